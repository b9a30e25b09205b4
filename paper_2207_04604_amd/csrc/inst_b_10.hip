// Kernel instantiations: ring degree 2^10, arithmetic ArithB.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_b_10()
{
    static const EngineOps ops = Launch<Engine<ArithB, 10, 3>>::full();
    return &ops;
}
}
