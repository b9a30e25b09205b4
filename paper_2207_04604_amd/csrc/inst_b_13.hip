// Kernel instantiations: ring degree 2^13, arithmetic ArithB.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_b_13()
{
    static const EngineOps ops = Launch<Engine<ArithB, 13, 3>>::full();
    return &ops;
}
}
