// Kernel instantiations: ring degree 2^14, arithmetic ArithB.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_b_14()
{
    static const EngineOps ops = Launch<Engine<ArithB, 14, 4>>::full();
    return &ops;
}
}
