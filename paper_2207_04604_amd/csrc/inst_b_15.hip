// Kernel instantiations: ring degree 2^15, arithmetic ArithB.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_b_15()
{
    static const EngineOps ops = Launch<Engine<ArithB, 15, 3, 12>>::transforms_only();
    return &ops;
}
}
