// Kernel instantiations: ring degree 2^16, arithmetic ArithB.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_b_16()
{
    static const EngineOps ops = Launch<Engine<ArithB, 16, 3, 12>>::transforms_only();
    return &ops;
}
}
