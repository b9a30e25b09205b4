// Kernel instantiations: ring degree 2^16, arithmetic ArithS.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_s_16()
{
    static const EngineOps ops = Launch<Engine<ArithS, 16, 3, 12>>::transforms_only();
    return &ops;
}
}
