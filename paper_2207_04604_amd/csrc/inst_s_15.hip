// Kernel instantiations: ring degree 2^15, arithmetic ArithS.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_s_15()
{
    static const EngineOps ops = Launch<Engine<ArithS, 15, 3, 12>>::transforms_only();
    return &ops;
}
}
