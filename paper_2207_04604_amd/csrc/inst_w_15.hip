// Kernel instantiations: ring degree 2^15, arithmetic Arith32.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_w_15()
{
    static const EngineOps ops = Launch<Engine<Arith32, 15, 3, 12>>::transforms_only();
    return &ops;
}
}
