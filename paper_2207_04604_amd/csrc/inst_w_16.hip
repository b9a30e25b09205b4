// Kernel instantiations: ring degree 2^16, arithmetic Arith32.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_w_16()
{
    static const EngineOps ops = Launch<Engine<Arith32, 16, 3, 12>>::transforms_only();
    return &ops;
}
}
