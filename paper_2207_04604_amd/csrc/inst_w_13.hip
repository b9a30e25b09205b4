// Kernel instantiations: ring degree 2^13, arithmetic Arith32.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_w_13()
{
    static const EngineOps ops = Launch<Engine<Arith32, 13, 3>>::full();
    return &ops;
}
}
