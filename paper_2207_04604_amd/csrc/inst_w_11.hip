// Kernel instantiations: ring degree 2^11, arithmetic Arith32.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_w_11()
{
    static const EngineOps ops = Launch<Engine<Arith32, 11, 3>>::full();
    return &ops;
}
}
