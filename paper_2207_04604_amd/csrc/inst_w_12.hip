// Kernel instantiations: ring degree 2^12, arithmetic Arith32.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_w_12()
{
    static const EngineOps ops = Launch<Engine<Arith32, 12, 3>>::full();
    return &ops;
}
}
