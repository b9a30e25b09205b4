// Kernel instantiations: ring degree 2^14, arithmetic Arith32.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_w_14()
{
    static const EngineOps ops = Launch<Engine<Arith32, 14, 4>>::full();
    return &ops;
}
}
