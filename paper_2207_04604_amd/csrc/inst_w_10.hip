// Kernel instantiations: ring degree 2^10, arithmetic Arith32.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_w_10()
{
    static const EngineOps ops = Launch<Engine<Arith32, 10, 3>>::full();
    return &ops;
}
}
