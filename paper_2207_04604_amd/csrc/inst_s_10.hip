// Kernel instantiations: ring degree 2^10, arithmetic ArithS.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_s_10()
{
    static const EngineOps ops = Launch<Engine<ArithS, 10, 3>>::full();
    return &ops;
}
}
