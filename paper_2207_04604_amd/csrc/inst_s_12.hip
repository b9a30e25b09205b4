// Kernel instantiations: ring degree 2^12, arithmetic ArithS.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_s_12()
{
    static const EngineOps ops = Launch<Engine<ArithS, 12, 3>>::full();
    return &ops;
}
}
