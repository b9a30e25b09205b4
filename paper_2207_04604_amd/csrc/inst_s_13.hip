// Kernel instantiations: ring degree 2^13, arithmetic ArithS.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_s_13()
{
    static const EngineOps ops = Launch<Engine<ArithS, 13, 3>>::full();
    return &ops;
}
}
