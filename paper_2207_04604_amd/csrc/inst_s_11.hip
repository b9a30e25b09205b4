// Kernel instantiations: ring degree 2^11, arithmetic ArithS.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_s_11()
{
    static const EngineOps ops = Launch<Engine<ArithS, 11, 3>>::full();
    return &ops;
}
}
