// Kernel instantiations: ring degree 2^14, arithmetic ArithS.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_s_14()
{
    static const EngineOps ops = Launch<Engine<ArithS, 14, 4>>::full();
    return &ops;
}
}
