// Kernel instantiations: ring degree 2^12, arithmetic ArithB.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_b_12()
{
    static const EngineOps ops = Launch<Engine<ArithB, 12, 3>>::full();
    return &ops;
}
}
