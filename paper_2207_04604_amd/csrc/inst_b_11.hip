// Kernel instantiations: ring degree 2^11, arithmetic ArithB.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_b_11()
{
    static const EngineOps ops = Launch<Engine<ArithB, 11, 3>>::full();
    return &ops;
}
}
