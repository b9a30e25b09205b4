// Kernel instantiations: ring degree 2^11, arithmetic ArithF.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_f_11()
{
    static const EngineOps ops = Launch<Engine<ArithF, 11, 3>>::full();
    return &ops;
}
}
