// Kernel instantiations: ring degree 2^13, arithmetic ArithF.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_f_13()
{
    static const EngineOps ops = Launch<Engine<ArithF, 13, 3>>::full();
    return &ops;
}
}
