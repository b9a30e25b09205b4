// Kernel instantiations: ring degree 2^15, arithmetic ArithF.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_f_15()
{
    static const EngineOps ops = Launch<Engine<ArithF, 15, 3, 12>>::transforms_only();
    return &ops;
}
}
