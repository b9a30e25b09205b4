// Kernel instantiations: ring degree 2^16, arithmetic ArithF.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_f_16()
{
    static const EngineOps ops = Launch<Engine<ArithF, 16, 3, 12>>::transforms_only();
    return &ops;
}
}
