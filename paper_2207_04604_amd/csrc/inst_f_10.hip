// Kernel instantiations: ring degree 2^10, arithmetic ArithF.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_f_10()
{
    static const EngineOps ops = Launch<Engine<ArithF, 10, 3>>::full();
    return &ops;
}
}
