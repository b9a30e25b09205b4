// Kernel instantiations: ring degree 2^12, arithmetic ArithF.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_f_12()
{
    static const EngineOps ops = Launch<Engine<ArithF, 12, 3>>::full();
    return &ops;
}
}
