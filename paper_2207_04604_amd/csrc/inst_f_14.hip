// Kernel instantiations: ring degree 2^14, arithmetic ArithF.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_f_14()
{
    static const EngineOps ops = Launch<Engine<ArithF, 14, 4>>::full();
    return &ops;
}
}
