// Kernel instantiations for ring degree 2^15.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_15()
{
    static const EngineOps ops = Launch<Engine<15, 4, 12>>::transforms_only();
    return &ops;
}
}
