// Kernel instantiations for ring degree 2^16.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_16()
{
    static const EngineOps ops = Launch<Engine<16, 4, 12>>::transforms_only();
    return &ops;
}
}
