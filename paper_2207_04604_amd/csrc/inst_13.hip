// Kernel instantiations for ring degree 2^13.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_13()
{
    static const EngineOps ops = Launch<Engine<13, 5>>::full();
    return &ops;
}
}
