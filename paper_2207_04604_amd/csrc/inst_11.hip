// Kernel instantiations for ring degree 2^11.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_11()
{
    static const EngineOps ops = Launch<Engine<11, 4>>::full();
    return &ops;
}
}
