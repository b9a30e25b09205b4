// Kernel instantiations for ring degree 2^12.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_12()
{
    static const EngineOps ops = Launch<Engine<12, 4>>::full();
    return &ops;
}
}
