// Kernel instantiations for ring degree 2^14.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_14()
{
    static const EngineOps ops = Launch<Engine<14, 5>>::full();
    return &ops;
}
}
