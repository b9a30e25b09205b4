// Kernel instantiations for ring degree 2^10.
#include "engine_inst.hpp"

namespace d2 {
const EngineOps *ops_10()
{
    static const EngineOps ops = Launch<Engine<10, 4>>::full();
    return &ops;
}
}
