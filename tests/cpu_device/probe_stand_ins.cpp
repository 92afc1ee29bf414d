// Test scaffolding (CPU only): the measurement aids of the library are timing loops in gfx950 assembly and have no
// place in a CPU build; the host code only needs their launchers to exist.
#include "ga_internal.h"

namespace ga {
hipError_t launch_probe_streams(uint32_t, uint32_t, uint32_t, bool, uint64_t, const float* const*, float* const*, hipStream_t) {
    return hipErrorNotSupported;
}
hipError_t launch_probe_valu(int, uint32_t, uint32_t, uint32_t*, hipStream_t) { return hipErrorNotSupported; }
}  // namespace ga
