// Host-only parts of the C ABI: version and last-HIP-error bookkeeping.
#include "common.h"

namespace svgear {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }
}  // namespace svgear

extern "C" int svgear_version(void) { return 1; }
extern "C" int svgear_last_hip_error(void) { return svgear::g_last_hip_error; }
