// Library identification and per-thread error state.
#include <hip/hip_version.h>

#include "common.h"

namespace det {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }
}  // namespace det

#define DET_STR2(x) #x
#define DET_STR(x) DET_STR2(x)

extern "C" const char* det_fingerprint(void)
{
    return "libdetinfer gfx950 hip-" DET_STR(HIP_VERSION_MAJOR) "." DET_STR(HIP_VERSION_MINOR) "." DET_STR(
        HIP_VERSION_PATCH) " canon-1 gemm-16x16x32-k64";
}

extern "C" int det_last_hip_error(void) { return det::g_last_hip_error; }
