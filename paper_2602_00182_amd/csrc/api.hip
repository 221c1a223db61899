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
        HIP_VERSION_PATCH) " canon-2 gemm-16x16x32-k64"
        // launch geometry revision: which tile shapes and kernel forms the row count (GEMM), the batch
        // (attention) select.  They move no output byte, but a receipt pins them all the same.
        " tiles-3(gemm:n128@256wg,rowcut,n64@m96/192,norm-in-kernel@4rows;qgemm:sp@8rows;attn:split@128wg,rows8@16rows)";
}

extern "C" int det_last_hip_error(void) { return det::g_last_hip_error; }
