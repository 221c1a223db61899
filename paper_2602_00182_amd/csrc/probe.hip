// Measurement aid, not part of the decode path: how fast one compute unit pulls L2-resident data into LDS.
// Every workgroup streams the same buffer (like the activation tile of a tall GEMM, which all column tiles
// re-read), 1 KB per wave instruction, either straight into LDS (LDS-DMA) or through registers and LDS
// stores.  bench.py times it and reports bytes per clock per compute unit next to the GEMM counters.
#include "common.h"
#include "stream.h"

namespace det {

template <int U>
__global__ __launch_bounds__(256) void fill_probe_regs(const uint4* __restrict__ src, int n16, int iters,
                                                       uint32_t* __restrict__ sink)
{
    __shared__ uint4 lds[4096];  // 64 KB
    const int tid = threadIdx.x;
    int pos = (int)((blockIdx.x * 977u) % (uint32_t)(n16 - 256 * U));
    for (int it = 0; it < iters; ++it) {
        uint4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = src[pos + u * 256 + tid];
#pragma unroll
        for (int u = 0; u < U; ++u) lds[(u * 256 + tid) & 4095] = r[u];
        pos += 256 * U;
        if (pos > n16 - 256 * U) pos = 0;
    }
    __syncthreads();
    if (lds[tid].x == 0x12345678u) sink[0] = 1;  // keeps the loop alive; the buffer never holds that value
}

template <int U>
__global__ __launch_bounds__(256) void fill_probe_dma(const uint4* __restrict__ src, int n16, int iters,
                                                      uint32_t* __restrict__ sink)
{
    __shared__ uint4 lds[4096];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t base = (uint32_t)(uintptr_t)(lds_char_t*)lds;
    int pos = (int)((blockIdx.x * 977u) % (uint32_t)(n16 - 256 * U));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            dma_block(src + pos + u * 256 + wave * 64, (uint32_t)lane * 16u,
                      base + (uint32_t)(((u * 256 + wave * 64) & 4095) * 16));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        pos += 256 * U;
        if (pos > n16 - 256 * U) pos = 0;
    }
    __syncthreads();
    if (lds[tid].x == 0x12345678u) sink[0] = 1;
}

}  // namespace det

using namespace det;

extern "C" int det_probe_lds_fill(const void* src, size_t src_bytes, int path, int workgroups, int iters,
                                  void* sink, void* stream)
{
    constexpr int U = 8;  // wave instructions in flight per wave: 32 KB per workgroup
    if (!src || !sink || iters < 1 || workgroups < 1 || (path != 0 && path != 1)) return DET_EINVAL;
    if (src_bytes < (size_t)2 * 256 * U * 16 || src_bytes > ((size_t)1 << 30)) return DET_ESHAPE;
    if (!aligned16(src)) return DET_EALIGN;
    const int n16 = (int)(src_bytes / 16);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (path == 0)
        hipLaunchKernelGGL(fill_probe_regs<U>, dim3(workgroups), dim3(256), 0, s, static_cast<const uint4*>(src), n16,
                           iters, static_cast<uint32_t*>(sink));
    else
        hipLaunchKernelGGL(fill_probe_dma<U>, dim3(workgroups), dim3(256), 0, s, static_cast<const uint4*>(src), n16,
                           iters, static_cast<uint32_t*>(sink));
    return check_launch();
}
