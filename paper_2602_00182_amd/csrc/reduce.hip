// RMSNorm and greedy argmax: one 256-thread workgroup per row; the sums use the balanced 256-leaf tree of
// fixed shape that the paper's section 6.5 (invariant 2) asks for, laid over four 64-wide wavefronts.
#include "common.h"

namespace det {

constexpr int kMaxVecPerThread = 8;  // H <= 8 * 256 * 8 = 16384

// Row i: thread t owns the 8-element vectors t, t+256, ... (element e -> lane (e/8) mod 256) and
// folds them in ascending e with fma(x,x,acc); then the 256-leaf tree; then
// y = bf16((x*r)*w) with r = 1/sqrt(ss/H + eps).
// QUANT: instead of y the kernel writes y's 8-bit block quantization (the bytes det_quant_act_q8 makes
// of y: per 64 consecutive elements d = max|y| / 127, code = clamp(rint(y / d))).  A block is the
// vectors of eight neighbouring threads, so its maximum is three exchanges inside the wave.
template <bool QUANT>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint4* __restrict__ x,
                                                      const uint4* __restrict__ w,
                                                      uint4* __restrict__ y, int H, float eps,
                                                      int8_t* __restrict__ codes, float* __restrict__ scales,
                                                      int ldd)
{
    __shared__ float scratch[4];
    const int nvec = H >> 3;
    const uint4* xr = x + (size_t)blockIdx.x * nvec;
    uint4* yr = y + (size_t)blockIdx.x * nvec;

    uint4 xv[kMaxVecPerThread], wv[kMaxVecPerThread];
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < kMaxVecPerThread; ++i) {  // the weights travel with the row, ahead of the reduction
        const int v = threadIdx.x + i * 256;
        if (v < nvec) wv[i] = w[v];
    }
#pragma unroll
    for (int i = 0; i < kMaxVecPerThread; ++i) {
        const int v = threadIdx.x + i * 256;
        if (v < nvec) {
            xv[i] = xr[v];
            acc = rms_fold(xv[i], acc);
        }
    }
    const float ss = block_tree_sum(acc, scratch);
    const float r = rms_scale(ss, H, eps);
#pragma unroll
    for (int i = 0; i < kMaxVecPerThread; ++i) {
        const int v = threadIdx.x + i * 256;
        if (v < nvec) {
            const uint4 yv = rms_apply(xv[i], wv[i], r);
            const uint32_t o[4] = {yv.x, yv.y, yv.z, yv.w};
            if constexpr (!QUANT) {
                yr[v] = yv;
            } else {
                float a[8];
                float amax = 0.0f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    a[2 * k] = bf16lo_to_f32(o[k]);
                    a[2 * k + 1] = bf16hi_to_f32(o[k]);
                    amax = fmaxf(amax, fmaxf(fabsf(a[2 * k]), fabsf(a[2 * k + 1])));
                }
                // H % 64 == 0: the eight threads of a block are all here or all absent
                amax = fmaxf(amax, __shfl_xor(amax, 1, kWave));
                amax = fmaxf(amax, __shfl_xor(amax, 2, kWave));
                amax = fmaxf(amax, __shfl_xor(amax, 4, kWave));
                const float df = amax / 127.0f;
                uint32_t c[2] = {0u, 0u};
                if (df != 0.0f) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const float q = rintf(a[k] / df);
                        const int iv = q < -127.0f ? -127 : (q > 127.0f ? 127 : (int)q);
                        c[k >> 2] |= (uint32_t)(iv & 0xFF) << (8 * (k & 3));
                    }
                }
                *reinterpret_cast<uint2*>(codes + (size_t)blockIdx.x * H + 8 * (size_t)v) = make_uint2(c[0], c[1]);
                if ((threadIdx.x & 7) == 0) scales[(size_t)(v >> 3) * ldd + blockIdx.x] = df;
            }
        }
    }
}

// (value, index) pair ordering: larger value wins; on equal values the smaller index wins.
// The operation is associative and commutative, so the reduction shape does not matter.
__device__ __forceinline__ void argmax_merge(float& bv, int& bi, float v, int i)
{
    if (i >= 0 && (bi < 0 || v > bv || (v == bv && i < bi))) {
        bv = v;
        bi = i;
    }
}

// One workgroup of kArgmaxThreads threads per row: a row of 32000 fp32 logits is 128 KB, and what
// bounds the kernel is how many of its bytes are in flight at once.
constexpr int kArgmaxThreads = 1024;
template <bool F32>
__global__ __launch_bounds__(kArgmaxThreads) void argmax_kernel(const void* __restrict__ logits,
                                                                int32_t* __restrict__ idx, int V, int vec)
{
    constexpr int T = kArgmaxThreads;
    __shared__ float sv[T / 64];
    __shared__ int si[T / 64];
    float bv = 0.0f;
    int bi = -1;  // -1: nothing but NaN seen so far
    // A thread's elements are visited in ascending index, so "strictly greater" keeps the lowest
    // index among its own; the merges below break the remaining ties by index.
    auto visit = [&](float v, int j) {
        if (v == v && (bi < 0 || v > bv)) {
            bv = v;
            bi = j;
        }
    };
    if (F32 && vec) {
        // 16-byte loads, four vectors in flight per thread
        const float4* row = reinterpret_cast<const float4*>(static_cast<const float*>(logits) + (size_t)blockIdx.x * V);
        const int nv = V >> 2;
        for (int v0 = threadIdx.x; v0 < nv; v0 += 4 * T) {
            float4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (v0 + u * T < nv) x[u] = row[v0 + u * T];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = v0 + u * T;
                if (q < nv) {
                    visit(x[u].x, 4 * q);
                    visit(x[u].y, 4 * q + 1);
                    visit(x[u].z, 4 * q + 2);
                    visit(x[u].w, 4 * q + 3);
                }
            }
        }
    } else if (!F32 && vec) {
        const uint4* row = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(logits) + (size_t)blockIdx.x * V);
        const int nv = V >> 3;
        for (int v0 = threadIdx.x; v0 < nv; v0 += 4 * T) {
            uint4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (v0 + u * T < nv) x[u] = row[v0 + u * T];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = v0 + u * T;
                if (q < nv) {
                    const uint32_t p[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        visit(bf16lo_to_f32(p[k]), 8 * q + 2 * k);
                        visit(bf16hi_to_f32(p[k]), 8 * q + 2 * k + 1);
                    }
                }
            }
        }
    } else {
        for (int j = threadIdx.x; j < V; j += T) {
            float v;
            if (F32)
                v = static_cast<const float*>(logits)[(size_t)blockIdx.x * V + j];
            else
                v = bf16_to_f32(static_cast<const uint16_t*>(logits)[(size_t)blockIdx.x * V + j]);
            visit(v, j);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(bv, off, kWave);
        const int oi = __shfl_xor(bi, off, kWave);
        argmax_merge(bv, bi, ov, oi);
    }
    if ((threadIdx.x & 63) == 0) {
        sv[threadIdx.x >> 6] = bv;
        si[threadIdx.x >> 6] = bi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < T / 64; ++k) argmax_merge(bv, bi, sv[k], si[k]);
        idx[blockIdx.x] = bi < 0 ? 0 : bi;
    }
}

}  // namespace det

using namespace det;

extern "C" int det_rmsnorm(const void* x, const void* w, void* y, int M, int H, float eps, void* stream)
{
    if (!x || !w || !y || M < 1 || H < 1) return DET_EINVAL;
    if (H % 8 != 0 || H > 8 * 256 * kMaxVecPerThread) return DET_ESHAPE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return DET_EALIGN;
    hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3(M), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(x), static_cast<const uint4*>(w), static_cast<uint4*>(y),
                       H, eps, nullptr, nullptr, 0);
    return check_launch();
}

extern "C" int det_rmsnorm_quant_q8(const void* x, const void* w, void* codes, void* scales, int M, int H, float eps,
                                    void* stream)
{
    if (!x || !w || !codes || !scales || M < 1 || H < 1) return DET_EINVAL;
    if (H % 64 != 0 || H > 8 * 256 * kMaxVecPerThread) return DET_ESHAPE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(codes) || !aligned16(scales)) return DET_EALIGN;
    hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3(M), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(x), static_cast<const uint4*>(w), nullptr, H, eps,
                       static_cast<int8_t*>(codes), static_cast<float*>(scales), (M + 3) & ~3);
    return check_launch();
}

extern "C" int det_argmax(const void* logits, int32_t* idx, int B, int V, int dtype, void* stream)
{
    if (!logits || !idx || B < 1 || V < 1) return DET_EINVAL;
    if (dtype != DET_BF16 && dtype != DET_F32) return DET_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // 16-byte loads when every row starts on a 16-byte boundary, element loads otherwise
    const int vec = aligned16(logits) && V % (dtype == DET_F32 ? 4 : 8) == 0;
    if (dtype == DET_F32)
        hipLaunchKernelGGL(argmax_kernel<true>, dim3(B), dim3(kArgmaxThreads), 0, s, logits, idx, V, vec);
    else
        hipLaunchKernelGGL(argmax_kernel<false>, dim3(B), dim3(kArgmaxThreads), 0, s, logits, idx, V, vec);
    return check_launch();
}
