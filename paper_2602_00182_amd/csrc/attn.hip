// Single-query attention over a KV cache in fixed 256-token chunks, and the softmax statistics it
// is built on.  Every reduction has a written order (the paper's section 6.5, invariants 2 and 3):
// scores on the matrix cores with one accumulator chain over the head dimension, chunk sums
// through the 256-leaf tree, chunk partials combined in ascending chunk order.  A chunk's
// arithmetic depends on nothing but that sequence's own cache rows and length.
#include <math.h>

#include <atomic>

#include "internal.h"
#include "stream.h"

namespace det {

constexpr int kChunk = 256;
constexpr int kD = 128;

// Softmax statistics of one chunk for G independent rows at once (the G query heads of a KV group in the
// attention kernel, G = 1 in the softmax entry point), one token per thread (leaf = threadIdx.x):
//   m_c = max of the valid scores;  e = det_expf(s - m_c) for a valid token, 0 otherwise;
//   l_c = the 256-leaf sum of e: inside a wavefront lane i takes lane i+off for off = 32, 16, .., 1, and
//         the four wave sums q0..q3 combine as (q0+q2)+(q1+q3).
// The G reductions are independent and share the barriers.  `scratch`: G x 4 floats of LDS; kScratchIdle
// says that no thread can still be reading it from an earlier call (saves the leading barrier).
// This is the only implementation of these statistics in the library: the attention kernel and
// det_softmax_f32 both call it.
template <int G, bool kScratchIdle>
__device__ __forceinline__ void chunk_stats(const float (&s)[G], bool valid, float (*scratch)[4], float (&m_c)[G],
                                            float (&e)[G], float (&l_c)[G])
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    float sv[G], red[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        sv[h] = valid ? s[h] : -INFINITY;
        red[h] = sv[h];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
#pragma unroll
        for (int h = 0; h < G; ++h) red[h] = fmaxf(red[h], __shfl_xor(red[h], off, kWave));
    if constexpr (!kScratchIdle) __syncthreads();
    if (lane == 0)
#pragma unroll
        for (int h = 0; h < G; ++h) scratch[h][wave] = red[h];
    __syncthreads();
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m_c[h] = fmaxf(fmaxf(scratch[h][0], scratch[h][1]), fmaxf(scratch[h][2], scratch[h][3]));
        e[h] = valid ? det_expf(sv[h] - m_c[h]) : 0.0f;
        red[h] = e[h];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
#pragma unroll
        for (int h = 0; h < G; ++h) red[h] = red[h] + __shfl_down(red[h], off, kWave);
    __syncthreads();  // the maxima in scratch have been read
    if (lane == 0)
#pragma unroll
        for (int h = 0; h < G; ++h) scratch[h][wave] = red[h];
    __syncthreads();
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float qa = scratch[h][0] + scratch[h][2];
        const float qb = scratch[h][1] + scratch[h][3];
        l_c[h] = qa + qb;
    }
}

// Combination of chunk statistics in ascending chunk order:
//   m = max_c m_c;  w_c = det_expf(m_c - m);  L = fold_c (L + w_c*l_c) from +0.
__device__ __forceinline__ float combine_max(const float* mc, int nc)
{
    float m = mc[0];
    for (int c = 1; c < nc; ++c) m = fmaxf(m, mc[c]);
    return m;
}

// ------------------------------------------------------------------ attention, pass 1

// Grid (chunk, kv head, sequence); 256 threads.  G = query heads per KV head.
//   scores: wave w takes tokens 64w..64w+63 of the chunk as four 16-token blocks; the K rows are
//           the row operand of v_mfma_f32_16x16x32_bf16 and the G query vectors (zero padded to
//           16) its column operand; four steps cover the 128 head dimensions in ascending order
//           (step i takes d = 32g + 8i + e for lane group g).
//   stats : chunk_stats per head, token = thread.
//   PV    : lane (p = lane/16, dg = lane%16) of wave w owns d = 8dg..8dg+7 and tokens
//           64w + 4it + p, it = 0..15, folded in ascending it with fma from +0; the four p are
//           summed as (p0+p2)+(p1+p3), then the four waves as (w0+w2)+(w1+w3).
template <int G, bool VLDS>
__global__ __launch_bounds__(256) void attn_chunk_kernel(const uint16_t* __restrict__ q,
                                                         const uint16_t* __restrict__ kcache,
                                                         const uint16_t* __restrict__ vcache,
                                                         const int32_t* __restrict__ seqlens,
                                                         const int32_t* __restrict__ slots,
                                                         float* __restrict__ ws_m, float* __restrict__ ws_l,
                                                         float* __restrict__ ws_o, int Hq, int Hkv, int Lmax,
                                                         int ncmax, float scale, int len_offset)
{
    __shared__ float sc[G][kChunk];       // scores, then e_j
    __shared__ float po[4][G][kD];        // per-wave partial outputs
    __shared__ float scratch[G][4];
    __shared__ uint4 vbuf[VLDS ? 4 : 1][VLDS ? 16 : 1][64];  // the chunk's V rows: wave, block of 4 tokens, lane

    // blockIdx.y names a group of G consecutive query heads; its KV head is the one those heads share.  A
    // launch with G = heads per KV head has one group per KV head; a launch with G = 1 on a model with
    // more gives every query head a workgroup of its own (same arithmetic per head, more workgroups).
    const int c = blockIdx.x, hgrp = blockIdx.y, b = blockIdx.z;
    const int kvh = (hgrp * G) / (Hq / Hkv);
    int len = seqlens[b] + len_offset;
    len = len > Lmax ? Lmax : len;
    const int t0 = c * kChunk;
    if (t0 >= len) return;  // uniform over the workgroup
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, lr = lane & 15;
    const int slot = slots ? slots[b] : b;  // which cache slot this row reads
    const size_t kv_base = ((size_t)slot * Hkv + kvh) * (size_t)Lmax * kD;
    const uint16_t* kp = kcache + kv_base;
    const uint16_t* vp = vcache + kv_base;

    // VLDS (launches with few workgroups, where latency and not bandwidth sets the time): the chunk's
    // V rows go straight into LDS (64 KB, LDS-DMA) before anything else, so that they travel while the
    // scores are computed.  Wave w loads what it will use itself: block `it` holds tokens 64w + 4it ..
    // +3, lane (g, lr) its 16 bytes d = 8lr..8lr+7 of token 4it + g -- the lane that reads it back.
    // Tokens past the length load nothing.  Large launches read V from global memory in the PV loop:
    // with 12 KB of LDS many workgroups share a compute unit and their phases overlap.
    if constexpr (VLDS) {
        const int wu = __builtin_amdgcn_readfirstlane(wave);  // the load takes wave-uniform base addresses
        const char* vsrc = reinterpret_cast<const char*>(vp + (size_t)(t0 + 64 * wu) * kD);
        const uint32_t vdst = (uint32_t)(uintptr_t)(lds_char_t*)&vbuf[0][0][0] + (uint32_t)wu * 16384u;
#pragma unroll
        for (int it = 0; it < 16; ++it)
            if (t0 + 64 * wave + 4 * it + g < len) dma_block(vsrc + it * 1024, (uint32_t)lane * 16u, vdst + it * 1024);
    }

    // query fragments: head lr (< G) of this KV group, d = 32g + 8i + e
    uint4 qf[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) qf[i] = make_uint4(0, 0, 0, 0);
    if (lr < G) {
        const uint4* qp = reinterpret_cast<const uint4*>(q + ((size_t)b * Hq + (size_t)hgrp * G + lr) * kD + 32 * g);
#pragma unroll
        for (int i = 0; i < 4; ++i) qf[i] = qp[i];
    }

#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const int tok = t0 + 64 * wave + 16 * tb + lr;
        uint4 kf[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) kf[i] = make_uint4(0, 0, 0, 0);
        if (tok < len) {
            const uint4* kr = reinterpret_cast<const uint4*>(kp + (size_t)tok * kD + 32 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) kf[i] = kr[i];
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[i]),
                                                          __builtin_bit_cast(bf16x8, qf[i]), acc, 0, 0, 0);
        // lane holds S[token = 16tb + 4g + v][head = lr]
        if (lr < G) {
#pragma unroll
            for (int v = 0; v < 4; ++v) sc[lr][64 * wave + 16 * tb + 4 * g + v] = acc[v] * scale;
        }
    }
    __syncthreads();

    const bool valid = t0 + tid < len;
    const size_t part = ((size_t)b * Hq + (size_t)hgrp * G) * ncmax + c;  // + h*ncmax
    {
        float sv[G], m_c[G], e[G], l_c[G];
#pragma unroll
        for (int h = 0; h < G; ++h) sv[h] = sc[h][tid];
        chunk_stats<G, true>(sv, valid, scratch, m_c, e, l_c);
#pragma unroll
        for (int h = 0; h < G; ++h) {
            sc[h][tid] = e[h];  // only this thread reads or writes slot tid until the barrier below
            if (tid == 0) {
                ws_m[part + (size_t)h * ncmax] = m_c[h];
                ws_l[part + (size_t)h * ncmax] = l_c[h];
            }
        }
    }
    __syncthreads();

    float o[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
        for (int d = 0; d < 8; ++d) o[h][d] = 0.0f;
    if constexpr (VLDS) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's V rows have landed
#pragma unroll 4
    for (int it = 0; it < 16; ++it) {
        const int tl = 64 * wave + 4 * it + g;
        if (t0 + tl < len) {
            uint4 vv;
            if constexpr (VLDS)
                vv = vbuf[wave][it][lane];
            else
                vv = *reinterpret_cast<const uint4*>(vp + (size_t)(t0 + tl) * kD + 8 * lr);
            const uint32_t pw[4] = {vv.x, vv.y, vv.z, vv.w};
            float vf[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                vf[2 * k] = bf16lo_to_f32(pw[k]);
                vf[2 * k + 1] = bf16hi_to_f32(pw[k]);
            }
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float e = sc[h][tl];
#pragma unroll
                for (int d = 0; d < 8; ++d) o[h][d] = __builtin_fmaf(e, vf[d], o[h][d]);
            }
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            float v = o[h][d];
            v = v + __shfl_down(v, 32, kWave);
            v = v + __shfl_down(v, 16, kWave);
            if (g == 0) po[wave][h][8 * lr + d] = v;
        }
    __syncthreads();
    for (int i = tid; i < G * kD; i += 256) {
        const int h = i / kD, d = i % kD;
        const float a = po[0][h][d] + po[2][h][d];
        const float bb = po[1][h][d] + po[3][h][d];
        ws_o[(part + (size_t)h * ncmax) * kD + d] = a + bb;
    }
}

// ------------------------------------------------------------------ attention, pass 2

// Grid (query head, sequence); 128 threads, thread = d.  The arithmetic is the ascending-chunk fold
// of the canonical order; only the data movement is parallel: the chunk maxima are reduced across
// the threads (max is exact, so order free), the weights w_c = det_expf(m_c - m) are computed one
// chunk per thread into LDS, and each thread then folds L and its own O[d] over the chunks in
// ascending order with the loads of 8 chunks in flight at a time.
// QUANT: instead of the bf16 output row the kernel writes its 8-bit block quantization (the bytes
// det_quant_act_q8 makes of it): a wave's 64 values are one block, so the block maximum is a wave
// reduction; `out` is then the int8 code array [B, Hq*128] and `scales` the block-major scale array
// with row stride ldd.
template <bool QUANT>
__global__ __launch_bounds__(128) void attn_combine_kernel(const int32_t* __restrict__ seqlens,
                                                           const float* __restrict__ ws_m,
                                                           const float* __restrict__ ws_l,
                                                           const float* __restrict__ ws_o,
                                                           void* __restrict__ out, int Hq, int Lmax,
                                                           int ncmax, int len_offset, float* __restrict__ scales,
                                                           int ldd)
{
    __shared__ float s_w[128];
    __shared__ float s_l[128];
    __shared__ float s_red[2];
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    int len = seqlens[b] + len_offset;
    len = len > Lmax ? Lmax : len;
    const size_t o_idx = ((size_t)b * Hq + h) * kD + d;
    auto store = [&](uint16_t y) {
        if constexpr (!QUANT) {
            static_cast<uint16_t*>(out)[o_idx] = y;
        } else {
            const float a = bf16_to_f32(y);
            float amax = fabsf(a);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, kWave));
            const float df = amax / 127.0f;
            int v = 0;
            if (df != 0.0f) {
                const float r = rintf(a / df);
                v = r < -127.0f ? -127 : (r > 127.0f ? 127 : (int)r);
            }
            static_cast<int8_t*>(out)[o_idx] = (int8_t)v;
            if ((d & 63) == 0) scales[(size_t)(2 * h + (d >> 6)) * ldd + b] = df;
        }
    };
    if (len <= 0) {  // uniform over the workgroup
        store(0);
        return;
    }
    const int nc = (len + kChunk - 1) / kChunk;
    const size_t part = ((size_t)b * Hq + h) * ncmax;
    float m = -INFINITY;
    for (int c = d; c < nc; c += 128) m = fmaxf(m, ws_m[part + c]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
    if ((d & 63) == 0) s_red[d >> 6] = m;
    __syncthreads();
    m = fmaxf(s_red[0], s_red[1]);

    float L = 0.0f, O = 0.0f;
    for (int c0 = 0; c0 < nc; c0 += 128) {
        const int n = min(128, nc - c0);
        __syncthreads();  // the previous tile's s_w / s_l are no longer read
        if (d < n) {
            s_w[d] = det_expf(ws_m[part + c0 + d] - m);
            s_l[d] = ws_l[part + c0 + d];
        }
        __syncthreads();
        const float* op = ws_o + (part + c0) * kD + d;
        int c = 0;
        for (; c + 8 <= n; c += 8) {
            float o[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) o[u] = op[(size_t)(c + u) * kD];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float w = s_w[c + u];
                const float wl = w * s_l[c + u];
                L = L + wl;
                const float wo = w * o[u];
                O = O + wo;
            }
        }
        for (; c < n; ++c) {
            const float w = s_w[c];
            const float wl = w * s_l[c];
            L = L + wl;
            const float wo = w * op[(size_t)c * kD];
            O = O + wo;
        }
    }
    store(f32_to_bf16_rne(O / L));
}

// ------------------------------------------------------------------ softmax on given scores

constexpr int kMaxChunksHook = 1024;

// One workgroup per row, chunks in ascending order; p holds e_j until the final rescale.
__global__ __launch_bounds__(256) void softmax_kernel(const float* __restrict__ s,
                                                      const int32_t* __restrict__ lens,
                                                      float* __restrict__ p, float* __restrict__ m_out,
                                                      float* __restrict__ l_out, int Lmax)
{
    __shared__ float mc[kMaxChunksHook];
    __shared__ float lc[kMaxChunksHook];
    __shared__ float scratch[1][4];
    const int r = blockIdx.x, tid = threadIdx.x;
    int len = lens[r];
    len = len > Lmax ? Lmax : len;
    if (len <= 0) {
        if (tid == 0) {
            m_out[r] = -INFINITY;
            l_out[r] = 0.0f;
        }
        return;
    }
    const float* sr = s + (size_t)r * Lmax;
    float* pr = p + (size_t)r * Lmax;
    const int nc = (len + kChunk - 1) / kChunk;
    for (int c = 0; c < nc; ++c) {
        const int j = c * kChunk + tid;
        const bool valid = j < len;
        const float sv[1] = {valid ? sr[j] : 0.0f};
        float m_c[1], e[1], l_c[1];
        chunk_stats<1, false>(sv, valid, scratch, m_c, e, l_c);
        if (valid) pr[j] = e[0];
        if (tid == 0) {
            mc[c] = m_c[0];
            lc[c] = l_c[0];
        }
    }
    __syncthreads();
    const float m = combine_max(mc, nc);
    float L = 0.0f;
    for (int c = 0; c < nc; ++c) {
        const float w = det_expf(mc[c] - m);
        const float wl = w * lc[c];
        L = L + wl;
    }
    for (int c = 0; c < nc; ++c) {
        const int j = c * kChunk + tid;
        if (j < len) {
            const float w = det_expf(mc[c] - m);
            const float we = w * pr[j];
            pr[j] = we / L;
        }
    }
    if (tid == 0) {
        m_out[r] = m;
        l_out[r] = L;
    }
}

static size_t attn_ws_floats(int B, int Hq, int Lmax)
{
    const size_t nc = (size_t)(Lmax + kChunk - 1) / kChunk;
    return (size_t)B * Hq * nc * (2 + kD);
}

// Chunk partials for det_attn_decode_static: a fixed array in the code object instead of a buffer the
// caller brings.  Every device the library runs on holds its own copy at its own address; in host code
// the name `scratch` is only a handle for hipGetSymbolAddress, never a pointer to pass to a kernel.
static __device__ __align__(256) unsigned char scratch[DET_ATTN_STATIC_WS_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of the current device's copy of `scratch`, looked up on the first call on that device.
static int static_scratch_ptr(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return DET_EHIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return DET_ESHAPE;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_last_hip_error((int)e);
            return DET_EHIP;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // two racing first calls store the same address
    }
    *out = p;
    return DET_OK;
}

}  // namespace det

using namespace det;

extern "C" size_t det_attn_decode_workspace_bytes(int B, int Hq, int D, int Lmax)
{
    if (B < 1 || Hq < 1 || D != kD || Lmax < 1) return 0;
    return attn_ws_floats(B, Hq, Lmax) * sizeof(float);
}

int det::attn_decode_impl(const void* q, const void* kcache, const void* vcache, const int32_t* seqlens,
                          const int32_t* slots, int len_offset, void* out, void* ws, size_t ws_bytes, int B, int Hq, int Hkv, int D,
                          int Lmax, float scale, hipStream_t s, void* qscales)
{
    if (!q || !kcache || !vcache || !seqlens || !out || !ws || B < 1 || Hq < 1 || Hkv < 1 || Lmax < 1)
        return DET_EINVAL;
    if (D != kD || Hq % Hkv != 0) return DET_ESHAPE;
    const int G = Hq / Hkv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return DET_ESHAPE;
    if (B > 65535 || Hkv > 65535 || Hq > 65535) return DET_ESHAPE;
    if (!aligned16(q) || !aligned16(kcache) || !aligned16(vcache) || !aligned16(out) || !aligned16(ws))
        return DET_EALIGN;
    if (ws_bytes < det_attn_decode_workspace_bytes(B, Hq, D, Lmax)) return DET_EWORKSPACE;
    const int ncmax = (Lmax + kChunk - 1) / kChunk;
    const size_t n = (size_t)B * Hq * ncmax;
    float* ws_m = static_cast<float*>(ws);
    float* ws_l = ws_m + n;
    float* ws_o = ws_l + n;
    // Launches of a few dozen workgroups (one sequence, short context) are all latency: every query head
    // then gets a workgroup of its own, which divides the statistics and the PV fold of a workgroup by G.
    const bool split_heads = G > 1 && (size_t)ncmax * Hkv * B <= 128;
    const dim3 grid(ncmax, split_heads ? Hq : Hkv, B);
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(kcache);
    const uint16_t* vv = static_cast<const uint16_t*>(vcache);
    // Which of the two data paths for V is a matter of time only: the arithmetic and its order are the
    // same, so a row's bytes do not depend on it.  At most two workgroups per compute unit: latency bound.
    const bool vlds = (size_t)grid.x * grid.y * grid.z <= 512;
#define DET_LAUNCH_ATTN(GG)                                                                                      \
    do {                                                                                                         \
        if (vlds)                                                                                                \
            hipLaunchKernelGGL((attn_chunk_kernel<GG, true>), grid, dim3(256), 0, s, qq, kk, vv, seqlens, slots, \
                               ws_m, ws_l, ws_o, Hq, Hkv, Lmax, ncmax, scale, len_offset);                      \
        else                                                                                                     \
            hipLaunchKernelGGL((attn_chunk_kernel<GG, false>), grid, dim3(256), 0, s, qq, kk, vv, seqlens, slots,\
                               ws_m, ws_l, ws_o, Hq, Hkv, Lmax, ncmax, scale, len_offset);                      \
    } while (0)
    switch (split_heads ? 1 : G) {
        case 1: DET_LAUNCH_ATTN(1); break;
        case 2: DET_LAUNCH_ATTN(2); break;
        case 4: DET_LAUNCH_ATTN(4); break;
        default: DET_LAUNCH_ATTN(8); break;
    }
#undef DET_LAUNCH_ATTN
    int rc = check_launch();
    if (rc != DET_OK) return rc;
    if (qscales) {
        if (!aligned16(qscales)) return DET_EALIGN;
        hipLaunchKernelGGL(attn_combine_kernel<true>, dim3(Hq, B), dim3(128), 0, s, seqlens, ws_m, ws_l, ws_o, out, Hq,
                           Lmax, ncmax, len_offset, static_cast<float*>(qscales), (B + 3) & ~3);
    } else {
        hipLaunchKernelGGL(attn_combine_kernel<false>, dim3(Hq, B), dim3(128), 0, s, seqlens, ws_m, ws_l, ws_o, out, Hq,
                           Lmax, ncmax, len_offset, nullptr, 0);
    }
    return check_launch();
}

extern "C" int det_attn_decode(const void* q, const void* kcache, const void* vcache, const int32_t* seqlens,
                               void* out, void* ws, size_t ws_bytes, int B, int Hq, int Hkv, int D, int Lmax,
                               float scale, void* stream)
{
    return attn_decode_impl(q, kcache, vcache, seqlens, nullptr, 0, out, ws, ws_bytes, B, Hq, Hkv, D, Lmax, scale,
                            static_cast<hipStream_t>(stream));
}

extern "C" int det_attn_decode_static(const void* q, const void* kcache, const void* vcache, const int32_t* seqlens,
                                      void* out, int B, int Hq, int Hkv, int D, int Lmax, float scale, void* stream)
{
    const size_t need = det_attn_decode_workspace_bytes(B, Hq, D, Lmax);
    if (need == 0) return (B < 1 || Hq < 1 || Lmax < 1) ? DET_EINVAL : DET_ESHAPE;
    if (need > (size_t)DET_ATTN_STATIC_WS_BYTES) return DET_EWORKSPACE;
    void* ws = nullptr;
    const int rc = static_scratch_ptr(&ws);
    if (rc != DET_OK) return rc;
    return attn_decode_impl(q, kcache, vcache, seqlens, nullptr, 0, out, ws, DET_ATTN_STATIC_WS_BYTES, B, Hq, Hkv, D,
                            Lmax, scale, static_cast<hipStream_t>(stream));
}

extern "C" int det_attn_decode_rows(const void* q, const void* kcache, const void* vcache, const int32_t* seqlens,
                                    const int32_t* slots, void* out, void* ws, size_t ws_bytes, int R, int Hq, int Hkv,
                                    int D, int Lmax, float scale, void* stream)
{
    if (!slots) return DET_EINVAL;
    return attn_decode_impl(q, kcache, vcache, seqlens, slots, 0, out, ws, ws_bytes, R, Hq, Hkv, D, Lmax, scale,
                            static_cast<hipStream_t>(stream));
}

extern "C" int det_attn_decode_quant_q8(const void* q, const void* kcache, const void* vcache, const int32_t* seqlens,
                                        const int32_t* slots, void* codes, void* scales, void* ws, size_t ws_bytes,
                                        int R, int Hq, int Hkv, int D, int Lmax, float scale, void* stream)
{
    if (!scales) return DET_EINVAL;
    return attn_decode_impl(q, kcache, vcache, seqlens, slots, 0, codes, ws, ws_bytes, R, Hq, Hkv, D, Lmax, scale,
                            static_cast<hipStream_t>(stream), scales);
}

extern "C" int det_softmax_f32(const float* s, const int32_t* lens, float* p, float* m_out, float* l_out,
                               int R, int Lmax, void* stream)
{
    if (!s || !lens || !p || !m_out || !l_out || R < 1 || Lmax < 1) return DET_EINVAL;
    if ((Lmax + kChunk - 1) / kChunk > kMaxChunksHook) return DET_ESHAPE;
    hipLaunchKernelGGL(softmax_kernel, dim3(R), dim3(256), 0, static_cast<hipStream_t>(stream), s, lens, p,
                       m_out, l_out, Lmax);
    return check_launch();
}
