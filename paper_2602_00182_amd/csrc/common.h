// Device-side building blocks shared by the kernels of libdetinfer: bf16 conversion, det_expf,
// the canonical 256-leaf tree, and the host-side error plumbing.
//
// Compile with -ffp-contract=off: every fp32 operation written here is individually rounded, and a
// fused multiply-add happens only where fmaf() is written.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/detinfer.h"

namespace det {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kWave = 64;
constexpr int kBlock = 256;  // threads per workgroup in every reduction kernel: 4 wavefronts

// ---------------------------------------------------------------- bf16 <-> fp32

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }

// Round to nearest, ties to even, on the upper 16 bits; NaN -> 0x7FC0; overflow -> +-inf.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return (uint32_t)f32_to_bf16_rne(lo) | ((uint32_t)f32_to_bf16_rne(hi) << 16);
}

// ---------------------------------------------------------------- det_expf

// exp(x) built only from an fp32 multiply, round-to-nearest-integer, fused multiply-adds and an
// integer add on the exponent field, so that it can be reproduced bit for bit anywhere:
//   n = rint(x*log2e);  r = fma(n,-ln2_hi,x);  r = fma(n,-ln2_lo,r);
//   p = degree-7 Taylor polynomial of exp(r), Horner form in fma;  result = p * 2^n by adding n to
//   the exponent bits.   x > 88.72 -> +inf;  x < -87 -> 0 (no subnormal results);  NaN -> 0x7FC00000.
__device__ __forceinline__ float det_expf(float x)
{
    if (x != x) return __uint_as_float(0x7FC00000u);
    if (x > 88.72f) return __uint_as_float(0x7F800000u);
    if (x < -87.0f) return 0.0f;
    const float n = __builtin_rintf(x * 0x1.715476p+0f);
    float r = __builtin_fmaf(n, -0x1.62e4p-1f, x);
    r = __builtin_fmaf(n, -0x1.7f7d1cp-20f, r);
    float p = 0x1.a01a02p-13f;
    p = __builtin_fmaf(p, r, 0x1.6c16c2p-10f);
    p = __builtin_fmaf(p, r, 0x1.111112p-7f);
    p = __builtin_fmaf(p, r, 0x1.555556p-5f);
    p = __builtin_fmaf(p, r, 0x1.555556p-3f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    return __uint_as_float((uint32_t)((int32_t)__float_as_uint(p) + (int32_t)n * (1 << 23)));
}

// ---------------------------------------------------------------- canonical reductions

// The value lane i+OFF holds, for the lanes i that the stride-halving tree needs at that level (i < OFF; what
// the other lanes receive is unspecified and never reaches lane 0).  Strides below 16 stay inside a row of
// sixteen lanes and are a modifier of the consuming instruction (row shift left: lane i reads lane i+OFF);
// 16 and 32 cross rows and go through the LDS crossbar.
template <int OFF>
__device__ __forceinline__ float lane_plus(float v)
{
    const int x = __builtin_bit_cast(int, v);
    if constexpr (OFF >= 16) {
        const int lane = (int)(threadIdx.x & (kWave - 1));
        return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(((lane + OFF) & (kWave - 1)) << 2, x));
    } else {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, x, 0x100 + OFF, 0xF, 0xF, true));
    }
}

// Sum of the 64 values of one wavefront as a balanced tree of fixed shape: level by level for the strides
// 32, 16, 8, 4, 2, 1, lane i adds the partial sum of lane i+stride to its own.  Lane 0 ends with the sum
// ((..(v0+v32)+(v16+v48)..)); other lanes hold values of no further use.
__device__ __forceinline__ float wave_tree_sum(float v)
{
    v = v + lane_plus<32>(v);
    v = v + lane_plus<16>(v);
    v = v + lane_plus<8>(v);
    v = v + lane_plus<4>(v);
    v = v + lane_plus<2>(v);
    v = v + lane_plus<1>(v);
    return v;
}

// Canonical sum of 256 leaves, one per thread of a 256-thread workgroup (leaf = threadIdx.x).
// Wave sums q0..q3 are combined as (q0+q2)+(q1+q3).  `scratch` is 4 floats of LDS; the function
// contains the barriers it needs and returns the sum to every thread.
__device__ __forceinline__ float block_tree_sum(float v, float* scratch)
{
    const float w = wave_tree_sum(v);
    __syncthreads();  // earlier readers of scratch are done
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[threadIdx.x >> 6] = w;
    __syncthreads();
    const float a = scratch[0] + scratch[2];
    const float b = scratch[1] + scratch[3];
    return a + b;
}

// Maximum of one value per thread over a 256-thread workgroup (exact, so order free).  NaN inputs
// are ignored by fmaxf semantics.  `scratch` is 4 floats of LDS.
__device__ __forceinline__ float block_max(float v, float* scratch)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(scratch[0], scratch[1]), fmaxf(scratch[2], scratch[3]));
}

// RMSNorm arithmetic shared by the kernel of its own and by the GEMM that normalizes its rows itself:
// the sum of squares of one 8-element vector folded into acc in ascending element order, and
// y = bf16((x*r)*w) of one vector.
__device__ __forceinline__ float rms_fold(const uint4& x, float acc)
{
    const uint32_t p[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float lo = bf16lo_to_f32(p[k]);
        const float hi = bf16hi_to_f32(p[k]);
        acc = __builtin_fmaf(lo, lo, acc);
        acc = __builtin_fmaf(hi, hi, acc);
    }
    return acc;
}
__device__ __forceinline__ float rms_scale(float ss, int H, float eps)
{
    const float mean = ss / (float)H;
    return 1.0f / __builtin_sqrtf(mean + eps);
}
__device__ __forceinline__ uint4 rms_apply(const uint4& x, const uint4& w, float r)
{
    const uint32_t p[4] = {x.x, x.y, x.z, x.w};
    const uint32_t q[4] = {w.x, w.y, w.z, w.w};
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float lo = (bf16lo_to_f32(p[k]) * r) * bf16lo_to_f32(q[k]);
        const float hi = (bf16hi_to_f32(p[k]) * r) * bf16hi_to_f32(q[k]);
        o[k] = pack_bf16x2(lo, hi);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// Epilogues.  kEpiStore: C = bf16(acc) or fp32 acc.  kEpiResidual: C = bf16(fp32(bf16(acc)) + fp32(R)),
// the bytes of the plain GEMM followed by the residual add.  kEpiSwiglu: the weight columns are packed
// gate_j, up_j interleaved, and Y[j] = bf16( silu(bf16(acc_gate_j)) * bf16(acc_up_j) ), the bytes of the
// plain GEMM followed by the SwiGLU step.  C (and R) may alias nothing the kernel reads except that C
// may be R itself: an output element is read and written by the same lane only.
constexpr int kEpiStore = 0, kEpiResidual = 1, kEpiSwiglu = 2;
// kEpiSwigluQuant (quantized GEMM with 128-column tiles only): the SwiGLU epilogue's bf16 values written as
// their 8-bit block quantization; a tile row holds exactly one block of 64 outputs.
constexpr int kEpiSwigluQuant = 3;
// kEpiRopeAppend (bf16 GEMM of the fused query/key/value projection): the weight columns of every
// 128-wide head are packed so that a rotation pair (d, d + 64) sits in adjacent columns 2d, 2d + 1;
// a lane's four columns are two pairs, which it rotates at the row's position and writes straight
// to where the layer wants them: query heads to qbuf, key heads (rotated) and value heads (as they
// are) to the row's cache slot at that position.  The bytes of the plain GEMM followed by the
// rotation and the append; C is not written.
constexpr int kEpiRopeAppend = 4;

struct gemm_rope_args {
    const int32_t* pos = nullptr;    // [M] position of each row (clamped to 0..Lmax-1)
    const int32_t* slots = nullptr;  // [M] cache slot of each row, or null: row b uses slot b
    const float* cos_t = nullptr;    // [Lmax, 64]
    const float* sin_t = nullptr;
    uint16_t* qbuf = nullptr;    // [M, Hq, 128]
    uint16_t* kcache = nullptr;  // [S, Hkv, Lmax, 128]
    uint16_t* vcache = nullptr;
    int Hq = 0, Hkv = 0, Lmax = 0;
};

// Rotate-half pair (i, i + D/2):
//   y_lo = bf16( fma(-x_hi, sin, x_lo*cos) ),  y_hi = bf16( fma(x_lo, sin, x_hi*cos) )
__device__ __forceinline__ void rope_pair(uint16_t xlo, uint16_t xhi, float c, float s, uint16_t& ylo,
                                          uint16_t& yhi)
{
    const float lo = bf16_to_f32(xlo), hi = bf16_to_f32(xhi);
    const float a = lo * c;
    const float b = hi * c;
    ylo = f32_to_bf16_rne(__builtin_fmaf(-hi, s, a));
    yhi = f32_to_bf16_rne(__builtin_fmaf(lo, s, b));
}

// kEpiRopeAppend for one lane: packed columns n..n+3 of head n / 128 are the pairs i0 = (n % 128) / 2
// and i0 + 1; p and slot are the row's (clamped) position and cache slot.
__device__ __forceinline__ void gemm_epilogue_rope_append(const float (&v)[4], const gemm_rope_args& ra, size_t row,
                                                          int p, int slot, int n)
{
    constexpr int D = 128, half = 64;
    const int head = n >> 7, i0 = (n & (D - 1)) >> 1;
    uint16_t x[4], lo0, hi0, lo1, hi1;
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = f32_to_bf16_rne(v[e]);
    uint16_t* dst;
    if (head < ra.Hq + ra.Hkv) {
        const float2 c = *reinterpret_cast<const float2*>(ra.cos_t + (size_t)p * half + i0);
        const float2 s = *reinterpret_cast<const float2*>(ra.sin_t + (size_t)p * half + i0);
        rope_pair(x[0], x[1], c.x, s.x, lo0, hi0);
        rope_pair(x[2], x[3], c.y, s.y, lo1, hi1);
        dst = head < ra.Hq ? ra.qbuf + (row * ra.Hq + head) * D
                           : ra.kcache + (((size_t)slot * ra.Hkv + (head - ra.Hq)) * ra.Lmax + p) * D;
    } else {
        lo0 = x[0], hi0 = x[1], lo1 = x[2], hi1 = x[3];
        dst = ra.vcache + (((size_t)slot * ra.Hkv + (head - ra.Hq - ra.Hkv)) * ra.Lmax + p) * D;
    }
    *reinterpret_cast<uint32_t*>(dst + i0) = lo0 | ((uint32_t)lo1 << 16);
    *reinterpret_cast<uint32_t*>(dst + half + i0) = hi0 | ((uint32_t)hi1 << 16);
}

__device__ __forceinline__ float silu_mul(float gate, float up)
{
    const float den = 1.0f + det_expf(-gate);
    const float sg = gate / den;
    return sg * up;
}

// The epilogue of one lane's four consecutive output columns v[0..3] of row `row`, first column n
// (both GEMM kernels end with a lane holding exactly that).
template <int EPI>
__device__ __forceinline__ void gemm_epilogue_store(const float (&v)[4], void* C, int ldc, const uint16_t* R, int ldr,
                                                    size_t row, int n, int out_f32)
{
    if constexpr (EPI == kEpiSwiglu) {
        const float g0 = bf16_to_f32(f32_to_bf16_rne(v[0])), u0 = bf16_to_f32(f32_to_bf16_rne(v[1]));
        const float g1 = bf16_to_f32(f32_to_bf16_rne(v[2])), u1 = bf16_to_f32(f32_to_bf16_rne(v[3]));
        uint32_t* dst = reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(C) + row * ldc + (n >> 1));
        *dst = pack_bf16x2(silu_mul(g0, u0), silu_mul(g1, u1));
    } else if constexpr (EPI == kEpiResidual) {
        const uint2 rv = *reinterpret_cast<const uint2*>(R + row * ldr + n);
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = bf16_to_f32(f32_to_bf16_rne(v[e]));
        y[0] = y[0] + bf16lo_to_f32(rv.x);
        y[1] = y[1] + bf16hi_to_f32(rv.x);
        y[2] = y[2] + bf16lo_to_f32(rv.y);
        y[3] = y[3] + bf16hi_to_f32(rv.y);
        uint2* dst = reinterpret_cast<uint2*>(static_cast<uint16_t*>(C) + row * ldc + n);
        *dst = make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
    } else if (out_f32) {
        float4* dst = reinterpret_cast<float4*>(static_cast<float*>(C) + row * ldc + n);
        *dst = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        uint2* dst = reinterpret_cast<uint2*>(static_cast<uint16_t*>(C) + row * ldc + n);
        *dst = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    }
}

// ---------------------------------------------------------------- host side

void set_last_hip_error(int e);

inline int check_launch()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return DET_EHIP;
    }
    return DET_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace det
