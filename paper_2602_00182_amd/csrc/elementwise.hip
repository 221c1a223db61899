// Elementwise steps of the decoder layer: rotary embedding (+ KV append), SwiGLU, residual add,
// embedding gather and the token bookkeeping of the greedy loop.  All arithmetic is fp32 with one
// rounding to bf16 per output; no step mixes data of different rows.
#include "internal.h"

namespace det {

// Grid (row); x, y: [R, nh, D] with row strides.
__global__ __launch_bounds__(256) void rope_kernel(const uint16_t* __restrict__ x, int ldx,
                                                   uint16_t* __restrict__ y, int ldy,
                                                   const int32_t* __restrict__ pos,
                                                   const float* __restrict__ cos_t,
                                                   const float* __restrict__ sin_t, int nh, int D, int Lmax)
{
    const int r = blockIdx.x, half = D >> 1;
    int p = pos[r];
    p = p < 0 ? 0 : (p >= Lmax ? Lmax - 1 : p);
    const uint16_t* xr = x + (size_t)r * ldx;
    uint16_t* yr = y + (size_t)r * ldy;
    for (int i = threadIdx.x; i < nh * half; i += 256) {
        const int h = i / half, k = i % half;
        rope_pair(xr[h * D + k], xr[h * D + k + half], cos_t[(size_t)p * half + k],
                  sin_t[(size_t)p * half + k], yr[h * D + k], yr[h * D + k + half]);
    }
}

// y = bf16( (g / (1 + det_expf(-g))) * u ), 8 elements per thread.  Grid (ceil(F/2048), R).
__global__ __launch_bounds__(256) void swiglu_kernel(const uint16_t* __restrict__ g, int ldg,
                                                     const uint16_t* __restrict__ u, int ldu,
                                                     uint16_t* __restrict__ y, int ldy, int F)
{
    const int r = blockIdx.y;
    const int e0 = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (e0 >= F) return;
    const uint4 gv = *reinterpret_cast<const uint4*>(g + (size_t)r * ldg + e0);
    const uint4 uv = *reinterpret_cast<const uint4*>(u + (size_t)r * ldu + e0);
    const uint32_t gp[4] = {gv.x, gv.y, gv.z, gv.w};
    const uint32_t up[4] = {uv.x, uv.y, uv.z, uv.w};
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float g0 = bf16lo_to_f32(gp[k]), g1 = bf16hi_to_f32(gp[k]);
        const float d0 = 1.0f + det_expf(-g0);
        const float d1 = 1.0f + det_expf(-g1);
        const float s0 = g0 / d0;
        const float s1 = g1 / d1;
        o[k] = pack_bf16x2(s0 * bf16lo_to_f32(up[k]), s1 * bf16hi_to_f32(up[k]));
    }
    *reinterpret_cast<uint4*>(y + (size_t)r * ldy + e0) = make_uint4(o[0], o[1], o[2], o[3]);
}

// z = bf16( fp32(x) + fp32(y) ), 8 elements per thread.
__global__ __launch_bounds__(256) void residual_kernel(const uint4* x, const uint4* y, uint4* z,
                                                       int64_t nvec)
{
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= nvec) return;
    const uint4 a = x[v], b = y[v];
    const uint32_t ap[4] = {a.x, a.y, a.z, a.w};
    const uint32_t bp[4] = {b.x, b.y, b.z, b.w};
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        o[k] = pack_bf16x2(bf16lo_to_f32(ap[k]) + bf16lo_to_f32(bp[k]),
                           bf16hi_to_f32(ap[k]) + bf16hi_to_f32(bp[k]));
    z[v] = make_uint4(o[0], o[1], o[2], o[3]);
}

// Grid (ceil(H/2048), B): exact copy of one table row per sequence.
__global__ __launch_bounds__(256) void embed_kernel(const uint4* __restrict__ table,
                                                    const int32_t* __restrict__ tokens,
                                                    uint4* __restrict__ out, int nvec, int V)
{
    const int b = blockIdx.y;
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= nvec) return;
    int t = tokens[b];
    t = t < 0 ? 0 : (t >= V ? V - 1 : t);
    out[(size_t)b * nvec + v] = table[(size_t)t * nvec + v];
}

__global__ __launch_bounds__(256) void next_token_kernel(const int32_t* __restrict__ prompts, int Tp,
                                                         const int32_t* __restrict__ prompt_lens,
                                                         const int32_t* __restrict__ last_sampled,
                                                         int32_t* __restrict__ tokens_out,
                                                         int32_t* __restrict__ positions_out,
                                                         int32_t* __restrict__ history, int Th, int t, int B)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int tok = (t < prompt_lens[b] && t < Tp) ? prompts[(size_t)b * Tp + t] : last_sampled[b];
    tokens_out[b] = tok;
    positions_out[b] = t;
    history[(size_t)b * Th + t] = tok;
}

// Decode after a one-pass prefill: sequence b sits at its own position.
__global__ __launch_bounds__(256) void advance_kernel(const int32_t* __restrict__ last_sampled,
                                                      const int32_t* __restrict__ base_positions, int j,
                                                      int32_t* __restrict__ tokens_out,
                                                      int32_t* __restrict__ positions_out, int B)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    tokens_out[b] = last_sampled[b];
    positions_out[b] = base_positions[b] + j;
}

}  // namespace det

using namespace det;


extern "C" int det_rope(const void* x, int ldx, void* y, int ldy, const int32_t* pos, const float* cos_t,
                        const float* sin_t, int R, int nh, int D, int Lmax, void* stream)
{
    if (!x || !y || !pos || !cos_t || !sin_t || R < 1 || nh < 1 || Lmax < 1) return DET_EINVAL;
    if (D != 128) return DET_ESHAPE;
    if (ldx < nh * D || ldy < nh * D) return DET_EINVAL;
    hipLaunchKernelGGL(rope_kernel, dim3(R), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(x), ldx, static_cast<uint16_t*>(y), ldy, pos, cos_t, sin_t,
                       nh, D, Lmax);
    return check_launch();
}

extern "C" int det_swiglu(const void* g, int ldg, const void* u, int ldu, void* y, int ldy, int R, int F,
                          void* stream)
{
    if (!g || !u || !y || R < 1 || F < 1) return DET_EINVAL;
    if (F % 8 != 0 || R > 65535) return DET_ESHAPE;
    if (!aligned16(g) || !aligned16(u) || !aligned16(y) || ldg % 8 || ldu % 8 || ldy % 8) return DET_EALIGN;
    if (ldg < F || ldu < F || ldy < F) return DET_EINVAL;
    hipLaunchKernelGGL(swiglu_kernel, dim3((F + 2047) / 2048, R), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(g), ldg,
                       static_cast<const uint16_t*>(u), ldu, static_cast<uint16_t*>(y), ldy, F);
    return check_launch();
}

extern "C" int det_residual_add(const void* x, const void* y, void* z, int64_t n, void* stream)
{
    if (!x || !y || !z || n < 1) return DET_EINVAL;
    if (n % 8 != 0) return DET_ESHAPE;
    if (!aligned16(x) || !aligned16(y) || !aligned16(z)) return DET_EALIGN;
    const int64_t nvec = n / 8;
    hipLaunchKernelGGL(residual_kernel, dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4*>(x),
                       static_cast<const uint4*>(y), static_cast<uint4*>(z), nvec);
    return check_launch();
}

extern "C" int det_embed_gather(const void* table, const int32_t* tokens, void* out, int B, int H, int V,
                                void* stream)
{
    if (!table || !tokens || !out || B < 1 || H < 1 || V < 1) return DET_EINVAL;
    if (H % 8 != 0 || B > 65535) return DET_ESHAPE;
    if (!aligned16(table) || !aligned16(out)) return DET_EALIGN;
    const int nvec = H / 8;
    hipLaunchKernelGGL(embed_kernel, dim3((nvec + 255) / 256, B), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4*>(table), tokens,
                       static_cast<uint4*>(out), nvec, V);
    return check_launch();
}

extern "C" int det_next_token(const int32_t* prompts, int Tp, const int32_t* prompt_lens,
                              const int32_t* last_sampled, int32_t* tokens_out, int32_t* positions_out,
                              int32_t* history, int Th, int t, int B, void* stream)
{
    if (!prompts || !prompt_lens || !last_sampled || !tokens_out || !positions_out || !history || B < 1 ||
        Tp < 1 || Th < 1)
        return DET_EINVAL;
    if (t < 0 || t >= Th) return DET_EINVAL;
    hipLaunchKernelGGL(next_token_kernel, dim3((B + 255) / 256), dim3(256), 0,
                       static_cast<hipStream_t>(stream), prompts, Tp, prompt_lens, last_sampled, tokens_out,
                       positions_out, history, Th, t, B);
    return check_launch();
}

extern "C" int det_decode_advance(const int32_t* last_sampled, const int32_t* base_positions, int j,
                                  int32_t* tokens_out, int32_t* positions_out, int B, void* stream)
{
    if (!last_sampled || !base_positions || !tokens_out || !positions_out || B < 1 || j < 0) return DET_EINVAL;
    hipLaunchKernelGGL(advance_kernel, dim3((B + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       last_sampled, base_positions, j, tokens_out, positions_out, B);
    return check_launch();
}
