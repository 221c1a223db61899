// Single-query attention over a KV cache in fixed 256-token chunks, and the softmax statistics it
// is built on.  Every reduction has a written order (the paper's section 6.5, invariants 2 and 3):
// scores on the matrix cores with one accumulator chain over the head dimension, chunk sums
// through the 256-leaf tree, chunk partials combined in ascending chunk order.  A chunk's
// arithmetic depends on nothing but that sequence's own cache rows and length.
#include <math.h>

#include <atomic>
#include <type_traits>

#include "internal.h"
#include "stream.h"

namespace det {

constexpr int kChunk = 256;
constexpr int kD = 128;
constexpr int kHalfTok = 128;  // tokens of the half chunk whose V^T sits in LDS at a time

// Softmax statistics of one 256-token chunk of one row, computed by ONE wavefront.  Lane 16r + i holds the
// scores of the tokens 64r + 16k + i, k = 0..3, of the chunk (s[k], valid[k]; chunk_token(lane, k)): the sixteen
// lanes of a row hold one group of 64 leaves of the 256-leaf tree, so the tree's strides 32 and 16 pair values
// of one lane, its strides 8, 4, 2, 1 are shifts inside a row of sixteen lanes (a modifier of the adding
// instruction), and only the four group sums cross rows, through scalar registers.
//   m_c = max of the valid scores (-inf if there is none);
//   e   = det_expf(s - m_c) for a valid token, 0 otherwise;
//   l_c = the 256-leaf sum of e: inside each group of 64 leaves, leaf j takes leaf j+off for off = 32, 16, .., 1,
//         and the four group sums q0..q3 combine as (q0+q2)+(q1+q3).
// m_c and l_c are returned in every lane.  No LDS, no barrier: the waves of a workgroup run it independently
// on different rows.  This is the only implementation of these statistics in the library: the attention kernel
// and det_softmax_f32 both call it.
__device__ __forceinline__ int chunk_token(int lane, int k) { return ((lane >> 4) << 6) + (k << 4) + (lane & 15); }
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ void chunk_stats(const float (&s)[4], const bool (&valid)[4], float& m_c, float (&e)[4],
                                            float& l_c)
{
    float sv[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) sv[k] = valid[k] ? s[k] : -INFINITY;
    float m = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));  // max is exact: any order
    m = fmaxf(m, lane_plus<8>(m));  // (a lane past its row's end reads 0 here and holds nothing of use afterwards:
    m = fmaxf(m, lane_plus<4>(m));  //  lane 0 of a row only ever takes lanes inside the row)
    m = fmaxf(m, lane_plus<2>(m));
    m = fmaxf(m, lane_plus<1>(m));
    m = fmaxf(fmaxf(lane_value(m, 0), lane_value(m, 16)), fmaxf(lane_value(m, 32), lane_value(m, 48)));
    m_c = m;
#pragma unroll
    for (int k = 0; k < 4; ++k) e[k] = valid[k] ? det_expf(sv[k] - m) : 0.0f;
    const float a = e[0] + e[2];  // stride 32: leaf j takes leaf j + 32, j = i and j = 16 + i
    const float b = e[1] + e[3];
    float t = a + b;              // stride 16
    t = t + lane_plus<8>(t);
    t = t + lane_plus<4>(t);
    t = t + lane_plus<2>(t);
    t = t + lane_plus<1>(t);
    const float qa = lane_value(t, 0) + lane_value(t, 32);
    const float qb = lane_value(t, 16) + lane_value(t, 48);
    l_c = qa + qb;
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

// One workgroup: one 256-token chunk of one cache slot's K/V, for up to RT query rows (tokens) times G
// query heads that share the KV head ("pairs").  Decode launches it with RT = 1 (every row has a cache slot
// of its own); the rows form with RT = 8 lets the rows of one prompt share each chunk of K and V (causal
// prefill: row i of a prompt has length p + i).  Grid (chunk, head group, row tile); 256 threads.
//
// The arithmetic of one (row, head, chunk) is the same whatever else sits in the workgroup:
//   scores: wave w takes tokens 64w..64w+63 of the chunk as four 16-token blocks; the K rows are the row
//           operand of v_mfma_f32_16x16x32_bf16 and sixteen pairs' query vectors its column operand; four
//           steps cover the 128 head dimensions in ascending order (step i takes d = 32g + 8i + e for lane
//           group g), one accumulator chain per (token, pair), then one multiply by the scale.
//   stats : chunk_stats, one wave per pair, a token valid iff it lies below that row's length.
//   PV    : on the matrix cores as well.  e_j (fp32, >= 0) is cut into three bf16 pieces by truncation,
//           e = hi + mid + lo exactly, so every product piece * v is exact in fp32; one accumulator chain
//           per (pair, d) runs over the chunk's eight 32-token steps in ascending order, each step adding
//           the hi, then the mid, then the lo products (V^T is the row operand, the pieces the column
//           operand).  Tokens at or past the row's length have e = 0 and add +0.
// Rows of a tile that name different slots are handled one slot after the other (same arithmetic, no
// sharing).  V rows at or past the longest length in the workgroup are never read (zeros instead), K rows
// likewise; what the cache holds there cannot reach an output.

// Index (in uint4 = eight tokens of one head dimension) into the transposed V half tile: 128 rows (d) of 16
// pieces (128 tokens), the pieces of a row rotated by d + d/8 so that both the transposing writes (rows 8
// apart, same piece) and the operand reads (sixteen consecutive rows, same piece) spread over the banks.
__device__ __forceinline__ int vt_index(int d, int piece) { return d * 16 + ((piece + d + (d >> 3)) & 15); }
// Index (in floats) of token tok in pair p's score row: the row's 16-byte pieces are rotated by p, so that
// sixteen pairs reading or writing the same tokens hit different banks.
__device__ __forceinline__ int sc_index(int p, int tok)
{
    return p * kChunk + ((((tok >> 2) + p) & 63) << 2) + (tok & 3);
}

template <int I>
__device__ __forceinline__ uint32_t u4_word(const uint4& v)
{
    return I == 0 ? v.x : (I == 1 ? v.y : (I == 2 ? v.z : v.w));
}

template <int G, int RT, bool DIRECT>
__global__ __launch_bounds__(256, RT == 1 ? 4 : 2) void attn_tile_kernel(const uint16_t* __restrict__ q,
                                                        const uint16_t* __restrict__ kcache,
                                                        const uint16_t* __restrict__ vcache,
                                                        const int32_t* __restrict__ seqlens,
                                                        const int32_t* __restrict__ slots,
                                                        float* __restrict__ ws_m, float* __restrict__ ws_l,
                                                        float* __restrict__ ws_o, uint16_t* __restrict__ out, int R,
                                                        int Hq, int Hkv, int Lmax, int ncmax, float scale,
                                                        int len_offset)
{
    constexpr int NP = G * RT;             // pairs (row, head) of the workgroup
    constexpr int CBK = (NP + 15) / 16;    // blocks of sixteen pairs
    constexpr int DPW = 2 * CBK;           // (pair block, 16-wide d block) units of one wave in PV: 8*CBK/4
    static_assert((G & (G - 1)) == 0 && CBK <= 4, "pair layout");
    __shared__ __align__(16) float sc[NP * kChunk];  // scores, then e_j
    __shared__ uint4 vt[128 * 16];                   // V^T of half a chunk: [d][token], 32 KB
    __shared__ float mc_s[NP], lc_s[NP];             // the pairs' chunk statistics (DIRECT only)
    const int c = blockIdx.x, hgrp = blockIdx.y, tile = blockIdx.z;
    const int kvh = (hgrp * G) / (Hq / Hkv);
    const int t0 = c * kChunk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, lr = lane & 15;

    // the tile's rows: length (0: no such row) and slot; a row is active if it has tokens in this chunk
    __shared__ int len[RT], slot[RT];
    if (tid < RT) {
        const int r = tile * RT + tid;
        int l = 0, sl = -1;
        if (r < R) {
            l = seqlens[r] + len_offset;
            l = l > Lmax ? Lmax : l;
            sl = slots ? slots[r] : r;
        }
        len[tid] = l;
        slot[tid] = sl;
    }
    __syncthreads();
    if constexpr (DIRECT) {
        // rows without any token get zeros, from the workgroups of chunk 0 (there is no second pass to do it)
        if (c == 0) {
#pragma unroll
            for (int ri = 0; ri < RT; ++ri) {
                const int r = tile * RT + ri;
                if (r < R && len[ri] <= 0)
                    for (int i = tid; i < G * kD; i += 256) out[((size_t)r * Hq + (size_t)hgrp * G) * kD + i] = 0;
            }
        }
    }
    bool any = false;
#pragma unroll
    for (int ri = 0; ri < RT; ++ri) any = any || len[ri] > t0;
    if (!any) return;  // uniform over the workgroup

    uint32_t done = 0;
    bool first_group = true;
#pragma unroll 1
    for (int first = 0; first < RT; ++first) {
        if (((done >> first) & 1u) || len[first] <= t0) continue;
        const int group_slot = slot[first];
        uint32_t mask = 0;
        int maxlen = 0;
#pragma unroll
        for (int ri = 0; ri < RT; ++ri) {
            const int l = len[ri];
            if (l > t0 && slot[ri] == group_slot) {
                mask |= 1u << ri;
                maxlen = l > maxlen ? l : maxlen;
            }
        }
        done |= mask;
        if (!first_group) __syncthreads();  // the previous group's LDS contents are no longer read
        first_group = false;

        const size_t kv_base = ((size_t)group_slot * Hkv + kvh) * (size_t)Lmax * kD;
        const uint16_t* kp = kcache + kv_base;
        const uint16_t* vp = vcache + kv_base;

        // ---- V: half a chunk at a time through registers into the transposed LDS tile.  A thread owns the
        // 8 x 8 block (tokens 8*oc .. +7 of the half) x (d = 8*o .. +7): eight 16-byte loads, one per token.
        const int o = lane & 15, oc = 4 * wave + (lane >> 4);
        uint4 vr[8];
        auto load_v = [&](int hf) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int tok = t0 + kHalfTok * hf + 8 * oc + j;
                vr[j] = make_uint4(0, 0, 0, 0);
                if (tok < maxlen) vr[j] = *reinterpret_cast<const uint4*>(vp + (size_t)tok * kD + 8 * o);
            }
        };
        auto store_vt = [&]() {
            auto row = [&](auto e_tag) {
                constexpr int E = decltype(e_tag)::value;
                uint32_t w[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const uint32_t a = u4_word<E / 2>(vr[2 * jj]), b = u4_word<E / 2>(vr[2 * jj + 1]);
                    w[jj] = (E & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
                }
                vt[vt_index(8 * o + E, oc)] = make_uint4(w[0], w[1], w[2], w[3]);
            };
            row(std::integral_constant<int, 0>{});
            row(std::integral_constant<int, 1>{});
            row(std::integral_constant<int, 2>{});
            row(std::integral_constant<int, 3>{});
            row(std::integral_constant<int, 4>{});
            row(std::integral_constant<int, 5>{});
            row(std::integral_constant<int, 6>{});
            row(std::integral_constant<int, 7>{});
        };
        load_v(0);  // travels while the scores are computed

        // ---- scores
        {
            uint4 qf[CBK][4];
#pragma unroll
            for (int cb = 0; cb < CBK; ++cb) {
                const int p = 16 * cb + lr;
                const int ri = p / G, h = p % G;
#pragma unroll
                for (int i = 0; i < 4; ++i) qf[cb][i] = make_uint4(0, 0, 0, 0);
                if (p < NP && ((mask >> ri) & 1u)) {
                    const uint4* qp = reinterpret_cast<const uint4*>(
                        q + ((size_t)(tile * RT + ri) * Hq + (size_t)hgrp * G + h) * kD + 32 * g);
#pragma unroll
                    for (int i = 0; i < 4; ++i) qf[cb][i] = qp[i];
                }
            }
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                const int tok = t0 + 64 * wave + 16 * tb + lr;
                uint4 kf[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) kf[i] = make_uint4(0, 0, 0, 0);
                if (tok < maxlen) {
                    const uint4* kr = reinterpret_cast<const uint4*>(kp + (size_t)tok * kD + 32 * g);
#pragma unroll
                    for (int i = 0; i < 4; ++i) kf[i] = kr[i];
                }
#pragma unroll
                for (int cb = 0; cb < CBK; ++cb) {
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[i]),
                                                                      __builtin_bit_cast(bf16x8, qf[cb][i]), acc, 0, 0, 0);
                    // lane holds S[token = 16tb + 4g + v][pair = 16cb + lr]
                    const int p = 16 * cb + lr;
                    if (p < NP)
                        *reinterpret_cast<float4*>(&sc[sc_index(p, 64 * wave + 16 * tb + 4 * g)]) =
                            make_float4(acc[0] * scale, acc[1] * scale, acc[2] * scale, acc[3] * scale);
                }
            }
        }
        store_vt();  // first half of V; nobody reads vt before the barriers below
        load_v(1);   // second half travels during the statistics and the first half of PV
        __syncthreads();

        // ---- statistics: wave w takes pairs w, w+4, ..; no barrier inside
#pragma unroll
        for (int pi = 0; pi < (NP + 3) / 4; ++pi) {
            const int p = 4 * pi + wave;
            if (p < NP) {  // uniform over the wave
                const int ri = p / G;
                const bool in_group = (mask >> ri) & 1u;
                const int l = len[ri];
                float sv[4], e[4], m_c, l_c;
                bool vd[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    vd[k] = in_group && t0 + chunk_token(lane, k) < l;
                    sv[k] = sc[sc_index(p, chunk_token(lane, k))];
                }
                chunk_stats(sv, vd, m_c, e, l_c);
#pragma unroll
                for (int k = 0; k < 4; ++k) sc[sc_index(p, chunk_token(lane, k))] = e[k];
                if (lane == 0 && in_group) {
                    const size_t part = ((size_t)(tile * RT + ri) * Hq + (size_t)hgrp * G + p % G) * ncmax + c;
                    ws_m[part] = m_c;
                    ws_l[part] = l_c;
                    if constexpr (DIRECT) {
                        mc_s[p] = m_c;
                        lc_s[p] = l_c;
                    }
                }
            }
        }
        __syncthreads();

        // ---- PV.  Wave w owns pair block pb and the 16-wide d blocks db0 .. db0+DPW-1.
        const int pb = CBK == 1 ? 0 : (CBK == 2 ? wave >> 1 : wave);
        const int db0 = CBK == 1 ? 2 * wave : (CBK == 2 ? 4 * (wave & 1) : 0);
        const int pp = 16 * pb + lr;  // this lane's pair as the column of the operand and of the output
        f32x4 acc[DPW];
#pragma unroll
        for (int u = 0; u < DPW; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto pv_half = [&](int hf) {
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const int tk = kHalfTok * hf + 32 * s4 + 8 * g;  // this lane's eight tokens of the step
                float ev[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) ev[k] = 0.0f;
                if (pp < NP) {
                    const float4 a = *reinterpret_cast<const float4*>(&sc[sc_index(pp, tk)]);
                    const float4 b = *reinterpret_cast<const float4*>(&sc[sc_index(pp, tk + 4)]);
                    ev[0] = a.x, ev[1] = a.y, ev[2] = a.z, ev[3] = a.w;
                    ev[4] = b.x, ev[5] = b.y, ev[6] = b.z, ev[7] = b.w;
                }
                uint32_t hi[8], mid[8], lo[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    hi[k] = __float_as_uint(ev[k]) & 0xFFFF0000u;
                    const float r1 = ev[k] - __uint_as_float(hi[k]);
                    mid[k] = __float_as_uint(r1) & 0xFFFF0000u;
                    lo[k] = __float_as_uint(r1 - __uint_as_float(mid[k]));  // at most 8 significant bits: exact in bf16
                }
                auto pack = [](const uint32_t (&x)[8]) {
                    return __builtin_bit_cast(bf16x8, make_uint4((x[0] >> 16) | (x[1] & 0xFFFF0000u), (x[2] >> 16) | (x[3] & 0xFFFF0000u),
                                                                 (x[4] >> 16) | (x[5] & 0xFFFF0000u), (x[6] >> 16) | (x[7] & 0xFFFF0000u)));
                };
                const bf16x8 phi = pack(hi), pmid = pack(mid), plo = pack(lo);
#pragma unroll
                for (int u = 0; u < DPW; ++u) {
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, vt[vt_index(16 * (db0 + u) + lr, 4 * s4 + g)]);
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, phi, acc[u], 0, 0, 0);
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pmid, acc[u], 0, 0, 0);
                    acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, plo, acc[u], 0, 0, 0);
                }
            }
        };
        pv_half(0);
        __syncthreads();  // every wave is done with the first half of V^T
        store_vt();
        __syncthreads();
        pv_half(1);

        // lane holds O[d = 16*(db0+u) + 4g + v][pair pp]
        bool mine = false;
        int my_row = 0, my_len = 0;
#pragma unroll
        for (int ri = 0; ri < RT; ++ri)
            if (pp < NP && pp / G == ri && ((mask >> ri) & 1u)) {
                mine = true;
                my_row = tile * RT + ri;
                my_len = len[ri];
            }
        if (DIRECT && mine && my_len <= kChunk) {
            // The row has this one chunk: what the second pass would compute from the single partial, computed
            // here with the same operations (m = m_c; w = det_expf(m_c - m); L = 0 + w*l_c; O = 0 + w*O_c;
            // out = bf16(O / L)), and the partial output is not written.
            const float w = det_expf(mc_s[pp] - mc_s[pp]);
            const float wl = w * lc_s[pp];
            const float L = 0.0f + wl;
            uint16_t* orow = out + ((size_t)my_row * Hq + (size_t)hgrp * G + pp % G) * kD + 4 * g;
#pragma unroll
            for (int u = 0; u < DPW; ++u) {
                float y[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float wo = w * acc[u][v];
                    const float O = 0.0f + wo;
                    y[v] = O / L;
                }
                *reinterpret_cast<uint2*>(orow + 16 * (db0 + u)) = make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
            }
        } else if (mine) {
            const size_t part = ((size_t)my_row * Hq + (size_t)hgrp * G + pp % G) * ncmax + c;
            float* op = ws_o + part * kD + 4 * g;
#pragma unroll
            for (int u = 0; u < DPW; ++u) {
                float2* dst = reinterpret_cast<float2*>(op + 16 * (db0 + u));  // 8-byte stores: ws_o is only that aligned
                dst[0] = make_float2(acc[u][0], acc[u][1]);
                dst[1] = make_float2(acc[u][2], acc[u][3]);
            }
        }
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
                                                           int ldd, int first_pass_wrote_short_rows)
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
    if (first_pass_wrote_short_rows && len <= kChunk) return;  // rows of at most one chunk are complete (uniform)
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

// One workgroup per row; wave w computes the statistics of chunks w, w+4, .. (chunk_stats), then the chunks
// are combined in ascending order; p holds e_j until the final rescale.
__global__ __launch_bounds__(256) void softmax_kernel(const float* __restrict__ s,
                                                      const int32_t* __restrict__ lens,
                                                      float* __restrict__ p, float* __restrict__ m_out,
                                                      float* __restrict__ l_out, int Lmax)
{
    __shared__ float mc[kMaxChunksHook];
    __shared__ float lc[kMaxChunksHook];
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    for (int c = wave; c < nc; c += 4) {
        float sv[4], e[4], m_c, l_c;
        bool vd[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = c * kChunk + chunk_token(lane, k);
            vd[k] = j < len;
            sv[k] = vd[k] ? sr[j] : 0.0f;
        }
        chunk_stats(sv, vd, m_c, e, l_c);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (vd[k]) pr[c * kChunk + chunk_token(lane, k)] = e[k];
        if (lane == 0) {
            mc[c] = m_c;
            lc[c] = l_c;
        }
    }
    __syncthreads();  // also orders this workgroup's writes of e_j before the reads below
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
    // Launch geometry (which workgroup computes a (row, head, chunk); never its arithmetic):
    //   * rows that name their slots (prefill: consecutive rows of a prompt share a slot) go eight to a
    //     workgroup from sixteen rows on, so that they share each chunk of K and V;
    //   * launches of a few dozen workgroups (one sequence, short context) are all latency: every query
    //     head then gets a workgroup of its own, which divides a workgroup's statistics and PV work by G.
    const bool tiled = slots != nullptr && B >= 16;
    const int RT = tiled ? 8 : 1;
    const bool split_heads = !tiled && G > 1 && (size_t)ncmax * Hkv * B <= 128;
    const dim3 grid(ncmax, split_heads ? Hq : Hkv, (B + RT - 1) / RT);
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(kcache);
    const uint16_t* vv = static_cast<const uint16_t*>(vcache);
    // Without the quantizing second pass, the first pass itself finishes every row of at most one chunk.
    const bool direct = qscales == nullptr;
    uint16_t* out16 = static_cast<uint16_t*>(out);
#define DET_LAUNCH_ATTN2(GG, RTV, DIR)                                                                              \
    hipLaunchKernelGGL((attn_tile_kernel<GG, RTV, DIR>), grid, dim3(256), 0, s, qq, kk, vv, seqlens, slots, ws_m, ws_l, \
                       ws_o, out16, B, Hq, Hkv, Lmax, ncmax, scale, len_offset)
#define DET_LAUNCH_ATTN(GG)                                \
    do {                                                   \
        if (tiled && direct)                               \
            DET_LAUNCH_ATTN2(GG, 8, true);                 \
        else if (tiled)                                    \
            DET_LAUNCH_ATTN2(GG, 8, false);                \
        else if (direct)                                   \
            DET_LAUNCH_ATTN2(GG, 1, true);                 \
        else                                               \
            DET_LAUNCH_ATTN2(GG, 1, false);                \
    } while (0)
    switch (split_heads ? 1 : G) {
        case 1: DET_LAUNCH_ATTN(1); break;
        case 2: DET_LAUNCH_ATTN(2); break;
        case 4: DET_LAUNCH_ATTN(4); break;
        default: DET_LAUNCH_ATTN(8); break;
    }
#undef DET_LAUNCH_ATTN
#undef DET_LAUNCH_ATTN2
    int rc = check_launch();
    if (rc != DET_OK) return rc;
    if (qscales) {
        if (!aligned16(qscales)) return DET_EALIGN;
        hipLaunchKernelGGL(attn_combine_kernel<true>, dim3(Hq, B), dim3(128), 0, s, seqlens, ws_m, ws_l, ws_o, out, Hq,
                           Lmax, ncmax, len_offset, static_cast<float*>(qscales), (B + 3) & ~3, 0);
    } else if (ncmax > 1) {  // with one chunk at most, every row is already complete
        hipLaunchKernelGGL(attn_combine_kernel<false>, dim3(Hq, B), dim3(128), 0, s, seqlens, ws_m, ws_l, ws_o, out, Hq,
                           Lmax, ncmax, len_offset, nullptr, 0, 1);
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
