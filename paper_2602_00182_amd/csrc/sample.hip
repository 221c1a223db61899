// Seeded temperature / top-k / top-p sampling in a canonical iteration order (the paper's section
// 6.6: a fixed-seed PRNG and a canonical order make the emitted token a function of (seed, decode
// policy) alone).  One 256-thread workgroup per row.
//
//   z_j = logits_j / T (NaN counts as -inf, -0 as +0);  candidates ordered by (z descending, index
//   ascending);  the first k = min(top_k, V) kept;  e_i = det_expf(z_i - z_0);  c_i = c_{i-1} + e_i
//   in rank order, sequential fp32 adds from +0;  n = smallest i+1 with c_i >= top_p * c_{k-1};
//   u = counter-based uniform of (seed, sequence id, step);  target = u * c_{n-1};  the token is the
//   candidate of the smallest rank i < n with c_i > target (rank n-1 if rounding leaves none).
//
// The order is total (index breaks ties), so the k kept candidates and their ranks are unique and any
// selection / sorting network gives them: here an 8-bit radix select on the 64-bit key
// (order-preserving image of z, then ~index) with integer LDS histograms, and a bitonic sort of the
// k survivors.  The prefix sums are one thread's adds in rank order.  sample_kernel reads the row once
// per radix pass and serves any V; sample_kernel_reg (rows of at most 65536 logits) keeps the keys in
// registers and takes wider digits.
#include <math.h>

#include "common.h"

namespace det {

constexpr int kMaxTopK = 1024;

// Order-preserving map fp32 -> uint32 (larger float, larger key) and its inverse.
__device__ __forceinline__ uint32_t order_key(float z)
{
    const uint32_t u = __float_as_uint(z);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float order_key_inv(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

__device__ __forceinline__ uint64_t candidate_key(float logit, float temperature, int j)
{
    float z = logit / temperature;
    if (z != z) z = -INFINITY;
    if (z == 0.0f) z = 0.0f;  // -0 and +0 are the same candidate value
    return ((uint64_t)order_key(z) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
}

__device__ __forceinline__ uint64_t splitmix64_mix(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void sample_kernel(const float* __restrict__ logits, int V, float temperature,
                                                     int top_k, float top_p, uint64_t seed,
                                                     const int32_t* __restrict__ seq_ids,
                                                     const int32_t* __restrict__ steps,
                                                     int32_t* __restrict__ tokens)
{
    __shared__ uint32_t hist[256];
    __shared__ uint64_t sel[kMaxTopK];
    __shared__ float ebuf[kMaxTopK];
    __shared__ int s_digit, s_need, s_bin, s_count;

    const int tid = threadIdx.x;
    const float* row = logits + (size_t)blockIdx.x * V;
    const int k = top_k < V ? top_k : V;

    // ---- radix select: the k-th largest key, 8 bits per pass from the top
    uint64_t prefix = 0;   // decided top bits of the k-th largest key
    int need = k;          // rank still to be found among the keys that share the prefix
    int shift = 56;
    bool all_of_bin = false;
    for (int pass = 0; pass < 8; ++pass, shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < V; j += 256) {
            const uint64_t key = candidate_key(row[j], temperature, j);
            if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        uint32_t above = 0;  // keys with the prefix and a larger digit than tid
        for (int b = tid + 1; b < 256; ++b) above += hist[b];
        const uint32_t mine = hist[tid];
        if ((int)above < need && need <= (int)(above + mine)) {
            s_digit = tid;
            s_need = need - (int)above;
            s_bin = (int)mine;
        }
        __syncthreads();
        prefix = (prefix << 8) | (uint64_t)s_digit;
        need = s_need;
        all_of_bin = s_bin == need;  // every key of this bin is wanted: no need to look at lower bits
        __syncthreads();
        if (all_of_bin) break;
    }
    const uint64_t threshold = all_of_bin ? (prefix << shift) : prefix;

    // ---- gather the k survivors (any order), pad to a power of two, sort descending
    if (tid == 0) s_count = 0;
    __syncthreads();
    for (int j = tid; j < V; j += 256) {
        const uint64_t key = candidate_key(row[j], temperature, j);
        if (key >= threshold) sel[atomicAdd(&s_count, 1)] = key;
    }
    int kp = 1;
    while (kp < k) kp <<= 1;
    __syncthreads();
    for (int i = k + tid; i < kp; i += 256) sel[i] = 0;  // below every real key
    __syncthreads();
    for (int size = 2; size <= kp; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < (kp >> 1); i += 256) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool desc = (lo & size) == 0;
                const uint64_t a = sel[lo], b = sel[hi];
                if ((a < b) == desc) {
                    sel[lo] = b;
                    sel[hi] = a;
                }
            }
            __syncthreads();
        }
    }

    // ---- probabilities in rank order
    const float z0 = order_key_inv((uint32_t)(sel[0] >> 32));
    for (int i = tid; i < k; i += 256) ebuf[i] = det_expf(order_key_inv((uint32_t)(sel[i] >> 32)) - z0);
    __syncthreads();
    if (tid == 0) {
        float acc = 0.0f;
        for (int i = 0; i < k; ++i) {
            acc = acc + ebuf[i];
            ebuf[i] = acc;  // c_i
        }
        const float cut = top_p * ebuf[k - 1];
        int n = k;
        for (int i = 0; i < k; ++i)
            if (ebuf[i] >= cut) {
                n = i + 1;
                break;
            }
        const uint64_t ctr = ((uint64_t)(uint32_t)seq_ids[blockIdx.x] << 32) | (uint64_t)(uint32_t)steps[blockIdx.x];
        const uint64_t r = splitmix64_mix(seed + (ctr + 1) * 0x9E3779B97F4A7C15ull);
        const float u = (float)(uint32_t)(r >> 40) * 0x1p-24f;
        const float target = u * ebuf[n - 1];
        int pick = n - 1;
        for (int i = 0; i < n; ++i)
            if (ebuf[i] > target) {
                pick = i;
                break;
            }
        tokens[blockIdx.x] = (int32_t)(0xFFFFFFFFu - (uint32_t)sel[pick]);
    }
}

// The same selection for rows of at most 1024*KPT logits, with the row read once: 1024 threads, each
// keeps the z keys of its KPT candidates (j = tid + 1024 i) in registers, so the radix passes, the
// gather and the division by the temperature touch no memory but the LDS histogram.  The sort and the
// exponentials use all threads; the prefix sums stay one thread's sequential adds in rank order (their
// order is part of the definition), the two searches over them are minimum reductions (the first
// index that satisfies a condition does not depend on how it is found).
constexpr int kSampleThreads = 1024;
template <int KPT>
__global__ __launch_bounds__(kSampleThreads) void sample_kernel_reg(const float* __restrict__ logits, int V,
                                                                    float temperature, int top_k, float top_p,
                                                                    uint64_t seed, const int32_t* __restrict__ seq_ids,
                                                                    const int32_t* __restrict__ steps,
                                                                    int32_t* __restrict__ tokens)
{
    constexpr int T = kSampleThreads;
    __shared__ uint32_t hist2[2][2 * kSampleThreads];  // the histogram of pass p is hist2[p & 1]; the other one is cleared meanwhile
    __shared__ uint64_t sel[kMaxTopK];
    __shared__ float ebuf[kMaxTopK];
    __shared__ int s_digit, s_need, s_bin, s_count, s_n, s_pick;
    __shared__ float s_cut, s_target;
    __shared__ uint32_t wave_tot[kSampleThreads / kWave];

    const int tid = threadIdx.x;
    const float* row = logits + (size_t)blockIdx.x * V;
    const int k = top_k < V ? top_k : V;

    uint32_t zk[KPT];  // high half of candidate_key; the low half is 0xFFFFFFFF - j
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int j = tid + T * i;
        zk[i] = j < V ? (uint32_t)(candidate_key(row[j], temperature, j) >> 32) : 0u;
    }
    auto key_of = [&](int i) { return ((uint64_t)zk[i] << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)(tid + T * i)); };

    // ---- radix select as in sample_kernel, with digits of 11, 11, 10 bits for each half of the key: the
    // top byte of a float (sign and seven exponent bits) takes a handful of values over a row of logits
    // and the increments of a pass would queue up on those few counters; three more bits spread them.
    // Thread t owns bins 2t and 2t+1 of the 2048.
    uint64_t prefix = 0;
    int need = k;
    int shift = 64;
    bool all_of_bin = false;
    hist2[0][2 * tid] = 0;
    hist2[0][2 * tid + 1] = 0;
    __syncthreads();
    for (int pass = 0; pass < 6; ++pass) {
        const int width = (pass % 3 == 2) ? 10 : 11;
        shift -= width;
        const uint32_t dmask = (1u << width) - 1u;
        uint32_t* hist = hist2[pass & 1];
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const bool in = tid + T * i < V;
            const uint64_t key = key_of(i);
            if (in && (pass == 0 || (key >> (shift + width)) == prefix)) atomicAdd(&hist[(uint32_t)(key >> shift) & dmask], 1u);
        }
        __syncthreads();
        // above(b) = keys with the prefix and a larger digit than b: suffix sums of the threads' pair sums inside
        // each wave, then the totals of the higher waves
        const uint32_t h_lo = hist[2 * tid], h_hi = hist[2 * tid + 1];
        uint32_t incl = h_lo + h_hi;
        {
            const int l = tid & (kWave - 1);
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t other = (uint32_t)__shfl_down((int)incl, off, kWave);
                if (l + off < kWave) incl += other;
            }
            if (l == 0) wave_tot[tid >> 6] = incl;
        }
        hist2[(pass + 1) & 1][2 * tid] = 0;  // next pass's histogram
        hist2[(pass + 1) & 1][2 * tid + 1] = 0;
        __syncthreads();
        {
            uint32_t above_hi = incl - (h_lo + h_hi);  // pairs of higher threads of this wave
            for (int w = (tid >> 6) + 1; w < T / kWave; ++w) above_hi += wave_tot[w];
            const uint32_t above_lo = above_hi + h_hi;
            if ((int)above_hi < need && need <= (int)(above_hi + h_hi)) {
                s_digit = 2 * tid + 1;
                s_need = need - (int)above_hi;
                s_bin = (int)h_hi;
            } else if ((int)above_lo < need && need <= (int)(above_lo + h_lo)) {
                s_digit = 2 * tid;
                s_need = need - (int)above_lo;
                s_bin = (int)h_lo;
            }
        }
        __syncthreads();
        // (s_digit, s_need, s_bin and wave_tot are next written a barrier or more into the next pass)
        prefix = (prefix << width) | (uint64_t)s_digit;
        need = s_need;
        all_of_bin = s_bin == need;  // every key of this bin is wanted: no need to look at lower bits
        if (all_of_bin) break;
    }
    // all 64 bits decided (shift == 0) or the rest left open
    const uint64_t threshold = all_of_bin ? (prefix << shift) : prefix;

    // ---- gather the k survivors (any order), pad to a power of two, sort descending
    if (tid == 0) s_count = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        if (tid + T * i < V) {
            const uint64_t key = key_of(i);
            if (key >= threshold) sel[atomicAdd(&s_count, 1)] = key;
        }
    }
    int kp = 1;
    while (kp < k) kp <<= 1;
    __syncthreads();
    for (int i = k + tid; i < kp; i += T) sel[i] = 0;  // below every real key
    __syncthreads();
    for (int size = 2; size <= kp; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < (kp >> 1); i += T) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool desc = (lo & size) == 0;
                const uint64_t a = sel[lo], b = sel[hi];
                if ((a < b) == desc) {
                    sel[lo] = b;
                    sel[hi] = a;
                }
            }
            __syncthreads();
        }
    }

    // ---- probabilities in rank order
    const float z0 = order_key_inv((uint32_t)(sel[0] >> 32));
    for (int i = tid; i < k; i += T) ebuf[i] = det_expf(order_key_inv((uint32_t)(sel[i] >> 32)) - z0);
    __syncthreads();
    if (tid == 0) {
        float acc = 0.0f;
        int i = 0;
        for (; i + 8 <= k; i += 8) {  // eight reads in flight, then their adds in order
            float e[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) e[u] = ebuf[i + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                acc = acc + e[u];
                e[u] = acc;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) ebuf[i + u] = e[u];  // c_i
        }
        for (; i < k; ++i) {
            acc = acc + ebuf[i];
            ebuf[i] = acc;
        }
        s_cut = top_p * ebuf[k - 1];
        s_n = k;
    }
    __syncthreads();
    {   // n = 1 + the first i with c_i >= cut (k if rounding leaves none)
        const float cut = s_cut;
        int best = k;
        for (int i = tid; i < k; i += T)
            if (ebuf[i] >= cut) {
                best = i + 1;
                break;
            }
        if (best < k) atomicMin(&s_n, best);
    }
    __syncthreads();
    const int n = s_n;
    if (tid == 0) {
        const uint64_t ctr = ((uint64_t)(uint32_t)seq_ids[blockIdx.x] << 32) | (uint64_t)(uint32_t)steps[blockIdx.x];
        const uint64_t r = splitmix64_mix(seed + (ctr + 1) * 0x9E3779B97F4A7C15ull);
        const float u = (float)(uint32_t)(r >> 40) * 0x1p-24f;
        s_target = u * ebuf[n - 1];
        s_pick = n - 1;
    }
    __syncthreads();
    {   // the first i < n with c_i > target (n-1 if rounding leaves none)
        const float target = s_target;
        for (int i = tid; i < n; i += T)
            if (ebuf[i] > target) {
                atomicMin(&s_pick, i);
                break;
            }
    }
    __syncthreads();
    if (tid == 0) tokens[blockIdx.x] = (int32_t)(0xFFFFFFFFu - (uint32_t)sel[s_pick]);
}

}  // namespace det

using namespace det;

extern "C" int det_sample(const float* logits, int B, int V, float temperature, int top_k, float top_p,
                          uint64_t seed, const int32_t* seq_ids, const int32_t* steps, int32_t* tokens,
                          void* stream)
{
    if (!logits || !seq_ids || !steps || !tokens || B < 1 || V < 1) return DET_EINVAL;
    if (!(temperature > 0.0f) || !(top_p > 0.0f) || !(top_p <= 1.0f)) return DET_EINVAL;
    if (top_k < 1 || top_k > kMaxTopK) return DET_ESHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (V <= kSampleThreads * 32)
        hipLaunchKernelGGL(sample_kernel_reg<32>, dim3(B), dim3(kSampleThreads), 0, s, logits, V, temperature, top_k, top_p,
                           seed, seq_ids, steps, tokens);
    else if (V <= kSampleThreads * 64)
        hipLaunchKernelGGL(sample_kernel_reg<64>, dim3(B), dim3(kSampleThreads), 0, s, logits, V, temperature, top_k, top_p,
                           seed, seq_ids, steps, tokens);
    else
        hipLaunchKernelGGL(sample_kernel, dim3(B), dim3(256), 0, s, logits, V, temperature, top_k, top_p, seed, seq_ids,
                           steps, tokens);
    return check_launch();
}
