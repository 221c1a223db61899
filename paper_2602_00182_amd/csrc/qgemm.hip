// Deterministic block-quantized GEMM for gfx950 (the paper's primary kernel family is the quantized
// one, section 6.4; its format is not given, this one is defined here):
//
//   weights      4-bit codes q in -8..7 and a bf16 scale s per 64 consecutive k of a column
//   activations  8-bit codes p in -127..127 and an fp32 scale d per 64 consecutive k of a row
//   C[i][n] = bf16(acc),  acc = 0;  for b ascending:  acc = fma( d[i][b]*s[b][n], float(P), acc ),
//   P = sum over the block of p*q in int32 (exact: v_mfma_i32_16x16x64_i8, one instruction per block)
//
// Every floating-point operation of the definition is an individually rounded IEEE fp32 operation
// in a written order and the contraction is integer, so a CPU reproduces the bytes exactly.
// Batch invariance follows as for the bf16 kernel: an output element's chain never depends on M.
//
// Kernel shape: as the bf16 GEMM (gemm.hip) -- a workgroup owns 16*CB columns and up to 256 rows,
// K in 64-deep stages streamed through an LDS ring by waves that only load -- with two differences.
// Weights arrive packed (544*CB bytes a stage: for each 16-column block, 8 bytes a lane of codes in
// matrix-core operand order, then 16 scales), so a chunk's weights are one contiguous run copied as
// it lies.  And the eight computing waves split the tile by column block first (wave w: column block
// w % CB, row blocks w / CB, w / CB + 8/CB, ...): at small M the work per stage is the unpacking of
// the codes, which a single wave could not do at the rate the weights stream in.  Tiles of at most 8
// rows and 2 column blocks go further and split the stages of a chunk over the waves (run_sp below):
// only the accumulation chain has a defined order, and it keeps it.
#include <type_traits>

#include "common.h"
#include "stream.h"

namespace det {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kQRing = 144;   // KB of LDS ring
constexpr int kQWaves = 8;    // waves that can compute
constexpr int kQLoaders = 4;  // waves that only load

// Columns-per-workgroup factor: the largest of 8, 4, 2, 1 that divides N/16 and leaves at least 160
// workgroups (see gemm_cols_per_block); 1 if there is none.
int qgemm_cols_per_block(int N)
{
    const int nb = N / 16;
    for (int cb = 8; cb > 1; cb >>= 1)
        if (nb % cb == 0 && nb / cb >= 160) return cb;
    return 1;
}

__host__ __device__ constexpr int qstage_w_bytes(int cb) { return 544 * cb; }

// ------------------------------------------------------------------------------------------------
// Weight quantizer + packer: one thread per (block b, column n).
// Packed layout: workgroup slab (16*cb columns) major, then stage; inside a stage, for column block
// j: 64 lanes x 8 bytes at j*512 (lane = 16*g + column%16 holds the codes of k = 16g .. 16g+15 of the
// stage: dword t = 0,1, byte i = 0..3: low nibble = code of k = 16g + 8t + i, high nibble = code of
// k = 16g + 8t + 4 + i, each stored as q + 8); then at 512*cb the scales, 16 bf16 per column block.
// gate_up_f > 0: packed column 2j is logical column j (gate) and 2j+1 is gate_up_f + j (up).
// rope_d > 0: within every head of rope_d columns, packed columns 2i and 2i+1 are the head's logical columns i
// and i + rope_d/2 (a rotation pair).
__global__ __launch_bounds__(256) void quant_pack_w4_kernel(const uint16_t* __restrict__ W, uint8_t* __restrict__ packed,
                                                            int N, int K, int cb, int gate_up_f, int rope_d)
{
    const int nblk = K >> 6;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)nblk * N) return;
    const int n = (int)(idx % N), b = (int)(idx / N);
    int nsrc = gate_up_f > 0 ? ((n & 1) ? gate_up_f + (n >> 1) : (n >> 1)) : n;
    if (rope_d > 0) {
        const int r = n % rope_d;
        nsrc = n - r + (r >> 1) + ((r & 1) ? rope_d >> 1 : 0);
    }
    float w[64];
    float amax = 0.0f;
#pragma unroll
    for (int k = 0; k < 64; ++k) {
        w[k] = bf16_to_f32(W[(size_t)(64 * b + k) * N + nsrc]);
        amax = fmaxf(amax, fabsf(w[k]));
    }
    const uint16_t sb = f32_to_bf16_rne(amax / 7.0f);
    const float sf = bf16_to_f32(sb);
    const int slab = n / (16 * cb), j = (n >> 4) % cb, c = n & 15;
    uint8_t* stage = packed + ((size_t)slab * nblk + b) * qstage_w_bytes(cb);
    uint32_t u[64];
#pragma unroll
    for (int k = 0; k < 64; ++k) {
        int v = 0;
        if (sf != 0.0f) {
            const float r = rintf(w[k] / sf);
            v = r < -8.0f ? -8 : (r > 7.0f ? 7 : (int)r);
        }
        u[k] = (uint32_t)(v + 8);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint32_t dw[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint32_t x = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) x |= (u[16 * g + 8 * t + i] | (u[16 * g + 8 * t + 4 + i] << 4)) << (8 * i);
            dw[t] = x;
        }
        *reinterpret_cast<uint2*>(stage + j * 512 + (16 * g + c) * 8) = make_uint2(dw[0], dw[1]);
    }
    *reinterpret_cast<uint16_t*>(stage + 512 * cb + j * 32 + c * 2) = sb;
}

// Test hook: the packed matrix back to logical codes q [K,N] (int8) and scales s [K/64,N] (bf16).
__global__ __launch_bounds__(256) void quant_unpack_w4_kernel(const uint8_t* __restrict__ packed, int8_t* __restrict__ q,
                                                              uint16_t* __restrict__ s, int N, int K, int cb)
{
    const int nblk = K >> 6;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)nblk * N) return;
    const int n = (int)(idx % N), b = (int)(idx / N);
    const int slab = n / (16 * cb), j = (n >> 4) % cb, c = n & 15;
    const uint8_t* stage = packed + ((size_t)slab * nblk + b) * qstage_w_bytes(cb);
    for (int g = 0; g < 4; ++g) {
        const uint2 d = *reinterpret_cast<const uint2*>(stage + j * 512 + (16 * g + c) * 8);
        const uint32_t dw[2] = {d.x, d.y};
        for (int t = 0; t < 2; ++t)
            for (int i = 0; i < 4; ++i) {
                const uint32_t byte = (dw[t] >> (8 * i)) & 0xFFu;
                q[(size_t)(64 * b + 16 * g + 8 * t + i) * N + n] = (int8_t)((int)(byte & 15u) - 8);
                q[(size_t)(64 * b + 16 * g + 8 * t + 4 + i) * N + n] = (int8_t)((int)(byte >> 4) - 8);
            }
    }
    s[(size_t)b * N + n] = *reinterpret_cast<const uint16_t*>(stage + 512 * cb + j * 32 + c * 2);
}

// Activation quantizer: one wave per (row, 64-k block); grid (blocks/4, M).  p [M,K] int8 row-major;
// d stored block-major, d[b*ldd + i], so that the scales of a tile's rows for one stage are contiguous.
__global__ __launch_bounds__(256) void quant_act_q8_kernel(const uint16_t* __restrict__ A, int lda, int8_t* __restrict__ p,
                                                           float* __restrict__ d, int ldd, int K)
{
    const int i = blockIdx.y, lane = threadIdx.x & 63;
    const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (b >= (K >> 6)) return;
    const float a = bf16_to_f32(A[(size_t)i * lda + 64 * b + lane]);
    float amax = fabsf(a);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    const float df = amax / 127.0f;
    int v = 0;
    if (df != 0.0f) {
        const float r = rintf(a / df);
        v = r < -127.0f ? -127 : (r > 127.0f ? 127 : (int)r);
    }
    p[(size_t)i * K + 64 * b + lane] = (int8_t)v;
    if (lane == 0) d[(size_t)b * ldd + i] = df;
}

// ------------------------------------------------------------------------------------------------
// Schedule of one 256-row tile, worked out on the host (see gemm.hip).
struct qgemm_plan {
    int mrem, RB;
    int SPC;         // stages per chunk
    int slot_bytes;  // bytes of a ring slot
    int nslots, nchunks, last_cnt;
    int tile_bytes;  // bytes of an activation tile: 1024 (16 rows), or 512 / 256 for a single row block of <= 8 / <= 4 rows
    uint32_t inv_4rb;  // floor(2^20/(4*RB))+1
    int nrg;         // row groups in use: min(8/CB, RB)
    int SG;          // stage groups: 8 / (CB * nrg) waves share a (column block, row group) pair, see run_sp
    int res_off;     // SG > 1: byte offset in the ring of the two result buffers
    int ncomp;       // waves that do not load
    int nload;
    uint32_t inv_nload;  // floor(2^20/nload)+1
};

static int q_wrun_bytes(int s_cnt, int cb) { return (s_cnt * qstage_w_bytes(cb) + 1023) & ~1023; }

static int up1k(int n) { return (n + 1023) & ~1023; }

static qgemm_plan make_qgemm_plan(int mrem, int cb, int K)
{
    qgemm_plan t;
    t.mrem = mrem;
    t.RB = (mrem + 15) >> 4;
    t.tile_bytes = t.RB == 1 ? (mrem <= 4 ? 256 : (mrem <= 8 ? 512 : 1024)) : 1024;
    t.inv_4rb = (1u << 20) / (uint32_t)(4 * t.RB) + 1u;
    // bytes of a chunk of spc stages: weight run, activation tiles, activation scales, each rounded up to 1 KB
    auto chunk_bytes = [&](int spc) { return q_wrun_bytes(spc, cb) + up1k(spc * t.RB * t.tile_bytes) + up1k(spc * t.RB * 64); };
    const int nstages = K >> 6;
    const int rg = 8 / cb;
    t.nrg = rg < t.RB ? rg : t.RB;
    // stage-parallel form (see run_sp) where the results stay small enough for chunks of twenty stages and
    // more: at most two column blocks of at most 8 rows
    t.SG = cb <= 2 && t.tile_bytes < 1024 ? 8 / cb : 1;
    t.res_off = 0;
    t.SPC = 1;
    if (t.SG > 1) {
        // four slots and two result buffers of 128 bytes per (stage, column block, row group, row kept)
        const int res_stage = 2 * t.tile_bytes * cb * t.nrg;
        while (4 * chunk_bytes(t.SPC + 1) + 2 * (t.SPC + 1) * res_stage <= kQRing * 1024 && t.SPC < 64) ++t.SPC;
        t.slot_bytes = chunk_bytes(t.SPC);
        t.nslots = 4;
        t.res_off = 4 * t.slot_bytes;
    } else {
        const int third = kQRing * 1024 / 3;  // the most stages whose chunk fits a third of the ring
        while (chunk_bytes(t.SPC + 1) <= third) ++t.SPC;
        t.slot_bytes = chunk_bytes(t.SPC);
        t.nslots = kQRing * 1024 / t.slot_bytes < 4 ? kQRing * 1024 / t.slot_bytes : 4;
    }
    t.nchunks = (nstages + t.SPC - 1) / t.SPC;
    t.last_cnt = nstages - (t.nchunks - 1) * t.SPC;
    // waves that do not load: one per (column block, row group, stage group), plus in the stage-parallel
    // form one wave per pair that only runs the ordered chain
    t.ncomp = cb * t.nrg * t.SG + (t.SG > 1 ? cb * t.nrg : 0);
    t.nload = kQWaves + kQLoaders - t.ncomp;
    t.inv_nload = (1u << 20) / (uint32_t)t.nload + 1u;
    return t;
}

// EPI: the epilogues of the bf16 kernel (plain store, residual add, SwiGLU on gate/up-interleaved columns),
// applied to the accumulator rounded to bf16, so each gives the bytes of the unfused sequence.
template <int CB, int EPI>
__global__ __launch_bounds__(64 * (kQWaves + kQLoaders)) void qgemm_kernel(
    const int8_t* __restrict__ qa, int K, const float* __restrict__ da, int ldd, const uint8_t* __restrict__ wp, void* C,
    int ldc, const uint16_t* R, int ldr, int out_f32, qgemm_plan plan_full, qgemm_plan plan_tail, float* qscales_out,
    gemm_rope_args ra)
{
    __shared__ uint4 ring[kQRing * 64];
    __shared__ float rowmax[EPI == kEpiSwigluQuant ? 8 * 256 : 1];  // row maxima of the eight waves, that epilogue only
    static_assert(EPI != kEpiSwigluQuant || CB == 8, "a 128-column tile holds one 64-output block per row");
    constexpr int RG = 8 / CB;        // row groups: wave w computes column block w % CB for row group w / CB
    constexpr int MAXR = 16 / RG;     // most row blocks a wave can own
    constexpr int WST = qstage_w_bytes(CB);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, lr = lane & 15;
    const int m0 = blockIdx.y * plan_full.mrem;  // full tiles hold plan_full.mrem rows (256 unless the rows are cut, see launch_qgemm)
    const qgemm_plan& tp = blockIdx.y + 1 == gridDim.y ? plan_tail : plan_full;
    const int mrem = tp.mrem, RB = tp.RB, SPC = tp.SPC, nslots = tp.nslots, nchunks = tp.nchunks;
    const int P = nslots - 1;
    const int nstages = K >> 6;
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(lds_char_t*)ring;
    auto chunk_stages = [&](int c) { return c < nchunks - 1 ? SPC : (c == nchunks - 1 ? tp.last_cnt : 0); };
    // LDS layout of a chunk of s_cnt stages: the weight run (s_cnt*WST bytes as they lie in memory,
    // rounded up to 1 KB), then the activation tiles (stage, row block: rows x 64 codes, the four
    // 16-byte pieces of row i swizzled: piece t at slot t ^ ((i/4)%4)), then the activation scales.
    auto wrun = [&](int s_cnt) { return (uint32_t)((s_cnt * WST + 1023) & ~1023); };
    // The activation tiles of a chunk follow its weight run and the activation scales follow the tiles:
    // tile (stage, row block) has TB bytes (16 rows of 64 codes; a single row block of at most 8 or 4
    // rows keeps only 8 or 4), the scales of a stage are 4 bytes for each of the 16*RB rows.
    const int TB = tp.tile_bytes;
    auto abytes_of = [&](int s_cnt) { return (uint32_t)((s_cnt * RB * TB + 1023) & ~1023); };
    auto sbytes_of = [&](int s_cnt) { return (uint32_t)((s_cnt * RB * 64 + 1023) & ~1023); };
    const int lrc = min(lr, (TB >> 6) - 1);  // row of the tile this lane reads (rows past a short tile repeat its last)

    if (wave >= tp.ncomp) {
        // ---------------------------------------------------------------- loading wave
        const int nload = tp.nload, lrank = wave - tp.ncomp;
        const char* wbytes = reinterpret_cast<const char*>(wp) + (size_t)blockIdx.x * nstages * WST;
        const char* abytes = reinterpret_cast<const char*>(qa) + (size_t)m0 * K;
        const char* dbytes = reinterpret_cast<const char*>(da + m0);
        const uint32_t lane16 = (uint32_t)lane * 16u;
        const int lrow = lane >> 2;  // row of this lane inside an activation tile
        const uint32_t a_lane_off = (uint32_t)lrow * (uint32_t)K + 16u * (uint32_t)((lane & 3) ^ ((lane >> 4) & 3));
        auto strided = [&](int n) { return n > lrank ? (int)(((uint32_t)(n - lrank + nload - 1) * tp.inv_nload) >> 20) : 0; };
        auto loads_for = [&](int s_cnt) {
            return strided((int)(wrun(s_cnt) >> 10)) + strided((int)(abytes_of(s_cnt) >> 10)) +
                   strided((int)(sbytes_of(s_cnt) >> 10));
        };
        // short tiles: a load covers 1024/TB stages; lane -> (stage lane/(TB/16), row (lane/4) % (TB/64), piece lane%4)
        const int srow = (lane >> 2) & ((TB >> 6) - 1);
        const int sst = lane / (TB >> 4);
        const uint32_t a_short_off = (uint32_t)srow * (uint32_t)K + 16u * (uint32_t)((lane & 3) ^ ((srow >> 2) & 3)) +
                                     64u * (uint32_t)sst;
        const int loads_full = loads_for(SPC), loads_last = loads_for(tp.last_cnt);
        auto wave_loads = [&](int c) { return c < nchunks - 1 ? loads_full : (c == nchunks - 1 ? loads_last : 0); };

        auto load_chunk = [&](int c, int slot_idx) {
            const int s_cnt = chunk_stages(c);
            if (s_cnt == 0) return;
            const int s0 = c * SPC;
            const uint32_t slot_addr = ring_addr + (uint32_t)slot_idx * (uint32_t)tp.slot_bytes;
            // weight run: 1 KB units of a contiguous byte range; the last unit may be short
            const uint32_t wlen = (uint32_t)(s_cnt * WST);
            const int nwu = (int)(wrun(s_cnt) >> 10);
            const char* wsrc = wbytes + (size_t)s0 * WST;
            // the whole units as one run of loads (three instructions each: the loaders' own instruction
            // stream is on the critical path of small tiles), the short last unit by the wave whose turn it is
            const int nfull = (int)(wlen >> 10);
            dma_run(wsrc, lane16 + (uint32_t)lrank * 1024u, (uint32_t)nload * 1024u, slot_addr + (uint32_t)lrank * 1024u,
                    (uint32_t)nload * 1024u, strided(nfull));
            if (nwu > nfull && nfull - nload * (int)(((uint32_t)nfull * tp.inv_nload) >> 20) == lrank) {
                const uint32_t off = (uint32_t)nfull << 10;
                if (off + lane16 < wlen) dma_block(wsrc + off, lane16, slot_addr + off);
            }
            // activation tiles; rows past M load nothing
            const uint32_t tiles = slot_addr + wrun(s_cnt);
            if (TB == 1024) {  // unit (stage, row block)
                int sl = 0, rb = lrank;
                while (rb >= RB) {
                    rb -= RB;
                    ++sl;
                }
                const int nt = s_cnt * RB;
                for (int u = lrank; u < nt; u += nload) {
                    if (16 * rb + lrow < mrem)
                        dma_block(abytes + (size_t)(16 * rb) * K + ((size_t)(s0 + sl) << 6), a_lane_off,
                                  tiles + ((uint32_t)u << 10));
                    rb += nload;
                    while (rb >= RB) {
                        rb -= RB;
                        ++sl;
                    }
                }
            } else {  // one row block of short tiles: unit = 1024/TB stages
                const int spu = 1024 / TB;
                const int nau = (int)(abytes_of(s_cnt) >> 10);
                for (int u = lrank; u < nau; u += nload)
                    if (srow < mrem && u * spu + sst < s_cnt)
                        dma_block(abytes + ((size_t)(s0 + u * spu) << 6), a_short_off, tiles + ((uint32_t)u << 10));
            }
            // activation scales: 16-byte piece p of the chunk's scale area = rows 4w .. 4w+3 of stage p / (4 RB),
            // w = p % (4 RB)
            const uint32_t scales = tiles + abytes_of(s_cnt);
            const int nsu = (int)(sbytes_of(s_cnt) >> 10);
            for (int u = lrank; u < nsu; u += nload) {
                const uint32_t pce = (uint32_t)(64 * u + lane);
                const uint32_t st = (pce * tp.inv_4rb) >> 20;
                const uint32_t w = pce - st * (uint32_t)(4 * RB);
                if ((int)st < s_cnt && (int)(4 * w) < mrem)
                    dma_block(dbytes + (size_t)s0 * ldd * 4, st * (uint32_t)ldd * 4u + 16u * w, scales + ((uint32_t)u << 10));
            }
        };

        for (int c = 0; c < P; ++c) load_chunk(c, c);
        const int younger_steady = (P - 1) * loads_full;
        int slot_c = 0, slot_new = P;
        for (int c = 0; c < nchunks; ++c) {
            int younger = younger_steady;
            if (c + P > nchunks - 1) {
                younger = 0;
                for (int dd = 1; dd < P; ++dd) younger += wave_loads(c + dd);
            }
            wait_loads_then_barrier(younger);
            load_chunk(c + P, slot_new);
            slot_new = slot_c;
            slot_c = slot_c + 1 == nslots ? 0 : slot_c + 1;
        }
        if (tp.SG > 1) __builtin_amdgcn_s_barrier();  // the barrier after which the last chunk's results are read
        if constexpr (EPI == kEpiSwigluQuant) __builtin_amdgcn_s_barrier();  // the epilogue's exchange of row maxima
        return;
    }

    // -------------------------------------------------------------------- computing wave
    const int nstagew = CB * tp.nrg * tp.SG;  // waves that work on stages; any further non-loading wave runs a chain
    const int pw = wave < nstagew ? wave : wave - nstagew;
    const int j = pw % CB, rg = (pw / CB) % tp.nrg;  // column block and row group of the wave
    const int cnt = (RB - rg + RG - 1) / RG;         // its row blocks: rg, rg + RG, ... (cnt >= 1 here)

    // Stage-parallel form for tiles with fewer row blocks than row groups (M <= 16*(8/CB - 1)): one wave
    // per (column block, row group) would leave most of the compute unit's vector units idle while it
    // works through every stage by itself.  The SG waves of a pair split the stages of a chunk
    // (stage sl -> wave sl % SG); for its stages a wave computes t = d*s and the block's integer
    // product as fp32 (exact) and leaves both in LDS.  After the next barrier the pair's chain wave
    // (a wave with no other work, so that the chain of chunk c runs beside the stage work of chunk
    // c+1) runs acc = fma(t, P, acc) over the chunk's stages in ascending order: the chain, the only
    // part whose order is defined, is the same sequence of operations as in the serial form.
    auto run_sp = [&]() {
        const int SG = tp.SG, npair = CB * tp.nrg;
        const bool chain_wave = wave >= nstagew;
        const int sg = wave / npair, pair = j + CB * rg;
        // results of a stage: for each pair RT = TB/64 rows x 16 columns of t, then of P; lane (g, lr) holds the
        // four columns 4g .. 4g+3 of row lr and takes part if its row is kept
        const int RT = TB >> 6;
        const int res_pair = RT * 128, res_stage = npair * res_pair;
        const bool row_kept = lr < RT;
        char* const resbase = reinterpret_cast<char*>(ring) + tp.res_off;
        const int res_chunk = SPC * res_stage;
        const int res_lane = pair * res_pair + (g * RT + lr) * 16;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        auto chain = [&](int c) {
            const int s_cnt = chunk_stages(c);
            if (!row_kept) return;
            const char* rr = resbase + (c & 1) * res_chunk + res_lane;
            const int stride = res_stage, pf_off = RT * 64;
            // eight stages' operands are read before their (ordered) chain runs, so that one LDS latency is
            // paid per eight stages
            constexpr int W = 8;
            int sl = 0;
            for (; sl + W <= s_cnt; sl += W) {
                float4 t[W], pf[W];
#pragma unroll
                for (int u = 0; u < W; ++u) {
                    t[u] = *reinterpret_cast<const float4*>(rr + u * stride);
                    pf[u] = *reinterpret_cast<const float4*>(rr + u * stride + pf_off);
                }
#pragma unroll
                for (int u = 0; u < W; ++u) {
                    acc[0] = __builtin_fmaf(t[u].x, pf[u].x, acc[0]);
                    acc[1] = __builtin_fmaf(t[u].y, pf[u].y, acc[1]);
                    acc[2] = __builtin_fmaf(t[u].z, pf[u].z, acc[2]);
                    acc[3] = __builtin_fmaf(t[u].w, pf[u].w, acc[3]);
                }
                rr += W * stride;
            }
            for (; sl < s_cnt; ++sl) {
                const float4 t = *reinterpret_cast<const float4*>(rr);
                const float4 pf = *reinterpret_cast<const float4*>(rr + pf_off);
                acc[0] = __builtin_fmaf(t.x, pf.x, acc[0]);
                acc[1] = __builtin_fmaf(t.y, pf.y, acc[1]);
                acc[2] = __builtin_fmaf(t.z, pf.z, acc[2]);
                acc[3] = __builtin_fmaf(t.w, pf.w, acc[3]);
                rr += stride;
            }
        };
        int slot_c = 0;
        for (int c = 0; c < nchunks; ++c) {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (chain_wave) {
                if (c > 0) chain(c - 1);
                continue;
            }
            const int s_cnt = chunk_stages(c);
            const char* slot = reinterpret_cast<const char*>(ring) + (size_t)slot_c * tp.slot_bytes;
            const char* tiles = slot + wrun(s_cnt);
            const char* scales = tiles + abytes_of(s_cnt);
            char* rw = resbase + (c & 1) * res_chunk + res_lane;
            // UU of the wave's stages at a time: all reads and matrix-core instructions first
            auto stages = [&](int sl, auto uu_tag) {
                constexpr int UU = decltype(uu_tag)::value;
                v4i wu[UU], xa[UU];
                uint2 sraw[UU];
                float dv[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const int s = sl + u * SG;
                    const char* wst = slot + s * WST;
                    const uint2 codes = *reinterpret_cast<const uint2*>(wst + j * 512 + lane * 8);
                    sraw[u] = *reinterpret_cast<const uint2*>(wst + 512 * CB + j * 32 + g * 8);
                    xa[u] = *reinterpret_cast<const v4i*>(tiles + (size_t)(s * RB + rg) * TB + 64 * lrc +
                                                          16 * (g ^ ((lrc >> 2) & 3)));
                    dv[u] = *reinterpret_cast<const float*>(scales + (size_t)s * RB * 64 + (16 * rg + lr) * 4);
                    // the stored nibble is q + 8: taken as it is, with -8 * (sum of the block's activation
                    // codes) as the matrix core's starting value, which is the same integer
                    wu[u][0] = (int)(codes.x & 0x0F0F0F0Fu);
                    wu[u][1] = (int)((codes.x >> 4) & 0x0F0F0F0Fu);
                    wu[u][2] = (int)(codes.y & 0x0F0F0F0Fu);
                    wu[u][3] = (int)((codes.y >> 4) & 0x0F0F0F0Fu);
                }
                v4i pr[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const int m8 = (int)0xF8F8F8F8u;
                    const v4i base = __builtin_amdgcn_mfma_i32_16x16x64_i8(v4i{m8, m8, m8, m8}, xa[u], v4i{0, 0, 0, 0}, 0, 0, 0);
                    pr[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wu[u], xa[u], base, 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const int s = sl + u * SG;
                    const float4 t = make_float4(dv[u] * bf16lo_to_f32(sraw[u].x), dv[u] * bf16hi_to_f32(sraw[u].x),
                                                 dv[u] * bf16lo_to_f32(sraw[u].y), dv[u] * bf16hi_to_f32(sraw[u].y));
                    const float4 pf = make_float4((float)pr[u][0], (float)pr[u][1], (float)pr[u][2], (float)pr[u][3]);
                    if (row_kept) {
                        *reinterpret_cast<float4*>(rw + (size_t)s * res_stage) = t;
                        *reinterpret_cast<float4*>(rw + (size_t)s * res_stage + RT * 64) = pf;
                    }
                }
            };
            int sl = sg;
            for (; sl + SG < s_cnt; sl += 2 * SG) stages(sl, std::integral_constant<int, 2>{});
            for (; sl < s_cnt; sl += SG) stages(sl, std::integral_constant<int, 1>{});
            slot_c = slot_c + 1 == nslots ? 0 : slot_c + 1;
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (!chain_wave) return;
        chain(nchunks - 1);
        const int n = blockIdx.x * (16 * CB) + 16 * j + 4 * g;
        const int rowl = 16 * rg + lr;
        if (rowl < mrem) {
            const size_t row = (size_t)(m0 + rowl);
            if constexpr (EPI == kEpiRopeAppend) {
                int p = ra.pos[row];
                p = p < 0 ? 0 : (p >= ra.Lmax ? ra.Lmax - 1 : p);
                gemm_epilogue_rope_append(acc, ra, row, p, ra.slots ? ra.slots[row] : (int)row, n);
            } else {
                gemm_epilogue_store<EPI>(acc, C, ldc, R, ldr, row, n, out_f32);
            }
        }
    };
    if (tp.SG > 1) {
        run_sp();
        return;
    }

    auto run = [&](auto nr_tag) {
        constexpr int NR = decltype(nr_tag)::value;  // cnt rounded up to a power of two; the surplus
                                                     // repeats the last row block and is not stored
        float acc[NR][4];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[r][v] = 0.0f;
        int rbs[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) rbs[r] = rg + RG * (r < cnt ? r : cnt - 1);

        int slot_c = 0;
        for (int c = 0; c < nchunks; ++c) {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const int s_cnt = chunk_stages(c);
            const char* slot = reinterpret_cast<const char*>(ring) + (size_t)slot_c * tp.slot_bytes;
            const char* tiles = slot + wrun(s_cnt);
            const char* scales = tiles + abytes_of(s_cnt);
            // UU stages at a time: all their LDS reads and matrix-core instructions first, so that the
            // latencies overlap, then the scaling chain of each output in ascending stage order
            auto stages = [&](int sl, auto uu_tag) {
                constexpr int UU = decltype(uu_tag)::value;
                constexpr int G = NR < 4 ? NR : 4;  // row blocks at a time
                // With one or two row blocks the wave's time goes into vector instructions, not the matrix
                // core: the stored nibbles q + 8 are then used as they are and the matrix core starts from
                // -8 * (sum of the block's activation codes), one more matrix instruction per row block
                // instead of twelve vector instructions per stage; the integer is the same.
                constexpr bool kBias = NR <= 2;
                auto expand = [](uint32_t x) { return (((x & 0x0F0F0F0Fu) | 0x80808080u) - 0x08080808u) ^ 0x80808080u; };
                v4i wq[UU];
                float sc[UU][4];
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const char* wst = slot + (sl + u) * WST;
                    const uint2 codes = *reinterpret_cast<const uint2*>(wst + j * 512 + lane * 8);
                    const uint2 sraw = *reinterpret_cast<const uint2*>(wst + 512 * CB + j * 32 + g * 8);
                    if constexpr (kBias) {
                        wq[u][0] = (int)(codes.x & 0x0F0F0F0Fu);
                        wq[u][1] = (int)((codes.x >> 4) & 0x0F0F0F0Fu);
                        wq[u][2] = (int)(codes.y & 0x0F0F0F0Fu);
                        wq[u][3] = (int)((codes.y >> 4) & 0x0F0F0F0Fu);
                    } else {
                        // 16 codes -> 16 signed bytes: per byte (u | 0x80) - 8, then the top bit flipped back
                        wq[u][0] = (int)expand(codes.x);
                        wq[u][1] = (int)expand(codes.x >> 4);
                        wq[u][2] = (int)expand(codes.y);
                        wq[u][3] = (int)expand(codes.y >> 4);
                    }
                    sc[u][0] = bf16lo_to_f32(sraw.x);
                    sc[u][1] = bf16hi_to_f32(sraw.x);
                    sc[u][2] = bf16lo_to_f32(sraw.y);
                    sc[u][3] = bf16hi_to_f32(sraw.y);
                }
#pragma unroll
                for (int r0 = 0; r0 < NR; r0 += G) {
                    v4i pr[UU][G];
                    float dv[UU][G];
#pragma unroll
                    for (int u = 0; u < UU; ++u)
#pragma unroll
                        for (int r = 0; r < G; ++r) {
                            const v4i xa = *reinterpret_cast<const v4i*>(tiles + (size_t)((sl + u) * RB + rbs[r0 + r]) * TB +
                                                                         64 * lrc + 16 * (g ^ ((lrc >> 2) & 3)));
                            dv[u][r] = *reinterpret_cast<const float*>(scales + (size_t)(sl + u) * RB * 64 +
                                                                       (16 * rbs[r0 + r] + lr) * 4);
                            if constexpr (kBias) {
                                const int m8 = (int)0xF8F8F8F8u;
                                const v4i base = __builtin_amdgcn_mfma_i32_16x16x64_i8(v4i{m8, m8, m8, m8}, xa, v4i{0, 0, 0, 0}, 0, 0, 0);
                                pr[u][r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wq[u], xa, base, 0, 0, 0);
                            } else {
                                pr[u][r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wq[u], xa, v4i{0, 0, 0, 0}, 0, 0, 0);
                            }
                        }
#pragma unroll
                    for (int u = 0; u < UU; ++u)
#pragma unroll
                        for (int r = 0; r < G; ++r)
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                acc[r0 + r][v] = __builtin_fmaf(dv[u][r] * sc[u][v], (float)pr[u][r][v], acc[r0 + r][v]);
                }
            };
            constexpr int U = NR == 1 ? 4 : (NR == 2 ? 2 : 1);
            int sl = 0;
            for (; sl + U <= s_cnt; sl += U) stages(sl, std::integral_constant<int, U>{});
            for (; sl < s_cnt; ++sl) stages(sl, std::integral_constant<int, 1>{});
            slot_c = slot_c + 1 == nslots ? 0 : slot_c + 1;
        }

        // Lane holds C[row = 16*rb + lr][n0 + 16j + 4g + v], v = 0..3.
        const int n = blockIdx.x * (16 * CB) + 16 * j + 4 * g;
        if constexpr (EPI == kEpiSwigluQuant) {
            // Columns are gate/up pairs: the lane holds outputs 8j + 2g and 8j + 2g + 1 of the tile's 64, the
            // tile row is one quantization block.  Its maximum: the lane's two values, the four lanes
            // of a row (g), then the eight waves (j) through LDS.  Here CB = 8: every wave owns all
            // row blocks (rbs[r] = r) and all of them take part in the barrier.
            float y[NR][2];
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const float g0 = bf16_to_f32(f32_to_bf16_rne(acc[r][0])), u0 = bf16_to_f32(f32_to_bf16_rne(acc[r][1]));
                const float g1 = bf16_to_f32(f32_to_bf16_rne(acc[r][2])), u1 = bf16_to_f32(f32_to_bf16_rne(acc[r][3]));
                y[r][0] = bf16_to_f32(f32_to_bf16_rne(silu_mul(g0, u0)));
                y[r][1] = bf16_to_f32(f32_to_bf16_rne(silu_mul(g1, u1)));
                float mx = fmaxf(fabsf(y[r][0]), fabsf(y[r][1]));
                mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                if (g == 0) rowmax[wave * 256 + 16 * rbs[r] + lr] = mx;
            }
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int rowl = 16 * rbs[r] + lr;
                float amax = rowmax[rowl];
#pragma unroll
                for (int w = 1; w < 8; ++w) amax = fmaxf(amax, rowmax[w * 256 + rowl]);
                const float df = amax / 127.0f;
                uint32_t c2 = 0;
                if (df != 0.0f) {
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const float qv = rintf(y[r][e] / df);
                        const int iv = qv < -127.0f ? -127 : (qv > 127.0f ? 127 : (int)qv);
                        c2 |= (uint32_t)(iv & 0xFF) << (8 * e);
                    }
                }
                if (r < cnt && rowl < mrem) {
                    const size_t row = (size_t)(m0 + rowl);
                    *reinterpret_cast<uint16_t*>(static_cast<int8_t*>(C) + row * ldc + (n >> 1)) = (uint16_t)c2;
                    if (j == 0 && g == 0) qscales_out[(size_t)blockIdx.x * ldr + row] = df;
                }
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int rowl = 16 * rbs[r] + lr;
            if (r < cnt && rowl < mrem) {
                const size_t row = (size_t)(m0 + rowl);
                const float v[4] = {acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
                if constexpr (EPI == kEpiRopeAppend) {
                    int p = ra.pos[row];
                    p = p < 0 ? 0 : (p >= ra.Lmax ? ra.Lmax - 1 : p);
                    gemm_epilogue_rope_append(v, ra, row, p, ra.slots ? ra.slots[row] : (int)row, n);
                } else {
                    gemm_epilogue_store<EPI>(v, C, ldc, R, ldr, row, n, out_f32);
                }
            }
        }
    };
    // the weight codes of a stage are expanded once per wave whatever the number of row blocks
    if (cnt == 1) {
        run(std::integral_constant<int, 1>{});
    } else if (cnt == 2) {
        run(std::integral_constant<int, 2>{});
    } else if (MAXR >= 4 && cnt <= 4) {
        run(std::integral_constant<int, (MAXR >= 4 ? 4 : MAXR)>{});
    } else if (MAXR >= 8 && cnt <= 8) {
        run(std::integral_constant<int, (MAXR >= 8 ? 8 : MAXR)>{});
    } else {
        run(std::integral_constant<int, MAXR>{});
    }
}

static int q_ldd(int M) { return (M + 3) & ~3; }

template <int CB, int EPI>
static void launch_qgemm(const void* qa, const void* da, int ldd, const void* wp, void* C, int ldc, const void* R, int ldr,
                         int M, int N, int K, int out_f32, hipStream_t s, float* qscales_out = nullptr,
                         const gemm_rope_args& ra = gemm_rope_args{})
{
    // Matrices too narrow to give every compute unit a column tile: the rows are cut into as many tiles as
    // fill the chip (a tile's rows are whole 16-row blocks; which tile a row falls in does not touch its
    // arithmetic).
    int tile_rows = 256;
    const int col_tiles = N / (16 * CB), row_blocks = (M + 15) / 16, fit = 256 / col_tiles;
    if (fit >= 2 && row_blocks >= 2) {
        const int row_tiles = row_blocks < fit ? row_blocks : fit;
        const int rows = 16 * ((row_blocks + row_tiles - 1) / row_tiles);
        tile_rows = rows < 256 ? rows : 256;
    }
    dim3 grid(N / (16 * CB), (M + tile_rows - 1) / tile_rows);
    const qgemm_plan full = make_qgemm_plan(tile_rows, CB, K);
    const qgemm_plan tail = make_qgemm_plan(M - tile_rows * ((M - 1) / tile_rows), CB, K);
    hipLaunchKernelGGL((qgemm_kernel<CB, EPI>), grid, dim3(64 * (kQWaves + kQLoaders)), 0, s,
                       static_cast<const int8_t*>(qa), K, static_cast<const float*>(da), ldd, static_cast<const uint8_t*>(wp),
                       C, ldc, static_cast<const uint16_t*>(R), ldr, out_f32, full, tail, qscales_out, ra);
}

// N: columns of the packed matrix (2F for the SwiGLU epilogue).
template <int EPI>
static int qgemm_dispatch(const void* codes, const void* scales, const void* packed_w, void* C, int ldc, const void* R,
                          int ldr, int M, int N, int K, int f32, hipStream_t s, const gemm_rope_args& ra = gemm_rope_args{})
{
    switch (qgemm_cols_per_block(N)) {
        case 1: launch_qgemm<1, EPI>(codes, scales, q_ldd(M), packed_w, C, ldc, R, ldr, M, N, K, f32, s, nullptr, ra); break;
        case 2: launch_qgemm<2, EPI>(codes, scales, q_ldd(M), packed_w, C, ldc, R, ldr, M, N, K, f32, s, nullptr, ra); break;
        case 4: launch_qgemm<4, EPI>(codes, scales, q_ldd(M), packed_w, C, ldc, R, ldr, M, N, K, f32, s, nullptr, ra); break;
        default: launch_qgemm<8, EPI>(codes, scales, q_ldd(M), packed_w, C, ldc, R, ldr, M, N, K, f32, s, nullptr, ra); break;
    }
    return check_launch();
}

static bool qgemm_shape_ok(int N, int K) { return N > 0 && K > 0 && N % 16 == 0 && K % 64 == 0 && K <= (1 << 22); }

}  // namespace det

using namespace det;

extern "C" size_t det_qgemm_packed_w_bytes(int N, int K)
{
    if (!qgemm_shape_ok(N, K)) return 0;
    return (size_t)(N / 16) * (K / 64) * qstage_w_bytes(1);
}

static int quant_pack_impl(const void* B_kn, void* packed, int N, int K, int gate_up_f, void* stream, int rope_d = 0)
{
    if (!B_kn || !packed) return DET_EINVAL;
    if (!qgemm_shape_ok(N, K)) return DET_ESHAPE;
    if (!aligned16(packed)) return DET_EALIGN;
    const size_t total = (size_t)N * (K / 64);
    hipLaunchKernelGGL(quant_pack_w4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(B_kn), static_cast<uint8_t*>(packed), N,
                       K, qgemm_cols_per_block(N), gate_up_f, rope_d);
    return check_launch();
}

extern "C" int det_quant_pack_w4_qkv(const void* B_kn, void* packed, int Hq, int Hkv, int D, int K, void* stream)
{
    if (Hq < 1 || Hkv < 1 || D != 128) return DET_ESHAPE;
    return quant_pack_impl(B_kn, packed, (Hq + 2 * Hkv) * D, K, 0, stream, D);
}

extern "C" int det_quant_pack_w4(const void* B_kn, void* packed, int N, int K, void* stream)
{
    return quant_pack_impl(B_kn, packed, N, K, 0, stream);
}

extern "C" int det_quant_pack_w4_gate_up(const void* B_kn, void* packed, int F, int K, void* stream)
{
    if (F < 1 || F % 8 != 0) return DET_ESHAPE;
    return quant_pack_impl(B_kn, packed, 2 * F, K, F, stream);
}

extern "C" int det_quant_unpack_w4(const void* packed, void* q, void* s, int N, int K, void* stream)
{
    if (!packed || !q || !s) return DET_EINVAL;
    if (!qgemm_shape_ok(N, K)) return DET_ESHAPE;
    const size_t total = (size_t)N * (K / 64);
    hipLaunchKernelGGL(quant_unpack_w4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint8_t*>(packed), static_cast<int8_t*>(q),
                       static_cast<uint16_t*>(s), N, K, qgemm_cols_per_block(N));
    return check_launch();
}

extern "C" size_t det_quant_act_codes_bytes(int M, int K) { return M > 0 && K > 0 ? (size_t)M * K : 0; }
extern "C" size_t det_quant_act_scales_bytes(int M, int K)
{
    return M > 0 && K > 0 && K % 64 == 0 ? (size_t)q_ldd(M) * (K / 64) * sizeof(float) : 0;
}

extern "C" int det_quant_act_q8(const void* A, int lda, void* codes, void* scales, int M, int K, void* stream)
{
    if (!A || !codes || !scales || M < 1) return DET_EINVAL;
    if (K < 64 || K % 64 != 0 || K > (1 << 22) || M > 65535) return DET_ESHAPE;
    if (lda < K) return DET_EINVAL;
    if (!aligned16(codes) || !aligned16(scales)) return DET_EALIGN;
    hipLaunchKernelGGL(quant_act_q8_kernel, dim3((K / 64 + 3) / 4, M), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(A), lda, static_cast<int8_t*>(codes), static_cast<float*>(scales), q_ldd(M),
                       K);
    return check_launch();
}

static int qgemm_args_ok(const void* codes, const void* scales, const void* packed_w, const void* C, int ldc, int M, int N,
                         int ncols_out, int K)
{
    if (!codes || !scales || !packed_w || !C || M < 1) return DET_EINVAL;
    if (!qgemm_shape_ok(N, K)) return DET_ESHAPE;
    if (ldc < ncols_out) return DET_EINVAL;
    if (!aligned16(codes) || !aligned16(scales) || !aligned16(packed_w) || !aligned16(C) || ldc % 4 != 0 || K % 16 != 0)
        return DET_EALIGN;
    return DET_OK;
}

extern "C" int det_qgemm_w4a8(const void* codes, const void* scales, const void* packed_w, void* C, int ldc, int M, int N,
                              int K, int out_dtype, void* stream)
{
    if (out_dtype != DET_BF16 && out_dtype != DET_F32) return DET_EINVAL;
    const int rc = qgemm_args_ok(codes, scales, packed_w, C, ldc, M, N, N, K);
    if (rc != DET_OK) return rc;
    return qgemm_dispatch<kEpiStore>(codes, scales, packed_w, C, ldc, nullptr, 0, M, N, K, out_dtype == DET_F32,
                                     static_cast<hipStream_t>(stream));
}

extern "C" int det_qgemm_w4a8_residual(const void* codes, const void* scales, const void* packed_w, const void* R, int ldr,
                                       void* C, int ldc, int M, int N, int K, void* stream)
{
    const int rc = qgemm_args_ok(codes, scales, packed_w, C, ldc, M, N, N, K);
    if (rc != DET_OK) return rc;
    if (!R || ldr < N) return DET_EINVAL;
    if (!aligned16(R) || ldr % 4 != 0) return DET_EALIGN;
    return qgemm_dispatch<kEpiResidual>(codes, scales, packed_w, C, ldc, R, ldr, M, N, K, 0,
                                        static_cast<hipStream_t>(stream));
}

extern "C" int det_qgemm_w4a8_swiglu(const void* codes, const void* scales, const void* packed_gate_up, void* Y, int ldy,
                                     int M, int F, int K, void* stream)
{
    if (F < 1 || F % 8 != 0 || F > (1 << 29)) return DET_ESHAPE;
    const int rc = qgemm_args_ok(codes, scales, packed_gate_up, Y, ldy, M, 2 * F, F, K);
    if (rc != DET_OK) return rc;
    return qgemm_dispatch<kEpiSwiglu>(codes, scales, packed_gate_up, Y, ldy, nullptr, 0, M, 2 * F, K, 0,
                                      static_cast<hipStream_t>(stream));
}

extern "C" int det_qgemm_w4a8_swiglu_quant_supported(int F, int K)
{
    return F >= 8 && F % 8 == 0 && F <= (1 << 29) && qgemm_shape_ok(2 * F, K) && qgemm_cols_per_block(2 * F) == 8;
}

extern "C" int det_qgemm_w4a8_swiglu_quant(const void* codes, const void* scales, const void* packed_gate_up, void* codes_out,
                                           void* scales_out, int M, int F, int K, void* stream)
{
    if (!scales_out) return DET_EINVAL;
    if (F < 1 || F % 64 != 0 || F > (1 << 29)) return DET_ESHAPE;
    const int rc = qgemm_args_ok(codes, scales, packed_gate_up, codes_out, F, M, 2 * F, F, K);
    if (rc != DET_OK) return rc;
    if (!det_qgemm_w4a8_swiglu_quant_supported(F, K)) return DET_ESHAPE;
    if (!aligned16(scales_out)) return DET_EALIGN;
    // the kernel's ldr argument carries the row stride of the output scales
    launch_qgemm<8, kEpiSwigluQuant>(codes, scales, q_ldd(M), packed_gate_up, codes_out, F, nullptr, q_ldd(M), M, 2 * F, K, 0,
                                     static_cast<hipStream_t>(stream), static_cast<float*>(scales_out));
    return check_launch();
}

extern "C" int det_qgemm_w4a8_qkv_rope_append(const void* codes, const void* scales, const void* packed_qkv, void* qbuf,
                                              void* kcache, void* vcache, const int32_t* positions, const int32_t* slots,
                                              const float* rope_cos, const float* rope_sin, int M, int Hq, int Hkv, int D,
                                              int Lmax, int K, void* stream)
{
    if (Hq < 1 || Hkv < 1 || D != 128 || Lmax < 1) return DET_ESHAPE;
    const int N = (Hq + 2 * Hkv) * D;
    const int rc = qgemm_args_ok(codes, scales, packed_qkv, qbuf, 4, M, N, 4, K);
    if (rc != DET_OK) return rc;
    if (!kcache || !vcache || !positions || !rope_cos || !rope_sin) return DET_EINVAL;
    if (!aligned16(kcache) || !aligned16(vcache) || !aligned16(rope_cos) || !aligned16(rope_sin)) return DET_EALIGN;
    gemm_rope_args ra;
    ra.pos = positions;
    ra.slots = slots;
    ra.cos_t = rope_cos;
    ra.sin_t = rope_sin;
    ra.qbuf = static_cast<uint16_t*>(qbuf);
    ra.kcache = static_cast<uint16_t*>(kcache);
    ra.vcache = static_cast<uint16_t*>(vcache);
    ra.Hq = Hq, ra.Hkv = Hkv, ra.Lmax = Lmax;
    return qgemm_dispatch<kEpiRopeAppend>(codes, scales, packed_qkv, qbuf, 4, nullptr, 0, M, N, K, 0,
                                          static_cast<hipStream_t>(stream), ra);
}
