// Deterministic bf16 GEMM for gfx950: C[M,N] = A[M,K] * B[K,N], fp32 accumulation on the matrix
// cores, one accumulator chain per output element in ascending K (the paper's section 6.5:
// invariant 1, fixed workgroup -> tile mapping with no inter-workgroup communication; invariant 3,
// no atomics).
//
// Shape of the kernel
//   * A workgroup (NW = 4 or 8 wavefronts) owns BN = 16*CB output columns and up to 256 rows; grid.x = N/BN,
//     grid.y = ceil(M/256).  CB and the LDS ring size are functions of N alone, so the
//     configuration never depends on M.
//   * K is cut into 64-deep stages.  Operands travel as 1 KB blocks, each already in the operand
//     order of v_mfma_f32_16x16x32_bf16 (lane l holds 8 consecutive k of row/column l%16, k group
//     l/16): a stage has 2*CB weight blocks and 2*RB activation blocks, RB = number of 16-row
//     blocks of the tile that hold data.  M decides RB and nothing else.
//   * Stages are grouped into chunks and streamed through a ring of up to 4 LDS slots with the
//     LDS-DMA form of the global load (global_load_lds_dwordx4: no staging registers, one wave
//     instruction fills one 1 KB block).  Up to 3 chunks are in flight while the waves compute on
//     a fourth; a wave waits only for its own loads of the oldest chunk (s_waitcnt vmcnt(n) with n
//     = its loads of the younger chunks), then the workgroup barrier makes the chunk visible.
//     The weight slab of a workgroup is one contiguous run of the packed matrix.
//   * Weights are the ROW operand of the MFMA (16 output columns of C), activations its COLUMN
//     operand (16 rows of C): a lane then holds 4 consecutive columns of one row of C and the
//     store is one 8- or 16-byte write.  Rows of the operand are independent in the matrix core,
//     so rows past M may hold anything: their lanes load nothing and their outputs are never
//     stored.
//   * 16-row blocks are dealt round-robin to the waves (block rb -> wave rb % NW).
//
// K order: matrix-core step t (t = 0 .. K/32-1, ascending) takes k in [32t, 32t+32); inside a step
// lane group g supplies k = 32t + 8g + e, e = 0..7.
#include <type_traits>

#include "common.h"

namespace det {

typedef __attribute__((address_space(3))) char lds_char_t;

// Columns-per-workgroup factor: the largest CB in 1..8 that divides N/16 and still leaves at least
// 192 workgroups across N (three quarters of the 256 compute units); 1 if there is none.
int gemm_cols_per_block(int N)
{
    const int nb = N / 16;
    int best = 1;
    for (int cb = 1; cb <= 8; ++cb)
        if (nb % cb == 0 && nb / cb >= 192) best = cb;
    return best;
}

// LDS ring size in 1 KB blocks.  144 KB by default (one workgroup per compute unit).  When N
// yields at least 1.5 workgroups per compute unit and CB is small, the ring is two stages of the
// largest tile, so that two workgroups share a compute unit's 160 KB of LDS.
// Wavefronts per workgroup: 4 for narrow tiles, 8 (two per SIMD, so that one can issue loads while
// the other feeds the matrix core) for wide ones, which measured faster from 64 rows up.
__host__ __device__ constexpr int gemm_waves(int cb) { return cb >= 4 ? 8 : 4; }

constexpr int kRingBig = 144;
__host__ __device__ constexpr int gemm_small_ring_blocks(int cb) { return 4 * (cb + 16); }
bool gemm_small_ring(int N)
{
    const int cb = gemm_cols_per_block(N);
    return cb <= 3 && N / (16 * cb) >= 384;
}

// One wave instruction: 64 lanes x 16 bytes from global memory straight into the 1 KB LDS block at
// byte address lds_addr (wave-uniform); lane l lands at lds_addr + 16 l.  Written as assembly so
// that the completion wait below can name a count instead of draining every load in flight.
__device__ __forceinline__ void dma_block(const void* gsrc, uint32_t lds_addr)
{
    uint32_t saved_m0;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %2, off\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved_m0)
        : "s"(lds_addr), "v"(gsrc)
        : "memory");
}

// Waits until at most n of this wave's loads are outstanding (the counter holds 0..63; anything
// above falls back to waiting for all of them), then the workgroup barrier.
#define DET_WB(n) \
    case n: asm volatile("s_waitcnt vmcnt(" #n ")\n\ts_barrier" ::: "memory"); break;
__device__ __forceinline__ void wait_loads_then_barrier(int n)
{
    switch (n) {
        DET_WB(1) DET_WB(2) DET_WB(3) DET_WB(4) DET_WB(5) DET_WB(6) DET_WB(7) DET_WB(8)
        DET_WB(9) DET_WB(10) DET_WB(11) DET_WB(12) DET_WB(13) DET_WB(14) DET_WB(15) DET_WB(16)
        DET_WB(17) DET_WB(18) DET_WB(19) DET_WB(20) DET_WB(21) DET_WB(22) DET_WB(23) DET_WB(24)
        DET_WB(25) DET_WB(26) DET_WB(27) DET_WB(28) DET_WB(29) DET_WB(30) DET_WB(31) DET_WB(32)
        DET_WB(33) DET_WB(34) DET_WB(35) DET_WB(36) DET_WB(37) DET_WB(38) DET_WB(39) DET_WB(40)
        DET_WB(41) DET_WB(42) DET_WB(43) DET_WB(44) DET_WB(45) DET_WB(46) DET_WB(47) DET_WB(48)
        DET_WB(49) DET_WB(50) DET_WB(51) DET_WB(52) DET_WB(53) DET_WB(54) DET_WB(55) DET_WB(56)
        DET_WB(57) DET_WB(58) DET_WB(59) DET_WB(60) DET_WB(61) DET_WB(62) DET_WB(63)
        default: asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory"); break;
    }
}
#undef DET_WB

// Epilogues.  kEpiStore: C = bf16(acc) or fp32 acc.  kEpiResidual: C = bf16(fp32(bf16(acc)) + fp32(R)),
// the bytes of the plain GEMM followed by the residual add.  kEpiSwiglu: the weight columns are packed
// gate_j, up_j interleaved, and Y[j] = bf16( silu(bf16(acc_gate_j)) * bf16(acc_up_j) ), the bytes of the
// plain GEMM followed by the SwiGLU step.  C (and R) may alias nothing the kernel reads except that C
// may be R itself: an output element is read and written by the same lane only.
constexpr int kEpiStore = 0, kEpiResidual = 1, kEpiSwiglu = 2;

__device__ __forceinline__ float silu_mul(float gate, float up)
{
    const float den = 1.0f + det_expf(-gate);
    const float sg = gate / den;
    return sg * up;
}

template <int CB, int RINGB, int EPI, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_kernel(const uint16_t* __restrict__ A, int lda,
                                                   const uint4* __restrict__ Bp, void* C, int ldc,
                                                   const uint16_t* R, int ldr, int M, int K, int out_f32)
{
    static_assert(RINGB >= 4 * (CB + 16), "the ring must hold two stages of the largest tile");
    __shared__ uint4 ring[RINGB * 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;   // k group of the lane
    const int lr = lane & 15;  // row of A / column-in-block of the weights
    const int m0 = blockIdx.y * 256;
    const int mrem = min(M - m0, 256);
    const int RB = (mrem + 15) >> 4;                 // 16-row blocks holding data
    const int nA = 2 * RB;                           // activation blocks per stage
    const int nb = 2 * CB + nA;                      // 1 KB blocks per stage
    const int SPC = max(1, (RINGB / 3) / nb);        // stages per chunk: three chunks fill the ring
    const int slot_blocks = SPC * nb;                // blocks per ring slot
    const int nslots = min(4, RINGB / slot_blocks);  // >= 2 by the static_assert
    const int P = nslots - 1;                        // chunks in flight
    const int nstages = K >> 6;
    const int nchunks = (nstages + SPC - 1) / SPC;
    const uint4* __restrict__ bsrc = Bp + (size_t)blockIdx.x * nstages * (2 * CB * 64);
    const uint16_t* __restrict__ abase = A + (size_t)m0 * lda;
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(lds_char_t*)ring;

    // Row blocks of this wave: rb = wave + 4r, active while rb < RB.
    const int nrb = RB > wave ? (RB - wave + NW - 1) / NW : 0;

    // Which waves issue loads: while fewer than NW row blocks hold data, the waves without a row block
    // (waves RB..NW-1) do all the loading and the computing waves only compute; from NW row blocks on,
    // every wave does both.  lrank < 0: this wave issues no loads.
    const int nload = RB >= NW ? NW : NW - RB;
    const int lrank = RB >= NW ? wave : wave - RB;

    auto chunk_stages = [&](int c) { return c < nchunks ? min(SPC, nstages - c * SPC) : 0; };
    // Loads this wave issues for a chunk of s_cnt stages: weight blocks q = lrank, lrank+nload, ...
    // below s_cnt*2*CB, one load each; activation pairs pp = lrank, lrank+nload, ... below s_cnt*RB,
    // two loads each (a pair always has a live lane: row 16*rb exists for rb < RB).
    // For narrow tiles, from NW row blocks on (every wave loads and computes) the split is per stage
    // instead: wave w takes the weight blocks f = w, w+NW, ... below 2*CB of each stage and the pairs of its own row
    // blocks, and issues them between the matrix-core steps of the stage it is computing.
    const bool interleaved = CB <= 3 && RB >= NW;  // wide tiles measured faster with burst issue
    const int nbw = 2 * CB > wave ? (2 * CB - wave + NW - 1) / NW : 0;  // weight blocks per stage, this wave
    auto strided = [&](int n) { return n > lrank ? (n - lrank + nload - 1) / nload : 0; };
    auto loads_for = [&](int s_cnt) {
        if (interleaved) return s_cnt * (nbw + 2 * nrb);
        return lrank < 0 ? 0 : strided(s_cnt * 2 * CB) + 2 * strided(s_cnt * RB);
    };
    // every chunk but the last has SPC stages, so two values cover all chunks
    const int loads_full = loads_for(SPC);
    const int loads_last = loads_for(nstages - (nchunks - 1) * SPC);
    auto wave_loads = [&](int c) { return c < nchunks - 1 ? loads_full : (c == nchunks - 1 ? loads_last : 0); };

    // LDS layout of a chunk of s_cnt stages inside its slot: first the s_cnt*2*CB weight blocks in
    // the order they lie in the packed matrix (stage, column block, step), then the s_cnt*2*RB
    // activation blocks (stage, row block, step).
    const uint4* wsrc = bsrc + lane;                          // this lane's slot in weight block 0
    const uint16_t* asrc = abase + (size_t)lr * lda + 8 * g;  // row lr, k group g of stage 0
    // One stage's loads of this wave under the per-stage split (stage sl of a chunk starting at
    // global stage s0 whose slot starts at slot_addr and holds nw weight blocks).
    auto issue_weight = [&](int s0, int sl, int t, uint32_t slot_addr) {
        const int f = wave + NW * t;
        if (f < 2 * CB)
            dma_block(wsrc + ((size_t)(s0 + sl) * (2 * CB) + f) * 64, slot_addr + (uint32_t)(sl * 2 * CB + f) * 1024u);
    };
    auto issue_pair = [&](int s0, int sl, int r, uint32_t slot_addr, int nw) {
        const int rb = wave + NW * r;
        if (16 * rb + lr < mrem) {  // lanes of rows past M load nothing: their LDS bytes are never used
            const uint16_t* src_a = asrc + (size_t)(16 * rb) * lda + ((s0 + sl) << 6);
            const uint32_t d = slot_addr + (uint32_t)nw * 1024u + (uint32_t)(sl * RB + rb) * 2048u;
            dma_block(src_a, d);
            dma_block(src_a + 32, d + 1024u);
        }
    };
    auto load_chunk = [&](int c, int slot_idx) {
        const int s_cnt = chunk_stages(c);
        if (s_cnt == 0 || lrank < 0) return;
        const int s0 = c * SPC;
        const int nw = s_cnt * 2 * CB;
        const uint32_t slot_addr = ring_addr + (uint32_t)(slot_idx * slot_blocks) * 1024u;
        if (interleaved) {  // burst form of the per-stage split (used to prime the ring)
            for (int sl = 0; sl < s_cnt; ++sl) {
                for (int t = 0; t < nbw; ++t) issue_weight(s0, sl, t, slot_addr);
                for (int r = 0; r < nrb; ++r) issue_pair(s0, sl, r, slot_addr, nw);
            }
            return;
        }
        const uint4* src = wsrc + ((size_t)s0 * (2 * CB) + lrank) * 64;
        uint32_t dst = slot_addr + (uint32_t)lrank * 1024u;
        for (int q = lrank; q < nw; q += nload) {
            dma_block(src, dst);
            src += nload * 64;
            dst += (uint32_t)nload * 1024u;
        }
        // activation blocks in pairs (both steps of one row block), pair pp = sl*RB + rb, so that the
        // two 64-byte halves of each 128-byte line of A are fetched back to back
        uint32_t adst = slot_addr + (uint32_t)nw * 1024u + (uint32_t)lrank * 2048u;
        int sl = 0, rb = lrank;
        while (rb >= RB) {
            rb -= RB;
            ++sl;
        }
        const int npair = s_cnt * RB;
        for (int pp = lrank; pp < npair; pp += nload) {
            if (16 * rb + lr < mrem) {  // lanes of rows past M load nothing: their LDS bytes are never used
                const uint16_t* src_a = asrc + (size_t)(16 * rb) * lda + ((s0 + sl) << 6);
                dma_block(src_a, adst);
                dma_block(src_a + 32, adst + 1024u);
            }
            adst += (uint32_t)nload * 2048u;
            rb += nload;
            while (rb >= RB) {
                rb -= RB;
                ++sl;
            }
        }
    };

    // The whole K loop and the store, for a wave with NRB row blocks (0: a wave that only loads).
    // NRB is a compile-time constant inside so that the loop bodies have no branches.
    auto run = [&](auto nrb_tag) {
        constexpr int NRB = decltype(nrb_tag)::value;
        constexpr int NR = NRB > 0 ? NRB : 1;
        struct Frags {
            bf16x8 wf[CB][2];
            bf16x8 xf[NR][2];
        };
        f32x4 acc[NR][CB];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int j = 0; j < CB; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

        // cn / slot_n: the chunk whose loads are issued between the steps (interleaved regime), -1: none
        auto compute_chunk = [&](int c, int slot_idx, int cn, int slot_n) {
            const int s_cnt = chunk_stages(c);
            const int sn_cnt = cn >= 0 ? chunk_stages(cn) : 0;
            const int sn0 = cn * SPC;
            const int nwn = sn_cnt * 2 * CB;
            const uint32_t slot_n_addr = ring_addr + (uint32_t)(slot_n * slot_blocks) * 1024u;
            const uint4* slot = ring + (size_t)(slot_idx * slot_blocks) * 64;
            const uint4* wbase = slot + lane;
            const uint4* abuf = slot + s_cnt * (2 * CB * 64) + 2 * wave * 64 + lane;
            auto read_stage = [&](Frags& fr, int sl) {
                const uint4* wp = wbase + sl * (2 * CB * 64);
#pragma unroll
                for (int j = 0; j < CB; ++j) {
                    fr.wf[j][0] = __builtin_bit_cast(bf16x8, wp[(2 * j) * 64]);
                    fr.wf[j][1] = __builtin_bit_cast(bf16x8, wp[(2 * j + 1) * 64]);
                }
                const uint4* ap = abuf + sl * nA * 64;
#pragma unroll
                for (int r = 0; r < NRB; ++r) {
                    fr.xf[r][0] = __builtin_bit_cast(bf16x8, ap[(2 * NW * r) * 64]);
                    fr.xf[r][1] = __builtin_bit_cast(bf16x8, ap[(2 * NW * r + 1) * 64]);
                }
                __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the steps they feed
            };
            // Steps of stage sl.  In the interleaved regime the loads of stage sl of chunk cn go out
            // between the groups of steps (pairs after the i = 0 groups, weight blocks after the i = 1
            // groups), so that address generation overlaps the matrix-core pipe.
            constexpr int NBW = (2 * CB + NW - 1) / NW;  // most weight blocks per stage any wave takes
            auto mfma_stage = [&](const Frags& fr, int sl) {
                const bool ld = sl < sn_cnt;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int r = 0; r < NRB; ++r) {
#pragma unroll
                        for (int j = 0; j < CB; ++j)
                            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr.wf[j][i], fr.xf[r][i], acc[r][j], 0, 0, 0);
                        if (ld) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (i == 0) {
                                issue_pair(sn0, sl, r, slot_n_addr, nwn);
                            } else {
                                issue_weight(sn0, sl, r, slot_n_addr);
                                if (r == NRB - 1) {
#pragma unroll
                                    for (int t = NRB; t < NBW; ++t) issue_weight(sn0, sl, t, slot_n_addr);
                                }
                            }
                        }
                    }
                __builtin_amdgcn_sched_barrier(0);
            };
            // Stages in ascending order, software pipelined: the LDS reads of stage s+D-1 are issued
            // before the steps of stage s (D = 4 for small tiles, whose steps are too few to cover the
            // LDS latency, else 2).  Reads past the last stage are redirected to the last stage: in
            // bounds and unused, which keeps the loop body free of branches.
            constexpr int D = (CB * NRB >= 4) ? 2 : 4;
            Frags f[D];
            const int last = s_cnt - 1;
#pragma unroll
            for (int d = 0; d < D - 1; ++d) read_stage(f[d], min(d, last));
            for (int sl = 0; sl < s_cnt; sl += D) {
#pragma unroll
                for (int u = 0; u < D; ++u) {
                    if (sl + u >= s_cnt) return;
                    read_stage(f[(u + D - 1) % D], min(sl + u + D - 1, last));
                    mfma_stage(f[u], sl + u);
                }
            }
        };

        for (int c = 0; c < P; ++c) load_chunk(c, c);
        int slot_c = 0;    // slot of chunk c
        int slot_new = P;  // slot of chunk c+P (the slot chunk c-1 used: nslots = P+1)
        for (int c = 0; c < nchunks; ++c) {
            // Loads issued after chunk c's: chunks c+1 .. c+P-1.  Once chunk c has landed here and
            // the barrier is passed, it has landed for every wave, and every wave is done with chunk
            // c-1, whose slot is the one chunk c+P goes into.
            int younger = 0;
            for (int d = 1; d < P; ++d) younger += wave_loads(c + d);
            wait_loads_then_barrier(younger);
            if constexpr (NRB > 0) {
                if (interleaved) {
                    compute_chunk(c, slot_c, c + P, slot_new);
                } else {
                    load_chunk(c + P, slot_new);
                    compute_chunk(c, slot_c, -1, 0);
                }
            } else {
                load_chunk(c + P, slot_new);
            }
            slot_new = slot_c;
            slot_c = slot_c + 1 == nslots ? 0 : slot_c + 1;
        }

        // Lane holds C[row = 16*rb + lr][n0 + 16j + 4g + v], v = 0..3.
        const int n0 = blockIdx.x * (16 * CB);
#pragma unroll
        for (int r = 0; r < NRB; ++r) {
            const int rowl = 16 * (wave + NW * r) + lr;
            if (rowl < mrem) {
                const size_t row = (size_t)(m0 + rowl);
#pragma unroll
                for (int j = 0; j < CB; ++j) {
                    const int n = n0 + 16 * j + 4 * g;
                    const f32x4 v = acc[r][j];
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
            }
        }
    };
    if constexpr (NW == 8) {
        switch (nrb) {
            case 0: run(std::integral_constant<int, 0>{}); break;
            case 1: run(std::integral_constant<int, 1>{}); break;
            default: run(std::integral_constant<int, 2>{}); break;
        }
    } else {
        switch (nrb) {
            case 0: run(std::integral_constant<int, 0>{}); break;
            case 1: run(std::integral_constant<int, 1>{}); break;
            case 2: run(std::integral_constant<int, 2>{}); break;
            case 3: run(std::integral_constant<int, 3>{}); break;
            default: run(std::integral_constant<int, 4>{}); break;
        }
    }
}

// One thread per 16 bytes of the packed matrix: gathers 8 K-consecutive elements of one column.
// gate_up_f > 0: packed column 2j is logical column j (gate) and 2j+1 is gate_up_f + j (up).
__global__ __launch_bounds__(256) void gemm_pack_kernel(const uint16_t* __restrict__ Bkn,
                                                        uint4* __restrict__ Bp, int N, int K, int cb,
                                                        int gate_up_f)
{
    const size_t total = (size_t)N * K / 8;
    const int stage_u4 = cb * 2 * 64;
    const int nstages = K >> 6;
    for (size_t u = (size_t)blockIdx.x * 256 + threadIdx.x; u < total; u += (size_t)gridDim.x * 256) {
        const size_t per_tile = (size_t)nstages * stage_u4;
        const int tile = (int)(u / per_tile);
        const int rem = (int)(u % per_tile);
        const int st = rem / stage_u4;
        const int f = rem % stage_u4;
        const int j = f >> 7;
        const int i = (f >> 6) & 1;
        const int lane = f & 63;
        int n = tile * 16 * cb + 16 * j + (lane & 15);
        if (gate_up_f > 0) n = (n & 1) ? gate_up_f + (n >> 1) : (n >> 1);
        const int k0 = 64 * st + 32 * i + 8 * (lane >> 4);
        uint16_t e[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) e[t] = Bkn[(size_t)(k0 + t) * N + n];
        uint4 o;
        o.x = e[0] | ((uint32_t)e[1] << 16);
        o.y = e[2] | ((uint32_t)e[3] << 16);
        o.z = e[4] | ((uint32_t)e[5] << 16);
        o.w = e[6] | ((uint32_t)e[7] << 16);
        Bp[u] = o;
    }
}

template <int CB, int RINGB, int EPI, int NW>
static void launch_gemm(const void* A, int lda, const void* Bp, void* C, int ldc, const void* R, int ldr, int M,
                        int N, int K, int out_f32, hipStream_t s)
{
    dim3 grid(N / (16 * CB), (M + 255) / 256);
    hipLaunchKernelGGL((gemm_kernel<CB, RINGB, EPI, NW>), grid, dim3(64 * NW), 0, s, static_cast<const uint16_t*>(A), lda,
                       static_cast<const uint4*>(Bp), C, ldc, static_cast<const uint16_t*>(R), ldr, M, K,
                       out_f32);
}

// Picks the kernel configuration from N alone and launches it.
template <int EPI>
static int gemm_dispatch(const void* A, int lda, const void* Bp, void* C, int ldc, const void* R, int ldr, int M,
                         int N, int K, int f32, hipStream_t s)
{
    const int cb = gemm_cols_per_block(N);
    const bool small = gemm_small_ring(N);
#define DET_GEMM_CASE(CBV)                                                                                  \
    case CBV:                                                                                               \
        if constexpr (CBV <= 3) {                                                                           \
            if (small) {                                                                                    \
                launch_gemm<CBV, gemm_small_ring_blocks(CBV), EPI, gemm_waves(CBV)>(A, lda, Bp, C, ldc, R, ldr, M, N, K, f32, s); \
                break;                                                                                      \
            }                                                                                               \
        }                                                                                                   \
        launch_gemm<CBV, kRingBig, EPI, gemm_waves(CBV)>(A, lda, Bp, C, ldc, R, ldr, M, N, K, f32, s);                       \
        break;
    switch (cb) {
        DET_GEMM_CASE(1)
        DET_GEMM_CASE(2)
        DET_GEMM_CASE(3)
        DET_GEMM_CASE(4)
        DET_GEMM_CASE(5)
        DET_GEMM_CASE(6)
        DET_GEMM_CASE(7)
        default:
            launch_gemm<8, kRingBig, EPI, gemm_waves(8)>(A, lda, Bp, C, ldc, R, ldr, M, N, K, f32, s);
            break;
    }
#undef DET_GEMM_CASE
    return check_launch();
}

static bool gemm_shape_ok(int N, int K) { return N > 0 && K > 0 && N % 16 == 0 && K % 64 == 0; }

}  // namespace det

using namespace det;

extern "C" size_t det_gemm_packed_b_bytes(int N, int K)
{
    if (!gemm_shape_ok(N, K)) return 0;
    return (size_t)2 * N * K;
}

static int pack_impl(const void* B_kn, void* B_packed, int N, int K, int gate_up_f, void* stream)
{
    if (!B_kn || !B_packed) return DET_EINVAL;
    if (!gemm_shape_ok(N, K)) return DET_ESHAPE;
    if (!aligned16(B_kn) || !aligned16(B_packed)) return DET_EALIGN;
    const size_t total = (size_t)N * K / 8;
    const int blocks = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL(gemm_pack_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(B_kn), static_cast<uint4*>(B_packed), N, K,
                       gemm_cols_per_block(N), gate_up_f);
    return check_launch();
}

extern "C" int det_gemm_pack_b(const void* B_kn, void* B_packed, int N, int K, void* stream)
{
    return pack_impl(B_kn, B_packed, N, K, 0, stream);
}

extern "C" int det_gemm_pack_gate_up(const void* B_kn, void* B_packed, int F, int K, void* stream)
{
    if (F < 1 || F % 8 != 0) return DET_ESHAPE;
    return pack_impl(B_kn, B_packed, 2 * F, K, F, stream);
}

static int gemm_args_ok(const void* A, int lda, const void* Bp, const void* C, int ldc, int M, int N, int K)
{
    if (!A || !Bp || !C || M < 1) return DET_EINVAL;
    if (!gemm_shape_ok(N, K)) return DET_ESHAPE;
    if (lda < K) return DET_EINVAL;
    if (!aligned16(A) || !aligned16(Bp) || !aligned16(C) || lda % 8 != 0 || ldc % 4 != 0) return DET_EALIGN;
    return DET_OK;
}

extern "C" int det_gemm_bf16(const void* A, int lda, const void* B_packed, void* C, int ldc, int M, int N,
                             int K, int out_dtype, void* stream)
{
    if (out_dtype != DET_BF16 && out_dtype != DET_F32) return DET_EINVAL;
    const int rc = gemm_args_ok(A, lda, B_packed, C, ldc, M, N, K);
    if (rc != DET_OK) return rc;
    if (ldc < N) return DET_EINVAL;
    return gemm_dispatch<kEpiStore>(A, lda, B_packed, C, ldc, nullptr, 0, M, N, K, out_dtype == DET_F32,
                                    static_cast<hipStream_t>(stream));
}

extern "C" int det_gemm_bf16_residual(const void* A, int lda, const void* B_packed, const void* R, int ldr,
                                      void* C, int ldc, int M, int N, int K, void* stream)
{
    const int rc = gemm_args_ok(A, lda, B_packed, C, ldc, M, N, K);
    if (rc != DET_OK) return rc;
    if (!R || ldc < N || ldr < N) return DET_EINVAL;
    if (!aligned16(R) || ldr % 4 != 0) return DET_EALIGN;
    return gemm_dispatch<kEpiResidual>(A, lda, B_packed, C, ldc, R, ldr, M, N, K, 0,
                                       static_cast<hipStream_t>(stream));
}

extern "C" int det_gemm_swiglu_bf16(const void* A, int lda, const void* B_gate_up, void* Y, int ldy, int M,
                                    int F, int K, void* stream)
{
    if (F < 1 || F % 8 != 0) return DET_ESHAPE;
    const int rc = gemm_args_ok(A, lda, B_gate_up, Y, ldy, M, 2 * F, K);
    if (rc != DET_OK) return rc;
    if (ldy < F) return DET_EINVAL;
    return gemm_dispatch<kEpiSwiglu>(A, lda, B_gate_up, Y, ldy, nullptr, 0, M, 2 * F, K, 0,
                                     static_cast<hipStream_t>(stream));
}
