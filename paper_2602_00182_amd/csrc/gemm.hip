// Deterministic bf16 GEMM for gfx950: C[M,N] = A[M,K] * B[K,N], fp32 accumulation on the matrix
// cores, one accumulator chain per output element in ascending K (the paper's section 6.5:
// invariant 1, fixed workgroup -> tile mapping with no inter-workgroup communication; invariant 3,
// no atomics).
//
// Shape of the kernel
//   * A workgroup owns BN = 16*CB output columns and up to 256 rows; grid.x = N/BN, grid.y =
//     ceil(M/256).  It has NW (4 or 8) wavefronts that can compute plus NL (2 or 4) that only load.
//     The packing (CB), the matrix-core shape and the K order are functions of N alone.  The tile a
//     launch cuts C into also looks at M (gemm_dispatch: narrow matrices cut their rows so that every
//     compute unit gets a workgroup, tall launches of narrow packings take 64- or 128-column tiles
//     over several slabs).  The tiling decides which workgroup and wave computes an element, never
//     the element's arithmetic, so its bytes are the same whichever ran.
//   * K is cut into 64-deep stages.  Operands travel as 1 KB blocks.  A weight block is already in
//     the operand order of v_mfma_f32_16x16x32_bf16 (lane l holds 8 consecutive k of column l%16, k
//     group l/16); an activation block is 8 rows x 64 k as they lie in A (whole 128-byte lines),
//     swizzled in LDS so that the operand reads are conflict free.  A stage has 2*CB weight blocks
//     and one activation block per 8 rows that hold data.  M decides the number of row blocks and
//     which waves compute, nothing else.
//   * Stages are grouped into chunks and streamed through a ring of up to 4 LDS slots with the
//     LDS-DMA form of the global load (global_load_lds_dwordx4: no staging registers, one wave
//     instruction fills one 1 KB block).  Up to 3 chunks are in flight while the computing waves
//     work on a fourth; a loading wave waits only for its own loads of the oldest chunk (s_waitcnt
//     vmcnt(n) with n = its loads of the younger chunks), then the workgroup barrier makes the chunk
//     visible.  The weight slab of a workgroup is one contiguous run of the packed matrix.
//   * 16-row blocks are dealt round-robin to the waves 0..NW-1 (block rb -> wave rb % NW).  A wave
//     with a row block only computes; every other wave only loads.  What bounds a tall tile is the
//     compute unit's memory pipe (about 25 bytes a clock into LDS for data that hits in L2, and
//     every load, hit or miss, completes in issue order), so the load queue must never run dry: a
//     wave that both loads and computes either blocks on a full queue with matrix-core work
//     unissued or computes while the queue drains.
//   * Weights are the ROW operand of the MFMA (16 output columns of C), activations its COLUMN
//     operand (16 rows of C): a lane then holds 4 consecutive columns of one row of C and the
//     store is one 8- or 16-byte write.  Rows of the operand are independent in the matrix core,
//     so rows past M may hold anything: their lanes load nothing and their outputs are never
//     stored.
//   * Fused forms of the same kernel, each giving the bytes of the unfused sequence: epilogues on the
//     accumulator rounded to bf16 (residual add, SwiGLU on gate/up-interleaved columns, rotation and cache
//     append on pair-interleaved query/key/value columns), and, up to four rows, the RMSNorm of the rows
//     computed by the workgroup itself in front of the K loop (template parameter NORM).
//
// K order: matrix-core step t (t = 0 .. K/32-1, ascending) takes k in [32t, 32t+32); inside a step
// lane group g supplies k = 32t + 8g + e, e = 0..7.
#include <type_traits>
#include <utility>

#include "common.h"
#include "stream.h"

namespace det {


// Columns-per-workgroup factor: the largest CB in 1..8 that divides N/16 and still leaves at least
// 160 workgroups across N; 1 if there is none.  160 compute units pulling weights keep HBM busy, and
// anything between 257 and 383 narrower tiles would run as a full round of workgroups plus a thin one
// (N = 11264: 176 tiles of 64 columns take 11.1 us at M = 1, 352 tiles of 32 columns 14.8 us).
int gemm_cols_per_block(int N)
{
    const int nb = N / 16;
    int best = 1;
    for (int cb = 1; cb <= 8; ++cb)
        if (nb % cb == 0 && nb / cb >= 160) best = cb;
    return best;
}

// LDS ring size in 1 KB blocks.  144 KB by default (one workgroup per compute unit).  When N
// yields at least 1.5 workgroups per compute unit and CB is small, the ring is two stages of the
// largest tile, so that two workgroups share a compute unit's 160 KB of LDS.
// Wavefronts per workgroup: 4 for narrow tiles, 8 (two per SIMD, so that one can issue loads while
// the other feeds the matrix core) for wide ones, which measured faster from 64 rows up.
__host__ __device__ constexpr int gemm_waves(int cb) { return cb >= 4 ? 8 : 4; }
// Wavefronts that never compute and only issue loads (on top of those above): one per SIMD for wide tiles.
__host__ __device__ constexpr int gemm_loader_waves(int cb, bool small_ring) { return small_ring ? 2 : 4; }

constexpr int kRingBig = 144;
__host__ __device__ constexpr int gemm_small_ring_blocks(int cb) { return 4 * (cb + 16); }
bool gemm_small_ring(int N)
{
    const int cb = gemm_cols_per_block(N);
    return cb <= 3 && N / (16 * cb) >= 384;
}


// LDS reads the compiler does not see.  Its own bookkeeping of the LDS counter waits for every read in
// flight before the first use of any of them once reads cross a loop back edge; written by hand, the
// wait before a matrix-core step can leave the reads of the following steps in flight.
//
// To the compiler the destination of such a read holds its value the moment the instruction is issued.
// Two rules follow, and every read in this file obeys both:
//   * the value is first used through tie(), an (empty) instruction placed after the wait that covers the
//     read, so that no use can be scheduled above the wait;
//   * EVERY read is tied that way, also one whose value is never fed to the matrix core.  A destination
//     that is dead right after the read is a free register to the compiler, which may then park an
//     address or a loop variable in it while the read is still in flight, and the returning data lands
//     on top of that value.  (Seen as rare wrong tiles when other kernels kept the compute unit's LDS
//     busy: the late return overwrote the address of the next chunk's first reads, which then read out
//     of range, i.e. zeros.)
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr)
{
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N>
__device__ __forceinline__ void wait_lds_reads()
{
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
template <class T>
__device__ __forceinline__ void tie(T& v)
{
    asm volatile("" : "+v"(v));
}
// Operands of one step: weight blocks 2 KB apart from waddr + WOFF (a constant of the instruction),
// activation tiles NW*2 KB apart from aaddr.
template <int NW, int WOFF, class Frags, int... J, int... Q>
__device__ __forceinline__ void read_frags_at(Frags& fr, uint32_t waddr, uint32_t aaddr, std::integer_sequence<int, J...>,
                                              std::integer_sequence<int, Q...>)
{
    ((fr.wf[J] = lds_read_b128<WOFF + J * 2048>(waddr)), ...);
    ((fr.xf[Q] = lds_read_b128<Q * NW * 2048>(aaddr)), ...);
}
template <int NW, class Frags, int... J, int... Q>
__device__ __forceinline__ void read_frags(Frags& fr, uint32_t waddr, uint32_t aaddr, std::integer_sequence<int, J...> w,
                                           std::integer_sequence<int, Q...> x)
{
    read_frags_at<NW, 0>(fr, waddr, aaddr, w, x);
}
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>), .., f(integral_constant<int, N-1>): a loop whose index is a constant in the body
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}
// Steps the operand reads of a small tile run ahead of the matrix core (see the kernel), by operand reads a step
__host__ __device__ constexpr int gemm_steps_ahead(int reads)
{
    return 15 / reads >= 7 ? 7 : (15 / reads >= 5 ? 5 : (15 / reads >= 3 ? 3 : 1));
}
template <class Frags, int... J, int... Q>
__device__ __forceinline__ void tie_frags(Frags& fr, std::integer_sequence<int, J...>, std::integer_sequence<int, Q...>)
{
    (tie(fr.wf[J]), ...);
    (tie(fr.xf[Q]), ...);
}

// Schedule of one 256-row tile: a function of the tile's row count, the kernel configuration and K,
// worked out on the host (the kernel's own prologue is on the critical path of a launch that lasts
// ten microseconds, and integer division is slow on the device).
struct gemm_tile_plan {
    int mrem;         // rows of the tile that hold data
    int RB, HB;       // 16-row blocks and 8-row half blocks that hold data
    int SPC;          // stages per chunk: three chunks fill the ring
    int slot_blocks;  // 1 KB blocks per ring slot
    int nslots;       // ring slots in use, 2..4
    int nchunks;
    int last_cnt;     // stages of the last chunk
    int nload;        // waves that load
    uint32_t inv_nload, inv_hb;  // floor(2^20/d)+1: n/d = (n * inv) >> 20, exact for the small n used here
};

// a_res: the activations do not travel through the ring (the kernel that normalizes its rows itself keeps them
// resident in the first K/64 blocks of its LDS): a stage is its weight blocks only, the ring is what is left,
// and only the NL waves that never compute load.
static gemm_tile_plan make_tile_plan(int mrem, int cb, int ringb, int nw, int nl, int K, bool a_res = false)
{
    gemm_tile_plan t;
    t.mrem = mrem;
    t.RB = (mrem + 15) >> 4;
    t.HB = (mrem + 7) >> 3;
    if (a_res) ringb -= K >> 6;
    const int nb = 2 * cb + (a_res ? 0 : 2 * t.RB);
    t.SPC = (ringb / 3) / nb > 1 ? (ringb / 3) / nb : 1;
    {
        // Small tiles run their operand reads in groups of stages (see the kernel's small-tile pipeline): a
        // chunk that is a whole number of groups takes the short loop.  Sized for the wave with the most row
        // blocks; data movement only.
        const int nrb0 = (t.RB + nw - 1) / nw;
        if (cb * nrb0 < 6) {
            const int gs = (gemm_steps_ahead(cb + nrb0) + 1) / 2;
            if (t.SPC >= 2 * gs) t.SPC -= t.SPC % gs;  // never gives up more than a third of a chunk
        }
    }
    t.slot_blocks = t.SPC * nb;
    t.nslots = ringb / t.slot_blocks < 4 ? ringb / t.slot_blocks : 4;
    const int nstages = K >> 6;
    t.nchunks = (nstages + t.SPC - 1) / t.SPC;
    t.last_cnt = nstages - (t.nchunks - 1) * t.SPC;
    t.nload = a_res ? nl : nw + nl - (t.RB < nw ? t.RB : nw);
    t.inv_nload = (1u << 20) / (uint32_t)t.nload + 1u;
    t.inv_hb = (1u << 20) / (uint32_t)t.HB + 1u;
    return t;
}

// Most loads one loading wave can have outstanding under a plan: its share of the nslots-1 chunks in flight
// (2*cb weight blocks and HB half blocks a stage, each kind dealt round-robin).  Must stay below the load
// counter's "do not wait" value (see wait_loads_then_barrier).
static bool plan_fits_load_counter(const gemm_tile_plan& t, int cb)
{
    const int per_chunk = (t.SPC * 2 * cb + t.nload - 1) / t.nload + t.SPC * ((t.HB + t.nload - 1) / t.nload) + 1;
    return t.nslots >= 2 && (t.nslots - 1) * per_chunk <= 62;
}

// PCB: column blocks per slab of the packed weights.  PCB == CB: the workgroup's weights are one slab.
// PCB < CB (tall launches of narrow matrices, see gemm_dispatch): the workgroup owns CB/PCB adjacent
// slabs of a matrix packed for narrower tiles, and its rows are a tile of plan_full.mrem rows.
//
// NORM: the rows of A are raw activations and the operand is their RMSNorm with the weight vector R and
// epsilon eps (the bytes det_rmsnorm would write, computed by the same routines in the same order).  Only for
// tiles of at most 4 rows and K <= 4096: the waves 0 .. NW-1 normalize the rows (256 threads a row, as the
// RMSNorm kernel has them) straight into LDS, where they stay for the whole K range in the first K/64
// blocks, one 8-row half block a stage; the ring behind them carries weights only, loaded by the NL waves
// that never compute, which start streaming before the rows are read.
template <int CB, int RINGB, int EPI, int NW, int NL, int PCB, bool NORM>
__global__ __launch_bounds__(64 * (NW + NL)) void gemm_kernel(const uint16_t* __restrict__ A, int lda,
                                                          const uint4* __restrict__ Bp, void* C, int ldc,
                                                          const uint16_t* R, int ldr, int K, int out_f32,
                                                          gemm_tile_plan plan_full, gemm_tile_plan plan_tail,
                                                          gemm_rope_args ra, float eps)
{
    static_assert(!NORM || (PCB == CB && NW % 4 == 0), "the normalizing form: one slab, whole teams of four waves");
    static_assert(RINGB >= 4 * (CB + 16), "the ring must hold two stages of the largest tile");
    static_assert(NL >= 1, "a tile of NW row blocks or more needs waves that only load");
    static_assert(CB % PCB == 0 && (PCB == CB || ((CB & (CB - 1)) == 0 && (PCB & (PCB - 1)) == 0)), "slab split by shifts");
    __shared__ uint4 ring[RINGB * 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;   // k group of the lane
    const int lr = lane & 15;  // row of A / column-in-block of the weights
    const int m0 = blockIdx.y * plan_full.mrem;  // full tiles are plan_full.mrem rows high (256 unless PCB < CB)
    const gemm_tile_plan& tp = blockIdx.y + 1 == gridDim.y ? plan_tail : plan_full;
    const int mrem = tp.mrem;
    const int RB = tp.RB;    // 16-row blocks holding data
    const int HB = tp.HB;    // 8-row half blocks holding data (one load each per stage)
    const int nA = 2 * RB;   // activation blocks per stage
    const int SPC = tp.SPC;  // stages per chunk
    const int slot_blocks = tp.slot_blocks;
    const int nslots = tp.nslots;  // >= 2 by the static_assert
    const int P = nslots - 1;      // chunks in flight
    const int nstages = K >> 6;
    const int nchunks = tp.nchunks;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_char_t*)ring;
    const uint32_t ring_addr = lds_base + (NORM ? (uint32_t)nstages * 1024u : 0u);  // behind the resident activations
    auto chunk_stages = [&](int c) { return c < nchunks - 1 ? SPC : (c == nchunks - 1 ? tp.last_cnt : 0); };

    // Roles.  Row block rb belongs to wave rb % NW (waves 0 .. NW-1); a wave with a row block only
    // computes, every other wave (waves min(RB,NW) .. NW+NL-1) only loads.  A load instruction blocks
    // its wave until the address unit accepts it, so a wave that issued a chunk's loads could not feed
    // the matrix core meanwhile, and one that computed first would leave the load queue empty
    // meanwhile; with the roles in different waves the loads of a chunk go out the moment its ring slot
    // is free and the compute units' memory pipe, which bounds tall tiles, never idles.
    // One barrier per chunk in both roles: passing barrier c means chunk c has landed for everyone
    // and everyone is done reading chunk c-1.
    const int ncomp = min(RB, NW);
    const int nrb = wave < ncomp ? (int)((unsigned)(RB - wave + NW - 1) / (unsigned)NW) : 0;

    // NORM: waves 0 .. NW-1 normalize the tile's rows into LDS.  A team of four waves is the 256 threads of
    // the RMSNorm kernel: thread t of the team owns the vectors t, t + 256 of a row, the wave sums go
    // through LDS and are combined as (q0+q2)+(q1+q3).  Team i takes the rows i, i + NW/4, ...  All loads are
    // issued before the first sum so that the rows cost one round trip.  Two barriers in here: the loads are
    // issued, and the hand-over of the wave sums; the rows themselves are published by the barrier that opens
    // chunk 0.
    __shared__ float norm_part[NORM ? 32 : 1];
    auto normalize_rows = [&]() {
        constexpr int NT = NW / 4;   // teams
        constexpr int RPT = 4 / NT;  // rows a team can own (the tile has at most four)
        const int team = wave >> 2, vt = tid & 255, nvec = K >> 3;
        const uint4* wn4 = reinterpret_cast<const uint4*>(R);
        uint4 wv[2], xv[RPT][2];
        float part[RPT];
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (vt + 256 * i < nvec) wv[i] = wn4[vt + 256 * i];
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int row = team + NT * q;
            if (row < mrem) {
                const uint4* xr = reinterpret_cast<const uint4*>(A + (size_t)(m0 + row) * lda);
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    if (vt + 256 * i < nvec) xv[q][i] = xr[vt + 256 * i];
            }
        }
        // The rows' loads are in the memory pipe: only now may the loading waves start the weight stream.  The pipe
        // returns loads in issue order, and a row load queued behind the first chunks of weights would wait
        // for all of them.
        asm volatile("s_barrier" ::: "memory");
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int row = team + NT * q;
            part[q] = 0.0f;
            if (row < mrem) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    if (vt + 256 * i < nvec) part[q] = rms_fold(xv[q][i], part[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const float w = wave_tree_sum(part[q]);
            if (lane == 0) norm_part[(team + NT * q) * 4 + (wave & 3)] = w;
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int row = team + NT * q;
            if (row < mrem) {
                const float* s4 = norm_part + row * 4;
                const float a = s4[0] + s4[2];
                const float b = s4[1] + s4[3];
                const float r = rms_scale(a + b, K, eps);
                const int z = ((row >> 1) & 3) << 1;  // the swizzle of the activation tiles (see above)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int v = vt + 256 * i;
                    if (v < nvec) ring[(v >> 3) * 64 + row * 8 + ((v & 7) ^ z)] = rms_apply(xv[q][i], wv[i], r);
                }
            }
        }
    };

    // LDS layout of a chunk of s_cnt stages inside its slot: first the s_cnt*2*CB weight blocks in
    // the order they lie in the packed matrix (stage, column block, step), then s_cnt*RB activation
    // tiles of 2 KB (stage, row block), each 16 rows x 64 k.
    //
    // Activation tile: two half blocks of 8 rows, one load instruction each; lane l of the load takes
    // 16 bytes of row l/8, so a quarter wave covers two whole 128-byte lines of A (the memory pipe
    // handles a quarter wave at a time, and sixteen lanes on sixteen different lines cost it nearly
    // twice the time).  The row sits at 128*(row%8) inside its half block with its eight 16-byte
    // pieces XOR-swizzled: piece p (k = 8p .. 8p+7 of the stage) lies at slot p ^ z(row),
    // z(row) = 2*((row/2)%4) + row/8, which spreads the sixteen rows a quarter wave reads for one
    // matrix-core step (same piece of rows 0..15) over all sixteen 16-byte bank groups.

    if (nrb == 0) {
        if constexpr (NORM) {
            if (wave < NW) {  // normalizes, then only keeps the barrier count
                normalize_rows();
                for (int c = 0; c < nchunks; ++c) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                return;
            }
        }
        // ---------------------------------------------------------------- loading wave
        const int nload = tp.nload;  // = NW + NL - ncomp (NORM: NL)
        const int lrank = NORM ? wave - NW : wave - ncomp;
        // first slab of this workgroup (a slab holds nstages stages of 2*PCB blocks)
        const char* wbytes = reinterpret_cast<const char*>(Bp + (size_t)blockIdx.x * (CB / PCB) * nstages * (2 * PCB * 64));
        const char* abytes = reinterpret_cast<const char*>(A + (size_t)m0 * lda);
        const size_t half_bytes = (size_t)lda * 16;  // 8 rows of A
        const uint32_t w_lane_off = (uint32_t)lane * 16u;
        const int lrow = lane >> 3;  // row of this lane inside a half block
        const uint32_t zl = (uint32_t)(((lane >> 4) & 3) << 1);
        const uint32_t a_lane_off0 = (uint32_t)lrow * (uint32_t)lda * 2u + 16u * ((uint32_t)(lane & 7) ^ zl);
        const uint32_t a_lane_off1 = (uint32_t)lrow * (uint32_t)lda * 2u + 16u * ((uint32_t)(lane & 7) ^ (zl | 1u));
        const uint32_t a_lane_off_mine = (lrank & 1) ? a_lane_off1 : a_lane_off0;
        // Split of a chunk's loads over the loading waves.  Weight blocks: q = lrank, lrank+nload, ...
        // below s_cnt*2*CB.  Half blocks: if every half block is whole and there are at least nload of
        // them, hb = lrank, lrank+nload, ... below HB in every stage (short loop: the loaders'
        // instruction count per load matters for tall tiles); else unit pp = sl*HB + hb = lrank,
        // lrank+nload, ... below s_cnt*HB.  A half block that holds data always has a live lane.
        const bool stage_split = (mrem & 7) == 0 && HB >= nload;
        auto strided = [&](int n) { return n > lrank ? (int)(((uint32_t)(n - lrank + nload - 1) * tp.inv_nload) >> 20) : 0; };
        // With the weights in several slabs (PCB < CB) the split is by position inside a stage instead:
        // u = lrank, lrank+nload, ... below 2*CB, the same for every stage, since block u of successive
        // stages is evenly spaced both in its slab and in LDS.
        const int nw_stage = strided(2 * CB);
        auto loads_for = [&](int s_cnt) {
            return (PCB == CB ? strided(s_cnt * 2 * CB) : s_cnt * nw_stage) +
                   (NORM ? 0 : (stage_split ? s_cnt * strided(HB) : strided(s_cnt * HB)));
        };
        // every chunk but the last has SPC stages, so two values cover all chunks
        const int loads_full = loads_for(SPC);
        const int loads_last = loads_for(tp.last_cnt);
        auto wave_loads = [&](int c) { return c < nchunks - 1 ? loads_full : (c == nchunks - 1 ? loads_last : 0); };
        const int nw_full = strided(SPC * 2 * CB);  // weight blocks of a chunk, this wave
        const int nw_last = strided(tp.last_cnt * 2 * CB);
        const int nh_stage = strided(HB);  // half blocks of a stage, this wave, under the stage split
        const int first_sl = (int)(((uint32_t)lrank * tp.inv_hb) >> 20);  // lrank / HB: first unit of a chunk under the unit split
        const int first_hb = lrank - first_sl * HB;

        auto load_chunk = [&](int c, int slot_idx) {
            const int s_cnt = chunk_stages(c);
            if (s_cnt == 0) return;
            const int s0 = c * SPC;
            const int nw = s_cnt * 2 * CB;
            const uint32_t slot_addr = ring_addr + (uint32_t)(slot_idx * slot_blocks) * 1024u;
            if constexpr (PCB == CB) {
                dma_run(wbytes, w_lane_off + (uint32_t)(s0 * (2 * CB) + lrank) * 1024u, (uint32_t)nload * 1024u,
                        slot_addr + (uint32_t)lrank * 1024u, (uint32_t)nload * 1024u, s_cnt == SPC ? nw_full : nw_last);
            } else {
                // block u of a stage = block u % 2PCB of that stage in slab u / 2PCB
                for (int u = lrank; u < 2 * CB; u += nload) {
                    const int j2 = u / (2 * PCB), t = u % (2 * PCB);
                    dma_run(wbytes + (size_t)j2 * nstages * (2 * PCB * 1024),
                            w_lane_off + (uint32_t)(s0 * (2 * PCB) + t) * 1024u, (uint32_t)(2 * PCB) * 1024u,
                            slot_addr + (uint32_t)u * 1024u, (uint32_t)(2 * CB) * 1024u, s_cnt);
                }
            }
            if constexpr (NORM) return;  // the activations are resident
            // Half block hb of stage sl comes from abytes + hb*half_bytes + 128*(s0+sl) and goes to block
            // 2*RB*sl + hb of the tile area; both are walked with running addresses.
            if (stage_split && (nload & 1) == 0) {  // all of this wave's half blocks have the parity of its rank
                uint32_t off = a_lane_off_mine + (uint32_t)lrank * (uint32_t)half_bytes + ((uint32_t)s0 << 7);
                uint32_t adst = slot_addr + (uint32_t)(nw + lrank) * 1024u;
                for (int sl = 0; sl < s_cnt; ++sl) {
                    dma_run(abytes, off, (uint32_t)nload * (uint32_t)half_bytes, adst, (uint32_t)nload * 1024u, nh_stage);
                    off += 128;
                    adst += (uint32_t)(2 * RB) * 1024u;
                }
                return;
            }
            if (stage_split) {
                const char* src0 = abytes + (size_t)lrank * half_bytes + ((size_t)s0 << 7);
                uint32_t dst0 = slot_addr + (uint32_t)(nw + lrank) * 1024u;
                for (int sl = 0; sl < s_cnt; ++sl) {
                    const char* asrc = src0;
                    uint32_t adst = dst0;
                    for (int hb = lrank; hb < HB; hb += nload) {
                        dma_block(asrc, (hb & 1) ? a_lane_off1 : a_lane_off0, adst);
                        asrc += (size_t)nload * half_bytes;
                        adst += (uint32_t)nload * 1024u;
                    }
                    src0 += 128;
                    dst0 += (uint32_t)(2 * RB) * 1024u;
                }
                return;
            }
            if (HB == 1) {  // at most 8 rows: one half block a stage, stages lrank, lrank+nload, ...
                if (lrow < mrem)
                    dma_run(abytes, a_lane_off0 + ((uint32_t)(s0 + lrank) << 7), (uint32_t)nload << 7,
                            slot_addr + (uint32_t)(nw + lrank * 2 * RB) * 1024u, (uint32_t)(nload * 2 * RB) * 1024u,
                            strided(s_cnt));
                return;
            }
            const int nhalf = s_cnt * HB;
            int hb = first_hb;
            const char* asrc = abytes + (size_t)hb * half_bytes + ((size_t)(s0 + first_sl) << 7);
            uint32_t adst = slot_addr + (uint32_t)(nw + first_sl * 2 * RB + hb) * 1024u;
            for (int pp = lrank; pp < nhalf; pp += nload) {
                // rows past M load nothing: their LDS bytes feed only outputs that are never stored
                if (8 * hb + lrow < mrem) dma_block(asrc, (hb & 1) ? a_lane_off1 : a_lane_off0, adst);
                hb += nload;
                asrc += (size_t)nload * half_bytes;
                adst += (uint32_t)nload * 1024u;
                while (hb >= HB) {  // next stage
                    hb -= HB;
                    asrc += 128 - (ptrdiff_t)((size_t)HB * half_bytes);
                    adst += (uint32_t)(2 * RB - HB) * 1024u;
                }
            }
        };

        if constexpr (NORM) asm volatile("s_barrier" ::: "memory");  // the rows' loads are issued (see normalize_rows)
        for (int c = 0; c < P; ++c) load_chunk(c, c);
        if constexpr (NORM) asm volatile("s_barrier" ::: "memory");  // the hand-over of the wave sums in normalize_rows
        const int younger_steady = (P - 1) * loads_full;  // while chunks c+1 .. c+P-1 are all full ones
        int slot_c = 0;    // slot of chunk c
        int slot_new = P;  // slot of chunk c+P (the slot chunk c-1 used: nslots = P+1)
        for (int c = 0; c < nchunks; ++c) {
            // Loads issued after chunk c's: chunks c+1 .. c+P-1.  Once chunk c has landed here and the
            // barrier is passed, it has landed for every loader, and every computing wave is done with
            // chunk c-1, whose slot is the one chunk c+P goes into.
            int younger = younger_steady;
            if (c + P > nchunks - 1) {  // the last chunks: fewer and shorter chunks behind chunk c
                younger = 0;
                for (int d = 1; d < P; ++d) younger += wave_loads(c + d);
            }
            wait_loads_then_barrier(younger);
            load_chunk(c + P, slot_new);
            slot_new = slot_c;
            slot_c = slot_c + 1 == nslots ? 0 : slot_c + 1;
        }
        return;
    }

    // -------------------------------------------------------------------- computing wave
    // NRB (row blocks of the wave) is a compile-time constant inside so that the loop bodies have no
    // branches.
    auto run = [&](auto nrb_tag) {
        constexpr int NRB = decltype(nrb_tag)::value;
        struct Frags {  // operands of one matrix-core step
            bf16x8 wf[CB];
            bf16x8 xf[NRB];
        };
        f32x4 acc[NRB][CB];
#pragma unroll
        for (int r = 0; r < NRB; ++r)
#pragma unroll
            for (int j = 0; j < CB; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

        // this lane's two pieces (k group g of step 0 and of step 1) of row lr in the tile of row block `wave`
        const int zr = (((lr >> 1) & 3) << 1) | (lr >> 3);
        const int a_lane = 2 * wave * 64 + 64 * (lr >> 3) + 8 * (lr & 7);
        const int a0_off = a_lane + (g ^ zr), a1_off = a_lane + ((g ^ zr) ^ 4);
        auto mm = [&](const Frags& fr) {
#pragma unroll
            for (int r = 0; r < NRB; ++r)
#pragma unroll
                for (int j = 0; j < CB; ++j)
                    acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr.wf[j], fr.xf[r], acc[r][j], 0, 0, 0);
            // The matrix-core instructions have no side effects the compiler must order, so it may sink them
            // below the reads that follow, which reuse the registers of `fr`: it would then rename those
            // registers and copy them around, and a copy of a register whose read is still in flight copies
            // stale data.  Tying the accumulators here (an empty instruction that "uses" them) pins the
            // instructions above it, in order, before every later read.
#pragma unroll
            for (int r = 0; r < NRB; ++r)
#pragma unroll
                for (int j = 0; j < CB; ++j) tie(acc[r][j]);
            __builtin_amdgcn_sched_barrier(0);
        };
        // all of this wave's LDS reads have returned, then the barrier that opens the next chunk
        auto open_chunk = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
        if constexpr (NORM) normalize_rows();

        if constexpr (CB * NRB >= 6) {
            // One two-deep pipeline over the whole K range: the operands of a step are read while the step
            // before it is in the matrix core, also across a chunk boundary (a chunk is a single stage for the
            // tallest tiles), so that no LDS latency is exposed.  The barrier that opens chunk c+1 therefore
            // sits before the last step of chunk c; the wave has issued, and waited for, all its reads of
            // chunk c-1 by then, which is what the loaders rely on.
            using wseq = std::make_integer_sequence<int, CB>;
            using xseq = std::make_integer_sequence<int, NRB>;
            static_assert(CB + NRB <= 14, "outstanding LDS reads must stay below the counter's no-wait value");
            Frags f0, f1;
            int slot_c = 0;
            int s_cnt = chunk_stages(0);
            open_chunk();
            uint32_t wa = ring_addr + (uint32_t)lane * 16u;                 // weight block 0 of the stage, this lane
            uint32_t xa = NORM ? lds_base : ring_addr + (uint32_t)(s_cnt * 2 * CB) * 1024u;  // activation tiles of the stage
            const uint32_t a_step = NORM ? 1024u : (uint32_t)nA * 1024u;
            const uint32_t x0 = (uint32_t)a0_off * 16u, x1 = (uint32_t)a1_off * 16u;
            read_frags<NW>(f0, wa, xa + x0, wseq{}, xseq{});
            for (int c = 0; c < nchunks; ++c) {
                int next_cnt = 0;
                for (int sl = 0; sl < s_cnt; ++sl) {
                    wait_lds_reads<0>();
                    tie_frags(f0, wseq{}, xseq{});
                    read_frags<NW>(f1, wa + 1024u, xa + x1, wseq{}, xseq{});
                    mm(f0);
                    wait_lds_reads<0>();
                    tie_frags(f1, wseq{}, xseq{});
                    if (sl + 1 < s_cnt) {
                        wa += (uint32_t)(2 * CB) * 1024u;
                        xa += a_step;
                        read_frags<NW>(f0, wa, xa + x0, wseq{}, xseq{});
                    } else if (c + 1 < nchunks) {
                        open_chunk();
                        slot_c = slot_c + 1 == nslots ? 0 : slot_c + 1;
                        next_cnt = chunk_stages(c + 1);
                        wa = ring_addr + (uint32_t)(slot_c * slot_blocks) * 1024u + (uint32_t)lane * 16u;
                        xa = NORM ? xa + 1024u : ring_addr + (uint32_t)(slot_c * slot_blocks + next_cnt * 2 * CB) * 1024u;
                        read_frags<NW>(f0, wa, xa + x0, wseq{}, xseq{});
                    }
                    mm(f1);
                }
                s_cnt = next_cnt;
            }
        } else {
            // Small tiles: a step has too few matrix-core instructions to cover the LDS latency, so the reads
            // run kAhead steps ahead, one pipeline per chunk (a chunk has many stages here).  The wait before a
            // step leaves the reads of the kAhead-1 steps after it in flight; the step's own look-ahead read is
            // issued after that wait, so at most kAhead*kReads <= 15 reads are ever outstanding and every wait
            // names a count below the counter's no-wait value.
            constexpr int kReads = CB + NRB;
            constexpr int kAhead = gemm_steps_ahead(kReads);
            constexpr int DS = kAhead + 1;  // even, so that the parity of a step is static in the unrolled loop
            constexpr int GS = DS / 2;      // stages of one unrolled group of DS steps
            static_assert(kAhead * kReads <= 15 && (kAhead - 1) * kReads <= 14, "LDS counter");
            static_assert(2 * GS * 2 * CB * 1024 + CB * 2048 < 65536, "weight offsets fit the read instruction's offset field");
            using wseq = std::make_integer_sequence<int, CB>;
            using xseq = std::make_integer_sequence<int, NRB>;
            const uint32_t x0 = (uint32_t)a0_off * 16u, x1 = (uint32_t)a1_off * 16u;
            const uint32_t a_stage = NORM ? 1024u : (uint32_t)nA * 1024u;  // activation tiles of one stage
            int slot_c = 0;
            for (int c = 0; c < nchunks; ++c) {
                open_chunk();
                const int s_cnt = chunk_stages(c);
                const uint32_t wb = ring_addr + (uint32_t)(slot_c * slot_blocks) * 1024u + (uint32_t)lane * 16u;
                const uint32_t xb = NORM ? lds_base + (uint32_t)(c * SPC) * 1024u
                                         : ring_addr + (uint32_t)(slot_c * slot_blocks + s_cnt * 2 * CB) * 1024u;
                Frags f[DS];
                // (the division is by a constant; the host makes the chunks whole groups wherever it can)
                const int ngroups = s_cnt / GS;
                if (ngroups * GS == s_cnt) {
                    // The chunk is a whole number of groups of DS steps.  Step k of group g consumes f[k] and
                    // issues the read of the step kAhead later: for k = 0 the group's own last step, for
                    // k >= 1 step k-1 of group g+1, which the last group does not have, so nothing is ever
                    // read that is not used.  Addresses: the weight blocks of a group and of the group after
                    // it sit at constant offsets from one running pointer; the activation tiles of a stage are
                    // nA KB apart (a run-time value), one running pointer per stage of this and the next group.
                    uint32_t wg = wb;
                    uint32_t xs[2 * GS];
#pragma unroll
                    for (int sg = 0; sg < 2 * GS; ++sg) xs[sg] = xb + (uint32_t)sg * a_stage;
                    static_for<DS - 1>([&](auto dc) {
                        constexpr int d = decltype(dc)::value;
                        read_frags_at<NW, ((d >> 1) * 2 * CB + (d & 1)) * 1024>(f[d], wg, xs[d >> 1] + ((d & 1) ? x1 : x0), wseq{}, xseq{});
                    });
                    for (int grp = 0; grp + 1 < ngroups; ++grp) {
                        static_for<DS>([&](auto kc) {
                            constexpr int k = decltype(kc)::value;
                            constexpr int t = k == 0 ? DS - 1 : DS + k - 1;  // the step read now, counted from this group's step 0
                            wait_lds_reads<(kAhead - 1) * kReads>();
                            tie_frags(f[k], wseq{}, xseq{});
                            read_frags_at<NW, ((t >> 1) * 2 * CB + (t & 1)) * 1024>(f[t % DS], wg, xs[t >> 1] + ((t & 1) ? x1 : x0), wseq{}, xseq{});
                            mm(f[k]);
                        });
                        wg += (uint32_t)(GS * 2 * CB) * 1024u;
#pragma unroll
                        for (int sg = 0; sg < 2 * GS; ++sg) xs[sg] += (uint32_t)GS * a_stage;
                    }
                    static_for<DS>([&](auto kc) {  // the last group
                        constexpr int k = decltype(kc)::value;
                        if constexpr (k == 0) {
                            wait_lds_reads<(kAhead - 1) * kReads>();
                            tie_frags(f[0], wseq{}, xseq{});
                            read_frags_at<NW, (((DS - 1) >> 1) * 2 * CB + 1) * 1024>(f[DS - 1], wg, xs[(DS - 1) >> 1] + x1, wseq{}, xseq{});
                        } else {
                            wait_lds_reads<(DS - 1 - k) * kReads>();
                            tie_frags(f[k], wseq{}, xseq{});
                        }
                        mm(f[k]);
                    });
                } else {
                    // Any other chunk (the last one of a K that is not a whole number of groups): the same
                    // pipeline with every address computed per step.  Reads past the chunk's last stage are
                    // redirected to the last stage: in bounds and never fed to the matrix core, which keeps
                    // the counts the same in every iteration; their registers are tied after the wait that
                    // ends the chunk like any other read's (see lds_read_b128).
                    const int last = s_cnt - 1;
                    auto rd_step = [&](Frags& fr, int u, int odd) {  // step u = 2*stage + odd; odd is static at every call
                        const int sl = min(u >> 1, last);
                        read_frags<NW>(fr, wb + (uint32_t)(sl * 2 * CB + odd) * 1024u, xb + (uint32_t)sl * a_stage + (odd ? x1 : x0),
                                       wseq{}, xseq{});
                    };
#pragma unroll
                    for (int d = 0; d < DS - 1; ++d) rd_step(f[d], d, d & 1);
                    const int nsteps = 2 * s_cnt;
                    for (int u0 = 0; u0 < nsteps; u0 += DS) {
#pragma unroll
                        for (int k = 0; k < DS; ++k) {
                            if (u0 + k < nsteps) {
                                wait_lds_reads<(kAhead - 1) * kReads>();
                                tie_frags(f[k], wseq{}, xseq{});
                                rd_step(f[(k + DS - 1) % DS], u0 + k + DS - 1, (k + DS - 1) & 1);
                                mm(f[k]);
                            }
                        }
                    }
                    wait_lds_reads<0>();
#pragma unroll
                    for (int d = 0; d < DS; ++d) tie_frags(f[d], wseq{}, xseq{});
                }
                slot_c = slot_c + 1 == nslots ? 0 : slot_c + 1;
            }
        }

        // Lane holds C[row = 16*rb + lr][n0 + 16j + 4g + v], v = 0..3.
        const int n0 = blockIdx.x * (16 * CB);
#pragma unroll
        for (int r = 0; r < NRB; ++r) {
            const int rowl = 16 * (wave + NW * r) + lr;
            if (rowl < mrem) {
                const size_t row = (size_t)(m0 + rowl);
                int p = 0, slot = 0;
                if constexpr (EPI == kEpiRopeAppend) {
                    p = ra.pos[row];
                    p = p < 0 ? 0 : (p >= ra.Lmax ? ra.Lmax - 1 : p);
                    slot = ra.slots ? ra.slots[row] : (int)row;
                }
#pragma unroll
                for (int j = 0; j < CB; ++j) {
                    const int n = n0 + 16 * j + 4 * g;
                    const f32x4 a4 = acc[r][j];
                    const float v[4] = {a4[0], a4[1], a4[2], a4[3]};
                    if constexpr (EPI == kEpiRopeAppend)
                        gemm_epilogue_rope_append(v, ra, row, p, slot, n);
                    else
                        gemm_epilogue_store<EPI>(v, C, ldc, R, ldr, row, n, out_f32);
                }
            }
        }
    };
    if constexpr (NORM) {
        run(std::integral_constant<int, 1>{});
    } else if constexpr (NW == 8) {
        if (nrb == 1)
            run(std::integral_constant<int, 1>{});
        else
            run(std::integral_constant<int, 2>{});
    } else {
        switch (nrb) {
            case 1: run(std::integral_constant<int, 1>{}); break;
            case 2: run(std::integral_constant<int, 2>{}); break;
            case 3: run(std::integral_constant<int, 3>{}); break;
            default: run(std::integral_constant<int, 4>{}); break;
        }
    }
}

// One thread per 16 bytes of the packed matrix: gathers 8 K-consecutive elements of one column.
// gate_up_f > 0: packed column 2j is logical column j (gate) and 2j+1 is gate_up_f + j (up).
// rope_d > 0: within every head of rope_d columns, packed columns 2i and 2i+1 are the head's logical
// columns i and i + rope_d/2 (a rotation pair).
__global__ __launch_bounds__(256) void gemm_pack_kernel(const uint16_t* __restrict__ Bkn,
                                                        uint4* __restrict__ Bp, int N, int K, int cb,
                                                        int gate_up_f, int rope_d)
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
        if (rope_d > 0) {
            const int r = n % rope_d;
            n = n - r + (r >> 1) + ((r & 1) ? rope_d >> 1 : 0);
        }
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

// Up to four rows: each workgroup repeats the normalization of every row, which is off the critical path only
// while it is shorter than the wait for the first weights (measured on the layer: 4 us gained at one row, 3 at
// two, 1 at four, 3 lost at eight).
constexpr int kNormRows = 4;
template <int CB, int RINGB, int EPI, int NW, int NL, int PCB = CB, bool NORM = false>
static bool launch_gemm(const void* A, int lda, const void* Bp, void* C, int ldc, const void* R, int ldr,
                        const gemm_rope_args& ra, int M, int N, int K, int out_f32, hipStream_t s,
                        int tile_rows = 256, float eps = 0.0f)
{
    // tile_rows: a multiple of 16 in 16..256 (the kernel handles 1..16 row blocks of 16 rows)
    dim3 grid(N / (16 * CB), (M + tile_rows - 1) / tile_rows);
    if (NORM && (M > kNormRows || grid.y != 1 || (K >> 6) + 4 * CB > RINGB)) return false;
    const gemm_tile_plan tail = make_tile_plan(M - tile_rows * ((M - 1) / tile_rows), CB, RINGB, NW, NL, K, NORM);
    const gemm_tile_plan full = NORM ? tail : make_tile_plan(tile_rows, CB, RINGB, NW, NL, K);  // NORM: the one tile is the tail
    if (!plan_fits_load_counter(full, CB) || !plan_fits_load_counter(tail, CB)) return false;
    hipLaunchKernelGGL((gemm_kernel<CB, RINGB, EPI, NW, NL, PCB, NORM>), grid, dim3(64 * (NW + NL)), 0, s,
                       static_cast<const uint16_t*>(A), lda, static_cast<const uint4*>(Bp), C, ldc,
                       static_cast<const uint16_t*>(R), ldr, K, out_f32, full, tail, ra, eps);
    return true;
}

// The launch that normalizes its rows itself (see the kernel): M <= 4, K <= 4096, R = the norm's weight vector.
template <int EPI>
static int gemm_dispatch_norm(const void* X, int ldx, const void* wn, float eps, const void* Bp, void* C, int ldc, int M,
                              int N, int K, hipStream_t s, const gemm_rope_args& ra, int f32 = 0)
{
    bool ok = true;
    switch (gemm_cols_per_block(N)) {
#define DET_GEMM_NORM_CASE(CBV)                                                                                        \
    case CBV:                                                                                                          \
        ok = launch_gemm<CBV, kRingBig, EPI, gemm_waves(CBV), gemm_loader_waves(CBV, false), CBV, true>(               \
            X, ldx, Bp, C, ldc, wn, 0, ra, M, N, K, f32, s, 256, eps);                                                 \
        break;
        DET_GEMM_NORM_CASE(1)
        DET_GEMM_NORM_CASE(2)
        DET_GEMM_NORM_CASE(3)
        DET_GEMM_NORM_CASE(4)
        DET_GEMM_NORM_CASE(5)
        DET_GEMM_NORM_CASE(6)
        DET_GEMM_NORM_CASE(7)
        default:
            DET_GEMM_NORM_CASE(8)
#undef DET_GEMM_NORM_CASE
    }
    return ok ? check_launch() : DET_ESHAPE;
}
static bool gemm_norm_fusable(int M, int K) { return M <= kNormRows && K <= 4096; }

// Picks the kernel configuration (packing from N, tiling from N and M) and launches it.
// fixed_tile: the one tiling per (N, K) that does not look at M: 256-row tiles of the packing's own width,
// whatever the row count (det_gemm_bf16_fixed_tile).
template <int EPI>
static int gemm_dispatch(const void* A, int lda, const void* Bp, void* C, int ldc, const void* R, int ldr, int M,
                         int N, int K, int f32, hipStream_t s, bool fixed_tile = false,
                         const gemm_rope_args& ra = gemm_rope_args{})
{
    bool ok = true;  // false: the schedule would overrun the kernel's load counter (no supported shape does)
    const int cb = gemm_cols_per_block(N);
    const bool small = gemm_small_ring(N);
    // What bounds a launch with many rows is the bytes each workgroup pulls through its compute unit's
    // memory pipe: every row of its tile of A and every column of its tile of the weights, once per K.
    // The tiling below picks, per (M, N), the tile shape that keeps that sum small while every compute
    // unit still gets a workgroup.  The packing is untouched (a workgroup streams as many adjacent slabs
    // as its tile is wide), and so is the arithmetic of an output element: the same chain of matrix-core
    // steps over ascending K in every instantiation, so its bytes do not depend on which ran.
    //
    // (1) Launches with enough rows that 128-column tiles of 256 rows still fill the chip (prefill): the
    //     widest tile moves the fewest bytes per flop, whatever the packing.
    if (!fixed_tile && !small && cb < 8 && 8 % cb == 0 && N % 128 == 0 &&
        (long long)((M + 255) / 256) * (N / 128) >= 256) {
        if (cb == 1)
            ok = launch_gemm<8, kRingBig, EPI, 8, 4, 1>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s);
        else if (cb == 2)
            ok = launch_gemm<8, kRingBig, EPI, 8, 4, 2>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s);
        else
            ok = launch_gemm<8, kRingBig, EPI, 8, 4, 4>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s);
        return ok ? check_launch() : DET_ESHAPE;
    }
    // (2) Matrices too narrow to give every compute unit a column tile (N / (16 cb) < 256): the rows are
    //     cut into as many tiles as fill the chip, which also shortens each workgroup's pass over A.
    const int row_blocks = (M + 15) / 16;
    int base_rows = 256;
    {
        const int fit = 256 / (N / (16 * cb));
        if (!fixed_tile && !small && fit >= 2 && row_blocks >= 2) {
            const int row_tiles = row_blocks < fit ? row_blocks : fit;
            const int rows = 16 * ((row_blocks + row_tiles - 1) / row_tiles);
            base_rows = rows < 256 ? rows : 256;
        }
    }
    // (3) Tall launches of 16- or 32-column packings: a 256-row x 16-column tile (all of A for a sliver of
    //     the weights) is the wrong shape from about a hundred rows on; 64-column tiles of M/row_tiles rows
    //     move up to half as many bytes (measured: K = 14336, N = 4096 at M = 256 in 63 us instead of 112).
    //     Taken from the row counts where the measured times cross, and only where the 64-column tiles
    //     move clearly fewer bytes per compute unit than the tiles of (2).
    const int sq_row_tiles = N % 64 == 0 && 256 / (N / 64) > 0 ? 256 / (N / 64) : 1;
    const int sq_even = 16 * ((row_blocks + sq_row_tiles - 1) / sq_row_tiles);
    const int sq_rows = sq_even < 256 ? sq_even : 256;  // a tile holds at most 16 row blocks
    const int base_live = base_rows < 16 * row_blocks ? base_rows : 16 * row_blocks;
    // bytes per compute unit ~ (rows + columns of a tile) x rounds of 256 workgroups
    auto rounds = [](long long wgs) { return (wgs + 255) / 256; };
    const long long sq_cost = (long long)(sq_rows + 64) * rounds((long long)(N / 64) * ((M + sq_rows - 1) / sq_rows));
    const long long base_cost =
        (long long)(base_live + 16 * cb) * rounds((long long)(N / (16 * cb)) * ((M + base_rows - 1) / base_rows));
    const bool sq_pays = 115 * sq_cost <= 100 * base_cost;
    if (!fixed_tile && !small && N % 64 == 0 && sq_pays && ((cb == 1 && M >= 96) || (cb == 2 && M >= 192))) {
        const int rows = sq_rows;
        if (cb == 1)
            ok = launch_gemm<4, kRingBig, EPI, 8, 4, 1>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s, rows);
        else
            ok = launch_gemm<4, kRingBig, EPI, 8, 4, 2>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s, rows);
        return ok ? check_launch() : DET_ESHAPE;
    }
#define DET_GEMM_CASE(CBV)                                                                                  \
    case CBV:                                                                                               \
        if constexpr (CBV <= 3) {                                                                           \
            if (small) {                                                                                    \
                ok = launch_gemm<CBV, gemm_small_ring_blocks(CBV), EPI, gemm_waves(CBV), gemm_loader_waves(CBV, true)>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s); \
                break;                                                                                      \
            }                                                                                               \
        }                                                                                                   \
        ok = launch_gemm<CBV, kRingBig, EPI, gemm_waves(CBV), gemm_loader_waves(CBV, false)>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s, base_rows);            \
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
            ok = launch_gemm<8, kRingBig, EPI, gemm_waves(8), gemm_loader_waves(8, false)>(A, lda, Bp, C, ldc, R, ldr, ra, M, N, K, f32, s, base_rows);
            break;
    }
#undef DET_GEMM_CASE
    return ok ? check_launch() : DET_ESHAPE;
}

static bool gemm_shape_ok(int N, int K) { return N > 0 && K > 0 && N % 16 == 0 && K % 64 == 0; }

}  // namespace det

using namespace det;

extern "C" size_t det_gemm_packed_b_bytes(int N, int K)
{
    if (!gemm_shape_ok(N, K)) return 0;
    return (size_t)2 * N * K;
}

static int pack_impl(const void* B_kn, void* B_packed, int N, int K, int gate_up_f, void* stream, int rope_d = 0)
{
    if (!B_kn || !B_packed) return DET_EINVAL;
    if (!gemm_shape_ok(N, K)) return DET_ESHAPE;
    if (!aligned16(B_kn) || !aligned16(B_packed)) return DET_EALIGN;
    const size_t total = (size_t)N * K / 8;
    const int blocks = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL(gemm_pack_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(B_kn), static_cast<uint4*>(B_packed), N, K,
                       gemm_cols_per_block(N), gate_up_f, rope_d);
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

extern "C" int det_gemm_pack_qkv(const void* B_kn, void* B_packed, int Hq, int Hkv, int D, int K, void* stream)
{
    if (Hq < 1 || Hkv < 1 || D != 128) return DET_ESHAPE;
    return pack_impl(B_kn, B_packed, (Hq + 2 * Hkv) * D, K, 0, stream, D);
}

static int gemm_args_ok(const void* A, int lda, const void* Bp, const void* C, int ldc, int M, int N, int K)
{
    if (!A || !Bp || !C || M < 1) return DET_EINVAL;
    if (!gemm_shape_ok(N, K)) return DET_ESHAPE;
    if (lda < K) return DET_EINVAL;
    if (lda > (1 << 22)) return DET_ESHAPE;  // the kernel keeps byte offsets inside a 256-row tile of A in 32 bits
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

extern "C" int det_gemm_bf16_fixed_tile(const void* A, int lda, const void* B_packed, void* C, int ldc, int M, int N,
                                        int K, int out_dtype, void* stream)
{
    if (out_dtype != DET_BF16 && out_dtype != DET_F32) return DET_EINVAL;
    const int rc = gemm_args_ok(A, lda, B_packed, C, ldc, M, N, K);
    if (rc != DET_OK) return rc;
    if (ldc < N) return DET_EINVAL;
    return gemm_dispatch<kEpiStore>(A, lda, B_packed, C, ldc, nullptr, 0, M, N, K, out_dtype == DET_F32,
                                    static_cast<hipStream_t>(stream), true);
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

extern "C" int det_gemm_qkv_rope_append(const void* A, int lda, const void* B_qkv, void* qbuf, void* kcache,
                                        void* vcache, const int32_t* positions, const int32_t* slots,
                                        const float* rope_cos, const float* rope_sin, int M, int Hq, int Hkv, int D,
                                        int Lmax, int K, void* stream)
{
    if (Hq < 1 || Hkv < 1 || D != 128 || Lmax < 1) return DET_ESHAPE;
    const int N = (Hq + 2 * Hkv) * D;
    const int rc = gemm_args_ok(A, lda, B_qkv, qbuf, 4, M, N, K);
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
    return gemm_dispatch<kEpiRopeAppend>(A, lda, B_qkv, qbuf, 4, nullptr, 0, M, N, K, 0,
                                         static_cast<hipStream_t>(stream), false, ra);
}

extern "C" int det_rmsnorm_gemm_qkv_rope_append(const void* x, int ldx, const void* w_norm, float eps, const void* B_qkv,
                                                void* h, void* qbuf, void* kcache, void* vcache,
                                                const int32_t* positions, const int32_t* slots, const float* rope_cos,
                                                const float* rope_sin, int M, int Hq, int Hkv, int D, int Lmax, int K,
                                                void* stream)
{
    if (!x || !w_norm || !h) return DET_EINVAL;
    if (!aligned16(w_norm) || !aligned16(h)) return DET_EALIGN;
    if (!gemm_norm_fusable(M, K)) {
        if (ldx != K) return DET_EINVAL;  // det_rmsnorm takes contiguous rows
        const int rc = det_rmsnorm(x, w_norm, h, M, K, eps, stream);
        if (rc != DET_OK) return rc;
        return det_gemm_qkv_rope_append(h, K, B_qkv, qbuf, kcache, vcache, positions, slots, rope_cos, rope_sin, M, Hq,
                                        Hkv, D, Lmax, K, stream);
    }
    if (Hq < 1 || Hkv < 1 || D != 128 || Lmax < 1) return DET_ESHAPE;
    const int N = (Hq + 2 * Hkv) * D;
    const int rc = gemm_args_ok(x, ldx, B_qkv, qbuf, 4, M, N, K);
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
    return gemm_dispatch_norm<kEpiRopeAppend>(x, ldx, w_norm, eps, B_qkv, qbuf, 4, M, N, K,
                                              static_cast<hipStream_t>(stream), ra);
}

extern "C" int det_rmsnorm_gemm_swiglu_bf16(const void* x, int ldx, const void* w_norm, float eps, const void* B_gate_up,
                                            void* h, void* Y, int ldy, int M, int F, int K, void* stream)
{
    if (!x || !w_norm || !h) return DET_EINVAL;
    if (!aligned16(w_norm) || !aligned16(h)) return DET_EALIGN;
    if (!gemm_norm_fusable(M, K)) {
        if (ldx != K) return DET_EINVAL;
        const int rc = det_rmsnorm(x, w_norm, h, M, K, eps, stream);
        if (rc != DET_OK) return rc;
        return det_gemm_swiglu_bf16(h, K, B_gate_up, Y, ldy, M, F, K, stream);
    }
    if (F < 1 || F % 8 != 0) return DET_ESHAPE;
    const int rc = gemm_args_ok(x, ldx, B_gate_up, Y, ldy, M, 2 * F, K);
    if (rc != DET_OK) return rc;
    if (ldy < F) return DET_EINVAL;
    return gemm_dispatch_norm<kEpiSwiglu>(x, ldx, w_norm, eps, B_gate_up, Y, ldy, M, 2 * F, K,
                                          static_cast<hipStream_t>(stream), gemm_rope_args{});
}

extern "C" int det_rmsnorm_gemm_bf16(const void* x, int ldx, const void* w_norm, float eps, const void* B_packed, void* h,
                                     void* C, int ldc, int M, int N, int K, int out_dtype, void* stream)
{
    if (!x || !w_norm || !h) return DET_EINVAL;
    if (out_dtype != DET_BF16 && out_dtype != DET_F32) return DET_EINVAL;
    if (!aligned16(w_norm) || !aligned16(h)) return DET_EALIGN;
    if (!gemm_norm_fusable(M, K)) {
        if (ldx != K) return DET_EINVAL;
        const int rc = det_rmsnorm(x, w_norm, h, M, K, eps, stream);
        if (rc != DET_OK) return rc;
        return det_gemm_bf16(h, K, B_packed, C, ldc, M, N, K, out_dtype, stream);
    }
    const int rc = gemm_args_ok(x, ldx, B_packed, C, ldc, M, N, K);
    if (rc != DET_OK) return rc;
    if (ldc < N) return DET_EINVAL;
    return gemm_dispatch_norm<kEpiStore>(x, ldx, w_norm, eps, B_packed, C, ldc, M, N, K, static_cast<hipStream_t>(stream),
                                         gemm_rope_args{}, out_dtype == DET_F32);
}
