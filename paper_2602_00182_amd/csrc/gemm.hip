// Deterministic bf16 GEMM for gfx950: C[M,N] = A[M,K] * B[K,N], fp32 accumulation on the matrix
// cores, one accumulator chain per output element in ascending K (the paper's section 6.5:
// invariant 1, fixed workgroup -> tile mapping with no inter-workgroup communication; invariant 3,
// no atomics).
//
// Shape of the kernel
//   * A workgroup (4 wavefronts) owns BN = 16*CB output columns and up to 256 rows; grid.x = N/BN,
//     grid.y = ceil(M/256).  CB and the LDS chunk size are functions of N alone, so the
//     configuration never depends on M.
//   * K is cut into 64-deep stages.  A stage is a run of 1 KB blocks, each already in the
//     operand order of v_mfma_f32_16x16x32_bf16 (lane l holds 8 consecutive k of row/column l%16,
//     k group l/16): 2*CB weight blocks followed by 2*RB activation blocks, RB = number of 16-row
//     blocks of the tile that hold data.  M decides RB and nothing else.
//   * Stages are streamed through two LDS chunk buffers with the LDS-DMA form of the global load
//     (global_load_lds_dwordx4: no staging registers, a wave instruction fills one 1 KB block):
//     while the waves compute on one buffer, the loads of the next chunk are in flight into the
//     other.  The weight slab of a workgroup is one contiguous run of the packed matrix.
//   * Weights are the ROW operand of the MFMA (16 output columns of C), activations its COLUMN
//     operand (16 rows of C): a lane then holds 4 consecutive columns of one row of C and the
//     store is one 8- or 16-byte write.  Rows of the operand are independent in the matrix core,
//     so rows past M may hold anything: their loads are clamped to row M-1 and never stored.
//   * 16-row blocks are dealt round-robin to the 4 waves (block rb -> wave rb % 4).
//
// K order: matrix-core step t (t = 0 .. K/32-1, ascending) takes k in [32t, 32t+32); inside a step
// lane group g supplies k = 32t + 8g + e, e = 0..7.
#include "common.h"

namespace det {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

// Columns-per-workgroup factor: the largest CB in 1..8 that divides N/16 and still leaves at least
// 240 workgroups across N (one per compute unit, roughly); 1 if there is none.
int gemm_cols_per_block(int N)
{
    const int nb = N / 16;
    int best = 1;
    for (int cb = 1; cb <= 8; ++cb)
        if (nb % cb == 0 && nb / cb >= 240) best = cb;
    return best;
}

// 1 KB blocks per LDS chunk buffer (there are two buffers).  A stage of the largest tile needs
// 2*(CB+16) blocks.  When N yields at least 1.5 workgroups per compute unit and CB is small, the
// buffers are kept small enough for two workgroups to share a compute unit's 160 KB of LDS.
__host__ __device__ constexpr int gemm_small_chunk_blocks(int cb) { return 2 * (cb + 16) + 2; }
int gemm_chunk_blocks(int N)
{
    const int cb = gemm_cols_per_block(N);
    if (cb <= 3 && N / (16 * cb) >= 384) return gemm_small_chunk_blocks(cb);
    return 64;
}

template <int CB, int CHB>
__global__ __launch_bounds__(256) void gemm_kernel(const uint16_t* __restrict__ A, int lda,
                                                   const uint4* __restrict__ Bp, void* __restrict__ C,
                                                   int ldc, int M, int K, int out_f32)
{
    static_assert(CHB >= 2 * (CB + 16), "a chunk buffer must hold one stage of the largest tile");
    __shared__ uint4 buf0[CHB * 64];
    __shared__ uint4 buf1[CHB * 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;   // k group of the lane
    const int lr = lane & 15;  // row of A / column-in-block of the weights
    const int m0 = blockIdx.y * 256;
    const int mrem = min(M - m0, 256);
    const int RB = (mrem + 15) >> 4;          // 16-row blocks holding data
    const int nb = 2 * (CB + RB);             // 1 KB blocks per stage
    const int SPC = CHB / nb;                 // stages per chunk (>= 1)
    const int nstages = K >> 6;
    const int nchunks = (nstages + SPC - 1) / SPC;
    const uint4* __restrict__ bsrc = Bp + (size_t)blockIdx.x * nstages * (2 * CB * 64);
    const uint16_t* __restrict__ abase = A + (size_t)m0 * lda;

    // Row blocks of this wave: rb = wave + 4r, active while rb < RB.
    const int nrb = RB > wave ? (RB - wave + 3) >> 2 : 0;

    f32x4 acc[4][CB];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < CB; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Issues the LDS-DMA loads of chunk c into `buf`: block F of the chunk (stage F / nb, block
    // F % nb of that stage) is loaded by wave F % 4.
    auto load_chunk = [&](uint4* buf, int c) {
        const int s_begin = c * SPC;
        const int s_cnt = min(SPC, nstages - s_begin);
        const int total = s_cnt * nb;
        int s = s_begin, f = wave;
        for (int F = wave; F < total; F += 4) {
            const void* src;
            if (f < 2 * CB) {
                src = bsrc + ((size_t)s * (2 * CB) + f) * 64 + lane;
            } else {
                const int a = f - 2 * CB;
                int row = 16 * (a >> 1) + lr;
                row = row < mrem ? row : mrem - 1;
                src = abase + (size_t)row * lda + (s << 6) + 32 * (a & 1) + 8 * g;
            }
            __builtin_amdgcn_global_load_lds((global_void_t*)src, (lds_void_t*)(buf + F * 64), 16, 0, 0);
            f += 4;
            if (f >= nb) {
                f -= nb;
                ++s;
            }
        }
    };

    auto compute_chunk = [&](const uint4* buf, int c) {
        if (nrb == 0) return;
        const int s_cnt = min(SPC, nstages - c * SPC);
        for (int s = 0; s < s_cnt; ++s) {
            const uint4* st = buf + s * nb * 64 + lane;
            bf16x8 wf[CB][2];
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                wf[j][0] = __builtin_bit_cast(bf16x8, st[(2 * j) * 64]);
                wf[j][1] = __builtin_bit_cast(bf16x8, st[(2 * j + 1) * 64]);
            }
            bf16x8 xf[4][2];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (r < nrb) {
                    const uint4* ap = st + (2 * CB + 2 * (wave + 4 * r)) * 64;
                    xf[r][0] = __builtin_bit_cast(bf16x8, ap[0]);
                    xf[r][1] = __builtin_bit_cast(bf16x8, ap[64]);
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (r < nrb) {
#pragma unroll
                        for (int j = 0; j < CB; ++j)
                            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j][i], xf[r][i], acc[r][j], 0, 0, 0);
                    }
        }
    };

    load_chunk(buf0, 0);
    for (int c = 0; c < nchunks; c += 2) {
        __syncthreads();  // chunk c has landed in buf0; every wave is done with buf1
        if (c + 1 < nchunks) load_chunk(buf1, c + 1);
        compute_chunk(buf0, c);
        if (c + 1 < nchunks) {
            __syncthreads();  // chunk c+1 has landed in buf1; every wave is done with buf0
            if (c + 2 < nchunks) load_chunk(buf0, c + 2);
            compute_chunk(buf1, c + 1);
        }
    }

    // Lane holds C[row = 16*rb + lr][n0 + 16j + 4g + v], v = 0..3.
    const int n0 = blockIdx.x * (16 * CB);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int rowl = 16 * (wave + 4 * r) + lr;
        if (r < nrb && rowl < mrem) {
            const size_t row = (size_t)(m0 + rowl);
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                const int n = n0 + 16 * j + 4 * g;
                const f32x4 v = acc[r][j];
                if (out_f32) {
                    float4* dst = reinterpret_cast<float4*>(static_cast<float*>(C) + row * ldc + n);
                    *dst = make_float4(v[0], v[1], v[2], v[3]);
                } else {
                    uint2* dst = reinterpret_cast<uint2*>(static_cast<uint16_t*>(C) + row * ldc + n);
                    *dst = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
                }
            }
        }
    }
}

// One thread per 16 bytes of the packed matrix: gathers 8 K-consecutive elements of one column.
__global__ __launch_bounds__(256) void gemm_pack_kernel(const uint16_t* __restrict__ Bkn,
                                                        uint4* __restrict__ Bp, int N, int K, int cb)
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
        const int n = tile * 16 * cb + 16 * j + (lane & 15);
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

template <int CB, int CHB>
static void launch_gemm(const void* A, int lda, const void* Bp, void* C, int ldc, int M, int N, int K,
                        int out_f32, hipStream_t s)
{
    dim3 grid(N / (16 * CB), (M + 255) / 256);
    hipLaunchKernelGGL((gemm_kernel<CB, CHB>), grid, dim3(256), 0, s, static_cast<const uint16_t*>(A), lda,
                       static_cast<const uint4*>(Bp), C, ldc, M, K, out_f32);
}

static bool gemm_shape_ok(int N, int K) { return N > 0 && K > 0 && N % 16 == 0 && K % 64 == 0; }

}  // namespace det

using namespace det;

extern "C" size_t det_gemm_packed_b_bytes(int N, int K)
{
    if (!gemm_shape_ok(N, K)) return 0;
    return (size_t)2 * N * K;
}

extern "C" int det_gemm_pack_b(const void* B_kn, void* B_packed, int N, int K, void* stream)
{
    if (!B_kn || !B_packed) return DET_EINVAL;
    if (!gemm_shape_ok(N, K)) return DET_ESHAPE;
    if (!aligned16(B_kn) || !aligned16(B_packed)) return DET_EALIGN;
    const size_t total = (size_t)N * K / 8;
    const int blocks = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL(gemm_pack_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t*>(B_kn), static_cast<uint4*>(B_packed), N, K,
                       gemm_cols_per_block(N));
    return check_launch();
}

extern "C" int det_gemm_bf16(const void* A, int lda, const void* B_packed, void* C, int ldc, int M, int N,
                             int K, int out_dtype, void* stream)
{
    if (!A || !B_packed || !C || M < 1) return DET_EINVAL;
    if (out_dtype != DET_BF16 && out_dtype != DET_F32) return DET_EINVAL;
    if (!gemm_shape_ok(N, K)) return DET_ESHAPE;
    if (lda < K || ldc < N) return DET_EINVAL;
    if (!aligned16(A) || !aligned16(B_packed) || !aligned16(C) || lda % 8 != 0 || ldc % 4 != 0)
        return DET_EALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int f32 = out_dtype == DET_F32;
    const int cb = gemm_cols_per_block(N);
    const bool small = gemm_chunk_blocks(N) != 64;
#define DET_GEMM_CASE(CBV)                                                                          \
    case CBV:                                                                                       \
        if constexpr (CBV <= 3) {                                                                   \
            if (small) {                                                                            \
                launch_gemm<CBV, gemm_small_chunk_blocks(CBV <= 3 ? CBV : 1)>(A, lda, B_packed, C, ldc, M, N, \
                                                                             K, f32, s);            \
                break;                                                                              \
            }                                                                                       \
        }                                                                                           \
        launch_gemm<CBV, 64>(A, lda, B_packed, C, ldc, M, N, K, f32, s);                            \
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
            launch_gemm<8, 64>(A, lda, B_packed, C, ldc, M, N, K, f32, s);
            break;
    }
#undef DET_GEMM_CASE
    return check_launch();
}
