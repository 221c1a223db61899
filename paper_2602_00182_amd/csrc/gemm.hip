// Deterministic bf16 GEMM for gfx950: C[M,N] = A[M,K] * B[K,N], fp32 accumulation on the matrix
// cores, one accumulator chain per output element in ascending K (the paper's section 6.5:
// invariant 1, fixed workgroup -> tile mapping with no inter-workgroup communication; invariant 3,
// no atomics).
//
// Shape of the kernel
//   * A workgroup (4 wavefronts) owns BN = 16*CB output columns and up to 256 rows; grid.x = N/BN,
//     grid.y = ceil(M/256).  CB is a function of N alone (gemm_cols_per_block), so the
//     configuration never depends on M.
//   * The weight slab of the workgroup is one contiguous run of the packed matrix.  It is streamed
//     through a double-buffered LDS ring in chunks of CS 64-deep K stages: all 256 threads issue
//     the 16-byte global loads of chunk c+1 before computing on chunk c.
//   * Weights are the ROW operand of v_mfma_f32_16x16x32_bf16 (16 output columns of C), the
//     activations are its COLUMN operand (16 rows of C): a lane then holds 4 consecutive columns of
//     one row of C, which makes the store one 8- or 16-byte write.
//   * 16-row blocks of the tile are dealt round-robin to the 4 waves (block rb -> wave rb % 4).
//     M only decides how many blocks exist; a block's arithmetic is identical wherever it sits.
//     Activation fragments go straight from global memory (L2) to registers: each is needed by
//     exactly one wave of the workgroup.
//
// K order inside a 64-deep stage s: matrix-core step 2s takes k = 64s + 16g + e, step 2s+1 takes
// k = 64s + 16g + 8 + e (g = lane/16 in 0..3, e in 0..7), so that a lane's two activation
// fragments are 32 contiguous bytes of a row of A.
#include "common.h"

namespace det {

__host__ __device__ constexpr int gemm_stage_u4(int cb) { return cb * 2 * 64; }  // uint4 per stage

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

// K stages per LDS chunk for a given CB: at most 32 KB per chunk (two chunks fit the 64 KB of
// statically declared LDS), even so that the chunk is a whole number of 16-byte loads per thread.
__host__ __device__ constexpr int gemm_chunk_stages(int cb)
{
    return cb == 1 ? 16 : cb == 2 ? 8 : cb <= 4 ? 4 : 2;
}

template <int CB>
__global__ __launch_bounds__(256) void gemm_kernel(const uint16_t* __restrict__ A, int lda,
                                                   const uint4* __restrict__ Bp, void* __restrict__ C,
                                                   int ldc, int M, int K, int out_f32)
{
    constexpr int CS = gemm_chunk_stages(CB);
    constexpr int STAGE_U4 = gemm_stage_u4(CB);
    constexpr int CHUNK_U4 = CS * STAGE_U4;
    constexpr int LOADS = CHUNK_U4 / 256;
    static_assert(CHUNK_U4 % 256 == 0, "chunk must be a whole number of loads per thread");
    __shared__ uint4 lds[2][CHUNK_U4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int g = lane >> 4;      // k group of the lane
    const int lr = lane & 15;     // row of A / column-in-block of the weights
    const int m0 = blockIdx.y * 256;
    const int nstages = K >> 6;
    const int total_u4 = nstages * STAGE_U4;
    const uint4* __restrict__ bsrc = Bp + (size_t)blockIdx.x * total_u4;

    // Row blocks of this wave: rb = wave + 4r.  Block r is active when its first row exists.
    const int mrem = M - m0;
    const uint16_t* arow[4];
    bool rvalid[4];
    int nrb = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 16 * (wave + 4 * r) + lr;
        if (16 * (wave + 4 * r) < mrem) nrb = r + 1;
        rvalid[r] = row < mrem;
        arow[r] = A + (size_t)(m0 + (rvalid[r] ? row : 0)) * lda + 16 * g;
    }

    f32x4 acc[4][CB];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < CB; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint4 pre[LOADS];
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int idx = i * 256 + tid;
        pre[i] = idx < total_u4 ? bsrc[idx] : zero4;
    }

    const int nchunks = (nstages + CS - 1) / CS;
    for (int ch = 0; ch < nchunks; ++ch) {
        uint4* buf = lds[ch & 1];
#pragma unroll
        for (int i = 0; i < LOADS; ++i) buf[i * 256 + tid] = pre[i];
        __syncthreads();
        if (ch + 1 < nchunks) {
            const int base = (ch + 1) * CHUNK_U4;
#pragma unroll
            for (int i = 0; i < LOADS; ++i) {
                const int idx = base + i * 256 + tid;
                pre[i] = idx < total_u4 ? bsrc[idx] : zero4;
            }
        }
        const int st_n = min(CS, nstages - ch * CS);
        if (nrb > 0) {
            for (int st = 0; st < st_n; ++st) {
                const int kbase = (ch * CS + st) << 6;
                bf16x8 wf[CB][2];
#pragma unroll
                for (int j = 0; j < CB; ++j) {
                    wf[j][0] = __builtin_bit_cast(bf16x8, buf[st * STAGE_U4 + (2 * j) * 64 + lane]);
                    wf[j][1] = __builtin_bit_cast(bf16x8, buf[st * STAGE_U4 + (2 * j + 1) * 64 + lane]);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (r < nrb) {
                        uint4 a0 = zero4, a1 = zero4;
                        if (rvalid[r]) {
                            const uint4* ap = reinterpret_cast<const uint4*>(arow[r] + kbase);
                            a0 = ap[0];
                            a1 = ap[1];
                        }
                        const bf16x8 x0 = __builtin_bit_cast(bf16x8, a0);
                        const bf16x8 x1 = __builtin_bit_cast(bf16x8, a1);
#pragma unroll
                        for (int j = 0; j < CB; ++j) {
                            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j][0], x0, acc[r][j], 0, 0, 0);
                            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j][1], x1, acc[r][j], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

    // Lane holds C[row = 16*rb + lr][n0 + 16j + 4g + v], v = 0..3.
    const int n0 = blockIdx.x * (16 * CB);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (r < nrb && rvalid[r]) {
            const size_t row = (size_t)(m0 + 16 * (wave + 4 * r) + lr);
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
    const int stage_u4 = gemm_stage_u4(cb);
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
        const int k0 = 64 * st + 16 * (lane >> 4) + 8 * i;
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

template <int CB>
static void launch_gemm(const void* A, int lda, const void* Bp, void* C, int ldc, int M, int N, int K,
                        int out_f32, hipStream_t s)
{
    dim3 grid(N / (16 * CB), (M + 255) / 256);
    hipLaunchKernelGGL(gemm_kernel<CB>, grid, dim3(256), 0, s, static_cast<const uint16_t*>(A), lda,
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
    switch (gemm_cols_per_block(N)) {
        case 1: launch_gemm<1>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
        case 2: launch_gemm<2>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
        case 3: launch_gemm<3>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
        case 4: launch_gemm<4>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
        case 5: launch_gemm<5>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
        case 6: launch_gemm<6>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
        case 7: launch_gemm<7>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
        default: launch_gemm<8>(A, lda, B_packed, C, ldc, M, N, K, f32, s); break;
    }
    return check_launch();
}
