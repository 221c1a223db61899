/*
 * libdetinfer -- deterministic, batch-invariant transformer decode step for AMD MI355X (gfx950).
 *
 * Every entry point is a pure function of its input bytes and shape arguments: the output bytes
 * never depend on the stream, the launch order, what else runs on the device, the contents of a
 * workspace before the call, or on the batch size (row i of an output is the same whether the call
 * carries 1 row or 256, and whatever the other rows hold).  This is the contract of the paper's
 * section 6.1 (inference as a pure function whose honest re-executions are bit-identical) carried
 * by the three kernel invariants of its section 6.5: a fixed mapping of workgroups to output tiles
 * with no communication between workgroups, canonical stride-halving tree reductions, and no
 * floating-point atomics.
 *
 * Conventions
 *   - Plain C ABI.  All pointers are DEVICE pointers unless a comment says "host".
 *   - The caller owns every buffer.  The library allocates nothing and only enqueues work on the
 *     caller's HIP stream (`stream` is a hipStream_t passed as void*; NULL is the default stream).
 *     No call synchronises; results are ready when the stream reaches them.
 *   - bf16 tensors are arrays of 16-bit patterns (upper half of an IEEE fp32), row-major.
 *   - Workspaces need no initialisation: kernels overwrite whatever they later read.
 *   - Every call returns DET_OK or an error code below and launches nothing on error.  After
 *     DET_EHIP, det_last_hip_error() returns the hipError_t value seen by the calling thread.
 *   - Pointers must be 16-byte aligned (DET_EALIGN otherwise).
 *   - The library keeps no state between calls, with three exceptions that never reach an output byte:
 *     the per-thread last HIP error; the per-device address of the fixed scratch array of
 *     det_attn_decode_static (looked up once); and det_sha256_force_portable(), a process-wide switch
 *     for tests that selects between two implementations of the same hash.
 */
#ifndef DETINFER_H
#define DETINFER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DET_OK 0
#define DET_EINVAL 1     /* null pointer, non-positive size, bad enum */
#define DET_ESHAPE 2     /* shape outside what the kernels support (see each call) */
#define DET_EALIGN 3     /* pointer or leading dimension not 16-byte aligned */
#define DET_EWORKSPACE 4 /* workspace smaller than the matching *_workspace_bytes() */
#define DET_EHIP 5       /* a HIP runtime call failed */

#define DET_BF16 0
#define DET_F32 1

/* ---------------------------------------------------------------------------------------------
 * Deterministic GEMM (section 6.5: custom GEMM kernels; invariants 1 and 3).
 *
 *   C[i][j] = sum_k A[i][k] * B[k][j],  bf16 inputs, fp32 accumulation, output rounded once to
 *   bf16 (nearest even) or left in fp32.
 *
 * Each output element has ONE fp32 accumulator that starts at +0 and takes K/32 matrix-core steps
 * in ascending order; step t adds the 32 products of a fixed set of k indices (k in
 * [64*(t/2), 64*(t/2)+64), see det_gemm_pack_b).  There is no split of K across workgroups or
 * waves and there are no atomics.
 *
 * What depends on (N, K) only: the packing, the matrix-core instruction, the K staging and the order
 * of the steps, i.e. everything that enters an element's arithmetic.  What det_gemm_bf16 (and the
 * fused forms below) ALSO choose from M is the tile a launch cuts C into, i.e. which workgroup and wave
 * computes an element: 256 rows x the packing's width by default; rows cut into shorter tiles when N
 * alone gives fewer than 256 workgroups and M >= 17; 64-column tiles from M >= 96 (16-column packings)
 * or M >= 192 (32-column packings); 128-column tiles when ceil(M/256) * N/128 >= 256.  The bytes of a
 * row do not depend on that choice (every tile shape runs the same chain for an element; the tests
 * compare every M in 1..256 with the M = 256 launch and with det_gemm_bf16_fixed_tile), but it IS a
 * launch geometry keyed on the batch size, so it is named here and in det_fingerprint(), and
 * det_gemm_bf16_fixed_tile below is the form without it.
 *
 *   A        [M, K] bf16, row stride lda elements (lda >= K, lda % 8 == 0)
 *   B_packed output of det_gemm_pack_b for the same (N, K)
 *   C        [M, N] bf16 (out_dtype DET_BF16) or fp32 (DET_F32), row stride ldc elements
 *            (ldc >= N, ldc % 4 == 0)
 *   Shapes: M >= 1, N % 16 == 0, K % 64 == 0; DET_ESHAPE otherwise.
 */
int det_gemm_bf16(const void *A, int lda, const void *B_packed, void *C, int ldc, int M, int N,
                  int K, int out_dtype, void *stream);

/* det_gemm_bf16 with ONE tiling per (N, K) that never looks at M (section 6.5, invariant 1 read
 * strictly: a fixed workgroup -> tile mapping whatever the batch): 256-row tiles of the packing's
 * width, M only decides how many 16-row blocks of a tile hold data.  Same arguments, same bytes; slower
 * from about a hundred rows on (the benchmark reports both). */
int det_gemm_bf16_fixed_tile(const void *A, int lda, const void *B_packed, void *C, int ldc, int M, int N,
                             int K, int out_dtype, void *stream);

/* Bytes of the packed form of a [K, N] bf16 matrix (= 2*K*N). 0 if the shape is unsupported. */
size_t det_gemm_packed_b_bytes(int N, int K);

/* One-time, layout-only, bit-preserving repack of a row-major [K, N] bf16 weight matrix into the
 * order the GEMM kernel streams it: each workgroup's column slab becomes one contiguous run, cut
 * into 64-deep K stages already in matrix-core operand order.  B_kn and B_packed must not
 * overlap. */
int det_gemm_pack_b(const void *B_kn, void *B_packed, int N, int K, void *stream);

/* Fused epilogues of the same kernel; each produces exactly the bytes of the unfused sequence.
 *
 * det_gemm_bf16_residual: C = bf16( fp32(bf16(A B)) + fp32(R) ), i.e. det_gemm_bf16 (bf16 out)
 *   followed by det_residual_add.  R [M, N] bf16 with row stride ldr (ldr % 4 == 0); C may be R.
 * det_gemm_pack_gate_up: packs a [K, 2F] bf16 matrix whose columns are F gate columns followed by
 *   F up columns, with gate_j and up_j made neighbours, for det_gemm_swiglu_bf16.  F % 8 == 0.
 * det_gemm_swiglu_bf16: Y[M, F] = det_swiglu( g, u ) with [g | u] = det_gemm_bf16(A, [Wgate | Wup])
 *   rounded to bf16 first.  B_gate_up is the output of det_gemm_pack_gate_up; ldy >= F, ldy % 4 == 0.
 * det_gemm_pack_qkv: packs a [K, (Hq+2Hkv) D] bf16 matrix whose columns are Hq query heads, Hkv key
 *   heads and Hkv value heads of D = 128 columns each, with the columns d and d + D/2 of every head
 *   (a rotation pair of det_rope) made neighbours, for det_gemm_qkv_rope_append.
 * det_gemm_qkv_rope_append: the layer's fused projection.  With qkv = det_gemm_bf16(A, Wqkv) (bf16),
 *   row i at position p = positions[i] (clamped to 0..Lmax-1) and cache slot s = slots[i] (slots NULL:
 *   s = i): qbuf[i] = det_rope(query heads of qkv[i], p); kcache[s][:, p, :] = det_rope(key heads, p);
 *   vcache[s][:, p, :] = value heads.  Exactly the bytes of those three steps; qkv itself is never
 *   stored.  qbuf [M, Hq, D] bf16; caches [S, Hkv, Lmax, D] bf16; rope_cos/sin [Lmax, D/2] fp32,
 *   16-byte aligned; no two rows of one call may name the same (slot, position).  D must be 128.
 */
int det_gemm_bf16_residual(const void *A, int lda, const void *B_packed, const void *R, int ldr,
                           void *C, int ldc, int M, int N, int K, void *stream);
int det_gemm_pack_gate_up(const void *B_kn, void *B_packed, int F, int K, void *stream);
int det_gemm_swiglu_bf16(const void *A, int lda, const void *B_gate_up, void *Y, int ldy, int M,
                         int F, int K, void *stream);
/* The projections that follow an RMSNorm (two in the layer, the output head after the last layer), with the
 * norm in the same call:
 *   det_rmsnorm_gemm_qkv_rope_append(x, ...) = det_gemm_qkv_rope_append(det_rmsnorm(x, w_norm, eps), ...)
 *   det_rmsnorm_gemm_swiglu_bf16(x, ...)     = det_gemm_swiglu_bf16(det_rmsnorm(x, w_norm, eps), ...)
 *   det_rmsnorm_gemm_bf16(x, ...)            = det_gemm_bf16(det_rmsnorm(x, w_norm, eps), ...)
 * byte for byte.  x [M, K] bf16 raw rows with row stride ldx; w_norm [K] bf16; h [M, K] bf16 scratch that
 * the call may or may not write (M <= 4 and K <= 4096: the GEMM's workgroups normalize the rows themselves,
 * one launch instead of two, and h is untouched; otherwise det_rmsnorm into h, then the GEMM, and ldx must
 * be K).  Other arguments and errors as the two GEMM calls. */
int det_rmsnorm_gemm_qkv_rope_append(const void *x, int ldx, const void *w_norm, float eps,
                                     const void *B_qkv, void *h, void *qbuf, void *kcache, void *vcache,
                                     const int32_t *positions, const int32_t *slots,
                                     const float *rope_cos, const float *rope_sin, int M, int Hq,
                                     int Hkv, int D, int Lmax, int K, void *stream);
int det_rmsnorm_gemm_swiglu_bf16(const void *x, int ldx, const void *w_norm, float eps,
                                 const void *B_gate_up, void *h, void *Y, int ldy, int M, int F, int K,
                                 void *stream);
int det_rmsnorm_gemm_bf16(const void *x, int ldx, const void *w_norm, float eps, const void *B_packed,
                          void *h, void *C, int ldc, int M, int N, int K, int out_dtype, void *stream);
int det_gemm_pack_qkv(const void *B_kn, void *B_packed, int Hq, int Hkv, int D, int K, void *stream);
int det_gemm_qkv_rope_append(const void *A, int lda, const void *B_qkv, void *qbuf, void *kcache,
                             void *vcache, const int32_t *positions, const int32_t *slots,
                             const float *rope_cos, const float *rope_sin, int M, int Hq, int Hkv,
                             int D, int Lmax, int K, void *stream);

/* ---------------------------------------------------------------------------------------------
 * RMSNorm (section 6.5, invariant 2: canonical tree reduction; tree of Fig. "kernel_tree").
 *
 *   y[i][e] = bf16( (x[i][e] * r_i) * w[e] ),  r_i = 1 / sqrt( mean_e x[i][e]^2 + eps )
 *
 * Sum of squares: element e belongs to lane (e/8) mod 256; a lane folds its elements in ascending
 * e with fma(x, x, acc) from +0; the 256 lane sums are reduced by six stride-halving levels inside
 * each group of 64 lanes (offsets 32..1) and the four group sums as (q0+q2)+(q1+q3).  mean = ss/H;
 * divide and square root are correctly rounded fp32.
 *
 *   x, y [M, H] bf16 contiguous; w [H] bf16.  H % 8 == 0, H <= 16384.
 */
int det_rmsnorm(const void *x, const void *w, void *y, int M, int H, float eps, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Single-query attention over a KV cache, grouped-query heads (the paper is silent on attention;
 * the reductions follow section 6.5's invariants).
 *
 * For sequence b and query head h (reading KV head h / (Hq/Hkv)), len = seqlens[b]:
 *   s_j = scale * (q . k_j), j < len, contraction on matrix cores with fp32 accumulation;
 *   chunk c = tokens [256c, min(256c+256, len)):  m_c = max s_j;  e_j = det_expf(s_j - m_c);
 *   l_c = tree-sum of e_j (same 256-leaf tree as RMSNorm, leaf = j - 256c);
 *   O_c[d] = sum_j e_j * v_jd on the matrix cores: e_j (fp32) is cut by truncation into three bf16 pieces
 *            with e_j = hi + mid + lo exactly, so every product piece * v is exact in fp32; one fp32
 *            accumulator per (head, d) from +0 takes the chunk's eight 32-token steps in ascending order,
 *            each step the hi, then the mid, then the lo products (tokens at or past len add +0);
 *   combine in ascending c:  m = max m_c;  w_c = det_expf(m_c - m);  L = sum w_c*l_c;
 *   O[d] = sum w_c*O_c[d];  out[d] = bf16(O[d] / L).
 * The number of chunks depends only on that sequence's length.  Cache contents at or past len are
 * never used.  len = 0 gives zeros.
 *
 *   q, out   [B, Hq, D] bf16
 *   kcache, vcache [B, Hkv, Lmax, D] bf16
 *   seqlens  [B] int32, 0 <= seqlens[b] <= Lmax (values above Lmax are clamped to Lmax)
 *   ws       det_attn_decode_workspace_bytes(B, Hq, D, Lmax) bytes.  After the call it holds the chunk
 *            partials, fp32, nc = ceil(Lmax/256): m_c [B, Hq, nc], then l_c [B, Hq, nc], then the
 *            unnormalised chunk outputs o_c [B, Hq, nc, D]; entries of chunks at or past the sequence's
 *            length are not written, and neither is the o_c of a sequence of at most 256 tokens: its
 *            single chunk is finished by the first pass with the operations the combination would
 *            apply to it (det_attn_decode_quant_q8 always takes the second pass).  (Tests read m_c and
 *            l_c there and compare them bit for bit with the reference statistics of the same scores.)
 *   Shapes: D == 128, Hq % Hkv == 0, Hq/Hkv in {1, 2, 4, 8}.
 */
size_t det_attn_decode_workspace_bytes(int B, int Hq, int D, int Lmax);
int det_attn_decode(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                    void *out, void *ws, size_t ws_bytes, int B, int Hq, int Hkv, int D, int Lmax,
                    float scale, void *stream);

/* The same operation on R rows that name their cache slot: row r reads slot slots[r] of caches
 * [S, Hkv, Lmax, D] with length seqlens[r].  Several rows may share a slot (the tokens of one prompt
 * at lengths 1..T: batch-invariant prefill, since each row is exactly the single-token operation).
 * 0 <= slots[r] < S is the caller's responsibility.  Workspace: det_attn_decode_workspace_bytes(R, ...).
 * From sixteen rows on, eight consecutive rows go to one workgroup, and those of them that name the same
 * slot share each 256-token chunk of K and V (causal prefill: one read of the prompt's cache per eight
 * query tokens instead of one per token).  Which rows share a workgroup changes no row's arithmetic. */
int det_attn_decode_rows(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                         const int32_t *slots, void *out, void *ws, size_t ws_bytes, int R, int Hq,
                         int Hkv, int D, int Lmax, float scale, void *stream);

/* det_attn_decode for callers that cannot provide or allocate a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation): the chunk partials live in a fixed array of
 * DET_ATTN_STATIC_WS_BYTES inside the library's code object, one copy per device, held until the
 * process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine); its
 * first call on a device looks up that device's copy of the array (hipGetSymbolAddress), so the device
 * `stream` belongs to must be the current device.  Output bytes are those of det_attn_decode.
 *   Limit: det_attn_decode_workspace_bytes(B, Hq, D, Lmax) <= DET_ATTN_STATIC_WS_BYTES, i.e.
 *   B * Hq * ceil(Lmax/256) <= 64527; DET_EWORKSPACE beyond it (nothing is launched).
 *   All calls on one device share the array, which keeps the previous call's partials; nothing in it
 *   needs clearing (each call overwrites what it later reads), but two calls that overlap in time on
 *   one device (different streams) race on it: serialise them.
 *   Other arguments and errors as det_attn_decode. */
#define DET_ATTN_STATIC_WS_BYTES (32u << 20)
int det_attn_decode_static(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                           void *out, int B, int Hq, int Hkv, int D, int Lmax, float scale, void *stream);

/* Test hook: the softmax statistics of det_attn_decode on caller-provided fp32 scores.  The per-chunk
 * statistics (m_c, e_j, l_c) come from the one device routine the attention kernel itself calls; the
 * combination over chunks is the same ascending fold, written for one row per workgroup.
 * s, p [R, Lmax] fp32; lens [R]; m_out, l_out [R] fp32.
 * p_j = (w_c * e_j) / L for j < lens[r]; entries at or past lens[r] are not written.
 * lens[r] = 0 gives m = -inf, L = 0.  Lmax <= 262144. */
int det_softmax_f32(const float *s, const int32_t *lens, float *p, float *m_out, float *l_out, int R,
                    int Lmax, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Greedy sampling (section 6.6: deterministic decoding in a canonical iteration order).
 * idx[b] = smallest index attaining the maximum of row b; -0 equals +0; NaN never wins; a row of
 * NaNs gives 0.  logits [B, V] fp32 (DET_F32) or bf16 (DET_BF16); idx [B] int32. */
int det_argmax(const void *logits, int32_t *idx, int B, int V, int dtype, void *stream);

/* Seeded sampling (section 6.6: a fixed-seed PRNG and a canonical iteration order make the token a
 * function of (seed, decode policy)).  Per row:
 *   z_j = logits_j / temperature (NaN counts as -inf);  candidates ordered by (z descending, index
 *   ascending);  the first k = min(top_k, V) kept;  e_i = det_expf(z_i - z_0);  c_i = c_{i-1} + e_i in
 *   rank order (sequential fp32 adds from +0);  n = smallest i+1 with c_i >= top_p * c_{k-1};
 *   u = (splitmix64 output for seed + ((seq_id << 32 | step) + 1) * 0x9E3779B97F4A7C15) >> 40, scaled by
 *   2^-24;  target = u * c_{n-1};  token = candidate of the smallest rank i < n with c_i > target
 *   (rank n-1 if none).  top_k = 1 is det_argmax.
 * The sample depends on (seed, seq_ids[b], steps[b]) and row b's logits only, never on the batch.
 *   logits [B, V] fp32; seq_ids, steps, tokens [B] int32.
 *   temperature > 0, 0 < top_p <= 1 (DET_EINVAL otherwise); 1 <= top_k <= 1024 (DET_ESHAPE). */
int det_sample(const float *logits, int B, int V, float temperature, int top_k, float top_p,
               uint64_t seed, const int32_t *seq_ids, const int32_t *steps, int32_t *tokens,
               void *stream);

/* ---------------------------------------------------------------------------------------------
 * Elementwise steps of the decoder layer, exported so each can be checked bit for bit.
 *
 * det_rope: rotary embedding, rotate-half pairing (i, i + D/2), on nh heads of one token per row.
 *   y_lo = bf16( fma(-x_hi, sin, x_lo*cos) ),  y_hi = bf16( fma(x_lo, sin, x_hi*cos) )
 *   x, y [R, nh, D] bf16 (row stride ldx / ldy elements); pos [R] int32 (< Lmax);
 *   cos_t, sin_t [Lmax, D/2] fp32 built by the caller.  D == 128.
 * det_swiglu: y = bf16( (g / (1 + det_expf(-g))) * u ); g, u, y [R, F] bf16 with row strides.
 * det_residual_add: z = bf16( fp32(x) + fp32(y) ), n elements, n % 8 == 0; z may alias x.
 */
int det_rope(const void *x, int ldx, void *y, int ldy, const int32_t *pos, const float *cos_t,
             const float *sin_t, int R, int nh, int D, int Lmax, void *stream);
int det_swiglu(const void *g, int ldg, const void *u, int ldu, void *y, int ldy, int R, int F,
               void *stream);
int det_residual_add(const void *x, const void *y, void *z, int64_t n, void *stream);

/* out[b][:] = table[tokens[b]][:]  (exact copy).  table [V, H] bf16; tokens [B] int32 in [0, V);
 * out [B, H] bf16.  H % 8 == 0.  Out-of-range ids are clamped into [0, V). */
int det_embed_gather(const void *table, const int32_t *tokens, void *out, int B, int H, int V,
                     void *stream);

/* ---------------------------------------------------------------------------------------------
 * One Llama-style decoder layer on one new token per sequence.
 *
 *   h = rmsnorm(x, w_norm1);  [q|k|v] = h Wqkv;  q, k = rope(q, k) at positions[b];
 *   k, v are written into the caches at row positions[b];
 *   a = attn_decode(q, caches, len = positions[b] + 1);
 *   x = x + a Wo;  h = rmsnorm(x, w_norm2);  [g|u] = h Wgu;  m = swiglu(g, u);  x = x + m Wdown.
 *
 * Every step is the operation documented above (the residual adds and the SwiGLU run as fused GEMM
 * epilogues with the bytes of the unfused steps), so the layer inherits their invariance: row b
 * of x and sequence b's cache rows do not depend on B or on the other sequences.
 */
typedef struct det_layer_cfg {
    int32_t H;      /* hidden size */
    int32_t Hq;     /* query heads */
    int32_t Hkv;    /* KV heads */
    int32_t D;      /* head dim (128) */
    int32_t F;      /* MLP inner size */
    int32_t Lmax;   /* rows per (sequence, KV head) in the caches and in the rope tables */
    float eps;      /* RMSNorm epsilon */
    float scale;    /* attention score scale, normally (float)(1/sqrt(D)) */
} det_layer_cfg;

typedef struct det_layer_weights {
    const void *w_norm1; /* [H] bf16 */
    const void *wqkv;    /* [K=H, N=(Hq+2Hkv)D] (columns: q heads, k heads, v heads) packed by
                          * det_gemm_pack_qkv */
    const void *wo;      /* packed [K=Hq*D, N=H] */
    const void *w_norm2; /* [H] bf16 */
    const void *wgu;     /* [K=H, N=2F] (columns: gate, up) packed by det_gemm_pack_gate_up */
    const void *wdown;   /* packed [K=F, N=H] */
} det_layer_weights;

size_t det_decoder_layer_workspace_bytes(const det_layer_cfg *cfg /* host */, int B);

/* One decoder layer as a pure function of (weights, x, caches, positions): section 6.1's contract (an
 * honest re-execution reproduces the bytes) composed from the operations above, which is what lets a
 * verifier re-run a single layer of a disputed step (section 6.1, layer-granular re-execution).
 *   w, cfg      host structs holding device pointers / sizes
 *   x_inout     [B, H] bf16, updated in place
 *   kcache, vcache [B, Hkv, Lmax, D] bf16, row positions[b] of every KV head of sequence b written
 *   positions   [B] int32, 0 <= positions[b] < Lmax
 *   rope_cos, rope_sin [Lmax, D/2] fp32
 */
int det_decoder_layer(const det_layer_weights *w, const det_layer_cfg *cfg, void *x_inout,
                      void *kcache, void *vcache, const int32_t *positions, const float *rope_cos,
                      const float *rope_sin, void *ws, size_t ws_bytes, int B, void *stream);

/* The layer on R rows that name their cache slot (caches [S, Hkv, Lmax, D]): row r is one token at
 * position positions[r] of the sequence in slot slots[r].  All keys and values of the call are
 * written before any row attends, so the T tokens of a prompt can go through in one call (rows at
 * positions 0..T-1 of one slot): every row's bytes are those of feeding the tokens one call at a
 * time.  No two rows may name the same (slot, position).  Workspace:
 * det_decoder_layer_workspace_bytes(cfg, R). */
int det_decoder_layer_rows(const det_layer_weights *w, const det_layer_cfg *cfg, void *x_inout,
                           void *kcache, void *vcache, const int32_t *positions, const int32_t *slots,
                           const float *rope_cos, const float *rope_sin, void *ws, size_t ws_bytes,
                           int R, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Token bookkeeping of the greedy decode loop, on the device so a step needs no host round trip.
 * For row b at step t:  tok = t < prompt_lens[b] ? prompts[b][t] : last_sampled[b];
 * tokens_out[b] = tok;  history[b][t] = tok;  positions_out[b] = t.
 *   prompts [B, Tp] int32; prompt_lens [B]; last_sampled [B] (the argmax of step t-1);
 *   history [B, Th] int32 with t < Th.
 */
int det_next_token(const int32_t *prompts, int Tp, const int32_t *prompt_lens,
                   const int32_t *last_sampled, int32_t *tokens_out, int32_t *positions_out,
                   int32_t *history, int Th, int t, int B, void *stream);

/* The same bookkeeping after a one-pass prefill, where every sequence sits at its own position (section
 * 6.6's loop with per-sequence step counters): tokens_out[b] = last_sampled[b];
 * positions_out[b] = base_positions[b] + j.  All arrays [B] int32; j >= 0. */
int det_decode_advance(const int32_t *last_sampled, const int32_t *base_positions, int j, int32_t *tokens_out,
                       int32_t *positions_out, int B, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Deterministic block-quantized GEMM (the paper's primary kernel family is the quantized one, section
 * 6.4 and Table 5; it gives no format, so one is defined here).
 *
 *   weights, block = 64 consecutive k of one column:   amax = max|w|; s = bf16(amax / 7);
 *       q = clamp(rint(w / s), -8, 7), 0 if s == 0                      (4-bit code, bf16 scale)
 *   activations, block = 64 consecutive k of one row:  amax = max|a|; d = amax / 127 (fp32);
 *       p = clamp(rint(a / d), -127, 127), 0 if d == 0                  (8-bit code, fp32 scale)
 *   C[i][n] = bf16(acc) (or acc as fp32), acc = 0; for blocks b ascending:
 *       acc = fma( d[i][b] * s[b][n], (float)(sum over the block of p*q, int32), acc )
 *   All of it IEEE fp32 with round-to-nearest-even; the result is a pure function of the operand
 *   bytes and is reproduced bit for bit by a plain CPU implementation.  NaN/Inf inputs and blocks
 *   whose largest magnitude is denormal are unspecified.
 *
 * det_quant_pack_w4: one-time; B_kn is bf16 row-major [K,N]; `packed` (det_qgemm_packed_w_bytes
 * bytes, 16-byte aligned, 4.25 bits per weight) is in the kernel's streaming order.  N % 16 == 0,
 * K % 64 == 0, else DET_ESHAPE.  det_quant_unpack_w4 is a test hook: codes int8 [K,N] and scales bf16
 * [K/64,N] back out of a packed matrix.
 * det_quant_act_q8: A bf16 [M,K] with row stride lda -> codes (det_quant_act_codes_bytes: int8
 * [M,K]) and scales (det_quant_act_scales_bytes: fp32, block-major with row stride (M+3)&~3, so a
 * test reads scale (i, b) at scales[b * ((M+3)&~3) + i]); both 16-byte aligned.
 * det_qgemm_w4a8: C [M,N] with row stride ldc (ldc % 4 == 0), out_dtype DET_BF16 or DET_F32; codes and
 * scales as written by det_quant_act_q8 for the same M and K.  Device pointers; work is enqueued on
 * `stream`. */
size_t det_qgemm_packed_w_bytes(int N, int K);
int det_quant_pack_w4(const void *B_kn, void *packed, int N, int K, void *stream);
int det_quant_unpack_w4(const void *packed, void *codes, void *scales, int N, int K, void *stream);
size_t det_quant_act_codes_bytes(int M, int K);
size_t det_quant_act_scales_bytes(int M, int K);
int det_quant_act_q8(const void *A, int lda, void *codes, void *scales, int M, int K, void *stream);
int det_qgemm_w4a8(const void *codes, const void *scales, const void *packed_w, void *C, int ldc, int M,
                   int N, int K, int out_dtype, void *stream);

/* Fused forms for the quantized decoder layer; each gives the bytes of the unfused sequence.
 * det_quant_pack_w4_gate_up: det_quant_pack_w4 of a [K, 2F] matrix (F gate columns, then F up columns)
 *   with gate_j and up_j made neighbours, for det_qgemm_w4a8_swiglu.  F % 8 == 0.
 * det_qgemm_w4a8_residual: C = det_residual_add(R, det_qgemm_w4a8(...) as bf16); C may be R.  R bf16 [M,N]
 *   with row stride ldr (ldr % 4 == 0).
 * det_qgemm_w4a8_swiglu: Y[M,F] = det_swiglu(g, u), [g | u] = det_qgemm_w4a8 of the [K, 2F] matrix as bf16;
 *   packed_gate_up from det_quant_pack_w4_gate_up; ldy >= F, ldy % 4 == 0.
 * det_rmsnorm_quant_q8: det_quant_act_q8(det_rmsnorm(x, w)) without the bf16 round trip through memory:
 *   codes int8 [M,H] and scales as det_quant_act_q8 writes them for (M, K = H).  H % 64 == 0, H <= 16384. */
int det_quant_pack_w4_gate_up(const void *B_kn, void *packed, int F, int K, void *stream);
int det_qgemm_w4a8_residual(const void *codes, const void *scales, const void *packed_w, const void *R,
                            int ldr, void *C, int ldc, int M, int N, int K, void *stream);
int det_qgemm_w4a8_swiglu(const void *codes, const void *scales, const void *packed_gate_up, void *Y,
                          int ldy, int M, int F, int K, void *stream);
/* det_quant_pack_w4_qkv / det_qgemm_w4a8_qkv_rope_append: the quantized layer's fused projection, as
 *   det_gemm_pack_qkv / det_gemm_qkv_rope_append are the bf16 layer's: the packing makes the columns d
 *   and d + D/2 of every head neighbours (the quantizer's blocks run along K, so codes and scales are
 *   those of det_quant_pack_w4 in another column order), and the GEMM's epilogue rotates the query and
 *   key heads at the row's position and writes query heads to qbuf, key and value heads to the row's
 *   cache slot: the bytes of det_qgemm_w4a8 (bf16 out), det_rope and the append.  D must be 128. */
int det_quant_pack_w4_qkv(const void *B_kn, void *packed, int Hq, int Hkv, int D, int K, void *stream);
int det_qgemm_w4a8_qkv_rope_append(const void *codes, const void *scales, const void *packed_qkv,
                                   void *qbuf, void *kcache, void *vcache, const int32_t *positions,
                                   const int32_t *slots, const float *rope_cos, const float *rope_sin,
                                   int M, int Hq, int Hkv, int D, int Lmax, int K, void *stream);
int det_rmsnorm_quant_q8(const void *x, const void *w, void *codes, void *scales, int M, int H, float eps,
                         void *stream);
/* det_attn_decode_quant_q8: det_quant_act_q8 of the [R, Hq*D] output of det_attn_decode_rows (slots may be
 *   NULL: row r reads cache slot r, as det_attn_decode), written as codes int8 [R, Hq*D] and scales for
 *   (M = R, K = Hq*D); other arguments and errors as det_attn_decode_rows. */
/* det_qgemm_w4a8_swiglu_quant: det_quant_act_q8 of the [M, F] output of det_qgemm_w4a8_swiglu, written as codes_out
 *   int8 [M, F] and scales_out for (M, K = F), without the bf16 round trip.  Only where the kernel's tile
 *   is 128 packed columns wide (then a tile row is exactly one 64-output block):
 *   det_qgemm_w4a8_swiglu_quant_supported(F, K) != 0, else DET_ESHAPE; F % 64 == 0.  codes_out / scales_out
 *   must not be the input codes / scales. */
int det_qgemm_w4a8_swiglu_quant_supported(int F, int K);
int det_qgemm_w4a8_swiglu_quant(const void *codes, const void *scales, const void *packed_gate_up,
                                void *codes_out, void *scales_out, int M, int F, int K, void *stream);
int det_attn_decode_quant_q8(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                             const int32_t *slots, void *codes, void *scales, void *ws, size_t ws_bytes,
                             int R, int Hq, int Hkv, int D, int Lmax, float scale, void *stream);

/* The decoder layer with every projection block-quantized (the engine the paper measures runs
 * quantized models, section 6.4): the steps of det_decoder_layer in the same order, each projection
 * det_qgemm_w4a8 on the det_quant_act_q8 codes of the bf16 activations it would have taken.  Weights:
 * w_norm1, w_norm2 bf16 [H]; wqkv from det_quant_pack_w4_qkv; wo, wdown from det_quant_pack_w4; wgu from
 * det_quant_pack_w4_gate_up.  Other arguments as det_decoder_layer_rows; slots may be NULL (row r is
 * the sequence in cache slot r).  Same invariance: a row's bytes and its cache rows do not depend on
 * R or on the other rows.  Workspace: det_qdecoder_layer_workspace_bytes(cfg, R). */
size_t det_qdecoder_layer_workspace_bytes(const det_layer_cfg *cfg /* host */, int R);
int det_qdecoder_layer(const det_layer_weights *w, const det_layer_cfg *cfg, void *x_inout, void *kcache,
                       void *vcache, const int32_t *positions, const int32_t *slots,
                       const float *rope_cos, const float *rope_sin, void *ws, size_t ws_bytes, int R,
                       void *stream);

/* ---------------------------------------------------------------------------------------------
 * Output commitment (the paper's section 6.7 records SHA256(prompt || logits || tokens) for every
 * execution, and a receipt commits to the output by its hash, section 4.1).  HOST code on HOST
 * pointers: SHA-256 (FIPS 180-4) is a serial chain, so the caller copies what it wants committed
 * to host memory (per step, overlapped with the next step) and feeds it here.
 *
 * det_sha256_init / _update / _final: streaming interface; the context is caller-owned plain data
 * (no allocation); after _final the context is spent and must be re-initialised.  DET_EINVAL for
 * null pointers or a spent context.  det_commit_sha256: the three byte strings hashed in the
 * paper's order in one call; a length may be 0 (its pointer is then ignored).  The digest is the 32
 * bytes in the standard's order (big-endian words).  The bytes hashed are the caller's: this
 * library's convention (tests, decode loop) is int32 little-endian token ids and fp32 little-endian
 * logits, step-major. */
typedef struct det_sha256_ctx {
    uint32_t h[8];
    uint64_t nbytes;
    uint8_t buf[64];
    uint32_t fill;
} det_sha256_ctx;
int det_sha256_init(det_sha256_ctx *ctx);
int det_sha256_update(det_sha256_ctx *ctx, const void *data, size_t bytes);
int det_sha256_final(det_sha256_ctx *ctx, uint8_t digest[32]);
int det_commit_sha256(const void *prompt, size_t prompt_bytes, const void *logits, size_t logits_bytes,
                      const void *tokens, size_t tokens_bytes, uint8_t digest[32]);
/* Test hook: nonzero makes the calls above use the portable compression function even where the
 * CPU has SHA instructions (process-wide). */
int det_sha256_force_portable(int on);

/* Measurement aid (not part of the decode path): `workgroups` workgroups of 256 threads each stream the
 * buffer src (src_bytes, at most 1 GiB, every workgroup the same bytes, so that they come from L2) into
 * their LDS `iters` times 32 KB, path 0 through registers and LDS stores, path 1 with LDS-DMA loads.
 * Moves workgroups * iters * 32768 bytes; the caller times it.  sink: 4 bytes, never written in practice. */
int det_probe_lds_fill(const void *src, size_t src_bytes, int path, int workgroups, int iters, void *sink,
                       void *stream);

/* Build identification: target architecture, ROCm version the library was built with, and the
 * kernel-configuration revision (echoes the paper's `system_fingerprint` response field, section
 * 7.1).  Static storage; host pointer. */
const char *det_fingerprint(void);

/* hipError_t value of the last failed HIP call on the calling thread (0 if none). */
int det_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DETINFER_H */
