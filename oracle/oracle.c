/*
 * CPU oracle for the deterministic decode path.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * path may call into this file; it exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg have an independent statement of what each operation computes.  It shares no
 * code, table or helper with the HIP kernels.
 *
 * Two kinds of function:
 *   T  "tolerance" references: the plain mathematical definition evaluated in fp64 from the exact
 *      bf16 inputs (GEMM, attention, the contractions inside the decoder layer).  The GPU reaches
 *      an fp32 approximation of these in a hardware-defined order, so they are compared within a
 *      stated bound, never by bytes (the paper reports a 0 % bit match across architectures,
 *      section 6.7, Table 4).
 *   X  bit-exact references: an fp32 emulation, step by step, of the canonical reduction order
 *      (RMSNorm, softmax statistics, argmax, det_expf, bf16 rounding, RoPE, SwiGLU, residual,
 *      seeded sampling, the quantizers and the quantized GEMM, whose contraction is integer).
 *
 * The canonical order follows the paper's three kernel invariants (section 6.5): a fixed mapping
 * of work to threads, a stride-halving binary-tree reduction (the four-line shuffle loop of
 * section 6.5, paragraph 2, written for a 64-wide wavefront; tree shape of Fig. "kernel_tree"),
 * and no atomics: every accumulation has a written order.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py (closed forms, brute
 * force, exact-arithmetic cases, library routines).  Nothing here is "parity unpinned" except
 * behaviour on NaN/Inf inputs, which the method leaves unspecified.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -mfma -mavx2 (no fast-math: every fp32 operation
 * below is individually rounded, and fmaf() is a single rounding).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- bit helpers */

static inline uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* bf16 -> fp32 is exact: the 16 bits become the upper half of the fp32 pattern. */
float orc_bf16_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }

/* X: fp32 -> bf16, round to nearest, ties to even; NaN -> 0x7FC0; overflow -> +-inf. */
uint16_t orc_bf16_rne(float f)
{
    uint32_t u = f32_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

void orc_bf16_rne_array(const float *x, uint16_t *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = orc_bf16_rne(x[i]);
}

/* fp64 -> bf16 with a single rounding (nearest even).  Used where a T reference in fp64 has to be
 * handed on as a bf16 activation (decoder layer): going through fp32 first could round twice. */
uint16_t orc_bf16_from_f64(double d)
{
    if (d != d) return 0x7FC0;
    if (d == 0.0) return signbit(d) ? 0x8000 : 0x0000;
    double a = fabs(d);
    if (a >= 3.3961775292304601e38) /* >= max bf16 + half an ulp */
        return signbit(d) ? 0xFF80 : 0x7F80;
    int e;
    (void)frexp(a, &e);               /* a = m * 2^e, m in [0.5,1) */
    int E = e - 1;                    /* a = (2m) * 2^E, 2m in [1,2) */
    if (E < -126) E = -126;           /* bf16 subnormals share the fp32 exponent floor */
    double q = ldexp(a, 7 - E);       /* mantissa scaled to integer units of one bf16 ulp */
    double r = nearbyint(q);          /* default rounding mode: nearest even */
    float f = (float)ldexp(r, E - 7); /* exact: at most 8 significant bits */
    uint16_t b = (uint16_t)(f32_bits(f) >> 16);
    return signbit(d) ? (uint16_t)(b | 0x8000) : b;
}

/* ---------------------------------------------------------------- det_expf (X) */

/* exp(x) from fp32 multiply, round-to-integer, fused multiply-add and an integer exponent add.
 * n = rint(x*log2e); r = x - n*ln2 in two fma steps; degree-7 Taylor polynomial of exp(r) in
 * Horner form; the result is the polynomial with n added to its exponent field.
 * x > 88.72 -> +inf, x < -87 -> 0 (so no subnormal results), NaN -> quiet NaN 0x7FC00000. */
float orc_expf(float x)
{
    if (x != x) return bits_f32(0x7FC00000u);
    if (x > 88.72f) return bits_f32(0x7F800000u);
    if (x < -87.0f) return 0.0f;
    const float log2e = 0x1.715476p+0f;
    const float ln2_hi = 0x1.62e4p-1f;
    const float ln2_lo = 0x1.7f7d1cp-20f;
    float t = x * log2e;
    float n = rintf(t);
    float r = fmaf(n, -ln2_hi, x);
    r = fmaf(n, -ln2_lo, r);
    float p = 0x1.a01a02p-13f;          /* 1/5040 */
    p = fmaf(p, r, 0x1.6c16c2p-10f);    /* 1/720  */
    p = fmaf(p, r, 0x1.111112p-7f);     /* 1/120  */
    p = fmaf(p, r, 0x1.555556p-5f);     /* 1/24   */
    p = fmaf(p, r, 0x1.555556p-3f);     /* 1/6    */
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    int32_t ni = (int32_t)n;
    return bits_f32((uint32_t)((int32_t)f32_bits(p) + ni * (1 << 23)));
}

void orc_expf_array(const float *x, float *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = orc_expf(x[i]);
}

/* ---------------------------------------------------------------- canonical tree (X) */

/* Sum of 256 fp32 leaves.  Within each aligned group of 64 leaves, six stride-halving levels
 * (offsets 32,16,8,4,2,1): leaf i takes leaf i+off for i mod 64 < off.  The four group sums
 * q0..q3 are then combined as (q0+q2)+(q1+q3), i.e. the same stride-halving rule on four leaves.
 * Every addition is a separately rounded fp32 add. */
float orc_tree256(const float *leaves)
{
    float t[256];
    memcpy(t, leaves, sizeof t);
    for (int off = 32; off > 0; off /= 2)
        for (int g = 0; g < 256; g += 64)
            for (int i = 0; i < off; ++i)
                t[g + i] = t[g + i] + t[g + i + off];
    float a = t[0] + t[128];
    float b = t[64] + t[192];
    return a + b;
}

/* ---------------------------------------------------------------- RMSNorm (X) */

/* y = bf16( (x*r)*w ), r = 1/sqrt(mean(x^2)+eps).
 * Sum of squares: element e belongs to lane (e/8) mod 256; each lane folds its elements in
 * ascending e into one fp32 accumulator with fma(x,x,acc) from +0; the 256 lane sums go through
 * the canonical tree.  mean = ss/H, r = 1/sqrt(mean+eps) with correctly rounded divide and sqrt;
 * two separately rounded multiplies, one rounding to bf16. */
float orc_sumsq(const uint16_t *x, int H)
{
    float acc[256];
    for (int l = 0; l < 256; ++l) acc[l] = 0.0f;
    for (int e = 0; e < H; ++e) {
        float v = orc_bf16_to_f32(x[e]);
        int lane = (e / 8) % 256;
        acc[lane] = fmaf(v, v, acc[lane]);
    }
    return orc_tree256(acc);
}

void orc_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int M, int H, float eps)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        const uint16_t *xi = x + (int64_t)i * H;
        float ss = orc_sumsq(xi, H);
        float mean = ss / (float)H;
        float r = 1.0f / sqrtf(mean + eps);
        for (int e = 0; e < H; ++e) {
            float v = orc_bf16_to_f32(xi[e]);
            float s = v * r;
            float o = s * orc_bf16_to_f32(w[e]);
            y[(int64_t)i * H + e] = orc_bf16_rne(o);
        }
    }
}

/* ---------------------------------------------------------------- chunked softmax (X) */

/* Statistics of one row of fp32 scores of length len, over fixed 256-token chunks.
 * Chunk c covers tokens [256c, min(256c+256,len)):  m_c = max score;  e_j = det_expf(s_j - m_c)
 * (0 for tokens at or past len);  l_c = tree256(e) with leaf index j - 256c.
 * Combine in ascending c:  m = max_c m_c;  w_c = det_expf(m_c - m);  L = sum_c w_c*l_c folded
 * from +0 with separate multiply and add.  p_j = (w_c*e_j)/L.
 * len <= 0: m = -inf, L = 0, nothing written to p. */
static void softmax_row(const float *s, int len, float *p, float *m_out, float *l_out)
{
    if (len <= 0) {
        *m_out = -INFINITY;
        *l_out = 0.0f;
        return;
    }
    int nc = (len + 255) / 256;
    float *mc = (float *)malloc(sizeof(float) * nc);
    float *lc = (float *)malloc(sizeof(float) * nc);
    float *e = (float *)malloc(sizeof(float) * (size_t)nc * 256);
    for (int c = 0; c < nc; ++c) {
        int lo = 256 * c, hi = lo + 256 < len ? lo + 256 : len;
        float m = s[lo];
        for (int j = lo + 1; j < hi; ++j)
            if (s[j] > m) m = s[j];
        mc[c] = m;
        float *ec = e + (size_t)c * 256;
        for (int t = 0; t < 256; ++t) {
            int j = lo + t;
            ec[t] = j < hi ? orc_expf(s[j] - m) : 0.0f;
        }
        lc[c] = orc_tree256(ec);
    }
    float m = mc[0];
    for (int c = 1; c < nc; ++c)
        if (mc[c] > m) m = mc[c];
    float L = 0.0f;
    for (int c = 0; c < nc; ++c) {
        float w = orc_expf(mc[c] - m);
        float wl = w * lc[c];
        L = L + wl;
    }
    if (p) {
        for (int c = 0; c < nc; ++c) {
            float w = orc_expf(mc[c] - m);
            int lo = 256 * c, hi = lo + 256 < len ? lo + 256 : len;
            for (int j = lo; j < hi; ++j) {
                float we = w * e[(size_t)c * 256 + (j - lo)];
                p[j] = we / L;
            }
        }
    }
    *m_out = m;
    *l_out = L;
    free(mc);
    free(lc);
    free(e);
}

/* s, p: [R, Lmax] fp32; lens: [R]; m_out, l_out: [R].  p entries at or past lens[r] are left
 * untouched. */
void orc_softmax_f32(const float *s, const int32_t *lens, float *p, float *m_out, float *l_out,
                     int R, int Lmax)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < R; ++r)
        softmax_row(s + (int64_t)r * Lmax, lens[r], p ? p + (int64_t)r * Lmax : NULL, m_out + r,
                    l_out + r);
}

/* ---------------------------------------------------------------- argmax (X) */

/* Smallest index attaining the maximum.  -0 == +0.  NaN never wins; a row of NaNs gives 0.
 * (max, lowest index) is associative and commutative, so any reduction tree gives this. */
void orc_argmax_f32(const float *logits, int32_t *idx, int B, int V)
{
    for (int b = 0; b < B; ++b) {
        const float *r = logits + (int64_t)b * V;
        int best = -1;
        float bv = 0.0f;
        for (int j = 0; j < V; ++j) {
            float v = r[j];
            if (v != v) continue;
            if (best < 0 || v > bv) { best = j; bv = v; }
        }
        idx[b] = best < 0 ? 0 : best;
    }
}

void orc_argmax_bf16(const uint16_t *logits, int32_t *idx, int B, int V)
{
    for (int b = 0; b < B; ++b) {
        const uint16_t *r = logits + (int64_t)b * V;
        int best = -1;
        float bv = 0.0f;
        for (int j = 0; j < V; ++j) {
            float v = orc_bf16_to_f32(r[j]);
            if (v != v) continue;
            if (best < 0 || v > bv) { best = j; bv = v; }
        }
        idx[b] = best < 0 ? 0 : best;
    }
}

/* ---------------------------------------------------------------- GEMM (T) */

/* C[i][j] = sum_k A[i][k]*B[k][j] in fp64 from bf16 inputs; Cabs[i][j] = sum_k |A[i][k]*B[k][j]|
 * (the magnitude the error bound is stated against).  A: [M,K] row-major with row stride lda;
 * B: [K,N] row-major; C, Cabs: [M,N].  Cabs may be NULL. */
void orc_gemm_f64(const uint16_t *A, int lda, const uint16_t *B, double *C, double *Cabs, int M,
                  int N, int K)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        double *c = C + (int64_t)i * N;
        double *ca = Cabs ? Cabs + (int64_t)i * N : NULL;
        for (int j = 0; j < N; ++j) c[j] = 0.0;
        if (ca)
            for (int j = 0; j < N; ++j) ca[j] = 0.0;
        for (int k = 0; k < K; ++k) {
            double a = (double)orc_bf16_to_f32(A[(int64_t)i * lda + k]);
            const uint16_t *b = B + (int64_t)k * N;
            for (int j = 0; j < N; ++j) {
                double t = a * (double)orc_bf16_to_f32(b[j]);
                c[j] += t;
                if (ca) ca[j] += fabs(t);
            }
        }
    }
}

/* The same definition at ns sampled positions (rows[s], cols[s]); used at sizes where the full
 * product would take too long on the host. */
void orc_gemm_f64_sample(const uint16_t *A, int lda, const uint16_t *B, const int32_t *rows,
                         const int32_t *cols, double *c, double *cabs, int ns, int N, int K)
{
#pragma omp parallel for schedule(static)
    for (int s = 0; s < ns; ++s) {
        int i = rows[s], j = cols[s];
        double acc = 0.0, aa = 0.0;
        for (int k = 0; k < K; ++k) {
            double t = (double)orc_bf16_to_f32(A[(int64_t)i * lda + k]) *
                       (double)orc_bf16_to_f32(B[(int64_t)k * N + j]);
            acc += t;
            aa += fabs(t);
        }
        c[s] = acc;
        if (cabs) cabs[s] = aa;
    }
}

/* ---------------------------------------------------------------- attention decode (T) */

/* One query token per sequence against its KV cache, grouped-query heads: query head h reads KV
 * head h / (Hq/Hkv).  s_j = scale * (q . k_j) for j < len;  p = softmax(s);  out = sum_j p_j v_j.
 * All in fp64.  outabs[d] = sum_j p_j |v_jd|.  len <= 0 gives zeros.
 * q: [B,Hq,D] bf16; kcache, vcache: [B,Hkv,Lmax,D] bf16; out, outabs: [B,Hq,D] fp64. */
void orc_attn_decode_f64(const uint16_t *q, const uint16_t *kcache, const uint16_t *vcache,
                         const int32_t *seqlens, double *out, double *outabs, int B, int Hq, int Hkv,
                         int D, int Lmax, float scale)
{
    int group = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            int len = seqlens[b];
            double *o = out + ((int64_t)b * Hq + h) * D;
            double *oa = outabs ? outabs + ((int64_t)b * Hq + h) * D : NULL;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            if (oa)
                for (int d = 0; d < D; ++d) oa[d] = 0.0;
            if (len <= 0) continue;
            int kvh = h / group;
            const uint16_t *kk = kcache + ((int64_t)b * Hkv + kvh) * (int64_t)Lmax * D;
            const uint16_t *vv = vcache + ((int64_t)b * Hkv + kvh) * (int64_t)Lmax * D;
            const uint16_t *qq = q + ((int64_t)b * Hq + h) * D;
            double *s = (double *)malloc(sizeof(double) * len);
            double m = -INFINITY;
            for (int j = 0; j < len; ++j) {
                double acc = 0.0;
                for (int d = 0; d < D; ++d)
                    acc += (double)orc_bf16_to_f32(qq[d]) *
                           (double)orc_bf16_to_f32(kk[(int64_t)j * D + d]);
                s[j] = (double)scale * acc;
                if (s[j] > m) m = s[j];
            }
            double denom = 0.0;
            for (int j = 0; j < len; ++j) {
                s[j] = exp(s[j] - m);
                denom += s[j];
            }
            for (int j = 0; j < len; ++j) {
                double p = s[j] / denom;
                for (int d = 0; d < D; ++d) {
                    double v = (double)orc_bf16_to_f32(vv[(int64_t)j * D + d]);
                    o[d] += p * v;
                    if (oa) oa[d] += p * fabs(v);
                }
            }
            free(s);
        }
    }
}

/* ---------------------------------------------------------------- elementwise (X) */

/* Rotary embedding, rotate-half pairing (i, i+D/2), on nh heads of one token per row.
 * x: [R, nh, D] bf16 in, y same shape out; pos[R]; cos_t, sin_t: [Lmax, D/2] fp32.
 *   y_lo = bf16( fma(-x_hi, sin, x_lo*cos) ),  y_hi = bf16( fma(x_lo, sin, x_hi*cos) ). */
void orc_rope(const uint16_t *x, uint16_t *y, const int32_t *pos, const float *cos_t,
              const float *sin_t, int R, int nh, int D)
{
    int half = D / 2;
    for (int r = 0; r < R; ++r)
        for (int h = 0; h < nh; ++h) {
            const uint16_t *xi = x + ((int64_t)r * nh + h) * D;
            uint16_t *yi = y + ((int64_t)r * nh + h) * D;
            for (int i = 0; i < half; ++i) {
                float c = cos_t[(int64_t)pos[r] * half + i];
                float s = sin_t[(int64_t)pos[r] * half + i];
                float lo = orc_bf16_to_f32(xi[i]);
                float hi = orc_bf16_to_f32(xi[i + half]);
                float a = lo * c;
                float b = hi * c;
                yi[i] = orc_bf16_rne(fmaf(-hi, s, a));
                yi[i + half] = orc_bf16_rne(fmaf(lo, s, b));
            }
        }
}

/* SiLU(g)*u: sig = g / (1 + det_expf(-g)) with a correctly rounded divide, one multiply by u,
 * one rounding to bf16.  g, u: n bf16 values each. */
void orc_swiglu(const uint16_t *g, const uint16_t *u, uint16_t *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        float gv = orc_bf16_to_f32(g[i]);
        float uv = orc_bf16_to_f32(u[i]);
        float den = 1.0f + orc_expf(-gv);
        float sg = gv / den;
        y[i] = orc_bf16_rne(sg * uv);
    }
}

/* Residual add: bf16( fp32(x) + fp32(y) ). */
void orc_residual(const uint16_t *x, const uint16_t *y, uint16_t *z, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        z[i] = orc_bf16_rne(orc_bf16_to_f32(x[i]) + orc_bf16_to_f32(y[i]));
}

/* ---------------------------------------------------------------- decoder layer (T around X) */

/* GEMM in fp64 whose result is handed on as a bf16 activation (single rounding). */
static void gemm_to_bf16(const uint16_t *A, const uint16_t *Bm, uint16_t *C, int M, int N, int K)
{
    double *c = (double *)malloc(sizeof(double) * (size_t)M * N);
    orc_gemm_f64(A, K, Bm, c, NULL, M, N, K);
    for (int64_t i = 0; i < (int64_t)M * N; ++i) C[i] = orc_bf16_from_f64(c[i]);
    free(c);
}

/* One Llama-style decoder layer on one new token per sequence:
 *   h = rmsnorm(x, w_norm1);  [q|k|v] = h Wqkv;  rope(q), rope(k) at positions[b];
 *   k, v written to the caches at positions[b];  a = attention(q, caches, len = positions[b]+1);
 *   x = x + a Wo;  h = rmsnorm(x, w_norm2);  [g|u] = h Wgu;  m = silu(g)*u;  x = x + m Wdown.
 * Contractions are fp64 references rounded once to bf16; every other step is the bit-exact
 * canonical form above.  Weights are logical [K,N] row-major bf16:
 *   wqkv [H,(Hq+2Hkv)D] with columns ordered q heads, k heads, v heads;  wo [Hq*D,H];
 *   wgu [H,2F] with columns ordered gate, up;  wdown [F,H].
 * x: [B,H] in/out.  kcache, vcache: [B,Hkv,Lmax,D] in/out. */
void orc_decoder_layer(uint16_t *x, const uint16_t *w_norm1, const uint16_t *wqkv,
                       const uint16_t *wo, const uint16_t *w_norm2, const uint16_t *wgu,
                       const uint16_t *wdown, uint16_t *kcache, uint16_t *vcache,
                       const int32_t *positions, const float *cos_t, const float *sin_t, int B,
                       int H, int Hq, int Hkv, int D, int F, int Lmax, float eps, float scale)
{
    int Nqkv = (Hq + 2 * Hkv) * D;
    uint16_t *h = (uint16_t *)malloc(2 * (size_t)B * H);
    uint16_t *qkv = (uint16_t *)malloc(2 * (size_t)B * Nqkv);
    uint16_t *qr = (uint16_t *)malloc(2 * (size_t)B * Hq * D);
    uint16_t *kr = (uint16_t *)malloc(2 * (size_t)B * Hkv * D);
    uint16_t *att = (uint16_t *)malloc(2 * (size_t)B * Hq * D);
    uint16_t *proj = (uint16_t *)malloc(2 * (size_t)B * H);
    uint16_t *gu = (uint16_t *)malloc(2 * (size_t)B * 2 * F);
    uint16_t *mm = (uint16_t *)malloc(2 * (size_t)B * F);
    double *ao = (double *)malloc(sizeof(double) * (size_t)B * Hq * D);
    int32_t *lens = (int32_t *)malloc(sizeof(int32_t) * B);

    orc_rmsnorm(x, w_norm1, h, B, H, eps);
    gemm_to_bf16(h, wqkv, qkv, B, Nqkv, H);
    for (int b = 0; b < B; ++b) {
        const uint16_t *row = qkv + (int64_t)b * Nqkv;
        orc_rope(row, qr + (int64_t)b * Hq * D, positions + b, cos_t, sin_t, 1, Hq, D);
        orc_rope(row + Hq * D, kr + (int64_t)b * Hkv * D, positions + b, cos_t, sin_t, 1, Hkv, D);
        for (int g = 0; g < Hkv; ++g) {
            int64_t dst = (((int64_t)b * Hkv + g) * Lmax + positions[b]) * D;
            memcpy(kcache + dst, kr + ((int64_t)b * Hkv + g) * D, 2 * (size_t)D);
            memcpy(vcache + dst, row + (Hq + Hkv) * D + g * D, 2 * (size_t)D);
        }
        lens[b] = positions[b] + 1;
    }
    orc_attn_decode_f64(qr, kcache, vcache, lens, ao, NULL, B, Hq, Hkv, D, Lmax, scale);
    for (int64_t i = 0; i < (int64_t)B * Hq * D; ++i) att[i] = orc_bf16_from_f64(ao[i]);
    gemm_to_bf16(att, wo, proj, B, H, Hq * D);
    orc_residual(x, proj, x, (int64_t)B * H);
    orc_rmsnorm(x, w_norm2, h, B, H, eps);
    gemm_to_bf16(h, wgu, gu, B, 2 * F, H);
    for (int b = 0; b < B; ++b)
        orc_swiglu(gu + (int64_t)b * 2 * F, gu + (int64_t)b * 2 * F + F, mm + (int64_t)b * F, F);
    gemm_to_bf16(mm, wdown, proj, B, H, F);
    orc_residual(x, proj, x, (int64_t)B * H);

    free(h); free(qkv); free(qr); free(kr); free(att); free(proj); free(gu); free(mm); free(ao);
    free(lens);
}

/* ---------------------------------------------------------------- seeded sampling (X) */

/* Counter-based uniform in [0,1): the splitmix64 output function applied to
 * seed + (((uint64)seq_id << 32 | (uint32)step) + 1) * 0x9E3779B97F4A7C15, top 24 bits scaled by 2^-24.
 * A sample depends on (seed, sequence id, step) only, never on the batch (section 6.6: fixed-seed
 * PRNG, reproducible per (seed, decode policy)). */
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

float orc_sample_uniform(uint64_t seed, int32_t seq_id, int32_t step)
{
    uint64_t ctr = ((uint64_t)(uint32_t)seq_id << 32) | (uint64_t)(uint32_t)step;
    uint64_t r = mix64(seed + (ctr + 1) * 0x9E3779B97F4A7C15ull);
    return (float)(r >> 40) * 0x1p-24f;
}

typedef struct { float z; int32_t idx; } zi_t;

/* canonical order of candidates: larger z first; equal z: smaller index first */
static int zi_cmp(const void *a, const void *b)
{
    const zi_t *x = (const zi_t *)a, *y = (const zi_t *)b;
    if (x->z > y->z) return -1;
    if (x->z < y->z) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* Temperature / top-k / top-p sampling in a canonical iteration order (section 6.6).
 *   z_j = logits_j / T (fp32 divide; NaN counts as -inf);  candidates sorted by (z desc, index asc);
 *   the first k = min(top_k, V) kept;  e_i = det_expf(z_i - z_0);  c_i = c_{i-1} + e_i in rank
 *   order (sequential fp32 adds from +0);  n = the smallest i+1 with c_i >= top_p * c_{k-1};
 *   target = u * c_{n-1};  the token is the candidate of the smallest rank i < n with
 *   c_i > target (rank n-1 if rounding leaves none).
 * logits [B,V] fp32; seq_ids, steps [B]; tokens [B]. */
void orc_sample(const float *logits, int B, int V, float temperature, int top_k, float top_p,
                uint64_t seed, const int32_t *seq_ids, const int32_t *steps, int32_t *tokens)
{
    for (int b = 0; b < B; ++b) {
        zi_t *c = (zi_t *)malloc(sizeof(zi_t) * (size_t)V);
        for (int j = 0; j < V; ++j) {
            float z = logits[(int64_t)b * V + j] / temperature;
            if (z != z) z = -INFINITY;
            c[j].z = z;
            c[j].idx = j;
        }
        qsort(c, (size_t)V, sizeof(zi_t), zi_cmp);
        int k = top_k < V ? top_k : V;
        float *cum = (float *)malloc(sizeof(float) * (size_t)k);
        float acc = 0.0f;
        for (int i = 0; i < k; ++i) {
            float e = orc_expf(c[i].z - c[0].z);
            acc = acc + e;
            cum[i] = acc;
        }
        float cut = top_p * cum[k - 1];
        int n = k;
        for (int i = 0; i < k; ++i)
            if (cum[i] >= cut) { n = i + 1; break; }
        float u = orc_sample_uniform(seed, seq_ids[b], steps[b]);
        float target = u * cum[n - 1];
        int pick = n - 1;
        for (int i = 0; i < n; ++i)
            if (cum[i] > target) { pick = i; break; }
        tokens[b] = c[pick].idx;
        free(cum);
        free(c);
    }
}

/* Threads the parallel loops above will use (reported with the CPU baseline). */
/* ---------------------------------------------------------------------------------------------
 * Deterministic quantized GEMM (the paper's primary kernel family is the quantized one: section
 * 6.4 names the quantized warp-synchronous kernels of its engine, Table 5 measures them).  The
 * paper gives no format; this one is defined here, integer where it can be so that the whole
 * operation has a bit-exact reference (X):
 *
 *   weights, block = 64 consecutive k of one column:  amax = max |w|;  s = bf16(amax / 7);
 *       q_k = clamp(rint(w_k / s), -8, 7)  (0 if s == 0);            w_k ~ s * q_k
 *   activations, block = 64 consecutive k of one row: amax = max |a|;  d = amax / 127 (fp32);
 *       p_k = clamp(rint(a_k / d), -127, 127)  (0 if d == 0);        a_k ~ d * p_k
 *   C[i][n] = bf16( acc ),  acc = 0;  for b = 0 .. K/64-1 ascending:
 *       P = sum_{k in block b} p_k * q_k            (int32, exact, any order)
 *       acc = fmaf( d[i][b] * s[b][n], (float)P, acc )     (one rounded multiply, one fma)
 *
 * All divisions and multiplies are IEEE fp32, rint is round-to-nearest-even.  NaN/Inf inputs and
 * blocks whose amax is denormal are unspecified.
 */
void orc_quant_w4(const uint16_t *W, int K, int N, int8_t *q, uint16_t *s)
{
    const int nb = K / 64;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int b = 0; b < nb; ++b) {
            float amax = 0.0f;
            for (int k = 64 * b; k < 64 * b + 64; ++k) {
                const float a = fabsf(orc_bf16_to_f32(W[(size_t)k * N + n]));
                if (a > amax) amax = a;
            }
            const uint16_t sb = orc_bf16_rne(amax / 7.0f);
            const float sf = orc_bf16_to_f32(sb);
            s[(size_t)b * N + n] = sb;
            for (int k = 64 * b; k < 64 * b + 64; ++k) {
                int v = 0;
                if (sf != 0.0f) {
                    const float r = nearbyintf(orc_bf16_to_f32(W[(size_t)k * N + n]) / sf);
                    v = r < -8.0f ? -8 : (r > 7.0f ? 7 : (int)r);
                }
                q[(size_t)k * N + n] = (int8_t)v;
            }
        }
}

void orc_quant_a8(const uint16_t *A, int lda, int M, int K, int8_t *p, float *d)
{
    const int nb = K / 64;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int b = 0; b < nb; ++b) {
            float amax = 0.0f;
            for (int k = 64 * b; k < 64 * b + 64; ++k) {
                const float a = fabsf(orc_bf16_to_f32(A[(size_t)i * lda + k]));
                if (a > amax) amax = a;
            }
            const float df = amax / 127.0f;
            d[(size_t)i * nb + b] = df;
            for (int k = 64 * b; k < 64 * b + 64; ++k) {
                int v = 0;
                if (df != 0.0f) {
                    const float r = nearbyintf(orc_bf16_to_f32(A[(size_t)i * lda + k]) / df);
                    v = r < -127.0f ? -127 : (r > 127.0f ? 127 : (int)r);
                }
                p[(size_t)i * K + k] = (int8_t)v;
            }
        }
}

/* p [M,K], d [M,K/64], q [K,N], s [K/64,N]  ->  acc fp32 [M,N] and its bf16 rounding c [M,N] */
void orc_qgemm_w4a8(const int8_t *p, const float *d, const int8_t *q, const uint16_t *s, int M, int N,
                    int K, float *acc_out, uint16_t *c)
{
    const int nb = K / 64;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int n = 0; n < N; ++n) {
            float acc = 0.0f;
            for (int b = 0; b < nb; ++b) {
                int32_t P = 0;
                for (int k = 64 * b; k < 64 * b + 64; ++k)
                    P += (int32_t)p[(size_t)i * K + k] * (int32_t)q[(size_t)k * N + n];
                const float scale = d[(size_t)i * nb + b] * orc_bf16_to_f32(s[(size_t)b * N + n]);
                acc = fmaf(scale, (float)P, acc);
            }
            acc_out[(size_t)i * N + n] = acc;
            c[(size_t)i * N + n] = orc_bf16_rne(acc);
        }
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
