// One decoder layer as a fixed sequence of the library's own operations on the caller's stream.
// Nothing here computes: the layer inherits determinism and batch invariance from its steps.
#include "internal.h"

namespace det {

static size_t up256(size_t n) { return (n + 255) & ~(size_t)255; }

struct LayerWs {
    size_t h, qbuf, att, mm, attn, attn_bytes, total;
};

static LayerWs layer_ws(const det_layer_cfg& c, int B)
{
    LayerWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += up256(bytes);
        return o;
    };
    w.h = take(2 * (size_t)B * c.H);
    w.qbuf = take(2 * (size_t)B * c.Hq * c.D);
    w.att = take(2 * (size_t)B * c.Hq * c.D);
    w.mm = take(2 * (size_t)B * c.F);
    w.attn_bytes = det_attn_decode_workspace_bytes(B, c.Hq, c.D, c.Lmax);
    w.attn = take(w.attn_bytes);
    w.total = off;
    return w;
}

// Workspace of the quantized layer: the bf16 buffers of the plain one that are still needed, plus one
// set of activation codes and scales (the widest projection input), reused by the four projections.
struct QLayerWs {
    size_t qbuf, mm, codes, scales, codes2, scales2, attn, attn_bytes, total;
};

static QLayerWs qlayer_ws(const det_layer_cfg& c, int R)
{
    QLayerWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += up256(bytes);
        return o;
    };
    const int nq = c.Hq * c.D;
    const int kmax = c.H > nq ? (c.H > c.F ? c.H : c.F) : (nq > c.F ? nq : c.F);
    w.qbuf = take(2 * (size_t)R * nq);
    w.mm = take(2 * (size_t)R * c.F);
    w.codes = take(det_quant_act_codes_bytes(R, kmax));
    w.scales = take(det_quant_act_scales_bytes(R, kmax));
    // the SwiGLU output's codes, written by the gate/up projection while it still reads the first set
    w.codes2 = take(det_quant_act_codes_bytes(R, c.F));
    w.scales2 = take(det_quant_act_scales_bytes(R, c.F));
    w.attn_bytes = det_attn_decode_workspace_bytes(R, c.Hq, c.D, c.Lmax);
    w.attn = take(w.attn_bytes);
    w.total = off;
    return w;
}

static bool layer_cfg_ok(const det_layer_cfg* c)
{
    return c && c->H > 0 && c->Hq > 0 && c->Hkv > 0 && c->D == 128 && c->F > 0 && c->Lmax > 0 &&
           c->Hq % c->Hkv == 0 && c->H % 64 == 0 && c->F % 64 == 0;  // F % 64: K of the down projection
}

}  // namespace det

using namespace det;

extern "C" size_t det_decoder_layer_workspace_bytes(const det_layer_cfg* cfg, int B)
{
    if (!layer_cfg_ok(cfg) || B < 1) return 0;
    return layer_ws(*cfg, B).total;
}

static int decoder_layer_impl(const det_layer_weights* w, const det_layer_cfg* cfg, void* x_inout, void* kcache,
                              void* vcache, const int32_t* positions, const int32_t* slots, const float* rope_cos,
                              const float* rope_sin, void* ws, size_t ws_bytes, int B, void* stream)
{
    if (!w || !cfg || !x_inout || !kcache || !vcache || !positions || !rope_cos || !rope_sin || !ws || B < 1)
        return DET_EINVAL;
    if (!w->w_norm1 || !w->wqkv || !w->wo || !w->w_norm2 || !w->wgu || !w->wdown) return DET_EINVAL;
    if (!layer_cfg_ok(cfg)) return DET_ESHAPE;
    if (!aligned16(ws) || !aligned16(x_inout)) return DET_EALIGN;
    const det_layer_cfg c = *cfg;
    const LayerWs l = layer_ws(c, B);
    if (ws_bytes < l.total) return DET_EWORKSPACE;
    char* base = static_cast<char*>(ws);
    void* h = base + l.h;
    void* qbuf = base + l.qbuf;
    void* att = base + l.att;
    void* mm = base + l.mm;
    void* aws = base + l.attn;
    const int nq = c.Hq * c.D;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc;
#define DET_TRY(call)                \
    do {                             \
        rc = (call);                 \
        if (rc != DET_OK) return rc; \
    } while (0)
    DET_TRY(det_rmsnorm_gemm_qkv_rope_append(x_inout, c.H, w->w_norm1, c.eps, w->wqkv, h, qbuf, kcache, vcache,
                                             positions, slots, rope_cos, rope_sin, B, c.Hq, c.Hkv, c.D, c.Lmax, c.H,
                                             stream));
    DET_TRY(attn_decode_impl(qbuf, kcache, vcache, positions, slots, 1, att, aws, l.attn_bytes, B, c.Hq, c.Hkv, c.D,
                             c.Lmax, c.scale, s));
    DET_TRY(det_gemm_bf16_residual(att, nq, w->wo, x_inout, c.H, x_inout, c.H, B, c.H, nq, stream));
    DET_TRY(det_rmsnorm_gemm_swiglu_bf16(x_inout, c.H, w->w_norm2, c.eps, w->wgu, h, mm, c.F, B, c.F, c.H, stream));
    DET_TRY(det_gemm_bf16_residual(mm, c.F, w->wdown, x_inout, c.H, x_inout, c.H, B, c.H, c.F, stream));
#undef DET_TRY
    return DET_OK;
}

extern "C" int det_decoder_layer(const det_layer_weights* w, const det_layer_cfg* cfg, void* x_inout,
                                 void* kcache, void* vcache, const int32_t* positions, const float* rope_cos,
                                 const float* rope_sin, void* ws, size_t ws_bytes, int B, void* stream)
{
    return decoder_layer_impl(w, cfg, x_inout, kcache, vcache, positions, nullptr, rope_cos, rope_sin, ws, ws_bytes, B,
                              stream);
}

extern "C" int det_decoder_layer_rows(const det_layer_weights* w, const det_layer_cfg* cfg, void* x_inout,
                                      void* kcache, void* vcache, const int32_t* positions, const int32_t* slots,
                                      const float* rope_cos, const float* rope_sin, void* ws, size_t ws_bytes,
                                      int R, void* stream)
{
    if (!slots) return DET_EINVAL;
    return decoder_layer_impl(w, cfg, x_inout, kcache, vcache, positions, slots, rope_cos, rope_sin, ws, ws_bytes, R,
                              stream);
}

extern "C" size_t det_qdecoder_layer_workspace_bytes(const det_layer_cfg* cfg, int R)
{
    if (!layer_cfg_ok(cfg) || R < 1) return 0;
    return qlayer_ws(*cfg, R).total;
}

extern "C" int det_qdecoder_layer(const det_layer_weights* w, const det_layer_cfg* cfg, void* x_inout, void* kcache,
                                  void* vcache, const int32_t* positions, const int32_t* slots, const float* rope_cos,
                                  const float* rope_sin, void* ws, size_t ws_bytes, int R, void* stream)
{
    if (!w || !cfg || !x_inout || !kcache || !vcache || !positions || !rope_cos || !rope_sin || !ws || R < 1)
        return DET_EINVAL;
    if (!w->w_norm1 || !w->wqkv || !w->wo || !w->w_norm2 || !w->wgu || !w->wdown) return DET_EINVAL;
    if (!layer_cfg_ok(cfg)) return DET_ESHAPE;
    if (!aligned16(ws) || !aligned16(x_inout)) return DET_EALIGN;
    const det_layer_cfg c = *cfg;
    const QLayerWs l = qlayer_ws(c, R);
    if (ws_bytes < l.total) return DET_EWORKSPACE;
    char* base = static_cast<char*>(ws);
    void* qbuf = base + l.qbuf;
    void* mm = base + l.mm;
    void* codes = base + l.codes;
    void* scales = base + l.scales;
    void* codes2 = base + l.codes2;
    void* scales2 = base + l.scales2;
    void* aws = base + l.attn;
    const int nq = c.Hq * c.D;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc;
#define DET_TRY(call)                \
    do {                             \
        rc = (call);                 \
        if (rc != DET_OK) return rc; \
    } while (0)
    DET_TRY(det_rmsnorm_quant_q8(x_inout, w->w_norm1, codes, scales, R, c.H, c.eps, stream));
    DET_TRY(det_qgemm_w4a8_qkv_rope_append(codes, scales, w->wqkv, qbuf, kcache, vcache, positions, slots, rope_cos,
                                           rope_sin, R, c.Hq, c.Hkv, c.D, c.Lmax, c.H, stream));
    DET_TRY(attn_decode_impl(qbuf, kcache, vcache, positions, slots, 1, codes, aws, l.attn_bytes, R, c.Hq, c.Hkv, c.D,
                             c.Lmax, c.scale, s, scales));
    DET_TRY(det_qgemm_w4a8_residual(codes, scales, w->wo, x_inout, c.H, x_inout, c.H, R, c.H, nq, stream));
    DET_TRY(det_rmsnorm_quant_q8(x_inout, w->w_norm2, codes, scales, R, c.H, c.eps, stream));
    if (det_qgemm_w4a8_swiglu_quant_supported(c.F, c.H)) {
        DET_TRY(det_qgemm_w4a8_swiglu_quant(codes, scales, w->wgu, codes2, scales2, R, c.F, c.H, stream));
    } else {
        DET_TRY(det_qgemm_w4a8_swiglu(codes, scales, w->wgu, mm, c.F, R, c.F, c.H, stream));
        DET_TRY(det_quant_act_q8(mm, c.F, codes2, scales2, R, c.F, stream));
    }
    DET_TRY(det_qgemm_w4a8_residual(codes2, scales2, w->wdown, x_inout, c.H, x_inout, c.H, R, c.H, c.F, stream));
#undef DET_TRY
    return DET_OK;
}
