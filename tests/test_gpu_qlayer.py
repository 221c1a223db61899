"""det_qdecoder_layer (the decoder layer on 4-bit weights and 8-bit activations) against the oracle's
quantized layer: everything up to attention is bit-exact (new cache rows), the output within the
layer bound; byte equality against the unfused sequence of individually pinned calls, across batch
compositions, and between one call on T rows of a slot and T single-token calls."""
import math

import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, bits_to_f64, down_bf16, step, up

pytestmark = pytest.mark.gpu

CFG = dict(H=4096, Hq=32, Hkv=8, D=128, F=14336, Lmax=2048, eps=1e-5,
           scale=float(np.float32(1.0 / math.sqrt(128.0))))


@pytest.fixture(scope="module")
def d():
    import paper_2602_00182_amd as d
    return d


@pytest.fixture(scope="module")
def layer(d):
    H, Hq, Hkv, D, F = (CFG[k] for k in ("H", "Hq", "Hkv", "D", "F"))
    s = ds.tensor_seed(7, 0)
    logical = dict(
        norm1=ds.normal_bf16_torch(s, (H,), 0.1, 1.0, DEV),
        wqkv=ds.normal_bf16_torch(s + 1, (H, (Hq + 2 * Hkv) * D), 0.02, 0.0, DEV),
        wo=ds.normal_bf16_torch(s + 2, (Hq * D, H), 0.02, 0.0, DEV),
        norm2=ds.normal_bf16_torch(s + 3, (H,), 0.1, 1.0, DEV),
        wgu=ds.normal_bf16_torch(s + 4, (H, 2 * F), 0.02, 0.0, DEV),
        wdown=ds.normal_bf16_torch(s + 5, (F, H), 0.02, 0.0, DEV),
    )
    packed = dict(norm1=logical["norm1"], norm2=logical["norm2"], wqkv=d.quant_pack_qkv(logical["wqkv"], Hq, Hkv, D),
                  wqkv_plain=d.quant_pack_weight(logical["wqkv"]),
                  wo=d.quant_pack_weight(logical["wo"]), wgu=d.quant_pack_gate_up(logical["wgu"]),
                  wgu_plain=d.quant_pack_weight(logical["wgu"]), wdown=d.quant_pack_weight(logical["wdown"]))
    struct = d.layer_weights(packed["norm1"], packed["wqkv"], packed["wo"], packed["norm2"], packed["wgu"],
                             packed["wdown"])
    cos_t, sin_t = ds.rope_tables(CFG["Lmax"], CFG["D"], 5.0e5)
    cfg = d.layer_cfg(CFG["H"], CFG["Hq"], CFG["Hkv"], CFG["D"], CFG["F"], CFG["Lmax"], CFG["eps"], CFG["scale"])
    return dict(logical=logical, packed=packed, struct=struct, cfg=cfg, cos=up(cos_t), sin=up(sin_t),
                cos_h=cos_t, sin_h=sin_t)


def seq_inputs(b):
    s = ds.tensor_seed(7, 100) + 10 * b
    x = ds.normal_bf16_torch(s, (CFG["H"],), 1.0, 0.0, DEV)
    k = ds.normal_bf16_torch(s + 1, (CFG["Hkv"], CFG["Lmax"], CFG["D"]), 1.0, 0.0, DEV)
    v = ds.normal_bf16_torch(s + 2, (CFG["Hkv"], CFG["Lmax"], CFG["D"]), 1.0, 0.0, DEV)
    return x, k, v


def batch_inputs(seq_ids):
    xs, ks, vs = zip(*[seq_inputs(b) for b in seq_ids])
    return torch.stack(xs).contiguous(), torch.stack(ks).contiguous(), torch.stack(vs).contiguous()


def run_layer(d, layer, seq_ids, positions):
    B = len(seq_ids)
    x, kc, vc = batch_inputs(seq_ids)
    ws = torch.empty(d.det_qdecoder_layer_workspace_bytes(layer["cfg"], B), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    d.det_qdecoder_layer(layer["struct"], layer["cfg"], x, kc, vc, up(np.asarray(positions, dtype=np.int32)), None,
                         layer["cos"], layer["sin"], ws)
    torch.cuda.synchronize()
    return x, kc, vc


def test_qlayer_vs_oracle(d, orc, layer):
    """B = 3 at positions 2047, 1000, 0.  RMSNorm, both quantizers, the quantized projection and the
    rotation are bit-exact against the oracle, so the new K and V rows must match it byte for byte.
    After attention (fp32 on the GPU, fp64 rounded once in the oracle) the two sides may differ by
    one bf16 ulp in a few attention outputs, which moves the codes of those 64-element blocks; the
    output is held to the element-wise bound of the bf16 layer test (oracle.model.layer_bound)."""
    seq_ids, positions = [0, 1, 2], [2047, 1000, 0]
    step("quantized decoder layer B=3 vs oracle")
    x, kc, vc = run_layer(d, layer, seq_ids, positions)
    x0, kc0, vc0 = (down_bf16(t) for t in batch_inputs(seq_ids))
    w = {k: (down_bf16(v) if v.dim() == 1 else orc.quant_w4(down_bf16(v))) for k, v in layer["logical"].items()}
    from oracle import model as om

    inter = {}
    ref = orc.qdecoder_layer(x0, w, kc0, vc0, np.asarray(positions, dtype=np.int32), layer["cos_h"],
                             layer["sin_h"], CFG, intermediates=inter)
    assert np.array_equal(down_bf16(kc), kc0) and np.array_equal(down_bf16(vc), vc0)   # oracle updated its copies
    got, reff = bits_to_f64(down_bf16(x)), bits_to_f64(ref)
    err = np.abs(got - reff)
    # the four roundings on an output's path (o, x1, dn, x2) one ulp each; the carried term is twice the
    # bf16 layer's because a one-ulp flip of an activation also re-rounds the 8-bit codes of its 64-element
    # block (each code by at most one step d = amax/127)
    bound = om.layer_bound(ref, inter, carried_rel=2.0 ** -7)
    print(f"[measured] quantized decoder layer vs oracle: max err/bound = {(err / bound).max():.3f}, "
          f"outputs that differ: {(err > 0).mean():.5f}", flush=True)
    assert (err <= bound).all(), (err / bound).max()
    assert (down_bf16(x) == ref).mean() > 0.9


def test_qlayer_equals_unfused_calls(d, layer):
    """The layer's bytes are those of the library's own single operations called one after the other
    (each of which has its own oracle test): RMSNorm, activation quantizer, quantized GEMM, rotation,
    cache write, attention, residual add, SwiGLU."""
    B, positions = 5, [2047, 7, 300, 0, 1999]
    H, Hq, Hkv, D, F, Lmax = (CFG[k] for k in ("H", "Hq", "Hkv", "D", "F", "Lmax"))
    step("quantized decoder layer B=5, fused")
    xf, kf, vf = run_layer(d, layer, list(range(B)), positions)
    step("quantized decoder layer B=5, one operation at a time")
    x, kc, vc = batch_inputs(list(range(B)))
    pk = layer["packed"]
    pos = up(np.asarray(positions, dtype=np.int32))

    def qlinear(a, packed, N):
        codes, scales = d.quant_activations(a.contiguous())
        out = torch.empty((a.shape[0], N), dtype=torch.bfloat16, device=DEV)
        d.det_qgemm_w4a8(codes, scales, packed, out, N)
        return out

    h = torch.empty_like(x)
    d.det_rmsnorm(x, pk["norm1"], h, CFG["eps"])
    qkv = qlinear(h, pk["wqkv_plain"], (Hq + 2 * Hkv) * D)
    q = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=DEV)
    k = torch.empty((B, Hkv, D), dtype=torch.bfloat16, device=DEV)
    d.det_rope(qkv[:, :Hq * D].reshape(B, Hq, D).contiguous(), q, pos, layer["cos"], layer["sin"])
    d.det_rope(qkv[:, Hq * D:(Hq + Hkv) * D].reshape(B, Hkv, D).contiguous(), k, pos, layer["cos"], layer["sin"])
    for b, p in enumerate(positions):
        kc[b, :, p] = k[b]
        vc[b, :, p] = qkv[b, (Hq + Hkv) * D:].reshape(Hkv, D)
    att = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(d.det_attn_decode_workspace_bytes(B, Hq, D, Lmax), dtype=torch.uint8, device=DEV)
    d.det_attn_decode(q, kc, vc, pos + 1, att, ws, CFG["scale"])
    o = qlinear(att.reshape(B, Hq * D), pk["wo"], H)
    d.det_residual_add(x, o, x)
    d.det_rmsnorm(x, pk["norm2"], h, CFG["eps"])
    gu = qlinear(h, pk["wgu_plain"], 2 * F)
    mm = torch.empty((B, F), dtype=torch.bfloat16, device=DEV)
    d.det_swiglu(gu[:, :F], gu[:, F:], mm)
    dn = qlinear(mm, pk["wdown"], H)
    d.det_residual_add(x, dn, x)
    torch.cuda.synchronize()
    assert torch.equal(kf.view(torch.int16), kc.view(torch.int16)) and torch.equal(vf.view(torch.int16), vc.view(torch.int16))
    assert torch.equal(xf.view(torch.int16), x.view(torch.int16))


@pytest.mark.parametrize("B", [32, 128])
def test_qlayer_bytes_across_batch_compositions(d, layer, B):
    step("quantized decoder layer alone")
    x1, k1, v1 = run_layer(d, layer, [0], [2047])
    want = (x1[0].clone(), k1[0, :, 2047].clone(), v1[0, :, 2047].clone())

    def check(xb, kb, vb, slot):
        for got, w_ in zip((xb[slot], kb[slot, :, 2047], vb[slot, :, 2047]), want):
            assert torch.equal(got.view(torch.int16), w_.view(torch.int16))

    step(f"quantized decoder layer inside B={B}, slot 0")
    check(*run_layer(d, layer, list(range(B)), [2047] * B), 0)
    step(f"quantized decoder layer inside B={B}, slot {B - 3}, other rows re-seeded, ragged positions")
    ids = [1000 + i for i in range(B)]
    slot = B - 3
    ids[slot] = 0
    pos = ds.uniform_int(78 + B, (B,), 0, 2047).tolist()
    pos[slot] = 2047
    xb, kb, vb = run_layer(d, layer, ids, pos)
    check(xb, kb, vb, slot)
    step("quantized decoder layer repeat x3")
    for _ in range(3):
        xr, kr, _ = run_layer(d, layer, ids, pos)
        assert torch.equal(xr.view(torch.int16), xb.view(torch.int16)) and torch.equal(kr.view(torch.int16), kb.view(torch.int16))


def test_qlayer_rows_prefill_equals_steps(d, layer):
    """T rows on one cache slot at positions 0..T-1 in one call (with a second slot interleaved) leave
    the hidden rows and cache bytes of T single-token calls."""
    T = 24
    s = ds.tensor_seed(7, 900)
    xs = ds.normal_bf16_torch(s, (2, T, CFG["H"]), 1.0, 0.0, DEV)
    shape = (1, CFG["Hkv"], CFG["Lmax"], CFG["D"])
    step("quantized layer, token by token, sequence 0")
    kc = torch.zeros(shape, dtype=torch.bfloat16, device=DEV)
    vc = torch.zeros_like(kc)
    ws1 = torch.empty(d.det_qdecoder_layer_workspace_bytes(layer["cfg"], 1), dtype=torch.uint8, device=DEV)
    want = []
    for t in range(T):
        x = xs[0, t:t + 1].clone()
        d.det_qdecoder_layer(layer["struct"], layer["cfg"], x, kc, vc, up(np.asarray([t], dtype=np.int32)), None,
                             layer["cos"], layer["sin"], ws1)
        want.append(x)
    want = torch.cat(want)
    step("quantized layer rows, two slots interleaved")
    kc2 = torch.zeros((2,) + shape[1:], dtype=torch.bfloat16, device=DEV)
    vc2 = torch.zeros_like(kc2)
    order = np.random.default_rng(4).permutation(2 * T)
    slots = (order // T).astype(np.int32)
    pos = (order % T).astype(np.int32)
    x = xs.reshape(2 * T, -1)[torch.from_numpy(order).to(DEV)].contiguous()
    ws = torch.empty(d.det_qdecoder_layer_workspace_bytes(layer["cfg"], 2 * T), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    d.det_qdecoder_layer(layer["struct"], layer["cfg"], x, kc2, vc2, up(pos), up(slots), layer["cos"], layer["sin"], ws)
    torch.cuda.synchronize()
    rows0 = np.argsort(order)[:T]
    assert torch.equal(x[torch.from_numpy(rows0).to(DEV)], want)
    assert torch.equal(kc2[0], kc[0]) and torch.equal(vc2[0], vc[0])


def test_qlayer_argument_errors(d, layer):
    from paper_2602_00182_amd._lib import lib
    import ctypes as C
    L = lib()
    assert L.det_qdecoder_layer_workspace_bytes(C.byref(layer["cfg"]), 0) == 0
    x, kc, vc = batch_inputs([0])
    pos = up(np.asarray([5], dtype=np.int32))
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    rc = L.det_qdecoder_layer(C.byref(layer["struct"]), C.byref(layer["cfg"]), x.data_ptr(), kc.data_ptr(), vc.data_ptr(),
                              pos.data_ptr(), None, layer["cos"].data_ptr(), layer["sin"].data_ptr(), small.data_ptr(),
                              small.numel(), 1, None)
    assert rc == 4                                                             # DET_EWORKSPACE
    rc = L.det_qdecoder_layer(C.byref(layer["struct"]), C.byref(layer["cfg"]), None, kc.data_ptr(), vc.data_ptr(),
                              pos.data_ptr(), None, layer["cos"].data_ptr(), layer["sin"].data_ptr(), small.data_ptr(),
                              small.numel(), 1, None)
    assert rc == 1                                                             # DET_EINVAL
    torch.cuda.synchronize()
