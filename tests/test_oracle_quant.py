"""Pins of the quantized-GEMM oracle (CPU only): exact cases, symmetries and scale equivariance of
the two quantizers, reconstruction bounds, and the quantized contraction against exact integer /
fp64 arithmetic done independently in numpy."""
import numpy as np
import pytest

import detsynth as ds


def bf16(x):
    return ds.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def f32(bits):
    return ds.bf16_bits_to_f32(bits)


def test_weight_quantizer_exact_cases(orc):
    rng = np.random.default_rng(1)
    K, N = 192, 24
    w = rng.integers(-7, 8, (K, N)).astype(np.float32)
    w[0::64, :] = 7.0                      # every block's largest magnitude is 7: scale exactly 1
    w[5::64, ::2] = -7.0
    q, s = orc.quant_w4(bf16(w))
    assert np.array_equal(f32(s), np.ones((K // 64, N), np.float32))
    assert np.array_equal(q.astype(np.float32), w)
    for e in (-9, 3):                      # a power-of-two factor moves into the scale only
        q2, s2 = orc.quant_w4(bf16(w * 2.0 ** e))
        assert np.array_equal(q2, q) and np.array_equal(f32(s2), np.full_like(f32(s), 2.0 ** e))
    zq, zs = orc.quant_w4(bf16(np.zeros((64, 3))))
    assert not zq.any() and not f32(zs).any()


def test_weight_quantizer_properties(orc):
    w = ds.normal_bf16(ds.tensor_seed(6, 1), (512, 96), 0.02, 0.0)
    q, s = orc.quant_w4(w)
    wf, sf = f32(w).astype(np.float64), np.repeat(f32(s).astype(np.float64), 64, axis=0)
    amax = np.abs(wf).reshape(8, 64, 96).max(axis=1)
    assert q.min() >= -7 and q.max() <= 7 and (np.abs(q).reshape(8, 64, 96).max(axis=1) == 7).all()
    assert (np.abs(f32(s) * 7.0 - amax) <= amax * 2.0 ** -8).all()          # the scale is bf16(amax/7)
    assert (np.abs(wf - sf * q) <= sf * 0.5 * (1 + 2.0 ** -20)).all()       # nearest code
    qn, sn = orc.quant_w4(w ^ 0x8000)                                       # sign symmetry
    assert np.array_equal(qn, -q) and np.array_equal(sn, s)
    perm = np.random.default_rng(2).permutation(96)                         # columns are independent
    qp, sp = orc.quant_w4(np.ascontiguousarray(w[:, perm]))
    assert np.array_equal(qp, q[:, perm]) and np.array_equal(sp, s[:, perm])


def test_activation_quantizer(orc):
    rng = np.random.default_rng(3)
    a = rng.integers(-127, 128, (5, 128)).astype(np.float32)
    a[:, 0] = 127.0
    a[:, 64] = -127.0
    p, d = orc.quant_a8(bf16(a))
    assert np.array_equal(d, np.ones((5, 2), np.float32)) and np.array_equal(p.astype(np.float32), a)
    p2, d2 = orc.quant_a8(bf16(a * 0.25))
    assert np.array_equal(p2, p) and np.array_equal(d2, np.full((5, 2), 0.25, np.float32))
    x = ds.normal_bf16(ds.tensor_seed(6, 2), (7, 256), 1.0, 0.0)
    p, d = orc.quant_a8(x)
    xf, df = f32(x).astype(np.float64), np.repeat(d.astype(np.float64), 64, axis=1)
    amax = np.abs(xf).reshape(7, 4, 64).max(axis=2)
    assert np.abs(p).max() <= 127 and (np.abs(p).reshape(7, 4, 64).max(axis=2) == 127).all()
    assert (np.abs(d.astype(np.float64) * 127.0 - amax) <= amax * 2.0 ** -23).all()
    assert (np.abs(xf - df * p) <= df * 0.5 * (1 + 2.0 ** -20)).all()
    pn, dn = orc.quant_a8(x ^ 0x8000)
    assert np.array_equal(pn, -p) and np.array_equal(dn, d)
    rows = [3, 0, 6]                                                        # rows are independent
    pr, dr = orc.quant_a8(np.ascontiguousarray(x[rows]))
    assert np.array_equal(pr, p[rows]) and np.array_equal(dr, d[rows])


def test_qgemm_exact_integer_case(orc):
    """Power-of-two scales and small integers: every product and partial sum is exact in fp32, so the
    result must equal the integer arithmetic done in numpy int64."""
    rng = np.random.default_rng(4)
    M, K, N = 5, 192, 7
    p = rng.integers(-127, 128, (M, K)).astype(np.int8)
    q = rng.integers(-8, 8, (K, N)).astype(np.int8)
    ed = rng.integers(-3, 2, (M, K // 64))
    es = rng.integers(-4, 1, (K // 64, N))
    d = (2.0 ** ed).astype(np.float32)
    s = bf16(2.0 ** es)
    acc, c = orc.qgemm_w4a8(p, d, q, s)
    P = np.einsum("ibk,bkn->ibn", p.astype(np.int64).reshape(M, K // 64, 64), q.astype(np.int64).reshape(K // 64, 64, N))
    want = (P * 2.0 ** (ed[:, :, None] + es[None, :, :])).sum(axis=1)       # exact in float64
    assert np.array_equal(acc.astype(np.float64), want)
    assert np.array_equal(c, orc.bf16_rne(want.astype(np.float32)))
    # transposed or mismatched operands would not survive this: one-hot rows pick single weights
    p1 = np.zeros((3, K), np.int8)
    p1[0, 5], p1[1, 70], p1[2, 191] = 1, -2, 3
    acc1, _ = orc.qgemm_w4a8(p1, np.ones((3, K // 64), np.float32), q, bf16(np.ones((K // 64, N))))
    assert np.array_equal(acc1, np.stack([q[5], -2 * q[70], 3 * q[191]]).astype(np.float32))


def test_qgemm_against_fp64_and_against_the_unquantized_product(orc):
    M, K, N = 9, 1024, 40
    x = ds.normal_bf16(ds.tensor_seed(6, 3), (M, K), 1.0, 0.0)
    w = ds.normal_bf16(ds.tensor_seed(6, 4), (K, N), 0.02, 0.0)
    p, d = orc.quant_a8(x)
    q, s = orc.quant_w4(w)
    acc, c = orc.qgemm_w4a8(p, d, q, s)
    nb = K // 64
    P = np.einsum("ibk,bkn->ibn", p.astype(np.int64).reshape(M, nb, 64), q.astype(np.int64).reshape(nb, 64, N))
    terms = d.astype(np.float64)[:, :, None] * f32(s).astype(np.float64)[None, :, :] * P
    ref = terms.sum(axis=1)
    # one rounded multiply and one fma per block: error <= (nb + 1) * 2^-24 * sum |terms|
    assert (np.abs(acc - ref) <= (nb + 1) * 2.0 ** -24 * np.abs(terms).sum(axis=1)).all()
    assert np.array_equal(c, orc.bf16_rne(acc))
    exact = f32(x).astype(np.float64) @ f32(w).astype(np.float64)           # what is being approximated
    rel = np.linalg.norm(ref - exact) / np.linalg.norm(exact)
    assert 0.01 < rel < 0.15, rel                                           # 4-bit weights: a few per cent


def test_quantized_layer_tracks_the_bf16_layer(orc):
    """qdecoder_layer is decoder_layer with quantized projections: on a small layer its branch update
    x' - x and its new cache rows stay within the quantization noise of the fp64-reference layer
    (4-bit weights: about 12 % of a projection's output), and far from it when a step is wrong (the
    same check fails with gate and up swapped or the rotation skipped, see the planted cases)."""
    cfg = dict(H=256, Hq=2, Hkv=1, D=128, F=192, Lmax=16, eps=1e-5, scale=float(np.float32(128.0 ** -0.5)))
    H, Hq, Hkv, D, F, Lmax = (cfg[k] for k in ("H", "Hq", "Hkv", "D", "F", "Lmax"))
    s0 = ds.tensor_seed(6, 40)
    w = dict(norm1=ds.normal_bf16(s0, (H,), 0.1, 1.0), norm2=ds.normal_bf16(s0 + 1, (H,), 0.1, 1.0),
             wqkv=ds.normal_bf16(s0 + 2, (H, (Hq + 2 * Hkv) * D), 0.06, 0.0),
             wo=ds.normal_bf16(s0 + 3, (Hq * D, H), 0.06, 0.0),
             wgu=ds.normal_bf16(s0 + 4, (H, 2 * F), 0.06, 0.0),
             wdown=ds.normal_bf16(s0 + 5, (F, H), 0.06, 0.0))
    B = 3
    x = ds.normal_bf16(s0 + 6, (B, H), 1.0, 0.0)
    kc = ds.normal_bf16(s0 + 7, (B, Hkv, Lmax, D), 1.0, 0.0)
    vc = ds.normal_bf16(s0 + 8, (B, Hkv, Lmax, D), 1.0, 0.0)
    pos = np.asarray([15, 4, 0], dtype=np.int32)
    cos_t, sin_t = ds.rope_tables(Lmax, D, 5.0e5)
    kr, vr = kc.copy(), vc.copy()
    ref = orc.decoder_layer(x, w, kr, vr, pos, cos_t, sin_t, cfg)

    def run(wq, cos=cos_t, sin=sin_t):
        kq, vq = kc.copy(), vc.copy()
        return orc.qdecoder_layer(x, wq, kq, vq, pos, cos, sin, cfg), kq, vq

    wq = {k: (v if v.ndim == 1 else orc.quant_w4(v)) for k, v in w.items()}
    got, kq, vq = run(wq)

    def rel(a, b):
        a, b = f32(a).astype(np.float64), f32(b).astype(np.float64)
        return np.sqrt(((a - b) ** 2).mean() / (b ** 2).mean())

    upd_ref = f32(ref).astype(np.float64) - f32(x)
    upd_got = f32(got).astype(np.float64) - f32(x)
    err = np.sqrt(((upd_got - upd_ref) ** 2).mean() / (upd_ref ** 2).mean())
    assert err < 0.3, err
    for b, p in enumerate(pos):
        assert rel(kq[b, :, p], kr[b, :, p]) < 0.25 and rel(vq[b, :, p], vr[b, :, p]) < 0.25
        mask = np.ones(Lmax, dtype=bool)
        mask[p] = False
        assert np.array_equal(kq[b][:, mask], kc[b][:, mask]) and np.array_equal(vq[b][:, mask], vc[b][:, mask])
    # planted mistakes in the inputs move the result far outside that bound
    swapped = dict(wq)
    gu = w["wgu"]
    swapped["wgu"] = orc.quant_w4(np.ascontiguousarray(np.concatenate([gu[:, F:], gu[:, :F]], axis=1)))
    bad, _, _ = run(swapped)
    assert np.sqrt((((f32(bad).astype(np.float64) - f32(x)) - upd_ref) ** 2).mean() / (upd_ref ** 2).mean()) > 0.5
    _, k_norot, _ = run(wq, np.ones_like(cos_t), np.zeros_like(sin_t))
    assert rel(k_norot[0, :, 15], kr[0, :, 15]) > 0.5
    # a layer whose output projections are zero leaves x unchanged and still appends the cache rows
    zeroed = dict(wq)
    zeroed["wo"] = orc.quant_w4(np.zeros_like(w["wo"]))
    zeroed["wdown"] = orc.quant_w4(np.zeros_like(w["wdown"]))
    same, kz, _ = run(zeroed)
    assert np.array_equal(same, x) and np.array_equal(kz, kq)
