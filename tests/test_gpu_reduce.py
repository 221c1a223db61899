"""RMSNorm, softmax statistics, argmax and the elementwise steps: the GPU must match the CPU
oracle's emulation of the canonical fp32 order bit for bit."""
import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, down_bf16, step, up, up_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def d():
    import paper_2602_00182_amd as d
    return d


@pytest.mark.parametrize("M,H", [(1, 4096), (16, 4096), (64, 4096), (7, 2048), (3, 8), (5, 264), (2, 16384), (130, 5632)])
def test_rmsnorm_bit_exact(d, orc, M, H):
    x = ds.normal_bf16(ds.tensor_seed(3, 0) + H, (M, H))
    w = ds.normal_bf16(ds.tensor_seed(3, 1) + H, (H,), 0.1, 1.0)
    step(f"rmsnorm M={M} H={H}")
    y = torch.empty((M, H), dtype=torch.bfloat16, device=DEV)
    d.det_rmsnorm(up_bf16(x), up_bf16(w), y, 1e-5)
    torch.cuda.synchronize()
    got = down_bf16(y)
    assert np.array_equal(got, orc.rmsnorm(x, w, 1e-5))
    # batch invariance: row 0 alone
    y1 = torch.empty((1, H), dtype=torch.bfloat16, device=DEV)
    d.det_rmsnorm(up_bf16(x[:1]), up_bf16(w), y1, 1e-5)
    torch.cuda.synchronize()
    assert np.array_equal(down_bf16(y1)[0], got[0])


def test_rmsnorm_order_sensitive_rows(d, orc):
    """Rows built so that a different lane mapping or tree shape changes the sum of squares by one
    fp32 ulp or more (big element next to small ones), at scales where that moves the output."""
    H = 4096
    rng = np.random.default_rng(17)
    x = ds.normal_bf16(400, (32, H))
    xf = ds.bf16_bits_to_f32(x)
    for r in range(32):
        j = rng.integers(0, H, 8)
        xf[r, j] *= np.float32(2.0 ** rng.integers(3, 9))
    x = ds.f32_to_bf16_bits(xf)
    w = ds.normal_bf16(401, (H,), 0.1, 1.0)
    y = torch.empty((32, H), dtype=torch.bfloat16, device=DEV)
    step("rmsnorm order-sensitive rows")
    d.det_rmsnorm(up_bf16(x), up_bf16(w), y, 1e-5)
    torch.cuda.synchronize()
    assert np.array_equal(down_bf16(y), orc.rmsnorm(x, w, 1e-5))


def test_softmax_bit_exact(d, orc):
    lens = np.array([1, 255, 256, 257, 511, 512, 513, 0, 4096, 5000, 32768, 30001], dtype=np.int32)
    Lmax = 32768
    R = len(lens)
    s = (ds.bf16_bits_to_f32(ds.normal_bf16(410, (R, Lmax))) * np.float32(3.0)).astype(np.float32)
    s += np.float32(1e-3) * np.arange(Lmax, dtype=np.float32)[None, :] / Lmax   # not just bf16 values
    s[5, 300] = 95.0          # a dominant score: everything else underflows to exactly 0
    s[9, :256] -= 120.0       # a whole chunk whose weight det_expf(m_c - m) is 0
    p0, m0, l0 = orc.softmax_f32(s, lens)
    sd = up(s)
    p = torch.zeros((R, Lmax), dtype=torch.float32, device=DEV)
    m = torch.empty(R, dtype=torch.float32, device=DEV)
    l = torch.empty(R, dtype=torch.float32, device=DEV)
    step("softmax_f32 hook")
    d.det_softmax_f32(sd, up(lens), p, m, l)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m0.view(np.uint32))
    assert np.array_equal(l.cpu().numpy().view(np.uint32), l0.view(np.uint32))
    assert np.array_equal(p.cpu().numpy().view(np.uint32), p0.view(np.uint32))


def test_expf_bit_exact_through_softmax(d, orc):
    """det_expf on a dense grid: a 2-token row (0, x) has e = (1, det_expf(x)) for x <= 0, so
    l - 1 = det_expf(x) exactly when det_expf(x) is a multiple of ulp(1)... instead compare p of the
    pair against the oracle's softmax, which exercises det_expf over the whole negative range."""
    n = 1 << 16
    x = -np.linspace(0.0, 90.0, n).astype(np.float32)
    s = np.zeros((n, 2), dtype=np.float32)
    s[:, 1] = x
    lens = np.full(n, 2, dtype=np.int32)
    p0, m0, l0 = orc.softmax_f32(s, lens)
    p = torch.zeros((n, 2), dtype=torch.float32, device=DEV)
    m = torch.empty(n, dtype=torch.float32, device=DEV)
    l = torch.empty(n, dtype=torch.float32, device=DEV)
    step("det_expf grid through softmax hook")
    d.det_softmax_f32(up(s), up(lens), p, m, l)
    torch.cuda.synchronize()
    assert np.array_equal(l.cpu().numpy().view(np.uint32), l0.view(np.uint32))
    assert np.array_equal(p.cpu().numpy().view(np.uint32), p0.view(np.uint32))


def test_argmax_bit_exact(d, orc):
    V = 32000
    x = ds.bf16_bits_to_f32(ds.normal_bf16(420, (64, V))).copy()
    x[1, :] = 2.5                       # all equal -> 0
    x[2, [100, 20000]] = 50.0           # tie -> lowest
    x[3, V - 1] = 60.0                  # last element
    x[4, :] = np.nan                    # all NaN -> 0
    x[5, :] = -5.0; x[5, 77] = np.nan; x[5, 31000] = -4.0
    x[6, :] = -1.0; x[6, 400] = -0.0; x[6, 900] = 0.0
    x[7, :] = -np.inf
    want = orc.argmax_f32(x)
    idx = torch.empty(64, dtype=torch.int32, device=DEV)
    step("argmax fp32")
    d.det_argmax(up(x), idx)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), want)
    assert want[:8].tolist()[1:] == [0, 100, V - 1, 0, 31000, 400, 0]
    xb = ds.normal_bf16(421, (16, V))   # bf16 logits tie often: lowest index must win
    step("argmax bf16")
    idx = torch.empty(16, dtype=torch.int32, device=DEV)
    d.det_argmax(up_bf16(xb), idx)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), orc.argmax_bf16(xb))
    for Vs in [1, 7, 255, 256, 257, 1000]:
        xs = ds.bf16_bits_to_f32(ds.normal_bf16(422 + Vs, (3, Vs))).copy()
        idx = torch.empty(3, dtype=torch.int32, device=DEV)
        d.det_argmax(up(xs), idx)
        torch.cuda.synchronize()
        assert np.array_equal(idx.cpu().numpy(), orc.argmax_f32(xs))


def test_rope_swiglu_residual_bit_exact(d, orc):
    D, Lmax = 128, 4096
    cos_t, sin_t = ds.rope_tables(Lmax, D)
    x = ds.normal_bf16(430, (33, 40, D))
    pos = ds.uniform_int(431, (33,), 0, Lmax - 1)
    y = torch.empty((33, 40, D), dtype=torch.bfloat16, device=DEV)
    step("rope")
    d.det_rope(up_bf16(x), y, up(pos), up(cos_t), up(sin_t))
    torch.cuda.synchronize()
    assert np.array_equal(down_bf16(y), orc.rope(x, pos, cos_t, sin_t))

    F = 14336
    gu = ds.normal_bf16(432, (9, 2 * F), 2.0)
    gu[0, :8] = ds.f32_to_bf16_bits(np.array([0, -0.0, 100, -100, 88, -88, 30, -30], dtype=np.float32))
    gud = up_bf16(gu)
    m = torch.empty((9, F), dtype=torch.bfloat16, device=DEV)
    step("swiglu")
    d.det_swiglu(gud[:, :F], gud[:, F:], m)
    torch.cuda.synchronize()
    assert np.array_equal(down_bf16(m), orc.swiglu(np.ascontiguousarray(gu[:, :F]), np.ascontiguousarray(gu[:, F:])))

    a = ds.normal_bf16(433, (50, 4096))
    b = ds.normal_bf16(434, (50, 4096), 0.01)
    z = torch.empty((50, 4096), dtype=torch.bfloat16, device=DEV)
    step("residual")
    d.det_residual_add(up_bf16(a), up_bf16(b), z)
    torch.cuda.synchronize()
    assert np.array_equal(down_bf16(z), orc.residual(a, b))
    za = up_bf16(a)
    d.det_residual_add(za, up_bf16(b), za)   # in place
    torch.cuda.synchronize()
    assert np.array_equal(down_bf16(za), orc.residual(a, b))


def test_embed_gather_and_next_token(d):
    V, H, B = 1000, 2048, 5
    table = ds.normal_bf16(440, (V, H))
    toks = np.array([0, 999, 5, 5, 123], dtype=np.int32)
    out = torch.empty((B, H), dtype=torch.bfloat16, device=DEV)
    step("embed gather")
    d.det_embed_gather(up_bf16(table), up(toks), out)
    torch.cuda.synchronize()
    assert np.array_equal(down_bf16(out), table[toks])
    prompts = np.arange(B * 6, dtype=np.int32).reshape(B, 6)
    plens = np.array([6, 1, 3, 2, 4], dtype=np.int32)
    last = np.array([900, 901, 902, 903, 904], dtype=np.int32)
    hist = torch.full((B, 10), -1, dtype=torch.int32, device=DEV)
    tok = torch.empty(B, dtype=torch.int32, device=DEV)
    pos = torch.empty(B, dtype=torch.int32, device=DEV)
    step("next token")
    d.det_next_token(up(prompts), up(plens), up(last), tok, pos, hist, 2)
    torch.cuda.synchronize()
    assert tok.cpu().tolist() == [2, 901, 14, 903, 26]
    assert pos.cpu().tolist() == [2] * B
    assert hist.cpu().numpy()[:, 2].tolist() == [2, 901, 14, 903, 26]
    assert (hist.cpu().numpy()[:, [0, 1, 3]] == -1).all()
