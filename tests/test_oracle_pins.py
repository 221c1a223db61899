"""Pins for the CPU oracle: each oracle function is checked against something that is not itself --
hand-worked values, closed forms, exact-arithmetic cases, brute force on tiny inputs, or a library
routine on a special case.  The paper prints no numeric example (its kernel section gives three
invariants and a reduction-tree figure), so there are no paper-printed values to pin to; the tree
cases below are worked by hand from the stride-halving loop of section 6.5, paragraph 2.
"""
import math

import numpy as np
import pytest

import detsynth as ds


def f32(x):
    return np.float32(x)


def bits(b):
    return np.array(b, dtype=np.uint16)


# ------------------------------------------------------------------ bf16 rounding

def test_bf16_rne_hand_cases(orc):
    cases = [
        (257.0, 0x4380),                   # 257 is a tie between 256 and 258: even mantissa -> 256
        (259.0, 0x4382),                   # tie between 258 (odd) and 260 (even) -> 260
        (1.0 + 2.0 ** -8, 0x3F80),         # tie, even below
        (1.0 + 3 * 2.0 ** -8, 0x3F82),     # tie, even above
        (1.0 + 2.0 ** -8 + 2.0 ** -23, 0x3F81),  # just above the tie
        (0.0, 0x0000), (-0.0, 0x8000),
        (float("inf"), 0x7F80), (float("-inf"), 0xFF80),
        (3.4028234663852886e38, 0x7F80),   # max fp32 rounds up to inf
        (-1.5, 0xBFC0),
    ]
    x = np.array([c[0] for c in cases], dtype=np.float32)
    got = orc.bf16_rne(x)
    assert got.tolist() == [c[1] for c in cases]
    nan = np.array([0x7FC00001, 0xFFFFFFFF, 0x7F800001], dtype=np.uint32).view(np.float32)
    assert orc.bf16_rne(nan).tolist() == [0x7FC0] * 3


def _rne_by_neighbours(x):
    """Independent formulation: pick, in fp64, the nearer of the two bf16 neighbours; ties go to
    the one with an even mantissa."""
    u = x.view(np.uint32)
    lo = (u & np.uint32(0xFFFF0000))
    hi = lo + np.uint32(0x10000)                       # next bf16 away from zero (may be inf)
    xl = lo.view(np.float32).astype(np.float64)
    xh = hi.view(np.float32).astype(np.float64)
    xd = x.astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        # distance to inf is measured to the value inf would have as a finite bf16 (2^128)
        xh_f = np.where(np.isinf(xh), np.sign(xd) * 2.0 ** 128, xh)
        dl = np.abs(xd - xl)
        dh = np.abs(xh_f - xd)
    pick_hi = (dh < dl) | ((dh == dl) & (((lo >> np.uint32(16)) & np.uint32(1)) == 1))
    return np.where(pick_hi, hi >> np.uint32(16), lo >> np.uint32(16)).astype(np.uint16)


def test_bf16_rne_against_neighbour_rule_and_torch(orc):
    import torch

    rng = np.random.default_rng(1)
    u = rng.integers(0, 2 ** 32, size=1 << 22, dtype=np.uint64).astype(np.uint32)
    # add every pattern whose low half is an exact tie or next to one, for a spread of exponents
    ties = (np.arange(0, 1 << 16, dtype=np.uint32) << np.uint32(16))[::7]
    u = np.concatenate([u, ties | np.uint32(0x8000), ties | np.uint32(0x7FFF), ties | np.uint32(0x8001)])
    x = u.view(np.float32)
    finite = np.isfinite(x)
    x = x[finite]
    got = orc.bf16_rne(x)
    assert np.array_equal(got, _rne_by_neighbours(x))
    t = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, t)


def test_bf16_from_f64_single_rounding(orc):
    # agrees with the fp32 rule wherever the double is an fp32 value
    rng = np.random.default_rng(2)
    x = rng.standard_normal(4096).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 4096).astype(np.float32)
    assert np.array_equal(orc.bf16_from_f64(x.astype(np.float64)), orc.bf16_rne(x))
    # a value that rounding through fp32 first would get wrong: just above a tie by 2^-40
    d = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(d) == np.float32(1.0 + 2.0 ** -8)            # fp32 lands on the tie ...
    assert orc.bf16_rne(np.array([d], dtype=np.float32))[0] == 0x3F80   # ... and goes down
    assert orc.bf16_from_f64(np.array([d]))[0] == 0x3F81               # single rounding goes up
    assert orc.bf16_from_f64(np.array([-d]))[0] == 0xBF81
    assert orc.bf16_from_f64(np.array([0.0, -0.0, 1e39, -1e39, np.nan])).tolist() == [0, 0x8000, 0x7F80, 0xFF80, 0x7FC0]
    # subnormal bf16: 2^-133 is the smallest; 2^-134 is a tie with zero -> even -> 0
    assert orc.bf16_from_f64(np.array([2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -133])).tolist() == [1, 0, 2]


# ------------------------------------------------------------------ det_expf

def test_expf_special_values(orc):
    x = np.array([0.0, -0.0, 88.73, 100.0, -87.01, -1000.0, np.inf, -np.inf], dtype=np.float32)
    y = orc.expf(x)
    assert y[0] == 1.0 and y[1] == 1.0
    assert np.isposinf(y[2]) and np.isposinf(y[3]) and np.isposinf(y[6])
    assert y[4] == 0.0 and y[5] == 0.0 and y[7] == 0.0
    n = orc.expf(np.array([np.nan], dtype=np.float32))
    assert n.view(np.uint32)[0] == 0x7FC00000


def test_expf_accuracy_vs_fp64_exp(orc):
    x = np.linspace(-87.0, 88.72, 3_000_001).astype(np.float32)
    rng = np.random.default_rng(3)
    x = np.concatenate([x, (rng.standard_normal(1_000_000) * 5).astype(np.float32),
                        -np.abs(rng.standard_normal(1_000_000) * 0.01).astype(np.float32)])
    x = x[(x >= -87.0) & (x <= 88.72)]
    y = orc.expf(x).astype(np.float64)
    ref = np.exp(x.astype(np.float64))
    ulp = np.spacing(ref.astype(np.float32)).astype(np.float64)
    err = np.abs(y - ref) / ulp
    assert err.max() <= 2.0, err.max()
    assert np.all(np.isfinite(y)) and np.all(y >= 2.0 ** -126)   # never subnormal, never inf


def test_expf_powers_of_two_are_scaled_exactly(orc):
    # exp(x + k*ln2) is not exactly 2^k exp(x) in fp32, but the exponent insertion must be: for
    # arguments that reduce to the same (r) the results differ by an exact power of two.  r = 0:
    # x = n*ln2_hi + n*ln2_lo is not representable, so use the reduction-free case n = 0 ...
    small = np.array([0.25, -0.25, 0.3, -0.34], dtype=np.float32)   # |x| < ln2/2 -> n = 0
    y = orc.expf(small).astype(np.float64)
    ref = np.exp(small.astype(np.float64))
    assert np.all(np.abs(y - ref) <= 1.5 * np.spacing(ref.astype(np.float32)))
    # ... and monotonic behaviour across the n = 0 / n = 1 seam at ln2/2
    seam = np.float32(0.5 * math.log(2.0))
    xs = np.array([np.nextafter(seam, f32(0)), seam, np.nextafter(seam, f32(1))], dtype=np.float32)
    ys = orc.expf(xs)
    assert ys[0] <= ys[1] <= ys[2]


# ------------------------------------------------------------------ canonical tree

def test_tree256_exact_integer_sums(orc):
    rng = np.random.default_rng(4)
    t = rng.integers(-1000, 1000, 256).astype(np.float32)
    assert orc.tree256(t) == np.float32(t.astype(np.int64).sum())
    t = np.zeros(256, dtype=np.float32)
    for i in range(256):
        t[:] = 0
        t[i] = 3.0
        assert orc.tree256(t) == 3.0    # every leaf is reached exactly once


def test_tree256_order_hand_worked(orc):
    """Cases where the stride-halving tree gives a different fp32 result from a left-to-right sum
    or an adjacent-pairs tree.  2^24 + 1 rounds back to 2^24 (tie to even), 2^24 + 2 is exact."""
    big = 2.0 ** 24

    def leaves(d):
        t = np.zeros(256, dtype=np.float32)
        for k, v in d.items():
            t[k] = v
        return t

    # level off=32 pairs 16 with 48 first: 1+1 = 2 survives, then 2^24 + 2 is exact.
    # (left-to-right and adjacent-pair trees meet 2^24 + 1 twice and give 2^24.)
    assert orc.tree256(leaves({0: big, 16: 1.0, 48: 1.0})) == f32(big + 2)
    # 1 and 33 are paired at the first level (off = 32): 2 survives to the last level
    assert orc.tree256(leaves({0: big, 1: 1.0, 33: 1.0})) == f32(big + 2)
    # 16 and 17 are NOT paired before meeting the big leaf's partial sums: leaf 16 joins leaf 0 at
    # off = 16 (2^24+1 -> 2^24), leaf 17 joins leaf 1 at off = 16 and reaches leaf 0 at off = 1.
    assert orc.tree256(leaves({0: big, 16: 1.0, 17: 1.0})) == f32(big)
    # 2 and 3: leaf 2 reaches leaf 0 at off = 2 (lost); leaf 3 reaches leaf 1 at off = 2, then
    # leaf 0 at off = 1 (lost).
    assert orc.tree256(leaves({0: big, 2: 1.0, 3: 1.0})) == f32(big)
    # 1 and 3 are paired at off = 2 (leaf 1 takes leaf 3): 2 survives
    assert orc.tree256(leaves({0: big, 1: 1.0, 3: 1.0})) == f32(big + 2)
    # group combine is (q0+q2)+(q1+q3): q1 and q3 meet first
    assert orc.tree256(leaves({0: big, 64: 1.0, 192: 1.0})) == f32(big + 2)
    # ... whereas q1 and q2 do not: q2 meets q0 first and is lost, then q1 is lost
    assert orc.tree256(leaves({0: big, 64: 1.0, 128: 1.0})) == f32(big)
    # q2, q3 do not meet first either
    assert orc.tree256(leaves({0: big, 128: 1.0, 192: 1.0})) == f32(big)


def test_tree256_close_to_fp64_sum(orc):
    rng = np.random.default_rng(5)
    for _ in range(20):
        t = rng.standard_normal(256).astype(np.float32)
        exact = t.astype(np.float64).sum()
        bound = 8 * 2.0 ** -24 * np.abs(t).astype(np.float64).sum()   # depth-8 tree
        assert abs(float(orc.tree256(t)) - exact) <= bound


# ------------------------------------------------------------------ RMSNorm

def test_sumsq_lane_mapping_hand_worked(orc):
    """Element e goes to lane (e/8) mod 256; a lane folds its elements in ascending order; the
    lanes then go through the tree.  4096^2 = 2^24, 1^2 = 1."""
    H = 4096
    one, big = 0x3F80, 0x4580   # bf16 bits of 1.0 and 4096.0

    def row(d):
        x = np.zeros(H, dtype=np.uint16)
        for k, v in d.items():
            x[k] = v
        return x

    # e = 1 shares lane 0 with e = 0: 2^24 + 1 -> 2^24; e = 2 likewise lost
    assert orc.sumsq(row({0: big, 1: one, 2: one})) == f32(2.0 ** 24)
    # e = 8 and e = 9 share lane 1: 1 + 1 = 2, joins lane 0 only at the last tree level: exact
    assert orc.sumsq(row({0: big, 8: one, 9: one})) == f32(2.0 ** 24 + 2)
    # e = 8 (lane 1) and e = 2056 = 8 + 2048 (lane 1 again, second sweep over the lanes)
    assert orc.sumsq(row({0: big, 8: one, 2056: one})) == f32(2.0 ** 24 + 2)
    # e = 8 (lane 1) and e = 16 (lane 2) meet the big value separately and are both lost
    assert orc.sumsq(row({0: big, 8: one, 16: one})) == f32(2.0 ** 24)
    # e = 8 (lane 1) and e = 8 + 8*32 (lane 33) are paired at the first level
    assert orc.sumsq(row({0: big, 8: one, 8 + 8 * 32: one})) == f32(2.0 ** 24 + 2)
    # H = 2048 has one sweep only: e = 2047 is lane 255
    x = np.zeros(2048, dtype=np.uint16)
    x[2047] = 0x4040   # 3.0
    assert orc.sumsq(x) == 9.0


def test_rmsnorm_closed_forms(orc):
    H = 4096
    two = np.full((1, H), 0x4000, dtype=np.uint16)        # x = 2 everywhere
    w1 = np.full(H, 0x3F80, dtype=np.uint16)
    y = orc.rmsnorm(two, w1, 0.0)                          # ss = 4H, mean = 4, r = 1/2
    assert np.all(y == 0x3F80)
    x = np.zeros((1, H), dtype=np.uint16)
    x[0, 77] = 0x4100                                      # one-hot 8: ss = 64, mean = 2^-6, r = 8
    w = np.full(H, 0x3FC0, dtype=np.uint16)                # w = 1.5
    y = orc.rmsnorm(x, w, 0.0)
    assert y[0, 77] == 0x42C0 and np.count_nonzero(y) == 1  # 96.0
    # eps sits inside the square root: x = 0 -> y = 0 (not NaN); x = 2^-3 one-hot at H = 2048
    z = orc.rmsnorm(np.zeros((1, H), dtype=np.uint16), w1, 1e-5)
    assert np.all(z == 0)


def test_rmsnorm_close_to_fp64_definition(orc):
    H = 4096
    x = ds.normal_bf16(11, (8, H))
    w = ds.normal_bf16(12, (H,), std=0.1, mean=1.0)
    y = orc.bf16_to_f32(orc.rmsnorm(x, w, 1e-5)).astype(np.float64)
    xf = ds.bf16_bits_to_f32(x).astype(np.float64)
    wf = ds.bf16_bits_to_f32(w).astype(np.float64)
    ref = xf / np.sqrt((xf ** 2).mean(axis=1, keepdims=True) + 1e-5) * wf
    assert np.all(np.abs(y - ref) <= 2.0 ** -8 * np.abs(ref) * 1.01 + 1e-30)
    # rows are independent: row 3 alone gives the same bytes
    assert np.array_equal(orc.rmsnorm(x[3:4], w, 1e-5)[0], orc.rmsnorm(x, w, 1e-5)[3])


# ------------------------------------------------------------------ softmax

def test_softmax_uniform_scores_exact(orc):
    for n in [1, 2, 64, 256, 512, 1024, 4096]:
        s = np.full((1, n), 3.25, dtype=np.float32)
        p, m, l = orc.softmax_f32(s, [n])
        assert m[0] == 3.25 and l[0] == n
        assert np.all(p == np.float32(1.0 / n))      # exact for a power of two


def test_softmax_lengths_and_mask(orc):
    rng = np.random.default_rng(6)
    Lmax = 600
    lens = [1, 255, 256, 257, 511, 512, 513, 0]
    s = rng.standard_normal((len(lens), Lmax)).astype(np.float32) * 3
    p, m, l = orc.softmax_f32(s, lens)
    from scipy.special import softmax
    for r, n in enumerate(lens):
        assert np.all(p[r, n:] == 0)
        if n == 0:
            assert np.isneginf(m[r]) and l[r] == 0
            continue
        ref = softmax(s[r, :n].astype(np.float64))
        assert np.abs(p[r, :n] - ref).max() <= 1e-6
        assert abs(p[r, :n].astype(np.float64).sum() - 1.0) <= 1e-6
        assert m[r] == s[r, :n].max()
        assert abs(l[r] - np.exp(s[r, :n].astype(np.float64) - m[r]).sum()) <= 1e-5 * l[r]
    # scores past the length must not matter, whatever they hold
    s2 = s.copy()
    for r, n in enumerate(lens):
        s2[r, n:] = np.nan
    p2, m2, l2 = orc.softmax_f32(s2, lens)
    assert np.array_equal(p, p2) and np.array_equal(m, m2) and np.array_equal(l, l2)


def test_softmax_one_hot_and_chunk_weights(orc):
    s = np.zeros((1, 1000), dtype=np.float32)
    s[0, 700] = 90.0                                  # 90 above everything: the rest underflows to 0
    p, m, l = orc.softmax_f32(s, [1000])
    assert p[0, 700] == 1.0 and np.count_nonzero(p) == 1 and l[0] == 1.0 and m[0] == 90.0
    # chunk 0 all 0, chunk 1 all -100: chunk 1's weight det_expf(-100) is exactly 0
    s = np.zeros((1, 512), dtype=np.float32)
    s[0, 256:] = -100.0
    p, m, l = orc.softmax_f32(s, [512])
    assert l[0] == 256.0 and np.all(p[0, :256] == np.float32(1 / 256)) and np.all(p[0, 256:] == 0)
    # chunk 0 all 0, chunk 1 all ln2-ish: the later chunk holds the maximum, so chunk 0 is
    # re-weighted by det_expf(0 - m) and chunk 1 by exactly 1
    s = np.zeros((1, 512), dtype=np.float32)
    s[0, 256:] = 1.0
    p, m, l = orc.softmax_f32(s, [512])
    w0 = orc.expf(np.array([-1.0], dtype=np.float32))[0]
    assert m[0] == 1.0
    assert l[0] == np.float32(np.float32(w0 * np.float32(256.0)) + np.float32(256.0))
    assert np.all(p[0, 256:] == np.float32(1.0) / l[0])
    assert np.all(p[0, :256] == w0 / l[0])


def test_softmax_long_row_sums_to_one(orc):
    s = ds.bf16_bits_to_f32(ds.normal_bf16(13, (2, 32768))).astype(np.float32)
    p, m, l = orc.softmax_f32(s, [32768, 30001])
    assert abs(p[0].astype(np.float64).sum() - 1.0) <= 1e-6
    assert abs(p[1].astype(np.float64).sum() - 1.0) <= 1e-6


# ------------------------------------------------------------------ argmax

def test_argmax_rules(orc):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((16, 32000)).astype(np.float32)
    assert np.array_equal(orc.argmax_f32(x), np.argmax(x, axis=1).astype(np.int32))
    t = np.zeros((6, 100), dtype=np.float32)
    t[0, :] = 5.0                                  # all equal -> 0
    t[1, [10, 50]] = 2.0                           # tie -> lowest index
    t[2, 99] = 1.0                                 # last element
    t[3, :] = -1.0; t[3, 40] = -0.0; t[3, 60] = 0.0   # -0 == +0 -> lowest index
    t[4, :] = np.nan                               # all NaN -> 0
    t[5, :] = -3.0; t[5, 5] = np.nan; t[5, 70] = -2.0   # NaN never wins
    assert orc.argmax_f32(t).tolist() == [0, 10, 99, 40, 0, 70]
    t2 = np.full((1, 10), -np.inf, dtype=np.float32)
    assert orc.argmax_f32(t2).tolist() == [0]
    xb = ds.normal_bf16(14, (8, 32000))
    assert np.array_equal(orc.argmax_bf16(xb), np.argmax(ds.bf16_bits_to_f32(xb), axis=1).astype(np.int32))


# ------------------------------------------------------------------ GEMM

def _b(x):
    return ds.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_gemm_hand_case(orc):
    A = _b([[1, 2, 3], [-1, 0.5, 4]])
    B = _b([[1, 0], [2, -1], [0.25, 8]])
    C, Ca = orc.gemm_f64(A, B)
    assert C.tolist() == [[1 + 4 + 0.75, -2 + 24], [-1 + 1 + 1, -0.5 + 32]]
    assert Ca.tolist() == [[5.75, 26], [3, 32.5]]


def test_gemm_identity_onehot_transpose(orc):
    K, N = 48, 40
    Bm = ds.normal_bf16(21, (K, N))
    eye = _b(np.eye(K))
    C, _ = orc.gemm_f64(eye, Bm)
    assert np.array_equal(C, ds.bf16_bits_to_f32(Bm).astype(np.float64))
    sel = np.zeros((3, K), dtype=np.float32)
    sel[0, 5] = 1; sel[1, 47] = 2; sel[2, 0] = -1
    C, _ = orc.gemm_f64(_b(sel), Bm)
    Bf = ds.bf16_bits_to_f32(Bm).astype(np.float64)
    assert np.array_equal(C, np.stack([Bf[5], 2 * Bf[47], -Bf[0]]))
    A = ds.normal_bf16(22, (17, K))
    C, Ca = orc.gemm_f64(A, Bm)
    Ct, _ = orc.gemm_f64(np.ascontiguousarray(Bm.T), np.ascontiguousarray(A.T))
    assert np.allclose(C, Ct.T, rtol=1e-14, atol=1e-14)
    Af = ds.bf16_bits_to_f32(A).astype(np.float64)
    assert np.allclose(C, Af @ Bf, rtol=1e-13, atol=1e-13)
    assert np.allclose(Ca, np.abs(Af) @ np.abs(Bf), rtol=1e-13, atol=1e-13)
    rows = np.array([0, 16, 3, 9]); cols = np.array([0, 39, 7, 20])
    c, ca = orc.gemm_f64_sample(A, Bm, rows, cols)
    assert np.allclose(c, C[rows, cols], rtol=1e-14) and np.allclose(ca, Ca[rows, cols], rtol=1e-14)


def test_gemm_integer_matrices_exact(orc):
    A = ds.small_int_bf16(23, (9, 300))
    Bm = ds.small_int_bf16(24, (300, 11))
    C, _ = orc.gemm_f64(A, Bm)
    ref = ds.bf16_bits_to_f32(A).astype(np.int64) @ ds.bf16_bits_to_f32(Bm).astype(np.int64)
    assert np.array_equal(C, ref.astype(np.float64))


# ------------------------------------------------------------------ attention decode

def _attn_inputs(seed, B, Hq, Hkv, D, Lmax):
    q = ds.normal_bf16(seed, (B, Hq, D))
    k = ds.normal_bf16(seed + 1, (B, Hkv, Lmax, D))
    v = ds.normal_bf16(seed + 2, (B, Hkv, Lmax, D))
    return q, k, v


def test_attention_closed_forms(orc):
    B, Hq, Hkv, D, Lmax = 2, 8, 2, 16, 40
    q, k, v = _attn_inputs(31, B, Hq, Hkv, D, Lmax)
    vf = ds.bf16_bits_to_f32(v).astype(np.float64)
    scale = 0.25
    # len = 1: output is v_0 of the right KV head (query head h reads KV head h // 4)
    out, oa = orc.attn_decode_f64(q, k, v, [1, 1], scale)
    for b in range(B):
        for h in range(Hq):
            assert np.array_equal(out[b, h], vf[b, h // 4, 0])
            assert np.array_equal(oa[b, h], np.abs(vf[b, h // 4, 0]))
    # q = 0: uniform scores -> column mean of V over the valid length
    out, _ = orc.attn_decode_f64(np.zeros_like(q), k, v, [40, 7], scale)
    assert np.allclose(out[0, 5], vf[0, 1, :40].mean(axis=0), rtol=1e-13, atol=1e-15)
    assert np.allclose(out[1, 2], vf[1, 0, :7].mean(axis=0), rtol=1e-13, atol=1e-15)
    # len = 0 -> zeros
    out, _ = orc.attn_decode_f64(q, k, v, [0, 3], scale)
    assert np.all(out[0] == 0)
    # dominant key: k_9 = 64*q direction makes token 9 win by > 700 in the exponent
    k2 = k.copy()
    qf = ds.bf16_bits_to_f32(q)
    k2[0, 0, 9] = ds.f32_to_bf16_bits(qf[0, 0] * 512)
    out, _ = orc.attn_decode_f64(q, k2, v, [40, 40], 1.0)
    assert np.allclose(out[0, 0], vf[0, 0, 9], rtol=0, atol=1e-200)
    # entries of the caches past the length must not matter
    k3, v3 = k.copy(), v.copy()
    k3[:, :, 20:] = 0x7FC0
    v3[:, :, 20:] = 0x7FC0
    a, _ = orc.attn_decode_f64(q, k, v, [20, 20], scale)
    b_, _ = orc.attn_decode_f64(q, k3, v3, [20, 20], scale)
    assert np.array_equal(a, b_)


def test_attention_vs_library_softmax(orc):
    from scipy.special import softmax
    B, Hq, Hkv, D, Lmax = 3, 8, 4, 32, 300
    q, k, v = _attn_inputs(41, B, Hq, Hkv, D, Lmax)
    lens = [300, 129, 1]
    scale = np.float32(1 / math.sqrt(D))
    out, oa = orc.attn_decode_f64(q, k, v, lens, scale)
    qf, kf, vf = (ds.bf16_bits_to_f32(t).astype(np.float64) for t in (q, k, v))
    for b in range(B):
        n = lens[b]
        for h in range(Hq):
            g = h // (Hq // Hkv)
            s = float(scale) * (kf[b, g, :n] @ qf[b, h])
            p = softmax(s)
            assert np.allclose(out[b, h], p @ vf[b, g, :n], rtol=1e-12, atol=1e-14)
            assert np.allclose(oa[b, h], p @ np.abs(vf[b, g, :n]), rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ elementwise

def test_rope_hand_cases(orc):
    D, Lmax = 16, 32
    cos_t, sin_t = ds.rope_tables(Lmax, D, 5.0e5)
    x = ds.normal_bf16(51, (4, 3, D))
    # position 0: cos = 1, sin = 0 -> identity
    assert np.array_equal(orc.rope(x, [0, 0, 0, 0], cos_t, sin_t), x)
    # a unit vector on element i rotates into (i, i + D/2) only: (cos, sin) of pos * theta^(-2i/D)
    for i in [0, 3, 7]:
        e = np.zeros((1, 1, D), dtype=np.uint16)
        e[0, 0, i] = 0x3F80
        y = orc.rope(e, [5], cos_t, sin_t)[0, 0]
        ang = 5 * (5.0e5 ** (-2.0 * i / D))
        assert y[i] == _b([math.cos(ang)])[0] and y[i + D // 2] == _b([math.sin(ang)])[0]
        assert np.count_nonzero(y) == 2
        e = np.zeros((1, 1, D), dtype=np.uint16)
        e[0, 0, i + D // 2] = 0x3F80
        y = orc.rope(e, [5], cos_t, sin_t)[0, 0]
        assert y[i] == _b([-math.sin(ang)])[0] and y[i + D // 2] == _b([math.cos(ang)])[0]
    # close to the exact rotation, and per-row positions are honoured
    pos = [1, 7, 20, 31]
    y = orc.bf16_to_f32(orc.rope(x, pos, cos_t, sin_t)).astype(np.float64)
    xf = ds.bf16_bits_to_f32(x).astype(np.float64)
    for r, p in enumerate(pos):
        ang = p * (5.0e5 ** (-2.0 * np.arange(D // 2) / D))
        lo, hi = xf[r, :, :D // 2], xf[r, :, D // 2:]
        ref = np.concatenate([lo * np.cos(ang) - hi * np.sin(ang), lo * np.sin(ang) + hi * np.cos(ang)], axis=1)
        assert np.all(np.abs(y[r] - ref) <= 2.0 ** -8 * np.abs(ref) + 2.0 ** -22 * (np.abs(lo).max() + np.abs(hi).max()))


def test_swiglu_and_residual(orc):
    g = _b([0.0, 1.0, -1.0, 30.0, -30.0, 100.0, -100.0, 2.5])
    u = _b([3.0, 2.0, 2.0, 1.5, 1.5, 1.0, 1.0, -4.0])
    y = orc.bf16_to_f32(orc.swiglu(g, u)).astype(np.float64)
    gf, uf = ds.bf16_bits_to_f32(g).astype(np.float64), ds.bf16_bits_to_f32(u).astype(np.float64)
    ref = gf / (1 + np.exp(-gf)) * uf
    assert y[0] == 0.0
    assert y[3] == 45.0            # silu(30) = 30 to fp32 precision; 30*1.5 exact
    assert y[5] == 100.0 and y[6] == 0.0   # det_expf(100) = inf -> -100/inf = -0
    assert np.all(np.abs(y - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-12)
    gg = ds.normal_bf16(61, (4096,), std=2.0)
    uu = ds.normal_bf16(62, (4096,))
    yy = orc.bf16_to_f32(orc.swiglu(gg, uu)).astype(np.float64)
    gf, uf = ds.bf16_bits_to_f32(gg).astype(np.float64), ds.bf16_bits_to_f32(uu).astype(np.float64)
    ref = gf / (1 + np.exp(-gf)) * uf
    assert np.all(np.abs(yy - ref) <= 2.0 ** -8 * np.abs(ref) * 1.001 + 1e-30)
    # residual: 1 + 2^-8 is a tie -> 1.0 ; 256 + 1 -> 256 (tie to even); 3 + 0.5 exact
    z = orc.residual(_b([1.0, 256.0, 3.0]), _b([2.0 ** -8, 1.0, 0.5]))
    assert z.tolist() == [0x3F80, 0x4380, 0x4060]


# ------------------------------------------------------------------ decoder layer glue

def _layer_setup(seed=71, B=3):
    cfg = dict(H=64, Hq=4, Hkv=2, D=16, F=96, Lmax=12, eps=1e-5, scale=float(np.float32(0.25)))
    H, Hq, Hkv, D, F, Lmax = (cfg[k] for k in ("H", "Hq", "Hkv", "D", "F", "Lmax"))
    w = dict(
        norm1=ds.normal_bf16(seed, (H,), 0.1, 1.0),
        wqkv=ds.normal_bf16(seed + 1, (H, (Hq + 2 * Hkv) * D), 0.2),
        wo=ds.normal_bf16(seed + 2, (Hq * D, H), 0.2),
        norm2=ds.normal_bf16(seed + 3, (H,), 0.1, 1.0),
        wgu=ds.normal_bf16(seed + 4, (H, 2 * F), 0.2),
        wdown=ds.normal_bf16(seed + 5, (F, H), 0.2),
    )
    x = ds.normal_bf16(seed + 6, (B, H))
    kc = ds.normal_bf16(seed + 7, (B, Hkv, Lmax, D))
    vc = ds.normal_bf16(seed + 8, (B, Hkv, Lmax, D))
    pos = np.array([0, 5, 11][:B], dtype=np.int32)
    cos_t, sin_t = ds.rope_tables(Lmax, D)
    return cfg, w, x, kc, vc, pos, cos_t, sin_t


def test_decoder_layer_matches_composition_of_ops(orc):
    """The layer's glue (column layout of the fused projections, which head reads which cache,
    where the new K/V rows land, where the residuals are added) against a composition written
    here from the per-op oracle functions and numpy's fp64 matmul."""
    cfg, w, x, kc, vc, pos, cos_t, sin_t = _layer_setup()
    H, Hq, Hkv, D, F, Lmax = (cfg[k] for k in ("H", "Hq", "Hkv", "D", "F", "Lmax"))
    B = x.shape[0]
    kc1, vc1 = kc.copy(), vc.copy()
    got = orc.decoder_layer(x, w, kc1, vc1, pos, cos_t, sin_t, cfg)

    def mm(a, b):
        return orc.bf16_from_f64(ds.bf16_bits_to_f32(a).astype(np.float64) @ ds.bf16_bits_to_f32(b).astype(np.float64))

    h = orc.rmsnorm(x, w["norm1"], cfg["eps"])
    qkv = mm(h, w["wqkv"])
    q = orc.rope(qkv[:, :Hq * D].reshape(B, Hq, D), pos, cos_t, sin_t)
    k = orc.rope(qkv[:, Hq * D:(Hq + Hkv) * D].reshape(B, Hkv, D), pos, cos_t, sin_t)
    v = qkv[:, (Hq + Hkv) * D:].reshape(B, Hkv, D)
    kc2, vc2 = kc.copy(), vc.copy()
    for b in range(B):
        kc2[b, :, pos[b]] = k[b]
        vc2[b, :, pos[b]] = v[b]
    assert np.array_equal(kc1, kc2) and np.array_equal(vc1, vc2)
    a, _ = orc.attn_decode_f64(q, kc2, vc2, pos + 1, cfg["scale"])
    a = orc.bf16_from_f64(a).reshape(B, Hq * D)
    x1 = orc.residual(x, mm(a, w["wo"]))
    h2 = orc.rmsnorm(x1, w["norm2"], cfg["eps"])
    gu = mm(h2, w["wgu"])
    m = orc.swiglu(gu[:, :F], gu[:, F:])
    x2 = orc.residual(x1, mm(m, w["wdown"]))
    assert np.array_equal(got, x2)


def test_decoder_layer_zero_projections_leave_x(orc):
    cfg, w, x, kc, vc, pos, cos_t, sin_t = _layer_setup(seed=81)
    w = dict(w)
    w["wo"] = np.zeros_like(w["wo"])
    w["wdown"] = np.zeros_like(w["wdown"])
    got = orc.decoder_layer(x, w, kc.copy(), vc.copy(), pos, cos_t, sin_t, cfg)
    assert np.array_equal(got, x)


def test_decoder_layer_rows_independent(orc):
    cfg, w, x, kc, vc, pos, cos_t, sin_t = _layer_setup(seed=91)
    full = orc.decoder_layer(x, w, kc.copy(), vc.copy(), pos, cos_t, sin_t, cfg)
    one = orc.decoder_layer(x[1:2], w, kc[1:2].copy(), vc[1:2].copy(), pos[1:2], cos_t, sin_t, cfg)
    assert np.array_equal(full[1], one[0])


def test_python_composed_layer_equals_the_c_layer_and_bound_is_sane(orc):
    """oracle.model.layer (the composition that also returns intermediates) gives the bytes of
    orc.decoder_layer, which the test above pins to numpy's matmul; its element-wise bound is at least one
    ulp of the output and far below the output's magnitude."""
    from oracle import model as om

    cfg, w, x, kc, vc, pos, cos_t, sin_t = _layer_setup(seed=101)
    kc1, vc1, kc2, vc2 = kc.copy(), vc.copy(), kc.copy(), vc.copy()
    want = orc.decoder_layer(x, w, kc1, vc1, pos, cos_t, sin_t, cfg)
    got, inter = om.layer(x, w, kc2, vc2, pos, cos_t, sin_t, cfg)
    assert np.array_equal(got, want) and np.array_equal(kc1, kc2) and np.array_equal(vc1, vc2)
    bound = om.layer_bound(got, inter)
    f = np.abs(ds.bf16_bits_to_f32(got).astype(np.float64))
    assert (bound >= om.ulp_bf16(got)).all() and np.median(bound / np.maximum(f, 1e-30)) < 0.1
    # ulp_bf16 against the definition: the distance to the next bf16 value of the same sign
    vals = ds.f32_to_bf16_bits(np.array([1.0, 1.5, 0.75, 3.0, 100.0, 2.0 ** -20], dtype=np.float32))
    nxt = ds.bf16_bits_to_f32(vals + 1).astype(np.float64) - ds.bf16_bits_to_f32(vals).astype(np.float64)
    assert np.array_equal(om.ulp_bf16(vals), nxt)


def test_model_step_glue(orc):
    """oracle.model.model_step: with the attention and MLP branches zeroed the logits are the lm_head
    product of the normalised embedding row of each token (embedding gather, final norm, lm_head
    orientation); rows are independent; and a second step at position 1 sees the cache row the first wrote."""
    from oracle import model as om

    cfg, w, x, kc, vc, pos, cos_t, sin_t = _layer_setup(seed=111)
    H, V = cfg["H"], 48
    Wt = dict(embed=ds.normal_bf16(120, (30, H)), lm_head=ds.normal_bf16(121, (H, V), 0.1),
              final_norm=ds.normal_bf16(122, (H,), 0.1, 1.0), layers=[w, w])
    zero = dict(w, wo=np.zeros_like(w["wo"]), wdown=np.zeros_like(w["wdown"]))
    Wz = dict(Wt, layers=[zero, zero])
    shape = (2, cfg["Hkv"], cfg["Lmax"], cfg["D"])
    new = lambda: [np.zeros(shape, dtype=np.uint16) for _ in range(2)]
    toks = np.array([7, 29])
    lg = om.model_step(Wz, cfg, toks, [0, 0], new(), new(), cos_t, sin_t)
    xn = ds.bf16_bits_to_f32(orc.rmsnorm(Wt["embed"][toks], Wt["final_norm"], cfg["eps"])).astype(np.float64)
    assert np.array_equal(lg, xn @ ds.bf16_bits_to_f32(Wt["lm_head"]).astype(np.float64))
    # full model: rows independent, and step 1 reads what step 0 wrote at cache row 0
    kcs, vcs = new(), new()
    l0 = om.model_step(Wt, cfg, toks, [0, 0], kcs, vcs, cos_t, sin_t)
    k1, v1 = [k[1:2].copy() * 0 for k in kcs], [v[1:2].copy() * 0 for v in vcs]
    assert np.array_equal(om.model_step(Wt, cfg, toks[1:], [0], k1, v1, cos_t, sin_t)[0], l0[1])
    assert all(np.array_equal(a[0], b[1]) for a, b in zip(k1, kcs))
    l1 = om.model_step(Wt, cfg, [3, 4], [1, 1], kcs, vcs, cos_t, sin_t)
    wiped = [k.copy() for k in kcs]
    for k in wiped:
        k[:, :, 0] = 0                                     # forget the first token's keys: the logits must change
    l1w = om.model_step(Wt, cfg, [3, 4], [1, 1], wiped, [v.copy() for v in vcs], cos_t, sin_t)
    assert not np.array_equal(l1, l1w)


# ------------------------------------------------------------------ input generator

def test_generator_host_and_torch_paths_agree():
    a = ds.normal_bf16(5, (257, 129), 0.02)
    b = ds.from_torch_bf16(ds.normal_bf16_torch(5, (257, 129), 0.02, device="cpu"))
    assert np.array_equal(a, b)
    assert np.array_equal(ds.normal_bf16_slice(5, 1000, 77, 0.02), a.reshape(-1)[1000:1077])
    f = ds.bf16_bits_to_f32(ds.normal_bf16(6, (1 << 18,)))
    assert abs(f.mean()) < 0.01 and abs(f.std() - 1) < 0.01
    ids = ds.uniform_int(7, (10000,), 16, 512)
    assert ids.min() == 16 and ids.max() == 512


# ------------------------------------------------------------------ stored digests of the oracle

def test_oracle_matches_stored_digests(orc):
    """tests/golden/oracle_golden.txt was written by a committed script that calls only the oracle;
    the oracle must keep producing those bytes unless a commit says why they changed."""
    import importlib.util
    import os

    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(here, "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = dict(line.split() for line in open(os.path.join(here, "oracle_golden.txt")) if not line.startswith("#"))
    got = dict(mod.digests())
    assert got == stored


# ------------------------------------------------------------------ seeded sampling

def test_sample_uniform_matches_independent_splitmix_and_is_uniform(orc):
    """The counter-based uniform against the input generator's own numpy splitmix64 (written
    separately from the same published algorithm), and its first two moments."""
    seed = 0x1234_5678_9ABC_DEF0
    for seq, step in [(0, 0), (5, 17), (63, 511), (2 ** 31 - 1, 2 ** 31 - 1)]:
        ctr = (seq << 32) | step
        h = ds._hash_np(seed, ctr, 1)[0]           # splitmix64 output number ctr for state seed
        want = np.float32(int(h) >> 40) * np.float32(2.0 ** -24)
        assert orc.sample_uniform(seed, seq, step) == want
    u = np.array([orc.sample_uniform(7, s, t) for s in range(40) for t in range(500)], dtype=np.float64)
    assert 0.0 <= u.min() and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005


def test_sample_closed_forms(orc):
    V = 1000
    rng = np.random.default_rng(8)
    x = rng.standard_normal((32, V)).astype(np.float32)
    ids = np.arange(32, dtype=np.int32)
    st = np.full(32, 3, dtype=np.int32)
    # top_k = 1 is greedy decoding, whatever the temperature, top_p or seed
    for T, p, seed in [(1.0, 1.0, 1), (0.3, 0.5, 99), (5.0, 1e-6, 2 ** 63 + 5)]:
        assert np.array_equal(orc.sample(x, T, 1, p, seed, ids, st), orc.argmax_f32(x))
    # a tiny top_p keeps the first candidate only
    assert np.array_equal(orc.sample(x, 1.0, 50, 1e-6, 4, ids, st), orc.argmax_f32(x))
    # all logits equal, top_k = 4: only the four lowest indices can come out, about equally often
    flat = np.zeros((4000, V), dtype=np.float32)
    tok = orc.sample(flat, 1.0, 4, 1.0, 11, np.arange(4000, dtype=np.int32), np.zeros(4000, dtype=np.int32))
    cnt = np.bincount(tok, minlength=V)
    assert cnt[4:].sum() == 0 and np.all(np.abs(cnt[:4] - 1000) < 5 * np.sqrt(1000 * 0.75))
    # two-point distribution: z = (0, -ln 2) -> probabilities (2/3, 1/3)
    two = np.full((6000, V), -200.0, dtype=np.float32)
    two[:, 10] = 0.0
    two[:, 700] = -np.float32(np.log(2.0))
    tok = orc.sample(two, 1.0, 40, 1.0, 5, np.arange(6000, dtype=np.int32), np.full(6000, 9, dtype=np.int32))
    assert set(np.unique(tok)) == {10, 700}
    assert abs((tok == 10).mean() - 2 / 3) < 5 * np.sqrt(2 / 9 / 6000)
    # temperature 0.5 squares the odds: (4/5, 1/5)
    tok = orc.sample(two, 0.5, 40, 1.0, 5, np.arange(6000, dtype=np.int32), np.full(6000, 9, dtype=np.int32))
    assert abs((tok == 10).mean() - 0.8) < 5 * np.sqrt(0.16 / 6000)
    # top_p: cumulative (2/3, 1) -> top_p = 0.6 keeps token 10 only, top_p = 0.7 keeps both
    assert np.all(orc.sample(two, 1.0, 40, 0.6, 5, np.arange(6000, dtype=np.int32), np.full(6000, 9, dtype=np.int32)) == 10)
    assert (orc.sample(two, 1.0, 40, 0.7, 5, np.arange(6000, dtype=np.int32), np.full(6000, 9, dtype=np.int32)) == 700).any()
    # a sample depends on (seed, sequence id, step), not on the row slot or the batch
    a = orc.sample(x, 0.9, 64, 0.95, 42, ids, st)
    perm = rng.permutation(32)
    assert np.array_equal(orc.sample(x[perm], 0.9, 64, 0.95, 42, ids[perm], st[perm]), a[perm])
    assert np.array_equal(orc.sample(x[5:6], 0.9, 64, 0.95, 42, ids[5:6], st[5:6]), a[5:6])
    assert not np.array_equal(orc.sample(x, 0.9, 64, 0.95, 43, ids, st), a)      # the seed matters
    # NaN logits are never sampled
    xn = x.copy()
    xn[:, ::2] = np.nan
    assert np.all(orc.sample(xn, 1.0, 64, 1.0, 1, ids, st) % 2 == 1)


def test_sample_cut_and_pick_comparisons_are_pinned_on_their_boundaries(orc):
    """Targets and cuts that land exactly on a prefix sum, and just beside it: the strictness of
    'c_i >= cut' and 'c_i > target' decides the token, and the expected tokens are worked out from
    integers in tests/sample_cases.py, not by the oracle."""
    import sample_cases as sc

    logits, steps, want, ids = sc.pick_boundary_case()
    assert len(set(want.tolist())) > 3 and want.min() >= 0
    got = orc.sample(logits, 1.0, 1024, 1.0, 0xC0FFEE, ids, steps)
    assert np.array_equal(got, want)
    cases, logits, steps, ids = sc.cut_boundary_case()
    for top_p, want in cases:
        assert 0 < (want == want.max()).sum() < want.size      # both sides of each threshold occur
        got = orc.sample(logits, 1.0, 4, top_p, 0xBEEF, ids, steps)
        assert np.array_equal(got, want), top_p
    assert cases[1][1].max() == 2 and cases[0][1].max() == 1
