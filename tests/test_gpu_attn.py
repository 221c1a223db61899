"""det_attn_decode against the fp64 oracle (bound: |err| <= 2^-8 |ref| + 2^-20 sum_j p_j |v_jd|),
its closed forms, and byte equality of a (sequence, head) across batch compositions."""
import math

import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, bits_to_f64, down_bf16, step, up, up_bf16, within_bound

pytestmark = pytest.mark.gpu

SCALE = float(np.float32(1.0 / math.sqrt(128.0)))


@pytest.fixture(scope="module")
def d():
    import paper_2602_00182_amd as d
    return d


def run_attn(d, q, k, v, lens, scale=SCALE, poison_ws=False):
    B, Hq, D = q.shape
    Lmax = k.shape[2]
    ws = torch.empty(d.det_attn_decode_workspace_bytes(B, Hq, D, Lmax), dtype=torch.uint8, device=DEV)
    if poison_ws:
        ws.fill_(0xFF)
    out = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=DEV)
    d.det_attn_decode(up_bf16(q), up_bf16(k), up_bf16(v), up(np.asarray(lens, dtype=np.int32)), out, ws, scale)
    torch.cuda.synchronize()
    return down_bf16(out)


def inputs(seed, B, Hq, Hkv, Lmax, D=128):
    return (ds.normal_bf16(seed, (B, Hq, D)), ds.normal_bf16(seed + 1, (B, Hkv, Lmax, D)),
            ds.normal_bf16(seed + 2, (B, Hkv, Lmax, D)))


@pytest.mark.parametrize("B,Hq,Hkv,Lmax,lens", [
    (1, 32, 8, 512, [512]),
    (4, 32, 8, 1024, [1, 255, 257, 1024]),
    (3, 8, 8, 600, [600, 513, 256]),
    (2, 16, 8, 300, [300, 2]),
    (2, 16, 2, 768, [700, 511]),
    (16, 32, 8, 4096, None),
])
def test_attention_vs_oracle(d, orc, B, Hq, Hkv, Lmax, lens):
    q, k, v = inputs(ds.tensor_seed(3, 10) + Lmax + B, B, Hq, Hkv, Lmax)
    if lens is None:   # ragged: lengths uniform in [1, Lmax]
        lens = ds.uniform_int(ds.tensor_seed(3, 13), (B,), 1, Lmax)
        lens[0] = Lmax
    step(f"attention B={B} Hq={Hq} Hkv={Hkv} Lmax={Lmax}")
    got = run_attn(d, q, k, v, lens, poison_ws=True)
    ref, refabs = orc.attn_decode_f64(q, k, v, lens, SCALE)
    ok = within_bound(bits_to_f64(got), ref, refabs)
    assert ok.all(), f"{(~ok).sum()} of {ok.size} outside the bound"


def test_attention_closed_forms(d, orc):
    B, Hq, Hkv, Lmax = 2, 32, 8, 1024
    q, k, v = inputs(500, B, Hq, Hkv, Lmax)
    step("attention len=1")
    got = run_attn(d, q, k, v, [1, 1])
    for h in range(Hq):
        assert np.array_equal(got[0, h], v[0, h // 4, 0]) and np.array_equal(got[1, h], v[1, h // 4, 0])
    step("attention len=0")
    got = run_attn(d, q, k, v, [0, 5])
    assert np.all(got[0] == 0)
    step("attention uniform scores")
    vi = ds.small_int_bf16(501, (B, Hkv, Lmax, 128), -8, 8)    # integer V: column sums exact in fp32
    got = run_attn(d, np.zeros_like(q), k, vi, [1024, 512])
    vf = ds.bf16_bits_to_f32(vi).astype(np.float64)
    for b, n in [(0, 1024), (1, 512)]:
        want = orc.bf16_rne((vf[b, :, :n].sum(axis=1) / n).astype(np.float32))   # exact: n is 2^k
        for h in range(Hq):
            assert np.array_equal(got[b, h], want[h // 4])
    step("attention dominant key")
    k2 = k.copy()
    qf = ds.bf16_bits_to_f32(q)
    k2[0, 2, 700] = ds.f32_to_bf16_bits(qf[0, 8] * 64)   # head 8 reads KV head 2
    got = run_attn(d, q, k2, v, [1024, 1024], scale=1.0)
    assert np.array_equal(got[0, 8], v[0, 2, 700])


def test_cache_past_len_is_ignored_and_batch_invariance(d, orc):
    B, Hq, Hkv, Lmax = 16, 32, 8, 2048
    q, k, v = inputs(510, B, Hq, Hkv, Lmax)
    lens = ds.uniform_int(511, (B,), 1, Lmax)
    lens[3] = 777
    step("attention batch 16")
    base = run_attn(d, q, k, v, lens)
    k2, v2 = k.copy(), v.copy()
    for b in range(B):
        k2[b, :, lens[b]:] = 0x7FC0     # NaN patterns past the length
        v2[b, :, lens[b]:] = 0xFF80     # -inf
    step("attention batch 16, poisoned tails")
    assert np.array_equal(run_attn(d, q, k2, v2, lens), base)
    step("attention sequence 3 alone")
    alone = run_attn(d, q[3:4], k[3:4], v[3:4], lens[3:4])
    assert np.array_equal(alone[0], base[3])
    step("attention sequence 3 in another slot among other sequences")
    q3, k3, v3 = inputs(520, 5, Hq, Hkv, Lmax)
    q3[4], k3[4], v3[4] = q[3], k[3], v[3]
    other = run_attn(d, q3, k3, v3, [5, 2048, 1, 300, lens[3]])
    assert np.array_equal(other[4], base[3])
    step("attention repeat x20")
    for _ in range(20):
        assert np.array_equal(run_attn(d, q, k, v, lens, poison_ws=True), base)


def test_long_context_sampled(d, orc):
    """L = 32768 at B = 2 (128 chunks per sequence): the oracle on sampled (sequence, head) pairs."""
    B, Hq, Hkv, Lmax = 2, 32, 8, 32768
    q, k, v = inputs(530, B, Hq, Hkv, Lmax)
    lens = [32768, 30001]
    step("attention L=32768")
    got = run_attn(d, q, k, v, lens)
    for b, heads in [(0, [0, 13, 31]), (1, [5, 22])]:
        for h in heads:
            g = h // 4
            ref, refabs = orc.attn_decode_f64(q[b:b + 1, h:h + 1], k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1],
                                              lens[b:b + 1], SCALE)
            assert within_bound(bits_to_f64(got[b, h]), ref[0, 0], refabs[0, 0]).all()


def test_full_size_batch64_context32768_sampled(d, orc):
    """The largest configuration bench.py times (B = 64, L = 32768: 8.6 GB of KV cache), generated
    on the device; the oracle recomputes sampled (sequence, head) pairs from the same counter-based
    generator on the host, so no input or expected value comes from the GPU."""
    B, Hq, Hkv, Lmax, D = 64, 32, 8, 32768, 128
    sq, sk, sv = ds.tensor_seed(3, 20), ds.tensor_seed(3, 21), ds.tensor_seed(3, 22)
    step("attention B=64 L=32768: generating 8.6 GB of cache on the device")
    q = ds.normal_bf16_torch(sq, (B, Hq, D), 1.0, 0.0, DEV)
    k = ds.normal_bf16_torch(sk, (B, Hkv, Lmax, D), 1.0, 0.0, DEV)
    v = ds.normal_bf16_torch(sv, (B, Hkv, Lmax, D), 1.0, 0.0, DEV)
    lens_h = ds.uniform_int(ds.tensor_seed(3, 23), (B,), Lmax // 2, Lmax)
    lens_h[0] = Lmax
    lens = up(lens_h)
    ws = torch.empty(d.det_attn_decode_workspace_bytes(B, Hq, D, Lmax), dtype=torch.uint8, device=DEV)
    out = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=DEV)
    step("attention B=64 L=32768: launch")
    d.det_attn_decode(q, k, v, lens, out, ws, SCALE)
    torch.cuda.synchronize()
    got = down_bf16(out)
    del k, v, ws
    torch.cuda.empty_cache()
    per_head = Lmax * D
    for b, h in [(0, 0), (17, 13), (63, 31), (40, 6)]:
        g = h // 4
        qh = ds.normal_bf16_slice(sq, (b * Hq + h) * D, D).reshape(1, 1, D)
        kh = ds.normal_bf16_slice(sk, (b * Hkv + g) * per_head, per_head).reshape(1, 1, Lmax, D)
        vh = ds.normal_bf16_slice(sv, (b * Hkv + g) * per_head, per_head).reshape(1, 1, Lmax, D)
        ref, refabs = orc.attn_decode_f64(qh, kh, vh, lens_h[b:b + 1], SCALE)
        assert within_bound(bits_to_f64(got[b, h]), ref[0, 0], refabs[0, 0]).all(), (b, h)


def test_rows_variant_slots(d, orc):
    """det_attn_decode_rows: identity slots give the bytes of det_attn_decode; a permuted slot table
    gives the permuted rows; rows that share one slot at lengths 1..R (the tokens of a prompt) each
    equal the single-row call on that slot at that length."""
    S, Hq, Hkv, Lmax = 6, 32, 8, 700
    q, k, v = inputs(560, S, Hq, Hkv, Lmax)
    lens = np.asarray([700, 1, 256, 257, 511, 40], dtype=np.int32)
    plain = run_attn(d, q, k, v, lens)

    def rows(qr, slots, seqlens):
        R = qr.shape[0]
        ws = torch.empty(d.det_attn_decode_workspace_bytes(R, Hq, 128, Lmax), dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)
        out = torch.empty((R, Hq, 128), dtype=torch.bfloat16, device=DEV)
        d.det_attn_decode_rows(up_bf16(qr), up_bf16(k), up_bf16(v), up(np.asarray(seqlens, dtype=np.int32)),
                               up(np.asarray(slots, dtype=np.int32)), out, ws, SCALE)
        torch.cuda.synchronize()
        return down_bf16(out)

    step("attention rows, identity slots")
    assert np.array_equal(rows(q, np.arange(S), lens), plain)
    step("attention rows, permuted slots")
    perm = np.asarray([4, 0, 5, 2, 2, 1])
    assert np.array_equal(rows(q[perm], perm, lens[perm]), plain[perm])
    step("attention rows, 300 rows on one slot at lengths 1..300")
    R = 300
    qr = ds.normal_bf16(565, (R, Hq, 128))
    got = rows(qr, np.full(R, 3), np.arange(1, R + 1))
    for r in (0, 1, 127, 255, 256, 299):
        q1 = np.repeat(qr[r:r + 1], S, axis=0)
        one = run_attn(d, q1, k, v, np.full(S, r + 1, dtype=np.int32))
        assert np.array_equal(got[r], one[3])
    # rows of the shared-chunk path against the fp64 definition: the first tiles, the tile that straddles
    # the chunk boundary at 256 tokens, and the last tile
    for r in list(range(0, 17)) + [250, 254, 255, 256, 257, 263, 264, 296, 299]:
        ref, refabs = orc.attn_decode_f64(qr[r:r + 1], k[3:4], v[3:4], [r + 1], SCALE)
        assert within_bound(bits_to_f64(got[r:r + 1]), ref, refabs).all(), r


def test_quantized_output_equals_quantizer_of_the_output(d, orc):
    """det_attn_decode_quant_q8 writes the activation codes and scales of the attention output: the
    oracle's quantizer applied to the bytes det_attn_decode returns (which the tests above hold to the
    attention bound), with and without slots, ragged lengths, a zero-length row."""
    B, Hq, Hkv, Lmax = 5, 16, 4, 700
    q, k, v = inputs(ds.tensor_seed(3, 60), B, Hq, Hkv, Lmax)
    lens = np.asarray([700, 1, 257, 0, 512], dtype=np.int32)
    step("attention with quantized output")
    plain = run_attn(d, q, k, v, lens)
    ws = torch.empty(d.det_attn_decode_workspace_bytes(B, Hq, 128, Lmax), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    codes = torch.full((B, Hq * 128), 99, dtype=torch.int8, device=DEV)
    scales = torch.full((d.det_quant_act_scales_bytes(B, Hq * 128) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    d.det_attn_decode_quant_q8(up_bf16(q), up_bf16(k), up_bf16(v), up(lens), None, codes, scales, ws, SCALE)
    torch.cuda.synchronize()
    po, do = orc.quant_a8(plain.reshape(B, Hq * 128))
    ldd = (B + 3) & ~3
    got_d = np.ascontiguousarray(scales.cpu().numpy().reshape(Hq * 2, ldd)[:, :B].T)
    assert np.array_equal(codes.cpu().numpy(), po) and np.array_equal(got_d.view(np.uint32), do.view(np.uint32))
    step("attention with quantized output, rows on permuted slots")
    slots = np.asarray([3, 0, 4, 1, 2], dtype=np.int32)
    codes2 = torch.empty_like(codes)
    scales2 = torch.empty_like(scales)
    d.det_attn_decode_quant_q8(up_bf16(q[slots]), up_bf16(k), up_bf16(v), up(lens[slots]), up(slots), codes2, scales2, ws,
                               SCALE)
    torch.cuda.synchronize()
    # row r now attends with the query and length of sequence slots[r] over cache slot slots[r]
    assert np.array_equal(codes2.cpu().numpy(), po[slots])
    got_d2 = np.ascontiguousarray(scales2.cpu().numpy().reshape(Hq * 2, ldd)[:, :B].T)
    assert np.array_equal(got_d2.view(np.uint32), do[slots].view(np.uint32))


@pytest.mark.parametrize("B,Hq,Hkv,Lmax,path", [
    (1, 32, 8, 1024, "one workgroup per query head, V through LDS"),
    (6, 32, 8, 1024, "4 heads per workgroup, V through LDS"),
    (20, 32, 8, 1024, "4 heads per workgroup, V from global memory"),
    (3, 8, 8, 600, "1 head per KV head"),
    (10, 16, 8, 512, "2 heads per workgroup"),
    (9, 16, 2, 2048, "8 heads per workgroup"),
])
def test_chunk_statistics_bitwise_against_reference_softmax(d, orc, B, Hq, Hkv, Lmax, path):
    """The attention kernel's own m_c and l_c, read out of the workspace, equal the reference statistics of
    the same scores bit for bit (section 6.5, invariant 2: the reduction tree), ragged lengths included.
    The scores are exact by construction: q and k hold small integers (every partial sum of a dot product
    is an integer below 2^24, so the accumulation order cannot matter) and the scale is a power of two, so
    the host computes the very fp32 scores the kernel does, with integer arithmetic.  The combined m and L
    of the same rows are checked through det_softmax_f32, which runs the same per-chunk device routine."""
    seed = ds.tensor_seed(3, 500) + 7 * B + Lmax
    qi = ds.uniform_int(seed, (B, Hq, 128), -3, 3)
    ki = ds.uniform_int(seed + 1, (B, Hkv, Lmax, 128), -3, 3)
    q = ds.f32_to_bf16_bits(qi.astype(np.float32))
    k = ds.f32_to_bf16_bits(ki.astype(np.float32))
    v = ds.normal_bf16(seed + 2, (B, Hkv, Lmax, 128))
    lens = ds.uniform_int(seed + 3, (B,), 1, Lmax)
    lens[0] = Lmax
    for i, special in enumerate([1, 255, 256, 257]):
        if i + 1 < B:
            lens[i + 1] = min(special, Lmax)
    scale = 0.125
    nc = (Lmax + 255) // 256
    ws = torch.empty(d.det_attn_decode_workspace_bytes(B, Hq, 128, Lmax), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    out = torch.empty((B, Hq, 128), dtype=torch.bfloat16, device=DEV)
    step(f"chunk statistics bitwise: B={B} Hq={Hq} Hkv={Hkv} Lmax={Lmax} ({path})")
    d.det_attn_decode(up_bf16(q), up_bf16(k), up_bf16(v), up(lens.astype(np.int32)), out, ws, scale)
    torch.cuda.synchronize()
    n = B * Hq * nc
    wsf = ws.cpu().numpy().view(np.float32)
    got_m = wsf[:n].reshape(B, Hq, nc)
    got_l = wsf[n:2 * n].reshape(B, Hq, nc)
    G = Hq // Hkv
    # exact scores [B, Hq, Lmax]: integer dot products times 2^-3
    s = np.empty((B, Hq, Lmax), dtype=np.float32)
    for h in range(Hq):
        s[:, h, :] = (np.einsum("bd,btd->bt", qi[:, h, :].astype(np.int64), ki[:, h // G, :, :].astype(np.int64))
                      .astype(np.float32) * np.float32(scale))
    # per chunk: a chunk alone is a one-chunk row, whose reference (m, L) are its (m_c, l_c)
    rows = s.reshape(B * Hq * nc, 256) if Lmax % 256 == 0 else None
    if rows is None:
        pad = np.zeros((B, Hq, nc * 256), dtype=np.float32)
        pad[:, :, :Lmax] = s
        rows = pad.reshape(B * Hq * nc, 256)
    clen = np.clip(lens[:, None, None] - 256 * np.arange(nc)[None, None, :], 0, 256)
    clen = np.broadcast_to(clen, (B, Hq, nc)).reshape(-1).astype(np.int32)
    _, ref_m, ref_l = orc.softmax_f32(rows, clen, want_p=False)
    live = clen > 0
    assert np.array_equal(got_m.reshape(-1)[live].view(np.uint32), ref_m[live].view(np.uint32)), "m_c"
    assert np.array_equal(got_l.reshape(-1)[live].view(np.uint32), ref_l[live].view(np.uint32)), "l_c"
    # chunks past the length are never written
    assert (wsf[:2 * n].view(np.uint32).reshape(2, -1)[:, ~live] == 0xFFFFFFFF).all()
    # combined m and L of the full rows
    R = B * Hq
    full = np.ascontiguousarray(s.reshape(R, Lmax))
    flen = np.repeat(lens.astype(np.int32), Hq)
    _, ref_M, ref_L = orc.softmax_f32(full, flen, want_p=False)
    p = torch.zeros((R, Lmax), dtype=torch.float32, device=DEV)
    m = torch.empty(R, dtype=torch.float32, device=DEV)
    l = torch.empty(R, dtype=torch.float32, device=DEV)
    d.det_softmax_f32(up(full), up(flen), p, m, l)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy().view(np.uint32), ref_M.view(np.uint32))
    assert np.array_equal(l.cpu().numpy().view(np.uint32), ref_L.view(np.uint32))
