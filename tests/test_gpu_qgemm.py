"""Block-quantized GEMM on the GPU against the bit-exact oracle: the two quantizers code for code,
the product byte for byte (bf16 and fp32 outputs), row-byte invariance over M = 1..256 and over the
content of the other rows, and repeatability."""
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


def gpu_quant_w(d, w_bits):
    K, N = w_bits.shape
    packed = d.quant_pack_weight(up_bf16(w_bits))
    q = torch.empty((K, N), dtype=torch.int8, device=DEV)
    s = torch.empty((K // 64, N), dtype=torch.bfloat16, device=DEV)
    d.det_quant_unpack_w4(packed, q, s)
    torch.cuda.synchronize()
    return packed, q.cpu().numpy(), down_bf16(s)


def gpu_quant_a(d, a_bits):
    M, K = a_bits.shape
    codes, scales = d.quant_activations(up_bf16(a_bits))
    torch.cuda.synchronize()
    ldd = (M + 3) & ~3
    return codes, scales, codes.cpu().numpy(), scales.cpu().numpy().reshape(K // 64, ldd)[:, :M].T.copy()


@pytest.mark.parametrize("K,N", [(256, 64), (512, 4096), (1024, 6144), (4096, 2048), (192, 28672)])
def test_weight_quantizer_matches_oracle(d, orc, K, N):
    w = ds.normal_bf16(ds.tensor_seed(6, 10) + K + N, (K, N), 0.02, 0.0)
    w[5, :] = 0x8000 | (w[5, :] & 0x7FFF)        # some structure: a negative row, a zero block, a big value
    w[64:128, 3] = 0
    w[130, 7] = 0x4040                         # 3.0
    step(f"weight quantizer K={K} N={N}")
    _, q, s = gpu_quant_w(d, w)
    qo, so = orc.quant_w4(w)
    assert np.array_equal(s, so) and np.array_equal(q, qo)


@pytest.mark.parametrize("M,K", [(1, 64), (3, 4096), (17, 1024), (256, 4096), (130, 14336)])
def test_activation_quantizer_matches_oracle(d, orc, M, K):
    a = ds.normal_bf16(ds.tensor_seed(6, 20) + M + K, (M, K), 1.0, 0.0)
    a[0, :64] = 0
    step(f"activation quantizer M={M} K={K}")
    _, _, p, dd = gpu_quant_a(d, a)
    po, do = orc.quant_a8(a)
    assert np.array_equal(dd.view(np.uint32), do.view(np.uint32)) and np.array_equal(p, po)


@pytest.mark.parametrize("M,K,N", [
    (1, 64, 16), (16, 512, 512), (5, 1024, 4096), (33, 2048, 6144), (64, 512, 28672), (200, 1024, 3072),
    (256, 4096, 4096), (256, 1024, 28672), (300, 512, 2048), (7, 14336, 256), (128, 2048, 32000),
    (257, 256, 4096), (260, 512, 6144), (8, 4096, 6144), (4, 2048, 3072), (2, 14336, 4096),
    (8, 128, 32), (5, 192, 6144), (3, 64, 4096), (9, 2048, 4096), (16, 14336, 4096), (48, 1024, 6144),
    (64, 5632, 2048), (40, 512, 1024), (130, 256, 2048), (33, 2048, 3072),
])
def test_qgemm_bytes_match_oracle(d, orc, M, K, N):
    a = ds.normal_bf16(ds.tensor_seed(6, 30) + M, (M, K), 1.0, 0.0)
    w = ds.normal_bf16(ds.tensor_seed(6, 31) + N, (K, N), 0.02, 0.0)
    step(f"qgemm M={M} K={K} N={N}")
    packed, _, _ = gpu_quant_w(d, w)
    codes, scales, _, _ = gpu_quant_a(d, a)
    c = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    cf = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    d.det_qgemm_w4a8(codes, scales, packed, c, N)
    d.det_qgemm_w4a8(codes, scales, packed, cf, N)
    torch.cuda.synchronize()
    p, dd = orc.quant_a8(a)
    q, s = orc.quant_w4(w)
    acc, cb = orc.qgemm_w4a8(p, dd, q, s)
    assert np.array_equal(cf.cpu().numpy().view(np.uint32), acc.view(np.uint32))
    assert np.array_equal(down_bf16(c), cb)


def test_qgemm_batch_invariance_and_repeats(d):
    K, N = 4096, 6144
    a = ds.normal_bf16(ds.tensor_seed(6, 40), (256, K), 1.0, 0.0)
    w = ds.normal_bf16(ds.tensor_seed(6, 41), (K, N), 0.02, 0.0)
    packed = d.quant_pack_weight(up_bf16(w))

    def run(rows_bits):
        M = rows_bits.shape[0]
        codes, scales = d.quant_activations(up_bf16(rows_bits))
        c = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
        d.det_qgemm_w4a8(codes, scales, packed, c, N)
        torch.cuda.synchronize()
        return down_bf16(c)

    step("qgemm M=256 reference")
    full = run(a)
    for M in (1, 2, 3, 8, 15, 16, 17, 64, 100, 128, 255):
        step(f"qgemm rows 0..{M - 1} alone")
        assert np.array_equal(run(a[:M]), full[:M]), M
    step("qgemm with other rows replaced and slots permuted")
    other = ds.normal_bf16(ds.tensor_seed(6, 42), (256, K), 3.0, 0.0)
    mixed = other.copy()
    mixed[[200, 7, 31]] = a[[0, 1, 2]]
    got = run(mixed)
    assert np.array_equal(got[[200, 7, 31]], full[[0, 1, 2]])
    step("qgemm 20 repeats")
    for _ in range(20):
        assert np.array_equal(run(a), full)


def test_qgemm_argument_errors(d):
    from paper_2602_00182_amd._lib import lib
    L = lib()
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    p = buf.data_ptr()
    assert L.det_qgemm_packed_w_bytes(100, 64) == 0 and L.det_qgemm_packed_w_bytes(64, 100) == 0   # N % 16, K % 64
    assert L.det_qgemm_packed_w_bytes(64, 128) == 4 * 2 * 544
    assert L.det_quant_pack_w4(p, p, 100, 64, None) == 2                       # DET_ESHAPE
    assert L.det_quant_pack_w4(None, p, 64, 64, None) == 1                     # DET_EINVAL
    assert L.det_quant_pack_w4(p, p + 4, 64, 64, None) == 3                    # DET_EALIGN
    assert L.det_quant_act_q8(p, 32, p, p, 1, 64, None) == 1                   # lda < K
    assert L.det_quant_act_q8(p, 64, p, p, 1, 96, None) == 2
    assert L.det_qgemm_w4a8(p, p, p, p, 60, 1, 64, 64, 0, None) == 1           # ldc < N
    assert L.det_qgemm_w4a8(p, p, p, p, 64, 1, 64, 64, 7, None) == 1           # out_dtype
    assert L.det_qgemm_w4a8(p, p, p, p, 64, 0, 64, 64, 0, None) == 1           # M < 1
    assert L.det_qgemm_w4a8(p, p, p, p, 66, 1, 64, 64, 0, None) == 3           # ldc % 4
    torch.cuda.synchronize()


@pytest.mark.parametrize("M,H", [(1, 4096), (5, 2048), (33, 64), (64, 16384), (130, 4096)])
def test_rmsnorm_quant_matches_oracle(d, orc, M, H):
    """det_rmsnorm_quant_q8 = the oracle's activation quantizer applied to the oracle's RMSNorm, code for
    code and scale bit for bit (and so equal to det_quant_act_q8 of det_rmsnorm)."""
    x = ds.normal_bf16(ds.tensor_seed(6, 50) + M, (M, H), 1.0, 0.0)
    w = ds.normal_bf16(ds.tensor_seed(6, 51) + H, (H,), 0.1, 1.0)
    x[0, :64] = 0                                  # a block of zeros: scale 0, codes 0
    step(f"rmsnorm+quant M={M} H={H}")
    codes = torch.full((M, H), 99, dtype=torch.int8, device=DEV)
    scales = torch.full((d.det_quant_act_scales_bytes(M, H) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    d.det_rmsnorm_quant_q8(up_bf16(x), up_bf16(w), codes, scales, 1e-5)
    torch.cuda.synchronize()
    ldd = (M + 3) & ~3
    got_d = scales.cpu().numpy().reshape(H // 64, ldd)[:, :M].T
    po, do = orc.quant_a8(orc.rmsnorm(x, w, 1e-5))
    assert np.array_equal(codes.cpu().numpy(), po)
    assert np.array_equal(np.ascontiguousarray(got_d).view(np.uint32), do.view(np.uint32))


@pytest.mark.parametrize("M,K,N", [(1, 256, 4096), (19, 1024, 6144), (70, 512, 12288), (130, 512, 28672),
                                   (300, 256, 2048)])
def test_qgemm_residual_epilogue_matches_oracle(d, orc, M, K, N):
    a = ds.normal_bf16(ds.tensor_seed(6, 60) + M, (M, K), 1.0, 0.0)
    w = ds.normal_bf16(ds.tensor_seed(6, 61) + N, (K, N), 0.02, 0.0)
    r = ds.normal_bf16(ds.tensor_seed(6, 62) + M, (M, N), 1.0, 0.0)
    step(f"qgemm residual epilogue M={M} K={K} N={N}")
    packed = d.quant_pack_weight(up_bf16(w))
    codes, scales = d.quant_activations(up_bf16(a))
    rd = up_bf16(r)
    out = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    d.det_qgemm_w4a8_residual(codes, scales, packed, rd, out, N)
    inplace = rd.clone()
    d.det_qgemm_w4a8_residual(codes, scales, packed, inplace, inplace, N)
    torch.cuda.synchronize()
    want = orc.residual(r, orc.qlinear(a, *orc.quant_w4(w)))
    assert np.array_equal(down_bf16(out), want) and np.array_equal(down_bf16(inplace), want)


@pytest.mark.parametrize("M,K,F", [(1, 256, 2048), (19, 512, 14336), (70, 1024, 5632), (200, 256, 3072),
                                   (130, 256, 6144)])
def test_qgemm_swiglu_epilogue_matches_oracle(d, orc, M, K, F):
    a = ds.normal_bf16(ds.tensor_seed(6, 70) + M, (M, K), 1.0, 0.0)
    w = ds.normal_bf16(ds.tensor_seed(6, 71) + F, (K, 2 * F), 0.05, 0.0)
    step(f"qgemm swiglu epilogue M={M} K={K} F={F}")
    packed = d.quant_pack_gate_up(up_bf16(w))
    codes, scales = d.quant_activations(up_bf16(a))
    y = torch.empty((M, F), dtype=torch.bfloat16, device=DEV)
    d.det_qgemm_w4a8_swiglu(codes, scales, packed, y, F)
    torch.cuda.synchronize()
    gu = orc.qlinear(a, *orc.quant_w4(w))
    want = orc.swiglu(np.ascontiguousarray(gu[:, :F]), np.ascontiguousarray(gu[:, F:]))
    assert np.array_equal(down_bf16(y), want)


@pytest.mark.parametrize("M,K,F", [(1, 256, 14336), (19, 512, 14336), (70, 256, 16000 * 2 // 2), (200, 256, 12288), (300, 256, 14336)])
def test_qgemm_swiglu_quant_epilogue_matches_oracle(d, orc, M, K, F):
    """The SwiGLU epilogue that writes activation codes: the oracle's quantizer applied to the oracle's
    SwiGLU of the quantized projection, code for code and scale bit for bit."""
    assert d.det_qgemm_w4a8_swiglu_quant_supported(F, K)
    a = ds.normal_bf16(ds.tensor_seed(6, 80) + M, (M, K), 1.0, 0.0)
    w = ds.normal_bf16(ds.tensor_seed(6, 81) + F, (K, 2 * F), 0.05, 0.0)
    w[:, 64:128] = 0                                # an all-zero output block: scale 0, codes 0
    step(f"qgemm swiglu+quant epilogue M={M} K={K} F={F}")
    packed = d.quant_pack_gate_up(up_bf16(w))
    codes, scales = d.quant_activations(up_bf16(a))
    co = torch.full((M, F), 99, dtype=torch.int8, device=DEV)
    so = torch.full((d.det_quant_act_scales_bytes(M, F) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    d.det_qgemm_w4a8_swiglu_quant(codes, scales, packed, co, so, F)
    torch.cuda.synchronize()
    gu = orc.qlinear(a, *orc.quant_w4(w))
    mm = orc.swiglu(np.ascontiguousarray(gu[:, :F]), np.ascontiguousarray(gu[:, F:]))
    po, do = orc.quant_a8(mm)
    ldd = (M + 3) & ~3
    got_d = np.ascontiguousarray(so.cpu().numpy().reshape(F // 64, ldd)[:, :M].T)
    assert np.array_equal(co.cpu().numpy(), po) and np.array_equal(got_d.view(np.uint32), do.view(np.uint32))


def test_qgemm_swiglu_quant_unsupported_shapes(d):
    from paper_2602_00182_amd._lib import lib
    assert not d.det_qgemm_w4a8_swiglu_quant_supported(5632, 2048)      # 32-column tiles
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    p = buf.data_ptr()
    assert lib().det_qgemm_w4a8_swiglu_quant(p, p, p, p, p, 1, 5632, 2048, None) == 2
    assert lib().det_qgemm_w4a8_swiglu_quant(p, p, p, p, None, 1, 14336, 256, None) == 1


@pytest.mark.parametrize("M,Hq,Hkv,K,Lmax,use_slots", [(1, 32, 8, 4096, 64, False), (5, 4, 2, 256, 40, True),
                                                       (8, 16, 4, 2048, 96, True), (33, 8, 2, 1024, 96, True),
                                                       (300, 32, 8, 4096, 320, False), (130, 2, 1, 512, 130, True)])
def test_qgemm_rope_append_epilogue_equals_unfused_bytes(d, M, Hq, Hkv, K, Lmax, use_slots):
    """det_qgemm_w4a8_qkv_rope_append on the pair-interleaved packing = det_qgemm_w4a8 on the plain packing,
    then det_rope on the query and key heads and a copy of the key and value heads into the caches, byte for
    byte (the quantized GEMM itself is compared with the oracle above); other cache rows keep their bytes."""
    D = 128
    N = (Hq + 2 * Hkv) * D
    A = up_bf16(ds.normal_bf16(820 + M, (M, K)))
    W = up_bf16(ds.normal_bf16(821 + Hq, (K, N), 0.05))
    codes, scales = d.quant_activations(A)
    cos_h, sin_h = ds.rope_tables(Lmax, D, 5.0e5)
    cos_t, sin_t = torch.from_numpy(cos_h).to(DEV), torch.from_numpy(sin_h).to(DEV)
    rng = np.random.default_rng(822 + M)
    if use_slots:
        S = max(2, (M + Lmax - 1) // Lmax + 1)
        cells = rng.permutation(S * Lmax)[:M]
        slots_h, pos_h = (cells // Lmax).astype(np.int32), (cells % Lmax).astype(np.int32)
    else:
        S = M
        slots_h, pos_h = np.arange(M, dtype=np.int32), rng.integers(0, Lmax, M).astype(np.int32)
        pos_h[0] = -3  # clamped to 0
    pos = torch.from_numpy(pos_h).to(DEV)
    slots = torch.from_numpy(slots_h).to(DEV) if use_slots else None
    kc0 = up_bf16(ds.normal_bf16(823, (S, Hkv, Lmax, D)))
    vc0 = up_bf16(ds.normal_bf16(824, (S, Hkv, Lmax, D)))
    step(f"qgemm rope/append epilogue M={M} Hq={Hq} Hkv={Hkv} K={K}")
    qkv = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    d.det_qgemm_w4a8(codes, scales, d.quant_pack_weight(W), qkv, N)
    qk = qkv[:, :(Hq + Hkv) * D].contiguous().view(M, Hq + Hkv, D)
    qk_rot = torch.empty_like(qk)
    d.det_rope(qk, qk_rot, pos, cos_t, sin_t)
    torch.cuda.synchronize()
    pc = torch.from_numpy(np.clip(pos_h, 0, Lmax - 1).astype(np.int64)).to(DEV)
    sl = torch.from_numpy(slots_h.astype(np.int64)).to(DEV)
    k_ref, v_ref = kc0.clone(), vc0.clone()
    k_ref[sl, :, pc, :] = qk_rot[:, Hq:, :]
    v_ref[sl, :, pc, :] = qkv[:, (Hq + Hkv) * D:].view(M, Hkv, D)
    qbuf = torch.zeros((M, Hq, D), dtype=torch.bfloat16, device=DEV)
    kc, vc = kc0.clone(), vc0.clone()
    d.det_qgemm_w4a8_qkv_rope_append(codes, scales, d.quant_pack_qkv(W, Hq, Hkv, D), qbuf, kc, vc, pos, slots, cos_t, sin_t)
    torch.cuda.synchronize()
    assert torch.equal(qbuf.view(torch.int16), qk_rot[:, :Hq, :].contiguous().view(torch.int16))
    assert torch.equal(kc.view(torch.int16), k_ref.view(torch.int16))
    assert torch.equal(vc.view(torch.int16), v_ref.view(torch.int16))
