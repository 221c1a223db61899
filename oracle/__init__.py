"""ctypes front end of the CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg; the product package never imports this.  Arrays are numpy: bf16 tensors travel
as uint16 bit patterns, fp32 as float32, fp64 as float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "oracle.c")

CFLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-mfma", "-mavx2", "-std=c11", "-shared", "-fPIC",
          "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    """Compile oracle.c into liboracle.so next to it."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _SO, "-lm"])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        _lib = C.CDLL(_SO)
        _lib.orc_bf16_to_f32.restype = C.c_float
        _lib.orc_bf16_to_f32.argtypes = [C.c_uint16]
        _lib.orc_bf16_rne.restype = C.c_uint16
        _lib.orc_bf16_rne.argtypes = [C.c_float]
        _lib.orc_bf16_from_f64.restype = C.c_uint16
        _lib.orc_bf16_from_f64.argtypes = [C.c_double]
        _lib.orc_expf.restype = C.c_float
        _lib.orc_expf.argtypes = [C.c_float]
        _lib.orc_tree256.restype = C.c_float
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_sumsq.restype = C.c_float
        _lib.orc_sample_uniform.restype = C.c_float
        _lib.orc_sample_uniform.argtypes = [C.c_uint64, C.c_int32, C.c_int32]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def bf16_rne(x) -> np.ndarray:
    x = _f32(x)
    y = np.empty(x.shape, dtype=np.uint16)
    lib().orc_bf16_rne_array(_p(x), _p(y), C.c_int64(x.size))
    return y


def bf16_from_f64(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    f = lib().orc_bf16_from_f64
    return np.array([f(float(v)) for v in x.reshape(-1)], dtype=np.uint16).reshape(x.shape)


def bf16_to_f32(b) -> np.ndarray:
    b = _u16(b)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def expf(x) -> np.ndarray:
    x = _f32(x)
    y = np.empty_like(x)
    lib().orc_expf_array(_p(x), _p(y), C.c_int64(x.size))
    return y


def tree256(leaves) -> np.float32:
    t = _f32(leaves)
    assert t.shape == (256,)
    return np.float32(lib().orc_tree256(_p(t)))


def sumsq(x) -> np.float32:
    x = _u16(x)
    assert x.ndim == 1
    return np.float32(lib().orc_sumsq(_p(x), C.c_int(x.size)))


def rmsnorm(x, w, eps: float) -> np.ndarray:
    x, w = _u16(x), _u16(w)
    M, H = x.shape
    assert w.shape == (H,)
    y = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(w), _p(y), C.c_int(M), C.c_int(H), C.c_float(eps))
    return y


def softmax_f32(s, lens, want_p: bool = True):
    """Returns (p, m, l).  p has zeros at and past lens[r]."""
    s, lens = _f32(s), _i32(lens)
    R, Lmax = s.shape
    p = np.zeros_like(s) if want_p else None
    m = np.empty(R, dtype=np.float32)
    l = np.empty(R, dtype=np.float32)
    lib().orc_softmax_f32(_p(s), _p(lens), _p(p) if want_p else None, _p(m), _p(l), C.c_int(R),
                          C.c_int(Lmax))
    return p, m, l


def argmax_f32(logits) -> np.ndarray:
    x = _f32(logits)
    B, V = x.shape
    idx = np.empty(B, dtype=np.int32)
    lib().orc_argmax_f32(_p(x), _p(idx), C.c_int(B), C.c_int(V))
    return idx


def argmax_bf16(logits) -> np.ndarray:
    x = _u16(logits)
    B, V = x.shape
    idx = np.empty(B, dtype=np.int32)
    lib().orc_argmax_bf16(_p(x), _p(idx), C.c_int(B), C.c_int(V))
    return idx


def gemm_f64(A, B, want_abs: bool = True):
    """A [M,K] bf16 bits, B [K,N] bf16 bits -> (C, Cabs) fp64."""
    A, B = _u16(A), _u16(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    Cm = np.empty((M, N), dtype=np.float64)
    Ca = np.empty((M, N), dtype=np.float64) if want_abs else None
    lib().orc_gemm_f64(_p(A), C.c_int(K), _p(B), _p(Cm), _p(Ca) if want_abs else None, C.c_int(M),
                       C.c_int(N), C.c_int(K))
    return Cm, Ca


def gemm_f64_sample(A, B, rows, cols):
    A, B = _u16(A), _u16(B)
    rows, cols = _i32(rows), _i32(cols)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2 and rows.shape == cols.shape
    assert rows.min() >= 0 and rows.max() < M and cols.min() >= 0 and cols.max() < N
    c = np.empty(rows.size, dtype=np.float64)
    ca = np.empty(rows.size, dtype=np.float64)
    lib().orc_gemm_f64_sample(_p(A), C.c_int(K), _p(B), _p(rows), _p(cols), _p(c), _p(ca),
                              C.c_int(rows.size), C.c_int(N), C.c_int(K))
    return c, ca


def attn_decode_f64(q, kcache, vcache, seqlens, scale: float):
    """q [B,Hq,D], caches [B,Hkv,Lmax,D] bf16 bits -> (out, outabs) fp64 [B,Hq,D]."""
    q, kcache, vcache, seqlens = _u16(q), _u16(kcache), _u16(vcache), _i32(seqlens)
    B, Hq, D = q.shape
    B2, Hkv, Lmax, D2 = kcache.shape
    assert B == B2 and D == D2 and vcache.shape == kcache.shape and Hq % Hkv == 0
    assert seqlens.shape == (B,) and seqlens.max(initial=0) <= Lmax
    out = np.empty((B, Hq, D), dtype=np.float64)
    oa = np.empty((B, Hq, D), dtype=np.float64)
    lib().orc_attn_decode_f64(_p(q), _p(kcache), _p(vcache), _p(seqlens), _p(out), _p(oa), C.c_int(B),
                              C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(Lmax), C.c_float(scale))
    return out, oa


def rope(x, pos, cos_t, sin_t) -> np.ndarray:
    """x [R,nh,D] bf16 bits, pos [R] -> rotated, same shape."""
    x, pos, cos_t, sin_t = _u16(x), _i32(pos), _f32(cos_t), _f32(sin_t)
    R, nh, D = x.shape
    assert cos_t.shape == sin_t.shape and cos_t.shape[1] == D // 2 and pos.max() < cos_t.shape[0]
    y = np.empty_like(x)
    lib().orc_rope(_p(x), _p(y), _p(pos), _p(cos_t), _p(sin_t), C.c_int(R), C.c_int(nh), C.c_int(D))
    return y


def swiglu(g, u) -> np.ndarray:
    g, u = _u16(g), _u16(u)
    assert g.shape == u.shape
    y = np.empty_like(g)
    lib().orc_swiglu(_p(g), _p(u), _p(y), C.c_int64(g.size))
    return y


def residual(x, y) -> np.ndarray:
    x, y = _u16(x), _u16(y)
    assert x.shape == y.shape
    z = np.empty_like(x)
    lib().orc_residual(_p(x), _p(y), _p(z), C.c_int64(x.size))
    return z


def decoder_layer(x, w, kcache, vcache, positions, cos_t, sin_t, cfg):
    """One decoder layer.  `w` is a dict of logical [K,N] bf16-bit weights: norm1, wqkv, wo, norm2,
    wgu, wdown.  `cfg` is a dict with H, Hq, Hkv, D, F, Lmax, eps, scale.  Returns the new x; the
    caches are updated in place."""
    x = _u16(x).copy()
    B, H = x.shape
    assert kcache.dtype == np.uint16 and kcache.flags.c_contiguous
    assert vcache.dtype == np.uint16 and vcache.flags.c_contiguous
    positions, cos_t, sin_t = _i32(positions), _f32(cos_t), _f32(sin_t)
    Hq, Hkv, D, F, Lmax = cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["F"], cfg["Lmax"]
    assert H == cfg["H"] and kcache.shape == (B, Hkv, Lmax, D) and vcache.shape == kcache.shape
    assert w["wqkv"].shape == (H, (Hq + 2 * Hkv) * D) and w["wo"].shape == (Hq * D, H)
    assert w["wgu"].shape == (H, 2 * F) and w["wdown"].shape == (F, H)
    assert positions.max() < Lmax and cos_t.shape == (Lmax, D // 2)
    lib().orc_decoder_layer(_p(x), _p(_u16(w["norm1"])), _p(_u16(w["wqkv"])), _p(_u16(w["wo"])),
                            _p(_u16(w["norm2"])), _p(_u16(w["wgu"])), _p(_u16(w["wdown"])),
                            _p(kcache), _p(vcache), _p(positions), _p(cos_t), _p(sin_t), C.c_int(B),
                            C.c_int(H), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(F),
                            C.c_int(Lmax), C.c_float(cfg["eps"]), C.c_float(cfg["scale"]))
    return x


def sample_uniform(seed: int, seq_id: int, step: int) -> np.float32:
    return np.float32(lib().orc_sample_uniform(C.c_uint64(seed & (2 ** 64 - 1)), int(seq_id), int(step)))


def sample(logits, temperature: float, top_k: int, top_p: float, seed: int, seq_ids, steps) -> np.ndarray:
    """Seeded temperature / top-k / top-p sampling; logits [B,V] fp32 -> tokens [B] int32."""
    x, seq_ids, steps = _f32(logits), _i32(seq_ids), _i32(steps)
    B, V = x.shape
    assert seq_ids.shape == (B,) and steps.shape == (B,) and top_k >= 1 and temperature > 0 and 0 < top_p <= 1
    out = np.empty(B, dtype=np.int32)
    lib().orc_sample(_p(x), C.c_int(B), C.c_int(V), C.c_float(temperature), C.c_int(top_k), C.c_float(top_p),
                     C.c_uint64(seed & (2 ** 64 - 1)), _p(seq_ids), _p(steps), _p(out))
    return out


def quant_w4(w_bits) -> tuple[np.ndarray, np.ndarray]:
    """Weight quantizer: W bf16 bits [K,N] -> (q int8 [K,N] in -8..7, s bf16 bits [K/64,N])."""
    w = _u16(w_bits)
    K, N = w.shape
    assert K % 64 == 0
    q = np.empty((K, N), dtype=np.int8)
    s = np.empty((K // 64, N), dtype=np.uint16)
    lib().orc_quant_w4(_p(w), C.c_int(K), C.c_int(N), _p(q), _p(s))
    return q, s


def quant_a8(a_bits) -> tuple[np.ndarray, np.ndarray]:
    """Activation quantizer: A bf16 bits [M,K] -> (p int8 [M,K] in -127..127, d fp32 [M,K/64])."""
    a = _u16(a_bits)
    M, K = a.shape
    assert K % 64 == 0
    p = np.empty((M, K), dtype=np.int8)
    d = np.empty((M, K // 64), dtype=np.float32)
    lib().orc_quant_a8(_p(a), C.c_int(K), C.c_int(M), C.c_int(K), _p(p), _p(d))
    return p, d


def qgemm_w4a8(p, d, q, s) -> tuple[np.ndarray, np.ndarray]:
    """Quantized GEMM on quantized operands -> (acc fp32 [M,N], C bf16 bits [M,N]), bit-exact reference."""
    p = np.ascontiguousarray(p, dtype=np.int8)
    q = np.ascontiguousarray(q, dtype=np.int8)
    d, s = _f32(d), _u16(s)
    M, K = p.shape
    N = q.shape[1]
    assert q.shape == (K, N) and d.shape == (M, K // 64) and s.shape == (K // 64, N)
    acc = np.empty((M, N), dtype=np.float32)
    c = np.empty((M, N), dtype=np.uint16)
    lib().orc_qgemm_w4a8(_p(p), _p(d), _p(q), _p(s), C.c_int(M), C.c_int(N), C.c_int(K), _p(acc), _p(c))
    return acc, c


def qlinear(a_bits, q, s) -> np.ndarray:
    """bf16 activations through a quantized projection: quantize the rows (quant_a8), contract with the
    weight codes and scales (qgemm_w4a8), return the bf16 bits of the result."""
    p, d = quant_a8(a_bits)
    return qgemm_w4a8(p, d, q, s)[1]


def qdecoder_layer(x, w, kcache, vcache, positions, cos_t, sin_t, cfg, intermediates=None):
    """One decoder layer with every projection block-quantized: the steps of decoder_layer in the same
    order, each projection replaced by qlinear on the bf16 activations it would have taken.  `w` holds
    norm1, norm2 (bf16 bits) and wqkv, wo, wgu, wdown as (codes int8 [K,N], scales bf16 bits [K/64,N])
    pairs from quant_w4 of the logical weights (wgu columns: F gate then F up).  Attention is the fp64
    reference rounded once to bf16.  Returns the new x; the caches are updated in place.  `intermediates`, if
    a dict, receives the branch values o, x1, dn (for the element-wise bound of oracle.model.layer_bound)."""
    x = _u16(x).copy()
    B, H = x.shape
    positions, cos_t, sin_t = _i32(positions), _f32(cos_t), _f32(sin_t)
    Hq, Hkv, D, F, Lmax = cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["F"], cfg["Lmax"]
    assert kcache.dtype == np.uint16 and kcache.flags.c_contiguous and kcache.shape == (B, Hkv, Lmax, D)
    assert vcache.dtype == np.uint16 and vcache.flags.c_contiguous and vcache.shape == kcache.shape
    h = rmsnorm(x, w["norm1"], cfg["eps"])
    qkv = qlinear(h, *w["wqkv"])
    q_rot = rope(np.ascontiguousarray(qkv[:, :Hq * D]).reshape(B, Hq, D), positions, cos_t, sin_t)
    k_rot = rope(np.ascontiguousarray(qkv[:, Hq * D:(Hq + Hkv) * D]).reshape(B, Hkv, D), positions, cos_t, sin_t)
    v_new = qkv[:, (Hq + Hkv) * D:].reshape(B, Hkv, D)
    for b in range(B):
        kcache[b, :, positions[b]] = k_rot[b]
        vcache[b, :, positions[b]] = v_new[b]
    att, _ = attn_decode_f64(q_rot, kcache, vcache, positions + 1, cfg["scale"])
    att = bf16_from_f64(att).reshape(B, Hq * D)
    o = qlinear(att, *w["wo"])
    x = residual(x, o)
    h = rmsnorm(x, w["norm2"], cfg["eps"])
    gu = qlinear(h, *w["wgu"])
    mm = swiglu(np.ascontiguousarray(gu[:, :F]), np.ascontiguousarray(gu[:, F:]))
    dn = qlinear(mm, *w["wdown"])
    if intermediates is not None:
        intermediates.update(o=o, x1=x, dn=dn)
    return residual(x, dn)


def commit_sha256(prompt: bytes, logits: bytes, tokens: bytes) -> bytes:
    """The digest the paper records per execution (section 6.7): SHA-256 of the three byte strings
    concatenated in that order.  The hash itself is the standard library's (a library primitive as a
    step); pinned by the FIPS 180-4 example digests in tests/golden/."""
    import hashlib
    return hashlib.sha256(bytes(prompt) + bytes(logits) + bytes(tokens)).digest()
