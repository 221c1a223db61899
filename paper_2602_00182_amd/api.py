"""Argument marshalling for libdetinfer.  One function per C entry point, same name.

Tensors must live on the GPU and be contiguous where the C call says so; nothing is copied or
converted here, and no arithmetic of the method happens in Python."""
from __future__ import annotations

import ctypes as C

import torch

from ._lib import LayerCfg, LayerWeights, Sha256Ctx, lib

__all__ = [
    "DetError", "det_gemm_bf16", "det_gemm_bf16_fixed_tile", "det_probe_lds_fill", "det_gemm_packed_b_bytes", "det_gemm_pack_b", "det_gemm_bf16_residual",
    "det_gemm_pack_gate_up", "det_gemm_swiglu_bf16", "pack_gate_up", "det_gemm_pack_qkv", "pack_qkv",
    "det_gemm_qkv_rope_append", "det_rmsnorm_gemm_qkv_rope_append", "det_rmsnorm_gemm_swiglu_bf16", "det_rmsnorm_gemm_bf16", "det_rmsnorm",
    "det_attn_decode_workspace_bytes", "det_attn_decode", "det_attn_decode_static", "det_attn_decode_rows", "det_decoder_layer_rows",
    "det_softmax_f32", "det_argmax", "det_sample", "det_rope",
    "det_swiglu", "det_residual_add", "det_embed_gather", "det_decoder_layer_workspace_bytes",
    "det_decoder_layer", "det_next_token", "det_decode_advance", "det_fingerprint", "det_last_hip_error", "layer_cfg",
    "layer_weights", "pack_weight", "det_sha256_init", "det_sha256_update", "det_sha256_final",
    "det_commit_sha256", "det_sha256_force_portable", "det_qgemm_packed_w_bytes", "det_quant_pack_w4",
    "det_quant_unpack_w4", "det_quant_act_codes_bytes", "det_quant_act_scales_bytes", "det_quant_act_q8",
    "det_qgemm_w4a8", "quant_pack_weight", "quant_pack_qkv", "det_quant_pack_w4_qkv", "det_qgemm_w4a8_qkv_rope_append", "quant_activations", "det_qgemm_w4a8_residual",
    "det_qgemm_w4a8_swiglu", "det_quant_pack_w4_gate_up", "quant_pack_gate_up", "det_rmsnorm_quant_q8",
    "det_qdecoder_layer_workspace_bytes", "det_qdecoder_layer", "det_attn_decode_quant_q8",
    "det_qgemm_w4a8_swiglu_quant_supported", "det_qgemm_w4a8_swiglu_quant",
]

_CODES = {1: "DET_EINVAL", 2: "DET_ESHAPE", 3: "DET_EALIGN", 4: "DET_EWORKSPACE", 5: "DET_EHIP"}
DET_BF16, DET_F32 = 0, 1


class DetError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        extra = f" (hipError {lib().det_last_hip_error()})" if code == 5 else ""
        super().__init__(f"{fn} failed: {_CODES.get(code, code)}{extra}")


def _check(fn: str, code: int) -> None:
    if code != 0:
        raise DetError(fn, code)


def _ptr(t: torch.Tensor, dtype=None) -> int:
    if not t.is_cuda:
        raise ValueError("libdetinfer takes device tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _contig(t: torch.Tensor, dtype=None) -> int:
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return _ptr(t, dtype)


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def det_qgemm_packed_w_bytes(N: int, K: int) -> int:
    return lib().det_qgemm_packed_w_bytes(N, K)


def det_quant_pack_w4(b_kn, packed, stream=None) -> None:
    K, N = b_kn.shape
    if packed.numel() * packed.element_size() < det_qgemm_packed_w_bytes(N, K):
        raise ValueError("packed buffer too small")
    _check("det_quant_pack_w4", lib().det_quant_pack_w4(_contig(b_kn, torch.bfloat16), _contig(packed), N, K,
                                                          _stream(stream)))


def det_quant_unpack_w4(packed, codes, scales, stream=None) -> None:
    K, N = codes.shape
    if scales.shape != (K // 64, N):
        raise ValueError("bad shapes")
    _check("det_quant_unpack_w4", lib().det_quant_unpack_w4(_contig(packed), _contig(codes, torch.int8),
                                                              _contig(scales, torch.bfloat16), N, K, _stream(stream)))


def det_quant_act_codes_bytes(M: int, K: int) -> int:
    return lib().det_quant_act_codes_bytes(M, K)


def det_quant_act_scales_bytes(M: int, K: int) -> int:
    return lib().det_quant_act_scales_bytes(M, K)


def det_quant_act_q8(a, codes, scales, stream=None) -> None:
    M, K = a.shape
    if a.stride(1) != 1 or codes.shape != (M, K) or scales.numel() * 4 < det_quant_act_scales_bytes(M, K):
        raise ValueError("bad shapes")
    _check("det_quant_act_q8", lib().det_quant_act_q8(_ptr(a, torch.bfloat16), a.stride(0), _contig(codes, torch.int8),
                                                        _contig(scales, torch.float32), M, K, _stream(stream)))


def det_qgemm_w4a8(codes, scales, packed_w, c, N: int, stream=None) -> None:
    M, K = codes.shape
    if c.shape != (M, N) or c.stride(1) != 1:
        raise ValueError("bad output shape")
    out_dtype = {torch.bfloat16: DET_BF16, torch.float32: DET_F32}[c.dtype]
    _check("det_qgemm_w4a8", lib().det_qgemm_w4a8(_contig(codes, torch.int8), _contig(scales, torch.float32),
                                                    _contig(packed_w), _ptr(c), c.stride(0), M, N, K, out_dtype,
                                                    _stream(stream)))


def det_qgemm_w4a8_residual(codes, scales, packed_w, r, c, N: int, stream=None) -> None:
    """c = bf16(fp32(bf16(qgemm)) + fp32(r)); c may be r."""
    M, K = codes.shape
    if c.shape != (M, N) or r.shape != (M, N) or c.stride(1) != 1 or r.stride(1) != 1:
        raise ValueError("bad output shape")
    _check("det_qgemm_w4a8_residual", lib().det_qgemm_w4a8_residual(
        _contig(codes, torch.int8), _contig(scales, torch.float32), _contig(packed_w), _ptr(r, torch.bfloat16),
        _ld(r, N), _ptr(c, torch.bfloat16), _ld(c, N), M, N, K, _stream(stream)))


def det_qgemm_w4a8_swiglu(codes, scales, packed_gate_up, y, F: int, stream=None) -> None:
    M, K = codes.shape
    if y.shape != (M, F) or y.stride(1) != 1:
        raise ValueError("bad output shape")
    _check("det_qgemm_w4a8_swiglu", lib().det_qgemm_w4a8_swiglu(
        _contig(codes, torch.int8), _contig(scales, torch.float32), _contig(packed_gate_up),
        _ptr(y, torch.bfloat16), _ld(y, F), M, F, K, _stream(stream)))


def det_qgemm_w4a8_swiglu_quant_supported(F: int, K: int) -> bool:
    return bool(lib().det_qgemm_w4a8_swiglu_quant_supported(F, K))


def det_qgemm_w4a8_swiglu_quant(codes, scales, packed_gate_up, codes_out, scales_out, F: int, stream=None) -> None:
    M, K = codes.shape
    if codes_out.shape != (M, F) or scales_out.numel() * 4 < det_quant_act_scales_bytes(M, F):
        raise ValueError("bad output shape")
    _check("det_qgemm_w4a8_swiglu_quant", lib().det_qgemm_w4a8_swiglu_quant(
        _contig(codes, torch.int8), _contig(scales, torch.float32), _contig(packed_gate_up),
        _contig(codes_out, torch.int8), _contig(scales_out, torch.float32), M, F, K, _stream(stream)))


def det_quant_pack_w4_gate_up(b_kn, packed, stream=None) -> None:
    K, N2 = b_kn.shape
    _check("det_quant_pack_w4_gate_up", lib().det_quant_pack_w4_gate_up(
        _contig(b_kn, torch.bfloat16), _contig(packed), N2 // 2, K, _stream(stream)))


def quant_pack_gate_up(b_kn: torch.Tensor) -> torch.Tensor:
    """Allocates and fills the packed 4-bit form of a [K, 2F] (gate | up) weight for det_qgemm_w4a8_swiglu."""
    K, N2 = b_kn.shape
    packed = torch.empty(det_qgemm_packed_w_bytes(N2, K), dtype=torch.uint8, device=b_kn.device)
    det_quant_pack_w4_gate_up(b_kn.contiguous(), packed)
    return packed


def det_rmsnorm_quant_q8(x, w, codes, scales, eps: float, stream=None) -> None:
    M, H = x.shape
    if w.shape != (H,) or codes.shape != (M, H) or scales.numel() * 4 < det_quant_act_scales_bytes(M, H):
        raise ValueError("bad RMSNorm/quantizer shapes")
    _check("det_rmsnorm_quant_q8", lib().det_rmsnorm_quant_q8(
        _contig(x, torch.bfloat16), _contig(w, torch.bfloat16), _contig(codes, torch.int8),
        _contig(scales, torch.float32), M, H, eps, _stream(stream)))


def det_attn_decode_quant_q8(q, kcache, vcache, seqlens, slots, codes, scales, ws, scale: float, stream=None) -> None:
    """Attention output [R, Hq*D] written as activation codes and scales; slots may be None."""
    R, Hq, D = q.shape
    _, Hkv, Lmax, D2 = kcache.shape
    if D2 != D or vcache.shape != kcache.shape or seqlens.shape != (R,) or codes.shape != (R, Hq * D):
        raise ValueError("bad attention shapes")
    if scales.numel() * 4 < det_quant_act_scales_bytes(R, Hq * D) or (slots is None and kcache.shape[0] < R):
        raise ValueError("bad attention shapes")
    _check("det_attn_decode_quant_q8", lib().det_attn_decode_quant_q8(
        _contig(q, torch.bfloat16), _contig(kcache, torch.bfloat16), _contig(vcache, torch.bfloat16),
        _contig(seqlens, torch.int32), None if slots is None else _contig(slots, torch.int32),
        _contig(codes, torch.int8), _contig(scales, torch.float32), _contig(ws), ws.numel() * ws.element_size(),
        R, Hq, Hkv, D, Lmax, scale, _stream(stream)))


def quant_pack_weight(b_kn: torch.Tensor) -> torch.Tensor:
    """Allocates the packed 4-bit matrix for a bf16 weight [K,N] and fills it (det_quant_pack_w4)."""
    K, N = b_kn.shape
    packed = torch.empty(det_qgemm_packed_w_bytes(N, K), dtype=torch.uint8, device=b_kn.device)
    det_quant_pack_w4(b_kn.contiguous(), packed)
    return packed


def det_quant_pack_w4_qkv(b_kn: torch.Tensor, packed: torch.Tensor, Hq: int, Hkv: int, D: int = 128, stream=None) -> None:
    K, N = b_kn.shape
    if N != (Hq + 2 * Hkv) * D or packed.numel() * packed.element_size() < det_qgemm_packed_w_bytes(N, K):
        raise ValueError("bad fused query/key/value weight")
    _check("det_quant_pack_w4_qkv", lib().det_quant_pack_w4_qkv(_contig(b_kn, torch.bfloat16), _contig(packed), Hq, Hkv, D, K,
                                                                 _stream(stream)))


def quant_pack_qkv(b_kn: torch.Tensor, Hq: int, Hkv: int, D: int = 128, stream=None) -> torch.Tensor:
    """Allocates and fills the packed 4-bit form of a [K, (Hq+2Hkv)D] weight for det_qgemm_w4a8_qkv_rope_append
    (the form det_qdecoder_layer takes as wqkv)."""
    K, N = b_kn.shape
    packed = torch.empty(det_qgemm_packed_w_bytes(N, K), dtype=torch.uint8, device=b_kn.device)
    det_quant_pack_w4_qkv(b_kn, packed, Hq, Hkv, D, stream)
    return packed


def det_qgemm_w4a8_qkv_rope_append(codes, scales, packed_qkv, qbuf, kcache, vcache, positions, slots, rope_cos, rope_sin,
                                   stream=None) -> None:
    """The quantized layer's fused projection (see det_gemm_qkv_rope_append); weight from quant_pack_qkv."""
    M, K = codes.shape
    _, Hq, D = qbuf.shape
    _, Hkv, Lmax, _ = kcache.shape
    if qbuf.shape[0] != M or vcache.shape != kcache.shape or positions.numel() != M:
        raise ValueError("bad fused projection operands")
    if slots is not None and slots.numel() != M:
        raise ValueError("bad slots")
    if rope_cos.shape != (Lmax, D // 2) or rope_sin.shape != (Lmax, D // 2):
        raise ValueError("bad rope tables")
    _check("det_qgemm_w4a8_qkv_rope_append", lib().det_qgemm_w4a8_qkv_rope_append(
        _contig(codes, torch.int8), _contig(scales, torch.float32), _contig(packed_qkv), _contig(qbuf, torch.bfloat16),
        _contig(kcache, torch.bfloat16), _contig(vcache, torch.bfloat16), _contig(positions, torch.int32),
        None if slots is None else _contig(slots, torch.int32), _contig(rope_cos, torch.float32),
        _contig(rope_sin, torch.float32), M, Hq, Hkv, D, Lmax, K, _stream(stream)))


def quant_activations(a: torch.Tensor):
    """Allocates codes and scales for a bf16 activation matrix [M,K] and fills them (det_quant_act_q8)."""
    M, K = a.shape
    codes = torch.empty((M, K), dtype=torch.int8, device=a.device)
    scales = torch.empty(det_quant_act_scales_bytes(M, K) // 4, dtype=torch.float32, device=a.device)
    det_quant_act_q8(a, codes, scales)
    return codes, scales


def _host_bytes(data):
    """(address, length, keep-alive) of a host byte string: bytes, bytearray, numpy array or CPU tensor."""
    if data is None:
        return None, 0, None
    if isinstance(data, torch.Tensor):
        if data.is_cuda or not data.is_contiguous():
            raise ValueError("the commitment hashes contiguous host memory")
        return data.data_ptr(), data.numel() * data.element_size(), data
    mv = memoryview(data)
    if not mv.contiguous:
        raise ValueError("the commitment hashes contiguous host memory")
    if mv.nbytes == 0:
        return None, 0, None
    buf = (C.c_char * mv.nbytes).from_buffer_copy(mv) if mv.readonly else (C.c_char * mv.nbytes).from_buffer(mv)
    return C.addressof(buf), mv.nbytes, buf


def det_sha256_init() -> Sha256Ctx:
    ctx = Sha256Ctx()
    _check("det_sha256_init", lib().det_sha256_init(C.byref(ctx)))
    return ctx


def det_sha256_update(ctx: Sha256Ctx, data) -> None:
    addr, n, keep = _host_bytes(data)
    _check("det_sha256_update", lib().det_sha256_update(C.byref(ctx), addr, n))
    del keep


def det_sha256_final(ctx: Sha256Ctx) -> bytes:
    out = (C.c_uint8 * 32)()
    _check("det_sha256_final", lib().det_sha256_final(C.byref(ctx), out))
    return bytes(out)


def det_commit_sha256(prompt, logits, tokens) -> bytes:
    """SHA256(prompt || logits || tokens) over host byte strings (None or empty: nothing hashed for that part)."""
    pa, pn, k1 = _host_bytes(prompt)
    la, ln, k2 = _host_bytes(logits)
    ta, tn, k3 = _host_bytes(tokens)
    out = (C.c_uint8 * 32)()
    _check("det_commit_sha256", lib().det_commit_sha256(pa, pn, la, ln, ta, tn, out))
    del k1, k2, k3
    return bytes(out)


def det_sha256_force_portable(on: bool) -> None:
    _check("det_sha256_force_portable", lib().det_sha256_force_portable(int(bool(on))))


def det_fingerprint() -> str:
    return lib().det_fingerprint().decode()


def det_last_hip_error() -> int:
    return lib().det_last_hip_error()


def det_gemm_packed_b_bytes(N: int, K: int) -> int:
    return lib().det_gemm_packed_b_bytes(N, K)


def det_gemm_pack_b(B_kn: torch.Tensor, B_packed: torch.Tensor, stream=None) -> None:
    K, N = B_kn.shape
    if B_packed.numel() * B_packed.element_size() < 2 * N * K:
        raise ValueError("B_packed too small")
    _check("det_gemm_pack_b", lib().det_gemm_pack_b(_contig(B_kn, torch.bfloat16), _contig(B_packed), N, K,
                                                     _stream(stream)))


def pack_weight(B_kn: torch.Tensor, stream=None) -> torch.Tensor:
    """Allocates the packed buffer for a [K, N] bf16 weight and fills it with det_gemm_pack_b."""
    K, N = B_kn.shape
    nbytes = det_gemm_packed_b_bytes(N, K)
    if nbytes == 0:
        raise DetError("det_gemm_packed_b_bytes", 2)
    out = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=B_kn.device)
    det_gemm_pack_b(B_kn, out, stream)
    return out


def det_gemm_bf16(A: torch.Tensor, B_packed: torch.Tensor, C_out: torch.Tensor, N: int, K: int,
                  stream=None, _entry: str = "det_gemm_bf16") -> None:
    """C_out[M, N] = A[M, K] @ B.  A and C_out may be row-strided views (stride(1) == 1)."""
    M = A.shape[0]
    if A.shape[1] != K or C_out.shape != (M, N) or A.stride(1) != 1 or C_out.stride(1) != 1:
        raise ValueError("bad GEMM operand shapes")
    if B_packed.numel() * B_packed.element_size() < 2 * N * K:
        raise ValueError("B_packed too small")
    if C_out.dtype == torch.bfloat16:
        od = DET_BF16
    elif C_out.dtype == torch.float32:
        od = DET_F32
    else:
        raise TypeError("C must be bf16 or fp32")
    lda = A.stride(0) if M > 1 else max(A.stride(0), K)
    ldc = C_out.stride(0) if M > 1 else max(C_out.stride(0), N)
    _check(_entry, getattr(lib(), _entry)(_ptr(A, torch.bfloat16), lda, _contig(B_packed), _ptr(C_out),
                                          ldc, M, N, K, od, _stream(stream)))


def det_probe_lds_fill(src: torch.Tensor, path: int, workgroups: int, iters: int, sink: torch.Tensor, stream=None) -> None:
    """Measurement aid: see the header.  src: any contiguous device tensor; sink: at least 4 bytes."""
    _check("det_probe_lds_fill", lib().det_probe_lds_fill(_contig(src), src.numel() * src.element_size(), path,
                                                           workgroups, iters, _contig(sink), _stream(stream)))


def det_gemm_bf16_fixed_tile(A: torch.Tensor, B_packed: torch.Tensor, C_out: torch.Tensor, N: int, K: int,
                             stream=None) -> None:
    """det_gemm_bf16 with the one tiling per (N, K) that does not look at M; same bytes."""
    det_gemm_bf16(A, B_packed, C_out, N, K, stream, _entry="det_gemm_bf16_fixed_tile")


def det_gemm_pack_gate_up(B_kn: torch.Tensor, B_packed: torch.Tensor, stream=None) -> None:
    K, N2 = B_kn.shape
    if N2 % 2 or B_packed.numel() * B_packed.element_size() < 2 * N2 * K:
        raise ValueError("bad gate/up weight")
    _check("det_gemm_pack_gate_up", lib().det_gemm_pack_gate_up(_contig(B_kn, torch.bfloat16), _contig(B_packed),
                                                                 N2 // 2, K, _stream(stream)))


def pack_gate_up(B_kn: torch.Tensor, stream=None) -> torch.Tensor:
    """Allocates and fills the packed form of a [K, 2F] (gate | up) weight for det_gemm_swiglu_bf16."""
    K, N2 = B_kn.shape
    if det_gemm_packed_b_bytes(N2, K) == 0:
        raise DetError("det_gemm_packed_b_bytes", 2)
    out = torch.empty(N2 * K, dtype=torch.bfloat16, device=B_kn.device)
    det_gemm_pack_gate_up(B_kn, out, stream)
    return out


def det_gemm_pack_qkv(B_kn: torch.Tensor, B_packed: torch.Tensor, Hq: int, Hkv: int, D: int = 128, stream=None) -> None:
    K, N = B_kn.shape
    if N != (Hq + 2 * Hkv) * D or B_packed.numel() * B_packed.element_size() < 2 * N * K:
        raise ValueError("bad fused query/key/value weight")
    _check("det_gemm_pack_qkv", lib().det_gemm_pack_qkv(_contig(B_kn, torch.bfloat16), _contig(B_packed), Hq, Hkv, D, K,
                                                         _stream(stream)))


def pack_qkv(B_kn: torch.Tensor, Hq: int, Hkv: int, D: int = 128, stream=None) -> torch.Tensor:
    """Allocates and fills the packed form of a [K, (Hq+2Hkv)D] weight for det_gemm_qkv_rope_append (the
    form det_decoder_layer takes as wqkv)."""
    K, N = B_kn.shape
    if det_gemm_packed_b_bytes(N, K) == 0:
        raise DetError("det_gemm_packed_b_bytes", 2)
    out = torch.empty(N * K, dtype=torch.bfloat16, device=B_kn.device)
    det_gemm_pack_qkv(B_kn, out, Hq, Hkv, D, stream)
    return out


def det_gemm_qkv_rope_append(A, B_qkv, qbuf, kcache, vcache, positions, slots, rope_cos, rope_sin, stream=None) -> None:
    """The layer's fused projection: A [M, K] times the weight of pack_qkv, query heads rotated into qbuf
    [M, Hq, D], key heads rotated and value heads copied into caches [S, Hkv, Lmax, D] at (slot, position).
    slots None: row i uses slot i."""
    M, K = A.shape
    _, Hq, D = qbuf.shape
    _, Hkv, Lmax, _ = kcache.shape
    if qbuf.shape[0] != M or vcache.shape != kcache.shape or A.stride(1) != 1 or positions.numel() != M:
        raise ValueError("bad fused projection operands")
    if slots is not None and slots.numel() != M:
        raise ValueError("bad slots")
    if rope_cos.shape != (Lmax, D // 2) or rope_sin.shape != (Lmax, D // 2):
        raise ValueError("bad rope tables")
    _check("det_gemm_qkv_rope_append", lib().det_gemm_qkv_rope_append(
        _ptr(A, torch.bfloat16), _ld(A, K), _contig(B_qkv), _contig(qbuf, torch.bfloat16),
        _contig(kcache, torch.bfloat16), _contig(vcache, torch.bfloat16), _contig(positions, torch.int32),
        None if slots is None else _contig(slots, torch.int32), _contig(rope_cos, torch.float32),
        _contig(rope_sin, torch.float32), M, Hq, Hkv, D, Lmax, K, _stream(stream)))


def det_rmsnorm_gemm_qkv_rope_append(x, w_norm, eps: float, B_qkv, h, qbuf, kcache, vcache, positions, slots, rope_cos,
                                     rope_sin, stream=None) -> None:
    """det_gemm_qkv_rope_append of det_rmsnorm(x, w_norm, eps); h [M, K] bf16 is scratch."""
    M, K = x.shape
    _, Hq, D = qbuf.shape
    _, Hkv, Lmax, _ = kcache.shape
    if qbuf.shape[0] != M or vcache.shape != kcache.shape or x.stride(1) != 1 or positions.numel() != M:
        raise ValueError("bad fused projection operands")
    if w_norm.shape != (K,) or h.shape != (M, K) or (slots is not None and slots.numel() != M):
        raise ValueError("bad norm operands")
    if rope_cos.shape != (Lmax, D // 2) or rope_sin.shape != (Lmax, D // 2):
        raise ValueError("bad rope tables")
    _check("det_rmsnorm_gemm_qkv_rope_append", lib().det_rmsnorm_gemm_qkv_rope_append(
        _ptr(x, torch.bfloat16), _ld(x, K), _contig(w_norm, torch.bfloat16), eps, _contig(B_qkv),
        _contig(h, torch.bfloat16), _contig(qbuf, torch.bfloat16), _contig(kcache, torch.bfloat16),
        _contig(vcache, torch.bfloat16), _contig(positions, torch.int32),
        None if slots is None else _contig(slots, torch.int32), _contig(rope_cos, torch.float32),
        _contig(rope_sin, torch.float32), M, Hq, Hkv, D, Lmax, K, _stream(stream)))


def det_rmsnorm_gemm_swiglu_bf16(x, w_norm, eps: float, B_gate_up, h, Y, F: int, stream=None) -> None:
    """det_gemm_swiglu_bf16 of det_rmsnorm(x, w_norm, eps); h [M, K] bf16 is scratch."""
    M, K = x.shape
    if Y.shape != (M, F) or x.stride(1) != 1 or Y.stride(1) != 1 or w_norm.shape != (K,) or h.shape != (M, K):
        raise ValueError("bad operand shapes")
    _check("det_rmsnorm_gemm_swiglu_bf16", lib().det_rmsnorm_gemm_swiglu_bf16(
        _ptr(x, torch.bfloat16), _ld(x, K), _contig(w_norm, torch.bfloat16), eps, _contig(B_gate_up),
        _contig(h, torch.bfloat16), _ptr(Y, torch.bfloat16), _ld(Y, F), M, F, K, _stream(stream)))


def det_rmsnorm_gemm_bf16(x, w_norm, eps: float, B_packed, h, C_out, N: int, stream=None) -> None:
    """det_gemm_bf16 of det_rmsnorm(x, w_norm, eps); h [M, K] bf16 is scratch; C_out bf16 or fp32."""
    M, K = x.shape
    if C_out.shape != (M, N) or x.stride(1) != 1 or C_out.stride(1) != 1 or w_norm.shape != (K,) or h.shape != (M, K):
        raise ValueError("bad operand shapes")
    if C_out.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("output must be bf16 or fp32")
    _check("det_rmsnorm_gemm_bf16", lib().det_rmsnorm_gemm_bf16(
        _ptr(x, torch.bfloat16), _ld(x, K), _contig(w_norm, torch.bfloat16), eps, _contig(B_packed),
        _contig(h, torch.bfloat16), C_out.data_ptr(), _ld(C_out, N), M, N, K,
        DET_F32 if C_out.dtype == torch.float32 else DET_BF16, _stream(stream)))


def _ld(t: torch.Tensor, cols: int) -> int:
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), cols)


def det_gemm_bf16_residual(A, B_packed, R, C_out, N: int, K: int, stream=None) -> None:
    """C_out = bf16(fp32(bf16(A @ B)) + fp32(R)); C_out may be R."""
    M = A.shape[0]
    if A.shape[1] != K or C_out.shape != (M, N) or R.shape != (M, N):
        raise ValueError("bad GEMM operand shapes")
    if A.stride(1) != 1 or C_out.stride(1) != 1 or R.stride(1) != 1:
        raise ValueError("rows must be contiguous")
    _check("det_gemm_bf16_residual", lib().det_gemm_bf16_residual(
        _ptr(A, torch.bfloat16), _ld(A, K), _contig(B_packed), _ptr(R, torch.bfloat16), _ld(R, N),
        _ptr(C_out, torch.bfloat16), _ld(C_out, N), M, N, K, _stream(stream)))


def det_gemm_swiglu_bf16(A, B_gate_up, Y, F: int, K: int, stream=None) -> None:
    """Y[M, F] = swiglu(bf16(A @ Wgate), bf16(A @ Wup)) with the weight packed by pack_gate_up."""
    M = A.shape[0]
    if A.shape[1] != K or Y.shape != (M, F) or A.stride(1) != 1 or Y.stride(1) != 1:
        raise ValueError("bad GEMM operand shapes")
    _check("det_gemm_swiglu_bf16", lib().det_gemm_swiglu_bf16(
        _ptr(A, torch.bfloat16), _ld(A, K), _contig(B_gate_up), _ptr(Y, torch.bfloat16), _ld(Y, F), M, F, K,
        _stream(stream)))


def det_rmsnorm(x: torch.Tensor, w: torch.Tensor, y: torch.Tensor, eps: float, stream=None) -> None:
    M, H = x.shape
    if w.shape != (H,) or y.shape != x.shape:
        raise ValueError("bad RMSNorm shapes")
    _check("det_rmsnorm", lib().det_rmsnorm(_contig(x, torch.bfloat16), _contig(w, torch.bfloat16),
                                             _contig(y, torch.bfloat16), M, H, eps, _stream(stream)))


def det_attn_decode_workspace_bytes(B: int, Hq: int, D: int, Lmax: int) -> int:
    return lib().det_attn_decode_workspace_bytes(B, Hq, D, Lmax)


def det_attn_decode(q, kcache, vcache, seqlens, out, ws, scale: float, stream=None) -> None:
    B, Hq, D = q.shape
    B2, Hkv, Lmax, D2 = kcache.shape
    if (B2, D2) != (B, D) or vcache.shape != kcache.shape or out.shape != q.shape or seqlens.shape != (B,):
        raise ValueError("bad attention shapes")
    _check("det_attn_decode", lib().det_attn_decode(
        _contig(q, torch.bfloat16), _contig(kcache, torch.bfloat16), _contig(vcache, torch.bfloat16),
        _contig(seqlens, torch.int32), _contig(out, torch.bfloat16), _contig(ws),
        ws.numel() * ws.element_size(), B, Hq, Hkv, D, Lmax, scale, _stream(stream)))


def det_attn_decode_static(q, kcache, vcache, seqlens, out, scale: float, stream=None) -> None:
    """det_attn_decode with the chunk partials in the library's fixed per-device array (allocates nothing)."""
    B, Hq, D = q.shape
    B2, Hkv, Lmax, D2 = kcache.shape
    if (B2, D2) != (B, D) or vcache.shape != kcache.shape or out.shape != q.shape or seqlens.shape != (B,):
        raise ValueError("bad attention shapes")
    _check("det_attn_decode_static", lib().det_attn_decode_static(
        _contig(q, torch.bfloat16), _contig(kcache, torch.bfloat16), _contig(vcache, torch.bfloat16),
        _contig(seqlens, torch.int32), _contig(out, torch.bfloat16), B, Hq, Hkv, D, Lmax, scale, _stream(stream)))


def det_attn_decode_rows(q, kcache, vcache, seqlens, slots, out, ws, scale: float, stream=None) -> None:
    R, Hq, D = q.shape
    S, Hkv, Lmax, D2 = kcache.shape
    if D2 != D or vcache.shape != kcache.shape or out.shape != q.shape or seqlens.shape != (R,) or slots.shape != (R,):
        raise ValueError("bad attention shapes")
    _check("det_attn_decode_rows", lib().det_attn_decode_rows(
        _contig(q, torch.bfloat16), _contig(kcache, torch.bfloat16), _contig(vcache, torch.bfloat16),
        _contig(seqlens, torch.int32), _contig(slots, torch.int32), _contig(out, torch.bfloat16), _contig(ws),
        ws.numel() * ws.element_size(), R, Hq, Hkv, D, Lmax, scale, _stream(stream)))


def det_softmax_f32(s, lens, p, m_out, l_out, stream=None) -> None:
    R, Lmax = s.shape
    if p.shape != s.shape or lens.shape != (R,) or m_out.shape != (R,) or l_out.shape != (R,):
        raise ValueError("bad softmax shapes")
    _check("det_softmax_f32", lib().det_softmax_f32(
        _contig(s, torch.float32), _contig(lens, torch.int32), _contig(p, torch.float32),
        _contig(m_out, torch.float32), _contig(l_out, torch.float32), R, Lmax, _stream(stream)))


def det_argmax(logits: torch.Tensor, idx: torch.Tensor, stream=None) -> None:
    B, V = logits.shape
    if idx.shape != (B,):
        raise ValueError("bad argmax shapes")
    if logits.dtype == torch.float32:
        dt = DET_F32
    elif logits.dtype == torch.bfloat16:
        dt = DET_BF16
    else:
        raise TypeError("logits must be fp32 or bf16")
    _check("det_argmax", lib().det_argmax(_contig(logits), _contig(idx, torch.int32), B, V, dt, _stream(stream)))


def det_sample(logits, temperature: float, top_k: int, top_p: float, seed: int, seq_ids, steps, tokens,
               stream=None) -> None:
    B, V = logits.shape
    for a in (seq_ids, steps, tokens):
        if a.shape != (B,):
            raise ValueError("bad sampling shapes")
    _check("det_sample", lib().det_sample(_contig(logits, torch.float32), B, V, temperature, top_k, top_p,
                                           seed & (2 ** 64 - 1), _contig(seq_ids, torch.int32),
                                           _contig(steps, torch.int32), _contig(tokens, torch.int32),
                                           _stream(stream)))


def det_rope(x, y, pos, cos_t, sin_t, stream=None) -> None:
    R, nh, D = x.shape
    Lmax = cos_t.shape[0]
    if y.shape != x.shape or pos.shape != (R,) or cos_t.shape != (Lmax, D // 2) or sin_t.shape != cos_t.shape:
        raise ValueError("bad rope shapes")
    _check("det_rope", lib().det_rope(_contig(x, torch.bfloat16), nh * D, _contig(y, torch.bfloat16), nh * D,
                                       _contig(pos, torch.int32), _contig(cos_t, torch.float32),
                                       _contig(sin_t, torch.float32), R, nh, D, Lmax, _stream(stream)))


def det_swiglu(g, u, y, stream=None) -> None:
    R, F = g.shape
    if u.shape != g.shape or y.shape != g.shape or g.stride(1) != 1 or u.stride(1) != 1 or y.stride(1) != 1:
        raise ValueError("bad swiglu shapes")
    _check("det_swiglu", lib().det_swiglu(_ptr(g, torch.bfloat16), g.stride(0), _ptr(u, torch.bfloat16),
                                           u.stride(0), _ptr(y, torch.bfloat16), y.stride(0), R, F,
                                           _stream(stream)))


def det_residual_add(x, y, z, stream=None) -> None:
    if y.shape != x.shape or z.shape != x.shape:
        raise ValueError("bad residual shapes")
    _check("det_residual_add", lib().det_residual_add(_contig(x, torch.bfloat16), _contig(y, torch.bfloat16),
                                                       _contig(z, torch.bfloat16), x.numel(), _stream(stream)))


def det_embed_gather(table, tokens, out, stream=None) -> None:
    V, H = table.shape
    B = tokens.shape[0]
    if out.shape != (B, H):
        raise ValueError("bad embedding shapes")
    _check("det_embed_gather", lib().det_embed_gather(_contig(table, torch.bfloat16), _contig(tokens, torch.int32),
                                                       _contig(out, torch.bfloat16), B, H, V, _stream(stream)))


def layer_cfg(H, Hq, Hkv, D, F, Lmax, eps, scale) -> LayerCfg:
    return LayerCfg(H, Hq, Hkv, D, F, Lmax, eps, scale)


def layer_weights(w_norm1, wqkv, wo, w_norm2, wgu, wdown) -> LayerWeights:
    """Device pointers of one layer's weights (projections already packed: wqkv, wo, wdown with
    pack_weight, wgu with pack_gate_up).  The struct keeps a reference to the six tensors, so they
    live as long as it does."""
    tensors = (w_norm1, wqkv, wo, w_norm2, wgu, wdown)
    s = LayerWeights(*[_contig(t) for t in tensors])
    s._keep = tensors
    return s


def det_decoder_layer_workspace_bytes(cfg: LayerCfg, B: int) -> int:
    return lib().det_decoder_layer_workspace_bytes(C.byref(cfg), B)


def det_decoder_layer(w: LayerWeights, cfg: LayerCfg, x, kcache, vcache, positions, rope_cos, rope_sin, ws,
                      stream=None) -> None:
    B = x.shape[0]
    if x.shape != (B, cfg.H) or kcache.shape != (B, cfg.Hkv, cfg.Lmax, cfg.D) or vcache.shape != kcache.shape:
        raise ValueError("bad layer shapes")
    if positions.shape != (B,) or rope_cos.shape != (cfg.Lmax, cfg.D // 2) or rope_sin.shape != rope_cos.shape:
        raise ValueError("bad layer shapes")
    _check("det_decoder_layer", lib().det_decoder_layer(
        C.byref(w), C.byref(cfg), _contig(x, torch.bfloat16), _contig(kcache, torch.bfloat16),
        _contig(vcache, torch.bfloat16), _contig(positions, torch.int32), _contig(rope_cos, torch.float32),
        _contig(rope_sin, torch.float32), _contig(ws), ws.numel() * ws.element_size(), B, _stream(stream)))


def det_decoder_layer_rows(w: LayerWeights, cfg: LayerCfg, x, kcache, vcache, positions, slots, rope_cos, rope_sin,
                           ws, stream=None) -> None:
    R = x.shape[0]
    if x.shape != (R, cfg.H) or kcache.shape[1:] != (cfg.Hkv, cfg.Lmax, cfg.D) or vcache.shape != kcache.shape:
        raise ValueError("bad layer shapes")
    if positions.shape != (R,) or slots.shape != (R,) or rope_cos.shape != (cfg.Lmax, cfg.D // 2):
        raise ValueError("bad layer shapes")
    _check("det_decoder_layer_rows", lib().det_decoder_layer_rows(
        C.byref(w), C.byref(cfg), _contig(x, torch.bfloat16), _contig(kcache, torch.bfloat16),
        _contig(vcache, torch.bfloat16), _contig(positions, torch.int32), _contig(slots, torch.int32),
        _contig(rope_cos, torch.float32), _contig(rope_sin, torch.float32), _contig(ws),
        ws.numel() * ws.element_size(), R, _stream(stream)))


def det_qdecoder_layer_workspace_bytes(cfg: LayerCfg, R: int) -> int:
    return lib().det_qdecoder_layer_workspace_bytes(C.byref(cfg), R)


def det_qdecoder_layer(w: LayerWeights, cfg: LayerCfg, x, kcache, vcache, positions, slots, rope_cos, rope_sin,
                       ws, stream=None) -> None:
    """The decoder layer on quantized weights; slots may be None (row r uses cache slot r)."""
    R = x.shape[0]
    if x.shape != (R, cfg.H) or kcache.shape[1:] != (cfg.Hkv, cfg.Lmax, cfg.D) or vcache.shape != kcache.shape:
        raise ValueError("bad layer shapes")
    if positions.shape != (R,) or rope_cos.shape != (cfg.Lmax, cfg.D // 2):
        raise ValueError("bad layer shapes")
    if slots is None:
        if kcache.shape[0] < R:
            raise ValueError("bad layer shapes")
        sl = None
    else:
        if slots.shape != (R,):
            raise ValueError("bad layer shapes")
        sl = _contig(slots, torch.int32)
    _check("det_qdecoder_layer", lib().det_qdecoder_layer(
        C.byref(w), C.byref(cfg), _contig(x, torch.bfloat16), _contig(kcache, torch.bfloat16),
        _contig(vcache, torch.bfloat16), _contig(positions, torch.int32), sl,
        _contig(rope_cos, torch.float32), _contig(rope_sin, torch.float32), _contig(ws),
        ws.numel() * ws.element_size(), R, _stream(stream)))


def det_decode_advance(last_sampled, base_positions, j: int, tokens_out, positions_out, stream=None) -> None:
    B = last_sampled.shape[0]
    for a in (last_sampled, base_positions, tokens_out, positions_out):
        if a.shape != (B,):
            raise ValueError("bad decode_advance shapes")
    _check("det_decode_advance", lib().det_decode_advance(
        _contig(last_sampled, torch.int32), _contig(base_positions, torch.int32), j,
        _contig(tokens_out, torch.int32), _contig(positions_out, torch.int32), B, _stream(stream)))


def det_next_token(prompts, prompt_lens, last_sampled, tokens_out, positions_out, history, t: int,
                   stream=None) -> None:
    B, Tp = prompts.shape
    Th = history.shape[1]
    for a in (prompt_lens, last_sampled, tokens_out, positions_out):
        if a.shape != (B,):
            raise ValueError("bad next_token shapes")
    if history.shape[0] != B:
        raise ValueError("bad next_token shapes")
    _check("det_next_token", lib().det_next_token(
        _contig(prompts, torch.int32), Tp, _contig(prompt_lens, torch.int32), _contig(last_sampled, torch.int32),
        _contig(tokens_out, torch.int32), _contig(positions_out, torch.int32), _contig(history, torch.int32),
        Th, t, B, _stream(stream)))
