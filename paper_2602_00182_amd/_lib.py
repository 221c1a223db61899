"""Loads libdetinfer.so (built in-tree by paper_2602_00182_amd.build) through ctypes.

There is no fallback: if the library is missing or a symbol is absent this raises."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdetinfer.so")


class LayerCfg(C.Structure):
    _fields_ = [("H", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("F", C.c_int32), ("Lmax", C.c_int32), ("eps", C.c_float), ("scale", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [("w_norm1", C.c_void_p), ("wqkv", C.c_void_p), ("wo", C.c_void_p),
                ("w_norm2", C.c_void_p), ("wgu", C.c_void_p), ("wdown", C.c_void_p)]


class Sha256Ctx(C.Structure):
    _fields_ = [("h", C.c_uint32 * 8), ("nbytes", C.c_uint64), ("buf", C.c_uint8 * 64), ("fill", C.c_uint32)]


_vp, _i, _f, _sz, _i64 = C.c_void_p, C.c_int, C.c_float, C.c_size_t, C.c_int64

# name -> (restype, argtypes); mirrors include/detinfer.h one to one
SIGNATURES = {
    "det_gemm_bf16": (_i, [_vp, _i, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "det_gemm_bf16_fixed_tile": (_i, [_vp, _i, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "det_gemm_packed_b_bytes": (_sz, [_i, _i]),
    "det_gemm_pack_b": (_i, [_vp, _vp, _i, _i, _vp]),
    "det_gemm_bf16_residual": (_i, [_vp, _i, _vp, _vp, _i, _vp, _i, _i, _i, _i, _vp]),
    "det_gemm_pack_gate_up": (_i, [_vp, _vp, _i, _i, _vp]),
    "det_gemm_swiglu_bf16": (_i, [_vp, _i, _vp, _vp, _i, _i, _i, _i, _vp]),
    "det_gemm_pack_qkv": (_i, [_vp, _vp, _i, _i, _i, _i, _vp]),
    "det_gemm_qkv_rope_append": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp]),
    "det_rmsnorm_gemm_qkv_rope_append": (_i, [_vp, _i, _vp, _f, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i,
                                              _i, _i, _i, _vp]),
    "det_rmsnorm_gemm_swiglu_bf16": (_i, [_vp, _i, _vp, _f, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "det_rmsnorm_gemm_bf16": (_i, [_vp, _i, _vp, _f, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "det_rmsnorm": (_i, [_vp, _vp, _vp, _i, _i, _f, _vp]),
    "det_attn_decode_workspace_bytes": (_sz, [_i, _i, _i, _i]),
    "det_attn_decode": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _sz, _i, _i, _i, _i, _i, _f, _vp]),
    "det_attn_decode_static": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _vp]),
    "det_attn_decode_rows": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _i, _i, _i, _i, _i, _f, _vp]),
    "det_softmax_f32": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _vp]),
    "det_argmax": (_i, [_vp, _vp, _i, _i, _i, _vp]),
    "det_sample": (_i, [_vp, _i, _i, _f, _i, _f, C.c_uint64, _vp, _vp, _vp, _vp]),
    "det_rope": (_i, [_vp, _i, _vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "det_swiglu": (_i, [_vp, _i, _vp, _i, _vp, _i, _i, _i, _vp]),
    "det_residual_add": (_i, [_vp, _vp, _vp, _i64, _vp]),
    "det_embed_gather": (_i, [_vp, _vp, _vp, _i, _i, _i, _vp]),
    "det_decoder_layer_workspace_bytes": (_sz, [C.POINTER(LayerCfg), _i]),
    "det_decoder_layer": (_i, [C.POINTER(LayerWeights), C.POINTER(LayerCfg), _vp, _vp, _vp, _vp, _vp, _vp,
                               _vp, _sz, _i, _vp]),
    "det_decoder_layer_rows": (_i, [C.POINTER(LayerWeights), C.POINTER(LayerCfg), _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                    _vp, _sz, _i, _vp]),
    "det_probe_lds_fill": (_i, [_vp, _sz, _i, _i, _i, _vp, _vp]),
    "det_next_token": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp]),
    "det_decode_advance": (_i, [_vp, _vp, _i, _vp, _vp, _i, _vp]),
    "det_qgemm_packed_w_bytes": (_sz, [_i, _i]),
    "det_quant_pack_w4": (_i, [_vp, _vp, _i, _i, _vp]),
    "det_quant_unpack_w4": (_i, [_vp, _vp, _vp, _i, _i, _vp]),
    "det_quant_act_codes_bytes": (_sz, [_i, _i]),
    "det_quant_act_scales_bytes": (_sz, [_i, _i]),
    "det_quant_act_q8": (_i, [_vp, _i, _vp, _vp, _i, _i, _vp]),
    "det_qgemm_w4a8": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "det_quant_pack_w4_gate_up": (_i, [_vp, _vp, _i, _i, _vp]),
    "det_qgemm_w4a8_residual": (_i, [_vp, _vp, _vp, _vp, _i, _vp, _i, _i, _i, _i, _vp]),
    "det_qgemm_w4a8_swiglu": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "det_quant_pack_w4_qkv": (_i, [_vp, _vp, _i, _i, _i, _i, _vp]),
    "det_qgemm_w4a8_qkv_rope_append": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp]),
    "det_rmsnorm_quant_q8": (_i, [_vp, _vp, _vp, _vp, _i, _i, _f, _vp]),
    "det_qgemm_w4a8_swiglu_quant_supported": (_i, [_i, _i]),
    "det_qgemm_w4a8_swiglu_quant": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp]),
    "det_attn_decode_quant_q8": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _i, _i, _i, _i, _i, _f, _vp]),
    "det_qdecoder_layer_workspace_bytes": (_sz, [C.POINTER(LayerCfg), _i]),
    "det_qdecoder_layer": (_i, [C.POINTER(LayerWeights), C.POINTER(LayerCfg), _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                _vp, _sz, _i, _vp]),
    "det_sha256_init": (_i, [C.POINTER(Sha256Ctx)]),
    "det_sha256_update": (_i, [C.POINTER(Sha256Ctx), _vp, _sz]),
    "det_sha256_final": (_i, [C.POINTER(Sha256Ctx), _vp]),
    "det_commit_sha256": (_i, [_vp, _sz, _vp, _sz, _vp, _sz, _vp]),
    "det_sha256_force_portable": (_i, [_i]),
    "det_fingerprint": (C.c_char_p, []),
    "det_last_hip_error": (_i, []),
}

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2602_00182_amd.build` "
                "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)  # AttributeError if the symbol is not exported
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib
