"""The C-ABI library loads and exports every entry point that include/detinfer.h declares, and the
Python binding mirrors the same names (no compute: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "detinfer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(det_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_contract_calls():
    names = _declared()
    for required in ["det_gemm_bf16", "det_rmsnorm", "det_attn_decode", "det_argmax", "det_decoder_layer"]:
        assert required in names


def test_library_exports_every_declared_symbol():
    from paper_2602_00182_amd import _lib

    assert os.path.exists(_lib.LIB_PATH), "build with python -m paper_2602_00182_amd.build"
    so = ctypes.CDLL(_lib.LIB_PATH)
    for name in _declared():
        assert hasattr(so, name), name
    assert sorted(_lib.SIGNATURES) == _declared()


def test_binding_mirrors_the_names():
    import paper_2602_00182_amd as d

    for name in _declared():
        assert callable(getattr(d, name)), name
    assert "gfx950" in d.det_fingerprint()
    assert d.det_gemm_packed_b_bytes(4096, 4096) == 2 * 4096 * 4096
    assert d.det_gemm_packed_b_bytes(4095, 4096) == 0
    assert d.det_attn_decode_workspace_bytes(2, 32, 128, 512) == 2 * 32 * 2 * 130 * 4
    assert d.det_attn_decode_workspace_bytes(2, 32, 64, 512) == 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_00182_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src, f
                assert "liboracle" not in src and "oracle.c" not in src, f
