"""det_attn_decode_static (the entry point for callers that cannot allocate: its chunk partials live in
a fixed per-device array inside the library) against det_attn_decode with a caller workspace: byte
equality on two calls in a row, the second with a smaller input, so the array still holds the first
call's partials when the second runs; and the size limit is refused without a launch."""
import math

import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, down_bf16, step, up, up_bf16

pytestmark = pytest.mark.gpu

SCALE = float(np.float32(1.0 / math.sqrt(128.0)))


@pytest.fixture(scope="module")
def d():
    import paper_2602_00182_amd as d
    return d


def _case(seed, B, Hq, Hkv, Lmax, lens):
    q = ds.normal_bf16(seed, (B, Hq, 128))
    k = ds.normal_bf16(seed + 1, (B, Hkv, Lmax, 128))
    v = ds.normal_bf16(seed + 2, (B, Hkv, Lmax, 128))
    return up_bf16(q), up_bf16(k), up_bf16(v), up(np.asarray(lens, dtype=np.int32))


def test_static_scratch_equals_workspace_variant_twice(d):
    big = _case(9100, 6, 32, 8, 2304, [2304, 1, 257, 1000, 2048, 511])
    small = _case(9200, 2, 16, 4, 600, [300, 600])
    for name, (q, k, v, lens) in (("first call, 6 x 2304", big), ("second call, 2 x 600", small)):
        B, Hq, D = q.shape
        Lmax = k.shape[2]
        ws = torch.empty(d.det_attn_decode_workspace_bytes(B, Hq, D, Lmax), dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)
        want = torch.empty_like(q)
        step(f"attention with caller workspace: {name}")
        d.det_attn_decode(q, k, v, lens, want, ws, SCALE)
        torch.cuda.synchronize()
        got = torch.full_like(q, float("nan"))
        step(f"attention with the static array: {name}")
        d.det_attn_decode_static(q, k, v, lens, got, SCALE)
        torch.cuda.synchronize()
        assert np.array_equal(down_bf16(got), down_bf16(want)), name


def test_static_scratch_limit_is_refused(d):
    lib = d.api.lib()
    # B * Hq * ceil(Lmax/256) = 8 * 32 * 256 = 65536 > 64527: one step past the array
    B, Hq, Hkv, Lmax = 8, 32, 8, 65536
    assert d.det_attn_decode_workspace_bytes(B, Hq, 128, Lmax) > (32 << 20)
    q = torch.zeros((B, Hq, 128), dtype=torch.bfloat16, device=DEV)
    tiny = torch.zeros(16, dtype=torch.bfloat16, device=DEV)   # never read: the call must refuse before launching
    lens = torch.zeros(B, dtype=torch.int32, device=DEV)
    out = torch.zeros_like(q)
    s = torch.cuda.current_stream().cuda_stream
    rc = lib.det_attn_decode_static(q.data_ptr(), tiny.data_ptr(), tiny.data_ptr(), lens.data_ptr(), out.data_ptr(),
                                    B, Hq, Hkv, 128, Lmax, SCALE, s)
    assert rc == 4   # DET_EWORKSPACE
    assert lib.det_attn_decode_static(q.data_ptr(), tiny.data_ptr(), tiny.data_ptr(), lens.data_ptr(), out.data_ptr(),
                                      B, Hq, Hkv, 64, Lmax, SCALE, s) == 2   # DET_ESHAPE: head dim
    torch.cuda.synchronize()
