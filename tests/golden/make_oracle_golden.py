"""Writes tests/golden/oracle_golden.txt: SHA-256 digests of the CPU oracle's outputs on seeded
inputs.  Calls only oracle/ and the input generator; nothing here comes from the GPU.  The file
guards the oracle against accidental change: a deliberate change to its arithmetic regenerates it
and says why in the commit message.  (The paper prints no numeric example to store instead.)

    python tests/golden/make_oracle_golden.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import detsynth as ds  # noqa: E402
import oracle  # noqa: E402


def cases():
    yield "bf16_rne", oracle.bf16_rne(np.linspace(-3.0, 3.0, 100001).astype(np.float32))
    yield "expf", oracle.expf(np.linspace(-87.0, 88.72, 200001).astype(np.float32))
    yield "tree256", np.array([oracle.tree256(ds.bf16_bits_to_f32(ds.normal_bf16(100 + i, (256,)))) for i in range(64)])
    x = ds.normal_bf16(11, (8, 4096))
    w = ds.normal_bf16(12, (4096,), 0.1, 1.0)
    yield "rmsnorm", oracle.rmsnorm(x, w, 1e-5)
    s = (ds.bf16_bits_to_f32(ds.normal_bf16(13, (6, 1500))) * np.float32(3)).astype(np.float32)
    p, m, l = oracle.softmax_f32(s, [1, 255, 256, 257, 1024, 1500])
    yield "softmax_p", p
    yield "softmax_m", m
    yield "softmax_l", l
    yield "argmax", oracle.argmax_bf16(ds.normal_bf16(14, (16, 32000)))
    A = ds.normal_bf16(15, (7, 320))
    B = ds.normal_bf16(16, (320, 48), 0.05)
    c, ca = oracle.gemm_f64(A, B)
    yield "gemm", c
    yield "gemm_abs", ca
    # (the fp64 attention reference calls libm's exp, whose last bit may differ between C libraries:
    # it is pinned by closed forms in the tests instead of a digest)
    cos_t, sin_t = ds.rope_tables(64, 128)
    yield "rope", oracle.rope(ds.normal_bf16(20, (3, 4, 128)), [0, 17, 63], cos_t, sin_t)
    g = ds.normal_bf16(21, (4096,), 2.0)
    u = ds.normal_bf16(22, (4096,))
    yield "swiglu", oracle.swiglu(g, u)
    yield "residual", oracle.residual(g, u)


def digests():
    return [(name, hashlib.sha256(np.ascontiguousarray(arr).tobytes()).hexdigest()) for name, arr in cases()]


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_golden.txt")
    with open(out, "w") as f:
        f.write("# written by tests/golden/make_oracle_golden.py from oracle/ alone; SHA-256 of raw output bytes\n")
        for name, d in digests():
            f.write(f"{name} {d}\n")
    print(out)
