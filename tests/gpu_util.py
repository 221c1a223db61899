"""Helpers of the GPU parity tests: uploads, downloads, the GEMM error bound."""
import numpy as np
import torch

import detsynth as ds

DEV = "cuda:0"


def up_bf16(bits):
    return ds.to_torch_bf16(bits, DEV)


def down_bf16(t):
    return ds.from_torch_bf16(t)


def up(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def bits_to_f64(bits):
    return ds.bf16_bits_to_f32(bits).astype(np.float64)


def within_bound(got_f64, ref, refabs):
    """|got - ref| <= 2^-8 |ref| + 2^-20 sum_k |a_ik b_kj|  (the stated floating-point bar)."""
    return np.abs(got_f64 - ref) <= 2.0 ** -8 * np.abs(ref) + 2.0 ** -20 * refabs


def step(msg):
    """Names the case on stdout before the GPU work starts, so a fault can be attributed."""
    print(f"[case] {msg}", flush=True)
