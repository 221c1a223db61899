"""Output commitment: the library's host-side SHA-256 against the FIPS 180-4 example digests and
against the oracle (hashlib) on ragged lengths and update boundaries, for both compression-function
paths (portable, and the CPU's SHA instructions where present); the oracle against the same
examples.  No GPU involved."""
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def fips_vectors():
    out = []
    for line in open(os.path.join(HERE, "golden", "sha256_fips180.txt")):
        if line.startswith("#") or not line.strip():
            continue
        spec, digest = line.split()
        if spec == "empty":
            msg = b""
        elif spec.startswith("ascii:"):
            msg = spec[6:].encode()
        else:
            _, ch, n = spec.split(":")
            msg = ch.encode() * int(n)
        out.append((msg, bytes.fromhex(digest)))
    return out


@pytest.fixture(scope="module")
def d():
    import paper_2602_00182_amd as d
    return d


def test_oracle_matches_fips_examples(orc):
    for msg, digest in fips_vectors():
        assert orc.commit_sha256(msg, b"", b"") == digest
        assert orc.commit_sha256(b"", msg, b"") == digest
        third = len(msg) // 3
        assert orc.commit_sha256(msg[:third], msg[third:2 * third], msg[2 * third:]) == digest


@pytest.mark.parametrize("portable", [True, False])
def test_library_matches_fips_examples(d, portable):
    d.det_sha256_force_portable(portable)
    try:
        for msg, digest in fips_vectors():
            assert d.det_commit_sha256(msg, None, None) == digest
            ctx = d.det_sha256_init()
            for i in range(0, len(msg), 4093):          # update boundaries off the block size
                d.det_sha256_update(ctx, msg[i:i + 4093])
            assert d.det_sha256_final(ctx) == digest
    finally:
        d.det_sha256_force_portable(False)


@pytest.mark.parametrize("portable", [True, False])
def test_library_matches_oracle_on_ragged_inputs(d, orc, portable):
    rng = np.random.default_rng(11)
    d.det_sha256_force_portable(portable)
    try:
        for n in list(range(0, 200)) + [255, 256, 257, 4095, 4096, 65537, 1 << 20]:
            data = rng.integers(0, 256, n, dtype=np.uint8).tobytes()
            a, b = sorted(rng.integers(0, n + 1, 2).tolist())
            want = orc.commit_sha256(data[:a], data[a:b], data[b:])
            assert d.det_commit_sha256(data[:a], data[a:b], data[b:]) == want, n
            ctx = d.det_sha256_init()
            pos = 0
            while pos < n:
                step = int(rng.integers(1, 130))
                d.det_sha256_update(ctx, data[pos:pos + step])
                pos += step
            assert d.det_sha256_final(ctx) == want, n
    finally:
        d.det_sha256_force_portable(False)


def test_numpy_and_tensor_inputs_and_errors(d, orc):
    import torch
    p = np.arange(7, dtype=np.int32)
    l = np.linspace(-1, 1, 33, dtype=np.float32)
    t = torch.arange(5, dtype=torch.int32)
    want = orc.commit_sha256(p.tobytes(), l.tobytes(), t.numpy().tobytes())
    assert d.det_commit_sha256(p, l, t) == want
    ctx = d.det_sha256_init()
    d.det_sha256_final(ctx)
    with pytest.raises(d.DetError):
        d.det_sha256_update(ctx, b"x")      # a spent context
    with pytest.raises(d.DetError):
        d.det_sha256_final(ctx)
