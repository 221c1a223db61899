"""Determinism under stress for attention, the decoder layer and the whole decode step (the GEMM has its
own such test): 100 repeats spread over three streams in shuffled launch order while another stream moves
256 MB back and forth, every result compared byte for byte with a quiet single-stream run (the paper's
same-host, batch-variance and co-scheduled-load conditions, sections 6.7, 10.1 and 10.2).  Each test stops
at its first mismatch."""
import math

import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, step, up

pytestmark = pytest.mark.gpu

SCALE = float(np.float32(1.0 / math.sqrt(128.0)))
REPS = 100


@pytest.fixture(scope="module")
def d():
    import paper_2602_00182_amd as d
    return d


class Hog:
    """A bandwidth hog on its own stream: one 256 MB device-to-device copy per repeat."""

    def __init__(self):
        self.stream = torch.cuda.Stream(device=DEV)
        self.a = torch.empty(256 << 20, dtype=torch.uint8, device=DEV)
        self.b = torch.empty_like(self.a)

    def kick(self):
        with torch.cuda.stream(self.stream):
            self.b.copy_(self.a)
            self.a.copy_(self.b)


def test_attention_repeats_streams_and_background_load(d):
    cases = []
    for (B, Hq, Hkv, L, seed) in [(16, 32, 8, 2048, 1), (1, 32, 8, 4096, 2), (5, 16, 4, 700, 3)]:
        s = ds.tensor_seed(3, 300) + 10 * seed
        q = ds.normal_bf16_torch(s, (B, Hq, 128), 1.0, 0.0, DEV)
        k = ds.normal_bf16_torch(s + 1, (B, Hkv, L, 128), 1.0, 0.0, DEV)
        v = ds.normal_bf16_torch(s + 2, (B, Hkv, L, 128), 1.0, 0.0, DEV)
        lens = ds.uniform_int(s + 3, (B,), 1, L)
        lens[0] = L
        cases.append((q, k, v, up(lens)))
    streams = [torch.cuda.Stream(device=DEV) for _ in range(3)]
    bufs = {}
    for ci, (q, k, v, lens) in enumerate(cases):
        B, Hq, _ = q.shape
        nbytes = d.det_attn_decode_workspace_bytes(B, Hq, 128, k.shape[2])
        for si in range(3):
            bufs[(ci, si)] = (torch.empty(nbytes, dtype=torch.uint8, device=DEV), torch.empty_like(q))
    want = []
    for ci, (q, k, v, lens) in enumerate(cases):
        ws, out = bufs[(ci, 0)]
        d.det_attn_decode(q, k, v, lens, out, ws, SCALE)
        want.append(out.clone())
    torch.cuda.synchronize()
    hog, rng = Hog(), np.random.default_rng(11)
    step("attention: 100 repeats over 3 streams with a background copy")
    for rep in range(REPS):
        hog.kick()
        launched = []
        for ci in rng.permutation(len(cases)):
            si = (rep + ci) % 3
            q, k, v, lens = cases[ci]
            ws, out = bufs[(ci, si)]
            with torch.cuda.stream(streams[si]):
                ws.fill_(0xFF if rep % 2 else 0)
                d.det_attn_decode(q, k, v, lens, out, ws, SCALE, streams[si])
            launched.append((ci, out))
        torch.cuda.synchronize()
        for ci, out in launched:
            assert torch.equal(out.view(torch.int16), want[ci].view(torch.int16)), f"repeat {rep}, case {ci}"


def test_decoder_layer_repeats_streams_and_background_load(d):
    H, Hq, Hkv, D, F, Lmax = 4096, 32, 8, 128, 14336, 2048
    s = ds.tensor_seed(4, 0)
    g = lambda i, shape, std=0.02, mean=0.0: ds.normal_bf16_torch(s + i, shape, std, mean, DEV)
    packed = [g(0, (H,), 0.0, 1.0), d.pack_qkv(g(1, (H, (Hq + 2 * Hkv) * D)), Hq, Hkv, D), d.pack_weight(g(2, (Hq * D, H))),
              g(3, (H,), 0.0, 1.0), d.pack_gate_up(g(4, (H, 2 * F))), d.pack_weight(g(5, (F, H)))]
    struct = d.layer_weights(*packed)
    cfg = d.layer_cfg(H, Hq, Hkv, D, F, Lmax, 1e-5, SCALE)
    cos_t, sin_t = ds.rope_tables(Lmax, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)
    streams = [torch.cuda.Stream(device=DEV) for _ in range(3)]
    cases = []
    for B in (1, 32):
        x0 = ds.normal_bf16_torch(s + 50 + B, (B, H), 1.0, 0.0, DEV)
        pos = up(ds.uniform_int(s + 60 + B, (B,), 0, Lmax - 1))
        per_stream = []
        for si in range(3):   # every stream owns its caches, workspace and x buffer; the cache contents are the same
            kc = ds.normal_bf16_torch(s + 70 + B, (B, Hkv, Lmax, D), 1.0, 0.0, DEV)
            vc = ds.normal_bf16_torch(s + 80 + B, (B, Hkv, Lmax, D), 1.0, 0.0, DEV)
            ws = torch.empty(d.det_decoder_layer_workspace_bytes(cfg, B), dtype=torch.uint8, device=DEV)
            per_stream.append((kc, vc, ws, torch.empty_like(x0)))
        cases.append((x0, pos, per_stream))
    want = []
    for x0, pos, per_stream in cases:
        kc, vc, ws, x = per_stream[0]
        x.copy_(x0)
        d.det_decoder_layer(struct, cfg, x, kc, vc, pos, cos_d, sin_d, ws)
        want.append((x.clone(), kc.clone()))
    torch.cuda.synchronize()
    hog, rng = Hog(), np.random.default_rng(12)
    step("decoder layer: 100 repeats over 3 streams with a background copy")
    for rep in range(REPS):
        hog.kick()
        launched = []
        for ci in rng.permutation(len(cases)):
            si = (rep + ci) % 3
            x0, pos, per_stream = cases[ci]
            kc, vc, ws, x = per_stream[si]
            with torch.cuda.stream(streams[si]):
                x.copy_(x0)
                d.det_decoder_layer(struct, cfg, x, kc, vc, pos, cos_d, sin_d, ws, streams[si])
            launched.append((ci, x, kc))
        torch.cuda.synchronize()
        for ci, x, kc in launched:
            assert torch.equal(x.view(torch.int16), want[ci][0].view(torch.int16)), f"repeat {rep}, case {ci}: x"
            if rep % 10 == 0:
                assert torch.equal(kc.view(torch.int16), want[ci][1].view(torch.int16)), f"repeat {rep}: cache"


def test_decode_step_repeats_streams_and_background_load(d):
    from paper_2602_00182_amd.decode import DecodeModel, ModelCfg

    H, Hq, Hkv, D, F, V, NL, Lm = 2048, 16, 4, 128, 5632, 32000, 8, 640
    s = ds.tensor_seed(5, 0)
    g = lambda i, shape, std=0.02, mean=0.0: ds.normal_bf16_torch(s + i, shape, std, mean, DEV)
    layers = []
    for l in range(NL):
        o = 10 + 10 * l
        layers.append(dict(norm1=g(o, (H,), 0.0, 1.0), wqkv=g(o + 1, (H, (Hq + 2 * Hkv) * D)), wo=g(o + 2, (Hq * D, H)),
                           norm2=g(o + 3, (H,), 0.0, 1.0), wgu=g(o + 4, (H, 2 * F)), wdown=g(o + 5, (F, H))))
    weights = dict(embed=g(1, (V, H), 1.0), lm_head=g(2, (H, V)), final_norm=g(3, (H,), 0.0, 1.0), layers=layers)
    model = DecodeModel(ModelCfg(H, Hq, Hkv, D, F, V, NL), weights)
    cos_t, sin_t = ds.rope_tables(Lm, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)
    streams = [torch.cuda.Stream(device=DEV) for _ in range(3)]
    cases = []
    for B in (1, 8):
        toks = up(ds.uniform_int(s + 900 + B, (B,), 0, V - 1))
        pos = up(ds.uniform_int(s + 910 + B, (B,), 0, Lm - 1))
        states = []
        for si in range(3):
            st = model.new_state(B, Lm, cos_d, sin_d)
            for i in range(NL):
                st.kcache[i].copy_(ds.normal_bf16_torch(s + 920 + i, tuple(st.kcache[i].shape), 1.0, 0.0, DEV))
                st.vcache[i].copy_(ds.normal_bf16_torch(s + 940 + i, tuple(st.vcache[i].shape), 1.0, 0.0, DEV))
            st.tokens.copy_(toks)
            st.positions.copy_(pos)
            states.append((st, torch.empty(B, dtype=torch.int32, device=DEV)))
        cases.append(states)
    want = []
    for states in cases:
        st, idx = states[0]
        st.forward()
        d.det_argmax(st.logits, idx)
        want.append((st.logits.clone(), idx.clone()))
    torch.cuda.synchronize()
    hog, rng = Hog(), np.random.default_rng(13)
    step("decode step (8 layers + lm_head + argmax): 100 repeats over 3 streams with a background copy")
    for rep in range(REPS):
        hog.kick()
        launched = []
        for ci in rng.permutation(len(cases)):
            si = (rep + ci) % 3
            st, idx = cases[ci][si]
            st.forward(streams[si])
            d.det_argmax(st.logits, idx, streams[si])
            launched.append((ci, st, idx))
        torch.cuda.synchronize()
        for ci, st, idx in launched:
            assert torch.equal(st.logits.view(torch.int32), want[ci][0].view(torch.int32)), f"repeat {rep}, case {ci}"
            assert torch.equal(idx, want[ci][1]), f"repeat {rep}, case {ci}: token"
