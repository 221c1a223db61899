"""The decode loop against the oracle: a tiny random-init model (2 layers, H = 256) run through
greedy_decode and prefill_decode on the GPU, and through a model step composed from the oracle's own
functions (oracle.model.model_step) on the CPU, teacher-forced on the GPU's tokens.  Every op of the loop
has its own oracle test; this one checks the composition (section 6.6's loop as the pure function of section
6.1): which token feeds which step, positions, the cache rows a step reads, the last-row gather after
prefill, the lm_head and the token selection.

Bars.  Logits (fp32 from the GPU, fp64 reference): |err| <= 2^-8 |ref| + 2^-9 rms(ref row).  A logit is a
256-term product of the normalised final hidden row; the two sides' hidden rows differ only where one of
the roundings on the way landed on the other side of a bf16 boundary (one ulp, 2^-7 relative, of one
element), which moves a logit by about 2^-7 |xn_k w_kj| ~ 2^-11 rms(row).  On this small model no such flip
happens with the committed seeds (measured and printed: max err = 2^-20 rms, fp32 against fp64
accumulation only); the bar leaves room for a handful of flips, while an indexing mistake (wrong position,
row, token or weight orientation) moves logits by about rms(row) itself, five hundred times the bar.  Tokens:
equal to the oracle's argmax wherever the oracle's top-2 margin exceeds twice that bar."""
import math

import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, step, up, up_bf16

pytestmark = pytest.mark.gpu

H, HQ, HKV, D, F, V, NL = 256, 2, 1, 128, 512, 512, 2
SCALE = float(np.float32(1.0 / math.sqrt(128.0)))
CFG = dict(H=H, Hq=HQ, Hkv=HKV, D=D, F=F, eps=1e-5, scale=SCALE)
N_NEW = 6
LENS = np.array([5, 12, 1, 9], dtype=np.int32)


@pytest.fixture(scope="module")
def weights_h():
    s = ds.tensor_seed(5, 7000)
    g = lambda i, shape, std=0.05, mean=0.0: ds.normal_bf16(s + i, shape, std, mean)
    layers = [dict(norm1=g(10 * l + 10, (H,), 0.1, 1.0), wqkv=g(10 * l + 11, (H, (HQ + 2 * HKV) * D)),
                   wo=g(10 * l + 12, (HQ * D, H)), norm2=g(10 * l + 13, (H,), 0.1, 1.0),
                   wgu=g(10 * l + 14, (H, 2 * F)), wdown=g(10 * l + 15, (F, H))) for l in range(NL)]
    return dict(embed=g(1, (V, H), 1.0), lm_head=g(2, (H, V), 0.06), final_norm=g(3, (H,), 0.1, 1.0), layers=layers)


@pytest.fixture(scope="module")
def model(weights_h):
    from paper_2602_00182_amd.decode import DecodeModel, ModelCfg

    wd = {k: (up_bf16(v) if k != "layers" else [{n: up_bf16(t) for n, t in lw.items()} for lw in v])
          for k, v in weights_h.items()}
    return DecodeModel(ModelCfg(H, HQ, HKV, D, F, V, NL, 1e-5, SCALE), wd)


def _prompts():
    return ds.uniform_int(ds.tensor_seed(5, 7100), (len(LENS), int(LENS.max())), 0, V - 1).astype(np.int32)


def _oracle_run(weights_h, toks, lens, gen):
    """Token-by-token reference of every sequence in one batch (step t: prompt token t, then the GPU's own
    generated tokens).  Returns fp64 logits [T, B, V]."""
    from oracle import model as om

    B = len(lens)
    T = int(lens.max()) + N_NEW - 1
    cos_t, sin_t = ds.rope_tables(T, D, 5.0e5)
    cfg = dict(CFG, Lmax=T)
    kcs = [np.zeros((B, HKV, T, D), dtype=np.uint16) for _ in range(NL)]
    vcs = [np.zeros((B, HKV, T, D), dtype=np.uint16) for _ in range(NL)]
    out = []
    for t in range(T):
        tok = [toks[b, t] if t < lens[b] else gen[b, min(t - lens[b], N_NEW - 1)] for b in range(B)]
        out.append(om.model_step(weights_h, cfg, tok, np.full(B, t, dtype=np.int32), kcs, vcs, cos_t, sin_t))
    return np.stack(out)


def _check(ref_logits_bt, gpu_logits, gpu_token, what):
    """ref_logits_bt, gpu_logits: [V]; the bar of the module docstring."""
    rms = np.sqrt((ref_logits_bt ** 2).mean())
    bar = 2.0 ** -8 * np.abs(ref_logits_bt) + 2.0 ** -9 * rms
    err = np.abs(gpu_logits.astype(np.float64) - ref_logits_bt)
    assert (err <= bar).all(), (what, (err / bar).max())
    order = np.argsort(-ref_logits_bt, kind="stable")
    margin = ref_logits_bt[order[0]] - ref_logits_bt[order[1]]
    decided = margin > 2 * bar.max()
    if decided:
        assert gpu_token == order[0], (what, gpu_token, order[0])
    _check.worst_rel_rms = max(getattr(_check, "worst_rel_rms", 0.0), float((err / rms).max()))
    return (err / bar).max(), bool(decided)


def test_decode_loop_against_oracle_model(model, weights_h):
    from paper_2602_00182_amd.decode import greedy_decode, prefill_decode

    toks, lens = _prompts(), LENS
    T = int(lens.max()) + N_NEW - 1
    cos_t, sin_t = ds.rope_tables(T, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)
    step("tiny model: token-by-token decode, 4 ragged prompts, logits kept at every step")
    gen, kept = greedy_decode(model, up(toks), up(lens), N_NEW, cos_d, sin_d, keep_logits_at=tuple(range(T)))
    torch.cuda.synchronize()
    gen = gen.cpu().numpy()
    step("tiny model: oracle-composed reference, teacher-forced on the GPU's tokens")
    ref = _oracle_run(weights_h, toks, lens, gen)
    worst, decided = 0.0, 0
    for b, l in enumerate(lens):
        for j in range(N_NEW):
            t = int(l) - 1 + j
            r, dec = _check(ref[t, b], kept[t][b].cpu().numpy(), gen[b, j], f"greedy b={b} step={t}")
            worst, decided = max(worst, r), decided + dec
    print(f"[measured] decode loop vs oracle model: max err/bar = {worst:.5f}, max err/rms(row) = 2^{math.log2(max(_check.worst_rel_rms, 1e-30)):.2f}, "
          f"tokens decided by margin: {decided} of {len(lens) * N_NEW}", flush=True)
    assert decided >= len(lens) * N_NEW // 2
    step("tiny model: one-pass prefill + decode")
    gen2, logits2 = prefill_decode(model, up(toks), up(lens), N_NEW, cos_d, sin_d, keep_logits=True)
    torch.cuda.synchronize()
    assert np.array_equal(gen2.cpu().numpy(), gen)
    for b, l in enumerate(lens):
        for j in range(N_NEW):
            _check(ref[int(l) - 1 + j, b], logits2[j][b].cpu().numpy(), gen[b, j], f"prefill b={b} token={j}")
    step("tiny model: B=1 (prompt 1 alone) on a side stream")
    side = torch.cuda.Stream(device=DEV)
    g1, k1 = greedy_decode(model, up(toks[1:2]), up(lens[1:2]), N_NEW, cos_d, sin_d,
                           keep_logits_at=(int(lens[1]) - 1, int(lens[1]) + 2), stream=side)
    side.synchronize()
    assert np.array_equal(g1.cpu().numpy()[0], gen[1])
    for t, lg in k1.items():
        assert np.array_equal(lg[0].cpu().numpy().view(np.uint32), kept[t][1].cpu().numpy().view(np.uint32))
