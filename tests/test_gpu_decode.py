"""Greedy decode of a random-init 8-layer Llama-style model: token streams (and logits bytes) of a
prompt are identical whether it runs alone or batched at 8 / 32 / 64 (the paper's end-to-end
determinism experiments, section 6.7, with batch composition as the perturbation)."""
import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, step, up

pytestmark = pytest.mark.gpu

H, HQ, HKV, D, F, V, NL = 2048, 16, 4, 128, 5632, 32000, 8
N_PROMPTS, N_NEW = 64, 128


@pytest.fixture(scope="module")
def weights():
    s = ds.tensor_seed(5, 0)
    g = lambda i, shape, std=0.02, mean=0.0: ds.normal_bf16_torch(s + i, shape, std, mean, DEV)
    layers = []
    for l in range(NL):
        o = 10 + 10 * l
        layers.append(dict(norm1=g(o, (H,), 0.0, 1.0), wqkv=g(o + 1, (H, (HQ + 2 * HKV) * D)),
                           wo=g(o + 2, (HQ * D, H)), norm2=g(o + 3, (H,), 0.0, 1.0), wgu=g(o + 4, (H, 2 * F)),
                           wdown=g(o + 5, (F, H))))
    return dict(embed=g(1, (V, H), 1.0), lm_head=g(2, (H, V)), final_norm=g(3, (H,), 0.0, 1.0), layers=layers)


@pytest.fixture(scope="module")
def model(weights):
    from paper_2602_00182_amd.decode import DecodeModel, ModelCfg

    return DecodeModel(ModelCfg(H, HQ, HKV, D, F, V, NL), weights)


@pytest.fixture(scope="module")
def qmodel(weights):
    from paper_2602_00182_amd.decode import DecodeModel, ModelCfg

    return DecodeModel(ModelCfg(H, HQ, HKV, D, F, V, NL), weights, quantized=True)


@pytest.fixture(scope="module")
def prompts():
    lens = ds.uniform_int(ds.tensor_seed(5, 500), (N_PROMPTS,), 16, 512)
    toks = ds.uniform_int(ds.tensor_seed(5, 501), (N_PROMPTS, 512), 0, V - 1)
    return toks, lens


def test_token_streams_identical_across_batchings(model, prompts):
    from paper_2602_00182_amd.decode import greedy_decode

    toks, lens = prompts
    cos_t, sin_t = ds.rope_tables(512 + N_NEW, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)

    def run(ids, keep=()):
        ids = list(ids)
        gen, kept = greedy_decode(model, up(toks[ids]), up(lens[ids]), N_NEW, cos_d, sin_d, keep_logits_at=keep)
        torch.cuda.synchronize()
        return gen.cpu().numpy(), {t: l.cpu().numpy() for t, l in kept.items()}

    keep = (15, 100, 300, 500, 600)
    step("greedy decode, all 64 prompts in one batch")
    full, full_logits = run(range(64), keep)
    assert full.shape == (64, N_NEW)
    assert len({tuple(r) for r in full}) > 32, "streams should differ between prompts"
    step("greedy decode, same batch again")
    again, again_logits = run(range(64), keep)
    assert np.array_equal(full, again)
    for t in keep:
        if t in full_logits:
            assert np.array_equal(full_logits[t].view(np.uint32), again_logits[t].view(np.uint32))
    for bs in (32, 8):
        for start in (0, 64 - bs):
            ids = list(range(start, start + bs))
            step(f"greedy decode, batch of {bs} starting at prompt {start}")
            part, part_logits = run(ids, keep)
            assert np.array_equal(part, full[ids]), f"token streams differ at batch size {bs}"
            for t, lg in part_logits.items():
                # rows still inside their own run at step t carry the same logits bytes
                live = [j for j, i in enumerate(ids) if t < lens[i] + N_NEW - 1]
                assert np.array_equal(lg[live].view(np.uint32), full_logits[t][[ids[j] for j in live]].view(np.uint32))
    step("greedy decode, shuffled batch of 32 drawn from all prompts")
    ids = np.random.default_rng(3).permutation(64)[:32].tolist()
    part, _ = run(ids)
    assert np.array_equal(part, full[ids])
    for i in (0, 17, 40, 63):
        step(f"greedy decode, prompt {i} alone")
        alone, alone_logits = run([i], keep)
        assert np.array_equal(alone[0], full[i]), f"prompt {i}: alone differs from batched"
        for t, lg in alone_logits.items():
            assert np.array_equal(lg[0].view(np.uint32), full_logits[t][i].view(np.uint32))


def test_seeded_sampling_streams_identical_across_batchings(model, prompts):
    """Seeded top-k / top-p decoding (section 6.6): for a fixed (seed, policy) a prompt's token stream
    is the same alone and in any batch, and changes with the seed."""
    from paper_2602_00182_amd.decode import SamplingPolicy, greedy_decode

    toks, lens = prompts
    n_new = 48
    cos_t, sin_t = ds.rope_tables(512 + n_new, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)

    def run(ids, seed=2026):
        ids = list(ids)
        pol = SamplingPolicy(0.8, 50, 0.95, seed, up(np.asarray(ids, dtype=np.int32)))
        gen, _ = greedy_decode(model, up(toks[ids]), up(lens[ids]), n_new, cos_d, sin_d, policy=pol)
        torch.cuda.synchronize()
        return gen.cpu().numpy()

    step("sampled decode, 16 prompts in one batch")
    full = run(range(16))
    step("sampled decode, same batch again")
    assert np.array_equal(run(range(16)), full)
    step("sampled decode, batch of 4")
    assert np.array_equal(run(range(8, 12)), full[8:12])
    step("sampled decode, prompt 5 alone")
    assert np.array_equal(run([5])[0], full[5])
    step("sampled decode, another seed")
    other = run(range(16), seed=2027)
    assert not np.array_equal(other, full)
    greedy, _ = greedy_decode(model, up(toks[:16]), up(lens[:16]), n_new, cos_d, sin_d)
    assert not np.array_equal(greedy.cpu().numpy(), full)


def test_prefill_rows_match_token_by_token(model, prompts):
    """Batch-invariant prefill: all prompt tokens of a batch go through each layer in one call (rows
    that name their cache slot) and the result is, byte for byte, that of feeding them one step at a
    time: same generated tokens, same logits, same KV-cache contents."""
    from paper_2602_00182_amd.decode import greedy_decode, prefill_decode

    toks, lens = prompts
    n_new = 24
    cos_t, sin_t = ds.rope_tables(512 + n_new, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)
    ids = list(range(8, 24))
    lens_b = lens[ids]
    keep = tuple(int(l) - 1 + j for l in lens_b for j in (0, 5, n_new - 1))
    step("token-by-token decode of 16 prompts")
    ref, ref_logits = greedy_decode(model, up(toks[ids]), up(lens_b), n_new, cos_d, sin_d, keep_logits_at=keep)
    torch.cuda.synchronize()
    step("prefill + decode of the same 16 prompts")
    gen, logits = prefill_decode(model, up(toks[ids]), up(lens_b), n_new, cos_d, sin_d, keep_logits=True)
    torch.cuda.synchronize()
    assert np.array_equal(gen.cpu().numpy(), ref.cpu().numpy())
    for b, l in enumerate(lens_b):
        for j in (0, 5, n_new - 1):
            a = logits[j][b].cpu().numpy().view(np.uint32)
            r = ref_logits[int(l) - 1 + j][b].cpu().numpy().view(np.uint32)
            assert np.array_equal(a, r), f"logits differ: prompt {ids[b]}, generated token {j}"
    step("prefill + decode, prompt 13 alone and a batch of 4")
    alone, _ = prefill_decode(model, up(toks[[13]]), up(lens[[13]]), n_new, cos_d, sin_d)
    assert np.array_equal(alone.cpu().numpy()[0], ref.cpu().numpy()[13 - 8])
    four, _ = prefill_decode(model, up(toks[[20, 9, 13, 16]]), up(lens[[20, 9, 13, 16]]), n_new, cos_d, sin_d)
    assert np.array_equal(four.cpu().numpy(), ref.cpu().numpy()[[12, 1, 5, 8]])


def test_receipts_identical_across_batchings(model, prompts, orc):
    """The paper's end-to-end check (section 6.7) in its own terms: the per-execution digest
    SHA256(prompt || logits || tokens) of a prompt is the same whether it runs alone or in any batch,
    equals the oracle's hash of the same downloaded bytes, and differs between prompts."""
    from paper_2602_00182_amd.decode import commit_outputs, prefill_decode

    toks, lens = prompts
    n_new = 12
    cos_t, sin_t = ds.rope_tables(512 + n_new, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)

    def run(ids):
        ids = list(ids)
        p, l = up(toks[ids]), up(lens[ids])
        gen, logits = prefill_decode(model, p, l, n_new, cos_d, sin_d, keep_logits=True)
        torch.cuda.synchronize()
        return commit_outputs(p, l, logits, gen), gen.cpu().numpy(), [x.cpu().numpy() for x in logits]

    step("receipts, 12 prompts in one batch")
    ids = list(range(30, 42))
    full, gen, logits = run(ids)
    assert len(set(full)) == len(full), "digests should differ between prompts"
    for b, i in enumerate(ids):
        want = orc.commit_sha256(toks[i, :lens[i]].astype("<i4").tobytes(),
                                 np.stack([x[b] for x in logits]).astype("<f4").tobytes(),
                                 gen[b].astype("<i4").tobytes())
        assert full[b] == want
    step("receipts, the same batch again")
    assert run(ids)[0] == full
    step("receipts, batch of 3 and one prompt alone")
    assert run([41, 30, 35])[0] == [full[11], full[0], full[5]]
    assert run([33])[0] == [full[3]]


def test_quantized_model_streams_across_batchings_and_prefill(qmodel, model, prompts):
    """The same model with every projection block-quantized (4-bit weights, 8-bit activations): token
    streams and logits bytes of a prompt are identical alone, in a batch of 12, in another order, and
    between token-by-token decoding and one-pass prefill; they differ from the bf16 model's."""
    from paper_2602_00182_amd.decode import greedy_decode, prefill_decode

    toks, lens = prompts
    n_new = 20
    cos_t, sin_t = ds.rope_tables(512 + n_new, D, 5.0e5)
    cos_d, sin_d = up(cos_t), up(sin_t)
    ids = list(range(20, 32))
    step("quantized model: prefill + decode of 12 prompts")
    full, full_logits = prefill_decode(qmodel, up(toks[ids]), up(lens[ids]), n_new, cos_d, sin_d, keep_logits=True)
    torch.cuda.synchronize()
    full = full.cpu().numpy()
    assert len({tuple(r) for r in full}) > 6
    step("quantized model: token-by-token decode of 4 of them")
    sub = [3, 0, 7, 11]
    sub_ids = [ids[i] for i in sub]
    keep = tuple(int(lens[i]) - 1 + j for i in sub_ids for j in (0, n_new - 1))
    tbt, tbt_logits = greedy_decode(qmodel, up(toks[sub_ids]), up(lens[sub_ids]), n_new, cos_d, sin_d, keep_logits_at=keep)
    torch.cuda.synchronize()
    assert np.array_equal(tbt.cpu().numpy(), full[sub])
    for row, i in enumerate(sub_ids):
        for j in (0, n_new - 1):
            a = tbt_logits[int(lens[i]) - 1 + j][row].cpu().numpy().view(np.uint32)
            b = full_logits[j][sub[row]].cpu().numpy().view(np.uint32)
            assert np.array_equal(a, b), f"logits differ: prompt {i}, generated token {j}"
    step("quantized model: one prompt alone, prefill")
    alone, _ = prefill_decode(qmodel, up(toks[[ids[5]]]), up(lens[[ids[5]]]), n_new, cos_d, sin_d)
    assert np.array_equal(alone.cpu().numpy()[0], full[5])
    step("bf16 model on the same prompts")
    ref, _ = prefill_decode(model, up(toks[ids]), up(lens[ids]), n_new, cos_d, sin_d)
    assert not np.array_equal(ref.cpu().numpy(), full)
