"""Greedy decode loop over libdetinfer (host orchestration only: every step runs in the library's
kernels, on one stream, with no host round trip inside the loop).

One step, for B sequences at step t (the paper's section 6.6: greedy decoding in a fixed order):
    token select -> embedding gather -> L x decoder layer -> final RMSNorm -> lm_head GEMM (fp32
    logits) -> argmax.
greedy_decode feeds prompts through the same step one token at a time; prefill_decode pushes all
prompt tokens of all sequences through each layer in one call (rows that name their cache slot) and
then decodes.  Either way a sequence's bytes are those of the single-sequence, token-by-token run,
whatever batch it sits in."""
from __future__ import annotations

import contextlib
import os
from dataclasses import dataclass

import torch

from . import api


@dataclass
class ModelCfg:
    H: int
    Hq: int
    Hkv: int
    D: int
    F: int
    V: int
    n_layers: int
    eps: float = 1e-5
    scale: float = 0.08838834764831845  # 1/sqrt(128)


class DecodeModel:
    """Weights of a Llama-style decoder, packed for det_gemm_bf16, or with quantized=True block-quantized
    to 4 bits and packed for det_qgemm_w4a8 (every projection, the lm_head included; embedding and norm
    weights stay bf16).

    `weights` holds logical row-major bf16 tensors on the GPU:
        embed [V,H], lm_head [H,V], final_norm [H], and per layer i:
        layers[i] = dict(norm1 [H], wqkv [H,(Hq+2Hkv)D], wo [Hq*D,H], norm2 [H], wgu [H,2F], wdown [F,H])
    """

    def __init__(self, cfg: ModelCfg, weights: dict, quantized: bool = False):
        self.cfg = cfg
        self.quantized = quantized
        pack = api.quant_pack_weight if quantized else api.pack_weight
        pack_gu = api.quant_pack_gate_up if quantized else api.pack_gate_up
        self.embed = weights["embed"].contiguous()
        self.final_norm = weights["final_norm"].contiguous()
        self.lm_head = pack(weights["lm_head"])
        self.layers = []
        for lw in weights["layers"]:
            wqkv = (api.quant_pack_qkv if quantized else api.pack_qkv)(lw["wqkv"], cfg.Hq, cfg.Hkv, cfg.D)
            packed = dict(norm1=lw["norm1"].contiguous(), wqkv=wqkv,
                          wo=pack(lw["wo"]), norm2=lw["norm2"].contiguous(),
                          wgu=pack_gu(lw["wgu"]), wdown=pack(lw["wdown"]))
            struct = api.layer_weights(packed["norm1"], packed["wqkv"], packed["wo"], packed["norm2"],
                                       packed["wgu"], packed["wdown"])
            self.layers.append((packed, struct))

    def layer_workspace_bytes(self, lcfg, rows: int) -> int:
        if self.quantized:
            return api.det_qdecoder_layer_workspace_bytes(lcfg, rows)
        return api.det_decoder_layer_workspace_bytes(lcfg, rows)

    def layer(self, struct, lcfg, x, kcache, vcache, positions, slots, rope_cos, rope_sin, ws, stream=None):
        """One decoder layer on rows x; slots None: row r is the sequence in cache slot r."""
        if self.quantized:
            api.det_qdecoder_layer(struct, lcfg, x, kcache, vcache, positions, slots, rope_cos, rope_sin, ws, stream)
        elif slots is None:
            api.det_decoder_layer(struct, lcfg, x, kcache, vcache, positions, rope_cos, rope_sin, ws, stream)
        else:
            api.det_decoder_layer_rows(struct, lcfg, x, kcache, vcache, positions, slots, rope_cos, rope_sin, ws,
                                       stream)

    def new_state(self, B: int, Lmax: int, rope_cos: torch.Tensor, rope_sin: torch.Tensor):
        return DecodeState(self, B, Lmax, rope_cos, rope_sin)


class DecodeState:
    """KV caches, workspace and step buffers for B sequences of up to Lmax tokens."""

    def __init__(self, model: DecodeModel, B: int, Lmax: int, rope_cos, rope_sin):
        c = model.cfg
        dev = model.embed.device
        self.model, self.B, self.Lmax = model, B, Lmax
        self.lcfg = api.layer_cfg(c.H, c.Hq, c.Hkv, c.D, c.F, Lmax, c.eps, c.scale)
        if rope_cos.shape != (Lmax, c.D // 2):
            raise ValueError("rope tables must be [Lmax, D/2]")
        self.rope_cos, self.rope_sin = rope_cos, rope_sin
        self.kcache = [torch.zeros((B, c.Hkv, Lmax, c.D), dtype=torch.bfloat16, device=dev)
                       for _ in range(c.n_layers)]
        self.vcache = [torch.zeros_like(k) for k in self.kcache]
        self.ws = torch.empty(model.layer_workspace_bytes(self.lcfg, B), dtype=torch.uint8, device=dev)
        self.x = torch.empty((B, c.H), dtype=torch.bfloat16, device=dev)
        self.xn = torch.empty((B, c.H), dtype=torch.bfloat16, device=dev)
        if model.quantized:  # the final norm's output as activation codes for the quantized lm_head
            self.xn_codes = torch.empty((B, c.H), dtype=torch.int8, device=dev)
            self.xn_scales = torch.empty(api.det_quant_act_scales_bytes(B, c.H) // 4, dtype=torch.float32, device=dev)
        self.logits = torch.empty((B, c.V), dtype=torch.float32, device=dev)
        self.tokens = torch.empty(B, dtype=torch.int32, device=dev)
        self.positions = torch.empty(B, dtype=torch.int32, device=dev)

    def forward(self, stream=None):
        """One decode step on self.tokens / self.positions; leaves fp32 logits in self.logits."""
        m, c = self.model, self.model.cfg
        api.det_embed_gather(m.embed, self.tokens, self.x, stream)
        for i, (_, struct) in enumerate(m.layers):
            m.layer(struct, self.lcfg, self.x, self.kcache[i], self.vcache[i], self.positions, None, self.rope_cos,
                    self.rope_sin, self.ws, stream)
        self.head(stream)

    def head(self, stream=None):
        """Final RMSNorm and lm_head on self.x; fp32 logits in self.logits."""
        m, c = self.model, self.model.cfg
        if m.quantized:
            api.det_rmsnorm_quant_q8(self.x, m.final_norm, self.xn_codes, self.xn_scales, c.eps, stream)
            api.det_qgemm_w4a8(self.xn_codes, self.xn_scales, m.lm_head, self.logits, c.V, stream)
        else:
            api.det_rmsnorm_gemm_bf16(self.x, m.final_norm, c.eps, m.lm_head, self.xn, self.logits, c.V, stream)


@dataclass
class SamplingPolicy:
    """Seeded decode policy: det_sample with these parameters instead of det_argmax.  `seq_ids`
    [B] int32 on the device names each sequence, so that its random stream does not depend on the
    batch it runs in."""
    temperature: float
    top_k: int
    top_p: float
    seed: int
    seq_ids: torch.Tensor


def greedy_decode(model: DecodeModel, prompts: torch.Tensor, prompt_lens: torch.Tensor, n_new: int,
                  rope_cos: torch.Tensor, rope_sin: torch.Tensor, keep_logits_at=(), stream=None,
                  policy: SamplingPolicy | None = None):
    """Runs B sequences together.  prompts [B, Tp] int32 (padded), prompt_lens [B] int32.
    With `policy`, tokens are drawn by det_sample (step = position) instead of det_argmax.

    Returns (generated [B, n_new] int32 on the device, {step: logits [B, V] fp32 clone}).
    Step t feeds prompt token t while t < len, else the token sampled at step t-1; sequence b's
    generated tokens are the samples of steps len_b-1 .. len_b+n_new-2."""
    # allocations, clones and the final gather are torch operations: they follow torch's current stream,
    # which is made the library's stream for the whole run
    with torch.cuda.stream(stream) if stream is not None else contextlib.nullcontext():
        return _greedy_decode(model, prompts, prompt_lens, n_new, rope_cos, rope_sin, keep_logits_at, stream, policy)


def _greedy_decode(model, prompts, prompt_lens, n_new, rope_cos, rope_sin, keep_logits_at, stream, policy):
    B, Tp = prompts.shape
    lens_host = prompt_lens.cpu()
    T = int(lens_host.max()) + n_new - 1
    if rope_cos.shape[0] < T:
        raise ValueError("rope tables shorter than the run")
    st = model.new_state(B, T, rope_cos[:T].contiguous(), rope_sin[:T].contiguous())
    dev = prompts.device
    sampled = torch.zeros((T, B), dtype=torch.int32, device=dev)
    history = torch.zeros((B, T), dtype=torch.int32, device=dev)
    kept = {}
    for t in range(T):
        last = sampled[t - 1] if t > 0 else sampled[0]
        api.det_next_token(prompts, prompt_lens, last, st.tokens, st.positions, history, t, stream)
        st.forward(stream)
        if policy is None:
            api.det_argmax(st.logits, sampled[t], stream)
        else:
            api.det_sample(st.logits, policy.temperature, policy.top_k, policy.top_p, policy.seed, policy.seq_ids,
                           st.positions, sampled[t], stream)
        if t in keep_logits_at:
            kept[t] = st.logits.clone()
    idx = (lens_host.to(torch.int64) - 1)[:, None] + torch.arange(n_new)[None, :]
    gen = sampled.t().contiguous().gather(1, idx.to(dev))
    return gen, kept


def _select(policy, logits, positions, out, stream):
    if policy is None:
        api.det_argmax(logits, out, stream)
    else:
        api.det_sample(logits, policy.temperature, policy.top_k, policy.top_p, policy.seed, policy.seq_ids,
                       positions, out, stream)


def prefill_decode(model: DecodeModel, prompts: torch.Tensor, prompt_lens: torch.Tensor, n_new: int,
                   rope_cos: torch.Tensor, rope_sin: torch.Tensor, stream=None,
                   policy: SamplingPolicy | None = None, keep_logits: bool = False):
    """Same results as greedy_decode, with the prompts processed in one pass.

    Prefill: row r is token prompts[b, p] with position p and cache slot b, for every b and p < len_b
    (R = sum of the lengths).  Each layer writes all keys and values first and then lets row r attend
    to positions 0..p of its slot, which is exactly what the token-by-token run computes for that
    token.  The last row of each sequence goes on to the final norm, lm_head and token selection.
    Decode: sequence b then advances from its own position len_b, one token per step.

    Returns (generated [B, n_new] int32 on the device, list of n_new logits clones [B, V] if
    keep_logits else [])."""
    with torch.cuda.stream(stream) if stream is not None else contextlib.nullcontext():
        return _prefill_decode(model, prompts, prompt_lens, n_new, rope_cos, rope_sin, stream, policy, keep_logits)


def _prefill_decode(model, prompts, prompt_lens, n_new, rope_cos, rope_sin, stream, policy, keep_logits):
    c = model.cfg
    B, _ = prompts.shape
    dev = prompts.device
    lens_host = prompt_lens.cpu().to(torch.int64)
    T = int(lens_host.max()) + n_new - 1
    if rope_cos.shape[0] < T:
        raise ValueError("rope tables shorter than the run")
    st = model.new_state(B, T, rope_cos[:T].contiguous(), rope_sin[:T].contiguous())

    # row tables, built on the host once (integer bookkeeping only)
    slots_h = torch.repeat_interleave(torch.arange(B), lens_host)
    starts = torch.cumsum(lens_host, 0) - lens_host
    pos_h = torch.arange(int(lens_host.sum())) - torch.repeat_interleave(starts, lens_host)
    R = int(lens_host.sum())
    row_tokens = prompts.cpu()[slots_h, pos_h].to(torch.int32).to(dev)
    row_slots = slots_h.to(torch.int32).to(dev)
    row_pos = pos_h.to(torch.int32).to(dev)
    last_rows = (starts + lens_host - 1).to(torch.int32).to(dev)

    xr = torch.empty((R, c.H), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(model.layer_workspace_bytes(st.lcfg, R), dtype=torch.uint8, device=dev)
    api.det_embed_gather(model.embed, row_tokens, xr, stream)
    for i, (_, struct) in enumerate(model.layers):
        model.layer(struct, st.lcfg, xr, st.kcache[i], st.vcache[i], row_pos, row_slots, st.rope_cos, st.rope_sin, ws,
                    stream)
    api.det_embed_gather(xr, last_rows, st.x, stream)  # row gather: the last token of each sequence
    st.head(stream)

    gen = torch.zeros((n_new, B), dtype=torch.int32, device=dev)
    kept = []
    base_pos = (lens_host - 1).to(torch.int32).to(dev)   # position of each sequence's last prompt token
    st.positions.copy_(base_pos)
    _select(policy, st.logits, st.positions, gen[0], stream)
    if keep_logits:
        kept.append(st.logits.clone())
    for j in range(1, n_new):
        api.det_decode_advance(gen[j - 1], base_pos, j, st.tokens, st.positions, stream)
        st.forward(stream)
        _select(policy, st.logits, st.positions, gen[j], stream)
        if keep_logits:
            kept.append(st.logits.clone())
    return gen.t().contiguous(), kept


def commit_outputs(prompts: torch.Tensor, prompt_lens: torch.Tensor, logits_steps, generated: torch.Tensor):
    """Per-sequence output commitment, the hash the paper records for every execution (section 6.7):
    SHA256(prompt || logits || tokens) with prompt = the sequence's own prompt ids (int32,
    little-endian), logits = the fp32 logits rows of its generated steps in step order, tokens = its
    generated ids (int32).  `logits_steps` is the list prefill_decode(keep_logits=True) returns.
    Downloads to host memory and hashes there (det_commit_sha256).  Returns a list of 32-byte digests;
    together with api.det_fingerprint() they are what a receipt would carry for the run."""
    B = prompts.shape[0]
    lens = prompt_lens.cpu().tolist()
    p_host = prompts.to(torch.int32).cpu().contiguous()
    g_host = generated.to(torch.int32).cpu().contiguous()
    l_host = torch.stack(list(logits_steps)).permute(1, 0, 2).contiguous().cpu()  # [B, steps, V]
    # one SHA-256 chain per sequence, the chains on separate host threads (the call releases the GIL)
    from concurrent.futures import ThreadPoolExecutor

    def one(b):
        return api.det_commit_sha256(p_host[b, :lens[b]].contiguous(), l_host[b], g_host[b])

    with ThreadPoolExecutor(max_workers=min(B, os.cpu_count() or 1, 16)) as pool:
        return list(pool.map(one, range(B)))
