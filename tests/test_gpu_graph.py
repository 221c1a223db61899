"""A decode step captured in a HIP graph and replayed gives the bytes of the eager step, on every
replay, with eager work and synchronisations in between (the library allocates nothing, records no
memset, and only enqueues on the caller's stream, so it can be captured as it is)."""
import math

import numpy as np
import pytest
import torch

import detsynth as ds
from gpu_util import DEV, step, up

pytestmark = pytest.mark.gpu


def test_decoder_layer_graph_replays_match_eager():
    import paper_2602_00182_amd as d

    H, Hq, Hkv, D, F, Lmax, B = 1024, 8, 2, 128, 2816, 512, 5
    scale = float(np.float32(1.0 / math.sqrt(D)))
    g = lambda i, shape, std=0.03, mean=0.0: ds.normal_bf16_torch(9000 + i, shape, std, mean, DEV)
    tensors = [g(0, (H,), 0.1, 1.0), d.pack_qkv(g(1, (H, (Hq + 2 * Hkv) * D)), Hq, Hkv, D), d.pack_weight(g(2, (Hq * D, H))),
               g(3, (H,), 0.1, 1.0), d.pack_gate_up(g(4, (H, 2 * F))), d.pack_weight(g(5, (F, H)))]
    w = d.layer_weights(*tensors)
    cfg = d.layer_cfg(H, Hq, Hkv, D, F, Lmax, 1e-5, scale)
    cos_t, sin_t = ds.rope_tables(Lmax, D)
    cos_d, sin_d = up(cos_t), up(sin_t)
    x0 = g(6, (B, H), 1.0)
    k0 = g(7, (B, Hkv, Lmax, D), 1.0)
    v0 = g(8, (B, Hkv, Lmax, D), 1.0)
    pos = up(np.array([511, 300, 0, 255, 256], dtype=np.int32))
    ws = torch.empty(d.det_decoder_layer_workspace_bytes(cfg, B), dtype=torch.uint8, device=DEV)
    x, kc, vc = x0.clone(), k0.clone(), v0.clone()
    logits = torch.empty((B, 2048), dtype=torch.float32, device=DEV)
    lm = d.pack_weight(g(9, (H, 2048)))
    idx = torch.empty(B, dtype=torch.int32, device=DEV)

    def run():
        d.det_decoder_layer(w, cfg, x, kc, vc, pos, cos_d, sin_d, ws)
        d.det_gemm_bf16(x, lm, logits, 2048, H)
        d.det_argmax(logits, idx)

    step("eager layer + logits + argmax")
    run()
    torch.cuda.synchronize()
    want = (x.clone(), kc.clone(), vc.clone(), logits.clone(), idx.clone())

    def reset():
        x.copy_(x0)
        kc.copy_(k0)
        vc.copy_(v0)
        logits.zero_()
        idx.zero_()
        ws.fill_(0xAB)

    step("capture")
    side = torch.cuda.Stream(device=DEV)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        reset()
        run()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        run()
    for rep in range(5):
        step(f"replay {rep}")
        reset()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (x, kc, vc, logits, idx)
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep} differs from eager"
        # eager work between replays
        junk = torch.empty(1 << 20, dtype=torch.float32, device=DEV).normal_()
        assert junk.numel() > 0


def test_quantized_layer_and_sampling_graph_replays_match_eager():
    """The same for the quantized layer, the quantized lm_head behind the fused RMSNorm quantizer, and
    seeded sampling."""
    import paper_2602_00182_amd as d

    H, Hq, Hkv, D, F, Lmax, B, V = 1024, 8, 2, 128, 4096, 512, 5, 4096
    scale = float(np.float32(1.0 / math.sqrt(D)))
    g = lambda i, shape, std=0.03, mean=0.0: ds.normal_bf16_torch(9100 + i, shape, std, mean, DEV)
    tensors = [g(0, (H,), 0.1, 1.0), d.quant_pack_qkv(g(1, (H, (Hq + 2 * Hkv) * D)), Hq, Hkv, D),
               d.quant_pack_weight(g(2, (Hq * D, H))), g(3, (H,), 0.1, 1.0), d.quant_pack_gate_up(g(4, (H, 2 * F))),
               d.quant_pack_weight(g(5, (F, H)))]
    w = d.layer_weights(*tensors)
    cfg = d.layer_cfg(H, Hq, Hkv, D, F, Lmax, 1e-5, scale)
    cos_t, sin_t = ds.rope_tables(Lmax, D)
    cos_d, sin_d = up(cos_t), up(sin_t)
    x0 = g(6, (B, H), 1.0)
    k0 = g(7, (B, Hkv, Lmax, D), 1.0)
    v0 = g(8, (B, Hkv, Lmax, D), 1.0)
    pos = up(np.array([511, 300, 0, 255, 256], dtype=np.int32))
    ws = torch.empty(d.det_qdecoder_layer_workspace_bytes(cfg, B), dtype=torch.uint8, device=DEV)
    x, kc, vc = x0.clone(), k0.clone(), v0.clone()
    wn = g(10, (H,), 0.1, 1.0)
    lm = d.quant_pack_weight(g(9, (H, V)))
    codes = torch.empty((B, H), dtype=torch.int8, device=DEV)
    scales = torch.empty(d.det_quant_act_scales_bytes(B, H) // 4, dtype=torch.float32, device=DEV)
    logits = torch.empty((B, V), dtype=torch.float32, device=DEV)
    tok = torch.empty(B, dtype=torch.int32, device=DEV)
    ids = up(np.arange(B, dtype=np.int32))

    def run():
        d.det_qdecoder_layer(w, cfg, x, kc, vc, pos, None, cos_d, sin_d, ws)
        d.det_rmsnorm_quant_q8(x, wn, codes, scales, 1e-5)
        d.det_qgemm_w4a8(codes, scales, lm, logits, V)
        d.det_sample(logits, 0.8, 40, 0.95, 77, ids, pos, tok)

    step("eager quantized layer + logits + sampling")
    run()
    torch.cuda.synchronize()
    want = (x.clone(), kc.clone(), vc.clone(), logits.clone(), tok.clone())

    def reset():
        x.copy_(x0)
        kc.copy_(k0)
        vc.copy_(v0)
        logits.zero_()
        tok.zero_()
        codes.zero_()
        ws.fill_(0xAB)

    step("capture")
    side = torch.cuda.Stream(device=DEV)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        reset()
        run()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        run()
    for rep in range(4):
        step(f"replay {rep}")
        reset()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip((x, kc, vc, logits, tok), want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep} differs from eager"
        junk = torch.empty(1 << 20, dtype=torch.float32, device=DEV).normal_()
        assert junk.numel() > 0
