"""The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a serving loop can capture them in a HIP graph.  Each graph is replayed
several times, with eager work and synchronisations in between, and every replay is compared
with the eager result."""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from paper_2407_12077_amd.workloads import CONFIGS, make_inputs, scaled

from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def test_decode_steps_in_a_graph(gpu_device):
    cfg = scaled(CONFIGS[4], B=8, T=4, H=4)
    inp = make_inputs(cfg)
    B, T, H, N = inp["r"].shape
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in "rkvx")
    u = to_dev(inp["u"], torch.float32)
    s0 = to_dev(inp["state_in"], torch.float32)
    steps = [[a[:, t].contiguous() for a in (r, k, v, x)] for t in range(T)]

    def run(state, outs):
        for t in range(T):
            wkv.wkv6_decode_bf16(B, H, N, *steps[t], u, state, outs[t])

    state_e = s0.clone()
    outs_e = [torch.empty((B, H, N), dtype=torch.bfloat16, device="cuda") for _ in range(T)]
    run(state_e, outs_e)
    torch.cuda.synchronize()

    state_g = s0.clone()
    outs_g = [torch.empty((B, H, N), dtype=torch.bfloat16, device="cuda") for _ in range(T)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(state_g, outs_g)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(state_g, outs_g)
    for replay in range(3):
        state_g.copy_(s0)                         # eager work between the replays
        for o in outs_g:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(state_g, state_e), replay
        for a, b in zip(outs_g, outs_e):
            assert torch.equal(a, b), replay


def test_prefill_in_a_graph(gpu_device):
    cfg = scaled(CONFIGS[4], B=2, T=300, H=3)
    inp = make_inputs(cfg)
    B, T, H, N = inp["r"].shape
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in "rkvx")
    u = to_dev(inp["u"], torch.float32)
    s_in = to_dev(inp["state_in"], torch.float32)
    out_e = torch.empty((B, T, H, N), dtype=torch.bfloat16, device="cuda")
    s_e = torch.empty_like(s_in)
    wkv.wkv6_prefill_bf16(B, T, H, N, r, k, v, x, u, s_in, out_e, s_e)
    torch.cuda.synchronize()

    out_g = torch.empty_like(out_e)
    s_g = torch.empty_like(s_in)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        wkv.wkv6_prefill_bf16(B, T, H, N, r, k, v, x, u, s_in, out_g, s_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        wkv.wkv6_prefill_bf16(B, T, H, N, r, k, v, x, u, s_in, out_g, s_g)
    for replay in range(3):
        out_g.fill_(float("nan"))
        s_g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e) and torch.equal(s_g, s_e), replay


def test_fused_layer_pieces_in_a_graph(gpu_device):
    """The Finch-C2 prefill with the decay logits formed in the kernel and the LayerNorm partials,
    their fold, and a key compression of as many tokens: three kernels captured as one graph."""
    from paper_2407_12077_amd.workloads import make_decay_lora_inputs, make_key_compress_inputs, make_uprime
    cfg = scaled(CONFIGS[4], B=3, T=130, H=4)
    inp = make_inputs(cfg)
    inp["uprime"] = make_uprime(cfg)
    inp.update(make_decay_lora_inputs(cfg))
    B, T, H, N = inp["r"].shape
    r, k, v, up, y, bo = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "uprime", "y", "b_omega"))
    lam, s_in = to_dev(inp["lam"], torch.float32), to_dev(inp["state_in"], torch.float32)
    kx, kw = make_key_compress_inputs(B * T, 256)
    hx, w_kd = to_dev(kx, torch.bfloat16), to_dev(kw, torch.bfloat16)

    def fresh():
        return (torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda"),
                torch.full((B, H, T, 2), float("nan"), dtype=torch.float32, device="cuda"),
                torch.full((B, T, 2), float("nan"), dtype=torch.float32, device="cuda"),
                torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda"),
                torch.full((B * T, 16), float("nan"), dtype=torch.bfloat16, device="cuda"))

    def run(bufs):
        out, mom, mr, s_out, c = bufs
        wkv.wkv6_finch_c2_prefill_lora_bf16(B, T, H, N, 64, r, k, v, y, lam, bo, up, s_in, out, mom, s_out)
        wkv.wkv6_layernorm_finalize(B, T, H, N, mom, 1e-5, mr)
        wkv.wkv6_key_compress_bf16(B * T, 256, hx, w_kd, c, wkv.WKV6_DTYPE_BF16)

    eager = fresh()
    run(eager)
    torch.cuda.synchronize()
    captured = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(captured)                             # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(captured)
    for replay in range(3):
        for t in captured:
            t.fill_(float("nan"))                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(captured, eager):
            assert torch.equal(a, b), replay


def test_layer_chain_in_a_graph(gpu_device):
    """All five calls of a Finch-C2 time-mix layer (decay front, fused prefill with LayerNorm partials,
    fold, normalisation, key compression) captured as one graph."""
    from paper_2407_12077_amd.workloads import (make_decay_front_inputs, make_decay_lora_inputs,
                                                make_key_compress_inputs, make_uprime)
    cfg = scaled(CONFIGS[2], B=2, T=200, H=4)
    B, T, H, N = cfg.B, cfg.T, cfg.H, cfg.N
    D, M = H * N, B * T
    fi, inp, lo = make_decay_front_inputs(cfg), make_inputs(cfg), make_decay_lora_inputs(cfg)
    bf, f32 = torch.bfloat16, torch.float32
    x, xp = to_dev(fi["x"], bf), to_dev(fi["x_prev"], bf)
    mu, lam_d = to_dev(fi["mu_x"], f32), to_dev(fi["lam_d"], f32)
    a_d, b_d, a_w = (to_dev(np.ascontiguousarray(fi[n].T), bf) for n in ("A_d", "B_d", "A_omega"))
    r, k, v, up = (to_dev(a, bf) for a in (inp["r"], inp["k"], inp["v"], make_uprime(cfg)))
    lam_w, b_w = to_dev(lo["lam"], f32), to_dev(lo["b_omega"], bf)
    gamma, beta = torch.ones(D, device="cuda"), torch.zeros(D, device="cuda")
    w_kd = to_dev(make_key_compress_inputs(16, D)[1], bf)

    def fresh():
        nan = lambda shape, dt: torch.full(shape, float("nan"), dtype=dt, device="cuda")
        return (nan((B, T, 64), bf), nan((B, T, H, N), bf), nan((B, H, T, 2), f32), nan((B, T, 2), f32),
                nan((B, H, N, N), f32), nan((B, T, D), bf), nan((M, D // 16), bf))

    def run(bufs):
        y, out, mom, mr, s_out, ln, c = bufs
        wkv.wkv6_decay_lora_input_bf16(B, T, D, 32, 64, x, xp, mu, lam_d, a_d, b_d, a_w, y, wkv.WKV6_DTYPE_BF16)
        wkv.wkv6_finch_c2_prefill_lora_bf16(B, T, H, N, 64, r, k, v, y, lam_w, b_w, up, None, out, mom, s_out)
        wkv.wkv6_layernorm_finalize(B, T, H, N, mom, 1e-5, mr)
        wkv.wkv6_layernorm_apply_bf16(B, T, H, N, out, mr, gamma, beta, ln, wkv.WKV6_DTYPE_BF16)
        wkv.wkv6_key_compress_bf16(M, D, ln, w_kd, c, wkv.WKV6_DTYPE_BF16)

    eager = fresh()
    run(eager)
    torch.cuda.synchronize()
    assert all(torch.isfinite(t.float()).all() for t in eager)
    captured = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(captured)                             # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(captured)
    for replay in range(3):
        for t in captured:
            t.fill_(float("nan"))                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(captured, eager):
            assert torch.equal(a, b), replay
