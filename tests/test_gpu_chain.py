"""The calls of one Finch-C2 time-mix layer chained on the GPU with nothing in between but the interface
tensors: decay front (x -> y), fused prefill with LayerNorm partials (r, kbar, v, y, u' -> out, state),
fold, normalisation, key compression of the normalised rows -- against the chained oracles
decay_lora_input_numpy -> decay_logits_numpy -> finch_c2_oracle -> layernorm_heads_numpy ->
key_compress_oracle.  Every stage is compared on the GPU's own input to that stage (the interface
tensors are bf16, so each carries one rounding the oracle chain is given too), which isolates the
kernels; the last assertion compares the end of the chain with the oracle chain run from the start."""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from oracle import (decay_logits_numpy, decay_lora_input_numpy, finch_c2_oracle, key_compress_oracle,
                    layernorm_heads_numpy)
from paper_2407_12077_amd.workloads import (CONFIGS, make_decay_front_inputs, make_decay_lora_inputs, make_inputs,
                                            make_key_compress_inputs, make_uprime, round_to_bf16, scaled)

from gpu_util import BF16_OUT_ROUNDING, TOL_BF16, in_arena, max_norm_err, to_dev

pytestmark = pytest.mark.gpu
EPS = 1e-5


@pytest.mark.parametrize("B,T,H,staggered", [(2, 300, 4, True), (1, 1000, 8, False), (3, 70, 32, True)])
def test_layer_chain(gpu_device, B, T, H, staggered):
    cfg = scaled(CONFIGS[2], B=B, T=T, H=H)
    N, D, R, M = 64, H * 64, 64, B * T
    fi, inp, lo = make_decay_front_inputs(cfg, seed=61), make_inputs(cfg, seed=62), make_decay_lora_inputs(cfg, seed=63)
    up = make_uprime(cfg, seed=64)
    _, w_kd = make_key_compress_inputs(16, D, seed=65)
    rng = np.random.default_rng(66)
    gamma = (1.0 + 0.3 * rng.standard_normal(D)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(D)).astype(np.float32)
    bf, f32 = torch.bfloat16, torch.float32
    big = [to_dev(fi["x"], bf), to_dev(inp["r"], bf), to_dev(inp["k"], bf), to_dev(inp["v"], bf), to_dev(up, bf),
           torch.full((B, T, H, N), float("nan"), dtype=bf, device="cuda"),
           torch.full((B, T, D), float("nan"), dtype=bf, device="cuda")]
    if staggered:
        arena, big = in_arena(big)
    x, r, k, v, upd, out, ln = big
    y = torch.full((B, T, R), float("nan"), dtype=bf, device="cuda")
    mom = torch.full((B, H, T, 2), float("nan"), dtype=f32, device="cuda")
    mr = torch.full((B, T, 2), float("nan"), dtype=f32, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=f32, device="cuda")
    c = torch.full((M, D // 16), float("nan"), dtype=bf, device="cuda")
    T_ = lambda a: np.ascontiguousarray(a.T)
    wkv.wkv6_decay_lora_input_bf16(B, T, D, 32, R, x, to_dev(fi["x_prev"], bf), to_dev(fi["mu_x"], f32),
                                   to_dev(fi["lam_d"], f32), to_dev(T_(fi["A_d"]), bf), to_dev(T_(fi["B_d"]), bf),
                                   to_dev(T_(fi["A_omega"]), bf), y, wkv.WKV6_DTYPE_BF16)
    wkv.wkv6_finch_c2_prefill_lora_bf16(B, T, H, N, R, r, k, v, y, to_dev(lo["lam"], f32), to_dev(lo["b_omega"], bf),
                                        upd, None, out, mom, s_out)
    wkv.wkv6_layernorm_finalize(B, T, H, N, mom, EPS, mr)
    wkv.wkv6_layernorm_apply_bf16(B, T, H, N, out, mr, to_dev(gamma, f32), to_dev(beta, f32), ln, wkv.WKV6_DTYPE_BF16)
    wkv.wkv6_key_compress_bf16(M, D, ln, to_dev(w_kd, bf), c, wkv.WKV6_DTYPE_BF16)
    torch.cuda.synchronize()
    host = lambda t: t.float().cpu().numpy()
    y_g, o_g, ln_g, c_g = host(y), host(out), host(ln).reshape(B, T, H, N), host(c)
    bar = TOL_BF16 + BF16_OUT_ROUNDING
    # stage by stage, each oracle fed the GPU's own interface tensor
    y_ref = decay_lora_input_numpy(fi["x"], fi["x_prev"], fi["mu_x"], fi["lam_d"], fi["A_d"], fi["B_d"], fi["A_omega"])
    d_g = decay_logits_numpy(y_g, lo["lam"], lo["b_omega"], H, N).astype(np.float32)
    o_ref, s_ref = finch_c2_oracle(inp["r"], inp["k"], inp["v"], d_g, up, None)
    ln_ref, _, _ = layernorm_heads_numpy(o_g, gamma, beta, EPS)
    c_ref = key_compress_oracle(ln_g.reshape(M, D), w_kd)
    errs = {"y": max_norm_err(y_g, y_ref), "out": max_norm_err(o_g, o_ref), "state": max_norm_err(host(s_out), s_ref),
            "layernorm": max_norm_err(ln_g, ln_ref), "compressed": max_norm_err(c_g, c_ref)}
    print(f"chain B={B} T={T} H={H} staggered={staggered}: " + " ".join(f"{n}={e:.2e}" for n, e in errs.items()), flush=True)
    assert errs["y"] <= bar and errs["out"] <= bar and errs["layernorm"] <= bar and errs["compressed"] <= bar
    assert errs["state"] <= TOL_BF16
    # end to end: the oracle chain from x, with the interface roundings the GPU chain has (y, out, ln in bf16)
    d_o = decay_logits_numpy(round_to_bf16(y_ref.astype(np.float32)), lo["lam"], lo["b_omega"], H, N).astype(np.float32)
    o_o, _ = finch_c2_oracle(inp["r"], inp["k"], inp["v"], d_o, up, None)
    ln_o, _, _ = layernorm_heads_numpy(round_to_bf16(o_o.astype(np.float32)), gamma, beta, EPS)
    c_o = key_compress_oracle(round_to_bf16(ln_o.astype(np.float32)).reshape(M, D), w_kd)
    end = max_norm_err(c_g, c_o)
    print(f"  end of the chain against the oracle chain from x: {end:.2e}", flush=True)
    # four bf16 interface roundings and four kernels in a row: four times the single-stage bar
    assert end <= 4 * bar
