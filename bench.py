#!/usr/bin/env python3
"""Benchmark of the WKV6 prefill hot path on one MI355X.

A "step" is one `wkv6_prefill_bf16` call: one layer's WKV6 recurrence over one batch of
synthetic Finch-1.6B-shaped inputs (B=8, T=4096, H=32, N=64, bf16 r/k/v/x, fp32 u and
state, zero initial state, bf16 output and fp32 final state written).  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2..5] [--entry NAME] [--preheat-ms MS]

Before the W warm-up steps the same step is launched back to back for --preheat-ms milliseconds
(default 300, untimed, reported as "preheat_ms"): an idle MI355X runs its first ~100 launches at
low clocks (per-launch time falls from ~210 us to its sustained value), so without it a short
run times the clock ramp, not the kernel.  The W warm-up steps and the K timed steps follow
unchanged.  After the timed region the output and final state of a few (batch, head) units of
the last timed step are compared with the fp64 oracle ("parity" in the JSON line).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
MFMA_F16_PEAK_TFLOPS = 2500.0   # dense fp16/bf16 MFMA

# HBM traffic per launch as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs, each
# scaled by the same counter's reading for a plain copy kernel of known size).  These are figures
# from the named summaries under profiles/, not something this run measures: the JSON line carries
# the file name next to the number, and null for workloads that were never profiled.
# value = FETCH_SIZE (KiB) x 2.0 (copy calibration) + WRITE_SIZE (KiB) x 1.0
PROFILED_TRAFFIC = {
    ("config 2", "wkv6_prefill_bf16"): (int(262300 * 1024 * 2.0 + 135200 * 1024 * 1.0), "profiles/chunked_kernel_config2.md"),
    ("config 3", "wkv6_prefill_bf16_split"): (int(1740783 * 1024 * 2.0 + 532536 * 1024 * 1.0), "profiles/chunked_kernel_configs_3_4_5.md"),
    ("config 2", "wkv6_finch_c2_prefill_bf16"): (int(327806 * 1024 * 2.0 + 135168 * 1024 * 1.0), "profiles/finch_c2_kernel_config2.md"),
    ("decode-step B=1024", "wkv6_decode_bf16"): (int(270381 * 1024 * 2.0 + 528416 * 1024 * 1.0), "profiles/decode_step_B1024.md"),
    ("decay-path front of config 2", "wkv6_decay_lora_input_bf16"): (int(126305 * 1024 * 2.0 + 6144 * 1024 * 1.0), "profiles/decay_input_config2_tokens.md"),
    ("LayerNorm apply on config 2", "wkv6_layernorm_apply_bf16"): (int(65750 * 1024 * 2.0 + 131072 * 1024 * 1.0), "profiles/layernorm_apply_config2.md"),
    ("key compression M=131072 D=2048", "wkv6_key_compress_bf16"): (int(265161 * 1024 * 2.0 + 32928 * 1024 * 1.0), "profiles/key_compress_131072_tokens.md"),
    ("key compression M=131072 D=4096", "wkv6_key_compress_bf16"): (int(572103 * 1024 * 2.0 + 65546 * 1024 * 1.0), "profiles/key_compress_131072_tokens.md"),
}
KERNEL_CHUNK = 32               # tokens per chunk of the chunked kernel (for the matrix-core flop count)


def profiled_traffic(workload_key, entry):
    value, source = PROFILED_TRAFFIC.get((workload_key, entry), (None, None))
    return value, source


def preheat(step, torch, ms):
    """Launch `step` back to back for about `ms` milliseconds (untimed) so the timed region starts at
    the chip's sustained clocks."""
    if ms <= 0:
        return 0
    n = 0
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(50):
            step()
        torch.cuda.synchronize()
        n += 50
    return n


def timed_region(step, steps, stream, torch):
    """Exactly `steps` launches between one pair of HIP events recorded on the launch stream, bracketed
    by synchronisations and the host clock.  Returns (average launch duration by the events in ms,
    host-clock ms per step, per-launch durations of a second, untimed pass of at most 100 launches
    with an event after every launch: a marker between two launches costs about 4 us, which is why
    the timed region itself carries only the outer pair)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = e0.elapsed_time(e1) / steps
    n = min(steps, 100)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    evs[0].record(stream)
    for i in range(n):
        step()
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    return kernel_ms, wall * 1e3 / steps, [evs[i].elapsed_time(evs[i + 1]) for i in range(n)]


def algorithmic_bytes(cfg, out_bytes, state_in, state_out=True, streams_in=4):
    """Bytes the method must move per launch: r,k,v,x (and u' in the Finch-C2 form) read once in
    bf16, the output written once, plus the fp32 state of every (batch, head) unit read and/or
    written once."""
    per_token_head = streams_in * cfg.N * 2 + cfg.N * out_bytes
    state = cfg.B * cfg.H * cfg.N * cfg.N * 4
    return cfg.token_heads * per_token_head + state * (int(state_in) + int(state_out))


def algorithmic_flops(cfg, chunk=KERNEL_CHUNK):
    """Matrix-core flops of the chunked form per launch: 4*C*N + 4*N*N per token and head."""
    return cfg.token_heads * (4 * chunk * cfg.N + 4 * cfg.N * cfg.N)


def cpu_baseline(cfg, inp, finch_c2=False):
    """The fp64 oracle, as it stands, timed on this host's cores on a bounded sample."""
    from oracle import finch_c2_oracle, wkv6_oracle
    cores = min(os.cpu_count() or 1, 16)
    budget_token_heads = 4_000_000              # about 10 s of CPU work on 8-16 cores
    nb = max(1, min(cfg.B, budget_token_heads // (cfg.T * cfg.H)))
    sample = {n: inp[n][:nb] for n in ("r", "k", "v", "x")}
    s0 = None if inp["state_in"] is None else inp["state_in"][:nb]
    t0 = time.perf_counter()
    if finch_c2:
        finch_c2_oracle(sample["r"], sample["k"], sample["v"], sample["x"], inp["uprime"][:nb], s0,
                        nthreads=cores)
    else:
        wkv6_oracle(sample["r"], sample["k"], sample["v"], sample["x"], inp["u"], s0, nthreads=cores)
    dt = time.perf_counter() - t0
    # one thread, on the first sequence only
    one = {n: inp[n][:1] for n in ("r", "k", "v", "x")}
    s1 = None if inp["state_in"] is None else inp["state_in"][:1]
    t1 = time.perf_counter()
    if finch_c2:
        finch_c2_oracle(one["r"], one["k"], one["v"], one["x"], inp["uprime"][:1], s1, nthreads=1)
    else:
        wkv6_oracle(one["r"], one["k"], one["v"], one["x"], inp["u"], s1, nthreads=1)
    dt1 = time.perf_counter() - t1
    return {"value": nb * cfg.T / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"first {nb} of {cfg.B} sequences of the same workload "
                      f"({nb * cfg.T * cfg.H} token-heads, fp64 sequential recurrence, {dt:.2f} s)",
            "value_single_thread": cfg.T / dt1}


def check_units(args, cfg, inp, out, s_out, finch_c2, decode, torch):
    """What the last timed step wrote, for a handful of (batch, head) units, against the fp64 oracle:
    max |gpu - oracle| / max |oracle| over those units, for the output and the final state."""
    import numpy as np
    from oracle import finch_c2_oracle, wkv6_oracle
    if args.entry in ("wkv6_finch_c2_prefill_lora_bf16", "wkv6_prefill_lora_bf16"):
        return None                       # logits formed in the kernel: covered by tests/test_gpu_decay_lora.py
    if decode:
        return None                       # the state is updated in place step after step: tests/test_gpu_decode_append.py
    B, H = cfg.B, cfg.H
    units = sorted({(0, 0), (B - 1, H - 1), (B // 2, 3 % H), (B // 3, 11 % H), (B - 1, 19 % H), (0, H // 2)})
    worst_o = worst_s = 0.0
    for (b, h) in units:
        sl = lambda a: np.ascontiguousarray(a[b:b + 1, :, h:h + 1])
        s0 = None if inp["state_in"] is None else np.ascontiguousarray(inp["state_in"][b:b + 1, h:h + 1])
        if finch_c2:
            o_ref, s_ref = finch_c2_oracle(sl(inp["r"]), sl(inp["k"]), sl(inp["v"]), sl(inp["x"]), sl(inp["uprime"]), s0,
                                           nthreads=1)
        else:
            o_ref, s_ref = wkv6_oracle(sl(inp["r"]), sl(inp["k"]), sl(inp["v"]), sl(inp["x"]), inp["u"][h:h + 1], s0,
                                       nthreads=1)
        got_o = out[b, :, h].float().cpu().numpy()
        worst_o = max(worst_o, float(np.abs(got_o - o_ref[0, :, 0]).max() / np.abs(o_ref).max()))
        got_s = s_out[b, h].cpu().numpy()
        worst_s = max(worst_s, float(np.abs(got_s - s_ref[0, 0]).max() / np.abs(s_ref).max()))
    out_is_bf16 = out.dtype == torch.bfloat16
    return {"units_checked": len(units), "err_out": worst_o, "err_state": worst_s,
            "tolerance_out": 2e-3 + (2.0 ** -8 if out_is_bf16 else 0.0), "tolerance_state": 2e-3,
            "against": "fp64 oracle on the same inputs, per unit max-normalised",
            "ok": bool(worst_o <= 2e-3 + (2.0 ** -8 if out_is_bf16 else 0.0) and worst_s <= 2e-3)}


def bench_decay_front(args, torch, wkv):
    """The operators in front of the decay path: y = tanh(ddlerp_d(x_t, x_{t-1}) A_omega) for the tokens of
    the chosen configuration; x and the weights resident in HBM, bf16 output."""
    import numpy as np
    from oracle import decay_lora_input_numpy
    from paper_2407_12077_amd.workloads import CONFIGS, make_decay_front_inputs
    cfg = CONFIGS[args.config]
    B, T, D = cfg.B, cfg.T, cfg.H * cfg.N
    fi = make_decay_front_inputs(cfg)
    dev = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).cuda()
    x, xp = dev(fi["x"], torch.bfloat16), dev(fi["x_prev"], torch.bfloat16)
    mu, lam = dev(fi["mu_x"], torch.float32), dev(fi["lam_d"], torch.float32)
    a_d, b_d, a_w = (dev(fi[n].T, torch.bfloat16) for n in ("A_d", "B_d", "A_omega"))
    y = torch.empty((B, T, 64), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        wkv.wkv6_decay_lora_input_bf16(B, T, D, 32, 64, x, xp, mu, lam, a_d, b_d, a_w, y, wkv.WKV6_DTYPE_BF16,
                                       stream.cuda_stream)

    preheat_launches = preheat(step, torch, args.preheat_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kernel_ms, ms_per_step, per_launch_ms = timed_region(step, args.steps, stream, torch)
    M = B * T
    abytes = M * D * 2 + M * 64 * 2 + B * D * 2 + 2 * D * 4 + (32 + 32 + 64) * D * 2
    aflops = 2 * M * D * (32 + 32 + 64)
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    traffic, traffic_source = profiled_traffic(f"decay-path front of config {cfg.index}", args.entry)
    result = {
        "metric": "decay-path front tokens/s (D=%d -> 32 -> D -> 64, bf16)" % D,
        "value": M / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "preheat_ms": args.preheat_ms, "preheat_launches": preheat_launches,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 tensors; f16 MFMA operands, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"decay-path front of config {cfg.index}: B={B} T={T} D={D}", "entry": args.entry,
                   "global_batch": B, "seq_len": T},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms_avg": kernel_ms,
                     "per_launch_event_ms_median": sorted(per_launch_ms)[len(per_launch_ms) // 2],
                     "per_launch_event_ms_min": min(per_launch_ms), "algorithmic_bytes": abytes,
                     "mfma_frac": aflops / (kernel_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS},
    }
    nb, nt = 1, min(T, 512)
    ref = decay_lora_input_numpy(fi["x"][:nb, :nt], fi["x_prev"][:nb], fi["mu_x"], fi["lam_d"], fi["A_d"], fi["B_d"],
                                 fi["A_omega"])
    got = y[:nb, :nt].float().cpu().numpy()
    result["parity"] = {"tokens_checked": nb * nt, "err": float(np.abs(got - ref).max() / np.abs(ref).max()),
                        "tolerance": 2e-3 + 2.0 ** -8, "against": "fp64 oracle, bf16 output"}
    if not args.no_cpu_baseline:
        nt = min(T, 4096)
        t0 = time.perf_counter()
        decay_lora_input_numpy(fi["x"][:1, :nt], fi["x_prev"][:1], fi["mu_x"], fi["lam_d"], fi["A_d"], fi["B_d"],
                               fi["A_omega"])
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": nt / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                  "sample": f"first {nt} tokens of the first sequence, fp64 NumPy, {dt:.2f} s"}
    print(json.dumps(result))


def bench_layernorm_apply(args, torch, wkv):
    """The LayerNorm of the output equation applied from per-token (mean, rstd): one streaming pass over
    the read-outs of the chosen configuration (bf16 in, bf16 out, D = H*N)."""
    import numpy as np
    from oracle import layernorm_heads_numpy
    from paper_2407_12077_amd.workloads import CONFIGS
    cfg = CONFIGS[args.config]
    B, T, H, N = cfg.B, cfg.T, cfg.H, cfg.N
    D = H * N
    eps = 1e-5
    rng = np.random.Generator(np.random.PCG64(20240712 + 4000 + cfg.index))
    nb, nt = 1, min(T, 256)                        # rows whose values come from the host (checked below)
    o = torch.randn((B, T, H, N), dtype=torch.float32, device="cuda").to(torch.bfloat16)
    head = (rng.standard_normal((nb, nt, H, N), dtype=np.float32) * np.float32(1.5) + np.float32(0.25))
    o[:nb, :nt] = torch.from_numpy(head).to(torch.bfloat16).cuda()
    of = o.float().view(B, T, D)
    mean = of.mean(dim=2)
    rstd = torch.rsqrt(of.var(dim=2, unbiased=False) + eps)
    mr = torch.stack([mean, rstd], dim=2).contiguous()
    del of
    gamma = (1.0 + 0.3 * rng.standard_normal(D)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(D)).astype(np.float32)
    g, bt = torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    y = torch.empty((B, T, D), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        wkv.wkv6_layernorm_apply_bf16(B, T, H, N, o, mr, g, bt, y, wkv.WKV6_DTYPE_BF16, stream.cuda_stream)

    preheat_launches = preheat(step, torch, args.preheat_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kernel_ms, ms_per_step, per_launch_ms = timed_region(step, args.steps, stream, torch)
    M = B * T
    abytes = M * D * 2 * 2 + M * 8 + 2 * D * 4
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    traffic, traffic_source = profiled_traffic(f"LayerNorm apply on config {cfg.index}", args.entry)
    result = {
        "metric": "LayerNorm-apply tokens/s (D=%d, bf16 in and out)" % D,
        "value": M / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "preheat_ms": args.preheat_ms, "preheat_launches": preheat_launches,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 tensors, f32 arithmetic", "data": "synthetic",
        "config": {"workload": f"read-outs of config {cfg.index}: B={B} T={T} D={D}", "entry": args.entry,
                   "global_batch": B, "seq_len": T},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms_avg": kernel_ms,
                     "per_launch_event_ms_median": sorted(per_launch_ms)[len(per_launch_ms) // 2],
                     "per_launch_event_ms_min": min(per_launch_ms), "algorithmic_bytes": abytes},
    }
    # the host-made rows against the oracle's LayerNorm over all heads (its own statistics, fp64)
    ob = o[:nb, :nt].float().cpu().numpy()
    ref, _, _ = layernorm_heads_numpy(ob, gamma, beta, eps)
    got = y[:nb, :nt].float().cpu().numpy().reshape(ref.shape)
    result["parity"] = {"tokens_checked": nb * nt, "err": float(np.abs(got - ref).max() / np.abs(ref).max()),
                        "tolerance": 2.0 ** -8 + 1e-4, "against": "fp64 oracle LayerNorm of the same bf16 read-outs"}
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            layernorm_heads_numpy(ob, gamma, beta, eps)
            reps += 1
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": reps * nb * nt / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{reps} x {nb * nt} tokens, fp64 NumPy, {dt:.2f} s"}
    print(json.dumps(result))


def bench_chain(args, torch, wkv):
    """The data path of one Finch-C2 time-mix layer with everything this library builds, as one step on
    one stream: decay front (x -> y), fused prefill with the LayerNorm partials (r, kbar, v, y, u' ->
    out, state), their fold, the normalisation, and -- standing in for the step behind the layer stack,
    on the normalised rows as hidden states -- the key compression.  Reports the step and each call."""
    import numpy as np
    from oracle import (decay_logits_numpy, decay_lora_input_numpy, finch_c2_oracle, key_compress_oracle,
                        layernorm_heads_numpy)
    from paper_2407_12077_amd.workloads import (CONFIGS, make_decay_front_inputs, make_decay_lora_inputs, make_inputs,
                                                make_key_compress_inputs, make_uprime, round_to_bf16)
    cfg = CONFIGS[args.config]
    B, T, H, N = cfg.B, cfg.T, cfg.H, cfg.N
    D, M, C, R, eps = H * N, B * T, H * N // 16, 64, 1e-5
    fi, inp, lo = make_decay_front_inputs(cfg), make_inputs(cfg), make_decay_lora_inputs(cfg)
    uprime = make_uprime(cfg)
    _, w_kd = make_key_compress_inputs(16, D)
    rng = np.random.Generator(np.random.PCG64(20240712 + 5000 + cfg.index))
    gamma = (1.0 + 0.3 * rng.standard_normal(D)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(D)).astype(np.float32)
    dev = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).cuda()
    bf, f32 = torch.bfloat16, torch.float32
    # the large [B][T][D] tensors in one arena laid out by the library (see wkv6_arena_layout)
    shapes = {"x": (B, T, D), "r": (B, T, H, N), "k": (B, T, H, N), "v": (B, T, H, N), "up": (B, T, H, N),
              "out": (B, T, H, N), "ln": (B, T, D)}
    total, offs = wkv.wkv6_arena_layout([M * D * 2] * len(shapes))
    arena = torch.empty(total + 4096, dtype=torch.uint8, device="cuda")
    first = (-arena.data_ptr()) % 4096
    t = {n: arena[first + o:first + o + M * D * 2].view(bf).view(sh) for (n, sh), o in zip(shapes.items(), offs)}
    for n, src in (("x", fi["x"]), ("r", inp["r"]), ("k", inp["k"]), ("v", inp["v"]), ("up", uprime)):
        t[n].copy_(dev(src, bf).view(shapes[n]))
    xp, mu, lam_d = dev(fi["x_prev"], bf), dev(fi["mu_x"], f32), dev(fi["lam_d"], f32)
    a_d, b_d, a_w = (dev(fi[n].T, bf) for n in ("A_d", "B_d", "A_omega"))
    lam_w, b_w = dev(lo["lam"], f32), dev(lo["b_omega"], bf)
    g, bt, wkd = dev(gamma, f32), dev(beta, f32), dev(w_kd, bf)
    y = torch.empty((B, T, R), dtype=bf, device="cuda")
    mom = torch.empty((B, H, T, 2), dtype=f32, device="cuda")
    mr = torch.empty((B, T, 2), dtype=f32, device="cuda")
    s_out = torch.empty((B, H, N, N), dtype=f32, device="cuda")
    c = torch.empty((M, C), dtype=bf, device="cuda")
    stream = torch.cuda.current_stream()
    q = stream.cuda_stream
    calls = [
        ("wkv6_decay_lora_input_bf16", lambda: wkv.wkv6_decay_lora_input_bf16(B, T, D, 32, R, t["x"], xp, mu, lam_d, a_d, b_d, a_w, y, wkv.WKV6_DTYPE_BF16, q)),
        ("wkv6_finch_c2_prefill_lora_bf16", lambda: wkv.wkv6_finch_c2_prefill_lora_bf16(B, T, H, N, R, t["r"], t["k"], t["v"], y, lam_w, b_w, t["up"], None, t["out"], mom, s_out, q)),
        ("wkv6_layernorm_finalize", lambda: wkv.wkv6_layernorm_finalize(B, T, H, N, mom, eps, mr, q)),
        ("wkv6_layernorm_apply_bf16", lambda: wkv.wkv6_layernorm_apply_bf16(B, T, H, N, t["out"], mr, g, bt, t["ln"], wkv.WKV6_DTYPE_BF16, q)),
        ("wkv6_key_compress_bf16", lambda: wkv.wkv6_key_compress_bf16(M, D, t["ln"], wkd, c, wkv.WKV6_DTYPE_BF16, q)),
    ]

    def step():
        for _, f in calls:
            f()

    preheat_launches = preheat(step, torch, args.preheat_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kernel_ms, ms_per_step, _ = timed_region(step, args.steps, stream, torch)
    per_call = {}
    for name, f in calls:                          # each call alone, back to back, for the breakdown
        for _ in range(20):
            f()
        torch.cuda.synchronize()
        per_call[name], _, _ = timed_region(f, min(args.steps, 100), stream, torch)
    step()
    torch.cuda.synchronize()
    abytes = {"wkv6_decay_lora_input_bf16": M * D * 2 + M * R * 2 + (32 + 32 + R) * D * 2,
              "wkv6_finch_c2_prefill_lora_bf16": 5 * M * D * 2 + M * R * 2 + R * D * 2 + B * H * N * N * 4 + M * H * 8,
              "wkv6_layernorm_finalize": M * H * 8 + M * 8,
              "wkv6_layernorm_apply_bf16": 2 * M * D * 2 + M * 8,
              "wkv6_key_compress_bf16": M * D * 2 + D * C * 2 + M * C * 2}
    total_bytes = sum(abytes.values())
    achieved = total_bytes / (kernel_ms * 1e-3) / 1e9
    result = {
        "metric": "Finch-C2 time-mix chain tokens/s per layer (H=%d,N=%d,bf16): decay front, fused prefill, LayerNorm, "
                  "key compression" % (H, N),
        "value": M / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "preheat_ms": args.preheat_ms, "preheat_launches": preheat_launches, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 tensors; f16/bf16 MFMA operands, f32 accumulate and state", "data": "synthetic",
        "config": {"workload": f"config {cfg.index} ({cfg.name}): B={B} T={T} H={H} N={N}, five calls per step",
                   "entry": "chain", "global_batch": B, "seq_len": T, "placement": "wkv6_arena_layout"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "traffic_source": None, "kernel_ms_avg": kernel_ms, "algorithmic_bytes": total_bytes,
                     "per_call": {n: {"ms": per_call[n], "algorithmic_bytes": abytes[n],
                                      "frac": abytes[n] / (per_call[n] * 1e-3) / 1e9 / HBM_PEAK_GBS} for n, _ in calls}},
    }
    # the first nt tokens of the first sequence through the chained oracles (each stage fed the rounding the
    # GPU's interface tensor carries, so a stage's error is its own)
    nt = min(T, 1024)
    sl = lambda a: a[:1, :nt]
    y_ref = decay_lora_input_numpy(sl(fi["x"]), fi["x_prev"][:1], fi["mu_x"], fi["lam_d"], fi["A_d"], fi["B_d"], fi["A_omega"])
    y_gpu = y[:1, :nt].float().cpu().numpy()
    d = decay_logits_numpy(y_gpu, lo["lam"], lo["b_omega"], H, N)
    o_ref, _ = finch_c2_oracle(sl(inp["r"]), sl(inp["k"]), sl(inp["v"]), d.astype(np.float32), sl(uprime), None)
    o_gpu = t["out"][:1, :nt].float().cpu().numpy()
    ln_ref, _, _ = layernorm_heads_numpy(o_gpu, gamma, beta, eps)
    ln_gpu = t["ln"][:1, :nt].float().cpu().numpy().reshape(1, nt, H, N)
    c_ref = key_compress_oracle(ln_gpu.reshape(nt, D), w_kd)
    c_gpu = c[:nt].float().cpu().numpy()
    err = lambda got, ref: float(np.abs(got - ref).max() / np.abs(ref).max())
    result["parity"] = {"tokens_checked": nt, "err_y": err(y_gpu, y_ref), "err_out": err(o_gpu, o_ref),
                        "err_layernorm": err(ln_gpu, ln_ref), "err_compressed": err(c_gpu, c_ref),
                        "tolerance": 2e-3 + 2.0 ** -8,
                        "against": "fp64 oracles, stage by stage on the GPU's own interface tensors, bf16 outputs"}
    result["parity"]["ok"] = all(result["parity"][k] <= result["parity"]["tolerance"]
                                 for k in ("err_y", "err_out", "err_layernorm", "err_compressed"))
    print(json.dumps(result))


def bench_key_compress(args, torch, wkv):
    """The step after the path: c = x W^KD for the tokens of the chosen configuration (B*T tokens,
    D = H*N), x and W^KD resident in HBM, bf16 output."""
    from oracle import key_compress_oracle
    from paper_2407_12077_amd.workloads import CONFIGS, make_key_compress_inputs
    cfg = CONFIGS[args.config]
    D = cfg.H * cfg.N
    # at least 131072 tokens unless --tokens says otherwise: with config 2's own 32768 tokens x is
    # 134 MB and partly served by the 256 MB last-level cache, which flatters the rate
    M = args.tokens if args.tokens > 0 else max(cfg.B * cfg.T, 131072)
    C = D // 16
    x, w = make_key_compress_inputs(M, D)
    xd = torch.from_numpy(x).to(torch.bfloat16).cuda()
    wd = torch.from_numpy(w).to(torch.bfloat16).cuda()
    c = torch.empty((M, C), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        wkv.wkv6_key_compress_bf16(M, D, xd, wd, c, wkv.WKV6_DTYPE_BF16, stream.cuda_stream)

    preheat_launches = preheat(step, torch, args.preheat_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kernel_ms, ms_per_step, per_launch_ms = timed_region(step, args.steps, stream, torch)
    traffic, traffic_source = profiled_traffic(f"key compression M={M} D={D}", args.entry)
    abytes = M * D * 2 + D * C * 2 + M * C * 2
    aflops = 2 * M * D * C
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    result = {
        "metric": "GOLD key compression tokens/s (D=%d, D/16=%d, bf16)" % (D, C),
        "value": M / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 operands, f32 accumulate", "data": "synthetic",
        "preheat_ms": args.preheat_ms, "preheat_launches": preheat_launches,
        "config": {"workload": f"key compression at the width of config {cfg.index}: M={M} tokens, D={D}",
                   "entry": args.entry, "tokens": M},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms_avg": kernel_ms,
                     "per_launch_event_ms_median": sorted(per_launch_ms)[len(per_launch_ms) // 2],
                     "per_launch_event_ms_min": min(per_launch_ms), "algorithmic_bytes": abytes,
                     "mfma_frac": aflops / (kernel_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS},
    }
    # rows of the last timed launch against the oracle
    rows = sorted({0, M - 1, *((i * 2654435761) % M for i in range(62))})
    import numpy as np
    got = c[rows].float().cpu().numpy()
    ref = key_compress_oracle(x[rows], w)
    result["parity"] = {"rows_checked": len(rows), "err": float(np.abs(got - ref).max() / np.abs(ref).max()),
                        "tolerance": 2.0 ** -8, "against": "fp64 oracle, bf16 output"}
    if not args.no_cpu_baseline:
        cores = min(os.cpu_count() or 1, 16)
        nrows = min(M, 4096)
        t0 = time.perf_counter()
        key_compress_oracle(x[:nrows], w, nthreads=cores)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": nrows / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                                  "sample": f"first {nrows} of {M} tokens, fp64 triple loop, {dt:.2f} s"}
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4, 5])
    ap.add_argument("--entry", default="wkv6_prefill_bf16",
                    choices=["wkv6_prefill_bf16", "wkv6_prefill_bf16_f32out", "wkv6_prefill_bf16_recurrent",
                             "wkv6_prefill_bf16_split", "wkv6_finch_c2_prefill_bf16",
                             "wkv6_finch_c2_prefill_bf16_f32out", "wkv6_finch_c2_prefill_bf16_moments",
                             "wkv6_finch_c2_prefill_lora_bf16", "wkv6_prefill_lora_bf16", "wkv6_decode_bf16", "wkv6_key_compress_bf16",
                             "wkv6_decay_lora_input_bf16", "wkv6_layernorm_apply_bf16", "chain"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--preheat-ms", type=float, default=300.0,
                    help="untimed back-to-back launches of the step for this long before the warm-up steps")
    ap.add_argument("--tokens", type=int, default=0, help="key compression only: number of tokens M")
    ap.add_argument("--aligned-placement", action="store_true",
                    help="time separate allocations instead of the library's arena layout")
    ap.add_argument("--no-placement-probe", action="store_true",
                    help="skip the second timed region (plain prefill entries) with separately allocated tensors")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain 512 MiB device copy (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path shards over (batch, head) "
                 "with no communication); use --gpus 1")

    import torch
    import paper_2407_12077_amd as wkv
    from paper_2407_12077_amd.workloads import CONFIGS, make_inputs, make_uprime

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2407_12077_amd.build import ensure_built
    ensure_built()                               # compiles only when no library is there
    wkv.load()                                   # fails loudly if the HIP library is missing
    if args.entry == "wkv6_key_compress_bf16":
        return bench_key_compress(args, torch, wkv)
    if args.entry == "wkv6_decay_lora_input_bf16":
        return bench_decay_front(args, torch, wkv)
    if args.entry == "wkv6_layernorm_apply_bf16":
        return bench_layernorm_apply(args, torch, wkv)
    if args.entry == "chain":
        return bench_chain(args, torch, wkv)
    cfg = CONFIGS[args.config]
    decode = args.entry == "wkv6_decode_bf16"
    if decode:
        # serving shape: one token for each of 1024 sequences with a carried state (config 4's
        # distributions); 1.07 GB of state traffic per step, well beyond the 256 MB last-level cache
        from paper_2407_12077_amd.workloads import scaled
        cfg = scaled(CONFIGS[4], B=1024, T=1, name="decode-step")
    inp = make_inputs(cfg)
    B, T, H, N = cfg.B, cfg.T, cfg.H, cfg.N

    def dev(a, dt):
        return None if a is None else torch.from_numpy(a).to(dt).cuda()

    r, k, v, x = (dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x"))
    u = dev(inp["u"], torch.float32)
    s_in = dev(inp["state_in"], torch.float32)
    finch_c2 = args.entry.startswith("wkv6_finch_c2")
    if finch_c2:
        inp["uprime"] = make_uprime(cfg)
        up = dev(inp["uprime"], torch.bfloat16)
    out_f32 = args.entry not in ("wkv6_prefill_bf16", "wkv6_prefill_bf16_split", "wkv6_finch_c2_prefill_bf16",
                                 "wkv6_finch_c2_prefill_bf16_moments", "wkv6_finch_c2_prefill_lora_bf16",
                                 "wkv6_prefill_lora_bf16", "wkv6_decode_bf16")
    out = torch.empty((B, T, H, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
    s_out = torch.empty((B, H, N, N), dtype=torch.float32, device="cuda")
    fn = getattr(wkv, args.entry)

    # The large tensors go where the library's placement helper puts them (one arena, tensor i at a
    # 4 KiB boundary + 128 B x (i mod 8)), unless --aligned-placement asks for separate allocations.
    staggered = not decode and not args.aligned_placement
    plain = {"r": r, "k": k, "v": v, "x": x, "out": out}
    if finch_c2:
        plain["up"] = up
    if staggered:
        order = ["r", "k", "v", "x"] + (["up"] if finch_c2 else []) + ["out"]
        sizes = [plain[n].numel() * plain[n].element_size() for n in order]
        total, offsets = wkv.wkv6_arena_layout(sizes)
        arena = torch.empty(total + 4096, dtype=torch.uint8, device="cuda")
        first = (-arena.data_ptr()) % 4096
        placed = {}
        for n, off, nb in zip(order, offsets, sizes):
            placed[n] = arena[first + off:first + off + nb].view(plain[n].dtype).view(plain[n].shape)
            if n != "out":
                placed[n].copy_(plain[n])
        r, k, v, x, out = placed["r"], placed["k"], placed["v"], placed["x"], placed["out"]
        if finch_c2:
            up = placed["up"]

    stream = torch.cuda.current_stream()         # the stream the kernels are launched on

    if args.entry == "wkv6_prefill_bf16_split":
        segments = wkv.wkv6_split_segments(B, T, H, N)
        ws_bytes = wkv.wkv6_split_workspace_bytes(B, T, H, N, segments)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")   # caller-owned workspace

        def step():
            fn(B, T, H, N, r, k, v, x, u, s_in, out, s_out, wkv.WKV6_DTYPE_BF16, segments, ws, ws_bytes,
               stream.cuda_stream)
    elif decode:
        segments = 1
        sq = lambda t: t.view(B, H, N)
        s_out = s_in                                 # updated in place

        def step():
            fn(B, H, N, sq(r), sq(k), sq(v), sq(x), u, s_in, sq(out), stream.cuda_stream)
    elif args.entry == "wkv6_finch_c2_prefill_bf16_moments":
        segments = 1
        moments = torch.empty((B, H, T, 2), dtype=torch.float32, device="cuda")
        mean_rstd = torch.empty((B, T, 2), dtype=torch.float32, device="cuda")

        def step():                              # the prefill with its LayerNorm partials, then their fold
            fn(B, T, H, N, r, k, v, x, up, s_in, out, moments, s_out, stream.cuda_stream)
            wkv.wkv6_layernorm_finalize(B, T, H, N, moments, 1e-5, mean_rstd, stream.cuda_stream)
    elif args.entry in ("wkv6_finch_c2_prefill_lora_bf16", "wkv6_prefill_lora_bf16"):
        segments = 1
        from paper_2407_12077_amd.workloads import make_decay_lora_inputs
        lora = make_decay_lora_inputs(cfg)
        y, b_omega = dev(lora["y"], torch.bfloat16), dev(lora["b_omega"], torch.bfloat16)
        lam = dev(lora["lam"], torch.float32)
        # x is not passed: the logits are formed in the kernel

        if finch_c2:
            def step():
                fn(B, T, H, N, 64, r, k, v, y, lam, b_omega, up, s_in, out, None, s_out, stream.cuda_stream)
        else:
            def step():
                fn(B, T, H, N, 64, r, k, v, y, lam, b_omega, u, s_in, out, s_out, stream.cuda_stream)
    elif finch_c2:
        segments = 1

        def step():
            fn(B, T, H, N, r, k, v, x, up, s_in, out, s_out, stream.cuda_stream)
    else:
        segments = 1

        def step():
            fn(B, T, H, N, r, k, v, x, u, s_in, out, s_out, stream.cuda_stream)

    if args.copy_probe:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.bfloat16, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    preheat_launches = preheat(step, torch, args.preheat_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kernel_ms, ms_per_step, per_launch_ms = timed_region(step, args.steps, stream, torch)

    abytes = algorithmic_bytes(cfg, 4 if out_f32 else 2, s_in is not None, streams_in=5 if finch_c2 else 4)
    if args.entry in ("wkv6_finch_c2_prefill_lora_bf16", "wkv6_prefill_lora_bf16"):
        # four bf16 streams per token-head instead of five; y once per token, the outer factor once
        abytes += -B * T * H * N * 2 + B * T * 64 * 2 + 64 * H * N * 2 + H * N * 4
    if args.entry == "wkv6_finch_c2_prefill_bf16_moments":
        abytes += B * T * H * 8 * 2 + B * T * 8      # partials written and read back once, two numbers per token
    aflops = algorithmic_flops(cfg)
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    workload_key = f"decode-step B={B}" if decode else f"config {cfg.index}"
    traffic, traffic_source = profiled_traffic(workload_key, args.entry)
    result = {
        "metric": "WKV6 prefill tokens/s per layer (H=%d,N=%d,bf16)" % (H, N),
        "value": B * T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "preheat_ms": args.preheat_ms,
        "preheat_launches": preheat_launches,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 tensors; f16 MFMA operands, f32 accumulate and state"
                 if args.entry not in ("wkv6_prefill_bf16_recurrent", "wkv6_decode_bf16")
                 else "bf16 tensors; f32 vector ALU, f32 state",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.index} ({cfg.name}): B={B} T={T} H={H} N={N}, "
                               f"{'nonzero' if s_in is not None else 'zero'} initial state",
                   "entry": args.entry, "segments": segments, "global_batch": B, "seq_len": T,
                   "placement": "wkv6_arena_layout: one arena, tensor i at a 4 KiB boundary + 128 B x (i mod 8)"
                                if staggered else "separate allocations"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms_avg": kernel_ms, "per_launch_event_ms_median": sorted(per_launch_ms)[len(per_launch_ms) // 2],
                     "per_launch_event_ms_min": min(per_launch_ms),
                     "algorithmic_bytes": abytes,
                     "mfma_frac": aflops / (kernel_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS},
    }
    result["parity"] = check_units(args, cfg, inp, out, s_out, finch_c2, decode, torch)
    if staggered and args.entry in ("wkv6_prefill_bf16", "wkv6_finch_c2_prefill_bf16") and not args.no_placement_probe:
        # Same call, same data, ordinary placement: every tensor an allocation of its own, so that all
        # bases agree in address bits 7..9 (what a caller gets who does not use wkv6_arena_layout).
        out_staggered, s_out_staggered = out, s_out.clone()
        r, k, v, x, out = plain["r"], plain["k"], plain["v"], plain["x"], plain["out"]
        if finch_c2:
            up = plain["up"]
        preheat(step, torch, args.preheat_ms)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        kernel_ms2, ms_per_step2, _ = timed_region(step, args.steps, stream, torch)
        result["aligned_placement"] = {
            "bases": "each tensor its own allocation (bases agree modulo 4 KiB)",
            "ms_per_step": ms_per_step2, "value": B * T / (ms_per_step2 * 1e-3),
            "frac": abytes / (kernel_ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "same_result": bool(torch.equal(out_staggered, out) and torch.equal(s_out_staggered, s_out))}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, inp, finch_c2)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
