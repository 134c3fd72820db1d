"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on the same
seeded inputs.  Tolerances are the stated ones: max |gpu - oracle| / max |oracle| <= 2e-3
for bf16 inputs (fp32 output and state) and <= 1e-5 for fp32 tensors.
"""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from oracle import wkv6_oracle
from paper_2407_12077_amd.workloads import CONFIGS, make_inputs, round_to_bf16, scaled

from gpu_util import (BF16_OUT_ROUNDING, TOL_BF16, TOL_F32, error_report, fmt_report, max_norm_err, run_entry,
                      to_dev)

pytestmark = pytest.mark.gpu


def check(entry, inp, tol, **kw):
    o_ref, s_ref = wkv6_oracle(inp["r"], inp["k"], inp["v"], inp["x"], inp["u"], inp.get("state_in"))
    o, s = run_entry(entry, inp, **kw)
    eo, es = max_norm_err(o, o_ref), max_norm_err(s, s_ref)
    print(f"{entry}: shape={inp['r'].shape} err_out={eo:.3e} err_state={es:.3e}", flush=True)
    assert np.isfinite(o).all() and np.isfinite(s).all()
    assert eo <= tol, f"out error {eo:.3e} > {tol}"
    assert es <= tol, f"state error {es:.3e} > {tol}"
    return eo, es


# ------------------------------------------------------------------ config 1 (fp32, full size)
def test_config1_fp32_full(gpu_device):
    inp = make_inputs(CONFIGS[1])
    check("wkv6_prefill_f32", inp, TOL_F32, in_dtype=torch.float32)


def test_fp32_with_initial_state_and_ragged_length(gpu_device):
    inp = make_inputs(scaled(CONFIGS[1], B=3, T=77, H=5, s0_std=0.5), seed=5)
    check("wkv6_prefill_f32", inp, TOL_F32, in_dtype=torch.float32)


def test_recurrent_kernel_on_bf16_inputs(gpu_device):
    inp = make_inputs(scaled(CONFIGS[2], B=2, T=300, H=3, s0_std=0.2), seed=6)
    check("wkv6_prefill_bf16_recurrent", inp, TOL_F32)


@pytest.mark.parametrize("T", [1, 6, 7, 15, 16, 17, 23, 24, 25, 40])
def test_token_by_token_forms_on_both_sides_of_their_switch(gpu_device, T):
    """The token-by-token entry points use a one-wave kernel below 16 tokens and a four-wave kernel
    with 8-token blocks from 16 on: lengths around the switch, with whole and ragged last blocks."""
    inp = make_inputs(scaled(CONFIGS[1], B=2, T=T, H=3, s0_std=0.4), seed=900 + T)
    check("wkv6_prefill_f32", inp, TOL_F32, in_dtype=torch.float32)
    inp = make_inputs(scaled(CONFIGS[2], B=2, T=T, H=3, s0_std=0.4), seed=950 + T)
    check("wkv6_prefill_bf16_recurrent", inp, TOL_F32)


# ------------------------------------------------------------------ chunked kernel, oracle-sized
@pytest.mark.parametrize("T", [1, 2, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 127, 128, 129, 200, 1000])
def test_chunked_lengths(gpu_device, T):
    inp = make_inputs(scaled(CONFIGS[2], B=2, T=T, H=3), seed=100 + T)
    check("wkv6_prefill_bf16_f32out", inp, TOL_BF16)


@pytest.mark.parametrize("cfg_index", [2, 4, 5])
def test_chunked_reduced_configs(gpu_device, cfg_index):
    cfg = CONFIGS[cfg_index]
    inp = make_inputs(scaled(cfg, B=2, T=777, H=min(cfg.H, 8)))
    check("wkv6_prefill_bf16_f32out", inp, TOL_BF16)


def test_chunked_bf16_output(gpu_device):
    inp = make_inputs(scaled(CONFIGS[2], B=2, T=333, H=4, s0_std=0.1), seed=21)
    o_ref, s_ref = wkv6_oracle(**inp)
    o, s = run_entry("wkv6_prefill_bf16", inp, out_dtype=torch.bfloat16)
    assert max_norm_err(s, s_ref) <= TOL_BF16
    assert max_norm_err(o, o_ref) <= TOL_BF16 + BF16_OUT_ROUNDING
    # against the oracle rounded the same way: the kernel's own share stays within tolerance
    assert max_norm_err(o, round_to_bf16(o_ref.astype(np.float32))) <= TOL_BF16 + BF16_OUT_ROUNDING
    o32, _ = run_entry("wkv6_prefill_bf16_f32out", inp)
    assert np.array_equal(o, round_to_bf16(o32.astype(np.float32)).astype(np.float64))


def test_chunked_matches_recurrent_kernel(gpu_device):
    inp = make_inputs(scaled(CONFIGS[4], B=3, T=512, H=4), seed=22)
    o1, s1 = run_entry("wkv6_prefill_bf16_f32out", inp)
    o2, s2 = run_entry("wkv6_prefill_bf16_recurrent", inp)
    assert max_norm_err(o1, o2) <= TOL_BF16 and max_norm_err(s1, s2) <= TOL_BF16


# ------------------------------------------------------------------ degenerate decays
@pytest.mark.parametrize("xval", [-np.inf, np.inf, 20.0, -30.0, 3.0])
@pytest.mark.parametrize("entry,tol,dt", [("wkv6_prefill_bf16_f32out", TOL_BF16, torch.bfloat16),
                                          ("wkv6_prefill_f32", TOL_F32, torch.float32)])
def test_constant_extreme_decay(gpu_device, xval, entry, tol, dt):
    inp = make_inputs(scaled(CONFIGS[2], B=1, T=150, H=2, s0_std=0.3), seed=31)
    inp["x"][:] = xval
    check(entry, inp, tol, in_dtype=dt)


def test_mixed_extreme_decays(gpu_device):
    rng = np.random.default_rng(32)
    inp = make_inputs(scaled(CONFIGS[2], B=2, T=260, H=2, s0_std=0.3), seed=32)
    choices = np.array([-np.inf, np.inf, -20.0, 10.0, 0.0, -1.0, 2.0], dtype=np.float32)
    inp["x"] = rng.choice(choices, size=inp["x"].shape).astype(np.float32)
    check("wkv6_prefill_bf16_f32out", inp, TOL_BF16)
    check("wkv6_prefill_bf16_recurrent", inp, TOL_F32)


def test_zero_inputs_keep_decayed_state(gpu_device):
    inp = make_inputs(scaled(CONFIGS[2], B=1, T=100, H=2, s0_std=1.0), seed=33)
    for n in ("r", "k", "v"):
        inp[n][:] = 0
    check("wkv6_prefill_bf16_f32out", inp, TOL_BF16)


# ------------------------------------------------------------------ state handling through the ABI
def test_state_passing_invariant_on_gpu(gpu_device):
    """[0,T) in one call == [0,T1) then [T1,T) with the carried state (strided entry, B>1)."""
    cfg = scaled(CONFIGS[2], B=3, T=448, H=4)
    inp = make_inputs(cfg, seed=41)
    B, T, H, N = inp["r"].shape
    o_ref, s_ref = wkv6_oracle(**inp)
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in "rkvx")
    u = to_dev(inp["u"], torch.float32)
    full_o = torch.empty((B, T, H, N), dtype=torch.float32, device="cuda")
    full_s = torch.empty((B, H, N, N), dtype=torch.float32, device="cuda")
    wkv.wkv6_prefill_bf16_f32out(B, T, H, N, r, k, v, x, u, None, full_o, full_s)
    for T1 in (64, 200, 447):
        o = torch.full((B, T, H, N), float("nan"), dtype=torch.float32, device="cuda")
        s = torch.empty((B, H, N, N), dtype=torch.float32, device="cuda")
        stride = T * H * N
        wkv.wkv6_prefill_bf16_strided(B, T1, H, N, r, k, v, x, u, None, o, s, stride, wkv.WKV6_DTYPE_F32)
        off = T1 * H * N
        tail = lambda t: t.view(-1)[off:]            # same batch stride, window starts at token T1
        wkv.wkv6_prefill_bf16_strided(B, T - T1, H, N, tail(r), tail(k), tail(v), tail(x), u, s,
                                      tail(o), s, stride, wkv.WKV6_DTYPE_F32)   # state in place
        torch.cuda.synchronize()
        assert max_norm_err(o.cpu().numpy(), o_ref) <= TOL_BF16
        assert max_norm_err(s.cpu().numpy(), s_ref) <= TOL_BF16
        assert max_norm_err(o.cpu().numpy(), full_o.cpu().numpy()) <= TOL_BF16
        assert max_norm_err(s.cpu().numpy(), full_s.cpu().numpy()) <= TOL_BF16


def test_null_state_out_and_inplace_state(gpu_device):
    inp = make_inputs(scaled(CONFIGS[4], B=2, T=130, H=3), seed=42)
    o_ref, s_ref = wkv6_oracle(**inp)
    for entry, tol, dt in (("wkv6_prefill_bf16_f32out", TOL_BF16, torch.bfloat16),
                           ("wkv6_prefill_bf16_recurrent", TOL_F32, torch.bfloat16)):
        o, s = run_entry(entry, inp, want_state=False, in_dtype=dt)
        assert s is None and max_norm_err(o, o_ref) <= tol
        o, s = run_entry(entry, inp, inplace_state=True, in_dtype=dt)
        assert max_norm_err(o, o_ref) <= tol and max_norm_err(s, s_ref) <= tol


def test_empty_sequence_passes_state_through(gpu_device):
    s_in = torch.randn(2, 3, 64, 64, device="cuda")
    u = torch.zeros(3, 64, device="cuda")
    s_out = torch.full_like(s_in, float("nan"))
    wkv.wkv6_prefill_bf16_f32out(2, 0, 3, 64, None, None, None, None, u, s_in, None, s_out)
    torch.cuda.synchronize()
    assert torch.equal(s_in, s_out)
    wkv.wkv6_prefill_f32(2, 0, 3, 64, None, None, None, None, u, None, None, s_out)
    torch.cuda.synchronize()
    assert (s_out == 0).all()
    wkv.wkv6_prefill_bf16(0, 5, 3, 64, None, None, None, None, u, None, None, None)   # empty batch


def test_runs_on_a_side_stream_and_is_deterministic(gpu_device):
    inp = make_inputs(scaled(CONFIGS[2], B=2, T=500, H=4), seed=43)
    B, T, H, N = inp["r"].shape
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in "rkvx")
    u = to_dev(inp["u"], torch.float32)
    outs = []
    side = torch.cuda.Stream()
    for i in range(3):
        o = torch.empty((B, T, H, N), dtype=torch.float32, device="cuda")
        s = torch.empty((B, H, N, N), dtype=torch.float32, device="cuda")
        if i == 2:
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                wkv.wkv6_prefill_bf16_f32out(B, T, H, N, r, k, v, x, u, None, o, s)
            side.synchronize()
        else:
            wkv.wkv6_prefill_bf16_f32out(B, T, H, N, r, k, v, x, u, None, o, s)
            torch.cuda.synchronize()
        outs.append((o.cpu(), s.cpu()))
    for o, s in outs[1:]:
        assert torch.equal(o, outs[0][0]) and torch.equal(s, outs[0][1])     # bit-identical


def test_finch_c2_reduction(gpu_device):
    """u = 0 and k pre-multiplied by (1 - w): state rows stay normalised (each entry is a
    convex combination of past values), so with v == 1 every state entry is 1 - prod w."""
    rng = np.random.default_rng(44)
    B, T, H, N = 1, 200, 2, 64
    x = round_to_bf16(rng.uniform(-5, 0, (B, T, H, N)).astype(np.float32))
    w = np.exp(-np.exp(x.astype(np.float64)))
    k = round_to_bf16((1 - w).astype(np.float32))
    inp = {"r": round_to_bf16(rng.standard_normal((B, T, H, N)).astype(np.float32) / 8), "k": k,
           "v": np.ones((B, T, H, N), np.float32), "x": x, "u": np.zeros((H, N), np.float32),
           "state_in": None}
    _, s = check("wkv6_prefill_bf16_f32out", inp, TOL_BF16)
    o, st = run_entry("wkv6_prefill_bf16_f32out", inp)
    expect = 1 - np.prod(w, axis=1)[0]                       # [H, N(key)]
    assert np.abs(st[0] - expect[:, :, None]).max() <= 3e-3  # k itself was rounded to bf16


# ------------------------------------------------------------------ token-split variant
def _run_split(inp, segments, out_dtype=torch.float32, want_state=True):
    B, T, H, N = inp["r"].shape
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in "rkvx")
    u = to_dev(inp["u"], torch.float32)
    s_in = to_dev(inp.get("state_in"), torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=out_dtype, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda") if want_state else None
    nbytes = wkv.wkv6_split_workspace_bytes(B, T, H, N, segments)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    code = wkv.WKV6_DTYPE_F32 if out_dtype == torch.float32 else wkv.WKV6_DTYPE_BF16
    wkv.wkv6_prefill_bf16_split(B, T, H, N, r, k, v, x, u, s_in, out, s_out, code, segments, ws, nbytes)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), (None if s_out is None else s_out.cpu().numpy().astype(np.float64))


@pytest.mark.parametrize("T,segments", [(4096, 4), (5000, 4), (1000, 7), (333, 3), (64, 2), (40, 8), (8192, 16)])
def test_split_matches_oracle(gpu_device, T, segments):
    inp = make_inputs(scaled(CONFIGS[4], B=2, T=T, H=3), seed=700 + T)
    o_ref, s_ref = wkv6_oracle(**inp)
    o, s = _run_split(inp, segments)
    eo, es = max_norm_err(o, o_ref), max_norm_err(s, s_ref)
    print(f"split T={T} segments={segments}: err_out={eo:.3e} err_state={es:.3e}", flush=True)
    assert eo <= TOL_BF16 and es <= TOL_BF16


def test_split_with_long_memory_channels(gpu_device):
    """Decays near 1 on half of the channels: the state entering a segment matters for its whole
    length, and the product of decays over a segment is far from zero."""
    inp = make_inputs(scaled(CONFIGS[5], B=1, T=4096, H=4), seed=71)
    inp["state_in"] = (np.random.default_rng(72).standard_normal((1, 4, 64, 64)) * 0.5).astype(np.float32)
    o_ref, s_ref = wkv6_oracle(**inp)
    o, s = _run_split(inp, 8)
    assert max_norm_err(o, o_ref) <= TOL_BF16 and max_norm_err(s, s_ref) <= TOL_BF16
    inp["x"][:] = -np.inf                      # w == 1 everywhere: nothing is ever forgotten
    o_ref, s_ref = wkv6_oracle(**inp)
    o, s = _run_split(inp, 8)
    assert max_norm_err(o, o_ref) <= TOL_BF16 and max_norm_err(s, s_ref) <= TOL_BF16


def test_split_bf16_out_and_no_state_out(gpu_device):
    inp = make_inputs(scaled(CONFIGS[2], B=1, T=3000, H=2), seed=73)
    o_ref, _ = wkv6_oracle(**inp)
    o, s = _run_split(inp, 5, out_dtype=torch.bfloat16, want_state=False)
    assert s is None and max_norm_err(o, o_ref) <= TOL_BF16 + BF16_OUT_ROUNDING


def test_split_state_in_place_and_short_last_segment(gpu_device):
    """state_out may be the state_in buffer: the fold reads the entering state before the full pass
    of the last segment (shorter than the others here) writes the final one over it."""
    inp = make_inputs(scaled(CONFIGS[4], B=2, T=1000, H=3, s0_std=0.4), seed=74)
    o_ref, s_ref = wkv6_oracle(**inp)
    B, T, H, N = inp["r"].shape
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in "rkvx")
    u = to_dev(inp["u"], torch.float32)
    state = to_dev(inp["state_in"], torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=torch.float32, device="cuda")
    segments = 3                                   # 352 + 352 + 296 tokens
    nbytes = wkv.wkv6_split_workspace_bytes(B, T, H, N, segments)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    wkv.wkv6_prefill_bf16_split(B, T, H, N, r, k, v, x, u, state, out, state, wkv.WKV6_DTYPE_F32, segments, ws, nbytes)
    torch.cuda.synchronize()
    assert max_norm_err(out.cpu().numpy().astype(np.float64), o_ref) <= TOL_BF16
    assert max_norm_err(state.cpu().numpy().astype(np.float64), s_ref) <= TOL_BF16


def test_tensors_beyond_four_gib(gpu_device):
    """Every tensor larger than 4 GiB (H = 544 heads, 65 536 tokens: 4.56 GB each), so byte offsets
    inside a tensor pass 2^32 and a token row is 68 KiB: the kernel re-bases its 32-bit buffer
    descriptors per chunk.  Inputs are drawn on the device (seeded); the units compared with the
    oracle are the first head, one in the middle and the last one, whose rows sit at the far end."""
    B, T, H, N = 1, 65536, 544, 64
    gen = torch.Generator(device="cuda").manual_seed(4242)
    def draw(scale, shift):
        t = torch.empty((B, T, H, N), dtype=torch.bfloat16, device="cuda")
        for t0 in range(0, T, 4096):                     # 0.57 GB of fp32 at a time
            blk = torch.rand((B, 4096, H, N), generator=gen, device="cuda") * scale + shift
            t[:, t0:t0 + 4096] = blk.to(torch.bfloat16)
        return t
    r, k, v = draw(2.0, -1.0), draw(2.0, -1.0), draw(2.0, -1.0)
    x = draw(7.0, -8.0)                                  # w between exp(-exp(-1)) and nearly 1
    u = (torch.rand((H, N), generator=gen, device="cuda") - 0.5).contiguous()
    out = torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
    assert r.numel() * 2 > (1 << 32)
    print("tensors of %.2f GB each" % (r.numel() * 2 / 1e9), flush=True)
    wkv.wkv6_prefill_bf16(B, T, H, N, r, k, v, x, u, None, out, s_out)
    torch.cuda.synchronize()
    for h in (0, 271, 543):
        one = {n: t[:, :, h:h + 1].float().cpu().numpy() for n, t in (("r", r), ("k", k), ("v", v), ("x", x))}
        o_ref, s_ref = wkv6_oracle(one["r"], one["k"], one["v"], one["x"], u[h:h + 1].cpu().numpy(), None)
        o = out[:, :, h:h + 1].float().cpu().numpy().astype(np.float64)
        s = s_out[:, h:h + 1].cpu().numpy().astype(np.float64)
        eo, es = max_norm_err(o, o_ref), max_norm_err(s, s_ref)
        print(f"head {h}: err_out={eo:.3e} err_state={es:.3e}", flush=True)
        assert np.isfinite(o).all() and np.isfinite(s).all()
        assert eo <= TOL_BF16 + BF16_OUT_ROUNDING and es <= TOL_BF16
    # every row was written
    assert bool(torch.isfinite(out[:, -1].float()).all()) and bool(torch.isfinite(out[:, 0].float()).all())
    del r, k, v, x, out
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ full-size configs, every unit
def _unit_slice(inp, b, h):
    one = {n: np.ascontiguousarray(inp[n][b:b + 1, :, h:h + 1]) for n in "rkvx"}
    one["u"] = np.ascontiguousarray(inp["u"][h:h + 1])
    one["state_in"] = None if inp["state_in"] is None else np.ascontiguousarray(inp["state_in"][b:b + 1, h:h + 1])
    return one


@pytest.mark.parametrize("cfg_index", [2, 3, 4, 5])
def test_full_size_config_every_unit(gpu_device, cfg_index):
    """The benchmark's launch configuration at full size: every output element and every final
    state entry of every (batch, head) unit against the oracle, for the fp32-out entry (the gate
    without output rounding) and for the benchmarked bf16-out entry.  Printed per tensor: the
    gated global figure, the worst per-unit figure (gated too), the worst per-token-row figure
    and the relative L2 error."""
    cfg = CONFIGS[cfg_index]
    inp = make_inputs(cfg)
    B, T, H, N = inp["r"].shape
    print(f"config {cfg_index}: oracle on every unit ...", flush=True)
    o_ref, s_ref = wkv6_oracle(**inp)              # all host cores
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in "rkvx")
    u = to_dev(inp["u"], torch.float32)
    s_in = to_dev(inp["state_in"], torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=torch.float32, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
    wkv.wkv6_prefill_bf16_f32out(B, T, H, N, r, k, v, x, u, s_in, out, s_out)
    out16 = torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    s_out16 = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
    wkv.wkv6_prefill_bf16(B, T, H, N, r, k, v, x, u, s_in, out16, s_out16)
    torch.cuda.synchronize()
    rep_o = error_report(out.cpu().numpy(), o_ref, "out")
    rep_s = error_report(s_out.cpu().numpy(), s_ref, "state")
    print(f"config {cfg_index} wkv6_prefill_bf16_f32out, all {B * H} units: out {fmt_report(rep_o)} | "
          f"state {fmt_report(rep_s)}", flush=True)
    assert rep_o["global"] <= TOL_BF16 and rep_o["unit"] <= TOL_BF16
    assert rep_s["global"] <= TOL_BF16 and rep_s["unit"] <= TOL_BF16
    rep_o16 = error_report(out16.float().cpu().numpy(), o_ref, "out")
    print(f"config {cfg_index} wkv6_prefill_bf16 (the benchmarked entry), all {B * H} units: out {fmt_report(rep_o16)}",
          flush=True)
    assert rep_o16["global"] <= TOL_BF16 + BF16_OUT_ROUNDING and rep_o16["unit"] <= TOL_BF16 + BF16_OUT_ROUNDING
    assert torch.equal(s_out16, s_out)
    assert torch.equal(out16, out.to(torch.bfloat16))          # the fp32 result rounded once
    del out16, s_out16
    if cfg_index == 3:
        # state at T/2 and the state-passing invariant: two calls with the carried state
        half = T // 2
        o2 = torch.empty_like(out)
        s_half = torch.empty_like(s_out)
        s_end = torch.empty_like(s_out)
        wkv.wkv6_prefill_bf16_f32out(B, half, H, N, r, k, v, x, u, None, o2, s_half)
        off = half * H * N
        tail = lambda t: t.view(-1)[off:]
        wkv.wkv6_prefill_bf16_f32out(B, T - half, H, N, tail(r), tail(k), tail(v), tail(x), u, s_half,
                                     tail(o2), s_end)
        torch.cuda.synchronize()
        assert max_norm_err(o2.cpu().numpy(), out.cpu().numpy()) <= 1e-6      # same chunk boundaries
        assert max_norm_err(s_end.cpu().numpy(), s_out.cpu().numpy()) <= 1e-6
        del o2
        first = {n: inp[n][:, :half] for n in "rkvx"}
        _, s_ref_half = wkv6_oracle(first["r"], first["k"], first["v"], first["x"], inp["u"], None)
        rep_h = error_report(s_half.cpu().numpy(), s_ref_half, "state")
        print(f"config 3 state at T/2: {fmt_report(rep_h)}", flush=True)
        assert rep_h["global"] <= TOL_BF16 and rep_h["unit"] <= TOL_BF16
        # the token-split entry in the benchmark's configuration, against the oracle itself
        segs = wkv.wkv6_split_segments(B, T, H, N)
        assert segs > 1
        nbytes = wkv.wkv6_split_workspace_bytes(B, T, H, N, segs)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for code, dt, extra in ((wkv.WKV6_DTYPE_F32, torch.float32, 0.0), (wkv.WKV6_DTYPE_BF16, torch.bfloat16, BF16_OUT_ROUNDING)):
            o3 = torch.full((B, T, H, N), float("nan"), dtype=dt, device="cuda")
            s3 = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
            wkv.wkv6_prefill_bf16_split(B, T, H, N, r, k, v, x, u, None, o3, s3, code, segs, ws, nbytes)
            torch.cuda.synchronize()
            rep_o3 = error_report(o3.float().cpu().numpy(), o_ref, "out")
            rep_s3 = error_report(s3.cpu().numpy(), s_ref, "state")
            print(f"config 3 wkv6_prefill_bf16_split ({segs} segments, out {dt}): out {fmt_report(rep_o3)} | "
                  f"state {fmt_report(rep_s3)}", flush=True)
            assert rep_o3["global"] <= TOL_BF16 + extra and rep_o3["unit"] <= TOL_BF16 + extra
            assert rep_s3["global"] <= TOL_BF16 and rep_s3["unit"] <= TOL_BF16
            del o3


def test_small_operands_meet_the_absolute_floor_of_fp16_tiles(gpu_device):
    """The header's second value-range clause.  The matrix-core operands are fp16: a scaled
    operand (r, k, v times a product of decays) below 2^-14 in magnitude is held to an absolute
    2^-25, not to a relative 2^-11.  Here the first tokens are 2^-12 of the last ones in amplitude,
    half the channels have long memory and half forget within a few tokens (decay products down
    to 1e-10 inside a chunk), so the early rows are small next to the tensor's maximum and many of
    their operands are below the normal range.  Gated: the usual global and per-unit figures, and
    every element against  tolerance x (its row's largest reference value) + the floor that
    follows from the 2^-25 steps (at most 64 channels x 32 tokens of products with one operand off
    by 2^-25 and the other at most max|r| or max|k|, times max|v|; the state read adds
    64 x 2^-25 x max|S|).  Printed: the worst per-row figure, which this floor, not the relative
    tolerance, explains."""
    B, T, H, N = 2, 384, 4, 64
    cfg = scaled(CONFIGS[5], B=B, T=T, H=H)
    inp = make_inputs(cfg, seed=505)
    ramp = (2.0 ** np.linspace(-12.0, 0.0, T)).astype(np.float32)[None, :, None, None]
    for n in "rkv":
        inp[n] = round_to_bf16(inp[n] * ramp)
    fast = np.random.default_rng(506).random((H, N)) < 0.5
    inp["x"] = round_to_bf16(np.where(fast[None, None], np.float32(1.5), inp["x"]))    # w = 0.011 per token
    o_ref, s_ref = wkv6_oracle(**inp)
    o, s = run_entry("wkv6_prefill_bf16_f32out", inp)
    rep_o, rep_s = error_report(o, o_ref, "out"), error_report(s, s_ref, "state")
    print(f"small early operands: out {fmt_report(rep_o)} | state {fmt_report(rep_s)}", flush=True)
    assert rep_o["global"] <= TOL_BF16 and rep_o["unit"] <= TOL_BF16
    assert rep_s["global"] <= TOL_BF16 and rep_s["unit"] <= TOL_BF16
    step = 2.0 ** -25
    amax = lambda n: float(np.abs(inp[n]).max())
    floor = 64 * 32 * step * (amax("r") + amax("k")) * amax("v") + 64 * step * (1 + amax("r")) * float(np.abs(s_ref).max())
    row_ref = np.abs(o_ref).max(axis=3, keepdims=True)
    excess = np.abs(o - o_ref) - (TOL_BF16 * row_ref + floor)
    print(f"  floor={floor:.3e}, smallest row scale={row_ref.min():.3e}, worst excess over the bound={excess.max():.3e}",
          flush=True)
    assert excess.max() <= 0


def test_operands_beyond_fp16_range_saturate(gpu_device):
    """The header's value-range clause: on the bf16 entry points operands larger than the fp16
    maximum saturate to +-65504 (no infinities, no NaNs): the result is that of the oracle run on
    the clamped inputs."""
    cfg = scaled(CONFIGS[2], B=1, T=160, H=2)
    inp = make_inputs(cfg)
    rng = np.random.default_rng(77)
    k = inp["k"].copy()
    hit = rng.random(k.shape) < 0.002
    k[hit] = np.where(rng.random(hit.sum()) < 0.5, 1.0e5, -3.0e5).astype(np.float32)
    inp["k"] = round_to_bf16(k)
    inp["v"] = inp["v"] * np.float32(0.125)        # keeps every state entry inside the fp16 range
    inp["u"] = np.clip(inp["u"], -1.0, 1.0)        # ... and the bonus-weighted key k*u
    o, s = run_entry("wkv6_prefill_bf16_f32out", inp)
    assert np.isfinite(o).all() and np.isfinite(s).all()
    clamped = dict(inp)
    clamped["k"] = np.clip(inp["k"], -65504.0, 65504.0)
    o_ref, s_ref = wkv6_oracle(**clamped)
    assert 1.0e3 < np.abs(s_ref).max() < 3.0e4
    assert max_norm_err(o, o_ref) <= TOL_BF16 and max_norm_err(s, s_ref) <= TOL_BF16


@pytest.mark.parametrize("B,T,H", [(70, 45, 4), (300, 20, 3), (40, 130, 8), (33, 32, 16), (600, 1, 2), (5, 40, 96), (12, 70, 64),
                                   (1, 40, 260), (2, 33, 260)])
def test_many_units_per_workgroup(gpu_device, B, T, H):
    """More (batch, head) units than compute units: each workgroup runs several units back to
    back without draining its pipeline; unit counts per workgroup differ by one, lengths ragged."""
    inp = make_inputs(scaled(CONFIGS[4], B=B, T=T, H=H))
    check("wkv6_prefill_bf16_f32out", inp, TOL_BF16)
    o16, s16 = run_entry("wkv6_prefill_bf16", inp, out_dtype=torch.bfloat16)
    o32, s32 = run_entry("wkv6_prefill_bf16_f32out", inp)
    assert np.array_equal(o16.astype(np.float32), round_to_bf16(o32.astype(np.float32)))
    assert np.array_equal(s16, s32)


def test_many_units_in_place_state_and_zero_state(gpu_device):
    inp = make_inputs(scaled(CONFIGS[4], B=90, T=70, H=4))
    o_ref, s_ref = wkv6_oracle(**inp)
    o, s = run_entry("wkv6_prefill_bf16_f32out", inp, inplace_state=True)
    assert max_norm_err(o, o_ref) <= TOL_BF16 and max_norm_err(s, s_ref) <= TOL_BF16
    inp["state_in"] = None
    check("wkv6_prefill_bf16_f32out", inp, TOL_BF16)


@pytest.mark.parametrize("entry", ["wkv6_prefill_bf16", "wkv6_finch_c2_prefill_bf16"])
def test_result_does_not_depend_on_placement(gpu_device, entry):
    """The same call with its tensors at the library's staggered arena offsets (bases that differ in
    address bits 7..9) and with ordinary, equally aligned tensors: identical bits."""
    from gpu_util import in_arena
    import paper_2407_12077_amd as wkv
    from paper_2407_12077_amd.workloads import make_uprime
    cfg = scaled(CONFIGS[2], B=3, T=700, H=12)
    inp = make_inputs(cfg, seed=77)
    c2 = "finch_c2" in entry
    B, T, H, N = inp["r"].shape
    names = ["r", "k", "v", "x"]
    if c2:
        inp["uprime"] = make_uprime(cfg, seed=78)
        names.append("uprime")
    plain = [to_dev(inp[n], torch.bfloat16) for n in names]
    u = to_dev(inp["u"], torch.float32)
    outs = []
    for staggered in (False, True):
        out = torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        if staggered:
            arena, views = in_arena(plain + [out])
            ins, out = views[:-1], views[-1]
            assert len({v.data_ptr() % 1024 for v in views}) == len(views)
        else:
            ins = plain
        s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
        getattr(wkv, entry)(B, T, H, N, ins[0], ins[1], ins[2], ins[3], ins[4] if c2 else u, None, out, s_out)
        torch.cuda.synchronize()
        outs.append((out.clone(), s_out))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert torch.isfinite(outs[0][0].float()).all()


def test_split_result_does_not_depend_on_placement(gpu_device):
    """The token split (three launches, caller workspace) with its tensors at the library's staggered
    arena offsets and with ordinary tensors: identical bits, out and final state."""
    from gpu_util import in_arena
    import paper_2407_12077_amd as wkv
    cfg = scaled(CONFIGS[3], T=3000, H=4)
    inp = make_inputs(cfg, seed=91)
    B, T, H, N = inp["r"].shape
    plain = [to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x")]
    u = to_dev(inp["u"], torch.float32)
    segments = 5
    ws_bytes = wkv.wkv6_split_workspace_bytes(B, T, H, N, segments)
    results = []
    for staggered in (False, True):
        out = torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        ins = plain
        if staggered:
            arena, views = in_arena(plain + [out])
            ins, out = views[:-1], views[-1]
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
        wkv.wkv6_prefill_bf16_split(B, T, H, N, ins[0], ins[1], ins[2], ins[3], u, None, out, s_out,
                                    wkv.WKV6_DTYPE_BF16, segments, ws, ws_bytes)
        torch.cuda.synchronize()
        results.append((out.clone(), s_out))
    assert torch.equal(results[0][0], results[1][0]) and torch.equal(results[0][1], results[1][1])
    assert torch.isfinite(results[0][0].float()).all() and torch.isfinite(results[0][1]).all()
