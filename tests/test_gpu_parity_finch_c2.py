"""GPU parity of the fused Finch-C2 entry points against the fp64 oracle (Method section,
Finch-C2 Time Mixing: k_t = kbar_t (1 - w_t), o_t = r_t . wkv_t + u'_t), through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from oracle import finch_c2_oracle
from paper_2407_12077_amd.workloads import CONFIGS, make_inputs, make_uprime, round_to_bf16, scaled

from gpu_util import BF16_OUT_ROUNDING, TOL_BF16, error_report, fmt_report, max_norm_err, to_dev

pytestmark = pytest.mark.gpu


def inputs(cfg, seed=None):
    inp = make_inputs(cfg, seed)
    inp["uprime"] = make_uprime(cfg, seed)
    return inp


def run_c2(inp, out_dtype=torch.float32, want_state=True, entry=None):
    B, T, H, N = inp["r"].shape
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    s_in = to_dev(inp.get("state_in"), torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=out_dtype, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda") if want_state else None
    if entry is None:
        entry = "wkv6_finch_c2_prefill_bf16_f32out" if out_dtype == torch.float32 else "wkv6_finch_c2_prefill_bf16"
    getattr(wkv, entry)(B, T, H, N, r, k, v, x, up, s_in, out, s_out)
    torch.cuda.synchronize()
    o = out.float().cpu().numpy().astype(np.float64)
    return o, (None if s_out is None else s_out.cpu().numpy().astype(np.float64))


def oracle(inp):
    return finch_c2_oracle(inp["r"], inp["k"], inp["v"], inp["x"], inp["uprime"], inp.get("state_in"))


def check(inp, tol=TOL_BF16):
    o_ref, s_ref = oracle(inp)
    o, s = run_c2(inp)
    eo, es = max_norm_err(o, o_ref), max_norm_err(s, s_ref)
    assert eo <= tol and es <= tol, (eo, es)
    return eo, es


@pytest.mark.parametrize("T", [1, 2, 7, 31, 32, 33, 63, 64, 65, 96, 97, 129, 200, 1000])
def test_lengths(gpu_device, T):
    check(inputs(scaled(CONFIGS[2], B=2, T=T, H=3)))


@pytest.mark.parametrize("cfg_index", [2, 4, 5])
def test_reduced_configs(gpu_device, cfg_index):
    dims = {2: dict(B=2, T=700, H=4), 4: dict(B=5, T=512, H=3), 5: dict(B=1, T=1500, H=6)}[cfg_index]
    eo, es = check(inputs(scaled(CONFIGS[cfg_index], **dims)))
    print(f"finch-c2 reduced config {cfg_index}: err_out={eo:.3e} err_state={es:.3e}", flush=True)


def test_bf16_output_is_the_fp32_result_rounded_once(gpu_device):
    inp = inputs(scaled(CONFIGS[4], B=3, T=333, H=2))
    o32, s32 = run_c2(inp, torch.float32)
    o16, s16 = run_c2(inp, torch.bfloat16)
    assert np.array_equal(o16.astype(np.float32), round_to_bf16(o32.astype(np.float32)))
    assert np.array_equal(s16, s32)
    o_ref, _ = oracle(inp)
    assert max_norm_err(o16, o_ref) <= TOL_BF16 + BF16_OUT_ROUNDING


def test_uprime_only(gpu_device):
    """r = 0: the output is u' exactly (bf16 values survive the fp32 add and the rounding)."""
    inp = inputs(scaled(CONFIGS[2], B=1, T=150, H=2))
    inp["r"] = np.zeros_like(inp["r"])
    o, _ = run_c2(inp, torch.bfloat16)
    assert np.array_equal(o.astype(np.float32), inp["uprime"])


@pytest.mark.parametrize("xval", [-np.inf, np.inf, 20.0, -30.0])
def test_constant_extreme_decay(gpu_device, xval):
    inp = inputs(scaled(CONFIGS[4], B=1, T=100, H=2))
    inp["x"] = np.full_like(inp["x"], xval)
    check(inp)


def test_mixed_extreme_decays(gpu_device):
    inp = inputs(scaled(CONFIGS[4], B=2, T=260, H=2))
    rng = np.random.default_rng(5)
    pick = rng.integers(0, 6, inp["x"].shape)
    x = inp["x"].copy()
    x[pick == 0] = -np.inf
    x[pick == 1] = np.inf
    x[pick == 2] = 12.0
    inp["x"] = x
    check(inp)


def test_state_passing_with_the_strided_entry(gpu_device):
    """Tokens [0, cut) and [cut, T) of one buffer, the second call from the carried state, equal
    one call over [0, T) (cut on a chunk boundary: same arithmetic; elsewhere: to tolerance)."""
    inp = inputs(scaled(CONFIGS[4], B=3, T=300, H=2))
    B, T, H, N = inp["r"].shape
    o_full, s_full = run_c2(inp)
    o_ref, s_ref = oracle(inp)
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    s_in = to_dev(inp["state_in"], torch.float32)
    for cut in (128, 77):
        out = torch.full((B, T, H, N), float("nan"), dtype=torch.float32, device="cuda")
        s_mid = torch.empty((B, H, N, N), dtype=torch.float32, device="cuda")
        s_end = torch.empty_like(s_mid)
        stride = T * H * N
        wkv.wkv6_finch_c2_prefill_bf16_strided(B, cut, H, N, r, k, v, x, up, s_in, out, s_mid, stride,
                                               wkv.WKV6_DTYPE_F32)
        off = cut * H * N
        tail = lambda t: t.view(-1)[off:]
        wkv.wkv6_finch_c2_prefill_bf16_strided(B, T - cut, H, N, tail(r), tail(k), tail(v), tail(x), tail(up),
                                               s_mid, tail(out), s_end, stride, wkv.WKV6_DTYPE_F32)
        torch.cuda.synchronize()
        o = out.cpu().numpy().astype(np.float64)
        s = s_end.cpu().numpy().astype(np.float64)
        assert max_norm_err(o, o_ref) <= TOL_BF16 and max_norm_err(s, s_ref) <= TOL_BF16
        if cut % 32 == 0:
            assert max_norm_err(o, o_full) <= 1e-6 and max_norm_err(s, s_full) <= 1e-6


@pytest.mark.parametrize("T,segments", [(4096, 4), (1000, 7), (333, 3), (40, 8)])
def test_split_matches_oracle(gpu_device, T, segments):
    inp = inputs(scaled(CONFIGS[4], B=2, T=T, H=2))
    B, T, H, N = inp["r"].shape
    o_ref, s_ref = oracle(inp)
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    s_in = to_dev(inp["state_in"], torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=torch.float32, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
    nbytes = wkv.wkv6_split_workspace_bytes(B, T, H, N, segments)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    wkv.wkv6_finch_c2_prefill_bf16_split(B, T, H, N, r, k, v, x, up, s_in, out, s_out, wkv.WKV6_DTYPE_F32,
                                         segments, ws, nbytes)
    torch.cuda.synchronize()
    eo = max_norm_err(out.cpu().numpy(), o_ref)
    es = max_norm_err(s_out.cpu().numpy(), s_ref)
    assert eo <= TOL_BF16 and es <= TOL_BF16, (eo, es)


def test_validation(gpu_device):
    z = torch.zeros((1, 8, 2, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(z)
    with pytest.raises(wkv.Wkv6Error) as e:
        wkv.wkv6_finch_c2_prefill_bf16(1, 8, 2, 64, z, z, z, z, None, None, out, None)
    assert e.value.status == 1
    with pytest.raises(wkv.Wkv6Error) as e:
        wkv.wkv6_finch_c2_prefill_bf16(1, 8, 2, 32, z, z, z, z, z, None, out, None)
    assert e.value.status == 3


def test_empty_sequence_passes_state_through(gpu_device):
    s_in = torch.randn((2, 3, 64, 64), device="cuda")
    s_out = torch.zeros_like(s_in)
    wkv.wkv6_finch_c2_prefill_bf16(2, 0, 3, 64, None, None, None, None, None, s_in, None, s_out)
    torch.cuda.synchronize()
    assert torch.equal(s_in, s_out)


@pytest.mark.parametrize("cfg_index", [2, 5])
def test_full_size_config_every_unit(gpu_device, cfg_index):
    """The benchmark's launch configuration at full size: every output element and final state
    entry of every (batch, head) unit against the oracle, for the bf16-out entry (the benchmarked
    one) and the fp32-out entry."""
    cfg = CONFIGS[cfg_index]
    inp = inputs(cfg)
    B, T, H, N = inp["r"].shape
    print(f"finch-c2 config {cfg_index}: oracle on every unit ...", flush=True)
    o_ref, s_ref = oracle(inp)
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    out = torch.full((B, T, H, N), float("nan"), dtype=torch.float32, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
    wkv.wkv6_finch_c2_prefill_bf16_f32out(B, T, H, N, r, k, v, x, up, None, out, s_out)
    out16 = torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    s_out16 = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
    wkv.wkv6_finch_c2_prefill_bf16(B, T, H, N, r, k, v, x, up, None, out16, s_out16)
    torch.cuda.synchronize()
    rep_o = error_report(out.cpu().numpy(), o_ref, "out")
    rep_s = error_report(s_out.cpu().numpy(), s_ref, "state")
    print(f"finch-c2 config {cfg_index} fp32 out, all {B * H} units: out {fmt_report(rep_o)} | state {fmt_report(rep_s)}",
          flush=True)
    assert rep_o["global"] <= TOL_BF16 and rep_o["unit"] <= TOL_BF16
    assert rep_s["global"] <= TOL_BF16 and rep_s["unit"] <= TOL_BF16
    rep_o16 = error_report(out16.float().cpu().numpy(), o_ref, "out")
    print(f"finch-c2 config {cfg_index} bf16 out, all {B * H} units: out {fmt_report(rep_o16)}", flush=True)
    assert rep_o16["global"] <= TOL_BF16 + BF16_OUT_ROUNDING and rep_o16["unit"] <= TOL_BF16 + BF16_OUT_ROUNDING
    assert torch.equal(s_out16, s_out) and torch.equal(out16, out.to(torch.bfloat16))


@pytest.mark.parametrize("entry", ["wkv6_finch_c2_prefill_bf16_f32out", "wkv6_finch_c2_append_bf16"])
def test_key_factor_of_long_memory_channels(gpu_device, entry):
    """Decay logits in U(-16, -10): w = exp(-exp(x)) is within 5e-5 of 1 and the key factor
    1 - w must not come from subtracting two nearly equal fp32 numbers.  With v = 1 and a
    constant key kbar every state row is kbar (1 - prod_t w_t), compared per key row (each row
    against its own magnitude, so no large row hides a small one).  kbar = 1024 keeps
    kbar (1 - w) inside the normal range of the fp16 operands."""
    B, T, H, N = 2, (100 if "prefill" in entry else 5), 3, 64
    rng = np.random.default_rng(16)
    x = round_to_bf16(rng.uniform(-16.0, -10.0, (B, T, H, N)).astype(np.float32))
    ones = np.ones((B, T, H, N), np.float32)
    inp = {"r": ones * np.float32(0.125), "k": ones * np.float32(1024.0), "v": ones, "x": x,
           "uprime": np.zeros((B, T, H, N), np.float32), "state_in": None}
    o_ref, s_ref = oracle(inp)
    w = np.exp(-np.exp(x.astype(np.float64)))
    closed = 1024.0 * -np.expm1(np.log(w).sum(axis=1))                    # [B, H, N] per key channel
    assert np.allclose(s_ref, closed[..., None] * np.ones(N), rtol=1e-8, atol=0)    # the oracle subtracts in fp64
    if "append" in entry:
        o, s = run_c2(inp, torch.bfloat16, entry=entry)
    else:
        o, s = run_c2(inp, entry=entry)
    rep_s = error_report(s, s_ref, "state")
    print(f"{entry}: long-memory key factor, state {fmt_report(rep_s)}", flush=True)
    assert rep_s["row"] <= TOL_BF16
    tol_o = TOL_BF16 if "prefill" in entry else TOL_BF16 + BF16_OUT_ROUNDING
    assert max_norm_err(o, o_ref) <= tol_o


@pytest.mark.parametrize("B,T,H", [(70, 45, 4), (300, 20, 3)])
def test_many_units_per_workgroup(gpu_device, B, T, H):
    inp = inputs(scaled(CONFIGS[4], B=B, T=T, H=H))
    check(inp)
    o32, _ = run_c2(inp, torch.float32)
    o16, _ = run_c2(inp, torch.bfloat16)
    assert np.array_equal(o16.astype(np.float32), round_to_bf16(o32.astype(np.float32)))
