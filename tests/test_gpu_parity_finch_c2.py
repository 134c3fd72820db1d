"""GPU parity of the fused Finch-C2 entry points against the fp64 oracle (Method section,
Finch-C2 Time Mixing: k_t = kbar_t (1 - w_t), o_t = r_t . wkv_t + u'_t), through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from oracle import finch_c2_oracle
from paper_2407_12077_amd.workloads import CONFIGS, make_inputs, make_uprime, round_to_bf16, scaled

from gpu_util import BF16_OUT_ROUNDING, TOL_BF16, max_norm_err, to_dev

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


def test_full_size_config2_sampled_units(gpu_device):
    """The benchmark's launch configuration at full size; the oracle recomputes a seeded sample
    of (batch, head) units in full."""
    cfg = CONFIGS[2]
    inp = inputs(cfg)
    B, T, H, N = inp["r"].shape
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    out = torch.empty((B, T, H, N), dtype=torch.bfloat16, device="cuda")
    s_out = torch.empty((B, H, N, N), dtype=torch.float32, device="cuda")
    wkv.wkv6_finch_c2_prefill_bf16(B, T, H, N, r, k, v, x, up, None, out, s_out)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(s_out).all()
    rng = np.random.default_rng(2002)
    units = {(0, 0), (B - 1, H - 1)}
    while len(units) < 10:
        units.add((int(rng.integers(B)), int(rng.integers(H))))
    worst_o = worst_s = 0.0
    for (b, h) in sorted(units):
        sl = lambda a: np.ascontiguousarray(a[b:b + 1, :, h:h + 1])
        o_ref, s_ref = finch_c2_oracle(sl(inp["r"]), sl(inp["k"]), sl(inp["v"]), sl(inp["x"]), sl(inp["uprime"]),
                                       None, nthreads=1)
        worst_o = max(worst_o, max_norm_err(out[b, :, h].float().cpu().numpy(), o_ref[0, :, 0]))
        worst_s = max(worst_s, max_norm_err(s_out[b, h].cpu().numpy(), s_ref[0, 0]))
    print(f"finch-c2 config 2: {len(units)} units, worst err_out={worst_o:.3e} err_state={worst_s:.3e}", flush=True)
    assert worst_o <= TOL_BF16 + BF16_OUT_ROUNDING and worst_s <= TOL_BF16


@pytest.mark.parametrize("B,T,H", [(70, 45, 4), (300, 20, 3)])
def test_many_units_per_workgroup(gpu_device, B, T, H):
    inp = inputs(scaled(CONFIGS[4], B=B, T=T, H=H))
    check(inp)
    o32, _ = run_c2(inp, torch.float32)
    o16, _ = run_c2(inp, torch.bfloat16)
    assert np.array_equal(o16.astype(np.float32), round_to_bf16(o32.astype(np.float32)))
