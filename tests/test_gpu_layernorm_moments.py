"""GPU parity of the Finch-C2 prefill that emits the partial statistics of the LayerNorm over all
heads (Method section, Finch-C2 Time Mixing, output equation), and of their fold into each
token's mean and 1/sqrt(var + eps), against the fp64 oracles, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from oracle import finch_c2_oracle, head_moments_numpy, layernorm_heads_numpy
from paper_2407_12077_amd.workloads import CONFIGS, make_inputs, make_uprime, round_to_bf16, scaled

from gpu_util import BF16_OUT_ROUNDING, TOL_BF16, max_norm_err, to_dev

pytestmark = pytest.mark.gpu
EPS = 1e-5


def inputs(cfg, seed=None):
    inp = make_inputs(cfg, seed)
    inp["uprime"] = make_uprime(cfg, seed)
    return inp


def run_moments(inp, eps=EPS):
    B, T, H, N = inp["r"].shape
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    s_in = to_dev(inp.get("state_in"), torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    mom = torch.full((B, H, T, 2), float("nan"), dtype=torch.float32, device="cuda")
    s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
    mr = torch.full((B, T, 2), float("nan"), dtype=torch.float32, device="cuda")
    wkv.wkv6_finch_c2_prefill_bf16_moments(B, T, H, N, r, k, v, x, up, s_in, out, mom, s_out)
    wkv.wkv6_layernorm_finalize(B, T, H, N, mom, eps, mr)
    # the plain entry on the same inputs: same kernel arithmetic, so the same bits
    out0 = torch.empty_like(out)
    s_out0 = torch.empty_like(s_out)
    wkv.wkv6_finch_c2_prefill_bf16(B, T, H, N, r, k, v, x, up, s_in, out0, s_out0)
    torch.cuda.synchronize()
    assert torch.equal(out, out0) and torch.equal(s_out, s_out0)
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    return f64(out), f64(mom), f64(mr), f64(s_out)


def check(inp, eps=EPS, rows=True):
    """Every output element is within delta = TOL_BF16 max|o| of the oracle (the parity bar), so:
    a head's sum of N values is within N delta; each deviation from the head mean within 2 delta,
    hence |m2 - m2_ref| <= sum (2 |dev| 2 delta + (2 delta)^2) <= 4 delta sqrt(N m2_ref) + 4 N delta^2.
    The normalised rows built from the GPU's bf16 output, mean and rstd meet the output's own bar."""
    B, T, H, N = inp["r"].shape
    o_ref, s_ref = finch_c2_oracle(inp["r"], inp["k"], inp["v"], inp["x"], inp["uprime"], inp.get("state_in"))
    sum_ref, m2_ref = head_moments_numpy(o_ref)
    out, mom, mr, s_out = run_moments(inp, eps)
    assert np.isfinite(mom).all() and np.isfinite(mr).all()
    delta = TOL_BF16 * np.abs(o_ref).max()
    assert np.abs(mom[..., 0] - sum_ref).max() <= N * delta
    assert (np.abs(mom[..., 1] - m2_ref) <= 4 * delta * np.sqrt(N * m2_ref) + 4 * N * delta ** 2).all()
    assert max_norm_err(s_out, s_ref) <= TOL_BF16
    rng = np.random.default_rng(7)
    gamma, beta = rng.standard_normal(H * N), rng.standard_normal(H * N)
    y_ref, mean_ref, rstd_ref = layernorm_heads_numpy(o_ref, gamma, beta, eps)
    y = ((out - mr[:, :, None, None, 0]) * mr[:, :, None, None, 1]) * gamma.reshape(H, N) + beta.reshape(H, N)
    e_mean = np.abs(mr[..., 0] - mean_ref).max() / np.abs(o_ref).max()
    e_rstd = np.abs(mr[..., 1] / rstd_ref - 1.0).max()
    e_y = max_norm_err(y, y_ref) if rows else 0.0
    assert e_mean <= TOL_BF16 and e_rstd <= TOL_BF16 and e_y <= TOL_BF16 + BF16_OUT_ROUNDING, (e_mean, e_rstd, e_y)
    return e_mean, e_rstd, e_y


@pytest.mark.parametrize("T", [1, 2, 31, 32, 33, 65, 100, 257])
def test_lengths(gpu_device, T):
    check(inputs(scaled(CONFIGS[2], B=2, T=T, H=3)))


@pytest.mark.parametrize("cfg_index", [2, 4, 5])
def test_reduced_configs(gpu_device, cfg_index):
    dims = {2: dict(B=2, T=700, H=4), 4: dict(B=5, T=512, H=3), 5: dict(B=1, T=1500, H=6)}[cfg_index]
    e = check(inputs(scaled(CONFIGS[cfg_index], **dims)))
    print(f"layernorm partials, reduced config {cfg_index}: err mean={e[0]:.2e} rstd={e[1]:.2e} y={e[2]:.2e}", flush=True)


@pytest.mark.parametrize("B,T,H", [(70, 45, 4), (300, 20, 3), (5, 40, 96)])
def test_many_units_per_workgroup(gpu_device, B, T, H):
    check(inputs(scaled(CONFIGS[4], B=B, T=T, H=H)))


def test_single_head(gpu_device):
    check(inputs(scaled(CONFIGS[2], B=3, T=50, H=1)))


def test_large_common_offset(gpu_device):
    """Second value 100 + noise: every head's mean is ~100 and its spread ~1; squared deviations
    taken from the head's own mean keep the variance (a raw sum of squares in fp32 would lose it).
    The bf16 output itself has a spacing of 0.5 at 100, so the normalised rows are not compared."""
    inp = inputs(scaled(CONFIGS[2], B=2, T=70, H=4))
    inp["uprime"] = round_to_bf16((inp["uprime"] + 100.0).astype(np.float32))
    e = check(inp, rows=False)
    assert e[1] <= 2e-4, e                        # rstd to better than the loose bar: no cancellation


def test_constant_rows_give_rstd_from_eps(gpu_device):
    """r = 0 and a constant second value: every token's D values are equal, variance 0."""
    inp = inputs(scaled(CONFIGS[2], B=1, T=40, H=2))
    inp["r"][:] = 0.0
    inp["uprime"][:] = 2.5
    _, mom, mr, _ = run_moments(inp, eps=1e-4)
    np.testing.assert_array_equal(mom[..., 0], 160.0)
    np.testing.assert_array_equal(mom[..., 1], 0.0)
    np.testing.assert_array_equal(mr[..., 0], 2.5)
    np.testing.assert_allclose(mr[..., 1], 100.0, rtol=1e-6)


def test_finalize_alone_against_the_oracle(gpu_device):
    """The fold on its own: partial moments from the oracle (rounded to fp32) in, token statistics
    out; fp32 arithmetic over H heads, so 1e-5 relative."""
    rng = np.random.default_rng(11)
    for (B, T, H) in [(1, 1, 1), (2, 300, 32), (3, 513, 7)]:
        o = rng.standard_normal((B, T, H, 64)) * rng.uniform(0.2, 4.0, (B, T, 1, 1)) + rng.standard_normal((B, 1, H, 1)) * 2.0
        s, m2 = head_moments_numpy(o)
        mom = np.stack([s, m2], axis=-1).astype(np.float32)
        s32, m232 = mom[..., 0].astype(np.float64), mom[..., 1].astype(np.float64)
        D = H * 64
        mean_ref = s32.sum(axis=1) / D                     # the identity of the partials, in fp64
        var_ref = (m232.sum(axis=1) + 64 * ((s32 / 64 - mean_ref[:, None, :]) ** 2).sum(axis=1)) / D
        _, mean_o, rstd_o = layernorm_heads_numpy(o, np.ones(D), np.zeros(D), EPS)
        np.testing.assert_allclose(mean_ref, mean_o, atol=1e-5)           # rounding the partials to fp32
        np.testing.assert_allclose(1 / np.sqrt(var_ref + EPS), rstd_o, rtol=1e-5)
        mr = torch.full((B, T, 2), float("nan"), dtype=torch.float32, device="cuda")
        wkv.wkv6_layernorm_finalize(B, T, H, 64, torch.from_numpy(mom).cuda(), EPS, mr)
        torch.cuda.synchronize()
        mr = mr.cpu().numpy().astype(np.float64)
        np.testing.assert_allclose(mr[..., 0], mean_o, atol=1e-5 * np.abs(o).max())
        np.testing.assert_allclose(mr[..., 1], rstd_o, rtol=1e-5)


def test_full_size_config2_sampled_units(gpu_device):
    """The benchmark's launch configuration at full size: the partial moments of a seeded sample
    of (batch, head) units against the oracle's."""
    cfg = CONFIGS[2]
    inp = inputs(cfg)
    B, T, H, N = inp["r"].shape
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    out = torch.empty((B, T, H, N), dtype=torch.bfloat16, device="cuda")
    mom = torch.full((B, H, T, 2), float("nan"), dtype=torch.float32, device="cuda")
    mr = torch.full((B, T, 2), float("nan"), dtype=torch.float32, device="cuda")
    wkv.wkv6_finch_c2_prefill_bf16_moments(B, T, H, N, r, k, v, x, up, None, out, mom, None)
    wkv.wkv6_layernorm_finalize(B, T, H, N, mom, EPS, mr)
    torch.cuda.synchronize()
    assert torch.isfinite(mom).all() and torch.isfinite(mr).all()
    rng = np.random.default_rng(2003)
    units = {(0, 0), (B - 1, H - 1)}
    while len(units) < 8:
        units.add((int(rng.integers(B)), int(rng.integers(H))))
    for (b, h) in sorted(units):
        sl = lambda a: np.ascontiguousarray(a[b:b + 1, :, h:h + 1])
        o_ref, _ = finch_c2_oracle(sl(inp["r"]), sl(inp["k"]), sl(inp["v"]), sl(inp["x"]), sl(inp["uprime"]),
                                   None, nthreads=1)
        s_ref, m2_ref = head_moments_numpy(o_ref)
        got = mom[b, h].cpu().numpy().astype(np.float64)
        delta = TOL_BF16 * np.abs(o_ref).max()
        assert np.abs(got[:, 0] - s_ref[0, 0]).max() <= N * delta
        assert (np.abs(got[:, 1] - m2_ref[0, 0]) <= 4 * delta * np.sqrt(N * m2_ref[0, 0]) + 4 * N * delta ** 2).all()
    # the fold of all 32 heads of a few tokens, from the GPU's own partials re-folded in fp64 by the identity
    m = mom.cpu().numpy().astype(np.float64)
    mean = m[..., 0].sum(axis=1) / (H * N)
    var = (m[..., 1].sum(axis=1) + N * ((m[..., 0] / N - mean[:, None, :]) ** 2).sum(axis=1)) / (H * N)
    got = mr.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(got[..., 0], mean, atol=1e-5 * np.abs(m[..., 0]).max() / N)
    np.testing.assert_allclose(got[..., 1], 1 / np.sqrt(var + EPS), rtol=1e-5)


def test_validation(gpu_device):
    B, T, H, N = 1, 8, 2, 64
    z = torch.zeros((B, T, H, N), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(z)
    mom = torch.empty((B, H, T, 2), dtype=torch.float32, device="cuda")
    with pytest.raises(wkv.Wkv6Error):                         # no moments buffer
        wkv.wkv6_finch_c2_prefill_bf16_moments(B, T, H, N, z, z, z, z, z, None, out, None, None)
    with pytest.raises(wkv.Wkv6Error):                         # head size
        wkv.wkv6_layernorm_finalize(B, T, H, 32, mom, EPS, mom)
    with pytest.raises(wkv.Wkv6Error):                         # negative eps
        wkv.wkv6_layernorm_finalize(B, T, H, N, mom, -1.0, mom)
    with pytest.raises(wkv.Wkv6Error):                         # missing output
        wkv.wkv6_layernorm_finalize(B, T, H, N, mom, EPS, None)
    wkv.wkv6_layernorm_finalize(B, 0, H, N, None, EPS, None)   # nothing to do
    wkv.wkv6_finch_c2_prefill_bf16_moments(B, 0, H, N, None, None, None, None, None, None, None, None, None)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ the statistics applied on the GPU
def run_applied(inp, gamma, beta, out_dtype, eps=EPS, in_place=False):
    """prefill with partial moments -> fold -> wkv6_layernorm_apply_bf16, all on the GPU."""
    B, T, H, N = inp["r"].shape
    r, k, v, x, up = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x", "uprime"))
    s_in = to_dev(inp.get("state_in"), torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    mom = torch.full((B, H, T, 2), float("nan"), dtype=torch.float32, device="cuda")
    mr = torch.full((B, T, 2), float("nan"), dtype=torch.float32, device="cuda")
    g, bt = to_dev(gamma, torch.float32), to_dev(beta, torch.float32)
    y = out.view(B, T, H * N) if in_place else torch.full((B, T, H * N), float("nan"), dtype=out_dtype, device="cuda")
    wkv.wkv6_finch_c2_prefill_bf16_moments(B, T, H, N, r, k, v, x, up, s_in, out, mom, None)
    wkv.wkv6_layernorm_finalize(B, T, H, N, mom, eps, mr)
    code = wkv.WKV6_DTYPE_F32 if out_dtype == torch.float32 else wkv.WKV6_DTYPE_BF16
    wkv.wkv6_layernorm_apply_bf16(B, T, H, N, out, mr, g, bt, y, code)
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64).reshape(B, T, H, N)


@pytest.mark.parametrize("dims", [dict(B=2, T=333, H=4), dict(B=1, T=70, H=32), dict(B=3, T=1, H=2), dict(B=1, T=1000, H=12)])
def test_layernorm_applied_end_to_end(gpu_device, dims):
    """From r, kbar, v, x, u' to LayerNorm(concat(heads)) with gain and offset, against the chained
    oracles finch_c2_oracle -> layernorm_heads_numpy.  The read-outs pass through bf16 between the two
    GPU kernels (that is the interface tensor), so the bar is the output's own (2e-3 + 2^-8), taken
    relative to the largest normalised value; the bf16 result carries one more rounding."""
    inp = inputs(scaled(CONFIGS[2], **dims), seed=31)
    B, T, H, N = inp["r"].shape
    rng = np.random.default_rng(32)
    gamma = (1.0 + 0.3 * rng.standard_normal(H * N)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(H * N)).astype(np.float32)
    o_ref, _ = finch_c2_oracle(inp["r"], inp["k"], inp["v"], inp["x"], inp["uprime"], None)
    y_ref, _, _ = layernorm_heads_numpy(o_ref, gamma, beta, EPS)
    y32 = run_applied(inp, gamma, beta, torch.float32)
    e32 = max_norm_err(y32, y_ref)
    y16 = run_applied(inp, gamma, beta, torch.bfloat16)
    e16 = max_norm_err(y16, y_ref)
    print(f"applied layernorm {dims}: fp32 out err={e32:.3e}, bf16 out err={e16:.3e}", flush=True)
    assert e32 <= TOL_BF16 + BF16_OUT_ROUNDING and e16 <= TOL_BF16 + 2 * BF16_OUT_ROUNDING
    assert np.array_equal(y16, round_to_bf16(y32.astype(np.float32)).astype(np.float64))
    # in place over the read-outs (bf16)
    assert np.array_equal(run_applied(inp, gamma, beta, torch.bfloat16, in_place=True), y16)
    # the normalised rows have the statistics a LayerNorm promises (gain 1, offset 0)
    y_plain = run_applied(inp, np.ones(H * N, np.float32), np.zeros(H * N, np.float32), torch.float32)
    flat = y_plain.reshape(B, T, H * N)
    assert np.abs(flat.mean(axis=2)).max() <= 5e-3 and np.abs(flat.var(axis=2) - 1.0).max() <= 2e-2


def test_layernorm_apply_validation(gpu_device):
    o = torch.zeros((1, 8, 2, 64), dtype=torch.bfloat16, device="cuda")
    mr = torch.zeros((1, 8, 2), dtype=torch.float32, device="cuda")
    g = torch.ones(128, dtype=torch.float32, device="cuda")
    y = torch.zeros((1, 8, 128), dtype=torch.bfloat16, device="cuda")
    wkv.wkv6_layernorm_apply_bf16(1, 8, 2, 64, o, mr, g, g, y, wkv.WKV6_DTYPE_BF16)
    wkv.wkv6_layernorm_apply_bf16(0, 8, 2, 64, None, None, None, None, None, wkv.WKV6_DTYPE_BF16)
    for args, status in [((1, 8, 2, 32, o, mr, g, g, y, 0), 3), ((1, 8, 2, 64, o, mr, g, g, y, 7), 3),
                         ((1, 8, 0, 64, o, mr, g, g, y, 0), 2), ((1, 8, 2, 64, o, None, g, g, y, 0), 1)]:
        with pytest.raises(wkv.Wkv6Error) as e:
            wkv.wkv6_layernorm_apply_bf16(*args)
        assert e.value.status == status
