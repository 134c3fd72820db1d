"""The token-split entry point that allocates nothing (its per-segment states live in a buffer that
is part of the library's code object) against the entry point that takes a caller workspace: same
kernels, same order, so every output element and the final state must agree bit for bit, and both
must sit within the stated tolerance of the fp64 oracle.  Two calls in a row share the library's
buffer, the second with a smaller input, so stale contents of the first would show."""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from gpu_util import TOL_BF16, max_norm_err, to_dev
from oracle import wkv6_oracle
from paper_2407_12077_amd.workloads import CONFIGS, make_inputs, scaled

pytestmark = pytest.mark.gpu


def _both(inp, segments):
    B, T, H, N = inp["r"].shape
    r, k, v, x = (to_dev(inp[n], torch.bfloat16) for n in ("r", "k", "v", "x"))
    u = to_dev(inp["u"], torch.float32)
    s_in = to_dev(inp.get("state_in"), torch.float32)
    res = []
    for noalloc in (True, False):
        out = torch.full((B, T, H, N), float("nan"), dtype=torch.float32, device="cuda")
        s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda")
        if noalloc:
            wkv.wkv6_prefill_bf16_split_noalloc(B, T, H, N, r, k, v, x, u, s_in, out, s_out, wkv.WKV6_DTYPE_F32,
                                                segments)
        else:
            nbytes = wkv.wkv6_split_workspace_bytes(B, T, H, N, segments)
            ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
            wkv.wkv6_prefill_bf16_split(B, T, H, N, r, k, v, x, u, s_in, out, s_out, wkv.WKV6_DTYPE_F32, segments,
                                        ws, nbytes)
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), s_out.cpu().numpy()))
    return res


def test_noalloc_split_twice_second_call_smaller(gpu_device):
    # first call: 2 x 7 segments x 6 heads with an entering state; second call: fewer, shorter segments
    shapes = [dict(B=2, T=1500, H=6, segments=7, cfg=4), dict(B=1, T=333, H=3, segments=3, cfg=2)]
    for i, sh in enumerate(shapes):
        inp = make_inputs(scaled(CONFIGS[sh["cfg"]], B=sh["B"], T=sh["T"], H=sh["H"]), seed=70 + i)
        print(f"noalloc split call {i}: B={sh['B']} T={sh['T']} H={sh['H']} segments={sh['segments']}", flush=True)
        (o_na, s_na), (o_ws, s_ws) = _both(inp, sh["segments"])
        assert np.array_equal(o_na, o_ws) and np.array_equal(s_na, s_ws)
        o_ref, s_ref = wkv6_oracle(**inp)
        eo, es = max_norm_err(o_na, o_ref), max_norm_err(s_na, s_ref)
        print(f"  err_out={eo:.3e} err_state={es:.3e}", flush=True)
        assert eo <= TOL_BF16 and es <= TOL_BF16


def test_noalloc_split_rejects_shapes_beyond_its_buffer(gpu_device):
    # 8 x 16 segments x 32 heads needs 68 MB of per-segment states: refused before anything is enqueued
    B, T, H, N, segments = 8, 16 * 64, 32, 64, 16
    assert wkv.wkv6_split_workspace_bytes(B, T, H, N, segments) > (8 << 20)
    t = torch.zeros((B, T, H, N), dtype=torch.bfloat16, device="cuda")
    u = torch.zeros((H, N), dtype=torch.float32, device="cuda")
    out = torch.full((B, T, H, N), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(wkv.Wkv6Error) as e:
        wkv.wkv6_prefill_bf16_split_noalloc(B, T, H, N, t, t, t, t, u, None, out, None, wkv.WKV6_DTYPE_BF16, segments)
    assert e.value.status == 6
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
