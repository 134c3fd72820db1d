"""GPU parity of the key-compression entry point against the fp64 oracle (Method section, GOLD
Key Compression: c_t = x_t W^KD).  bf16 products are exact in fp32 and the accumulation is fp32,
so the fp32 output is held to 1e-5 (max-normalised) and the bf16 output must be the fp32 output
rounded once."""
import numpy as np
import pytest
import torch

import paper_2407_12077_amd as wkv
from oracle import key_compress_oracle
from paper_2407_12077_amd.workloads import make_key_compress_inputs, round_to_bf16

from gpu_util import max_norm_err, to_dev

pytestmark = pytest.mark.gpu


def run(x, w, out_dtype):
    M, D = x.shape
    xd, wd = to_dev(x, torch.bfloat16), to_dev(w, torch.bfloat16)
    c = torch.full((M, D // 16), float("nan"), dtype=out_dtype, device="cuda")
    code = wkv.WKV6_DTYPE_F32 if out_dtype == torch.float32 else wkv.WKV6_DTYPE_BF16
    wkv.wkv6_key_compress_bf16(M, D, xd, wd, c, code)
    torch.cuda.synchronize()
    return c.float().cpu().numpy()


@pytest.mark.parametrize("M,D", [(1, 2048), (127, 2048), (128, 2048), (129, 2048), (1000, 2048), (300, 4096), (200, 256),
                                 (333, 768), (500, 1024), (130, 2304), (1100, 4096)])
def test_matches_oracle(gpu_device, M, D):
    x, w = make_key_compress_inputs(M, D, seed=500 + M)
    ref = key_compress_oracle(x, w)
    c32 = run(x, w, torch.float32)
    assert max_norm_err(c32, ref) <= 1e-5
    c16 = run(x, w, torch.bfloat16)
    assert np.array_equal(c16, round_to_bf16(c32))


def test_selector_matrix_copies_channels(gpu_device):
    """W with one 1 per column: every output is one bf16 input copied exactly."""
    M, D = 200, 2048
    x, _ = make_key_compress_inputs(M, D, seed=77)
    pick = np.random.default_rng(78).integers(0, D, D // 16)
    w = np.zeros((D, D // 16), np.float32)
    w[pick, np.arange(D // 16)] = 1.0
    assert np.array_equal(run(x, w, torch.bfloat16), x[:, pick])


def test_empty_and_validation(gpu_device):
    z = torch.zeros((4, 2048), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((2048, 128), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    wkv.wkv6_key_compress_bf16(0, 2048, None, None, None, wkv.WKV6_DTYPE_BF16)
    for args, status in [((4, 1000, z, w, c, 0), 3), ((4, 2048, z, w, c, 9), 3), ((4, 2048, None, w, c, 0), 1),
                         ((-1, 2048, z, w, c, 0), 2)]:
        with pytest.raises(wkv.Wkv6Error) as e:
            wkv.wkv6_key_compress_bf16(*args)
        assert e.value.status == status


@pytest.mark.parametrize("M,D", [(32768, 2048), (65536, 4096)])
def test_full_size_every_row(gpu_device, M, D):
    """The benchmark's sizes (the tokens of config 2 at D = 2048 and of config 5 at D = 4096):
    every row against the oracle."""
    x, w = make_key_compress_inputs(M, D)
    print(f"key compression M={M} D={D}: oracle on every row ...", flush=True)
    ref = key_compress_oracle(x, w)
    c32 = run(x, w, torch.float32)
    err = max_norm_err(c32, ref)
    rows = np.abs(c32 - ref).max(axis=1) / np.abs(ref).max(axis=1)
    print(f"key compression M={M} D={D}: global={err:.3e} worst row={rows.max():.3e} "
          f"rel_l2={np.linalg.norm(c32 - ref) / np.linalg.norm(ref):.3e}", flush=True)
    assert err <= 1e-5 and rows.max() <= 1e-5
    c16 = run(x, w, torch.bfloat16)
    assert np.array_equal(c16, round_to_bf16(c32))


def test_input_beyond_four_gib(gpu_device):
    """x of 4.83 GB (1 179 648 tokens of width 2048, drawn on the device from a seed): byte offsets into x
    pass 2^32.  The first, a middle and the last row tile are compared with the oracle."""
    M, D = 9216 * 128, 2048
    _, w = make_key_compress_inputs(16, D, seed=77)
    gen = torch.Generator(device="cuda").manual_seed(99)
    x = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
    for m0 in range(0, M, 65536):
        x[m0:m0 + 65536] = torch.randn((65536, D), generator=gen, device="cuda").to(torch.bfloat16)
    assert x.numel() * 2 > (1 << 32)
    wd = to_dev(w, torch.bfloat16)
    c = torch.full((M, D // 16), float("nan"), dtype=torch.float32, device="cuda")
    wkv.wkv6_key_compress_bf16(M, D, x, wd, c, wkv.WKV6_DTYPE_F32)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(c).all())
    for m0 in (0, (M // 2 // 128) * 128 + 64, M - 128):
        ref = key_compress_oracle(x[m0:m0 + 128].float().cpu().numpy(), w)
        err = max_norm_err(c[m0:m0 + 128].cpu().numpy(), ref)
        print(f"rows {m0}..{m0 + 127}: err={err:.3e}", flush=True)
        assert err <= 1e-5
    del x, c
    torch.cuda.empty_cache()
