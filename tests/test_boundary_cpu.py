"""CPU-side checks of the boundary: the C-ABI library loads, exports every symbol the header
declares, and rejects bad arguments before touching a GPU (validation runs first, so these
calls enqueue nothing and need no device)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2407_12077_amd as wkv
from paper_2407_12077_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "wkv6.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wkv6_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = header_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_version_and_status_strings():
    assert wkv.wkv6_version() >= 100
    assert wkv.status_string(0) == "ok"
    for code in range(1, 7):
        assert wkv.status_string(code) not in ("ok", "unknown status")
    assert wkv.status_string(99) == "unknown status"


def _raw(name):
    return getattr(binding.load(), name)


P = ctypes.c_void_p
A = P(0x1000)          # aligned, never dereferenced: validation fails before any launch


@pytest.mark.parametrize("name", ["wkv6_prefill_bf16", "wkv6_prefill_bf16_f32out",
                                  "wkv6_prefill_f32", "wkv6_prefill_bf16_recurrent"])
def test_validation_happens_before_any_launch(name):
    f = _raw(name)
    assert f(1, 8, 2, 32, A, A, A, A, A, None, A, A, None) == 3          # N != 64
    assert f(-1, 8, 2, 64, A, A, A, A, A, None, A, A, None) == 2
    assert f(1, -8, 2, 64, A, A, A, A, A, None, A, A, None) == 2
    assert f(1, 8, 0, 64, A, A, A, A, A, None, A, A, None) == 2
    assert f(1, 8, 2, 64, None, A, A, A, A, None, A, A, None) == 1
    assert f(1, 8, 2, 64, A, A, A, A, None, None, A, A, None) == 1
    assert f(1, 8, 2, 64, A, A, A, A, A, None, None, A, None) == 1
    assert f(1, 8, 2, 64, P(0x1004), A, A, A, A, None, A, A, None) == 5
    assert f(1, 8, 2, 64, A, A, A, A, A, P(0x1008), A, A, None) == 5
    assert f(0, 8, 2, 64, None, None, None, None, A, None, None, None, None) == 0   # empty batch
    assert f(70000, 8, 70000, 64, A, A, A, A, A, None, A, A, None) == 2              # grid overflow


@pytest.mark.parametrize("name", ["wkv6_finch_c2_prefill_bf16", "wkv6_finch_c2_prefill_bf16_f32out"])
def test_finch_c2_validation_happens_before_any_launch(name):
    f = _raw(name)
    assert f(1, 8, 2, 32, A, A, A, A, A, None, A, A, None) == 3          # N != 64
    assert f(1, -8, 2, 64, A, A, A, A, A, None, A, A, None) == 2
    assert f(1, 8, 2, 64, A, None, A, A, A, None, A, A, None) == 1       # kbar
    assert f(1, 8, 2, 64, A, A, A, A, None, None, A, A, None) == 1       # uprime
    assert f(1, 8, 2, 64, A, A, A, A, P(0x1002), None, A, A, None) == 5  # uprime alignment
    assert f(0, 8, 2, 64, None, None, None, None, None, None, None, None, None) == 0
    g = _raw("wkv6_finch_c2_prefill_bf16_strided")
    assert g(2, 8, 2, 64, A, A, A, A, A, None, A, A, 8 * 2 * 64 - 8, 1, None) == 2
    assert g(2, 8, 2, 64, A, A, A, A, A, None, A, A, 8 * 2 * 64, 7, None) == 3


def test_decode_and_append_validation():
    f = _raw("wkv6_decode_bf16")
    assert f(2, 3, 64, A, A, A, A, A, None, A, None) == 1                # state is required
    assert f(2, 3, 32, A, A, A, A, A, A, A, None) == 3
    assert f(2, 0, 64, A, A, A, A, A, A, A, None) == 2
    assert f(2, 3, 64, A, A, A, A, None, A, A, None) == 1                # u
    g = _raw("wkv6_finch_c2_decode_bf16")
    assert g(2, 3, 64, A, A, A, A, None, A, A, None) == 1                # uprime
    assert g(2, 3, 64, A, A, A, A, A, None, A, None) == 1
    h = _raw("wkv6_append_bf16")
    assert h(1, 8, 2, 32, A, A, A, A, A, None, A, A, None) == 3
    assert h(1, 8, 2, 64, A, None, A, A, A, None, A, A, None) == 1
    assert _raw("wkv6_finch_c2_append_bf16")(1, 8, 2, 64, A, A, A, A, None, None, A, A, None) == 1


def test_key_compress_validation():
    f = _raw("wkv6_key_compress_bf16")
    assert f(4, 1000, A, A, A, 0, None) == 3               # D not a multiple of 256
    assert f(4, 2048, A, A, A, 5, None) == 3               # dtype code
    assert f(-4, 2048, A, A, A, 0, None) == 2
    assert f(4, 2048, A, None, A, 0, None) == 1
    assert f(4, 2048, P(0x1008), A, A, 0, None) == 5
    assert f(0, 2048, None, None, None, 0, None) == 0


def test_strided_entry_validation():
    f = _raw("wkv6_prefill_bf16_strided")
    assert f(2, 8, 2, 64, A, A, A, A, A, None, A, A, 8 * 2 * 64 - 8, 1, None) == 2   # stride < T*H*N
    assert f(2, 8, 2, 64, A, A, A, A, A, None, A, A, 8 * 2 * 64 + 4, 1, None) == 5   # stride % 8
    assert f(2, 8, 2, 64, A, A, A, A, A, None, A, A, 8 * 2 * 64, 7, None) == 3       # dtype code


def test_binding_raises_with_status():
    with pytest.raises(wkv.Wkv6Error) as e:
        binding._check(3)
    assert e.value.status == 3


def test_oracle_is_not_reachable_from_the_product():
    """The package must not import the oracle (no CPU fallback)."""
    pkg = os.path.join(ROOT, "paper_2407_12077_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|libwkv6_oracle|wkv6_oracle", text, re.M), \
                    f"{fn} reaches into the oracle"


def test_arena_layout():
    """The placement helper: 4 KiB-aligned slots, tensor i shifted by 128 (i mod 8) bytes, no overlap,
    total a multiple of 4 KiB; rejected argument sets return -1."""
    sizes = [1000, 4096, 1, 0, 134217728, 77, 4097, 5, 12345, 16]
    total, offs = wkv.wkv6_arena_layout(sizes)
    assert total % 4096 == 0 and len(offs) == len(sizes)
    end = 0
    for j, (o, b) in enumerate(zip(offs, sizes)):
        assert o % 4096 == 128 * (j % 8) and o >= end and o - end < 4096 + 1024
        end = o + b
    assert end <= total < end + 4096
    assert {o % 1024 for o in offs[:6]} == {0, 128, 256, 384, 512, 640}      # six streams, six different eighths
    assert wkv.wkv6_arena_layout([]) == (0, [])
    assert wkv.wkv6_arena_layout([10, -1])[0] == -1
    assert wkv.wkv6_arena_layout([1] * 65)[0] == -1
    assert binding.load().wkv6_arena_layout(2, None, None) == -1


def test_split_helpers_and_validation():
    lib = binding.load()
    assert wkv.wkv6_split_segments(1, 131072, 32, 64) == 8          # 32 units on 256 CUs
    assert wkv.wkv6_split_segments(8, 4096, 32, 64) == 1            # already one unit per CU
    assert wkv.wkv6_split_segments(1, 1024, 32, 64) == 1            # too short to split
    assert wkv.wkv6_split_workspace_bytes(1, 131072, 32, 64, 8) == 8 * 32 * (4096 + 64) * 4
    assert wkv.wkv6_split_workspace_bytes(1, 100, 2, 64, 8) == 4 * 2 * (4096 + 64) * 4   # 32-token segments
    assert wkv.wkv6_split_workspace_bytes(1, 100, 2, 32, 8) == -1
    f = lib.wkv6_prefill_bf16_split
    assert f(1, 4096, 2, 64, A, A, A, A, A, None, A, A, 1, 4, None, 0, None) == 1        # no workspace
    assert f(1, 4096, 2, 64, A, A, A, A, A, None, A, A, 1, 4, A, 16, None) == 2           # too small
    assert f(1, 4096, 2, 64, A, A, A, A, A, None, A, A, 9, 4, A, 1 << 30, None) == 3      # dtype code
    assert f(1, 4096, 2, 64, A, A, A, A, A, None, A, A, 1, 0, A, 1 << 30, None) == 2      # segments < 1
    assert f(1, 4096, 2, 32, A, A, A, A, A, None, A, A, 1, 4, A, 1 << 30, None) == 3      # N != 64


def test_layernorm_moments_validation():
    f = _raw("wkv6_finch_c2_prefill_bf16_moments")
    assert f(1, 8, 2, 64, A, A, A, A, A, None, A, None, A, None) == 1          # moments required when T > 0
    assert f(1, 8, 2, 64, A, A, A, A, A, None, A, P(0x1004), A, None) == 5
    assert f(1, 8, 2, 32, A, A, A, A, A, None, A, A, A, None) == 3
    assert f(0, 8, 2, 64, None, None, None, None, None, None, None, None, None, None) == 0
    g = _raw("wkv6_layernorm_finalize")
    assert g(1, 8, 2, 32, A, ctypes.c_float(1e-5), A, None) == 3
    assert g(1, 8, 0, 64, A, ctypes.c_float(1e-5), A, None) == 2
    assert g(70000, 8, 2, 64, A, ctypes.c_float(1e-5), A, None) == 2             # grid limit
    assert g(1, 8, 2, 64, A, ctypes.c_float(-1.0), A, None) == 2
    assert g(1, 8, 2, 64, A, ctypes.c_float(float("nan")), A, None) == 2
    assert g(1, 8, 2, 64, None, ctypes.c_float(1e-5), A, None) == 1
    assert g(1, 8, 2, 64, A, ctypes.c_float(1e-5), P(0x1008), None) == 5
    assert g(1, 0, 2, 64, None, ctypes.c_float(1e-5), None, None) == 0


def test_layernorm_apply_validation():
    f = _raw("wkv6_layernorm_apply_bf16")
    assert f(1, 8, 2, 32, A, A, A, A, A, 0, None) == 3
    assert f(1, 8, 2, 64, A, A, A, A, A, 4, None) == 3
    assert f(1, -1, 2, 64, A, A, A, A, A, 0, None) == 2
    assert f(1, 8, 2, 64, A, A, None, A, A, 0, None) == 1
    assert f(1, 8, 2, 64, A, P(0x1004), A, A, A, 0, None) == 5
    assert f(0, 8, 2, 64, None, None, None, None, None, 0, None) == 0


def test_fused_decay_path_validation():
    f = _raw("wkv6_finch_c2_prefill_lora_bf16")
    ok = (A, A, A, A, A, A, A, None, A, None, A, None)    # r kbar v y lambda b_omega uprime state_in out moments state_out stream
    assert f(1, 8, 2, 64, 32, *ok) == 3                                          # rank
    assert f(1, 8, 2, 32, 64, *ok) == 3                                          # head size
    assert f(1, -8, 2, 64, 64, *ok) == 2
    assert f(1, 8, 2, 64, 64, A, A, A, None, A, A, A, None, A, None, A, None) == 1   # y
    assert f(1, 8, 2, 64, 64, A, A, A, A, None, A, A, None, A, None, A, None) == 1   # lambda
    assert f(1, 8, 2, 64, 64, A, A, A, A, A, None, A, None, A, None, A, None) == 1   # b_omega
    assert f(1, 8, 2, 64, 64, A, A, A, P(0x1008), A, A, A, None, A, None, A, None) == 5
    assert f(1, 8, 2, 64, 64, A, A, A, A, A, A, A, None, A, P(0x1004), A, None) == 5   # moments alignment
    assert f(0, 8, 2, 64, 64, *([None] * 12)) == 0


def test_decay_front_validation_and_recipe():
    f = _raw("wkv6_decay_lora_input_bf16")
    ok = (A, None, A, A, A, A, A, A, 0, None)     # x x_prev mu_x lambda_d a_d b_d a_omega y out_dtype stream
    assert f(1, 8, 2048, 16, 64, *ok) == 3                                        # inner rank
    assert f(1, 8, 2048, 32, 32, *ok) == 3                                        # outer rank
    assert f(1, 8, 2000, 32, 64, *ok) == 3                                        # width not a multiple of 128
    assert f(1, 8, 2048, 32, 64, A, None, A, A, A, A, A, A, 5, None) == 3          # dtype code
    assert f(-1, 8, 2048, 32, 64, *ok) == 2
    assert f(1, 8, 2048, 32, 64, None, None, A, A, A, A, A, A, 0, None) == 1       # x
    assert f(1, 8, 2048, 32, 64, A, None, A, A, A, None, A, A, 0, None) == 1       # b_d
    assert f(1, 8, 2048, 32, 64, A, P(0x1008), A, A, A, A, A, A, 0, None) == 5     # x_prev alignment
    assert f(1, 0, 2048, 32, 64, *([None] * 8), 0, None) == 0
    from paper_2407_12077_amd.workloads import CONFIGS, make_decay_front_inputs, round_to_bf16, scaled
    cfg = scaled(CONFIGS[2], B=2, T=9, H=2)
    a, b = make_decay_front_inputs(cfg), make_decay_front_inputs(cfg)
    assert a["x"].shape == (2, 9, 128) and a["x_prev"].shape == (2, 128) and a["A_d"].shape == (128, 32)
    assert a["B_d"].shape == (32, 128) and a["A_omega"].shape == (128, 64) and a["mu_x"].shape == (128,)
    for k in a:
        assert a[k].dtype == np.float32 and np.array_equal(a[k], b[k])
    for k in ("x", "x_prev", "A_d", "B_d", "A_omega"):
        assert np.array_equal(a[k], round_to_bf16(a[k]))
    assert 0 <= a["mu_x"].min() and a["mu_x"].max() <= 1 and 0 <= a["lam_d"].min() and a["lam_d"].max() <= 1


def test_decay_lora_workload_recipe():
    from paper_2407_12077_amd.workloads import CONFIGS, make_decay_lora_inputs, round_to_bf16, scaled
    cfg = scaled(CONFIGS[2], B=2, T=50, H=3)
    a, b = make_decay_lora_inputs(cfg), make_decay_lora_inputs(cfg)
    assert a["y"].shape == (2, 50, 64) and a["lam"].shape == (3 * 64,) and a["b_omega"].shape == (64, 3 * 64)
    for k in a:
        assert a[k].dtype == np.float32 and np.array_equal(a[k], b[k])            # seeded
    assert np.array_equal(a["y"], round_to_bf16(a["y"])) and np.array_equal(a["b_omega"], round_to_bf16(a["b_omega"]))
    assert np.abs(a["y"]).max() <= 1.0 and -5.5 <= a["lam"].min() and a["lam"].max() <= 0.5
    assert not np.array_equal(a["y"], make_decay_lora_inputs(cfg, seed=1)["y"])
