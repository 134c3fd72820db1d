"""Helpers shared by the GPU tests: upload seeded inputs, call the C ABI through the thin
binding, download, and compare with the oracle using the max-normalised error."""
import numpy as np
import torch

import paper_2407_12077_amd as wkv

TOL_BF16 = 2e-3     # bf16 inputs, fp32 output and state, vs the fp64 oracle
TOL_F32 = 1e-5      # fp32 tensors
BF16_OUT_ROUNDING = 2.0 ** -8   # extra allowance when the output itself is rounded to bf16


def max_norm_err(got, ref):
    """max |got - ref| / max |ref|  (the tolerance's definition of relative error)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = np.abs(ref).max()
    if denom == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / denom)


def error_report(got, ref, kind):
    """Every error figure the parity tests print for one tensor against the oracle's:

    global   max |got - ref| / max |ref| over the whole tensor (the gated definition)
    unit     the same ratio taken per (batch, head) unit, worst unit (gated at the same tolerance:
             a unit whose values are small next to the tensor's largest cannot hide)
    row      per token row (out) or per key row (state): max over the 64 channels of |got - ref| over
             the max of |ref| in that row, worst row (reported; rows of near-zero reference values
             make it large without meaning anything, so it is not gated)
    rel_l2   ||got - ref||_2 / ||ref||_2

    kind: "out" for [B, T, H, N] tensors, "state" for [B, H, N, N]."""
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(np.asarray(got, dtype=np.float64) - ref)
    aref = np.abs(ref)
    unit_axes = (1, 3) if kind == "out" else (2, 3)
    d_row, r_row = diff.max(axis=3), aref.max(axis=3)
    unit_axis_of_rows = 1 if kind == "out" else 2
    d_unit, r_unit = d_row.max(axis=unit_axis_of_rows), r_row.max(axis=unit_axis_of_rows)
    assert d_unit.shape == diff.max(axis=unit_axes).shape
    tiny = np.finfo(np.float64).tiny
    l2 = float(np.sqrt(np.square(diff).sum() / max(np.square(ref).sum(), tiny)))
    return {"global": float(d_unit.max() / max(r_unit.max(), tiny)),
            "unit": float((d_unit / np.maximum(r_unit, tiny)).max()),
            "row": float((d_row / np.maximum(r_row, tiny)).max()),
            "rel_l2": l2}


def fmt_report(rep):
    return " ".join(f"{k}={v:.3e}" for k, v in rep.items())


def to_dev(a, dtype):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(dtype).cuda()


def in_arena(tensors):
    """Copies of the given device tensors inside one arena, placed by the library's wkv6_arena_layout
    (4 KiB slots, tensor i shifted by 128 (i mod 8) bytes).  Returns (arena, [views])."""
    import paper_2407_12077_amd as wkv
    sizes = [t.numel() * t.element_size() for t in tensors]
    total, offs = wkv.wkv6_arena_layout(sizes)
    assert total >= 0
    arena = torch.empty(total + 4096, dtype=torch.uint8, device="cuda")
    first = (-arena.data_ptr()) % 4096
    views = []
    for t, o, b in zip(tensors, offs, sizes):
        v = arena[first + o:first + o + b].view(t.dtype).view(t.shape)
        v.copy_(t)
        views.append(v)
    return arena, views


def run_entry(entry, inp, out_dtype=torch.float32, in_dtype=torch.bfloat16, want_state=True,
              inplace_state=False):
    """Run one entry point on the arrays of ``inp`` (dict from make_inputs).  Returns
    (out, state_out) as float64 NumPy arrays (state_out None if not requested)."""
    B, T, H, N = inp["r"].shape
    r, k, v, x = (to_dev(inp[n], in_dtype) for n in ("r", "k", "v", "x"))
    u = to_dev(inp["u"], torch.float32)
    s_in = to_dev(inp.get("state_in"), torch.float32)
    out = torch.full((B, T, H, N), float("nan"), dtype=out_dtype, device="cuda")
    if inplace_state:
        assert s_in is not None
        s_out = s_in
    else:
        s_out = torch.full((B, H, N, N), float("nan"), dtype=torch.float32, device="cuda") if want_state else None
    getattr(wkv, entry)(B, T, H, N, r, k, v, x, u, s_in, out, s_out)
    torch.cuda.synchronize()
    o = out.float().cpu().numpy().astype(np.float64)
    s = None if s_out is None else s_out.cpu().numpy().astype(np.float64)
    return o, s
