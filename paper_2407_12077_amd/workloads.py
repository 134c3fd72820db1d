"""Seeded synthetic inputs for the WKV6 prefill path.

This module holds no arithmetic of the method: it only draws random tensors
with the shapes and value distributions of the five benchmark configurations
and rounds them once to their storage dtype.  Both the GPU tests / benchmark
and the CPU oracle's callers take their inputs from here, so the two sides
see bit-identical values.

The paper's own workloads are activations of trained Finch / GoldFinch
models on text corpora; neither weights nor corpora are available, so these
synthetic tensors stand in for them.

Draw order (fixed): r, k, v, x, u, S0 from ``numpy.random.Generator(PCG64(seed))``
with ``seed = 20240712 + config index`` unless overridden.
"""
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 20240712


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    B: int
    T: int
    H: int
    N: int
    dtype: str            # storage dtype of r,k,v,x: "f32" or "bf16"
    x_kind: str           # "uniform" (U(-6,1)) or "bimodal" (per-channel long/short memory)
    u_std: float
    s0_std: float         # 0 => zero initial state (state_in = None)

    @property
    def tokens(self):
        return self.B * self.T

    @property
    def token_heads(self):
        return self.B * self.T * self.H


CONFIGS = {
    1: Workload(1, "tiny-f32", 1, 256, 4, 64, "f32", "uniform", 0.5, 0.0),
    2: Workload(2, "finch-1.6b-layer", 8, 4096, 32, 64, "bf16", "uniform", 0.5, 0.0),
    3: Workload(3, "long-context", 1, 131072, 32, 64, "bf16", "uniform", 0.5, 0.0),
    4: Workload(4, "many-short-requests", 256, 512, 32, 64, "bf16", "uniform", 0.5, 0.1),
    5: Workload(5, "larger-model-stress", 4, 16384, 64, 64, "bf16", "bimodal", 1.0, 0.0),
}


def round_to_bf16(a):
    """Round a float32 array to the nearest bf16 value (ties to even), kept as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    out = ((bits + bias) & np.uint32(0xFFFF0000)).view(np.float32)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, a, out)
    return out.reshape(a.shape)


def bf16_bits(a):
    """uint16 bit patterns of an array already holding bf16-representable float32 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(a.shape)


def scaled(cfg, **dims):
    """The same workload with some of B, T, H overridden (reduced or ragged test sizes)."""
    return replace(cfg, **dims)


def make_inputs(cfg, seed=None):
    """Draw one batch for ``cfg``.  Returns a dict of float32 NumPy arrays:

    r, k, v, x : [B, T, H, N]  (already rounded to ``cfg.dtype``)
    u          : [H, N]  fp32
    state_in   : [B, H, N, N] fp32, or None when the workload starts from zero state
    """
    if seed is None:
        seed = BASE_SEED + cfg.index
    rng = np.random.Generator(np.random.PCG64(seed))
    shape = (cfg.B, cfg.T, cfg.H, cfg.N)
    inv_sqrt_n = np.float32(1.0 / np.sqrt(cfg.N))

    def gauss():
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= inv_sqrt_n
        return a

    r, k, v = gauss(), gauss(), gauss()

    x = rng.random(shape, dtype=np.float32)
    if cfg.x_kind == "uniform":
        x *= np.float32(7.0)
        x -= np.float32(6.0)                       # U(-6, 1)
    elif cfg.x_kind == "bimodal":
        long_memory = rng.random((cfg.H, cfg.N)) < 0.5
        lo = np.where(long_memory, -10.0, 0.0).astype(np.float32)   # U(-10,-3) or U(0,2)
        span = np.where(long_memory, 7.0, 2.0).astype(np.float32)
        x *= span[None, None]
        x += lo[None, None]
    else:
        raise ValueError(cfg.x_kind)

    u = (rng.standard_normal((cfg.H, cfg.N)) * cfg.u_std).astype(np.float32)
    state_in = None
    if cfg.s0_std > 0:
        state_in = rng.standard_normal((cfg.B, cfg.H, cfg.N, cfg.N), dtype=np.float32)
        state_in *= np.float32(cfg.s0_std)

    if cfg.dtype == "bf16":
        r, k, v, x = (round_to_bf16(a) for a in (r, k, v, x))
    elif cfg.dtype != "f32":
        raise ValueError(cfg.dtype)
    return {"r": r, "k": k, "v": v, "x": x, "u": u, "state_in": state_in}


def make_uprime(cfg, seed=None):
    """Second value u' of the Finch-C2 form for ``cfg``: [B, T, H, N], N(0,1)/sqrt(N) like v
    (it is a value-projection output plus a low-rank term), rounded to ``cfg.dtype``.  Drawn from
    its own generator, ``PCG64(seed + 1000)``, so the draws of ``make_inputs`` do not move."""
    if seed is None:
        seed = BASE_SEED + cfg.index
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    a = rng.standard_normal((cfg.B, cfg.T, cfg.H, cfg.N), dtype=np.float32)
    a *= np.float32(1.0 / np.sqrt(cfg.N))
    return round_to_bf16(a) if cfg.dtype == "bf16" else a


def make_decay_lora_inputs(cfg, seed=None, rank=64):
    """Inputs of the fused decay path for ``cfg``: low-rank activations y [B, T, rank] (tanh of
    N(0,1) draws, so inside (-1, 1) like the tanh(. A) they stand in for), per-channel base logits
    lam [H*N] ~ U(-5.5, 0.5) and the outer factor b_omega [rank, H*N] ~ N(0, 0.2^2), which puts the
    token-dependent part of the logit at a standard deviation of about 1 around its base (the
    logits then span roughly the U(-6, 1) range of the plain workloads).  y and b_omega are rounded
    to bf16; all are float32 arrays.  Own generator, ``PCG64(seed + 2000)``."""
    if seed is None:
        seed = BASE_SEED + cfg.index
    rng = np.random.Generator(np.random.PCG64(seed + 2000))
    y = np.tanh(rng.standard_normal((cfg.B, cfg.T, rank), dtype=np.float32))
    lam = (rng.random(cfg.H * cfg.N, dtype=np.float32) * np.float32(6.0) - np.float32(5.5)).astype(np.float32)
    b_omega = rng.standard_normal((rank, cfg.H * cfg.N), dtype=np.float32) * np.float32(0.2)
    return {"y": round_to_bf16(y), "lam": lam, "b_omega": round_to_bf16(b_omega)}


def make_decay_front_inputs(cfg, seed=None, inner_rank=32, rank=64):
    """Inputs of the operators in front of the decay path for ``cfg`` (D = H*N): the time-mix input
    x [B, T, D] ~ N(0, 1) (a LayerNorm output stands behind it in the model), the row x_prev [B, D]
    before each sequence, the interpolation weights mu_x ~ U(0, 1) and lam_d ~ U(0, 1) (both are
    per-channel mixing ratios between a token and its predecessor), and the three low-rank factors in
    the paper's orientation: A_d [D, inner_rank] ~ N(0, 1/D) (unit-scale pre-activations),
    B_d [inner_rank, D] ~ N(0, 0.1^2), A_omega [D, rank] ~ N(0, 1/D).  x, x_prev and the matrices are
    rounded to bf16; everything is returned as float32 arrays.  Own generator, ``PCG64(seed + 3000)``."""
    if seed is None:
        seed = BASE_SEED + cfg.index
    rng = np.random.Generator(np.random.PCG64(seed + 3000))
    D = cfg.H * cfg.N
    x = rng.standard_normal((cfg.B, cfg.T, D), dtype=np.float32)
    x_prev = rng.standard_normal((cfg.B, D), dtype=np.float32)
    mu_x = rng.random(D, dtype=np.float32)
    lam_d = rng.random(D, dtype=np.float32)
    inv = np.float32(1.0 / np.sqrt(D))
    A_d = rng.standard_normal((D, inner_rank), dtype=np.float32) * inv
    B_d = rng.standard_normal((inner_rank, D), dtype=np.float32) * np.float32(0.1)
    A_omega = rng.standard_normal((D, rank), dtype=np.float32) * inv
    return {"x": round_to_bf16(x), "x_prev": round_to_bf16(x_prev), "mu_x": mu_x, "lam_d": lam_d,
            "A_d": round_to_bf16(A_d), "B_d": round_to_bf16(B_d), "A_omega": round_to_bf16(A_omega)}


def make_key_compress_inputs(M, D, seed=BASE_SEED + 100):
    """Inputs of the GOLD key compression for M tokens of a model of width D: hidden states
    x [M, D] ~ N(0, 1) (a residual-stream activation stands in for the last Finch-C2 layer's
    output) and the compression matrix w_kd [D, D/16] ~ N(0, 1/D) (so the compressed entries have
    unit scale), both rounded to bf16 and returned as float32 arrays."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((M, D), dtype=np.float32)
    w = rng.standard_normal((D, D // 16), dtype=np.float32)
    w *= np.float32(1.0 / np.sqrt(D))
    return round_to_bf16(x), round_to_bf16(w)
