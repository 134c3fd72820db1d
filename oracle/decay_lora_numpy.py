"""Decay logits from the low-rank decay path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Finch-C2 Time Mixing defines  lora(x) = lambda + tanh(x A) B  and the decay logit
d_t = lora_omega(ddlerp_d(x_t, x_{t-1})), from which w_t = exp(-exp(d_t)).  With
z_t = ddlerp_d(x_t, x_{t-1}) (D entries) and y_t = tanh(z_t A_omega) (R entries, shared by all
heads), the last factor is

    d_t[c] = lambda[c] + sum_{k=0}^{R-1} y_t[k] * B_omega[k][c],        c = h*N + n  in [0, D).

``lora_numpy``            the operator as printed: lambda + tanh(x A) B.
``decay_logits_numpy``    the last factor alone, from y: what the fused GPU entry computes before
                          its decay map.  Returned per head as [B, T, H, N].

float64 throughout; sums written as explicit accumulation over k.  Nothing here is shared with or
imported by the GPU library.  Pins: tests/test_oracle_pins_decay_lora.py.
"""
import numpy as np


def lora_numpy(x, lam, A, Bm):
    """x [..., D_in]; A [D_in, R]; Bm [R, D_out]; lam [D_out] -> [..., D_out]."""
    x = np.asarray(x, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    Bm = np.asarray(Bm, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    hidden = np.zeros(x.shape[:-1] + (A.shape[1],), dtype=np.float64)
    for i in range(A.shape[0]):
        hidden += x[..., i:i + 1] * A[i]
    y = np.tanh(hidden)
    out = np.broadcast_to(lam, x.shape[:-1] + (Bm.shape[1],)).copy()
    for k in range(Bm.shape[0]):
        out += y[..., k:k + 1] * Bm[k]
    return out


def decay_logits_numpy(y, lam, Bm, H, N):
    """y [B, T, R]; lam [H*N]; Bm [R, H*N] -> d [B, T, H, N] (head h owns columns h*N .. h*N+N-1)."""
    y = np.asarray(y, dtype=np.float64)
    Bm = np.asarray(Bm, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    Bsz, T, R = y.shape
    if Bm.shape != (R, H * N) or lam.shape != (H * N,):
        raise ValueError(f"expected Bm ({R}, {H * N}) and lam ({H * N},), got {Bm.shape} and {lam.shape}")
    d = np.broadcast_to(lam, (Bsz, T, H * N)).copy()
    for k in range(R):
        d += y[:, :, k:k + 1] * Bm[k]
    return d.reshape(Bsz, T, H, N)
