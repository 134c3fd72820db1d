"""LayerNorm over the concatenated heads -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

The Finch-C2 output equation (Finch-C2 Time Mixing, last equation) applies one LayerNorm to
the concatenation of all heads' read-outs of a token before the output projection:

    z_t = concat_h( r_t . wkv_t + u'_t )            D = H*N entries
    y_t = (z_t - mean(z_t)) / sqrt(var(z_t) + eps) * gamma + beta

with mean and var taken over the D entries of the token (var divides by D, the usual
LayerNorm convention; the paper names the operator only), gamma and beta of D entries.

Written out per token in float64 with explicit sums; nothing here is shared with or imported
by the GPU library.

``layernorm_heads_numpy``  the definition above.
``head_moments_numpy``     per (batch, head, token): the sum of the head's N entries and the
                           sum of squared deviations from the head's own mean -- the partial
                           statistics from which the token's mean and variance follow by the
                           pairwise-combination identity (Chan, Golub, LeVeque 1979).

Parity pins (tests/test_oracle_pins_layernorm.py): a hand-computed token, zero mean / unit
variance of the result, shift and scale invariance, a constant token, the library LayerNorm
in float64, per-head normalisation told apart, the moments against the two-pass variance, and
planted mistakes.
"""
import numpy as np


def layernorm_heads_numpy(o, gamma, beta, eps):
    """o [B,T,H,N]; gamma, beta [H*N]; returns (y [B,T,H,N], mean [B,T], rstd [B,T]) float64."""
    o = np.asarray(o, dtype=np.float64)
    B, T, H, N = o.shape
    D = H * N
    gamma = np.asarray(gamma, dtype=np.float64).reshape(D)
    beta = np.asarray(beta, dtype=np.float64).reshape(D)
    y = np.empty((B, T, D), dtype=np.float64)
    mean = np.empty((B, T), dtype=np.float64)
    rstd = np.empty((B, T), dtype=np.float64)
    for b in range(B):
        for t in range(T):
            z = o[b, t].reshape(D)                 # heads side by side: head h owns entries h*N .. h*N+N-1
            m = z.sum() / D
            var = ((z - m) ** 2).sum() / D
            rs = 1.0 / np.sqrt(var + eps)
            y[b, t] = (z - m) * rs * gamma + beta
            mean[b, t] = m
            rstd[b, t] = rs
    return y.reshape(B, T, H, N), mean, rstd


def head_moments_numpy(o):
    """o [B,T,H,N]; returns (s [B,H,T], m2 [B,H,T]): s = sum_n o, m2 = sum_n (o - s/N)^2."""
    o = np.asarray(o, dtype=np.float64)
    B, T, H, N = o.shape
    s = np.empty((B, H, T), dtype=np.float64)
    m2 = np.empty((B, H, T), dtype=np.float64)
    for b in range(B):
        for t in range(T):
            for h in range(H):
                z = o[b, t, h]
                tot = z.sum()
                s[b, h, t] = tot
                m2[b, h, t] = ((z - tot / N) ** 2).sum()
    return s, m2
