"""NumPy fp64 twin of the WKV6 oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Written independently of ``wkv6_oracle.c`` from the same equations (Finch-C2
Time Mixing: decay map, wkv_t, read-out), vectorised over the channel axes but
still one token at a time, so that a slip in either shows up as a mismatch.
"""
import numpy as np


def wkv6_numpy(r, k, v, x, u, state_in=None):
    """out[b,t,h,:] = r_t . (S_{t-1} + diag(u) k_t^T v_t);  S_t = diag(w_t) S_{t-1} + k_t^T v_t.

    Shapes as in ``wkv6_oracle``.  Returns (out, state_out) in float64.
    """
    r = np.asarray(r, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    B, T, H, N = r.shape
    S = (np.zeros((B, H, N, N)) if state_in is None
         else np.array(state_in, dtype=np.float64).reshape(B, H, N, N))
    out = np.empty((B, T, H, N))
    with np.errstate(over="ignore"):
        w = np.exp(-np.exp(x))                      # decay in [0, 1], per key channel
    for t in range(T):
        kv = k[:, t, :, :, None] * v[:, t, :, None, :]          # [B,H,i,j] outer product
        seen = S + u[None, :, :, None] * kv                     # bonus on the current token
        out[:, t] = np.einsum("bhi,bhij->bhj", r[:, t], seen)
        S = w[:, t, :, :, None] * S + kv                        # decay rows, then add
    return out, S


def finch_c2_numpy(r, kbar, v, x, uprime, state_in=None):
    """Finch-C2 per-head time mix: k_t = kbar_t (1 - w_t); out_t = r_t . S_{t-1} + u'_t;
    S_t = diag(w_t) S_{t-1} + k_t^T v_t.  Returns (out, state_out) in float64."""
    r = np.asarray(r, dtype=np.float64)
    kbar = np.asarray(kbar, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    uprime = np.asarray(uprime, dtype=np.float64)
    B, T, H, N = r.shape
    S = (np.zeros((B, H, N, N)) if state_in is None
         else np.array(state_in, dtype=np.float64).reshape(B, H, N, N))
    out = np.empty((B, T, H, N))
    with np.errstate(over="ignore"):
        w = np.exp(-np.exp(x))
    k = kbar * (1.0 - w)                                   # key times one minus the decay
    for t in range(T):
        out[:, t] = np.einsum("bhi,bhij->bhj", r[:, t], S) + uprime[:, t]
        S = w[:, t, :, :, None] * S + k[:, t, :, :, None] * v[:, t, :, None, :]
    return out, S
