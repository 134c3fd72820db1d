"""Token shift, ddlerp and the inner factor of the decay path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Finch-C2 Time Mixing defines the operators

    lerp(a, b, t)   = a + (b - a) * t
    lora(x)         = lambda + tanh(x A) B
    ddlerp(a, b)    = a + (b - a) * lora(a + (b - a) * mu_x)

and the decay logit d_t = lora_omega(ddlerp_d(x_t, x_{t-1})).  With the token-shifted input
x_{t-1} (the previous token of the same sequence; before the first token the caller's carried row
``x_prev`` or, if there is none, zero: the paper writes x_{t-1} without saying what precedes the
first token, and Finch, from which the operators are taken, shifts in zeros or the carried last
token), this module evaluates

    z_t = ddlerp_d(x_t, x_{t-1})                       D entries
    y_t = tanh(z_t A_omega)                            R entries, shared by all heads

so that  d_t = lambda_omega + y_t B_omega  (``decay_logits_numpy``) completes the printed operator.

Every function is float64 NumPy with sums written as explicit accumulation; matrices are in the
paper's orientation (x on the left: A is [D, r], B is [r, D]).  Nothing here is shared with or
imported by the GPU library.  Pins: tests/test_oracle_pins_ddlerp.py.
"""
import numpy as np


def _matmul(x, W):
    """x [..., K] times W [K, N] as an explicit sum over K."""
    out = np.zeros(x.shape[:-1] + (W.shape[1],), dtype=np.float64)
    for i in range(W.shape[0]):
        out += x[..., i:i + 1] * W[i]
    return out


def lerp_numpy(a, b, t):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return a + (b - a) * np.asarray(t, dtype=np.float64)


def token_shift_numpy(x, x_prev=None):
    """x [B, T, D] -> the previous token of every position, [B, T, D]; position 0 gets x_prev [B, D]
    (zeros when None)."""
    x = np.asarray(x, dtype=np.float64)
    shifted = np.zeros_like(x)
    shifted[:, 1:] = x[:, :-1]
    if x_prev is not None and x.shape[1] > 0:
        shifted[:, 0] = np.asarray(x_prev, dtype=np.float64)
    return shifted


def ddlerp_numpy(a, b, mu_x, lam, A, Bm):
    """ddlerp(a, b) = a + (b - a) * lora(a + (b - a) * mu_x) with lora = lam + tanh(. A) Bm.
    a, b [..., D]; mu_x, lam [D]; A [D, r]; Bm [r, D]."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    Bm = np.asarray(Bm, dtype=np.float64)
    inner = a + (b - a) * np.asarray(mu_x, dtype=np.float64)
    mix = np.asarray(lam, dtype=np.float64) + _matmul(np.tanh(_matmul(inner, A)), Bm)
    return a + (b - a) * mix


def decay_lora_input_numpy(x, x_prev, mu_x, lam_d, A_d, B_d, A_omega):
    """y_t = tanh(ddlerp_d(x_t, x_{t-1}) A_omega) for every token: x [B, T, D] -> y [B, T, R]."""
    x = np.asarray(x, dtype=np.float64)
    z = ddlerp_numpy(x, token_shift_numpy(x, x_prev), mu_x, lam_d, A_d, B_d)
    return np.tanh(_matmul(z, np.asarray(A_omega, dtype=np.float64)))
