"""Pins for the Finch-C2 oracle (Method section, Finch-C2 Time Mixing: k_t carries the factor
(1 - w_t), wkv_t is the printed double sum/product, the read-out is r_t . wkv_t + u'_t).

Same scheme as the WKV6 pins: every pin is a function of an implementation
``f(r, kbar, v, x, uprime, state_in) -> (out, state_out)``; the C oracle (1 and 3 threads) and
its NumPy twin must pass all of them, every planted mistake must fail at least one.
"""
import numpy as np
import pytest

from oracle import finch_c2_numpy, finch_c2_oracle, wkv6_oracle


def draw(rng, B, T, H, N, s0=False, xlo=-6.0, xhi=1.0):
    r, kbar, v, up = (rng.standard_normal((B, T, H, N)).astype(np.float32) for _ in range(4))
    x = rng.uniform(xlo, xhi, (B, T, H, N)).astype(np.float32)
    s = rng.standard_normal((B, H, N, N)).astype(np.float32) if s0 else None
    return r, kbar, v, x, up, s


def printed_definition(r, kbar, v, x, up):
    """wkv_t = sum_{i<t} diag(prod_{j=i+1}^{t-1} w_j) k_i^T v_i with k_i = kbar_i (1 - w_i),
    o_t = r_t . wkv_t + u'_t, evaluated literally (explicit products, no running state);
    the final state is wkv_{T+1}."""
    r, kbar, v, x, up = (np.asarray(a, dtype=np.float64) for a in (r, kbar, v, x, up))
    B, T, H, N = r.shape
    w = np.exp(-np.exp(x))
    out = np.zeros((B, T, H, N))
    state = np.zeros((B, H, N, N))
    for b in range(B):
        for h in range(H):
            for t in range(T + 1):
                wkv = np.zeros((N, N))
                for i in range(t):
                    prod = np.ones(N)
                    for j in range(i + 1, t):
                        prod = prod * w[b, j, h]
                    k_i = kbar[b, i, h] * (1.0 - w[b, i, h])
                    wkv += prod[:, None] * np.outer(k_i, v[b, i, h])
                if t == T:
                    state[b, h] = wkv
                else:
                    out[b, t, h] = r[b, t, h] @ wkv + up[b, t, h]
    return out, state


def close(a, b, tol=1e-12):
    np.testing.assert_allclose(a, b, rtol=0, atol=tol * max(1.0, np.abs(b).max()))


# ----------------------------------------------------------------------------- pins
def pin_printed_sum(f):
    rng = np.random.default_rng(31)
    for (B, T, H, N) in [(1, 9, 2, 2), (2, 11, 2, 4), (1, 4, 1, 64), (1, 16, 3, 3)]:
        r, kbar, v, x, up, _ = draw(rng, B, T, H, N)
        o_ref, s_ref = printed_definition(r, kbar, v, x, up)
        o, s = f(r, kbar, v, x, up, None)
        close(o, o_ref)
        close(s, s_ref)


def pin_t1_closed_form(f):
    """One token: o_1 = r_1 . S_0 + u'_1;  S_1 = diag(w_1) S_0 + (kbar_1 (1 - w_1))^T v_1."""
    rng = np.random.default_rng(32)
    B, T, H, N = 2, 1, 3, 5
    r, kbar, v, x, up, s0 = draw(rng, B, T, H, N, s0=True)
    o, s = f(r, kbar, v, x, up, s0)
    w = np.exp(-np.exp(x.astype(np.float64)))[:, 0]                       # [B,H,N]
    o_ref = np.einsum("bhi,bhij->bhj", r[:, 0].astype(np.float64), s0.astype(np.float64)) + up[:, 0]
    k = kbar[:, 0].astype(np.float64) * (1.0 - w)
    s_ref = w[..., None] * s0 + k[..., None] * v[:, 0].astype(np.float64)[:, :, None, :]
    close(o[:, 0], o_ref)
    close(s, s_ref)


def pin_reduces_to_finch_with_scaled_key(f):
    """Finch-C2 is the Finch recurrence with bonus u = 0, the key pre-multiplied by (1 - w) and
    u' added to the read-out.  The pre-multiplied key is made exact in float32 by choosing
    decays w in {0, 1/2, 1} and keys with few significant bits."""
    rng = np.random.default_rng(33)
    B, T, H, N = 2, 13, 2, 4
    r, _, v, _, up, s0 = draw(rng, B, T, H, N, s0=True)
    x_half = np.float32(np.log(np.log(2.0)))
    choice = rng.integers(0, 3, (B, T, H, N))
    x = np.where(choice == 0, np.float32(-np.inf), np.where(choice == 1, x_half, np.float32(np.inf))).astype(np.float32)
    kbar = (rng.integers(-64, 65, (B, T, H, N)) / 16.0).astype(np.float32)
    w = np.exp(-np.exp(x.astype(np.float64)))
    k_scaled = kbar.astype(np.float64) * (1.0 - w)
    # float32(x_half) gives w = 1/2 only up to ~1e-8, so compare with a tolerance that covers
    # the rounding of the pre-scaled key to float32
    o_ref, s_ref = wkv6_oracle(r, k_scaled.astype(np.float32), v, x, np.zeros((H, N), np.float32), s0)
    o, s = f(r, kbar, v, x, up, s0)
    close(o, o_ref + up.astype(np.float64), 1e-6)
    close(s, s_ref, 1e-6)


def pin_w_one_never_writes_the_state(f):
    """x = -inf: w = 1, the key factor (1 - w) is 0, so the state stays S_0 and every read-out
    is r_t . S_0 + u'_t."""
    rng = np.random.default_rng(34)
    B, T, H, N = 1, 7, 2, 4
    r, kbar, v, _, up, s0 = draw(rng, B, T, H, N, s0=True)
    x = np.full((B, T, H, N), -np.inf, np.float32)
    o, s = f(r, kbar, v, x, up, s0)
    close(s, s0.astype(np.float64))
    o_ref = np.einsum("bthi,bhij->bthj", r.astype(np.float64), s0.astype(np.float64)) + up
    close(o, o_ref)


def pin_w_zero_keeps_last_token_only(f):
    """x = +inf: w = 0, the key factor is 1: S_t = kbar_t^T v_t and o_t = (r_t . kbar_{t-1}) v_{t-1} + u'_t."""
    rng = np.random.default_rng(35)
    B, T, H, N = 1, 6, 2, 3
    r, kbar, v, _, up, _ = draw(rng, B, T, H, N)
    x = np.full((B, T, H, N), np.inf, np.float32)
    o, s = f(r, kbar, v, x, up, None)
    r64, k64, v64 = (a.astype(np.float64) for a in (r, kbar, v))
    close(o[:, 0], up[:, 0].astype(np.float64))
    dots = np.einsum("bthi,bthi->bth", r64[:, 1:], k64[:, :-1])
    close(o[:, 1:], dots[..., None] * v64[:, :-1] + up[:, 1:])
    close(s, k64[:, -1][..., None] * v64[:, -1][:, :, None, :])


def pin_constant_value_normalisation(f):
    """kbar = 1, v = c (constant over time): the weights (1 - w_i) prod_{j>i} w_j telescope, so
    S_t[i][:] = (1 - prod_{s<=t} w_s[i]) c, a convex mixture: the reason for the (1 - w) factor."""
    rng = np.random.default_rng(36)
    B, T, H, N = 1, 15, 2, 3
    x = rng.uniform(-4, 1, (B, T, H, N)).astype(np.float32)
    w = np.exp(-np.exp(x.astype(np.float64)))
    c = rng.standard_normal((H, N)).astype(np.float32)
    v = np.broadcast_to(c[None, None], (B, T, H, N)).copy()
    kbar = np.ones((B, T, H, N), np.float32)
    r = np.zeros((B, T, H, N), np.float32)
    r[..., 1] = 1.0                                          # reads row 1 of the state
    up = np.zeros((B, T, H, N), np.float32)
    o, s = f(r, kbar, v, x, up, None)
    mass = 1.0 - np.cumprod(w, axis=1)                       # [B,T,H,N(key)]
    close(s, mass[:, -1][..., None] * c.astype(np.float64)[None, :, None, :])
    prev = np.concatenate([np.zeros_like(mass[:, :1]), mass[:, :-1]], axis=1)[..., 1]   # row 1, before t
    close(o, prev[..., None] * c.astype(np.float64)[None, None])


def pin_state_passing(f):
    """Running [0, cut) and then [cut, T) from the carried state equals one run over [0, T)."""
    rng = np.random.default_rng(37)
    B, T, H, N = 2, 14, 2, 4
    r, kbar, v, x, up, s0 = draw(rng, B, T, H, N, s0=True)
    o, s = f(r, kbar, v, x, up, s0)
    cut = 5
    o1, s1 = f(r[:, :cut], kbar[:, :cut], v[:, :cut], x[:, :cut], up[:, :cut], s0)
    close(o[:, :cut], o1)
    # second half from the carried state (rounded to float32: tolerance of that rounding)
    o2, s2 = f(r[:, cut:], kbar[:, cut:], v[:, cut:], x[:, cut:], up[:, cut:], s1.astype(np.float32))
    close(o[:, cut:], o2, 1e-6)
    close(s, s2, 1e-6)


def pin_uprime_is_added_once_per_value_channel(f):
    """out is affine in u' with slope exactly 1 on the same (b,t,h,j) and 0 elsewhere; the state
    does not depend on u'."""
    rng = np.random.default_rng(38)
    B, T, H, N = 1, 5, 2, 3
    r, kbar, v, x, up, s0 = draw(rng, B, T, H, N, s0=True)
    o0, s_a = f(r, kbar, v, x, np.zeros_like(up), s0)
    o1, s_b = f(r, kbar, v, x, up, s0)
    close(o1 - o0, up.astype(np.float64))
    close(s_a, s_b)


PINS = [pin_printed_sum, pin_t1_closed_form, pin_reduces_to_finch_with_scaled_key,
        pin_w_one_never_writes_the_state, pin_w_zero_keeps_last_token_only,
        pin_constant_value_normalisation, pin_state_passing,
        pin_uprime_is_added_once_per_value_channel]


def c_oracle(r, kbar, v, x, up, s0):
    return finch_c2_oracle(r, kbar, v, x, up, s0, nthreads=3)


def c_oracle_single_thread(r, kbar, v, x, up, s0):
    return finch_c2_oracle(r, kbar, v, x, up, s0, nthreads=1)


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
@pytest.mark.parametrize("impl", [c_oracle, c_oracle_single_thread, finch_c2_numpy], ids=lambda f: f.__name__)
def test_pin(impl, pin):
    pin(impl)


# ------------------------------------------------------------ planted mistakes (CPU only)
def wrong_variant(kind):
    def f(r, kbar, v, x, up, s0):
        r, kbar, v, x, up = (np.asarray(a, dtype=np.float64) for a in (r, kbar, v, x, up))
        B, T, H, N = r.shape
        S = np.zeros((B, H, N, N)) if s0 is None else np.array(s0, dtype=np.float64)
        if kind == "ignore_state_in":
            S = np.zeros((B, H, N, N))
        out = np.empty((B, T, H, N))
        with np.errstate(over="ignore"):
            w = np.exp(-np.exp(x))
        for t in range(T):
            wt = w[:, t]
            if kind == "no_one_minus_w":
                k = kbar[:, t]
            elif kind == "w_instead_of_one_minus_w":
                k = kbar[:, t] * wt
            elif kind == "one_minus_previous_w":
                k = kbar[:, t] * (1.0 - (w[:, t - 1] if t > 0 else 0.0))
            else:
                k = kbar[:, t] * (1.0 - wt)
            kv = k[..., :, None] * v[:, t][..., None, :]
            if kind == "factor_on_value_axis":
                kv = kbar[:, t][..., :, None] * (v[:, t] * (1.0 - wt))[..., None, :]
            read = S + kv if kind == "read_after_add" else S
            o = np.einsum("bhi,bhij->bhj", r[:, t], read)
            if kind == "no_uprime":
                pass
            elif kind == "uprime_gated_by_r":
                o = o + r[:, t] * up[:, t]
            elif kind == "uprime_previous_token":
                o = o + (up[:, t - 1] if t > 0 else 0.0)
            else:
                o = o + up[:, t]
            out[:, t] = o
            if kind == "decay_before_read":
                out[:, t] = np.einsum("bhi,bhij->bhj", r[:, t], wt[..., None] * S) + up[:, t]
            if kind == "uprime_enters_state":
                kv = kv + k[..., :, None] * up[:, t][..., None, :]
            if kind == "decay_on_value_axis":
                S = S * wt[..., None, :] + kv
            else:
                S = wt[..., None] * S + kv
        if kind == "state_out_transposed":
            S = S.transpose(0, 1, 3, 2).copy()
        return out, S
    return f


MISTAKES = ["ignore_state_in", "no_one_minus_w", "w_instead_of_one_minus_w", "one_minus_previous_w",
            "factor_on_value_axis", "read_after_add", "no_uprime", "uprime_gated_by_r",
            "uprime_previous_token", "decay_before_read", "uprime_enters_state",
            "decay_on_value_axis", "state_out_transposed"]


def test_unplanted_variant_passes_all_pins():
    for pin in PINS:
        pin(wrong_variant("none"))


@pytest.mark.parametrize("kind", MISTAKES)
def test_each_planted_mistake_fails_a_pin(kind):
    failed = []
    for pin in PINS:
        try:
            pin(wrong_variant(kind))
        except AssertionError:
            failed.append(pin.__name__)
    assert failed, f"no pin notices the planted mistake '{kind}'"


def test_c_oracle_matches_numpy_twin():
    rng = np.random.default_rng(40)
    r, kbar, v, x, up, s0 = draw(rng, 2, 40, 3, 64, s0=True)
    o1, s1 = finch_c2_oracle(r, kbar, v, x, up, s0)
    o2, s2 = finch_c2_numpy(r, kbar, v, x, up, s0)
    assert np.abs(o1 - o2).max() <= 1e-13 * max(1.0, np.abs(o1).max())
    assert np.abs(s1 - s2).max() <= 1e-13 * max(1.0, np.abs(s1).max())


def test_oracle_rejects_bad_arguments():
    z = np.zeros((1, 2, 1, 4), np.float32)
    with pytest.raises(ValueError):
        finch_c2_oracle(z, z, z[:, :1], z, z)
    with pytest.raises(ValueError):
        finch_c2_oracle(z, z, z, z, z, np.zeros((1, 1, 4, 3), np.float32))
