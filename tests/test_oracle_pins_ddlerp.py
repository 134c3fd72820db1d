"""Pins for the oracle of the operators in front of the decay path (Finch-C2 Time Mixing: lerp,
lora, ddlerp, and d_t = lora_omega(ddlerp_d(x_t, x_{t-1}))): token shift, ddlerp with its inner
lora, and y = tanh(z A_omega).  Each pin fixes the result by something other than the oracle's own
formula: a hand-worked case, special cases that collapse to a plain lerp or a plain shift, the
first-token boundary, sequence splitting with a carried row, the library product, and the chain into
the last factor of the printed operator.  Planted mistakes are each shown to fail a pin."""
import os

import numpy as np
import pytest

from oracle import (decay_logits_numpy, decay_lora_input_numpy, ddlerp_numpy, lerp_numpy, lora_numpy,
                    token_shift_numpy)

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "ddlerp_hand_case.txt")


def read_golden():
    vals = {}
    for line in open(GOLDEN):
        if line.startswith("#") or ":" not in line:
            continue
        name, rest = line.split(":")
        vals[name.strip()] = np.array([float(t) for t in rest.split()])
    return vals


def pin_hand_case(front, ddlerp, shift):
    g = read_golden()
    x = g["x"].reshape(1, 3, 2)
    A_d, B_d, A_w = g["A_d"].reshape(2, 1), g["B_d"].reshape(1, 2), g["A_omega"].reshape(2, 1)
    z = ddlerp(x, shift(x, None), g["mu_x"], g["lambda_d"], A_d, B_d)
    np.testing.assert_allclose(z.reshape(-1), g["z"], rtol=0, atol=1e-14)
    y = front(x, None, g["mu_x"], g["lambda_d"], A_d, B_d, A_w)
    assert y.shape == (1, 3, 1)
    np.testing.assert_allclose(y.reshape(-1), g["y"], rtol=0, atol=1e-14)


def pin_collapses_to_lerp_and_shift(front, ddlerp, shift):
    rng = np.random.default_rng(5)
    Bsz, T, D, r, R = 2, 6, 5, 3, 4
    x = rng.integers(-3, 4, (Bsz, T, D)).astype(np.float64)
    xs = shift(x, None)
    mu = rng.uniform(0, 1, D)
    A_d = rng.standard_normal((D, r))
    lam = rng.integers(-2, 3, D).astype(np.float64)
    zero_B = np.zeros((r, D))
    # outer factor of the inner lora zero: the mix is lambda, whatever mu_x and A_d are
    np.testing.assert_array_equal(ddlerp(x, xs, mu, lam, A_d, zero_B), x + (xs - x) * lam)
    # ... lambda = 0 returns the token itself, lambda = 1 the previous token (a pure shift)
    np.testing.assert_array_equal(ddlerp(x, xs, mu, np.zeros(D), A_d, zero_B), x)
    np.testing.assert_array_equal(ddlerp(x, xs, mu, np.ones(D), A_d, zero_B), xs)
    # equal neighbours: nothing to interpolate
    np.testing.assert_array_equal(ddlerp(x, x, mu, lam, A_d, rng.standard_normal((r, D))), x)
    # the shift itself: position t holds token t - 1, position 0 holds zero or the carried row
    assert np.array_equal(xs[:, 1:], x[:, :-1]) and not xs[:, 0].any()
    carried = rng.integers(-3, 4, (Bsz, D)).astype(np.float64)
    assert np.array_equal(shift(x, carried)[:, 0], carried) and np.array_equal(shift(x, carried)[:, 1:], x[:, :-1])
    # lerp: the end points and the midpoint
    a, b = x[0, 0], x[0, 1]
    np.testing.assert_array_equal(lerp_numpy(a, b, 0.0), a)
    np.testing.assert_array_equal(lerp_numpy(a, b, 1.0), b)
    np.testing.assert_array_equal(lerp_numpy(a, b, 0.5), (a + b) / 2)


def pin_mu_selects_the_lora_input(front, ddlerp, shift):
    """mu_x = 0 feeds the token itself to the inner lora, mu_x = 1 the previous token: the mix is then
    lora_numpy (the printed operator, pinned on its own) of that row."""
    rng = np.random.default_rng(6)
    Bsz, T, D, r = 1, 5, 6, 2
    x = rng.standard_normal((Bsz, T, D))
    xs = shift(x, None)
    lam, A_d, B_d = rng.standard_normal(D), rng.standard_normal((D, r)), rng.standard_normal((r, D))
    for mu, src in ((np.zeros(D), x), (np.ones(D), xs)):
        want = x + (xs - x) * lora_numpy(src, lam, A_d, B_d)
        np.testing.assert_allclose(ddlerp(x, xs, mu, lam, A_d, B_d), want, rtol=0, atol=1e-13)


def pin_first_token_and_state_passing(front, ddlerp, shift):
    rng = np.random.default_rng(7)
    Bsz, T, D, r, R = 2, 9, 8, 3, 5
    x = rng.standard_normal((Bsz, T, D))
    mu, lam = rng.uniform(0, 1, D), rng.standard_normal(D)
    A_d, B_d, A_w = rng.standard_normal((D, r)), rng.standard_normal((r, D)) * 0.3, rng.standard_normal((D, R)) * 0.3
    y = front(x, None, mu, lam, A_d, B_d, A_w)
    # first token with nothing before it: z_0 = x_0 (1 - lora(x_0 (1 - mu)))
    z0 = x[:, 0] * (1.0 - lora_numpy(x[:, 0] * (1.0 - mu), lam, A_d, B_d))
    np.testing.assert_allclose(y[:, 0], np.tanh(z0 @ A_w), rtol=0, atol=1e-13)
    # a token depends on itself and its predecessor only; splitting a sequence and carrying the last row
    cut = 4
    np.testing.assert_array_equal(front(x[:, :cut], None, mu, lam, A_d, B_d, A_w), y[:, :cut])
    np.testing.assert_array_equal(front(x[:, cut:], x[:, cut - 1], mu, lam, A_d, B_d, A_w), y[:, cut:])
    x2 = x.copy()
    x2[:, 6] += 1.0
    y2 = front(x2, None, mu, lam, A_d, B_d, A_w)
    changed = np.abs(y2 - y).max(axis=(0, 2)) > 0
    assert changed.tolist() == [False] * 6 + [True, True, False]
    # batches are independent
    np.testing.assert_array_equal(front(x[1:], None, mu, lam, A_d, B_d, A_w), y[1:])


def pin_library_and_chain(front, ddlerp, shift):
    """Against library products, and chained into the last factor: lambda_omega + y B_omega equals the
    printed lora_omega applied to z."""
    rng = np.random.default_rng(8)
    Bsz, T, H, N, r, R = 2, 7, 2, 4, 3, 6
    D = H * N
    x = rng.standard_normal((Bsz, T, D))
    mu, lam = rng.uniform(0, 1, D), rng.standard_normal(D)
    A_d, B_d = rng.standard_normal((D, r)), rng.standard_normal((r, D)) * 0.3
    A_w, B_w, lam_w = rng.standard_normal((D, R)) * 0.3, rng.standard_normal((R, D)), rng.uniform(-6, 1, D)
    xs = np.concatenate([np.zeros((Bsz, 1, D)), x[:, :-1]], axis=1)
    inner = x + (xs - x) * mu
    z = x + (xs - x) * (lam + np.tanh(inner @ A_d) @ B_d)
    np.testing.assert_allclose(ddlerp(x, shift(x, None), mu, lam, A_d, B_d), z, rtol=0, atol=1e-13)
    y = front(x, None, mu, lam, A_d, B_d, A_w)
    np.testing.assert_allclose(y, np.tanh(z @ A_w), rtol=0, atol=1e-13)
    assert np.abs(y).max() < 1.0
    d = decay_logits_numpy(y, lam_w, B_w, H, N)
    np.testing.assert_allclose(d.reshape(Bsz, T, D), lora_numpy(z, lam_w, A_w, B_w), rtol=0, atol=1e-12)


PINS = [pin_hand_case, pin_collapses_to_lerp_and_shift, pin_mu_selects_the_lora_input,
        pin_first_token_and_state_passing, pin_library_and_chain]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(decay_lora_input_numpy, ddlerp_numpy, token_shift_numpy)


# ---------------------------------------------------------------- planted mistakes
def _mm(x, W):
    return np.asarray(x, dtype=np.float64) @ np.asarray(W, dtype=np.float64)


def _variants():
    def make(shift=None, ddlerp=None, outer=None):
        sh = shift or token_shift_numpy
        dd = ddlerp or ddlerp_numpy

        def front(x, x_prev, mu, lam, A_d, B_d, A_w):
            x = np.asarray(x, dtype=np.float64)
            z = dd(x, sh(x, x_prev), mu, lam, A_d, B_d)
            return (outer or (lambda q: np.tanh(_mm(q, A_w))))(z) if outer is None else outer(z, A_w)
        return front, dd, sh

    def shift_forward(x, x_prev=None):            # next token instead of the previous one
        x = np.asarray(x, dtype=np.float64)
        s = np.zeros_like(x)
        s[:, :-1] = x[:, 1:]
        return s

    def shift_ignores_carry(x, x_prev=None):
        return token_shift_numpy(x, None)

    def shift_across_batches(x, x_prev=None):     # flattens batch and time before shifting
        x = np.asarray(x, dtype=np.float64)
        flat = x.reshape(1, -1, x.shape[-1])
        return token_shift_numpy(flat, None if x_prev is None else np.asarray(x_prev)[0]).reshape(x.shape)

    def dd_swapped(a, b, mu, lam, A, Bm):         # ddlerp(b, a)
        return ddlerp_numpy(b, a, mu, lam, A, Bm)

    def dd_mu_on_a(a, b, mu, lam, A, Bm):         # inner = a * mu + (b - a)
        a, b = np.asarray(a, float), np.asarray(b, float)
        return a + (b - a) * (lam + _mm(np.tanh(_mm(a * mu + (b - a), A)), Bm))

    def dd_no_tanh(a, b, mu, lam, A, Bm):
        a, b = np.asarray(a, float), np.asarray(b, float)
        return a + (b - a) * (lam + _mm(_mm(a + (b - a) * mu, A), Bm))

    def dd_no_lambda(a, b, mu, lam, A, Bm):
        a, b = np.asarray(a, float), np.asarray(b, float)
        return a + (b - a) * _mm(np.tanh(_mm(a + (b - a) * mu, A)), Bm)

    def dd_mix_outside(a, b, mu, lam, A, Bm):     # (a + (b - a)) * lora(...)
        a, b = np.asarray(a, float), np.asarray(b, float)
        return (a + (b - a)) * (lam + _mm(np.tanh(_mm(a + (b - a) * mu, A)), Bm))

    def dd_one_minus_mu(a, b, mu, lam, A, Bm):
        return ddlerp_numpy(a, b, 1.0 - np.asarray(mu, float), lam, A, Bm)

    def outer_no_tanh(z, A_w):
        return _mm(z, A_w)

    def outer_tanh_first(z, A_w):
        return _mm(np.tanh(z), A_w)

    return {
        "shift_forward": make(shift=shift_forward),
        "shift_ignores_carry": make(shift=shift_ignores_carry),
        "shift_across_batches": make(shift=shift_across_batches),
        "ddlerp_arguments_swapped": make(ddlerp=dd_swapped),
        "mu_on_the_token": make(ddlerp=dd_mu_on_a),
        "inner_tanh_dropped": make(ddlerp=dd_no_tanh),
        "lambda_dropped": make(ddlerp=dd_no_lambda),
        "mix_multiplies_the_sum": make(ddlerp=dd_mix_outside),
        "one_minus_mu": make(ddlerp=dd_one_minus_mu),
        "outer_tanh_dropped": make(outer=outer_no_tanh),
        "outer_tanh_before_the_product": make(outer=outer_tanh_first),
    }


@pytest.mark.parametrize("name", sorted(_variants()))
def test_each_planted_mistake_fails_a_pin(name):
    front, dd, sh = _variants()[name]
    failed = 0
    for pin in PINS:
        try:
            pin(front, dd, sh)
        except AssertionError:
            failed += 1
    assert failed >= 1, f"planted mistake {name} passes every pin"
