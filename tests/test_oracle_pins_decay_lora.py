"""Pins for the decay-logit oracle (Finch-C2 Time Mixing: lora(x) = lambda + tanh(x A) B,
d_t = lora_omega(ddlerp_d(x_t, x_{t-1})); the fused GPU entry takes y = tanh(. A) and forms
d = lambda + y B per head)."""
import numpy as np
import pytest

from oracle import decay_logits_numpy, finch_c2_numpy, lora_numpy


def logits(y, lam, Bm, H, N):
    return decay_logits_numpy(y, lam, Bm, H, N)


def pin_hand_case(f):
    """R = 2, H = 2, N = 2 (D = 4), one batch, two tokens.  y_0 = (1, 2), y_1 = (-1, 0.5);
    B rows (1, 2, 3, 4) and (10, 20, 30, 40); lambda = (0.5, -0.5, 0, 1):
    token 0: (1 + 20, 2 + 40, 3 + 60, 4 + 80) + lambda = (21.5, 41.5, 63, 85)
    token 1: (-1 + 5, -2 + 10, -3 + 15, -4 + 20) + lambda = (4.5, 7.5, 12, 17)."""
    y = np.array([[[1.0, 2.0], [-1.0, 0.5]]])
    Bm = np.array([[1.0, 2.0, 3.0, 4.0], [10.0, 20.0, 30.0, 40.0]])
    lam = np.array([0.5, -0.5, 0.0, 1.0])
    d = f(y, lam, Bm, 2, 2)
    assert d.shape == (1, 2, 2, 2)
    np.testing.assert_array_equal(d[0, 0], [[21.5, 41.5], [63.0, 85.0]])     # head 0 = columns 0,1; head 1 = columns 2,3
    np.testing.assert_array_equal(d[0, 1], [[4.5, 7.5], [12.0, 17.0]])


def pin_special_cases(f):
    rng = np.random.default_rng(71)
    Bsz, T, R, H, N = 2, 5, 8, 3, 4
    y = rng.integers(-4, 5, (Bsz, T, R)).astype(np.float64)
    Bm = rng.integers(-4, 5, (R, H * N)).astype(np.float64)
    lam = rng.integers(-4, 5, H * N).astype(np.float64)
    # y = 0: the logits are lambda for every token
    np.testing.assert_array_equal(f(np.zeros_like(y), lam, Bm, H, N), np.broadcast_to(lam.reshape(H, N), (Bsz, T, H, N)))
    # a one-hot y picks a row of B
    e = np.zeros((1, 1, R)); e[0, 0, 5] = 1.0
    np.testing.assert_array_equal(f(e, np.zeros(H * N), Bm, H, N).reshape(H * N), Bm[5])
    # linear in y and in B (integers: exact); lambda enters once
    y2 = rng.integers(-4, 5, (Bsz, T, R)).astype(np.float64)
    z = np.zeros(H * N)
    np.testing.assert_array_equal(f(y + y2, z, Bm, H, N), f(y, z, Bm, H, N) + f(y2, z, Bm, H, N))
    np.testing.assert_array_equal(f(y, lam, Bm, H, N) - f(y, z, Bm, H, N), np.broadcast_to(lam.reshape(H, N), (Bsz, T, H, N)))
    # a token depends on no other token or batch
    np.testing.assert_array_equal(f(y, lam, Bm, H, N)[1:2, 2:4], f(y[1:2, 2:4], lam, Bm, H, N))


def pin_library_product(f):
    rng = np.random.default_rng(72)
    for (Bsz, T, R, H, N) in [(1, 3, 64, 2, 64), (2, 7, 64, 32, 64), (1, 4, 32, 1, 16)]:
        y = np.tanh(rng.standard_normal((Bsz, T, R)))
        Bm = rng.standard_normal((R, H * N)) * 0.2
        lam = rng.uniform(-6, 1, H * N)
        ref = (lam + y @ Bm).reshape(Bsz, T, H, N)
        np.testing.assert_allclose(f(y, lam, Bm, H, N), ref, rtol=0, atol=1e-13)


def pin_is_the_last_factor_of_the_printed_operator(f):
    """lora(x) = lambda + tanh(x A) B: feeding y = tanh(x A) (library tanh and product) to the
    logits function reproduces lora_numpy of x."""
    rng = np.random.default_rng(73)
    Bsz, T, D, R, H, N = 2, 4, 32, 8, 2, 16
    x = rng.standard_normal((Bsz, T, D))
    A = rng.standard_normal((D, R)) * 0.3
    Bm = rng.standard_normal((R, H * N)) * 0.2
    lam = rng.uniform(-6, 1, H * N)
    full = lora_numpy(x, lam, A, Bm)
    np.testing.assert_allclose(f(np.tanh(x @ A), lam, Bm, H, N).reshape(Bsz, T, H * N), full, rtol=0, atol=1e-13)
    # tanh saturates: a huge x A gives y = +-1 and the logits lambda +- column sums of B
    big = lora_numpy(np.full((1, 1, D), 1e3), lam, np.abs(A), Bm)
    np.testing.assert_allclose(big.reshape(-1), lam + Bm.sum(axis=0), rtol=0, atol=1e-12)


def pin_logits_drive_the_decay_of_the_time_mix(f):
    """End to end with the Finch-C2 oracle on one channel pair: with r = 1, kbar = 1, v = 1,
    u' = 0 and a constant logit d (y = 0, lambda = d) the read-out at token t is the geometric
    sum (1 - w) (1 + w + ... + w^(t-1)) N = (1 - w^t) N with w = exp(-exp(d))."""
    H, N, T = 1, 2, 6
    lam = np.array([-1.0, 0.5])
    d = f(np.zeros((1, T, 4)), lam, np.ones((4, H * N)), H, N)
    ones = np.ones((1, T, H, N))
    o, _ = finch_c2_numpy(ones, ones, ones, d, np.zeros((1, T, H, N)))
    w = np.exp(-np.exp(lam))
    for t in range(T):
        np.testing.assert_allclose(o[0, t, 0], np.full(N, ((1 - w ** t)).sum()), rtol=1e-13, atol=1e-15)


PINS = [pin_hand_case, pin_special_cases, pin_library_product, pin_is_the_last_factor_of_the_printed_operator,
        pin_logits_drive_the_decay_of_the_time_mix]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(logits)


def wrong_variant(kind):
    def f(y, lam, Bm, H, N):
        y = np.asarray(y, dtype=np.float64)
        Bm = np.asarray(Bm, dtype=np.float64)
        lam = np.asarray(lam, dtype=np.float64)
        Bsz, T, R = y.shape
        d = lam + y @ Bm
        if kind == "lambda_dropped":
            d = y @ Bm
        if kind == "lambda_scaled_by_y":
            d = (1.0 + y.sum(axis=-1, keepdims=True)) * lam + y @ Bm
        if kind == "b_read_transposed":
            d = lam + y @ Bm.reshape(H * N, R).T
        if kind == "tanh_applied_again":
            d = lam + np.tanh(y) @ Bm
        if kind == "heads_interleaved":
            return d.reshape(Bsz, T, N, H).transpose(0, 1, 3, 2)
        if kind == "tokens_shifted":
            d = lam + np.roll(y, 1, axis=1) @ Bm
        if kind == "last_rank_dropped":
            d = lam + y[..., :-1] @ Bm[:-1]
        return d.reshape(Bsz, T, H, N)
    return f


MISTAKES = ["lambda_dropped", "lambda_scaled_by_y", "b_read_transposed", "tanh_applied_again", "heads_interleaved",
            "tokens_shifted", "last_rank_dropped"]


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


def test_shapes_are_checked():
    with pytest.raises(ValueError):
        decay_logits_numpy(np.zeros((1, 2, 4)), np.zeros(8), np.zeros((4, 6)), 2, 4)
