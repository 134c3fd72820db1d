"""Pins for the LayerNorm-over-all-heads oracle (Finch-C2 Time Mixing, output equation:
o_t = LayerNorm(concat_h(r_t wkv_t + u'_t)) W^O) and for the per-head partial moments from which
the token statistics are combined."""
import numpy as np
import pytest
import torch

from oracle import head_moments_numpy, layernorm_heads_numpy


def ln(o, gamma, beta, eps):
    return layernorm_heads_numpy(o, gamma, beta, eps)


def moments(o):
    return head_moments_numpy(o)


def ones_zeros(D):
    return np.ones(D), np.zeros(D)


def pin_hand_token(f, g):
    """One token, two heads of two channels: z = (1, 2, 3, 4).  mean 2.5, deviations
    (-1.5, -0.5, 0.5, 1.5), variance (2.25 + 0.25 + 0.25 + 2.25)/4 = 1.25 = 5/4, so with eps = 0
    y = deviations * 2/sqrt(5) = (-3, -1, 1, 3)/sqrt(5)."""
    o = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 2, 2)
    y, mean, rstd = f(o, *ones_zeros(4), 0.0)
    np.testing.assert_allclose(y.reshape(4), np.array([-3.0, -1.0, 1.0, 3.0]) / np.sqrt(5.0), rtol=0, atol=1e-15)
    assert mean[0, 0] == 2.5
    np.testing.assert_allclose(rstd[0, 0], 2.0 / np.sqrt(5.0), rtol=1e-15)
    # with gain (2, 2, 0.5, 0.5), offset (0, 1, 0, 1) and eps = 1.25 (variance + eps = 2.5 = 5/2):
    y, _, rstd = f(o, [2.0, 2.0, 0.5, 0.5], [0.0, 1.0, 0.0, 1.0], 1.25)
    s = np.sqrt(2.0 / 5.0)
    np.testing.assert_allclose(y.reshape(4), [-3.0 * s, 1.0 - 1.0 * s, 0.25 * s, 1.0 + 0.75 * s], rtol=0, atol=1e-15)
    # per-head moments of the same token: head 0 = (1, 2): sum 3, deviations -+0.5 -> 0.5;
    # head 1 = (3, 4): sum 7, 0.5
    s_h, m2_h = g(o)
    np.testing.assert_array_equal(s_h.reshape(2), [3.0, 7.0])
    np.testing.assert_array_equal(m2_h.reshape(2), [0.5, 0.5])


def pin_result_is_standardised(f, g):
    """gain 1, offset 0: every token's result has mean 0 and mean square var/(var + eps)."""
    rng = np.random.default_rng(61)
    B, T, H, N = 2, 5, 3, 8
    o = rng.standard_normal((B, T, H, N)) * 3.0 + 1.5
    for eps in (0.0, 1e-5, 0.7):
        y, _, _ = f(o, *ones_zeros(H * N), eps)
        z = o.reshape(B, T, H * N)
        var = z.var(axis=-1)                                   # numpy's two-pass population variance
        yy = y.reshape(B, T, H * N)
        np.testing.assert_allclose(yy.mean(axis=-1), 0.0, atol=1e-14)
        np.testing.assert_allclose((yy ** 2).mean(axis=-1), var / (var + eps), rtol=1e-12)


def pin_shift_and_scale_invariance(f, g):
    rng = np.random.default_rng(62)
    o = rng.standard_normal((1, 4, 2, 16))
    gam, bet = rng.standard_normal(32), rng.standard_normal(32)
    y0, m0, r0 = f(o, gam, bet, 0.0)
    y1, m1, r1 = f(o + 7.25, gam, bet, 0.0)
    np.testing.assert_allclose(y1, y0, atol=1e-12)
    np.testing.assert_allclose(m1, m0 + 7.25, atol=1e-13)
    y2, _, r2 = f(-4.0 * o, gam, bet, 0.0)
    np.testing.assert_allclose(y2 - bet.reshape(2, 16), -(y0 - bet.reshape(2, 16)), atol=1e-12)
    np.testing.assert_allclose(r2, r0 / 4.0, rtol=1e-13)
    # tokens are independent: a slice of tokens gives the same rows
    np.testing.assert_array_equal(f(o[:, 1:3], gam, bet, 0.0)[0], y0[:, 1:3])


def pin_constant_token(f, g):
    """All D entries equal: variance 0, the result is the offset and rstd = 1/sqrt(eps)."""
    o = np.full((1, 2, 4, 4), -3.5)
    bet = np.arange(16.0)
    y, mean, rstd = f(o, np.full(16, 9.0), bet, 1e-4)
    np.testing.assert_array_equal(y.reshape(2, 16), np.stack([bet, bet]))
    np.testing.assert_array_equal(mean, -3.5)
    np.testing.assert_allclose(rstd, 100.0, rtol=1e-15)
    s_h, m2_h = g(o)
    np.testing.assert_array_equal(s_h, -14.0)
    np.testing.assert_array_equal(m2_h, 0.0)


def pin_library_layernorm(f, g):
    rng = np.random.default_rng(63)
    for (B, T, H, N) in [(1, 1, 1, 64), (2, 3, 4, 64), (1, 2, 32, 64)]:
        D = H * N
        o = rng.standard_normal((B, T, H, N)) * rng.uniform(0.1, 5.0, (B, T, 1, 1)) + rng.standard_normal((B, T, H, 1))
        gam, bet = rng.standard_normal(D), rng.standard_normal(D)
        ref = torch.nn.functional.layer_norm(torch.from_numpy(o.reshape(B, T, D)), (D,), torch.from_numpy(gam),
                                             torch.from_numpy(bet), 1e-5).numpy()
        y, _, _ = f(o, gam, bet, 1e-5)
        np.testing.assert_allclose(y.reshape(B, T, D), ref, rtol=0, atol=1e-12)


def pin_heads_share_one_normalisation(f, g):
    """Two heads with different offsets: normalising each head on its own (a GroupNorm) would
    erase the offsets; the LayerNorm over the concatenation keeps them.  Head 0 = (-1, 1) - 10,
    head 1 = (-1, 1) + 10: mean 0, variance (81 + 121 + 81 + 121)/4 = 101."""
    o = np.array([-11.0, -9.0, 9.0, 11.0]).reshape(1, 1, 2, 2)
    y, _, _ = f(o, *ones_zeros(4), 0.0)
    np.testing.assert_allclose(y.reshape(4), np.array([-11.0, -9.0, 9.0, 11.0]) / np.sqrt(101.0), rtol=1e-15)


def pin_moments_combine_to_token_statistics(f, g):
    """sum_h s_h = D mean;  sum_h m2_h + N sum_h (s_h/N - mean)^2 = D var (pairwise-combination
    identity), checked against numpy's own mean and variance of the concatenation."""
    rng = np.random.default_rng(64)
    B, T, H, N = 2, 6, 5, 16
    o = rng.standard_normal((B, T, H, N)) * 2.0 + rng.standard_normal((1, 1, H, 1)) * 3.0
    s_h, m2_h = g(o)
    assert s_h.shape == (B, H, T) and m2_h.shape == (B, H, T)
    z = o.reshape(B, T, H * N)
    mean = s_h.sum(axis=1) / (H * N)
    np.testing.assert_allclose(mean, z.mean(axis=-1), atol=1e-13)
    m2 = m2_h.sum(axis=1) + N * ((s_h / N - mean[:, None, :]) ** 2).sum(axis=1)
    np.testing.assert_allclose(m2 / (H * N), z.var(axis=-1), rtol=1e-12)
    # each head's pair on its own: numpy's sum and variance of that head
    np.testing.assert_allclose(s_h, np.transpose(o.sum(axis=-1), (0, 2, 1)), atol=1e-13)
    np.testing.assert_allclose(m2_h, np.transpose(o.var(axis=-1) * N, (0, 2, 1)), rtol=1e-12)
    # and the LayerNorm's own statistics agree with them
    _, mu, rstd = f(o, *ones_zeros(H * N), 1e-5)
    np.testing.assert_allclose(mu, mean, atol=1e-13)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(m2 / (H * N) + 1e-5), rtol=1e-12)


PINS = [pin_hand_token, pin_result_is_standardised, pin_shift_and_scale_invariance, pin_constant_token,
        pin_library_layernorm, pin_heads_share_one_normalisation, pin_moments_combine_to_token_statistics]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(ln, moments)


def wrong_ln(kind):
    def f(o, gamma, beta, eps):
        o = np.asarray(o, dtype=np.float64)
        B, T, H, N = o.shape
        D = H * N
        z = o.reshape(B, T, D)
        gamma = np.asarray(gamma, dtype=np.float64).reshape(D)
        beta = np.asarray(beta, dtype=np.float64).reshape(D)
        m = z.mean(axis=-1, keepdims=True)
        dev = z - m
        var = (dev ** 2).sum(axis=-1, keepdims=True) / D
        if kind == "unbiased_variance":
            var = (dev ** 2).sum(axis=-1, keepdims=True) / (D - 1)
        if kind == "second_moment_for_variance":
            var = (z ** 2).sum(axis=-1, keepdims=True) / D
        rs = 1.0 / np.sqrt(var + eps)
        if kind == "eps_outside_root":
            rs = 1.0 / (np.sqrt(var) + eps)
        if kind == "mean_not_removed":
            dev = z
        y = dev * rs * gamma + beta
        if kind == "per_head_normalisation":
            zh = o - o.mean(axis=-1, keepdims=True)
            y = (zh / np.sqrt(o.var(axis=-1, keepdims=True) + eps)).reshape(B, T, D) * gamma + beta
        if kind == "gain_and_offset_swapped":
            y = dev * rs * beta + gamma
        if kind == "gain_per_head_channel_transposed":
            y = dev * rs * gamma.reshape(H, N).T.reshape(D) + beta if H == N else dev * rs * gamma[::-1] + beta
        if kind == "offset_inside_scaling":
            y = (dev + beta) * rs * gamma
        return y.reshape(B, T, H, N), m[..., 0], rs[..., 0]
    return f


def wrong_moments(kind):
    def g(o):
        o = np.asarray(o, dtype=np.float64)
        N = o.shape[-1]
        s = np.transpose(o.sum(axis=-1), (0, 2, 1))
        m2 = np.transpose(((o - o.mean(axis=-1, keepdims=True)) ** 2).sum(axis=-1), (0, 2, 1))
        if kind == "raw_square_sum":
            m2 = np.transpose((o ** 2).sum(axis=-1), (0, 2, 1))
        if kind == "variance_instead_of_m2":
            m2 = m2 / N
        if kind == "mean_instead_of_sum":
            s = s / N
        if kind == "token_major_layout":
            s, m2 = np.transpose(s, (0, 2, 1)), np.transpose(m2, (0, 2, 1))
        return s, m2
    return g


LN_MISTAKES = ["unbiased_variance", "second_moment_for_variance", "eps_outside_root", "mean_not_removed",
               "per_head_normalisation", "gain_and_offset_swapped", "gain_per_head_channel_transposed",
               "offset_inside_scaling"]
MOMENT_MISTAKES = ["raw_square_sum", "variance_instead_of_m2", "mean_instead_of_sum", "token_major_layout"]


def test_unplanted_variants_pass_all_pins():
    for pin in PINS:
        pin(wrong_ln("none"), wrong_moments("none"))


@pytest.mark.parametrize("kind", LN_MISTAKES)
def test_each_planted_layernorm_mistake_fails_a_pin(kind):
    failed = []
    for pin in PINS:
        try:
            pin(wrong_ln(kind), moments)
        except AssertionError:
            failed.append(pin.__name__)
    assert failed, f"no pin notices the planted mistake '{kind}'"


@pytest.mark.parametrize("kind", MOMENT_MISTAKES)
def test_each_planted_moment_mistake_fails_a_pin(kind):
    failed = []
    for pin in PINS:
        try:
            pin(ln, wrong_moments(kind))
        except AssertionError:
            failed.append(pin.__name__)
    assert failed, f"no pin notices the planted mistake '{kind}'"
