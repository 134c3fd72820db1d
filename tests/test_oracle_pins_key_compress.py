"""Pins for the key-compression oracle (Method section, GOLD Key Compression:
c_t = x_t W^KD, W^KD with D rows and D/16 columns)."""
import numpy as np
import pytest

from oracle import key_compress_oracle


def c_oracle(x, w):
    return key_compress_oracle(x, w, nthreads=3)


def c_oracle_single_thread(x, w):
    return key_compress_oracle(x, w, nthreads=1)


def pin_hand_case(f):
    """D = 32, D/16 = 2 columns, two tokens, integers small enough to do by hand:
    token 0 = (1, 2, ..., 32), token 1 = all ones; column 0 of W = all ones, column 1 = (d mod 2)."""
    x = np.stack([np.arange(1, 33), np.ones(32)]).astype(np.float32)
    w = np.stack([np.ones(32), np.arange(32) % 2], axis=1).astype(np.float32)
    c = f(x, w)
    # sum 1..32 = 528; entries at odd d (values 2,4,..,32) sum to 272; token 1: 32 and 16
    assert c.shape == (2, 2)
    np.testing.assert_array_equal(c, np.array([[528.0, 272.0], [32.0, 16.0]]))


def pin_selector_matrix(f):
    """W with a single one per column copies that channel of x: c[:, n] = x[:, pick[n]]."""
    rng = np.random.default_rng(51)
    D, C = 64, 4
    x = rng.standard_normal((7, D)).astype(np.float32)
    pick = np.array([5, 0, 63, 17])
    w = np.zeros((D, C), np.float32)
    w[pick, np.arange(C)] = 1.0
    np.testing.assert_array_equal(f(x, w), x[:, pick].astype(np.float64))


def pin_linearity_and_token_independence(f):
    rng = np.random.default_rng(52)
    D, C = 48, 3
    x1, x2 = (rng.integers(-8, 9, (5, D)).astype(np.float32) for _ in range(2))
    w1, w2 = (rng.integers(-8, 9, (D, C)).astype(np.float32) for _ in range(2))
    np.testing.assert_array_equal(f(x1 + x2, w1), f(x1, w1) + f(x2, w1))      # integers: exact
    np.testing.assert_array_equal(f(x1, w1 + w2), f(x1, w1) + f(x1, w2))
    np.testing.assert_array_equal(f(x1, w1)[2:4], f(x1[2:4], w1))             # a token depends on no other


def pin_library_matrix_product(f):
    rng = np.random.default_rng(53)
    for (M, D) in [(1, 16), (9, 256), (33, 2048)]:
        x = rng.standard_normal((M, D)).astype(np.float32)
        w = (rng.standard_normal((D, D // 16)) / np.sqrt(D)).astype(np.float32)
        ref = x.astype(np.float64) @ w.astype(np.float64)
        np.testing.assert_allclose(f(x, w), ref, rtol=0, atol=1e-12 * max(1.0, np.abs(ref).max()))


def pin_leading_axes(f):
    rng = np.random.default_rng(54)
    x = rng.standard_normal((2, 3, 32)).astype(np.float32)
    w = rng.standard_normal((32, 2)).astype(np.float32)
    c = f(x, w)
    assert c.shape == (2, 3, 2)
    np.testing.assert_allclose(c[1, 2], x[1, 2].astype(np.float64) @ w.astype(np.float64), atol=1e-13)


PINS = [pin_hand_case, pin_selector_matrix, pin_linearity_and_token_independence,
        pin_library_matrix_product, pin_leading_axes]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
@pytest.mark.parametrize("impl", [c_oracle, c_oracle_single_thread], ids=lambda f: f.__name__)
def test_pin(impl, pin):
    pin(impl)


def wrong_variant(kind):
    def f(x, w):
        x = np.asarray(x, dtype=np.float64)
        w = np.asarray(w, dtype=np.float64)
        lead, D = x.shape[:-1], x.shape[-1]
        x2 = x.reshape(-1, D)
        if kind == "w_read_transposed":               # W stored [D][C] but indexed as [C][D]
            c = x2 @ w.reshape(w.shape[1], w.shape[0]).T
        elif kind == "drops_last_channel":
            c = x2[:, :-1] @ w[:-1]
        elif kind == "tokens_mixed":
            c = np.roll(x2, 1, axis=0) @ w
        elif kind == "float32_accumulate":
            c = np.zeros((x2.shape[0], w.shape[1]), np.float32)
            for d in range(D):
                c += (x2[:, d:d + 1] * w[d:d + 1]).astype(np.float32)
            c = c.astype(np.float64)
        elif kind == "columns_reversed":
            c = (x2 @ w)[:, ::-1]
        else:
            c = x2 @ w
        return c.reshape(*lead, w.shape[1])
    return f


MISTAKES = ["w_read_transposed", "drops_last_channel", "tokens_mixed", "float32_accumulate", "columns_reversed"]


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


def test_oracle_rejects_bad_shapes():
    with pytest.raises(ValueError):
        key_compress_oracle(np.zeros((3, 32), np.float32), np.zeros((16, 2), np.float32))
