"""Pins of the oracle's row normalisation and of the surrogate applied on top of it.

RMS normalisation has a closed form, so the pins are the mathematics: a hand loop, the
unit-mean-square property, invariance to the scale of a row, the identity on rows that
already have unit mean square, linearity in the gain, and the limit of a large eps."""
import math

import numpy as np

from oracle import kvzap_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def test_hand_loop():
    r = _rng(0)
    T, Dh, eps = 7, 24, 1e-3
    x = r.normal(size=(T, Dh)) * r.uniform(0.1, 30.0, size=(T, 1))
    g = r.normal(size=Dh)
    y = O.rmsnorm(x, g, eps)
    inv = O.rstd(x, eps)
    for t in range(T):
        ms = 0.0
        for k in range(Dh):
            ms += x[t, k] * x[t, k]
        ms /= Dh
        s = 1.0 / math.sqrt(ms + eps)
        assert abs(inv[t] - s) <= 1e-15 * s
        for k in range(Dh):
            assert abs(y[t, k] - x[t, k] * s * g[k]) <= 1e-14 * (1 + abs(y[t, k]))


def test_unit_mean_square_and_scale_invariance():
    r = _rng(1)
    x = r.normal(size=(50, 64))
    ones = np.ones(64)
    y = O.rmsnorm(x, ones, 0.0)
    np.testing.assert_allclose(np.mean(y * y, axis=1), 1.0, rtol=1e-13)
    for c in (1e-3, 7.5, -2.0, 1e6):
        yc = O.rmsnorm(c * x, ones, 0.0)
        np.testing.assert_allclose(yc, np.sign(c) * y, rtol=1e-12, atol=1e-15)
    # a row that already has unit mean square is left alone; the sign of every entry survives
    np.testing.assert_allclose(O.rmsnorm(y, ones, 0.0), y, rtol=1e-13)
    assert (np.sign(y) == np.sign(x)).all()


def test_gain_is_a_diagonal_map_and_eps_shrinks():
    r = _rng(2)
    x = r.normal(size=(9, 32)); g = r.normal(size=32)
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-6), O.rmsnorm(x, np.ones(32), 1e-6) * g, rtol=1e-14)
    np.testing.assert_allclose(O.rmsnorm(x, 2 * g, 1e-6), 2 * O.rmsnorm(x, g, 1e-6), rtol=1e-14)
    # eps much larger than the mean square: y ~ x * gain / sqrt(eps)
    big = 1e8
    np.testing.assert_allclose(O.rmsnorm(x, g, big), x * g / math.sqrt(big), rtol=1e-7)
    # a zero row stays zero for eps > 0
    z = np.zeros((1, 32))
    assert (O.rmsnorm(z, g, 1e-6) == 0).all() and O.rstd(z, 1e-6)[0] == 1e3


def test_surrogate_on_normalised_rows():
    r = _rng(3)
    T, Dh, M, H, eps = 40, 64, 16, 3, 1e-5
    x = r.normal(size=(T, Dh)) * r.uniform(0.5, 20.0, size=(T, 1))
    g = r.normal(size=Dh)
    W1 = r.normal(size=(Dh, M)) / math.sqrt(Dh); b1 = 0.1 * r.normal(size=M)
    W2 = r.normal(size=(M, H)) / math.sqrt(M); b2 = 0.1 * r.normal(size=H)
    S = O.score_mlp_rmsnorm(x, g, eps, W1, b1, W2, b2)
    # definition: the surrogate of the normalised rows, position by position
    for t in (0, 17, T - 1):
        y = x[t] / math.sqrt(float(np.mean(x[t] ** 2)) + eps) * g
        z = y @ W1 + b1
        want = (0.5 * z * (1 + np.vectorize(math.erf)(z / math.sqrt(2)))) @ W2 + b2
        np.testing.assert_allclose(S[:, t], want, rtol=1e-12, atol=1e-14)
    # the gain can be moved into the first projection's rows, the row scale behind it:
    # z = rstd * (x @ (gain[:, None] * W1)) + b1  (what a fused kernel may compute)
    z2 = O.rstd(x, eps)[:, None] * (x @ (g[:, None] * W1)) + b1
    np.testing.assert_allclose(S, (O.gelu(z2) @ W2 + b2).T, rtol=1e-11, atol=1e-13)
    # with eps = 0 the scores do not depend on a positive rescaling of a token's state
    S0 = O.score_mlp_rmsnorm(x, g, 0.0, W1, b1, W2, b2)
    Sc = O.score_mlp_rmsnorm(x * r.uniform(0.1, 9.0, size=(T, 1)), g, 0.0, W1, b1, W2, b2)
    np.testing.assert_allclose(S0, Sc, rtol=1e-10, atol=1e-12)
