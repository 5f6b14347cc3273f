"""Pins of the update oracle (Sec. 6.2 and 6.3) against closed forms of the recurrences and of the schedules."""
import math

import numpy as np

from oracle import update


def test_polynomial_decay_closed_forms():
    eta0 = 0.8
    assert update.lr_polynomial(eta0, 3.0, 3.0, 40.0, 11.0) == eta0             # decay starts at e_start
    assert update.lr_polynomial(eta0, 40.0, 3.0, 40.0, 11.0) == 0.0             # and ends at e_end
    assert update.lr_polynomial(eta0, 1.0, 3.0, 40.0, 11.0) == eta0
    assert abs(update.lr_polynomial(eta0, 21.5, 3.0, 40.0, 1.0) - eta0 / 2) < 1e-15      # linear: half way
    assert abs(update.lr_polynomial(eta0, 21.5, 3.0, 40.0, 2.0) - eta0 / 4) < 1e-15      # quadratic: a quarter
    assert abs(update.lr_polynomial(eta0, 30.75, 3.0, 40.0, 3.0) - eta0 / 64) < 1e-15    # (1 - 3/4)^3
    es = np.linspace(3.0, 40.0, 50)
    vals = [update.lr_polynomial(eta0, e, 3.0, 40.0, 4.0) for e in es]
    assert all(a > b for a, b in zip(vals[:-1], vals[1:]))                     # strictly decreasing in between


def test_momentum_keeps_its_ratio_to_the_learning_rate():
    eta0, m0 = 0.8, 0.97
    for e in (0.0, 5.0, 17.0, 39.0):
        eta = update.lr_polynomial(eta0, e, 3.0, 40.0, 11.0)
        m = update.momentum_coupled(m0, eta0, eta)
        assert abs(m / eta - m0 / eta0) < 1e-12
    assert update.momentum_coupled(m0, eta0, eta0) == m0


def test_update_special_cases():
    rng = np.random.default_rng(0)
    W, Wp, U = rng.standard_normal((5, 7)), rng.standard_normal((5, 7)), rng.standard_normal((5, 7))
    new, prev = update.update_weights(W, Wp, U, 0.0, 0.0, 5, False)
    assert np.array_equal(new, W) and np.array_equal(prev, W)
    new, _ = update.update_weights(W, Wp, U, 0.25, 0.0, 5, False)
    assert np.allclose(new, W - 0.25 * U, rtol=0, atol=1e-15)                   # plain natural-gradient step
    new, _ = update.update_weights(W, W, U, 0.0, 0.9, 5, False)
    assert np.array_equal(new, W)                                              # no velocity yet: nothing moves
    new, _ = update.update_weights(W, Wp, 0 * U, 0.0, 1.0, 5, False)
    assert np.allclose(new, 2 * W - Wp, atol=1e-15)                            # m = 1: the last displacement again


def test_momentum_recurrence_closed_forms():
    """U = 0: the displacement shrinks by m each step, w_t = w_0 + v_0 (1 - m^t) / (1 - m).
    m = 0, constant U: w_t = w_0 - t eta U."""
    rng = np.random.default_rng(1)
    w0, v0, U = rng.standard_normal((3, 4)), rng.standard_normal((3, 4)), rng.standard_normal((3, 4))
    m = 0.6
    W, Wp = w0.copy(), w0 - v0
    for t in range(1, 12):
        W, Wp = update.update_weights(W, Wp, 0 * U, 0.1, m, 3, False)
        assert np.allclose(W, w0 + v0 * m * (1 - m ** t) / (1 - m), rtol=0, atol=1e-13)
    W, Wp = w0.copy(), w0.copy()
    for t in range(1, 9):
        W, Wp = update.update_weights(W, Wp, U, 0.05, 0.0, 3, False)
        assert np.allclose(W, w0 - t * 0.05 * U, rtol=0, atol=1e-13)
    # both: the heavy-ball sum  w_t = w_0 - eta U sum_{j<t} (1 - m^(t-j)) / (1 - m)
    W, Wp = w0.copy(), w0.copy()
    for t in range(1, 9):
        W, Wp = update.update_weights(W, Wp, U, 0.05, m, 3, False)
        s = sum((1 - m ** (t - j)) / (1 - m) for j in range(t))
        assert np.allclose(W, w0 - 0.05 * U * s, rtol=0, atol=1e-13)


def test_rescaling_gives_the_prescribed_norm_and_direction():
    rng = np.random.default_rng(2)
    W, Wp, U = rng.standard_normal((6, 9)), rng.standard_normal((6, 9)), rng.standard_normal((6, 9))
    plain, _ = update.update_weights(W, Wp, U, 0.1, 0.5, 6, False)
    new, prev = update.update_weights(W, Wp, U, 0.1, 0.5, 6, True)
    n = np.linalg.norm(plain)
    assert abs(np.linalg.norm(new) - math.sqrt(12.0) * n / (n + 1e-9)) < 1e-12
    assert np.allclose(new / np.linalg.norm(new), plain / n, atol=1e-14)       # direction kept
    assert np.array_equal(prev, W)
    # only the direction of the updated weights matters (up to eps)
    big, _ = update.update_weights(10 * W, 10 * Wp, 10 * U, 0.1, 0.5, 6, True)
    assert np.allclose(big, new, rtol=1e-9)
    # all-zero weights stay zero (eps keeps the division finite)
    z, _ = update.update_weights(0 * W, 0 * W, 0 * U, 0.1, 0.5, 6, True)
    assert np.array_equal(z, 0 * W)
