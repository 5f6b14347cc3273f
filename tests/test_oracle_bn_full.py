"""Pins of the oracle for the whole-layer BatchNorm Fisher (Sec. 4.2, the variant before the unit-wise approximation)."""
import numpy as np
import torch

import oracle
from oracle import bn_full


def _grads(N, c, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((N, c)), rng.standard_normal((N, c)) * 0.7 + 0.1


def test_fisher_is_the_mean_outer_product_of_autograd_per_sample_gradients():
    """y = gamma * xhat + beta in front of a loss: per-sample gradients w.r.t. (gamma_1, beta_1, gamma_2, ...) by autograd."""
    torch.manual_seed(0)
    N, c, hw = 5, 3, 4
    xhat = torch.randn(N, c, hw, dtype=torch.float64)
    w = torch.randn(2 * c, dtype=torch.float64, requires_grad=True)       # the paper's ordering of the layer's parameters
    target = torch.randn(N, c, hw, dtype=torch.float64)
    rows, dys = [], []
    for n in range(N):
        y = w[0::2].view(c, 1) * xhat[n] + w[1::2].view(c, 1)
        y.retain_grad()
        loss = ((y - target[n]) ** 3).sum()
        (g,) = torch.autograd.grad(loss, w, retain_graph=True)
        (dy,) = torch.autograd.grad(loss, y)
        rows.append(g.numpy())
        dys.append(dy.numpy())
    G = np.stack(rows)
    F_ref = sum(np.outer(r, r) for r in G) / N
    gg, gb = oracle.bn_reduce_nchw(np.stack(dys), xhat.numpy())
    assert np.allclose(bn_full.interleave(gg, gb), G, rtol=1e-12, atol=1e-12)
    assert np.allclose(bn_full.fisher_batch(gg, gb), F_ref, rtol=1e-12, atol=1e-12)


def test_diagonal_blocks_are_the_unit_wise_statistics():
    gg, gb = _grads(7, 5, 1)
    F = bn_full.fisher_batch(gg, gb)
    assert np.array_equal(F, F.T)
    Fu, _, _ = oracle.bn_unitwise_precondition(gg, gb, 0.0, 0.1)
    for i in range(5):
        blk = F[2 * i:2 * i + 2, 2 * i:2 * i + 2]
        assert np.allclose([blk[0, 0], blk[0, 1], blk[1, 1]], [np.mean(gg[:, i] ** 2), np.mean(gg[:, i] * gb[:, i]),
                                                              np.mean(gb[:, i] ** 2)], rtol=1e-13)
        assert np.allclose([blk[0, 0], blk[0, 1], blk[1, 1]], Fu[i], rtol=1e-13)
    # an off-diagonal entry, typed out: gamma of channel 1 against beta of channel 3
    assert np.isclose(F[2, 7], np.mean(gg[:, 1] * gb[:, 3]), rtol=1e-13)
    assert np.isclose(F[7, 2], F[2, 7])


def test_channels_that_never_fire_together_reduce_to_the_two_by_two_closed_form():
    """Each sample carries gradient for one channel only: F is block diagonal and Eq. 17's formula applies per channel."""
    N, c = 12, 4
    rng = np.random.default_rng(2)
    gg, gb = np.zeros((N, c)), np.zeros((N, c))
    for n in range(N):
        gg[n, n % c], gb[n, n % c] = rng.standard_normal(2)
    lam = 0.03
    F, inv, og, ob = bn_full.bn_full_precondition(gg, gb, 0.0, lam)
    for i in range(c):
        for j in range(c):
            if i != j:
                assert np.all(F[2 * i:2 * i + 2, 2 * j:2 * j + 2] == 0.0)
        a, b, d = np.mean(gg[:, i] ** 2) + lam, np.mean(gg[:, i] * gb[:, i]), np.mean(gb[:, i] ** 2) + lam
        det = a * d - b * b
        mg, mb = gg[:, i].mean(), gb[:, i].mean()
        assert np.isclose(og[i], (d * mg - b * mb) / det, rtol=1e-11)
        assert np.isclose(ob[i], (-b * mg + a * mb) / det, rtol=1e-11)
    _, ug, ub = oracle.bn_unitwise_precondition(gg, gb, 0.0, lam)
    assert np.allclose(og, ug, rtol=1e-11) and np.allclose(ob, ub, rtol=1e-11)


def test_single_sample_is_sherman_morrison():
    """N = 1: (g g^T + lam I)^-1 g = g / (lam + |g|^2)."""
    gg, gb = _grads(1, 6, 3)
    lam = 0.25
    _, _, og, ob = bn_full.bn_full_precondition(gg, gb, 0.0, lam)
    s = lam + np.sum(gg ** 2) + np.sum(gb ** 2)
    assert np.allclose(og, gg[0] / s, rtol=1e-12) and np.allclose(ob, gb[0] / s, rtol=1e-12)


def test_woodbury_route_through_the_sample_space():
    """(lam I + D^T D / N)^-1 v = (v - D^T (N lam I + D D^T)^-1 D v) / lam, an N x N solve instead of 2c x 2c."""
    N, c = 4, 9
    gg, gb = _grads(N, c, 4)
    lam = 0.05
    _, inv, og, ob = bn_full.bn_full_precondition(gg, gb, 0.0, lam)
    D = np.empty((N, 2 * c))
    D[:, 0::2], D[:, 1::2] = gg, gb
    v = D.mean(axis=0)
    u = (v - D.T @ np.linalg.solve(N * lam * np.eye(N) + D @ D.T, D @ v)) / lam
    assert np.allclose(og, u[0::2], rtol=1e-10) and np.allclose(ob, u[1::2], rtol=1e-10)
    assert np.allclose(inv @ (D.T @ D / N + lam * np.eye(2 * c)), np.eye(2 * c), atol=1e-10)


def test_running_average_and_damping_limits():
    gg, gb = _grads(6, 3, 5)
    F1 = bn_full.fisher_batch(gg, gb)
    prev = np.arange(36, dtype=np.float64).reshape(6, 6)
    prev = prev + prev.T + 40 * np.eye(6)
    F, _, _, _ = bn_full.bn_full_precondition(gg, gb, 0.9, 1.0, prev)
    assert np.allclose(F, 0.9 * prev + 0.1 * F1, rtol=1e-14)
    F, _, _, _ = bn_full.bn_full_precondition(gg, gb, 0.0, 1.0, prev)
    assert np.allclose(F, F1, rtol=1e-14)
    F, _, _, _ = bn_full.bn_full_precondition(gg, gb, 1.0, 1.0, prev)
    assert np.allclose(F, prev, rtol=1e-14)
    lam = 1e9                                                            # damping dominates: u -> mean gradient / lam
    _, _, og, ob = bn_full.bn_full_precondition(gg, gb, 0.0, lam)
    assert np.allclose(og * lam, gg.mean(0), rtol=1e-6) and np.allclose(ob * lam, gb.mean(0), rtol=1e-6)
