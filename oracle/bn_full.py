"""Float64 CPU oracle for natural gradient on BatchNorm parameters with the whole layer Fisher
-- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Sec. 4.2 ("Practical FIM Estimation for BatchNorm Layers"): before the unit-wise approximation is
introduced, the parameters of a BatchNorm layer with c channels are one vector
w = (gamma_1, beta_1, ..., gamma_c, beta_c) and its Fisher block is the dense 2c x 2c matrix of
Eq. 5 (the empirical estimate: the mean over the mini-batch of the outer product of the
per-sample gradient with itself).  This is the variant the experiments call "fullBN".
Only the tests may import this module; it imports nothing from the GPU package.

Readings where the paper is silent (the same ones the library takes):
  * damping is plain Tikhonov, (F + lambda I)^-1, as for the unit-wise blocks (the split of the
    damping between two Kronecker factors has no counterpart for an unfactored block);
  * the running average of F follows the rule used for every other statistic:
    F <- decay * F + (1 - decay) * F_batch;
  * the gradient that is preconditioned is the mean over the mini-batch of the per-sample gradients.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def interleave(g_gamma, g_beta) -> np.ndarray:
    """Per-sample gradients [N, c] + [N, c] -> [N, 2c] in the order of w: (gamma_i, beta_i) next to each other."""
    gg = np.asarray(g_gamma, dtype=np.float64)
    gb = np.asarray(g_beta, dtype=np.float64)
    assert gg.shape == gb.shape and gg.ndim == 2
    N, c = gg.shape
    D = np.empty((N, 2 * c), dtype=np.float64)
    for i in range(c):
        D[:, 2 * i] = gg[:, i]
        D[:, 2 * i + 1] = gb[:, i]
    return D


def fisher_batch(g_gamma, g_beta) -> np.ndarray:
    """F = (1/N) sum_n g_n g_n^T with g_n the per-sample gradient w.r.t. w (Eq. 5 for this layer)."""
    D = interleave(g_gamma, g_beta)
    N = D.shape[0]
    F = np.zeros((D.shape[1], D.shape[1]), dtype=np.float64)
    for n in range(N):
        F += np.outer(D[n], D[n])
    return F / N


def bn_full_precondition(g_gamma, g_beta, decay: float, lam: float,
                         F_ema: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Returns (F_ema_new [2c, 2c], (F_ema_new + lam I)^-1, out_gamma [c], out_beta [c])."""
    F_b = fisher_batch(g_gamma, g_beta)
    n = F_b.shape[0]
    F_old = np.zeros_like(F_b) if F_ema is None else np.asarray(F_ema, dtype=np.float64).reshape(n, n)
    F_new = decay * F_old + (1.0 - decay) * F_b
    inv = np.linalg.inv(F_new + lam * np.eye(n))
    inv = 0.5 * (inv + inv.T)
    g_mean = interleave(g_gamma, g_beta).mean(axis=0)
    u = inv @ g_mean
    return F_new, inv, u[0::2].copy(), u[1::2].copy()
