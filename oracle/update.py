"""Float64 CPU oracle for the end of the optimisation step -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Sec. 6.2 ("Learning rate and momentum": polynomial decay, momentum tied to the learning rate,
the parameter update) and Sec. 6.3 ("Weights rescaling"), written out from the equations.
Only the tests may import this module; it imports nothing from the GPU package.

Readings where the paper is silent (the same ones the library takes):
  * a layer's w is the matrix [d_out, d_in k^2 (+1)] the preconditioned gradient U has, bias
    column included if the layer has one (the paper ignores biases); ||w|| is its Frobenius norm;
  * v^(t) = w^(t) - w^(t-1) uses the weights as they were stored, i.e. after the rescaling of the
    step before;
  * the learning rate formula is used as printed for e_start <= e <= e_end; before e_start it is
    eta^(0), after e_end it is 0.
"""
from __future__ import annotations

import math
from typing import Tuple

import numpy as np


def lr_polynomial(eta0: float, e: float, e_start: float, e_end: float, p_decay: float) -> float:
    """eta^(e) = eta^(0) (1 - (e - e_start) / (e_end - e_start))^p_decay."""
    if e <= e_start:
        return eta0
    if e >= e_end:
        return 0.0
    return eta0 * (1.0 - (e - e_start) / (e_end - e_start)) ** p_decay


def momentum_coupled(m0: float, eta0: float, eta: float) -> float:
    """m^(e) = m^(0) / eta^(0) * eta^(e)."""
    return m0 / eta0 * eta


def update_weights(W, W_prev, U, eta: float, momentum: float, d_out: int, rescale: bool,
                   eps: float = 1e-9) -> Tuple[np.ndarray, np.ndarray]:
    """w^(t+1) = w^(t) - eta U + m (w^(t) - w^(t-1)), then (optionally) w^(t+1) <- sqrt(2 d_out) w^(t+1) / (||w^(t+1)|| + eps).

    Returns (w^(t+1), w^(t)): the new weights and what the next step uses as its previous ones."""
    W = np.asarray(W, dtype=np.float64)
    W_prev = np.asarray(W_prev, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    v = W - W_prev
    new = W - eta * U + momentum * v
    if rescale:
        norm = math.sqrt(float(np.sum(new * new)))
        new = math.sqrt(2.0 * d_out) * new / (norm + eps)
    return new, W.copy()
