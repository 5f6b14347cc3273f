"""Float64 CPU oracle for the adaptive refresh of stale statistics -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Plain numpy / Python, written out from the definitions of the paper (Sec. 4.3 "Natural Gradient
with Stale Statistics": Algorithm 1, Algorithm 2 and the similarity criterion under them).
Only the tests may import this module; it imports nothing from the GPU package.

Readings where the paper is silent (the same ones the library takes):
  * a statistic that has no predecessor yet (X_-1 or X_-2 undefined at the first refreshes)
    counts as "not similar" to it;
  * every interval starts at 1 (Delta = Delta_-1 = 1), every statistic is due at step 1;
  * Algorithm 2's header names its interval inputs Delta_-1, Delta_-2 while Algorithm 1 passes
    (Delta, Delta_-1): on entry they are the two most recent intervals, most recent first, and
    the result is (new interval, the most recent one of the inputs);
  * ||B||_F = 0: the ratio is 0 if X equals B as well, else +infinity.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np


def frobenius_ratio(X, B) -> float:
    """||X - B||_F / ||B||_F with ||M||_F = sqrt(sum_ij M_ij^2)  (criterion below Algorithm 2)."""
    X = np.asarray(X, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    assert X.shape == B.shape
    num = 0.0
    den = 0.0
    for x_row, b_row in zip(X.reshape(X.shape[0], -1), B.reshape(B.shape[0], -1)):
        d = x_row - b_row
        num += float(np.sum(d * d))
        den += float(np.sum(b_row * b_row))
    if den == 0.0:
        return 0.0 if num == 0.0 else math.inf
    return math.sqrt(num) / math.sqrt(den)


def is_similar(X, B, alpha: float) -> bool:
    """A is "similar to" B when ||A - B||_F / ||B||_F < alpha; an undefined B is never similar."""
    if B is None:
        return False
    return frobenius_ratio(X, B) < alpha


def next_interval(similar_last: bool, similar_before_last: bool, delta_m1: int, delta_m2: int) -> int:
    """Algorithm 2: the acceptable interval until the next refresh.

    delta_m1 is the last interval, delta_m2 the one before it."""
    if not similar_last:
        return max(1, delta_m1 // 2)
    if not similar_before_last:
        return delta_m1
    return delta_m1 + delta_m2


class RefreshState:
    """What Algorithm 1 keeps per statistic X: the step of its next refresh and its two most recent intervals."""

    def __init__(self):
        self.t_next = 1
        self.delta = 1
        self.delta_m1 = 1

    def due(self, t: int) -> bool:
        return t == self.t_next

    def refreshed(self, similar_last: bool, similar_before_last: bool) -> None:
        """The body of Algorithm 1's `if t == t_X` after the statistic has been recomputed."""
        new = next_interval(similar_last, similar_before_last, self.delta, self.delta_m1)
        self.delta, self.delta_m1 = new, self.delta
        self.t_next += self.delta


def run_schedule(statistic_at, n_steps: int, alpha: float) -> Tuple[List[int], List[int]]:
    """Algorithm 1 for one statistic: statistic_at(t) is the value a refresh at step t yields.

    Returns the steps at which the statistic was refreshed and the interval chosen at each."""
    st = RefreshState()
    X1: Optional[np.ndarray] = None
    X2: Optional[np.ndarray] = None
    steps: List[int] = []
    deltas: List[int] = []
    for t in range(1, n_steps + 1):
        if st.due(t):
            X = np.asarray(statistic_at(t), dtype=np.float64)
            st.refreshed(is_similar(X, X1, alpha), is_similar(X, X2, alpha))
            X1, X2 = X, X1
            steps.append(t)
            deltas.append(st.delta)
    return steps, deltas


def staleness(Xs: Sequence, X1s: Sequence, X2s: Sequence) -> np.ndarray:
    """For each statistic i: (ratio to X_-1, ratio to X_-2); +infinity where the predecessor is undefined."""
    out = np.empty((len(Xs), 2), dtype=np.float64)
    for i, X in enumerate(Xs):
        out[i, 0] = math.inf if X1s[i] is None else frobenius_ratio(X, X1s[i])
        out[i, 1] = math.inf if X2s[i] is None else frobenius_ratio(X, X2s[i])
    return out
