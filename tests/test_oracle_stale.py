"""Pins of the stale-statistics oracle (Sec. 4.3, Algorithms 1 and 2) against things other than itself:
a library norm, closed forms, and interval sequences worked out by hand from the algorithm's text."""
import math
import os

import numpy as np
import pytest

from oracle import stale


def _alpha():
    with open(os.path.join(os.path.dirname(__file__), "golden", "stale_facts.txt")) as f:
        for line in f:
            if line.startswith("stale_alpha"):
                return float(line.split("=")[1])
    raise AssertionError("stale_alpha missing")


ALPHA = _alpha()


@pytest.mark.parametrize("shape", [(1, 1), (3, 3), (17, 17), (65, 65), (130, 130)])
def test_ratio_equals_library_frobenius_norms(shape):
    rng = np.random.default_rng(shape[0])
    X, B = rng.standard_normal(shape), rng.standard_normal(shape)
    ref = np.linalg.norm(X - B, "fro") / np.linalg.norm(B, "fro")
    assert abs(stale.frobenius_ratio(X, B) - ref) <= 1e-13 * ref


def test_ratio_closed_forms():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((9, 9))
    assert stale.frobenius_ratio(X, X) == 0.0
    for c in (0.5, 2.0, -3.0, 1.0625):
        # ||X - cX|| / ||cX|| = |1 - c| / |c|
        assert abs(stale.frobenius_ratio(X, c * X) - abs(1 - c) / abs(c)) <= 1e-13
    E = np.zeros((4, 4)); E[1, 2] = 1.0
    F = np.zeros((4, 4)); F[3, 0] = 1.0
    assert abs(stale.frobenius_ratio(E, F) - math.sqrt(2.0)) <= 1e-15      # two different unit matrices
    assert abs(stale.frobenius_ratio(3 * E + 4 * F, F) - math.sqrt(9 + 9)) <= 1e-14
    Z = np.zeros((4, 4))
    assert stale.frobenius_ratio(Z, Z) == 0.0 and stale.frobenius_ratio(E, Z) == math.inf
    # not symmetric in its arguments: the norm of the *second* one divides
    assert abs(stale.frobenius_ratio(2 * E, E) - 1.0) <= 1e-15 and abs(stale.frobenius_ratio(E, 2 * E) - 0.5) <= 1e-15


def test_similarity_threshold_is_strict_and_undefined_is_dissimilar():
    X = np.eye(3)
    assert stale.is_similar(X, X / (1 + 0.0999), ALPHA)            # ratio 0.0999
    assert not stale.is_similar(X, X / (1 + 0.1001), ALPHA)        # ratio 0.1001
    assert not stale.is_similar(X, None, ALPHA)
    # "< alpha", not "<=": ratio exactly 0.5 against alpha = 0.5
    assert not stale.is_similar(np.array([[1.5]]), np.array([[1.0]]), 0.5)


def test_interval_rule_cases():
    # not similar to the last: halve, floor, at least 1
    assert [stale.next_interval(False, s2, d, 7) for d in (1, 2, 3, 5, 8, 13) for s2 in (False, True)] == \
        [1, 1, 1, 1, 1, 1, 2, 2, 4, 4, 6, 6]
    # similar to the last, not to the one before: keep
    assert [stale.next_interval(True, False, d, 99) for d in (1, 4, 13)] == [1, 4, 13]
    # similar to both: sum of the two last intervals
    assert stale.next_interval(True, True, 5, 3) == 8 and stale.next_interval(True, True, 1, 1) == 2


def test_constant_statistic_gives_fibonacci_refresh_steps():
    """A statistic that never changes: the first refresh has no predecessor (interval 1), the second none
    before the last (keep 1), after that the interval is the sum of the two before it."""
    steps, deltas = stale.run_schedule(lambda t: np.eye(4), 60, ALPHA)
    assert steps == [1, 2, 3, 5, 8, 13, 21, 34, 55]
    assert deltas == [1, 1, 2, 3, 5, 8, 13, 21, 34]


def test_ever_changing_statistic_is_refreshed_every_step():
    rng = np.random.default_rng(0)
    steps, deltas = stale.run_schedule(lambda t: rng.standard_normal((5, 5)), 12, ALPHA)
    assert steps == list(range(1, 13)) and deltas == [1] * 12


def test_jump_halves_then_recovers():
    """Worked by hand: constant until step 20, another constant from step 20 on.
    Refreshes 1,2,3,5,8,13 as above (interval 8 chosen at 13 -> next at 21).  At 21 the value differs from the
    one of step 13: halve 8 -> 4, next 25.  At 25: same as at 21 but not as at 13: keep 4, next 29.  At 29:
    same as both: 4 + 4 = 8, next 37.  At 37: 8 + 4 = 12, next 49."""
    val = lambda t: np.eye(3) if t < 20 else 2.0 * np.eye(3)
    steps, deltas = stale.run_schedule(val, 50, ALPHA)
    assert steps == [1, 2, 3, 5, 8, 13, 21, 25, 29, 37, 49]
    assert deltas == [1, 1, 2, 3, 5, 8, 4, 4, 8, 12, 20]


def test_slow_drift_keeps_a_bounded_interval():
    """X_t = (1 + 0.03 t) I: a refresh after an interval D from step s sees the ratio 0.03 D / (1 + 0.03 s) to the
    last value, so the interval cannot stay above (1 + 0.03 s) * alpha / 0.03 for long: it is halved again."""
    steps, deltas = stale.run_schedule(lambda t: (1.0 + 0.03 * t) * np.eye(2), 200, ALPHA)
    for s, s_next in zip(steps[:-1], steps[1:]):
        ratio = 0.03 * (s_next - s) / (1.0 + 0.03 * s)
        # an interval that turned out too long is never followed by a longer one
        if ratio >= ALPHA:
            k = steps.index(s_next)
            assert deltas[k] <= max(1, (s_next - s) // 2)
    assert max(deltas) < 200 and len(steps) < 200


def test_staleness_table():
    rng = np.random.default_rng(3)
    X = [rng.standard_normal((6, 6)), rng.standard_normal((3, 3))]
    P = [X[0] * 1.25, None]
    Q = [None, X[1] - 1.0]
    out = stale.staleness(X, P, Q)
    assert abs(out[0, 0] - 0.2) <= 1e-14 and out[0, 1] == math.inf and out[1, 0] == math.inf
    assert abs(out[1, 1] - 3.0 / np.linalg.norm(Q[1], "fro")) <= 1e-14
