"""GPU parity of the stale-statistics path (Sec. 4.3): the staleness ratios against the float64
oracle, and Algorithm 1 driven by the library (device ratios + host state) against the oracle's run."""
import math

import numpy as np
import pytest
import torch

from oracle import stale
from paper_2002_06015_amd import kfac, workloads as wl

pytestmark = pytest.mark.gpu

ALPHA = 0.1
TOL = 1e-11     # double accumulation of exactly converted floats: only the order of the sums differs


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    kfac.lib()   # fails loudly if the HIP library is not built
    return torch.device("cuda")


def _close(got, ref):
    if math.isinf(ref):
        return math.isinf(got) and got > 0
    return abs(got - ref) <= TOL * max(ref, 1e-300)


def _run(ctx, dims, X, P, Q):
    dv = lambda m: None if m is None else torch.from_numpy(np.ascontiguousarray(m, dtype=np.float32)).cuda()
    dX, dP, dQ = [dv(m) for m in X], [dv(m) for m in P], [dv(m) for m in Q]
    out = torch.full((2 * len(dims),), -1.0, dtype=torch.float64, device="cuda")
    kfac.kfac_staleness(ctx, dims, dX, None if all(m is None for m in dP) else dP,
                        None if all(m is None for m in dQ) else dQ, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().reshape(-1, 2)


def test_staleness_matches_oracle(gpu):
    """Sizes from one element to several chunks with ragged tails (n^2 % 4 != 0, n^2 % 4096 != 0), missing
    predecessors, a zero predecessor, an identical one."""
    dims = [1, 2, 3, 63, 64, 65, 130, 577, 1153, 64, 7, 7, 129]
    rng = np.random.default_rng(42)
    X = [rng.standard_normal((d, d)).astype(np.float32) for d in dims]
    P = [x + 0.05 * rng.standard_normal(x.shape).astype(np.float32) for x in X]
    Q = [x * np.float32(1.5) for x in X]
    P[1] = None                       # no predecessor yet
    Q[2] = None
    P[9] = X[9].copy()                # identical: ratio exactly 0
    Q[10] = np.zeros_like(X[10])      # zero predecessor, X != 0: +inf
    X[11] = np.zeros_like(X[11]); P[11] = np.zeros_like(X[11])   # both zero: 0
    layers = [wl.fc_layer(2, 1200, 1200, bias=0)]   # a context whose workspace covers the partial sums
    ctx = kfac.Context(layers)
    got = _run(ctx, dims, X, P, Q)
    ref = stale.staleness(X, P, Q)
    for i in range(len(dims)):
        assert _close(got[i, 0], ref[i, 0]) and _close(got[i, 1], ref[i, 1]), (i, got[i], ref[i])
    assert got[9, 0] == 0.0 and got[11, 0] == 0.0 and math.isinf(got[10, 1]) and math.isinf(got[1, 0])
    # the same inputs give the same bits
    again = _run(ctx, dims, X, P, Q)
    assert np.array_equal(got, again, equal_nan=True)
    ctx.close()


def test_algorithm_1_on_the_gpu_matches_oracle(gpu):
    """Three statistics with different dynamics over 60 steps: the library's state machine, fed with the ratios the
    GPU computes, refreshes them at the same steps and with the same intervals as the oracle's run."""
    n_steps = 60
    rng = np.random.default_rng(7)
    base = [rng.standard_normal((33, 33)).astype(np.float32), rng.standard_normal((130, 130)).astype(np.float32),
            rng.standard_normal((65, 65)).astype(np.float32)]
    noise = [rng.standard_normal((n_steps + 1, 65, 65)).astype(np.float32)]
    def value(i, t):
        if i == 0:
            return base[0]                                               # never changes
        if i == 1:
            return base[1] if t < 20 else (base[1] * np.float32(2.0))    # one jump
        return base[2] + np.float32(0.02 * t) * base[2] + np.float32(1e-3) * noise[0][t]   # steady drift
    ctx = kfac.Context([wl.fc_layer(2, 200, 200, bias=0)])
    states = kfac.kfac_refresh_init(3)
    prev1, prev2 = [None] * 3, [None] * 3
    steps, deltas = [[] for _ in range(3)], [[] for _ in range(3)]
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    for t in range(1, n_steps + 1):
        for i in range(3):
            if not kfac.kfac_refresh_due(states[i], t):
                continue
            X = torch.from_numpy(value(i, t)).cuda()
            kfac.kfac_staleness(ctx, [X.shape[0]], [X], None if prev1[i] is None else [prev1[i]],
                                None if prev2[i] is None else [prev2[i]], out)
            r = out.cpu().numpy()
            kfac.kfac_refresh_advance(states[i], float(r[0]), float(r[1]), ALPHA)
            prev1[i], prev2[i] = X, prev1[i]
            steps[i].append(t); deltas[i].append(states[i].delta)
    ctx.close()
    for i in range(3):
        ref_steps, ref_deltas = stale.run_schedule(lambda t: value(i, t), n_steps, ALPHA)
        assert steps[i] == ref_steps and deltas[i] == ref_deltas, (i, steps[i], ref_steps)
    assert steps[0] == [1, 2, 3, 5, 8, 13, 21, 34, 55]


def test_staleness_full_resnet50_factor_set(gpu):
    """All 108 factors of configuration 4 (dims 64 .. 4609, 155 M elements) against their two predecessors in one call."""
    layers = wl.config_layers(4)
    dims = [L.dA for L in layers] + [L.dG for L in layers]
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    X = [torch.randn(d, d, device="cuda", generator=g) for d in dims]
    P = [x + 0.03 * torch.randn(x.shape, device="cuda", generator=g) for x in X]
    Q = [x * 0.8 for x in X]
    ctx = kfac.Context(layers)
    out = torch.zeros(2 * len(dims), dtype=torch.float64, device="cuda")
    kfac.kfac_staleness(ctx, dims, X, P, Q, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(-1, 2)
    kfac.kfac_staleness(ctx, dims, X, P, Q, out)
    torch.cuda.synchronize()
    assert np.array_equal(got, out.cpu().numpy().reshape(-1, 2))
    # every Q ratio is |1 - 0.8| / 0.8 up to the rounding of 0.8 x in fp32; the oracle on a sample of the matrices
    for i in list(range(0, len(dims), 9)) + [int(np.argmax(dims))]:
        ref1 = stale.frobenius_ratio(X[i].cpu().numpy(), P[i].cpu().numpy())
        ref2 = stale.frobenius_ratio(X[i].cpu().numpy(), Q[i].cpu().numpy())
        assert _close(got[i, 0], ref1) and _close(got[i, 1], ref2), (i, got[i], ref1, ref2)
    assert np.all(np.abs(got[:, 1] - 0.25) < 1e-6)
    ctx.close()
