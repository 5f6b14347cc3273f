"""kfac_staleness_static (the entry point that allocates nothing: chunk sums in the library's fixed
device array) against kfac_staleness (chunk sums in the caller's workspace), through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import stale
from paper_2002_06015_amd import kfac, workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-11    # the bar of the staleness parity tests (double sums of exactly converted floats)


def _mats(dims, seed):
    rng = np.random.default_rng(seed)
    X = [rng.standard_normal((d, d)).astype(np.float32) for d in dims]
    P = [x + 0.05 * rng.standard_normal(x.shape).astype(np.float32) for x in X]
    Q = [x * np.float32(1.5) for x in X]
    return X, P, Q


def _both(ctx, dims, X, P, Q):
    dv = lambda m: None if m is None else torch.from_numpy(m).cuda()
    dX, dP, dQ = [dv(m) for m in X], [dv(m) for m in P], [dv(m) for m in Q]
    ref = torch.full((2 * len(dims),), -1.0, dtype=torch.float64, device="cuda")
    got = torch.full((2 * len(dims),), -2.0, dtype=torch.float64, device="cuda")
    kfac.kfac_staleness(ctx, dims, dX, dP, dQ, ref)
    kfac.kfac_staleness_static(None, dims, dX, dP, dQ, got)
    torch.cuda.synchronize()
    return got.cpu().numpy().reshape(-1, 2), ref.cpu().numpy().reshape(-1, 2)


def _same(got, ref):
    for g, r in zip(got.ravel(), ref.ravel()):
        if np.isinf(r):
            assert np.isinf(g) and g > 0
        else:
            assert abs(g - r) <= TOL * max(abs(r), 1e-300), (g, r)


def test_static_scratch_staleness_matches_the_workspace_entry_point():
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    ctx = kfac.Context([wl.fc_layer(2, 2400, 2400, bias=0)])
    # first call: 70 matrices (more than one launch's table), several chunks each, ragged tails,
    # missing predecessors; 2305^2 alone is 1298 chunks
    dims = [1, 2, 3, 63, 64, 65, 130, 577, 1153, 2305] + [97 + 3 * i for i in range(60)]
    X, P, Q = _mats(dims, 5)
    P[1] = None
    Q[2] = None
    Q[7] = np.zeros_like(X[7])
    got, ref = _both(ctx, dims, X, P, Q)
    _same(got, ref)
    want = stale.staleness(X, P, Q)
    _same(got, want)
    # second call, smaller input: whatever the first call left in the array must not matter
    dims2 = [65, 7, 130]
    X2, P2, Q2 = _mats(dims2, 6)
    got2, ref2 = _both(ctx, dims2, X2, P2, Q2)
    _same(got2, ref2)
    _same(got2, stale.staleness(X2, P2, Q2))
    ctx.close()


def test_static_scratch_staleness_rejects_what_does_not_fit():
    """Host-side checks only: nothing is launched for a rejected call."""
    L = kfac.lib()
    dims = (ctypes.c_int32 * 1)(8193)
    one = (ctypes.c_void_p * 1)(256)
    st = L.kfac_staleness_static(None, 1, ctypes.addressof(dims), ctypes.addressof(one), None, None, ctypes.c_void_p(512))
    assert st == kfac.KFAC_ERR_WORKSPACE
    dims[0] = 64
    assert L.kfac_staleness_static(None, 0, ctypes.addressof(dims), ctypes.addressof(one), None, None,
                                   ctypes.c_void_p(512)) == kfac.KFAC_ERR_INVALID
    assert L.kfac_staleness_static(None, 1, ctypes.addressof(dims), ctypes.addressof(one), None, None,
                                   None) == kfac.KFAC_ERR_INVALID
    same = (ctypes.c_void_p * 1)(256)
    assert L.kfac_staleness_static(None, 1, ctypes.addressof(dims), ctypes.addressof(one), ctypes.addressof(same), None,
                                   ctypes.c_void_p(512)) == kfac.KFAC_ERR_INVALID
