"""CPU-only checks of the C-ABI boundary: the library loads, exports what the header
declares, sizes workspaces, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2002_06015_amd import kfac, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "kfac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(kfac_[a-z0-9_]+|bn_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = kfac.lib()
    declared = _declared_functions()
    assert set(declared) == set(kfac.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings():
    assert kfac.status_string(kfac.KFAC_OK) == "ok"
    for s in range(5):
        assert kfac.status_string(s)


def test_layer_dims_and_validation():
    assert kfac.kfac_layer_dims(wl.conv_layer(32, 64, 64, 3, 1, 1, 56)) == (577, 64, 56, 56)
    assert kfac.kfac_layer_dims(wl.fc_layer(32, 2048, 1000)) == (2049, 1000, 1, 1)
    assert kfac.kfac_layer_dims(wl.conv_layer(2, 3, 64, 7, 2, 3, 224)) == (148, 64, 112, 112)
    assert kfac.kfac_layer_dims(wl.conv_layer(2, 3, 4, 3, 2, 0, 6, bias=0)) == (27, 4, 2, 2)
    for bad in [(0, 3, 4, 3, 1, 1, 5, 5, 1), (2, 0, 4, 3, 1, 1, 5, 5, 1), (2, 3, 4, 3, 0, 1, 5, 5, 1),
                (2, 3, 4, 7, 1, 0, 5, 5, 1), (2, 3, 4, 3, 1, -1, 5, 5, 1), (2, 3, 4, 3, 1, 1, 5, 5, 2)]:
        with pytest.raises(kfac.KfacError):
            kfac.kfac_layer_dims(bad)


def test_workspace_bytes():
    assert kfac.kfac_workspace_bytes([(0, 1, 1, 1, 1, 0, 1, 1, 1)]) == 0
    small = kfac.kfac_workspace_bytes(wl.config_layers(1))
    c2 = kfac.kfac_workspace_bytes(wl.config_layers(2))
    c4 = kfac.kfac_workspace_bytes(wl.config_layers(4))
    assert 0 < small < c2 < c4 < 16 * 2 ** 30
    # fp32: the zero-padded image of the 3x3 layer (32 x 64 planes of 58 x 58) must fit; the
    # patch matrix is not built.  bf16: patches (576 x 100352 bf16) must fit
    assert 32 * 64 * 58 * 58 * 4 <= c2 < 576 * 100352 * 4
    assert kfac.kfac_workspace_bytes(wl.config_layers(2), kfac.KFAC_BF16) >= 576 * 100352 * 2


def _fake_ctx(nbytes=1 << 20):
    """A context on a made-up (aligned, never dereferenced) workspace address: enough to
    exercise validation, which must fail before any GPU call."""
    h = ctypes.c_void_p()
    st = kfac.lib().kfac_create(ctypes.addressof(h), None, ctypes.c_void_p(0x100000), nbytes)
    assert st == kfac.KFAC_OK
    return h


def test_create_rejects_bad_arguments():
    h = ctypes.c_void_p()
    L = kfac.lib()
    assert L.kfac_create(None, None, ctypes.c_void_p(0x100000), 1024) == kfac.KFAC_ERR_INVALID
    assert L.kfac_create(ctypes.addressof(h), None, None, 1024) == kfac.KFAC_ERR_INVALID
    assert L.kfac_create(ctypes.addressof(h), None, ctypes.c_void_p(0x100001), 1024) == kfac.KFAC_ERR_INVALID
    assert L.kfac_create(ctypes.addressof(h), None, ctypes.c_void_p(0x100000), 0) == kfac.KFAC_ERR_INVALID
    L.kfac_destroy(None)


def test_calls_reject_bad_arguments_without_a_gpu():
    L = kfac.lib()
    h = _fake_ctx()
    lay = kfac.kfac_layer(*wl.fc_layer(4, 8, 3))
    lp = ctypes.addressof(lay)
    fake = (ctypes.c_void_p * 1)(0x200000)
    fp = ctypes.addressof(fake)
    null1 = (ctypes.c_void_p * 1)(None)
    np_ = ctypes.addressof(null1)
    INV = kfac.KFAC_ERR_INVALID
    # kfac_stats
    assert L.kfac_stats(None, 1, lp, 0, fp, fp, 0.0, 0, fp, fp) == INV
    assert L.kfac_stats(h, 0, lp, 0, fp, fp, 0.0, 0, fp, fp) == INV
    assert L.kfac_stats(h, 1, None, 0, fp, fp, 0.0, 0, fp, fp) == INV
    assert L.kfac_stats(h, 1, lp, 7, fp, fp, 0.0, 0, fp, fp) == INV
    assert L.kfac_stats(h, 1, lp, 0, fp, fp, 1.0, 0, fp, fp) == INV          # decay must be < 1
    assert L.kfac_stats(h, 1, lp, 0, fp, fp, -0.1, 0, fp, fp) == INV
    assert L.kfac_stats(h, 1, lp, 0, fp, fp, float("nan"), 0, fp, fp) == INV
    assert L.kfac_stats(h, 1, lp, 0, None, None, 0.0, 0, fp, fp) == INV       # nothing to do
    assert L.kfac_stats(h, 1, lp, 0, fp, fp, 0.0, 0, None, fp) == INV          # act given, A_ema missing
    assert L.kfac_stats(h, 1, lp, 0, fp, fp, 0.0, 0, fp, np_) == INV
    # the NHWC entry points validate like the NCHW ones
    assert L.kfac_stats_nhwc(None, 1, lp, 0, fp, fp, 0.0, 0, fp, fp) == INV
    assert L.kfac_stats_nhwc(h, 1, lp, 7, fp, fp, 0.0, 0, fp, fp) == INV
    assert L.kfac_stats_nhwc(h, 1, lp, 0, fp, fp, 1.0, 0, fp, fp) == INV
    assert L.kfac_stats_nhwc(h, 1, lp, 0, fp, fp, 0.0, 0, None, fp) == INV
    assert L.kfac_step_nhwc(None, 1, lp, 0, fp, fp, 0.0, 0, fp, fp, None, 1e-3, fp, fp, None, None, fp, fp) == INV
    assert L.kfac_step_nhwc(h, 1, lp, 0, fp, fp, 0.0, 0, fp, fp, None, -1.0, fp, fp, None, None, fp, fp) == INV
    assert L.kfac_step_nhwc(h, 1, lp, 0, fp, None, 0.0, 0, fp, fp, None, 1e-3, fp, fp, None, None, fp, fp) == INV
    one = (ctypes.c_int32 * 1)(4)
    op = ctypes.addressof(one)
    assert L.bn_unitwise_reduce_nhwc(None, 1, 2, op, op, fp, fp, fp, fp) == INV
    assert L.bn_unitwise_reduce_nhwc(h, 1, 0, op, op, fp, fp, fp, fp) == INV
    assert L.bn_unitwise_reduce_nhwc(h, 1, 2, op, op, fp, None, fp, fp) == INV
    # kfac_invert
    assert L.kfac_invert(h, 1, lp, fp, fp, -1.0, fp, fp, None, None) == INV
    assert L.kfac_invert(h, 1, lp, fp, fp, 1e-3, fp, fp, None, None) == INV   # in == out
    assert L.kfac_invert(h, 1, lp, None, fp, 1e-3, fp, fp, None, None) == INV
    assert L.kfac_invert(h, 1, lp, np_, fp, 1e-3, fp, fp, None, None) == INV
    # kfac_precondition
    assert L.kfac_precondition(h, 1, lp, fp, fp, None, fp) == INV
    assert L.kfac_precondition(h, 1, lp, fp, fp, fp, np_) == INV
    assert L.kfac_precondition(h, -1, lp, fp, fp, fp, fp) == INV
    # kfac_step: the union of the three checks
    ok = [h, 1, lp, 0, fp, fp, 0.0, 0, fp, fp, None, 1e-3, fp, fp, None, None, fp, fp]
    other = (ctypes.c_void_p * 1)(0x400000)
    op = ctypes.addressof(other)

    def step_with(**kw):
        a = list(ok)
        a[12], a[13] = op, op                      # inverses distinct from the factors
        names = ["ctx", "n", "L", "in", "act", "grad_out", "decay", "gsm", "A", "G", "mask", "gamma", "Ai", "Gi",
                 "pi", "info", "gW", "out"]
        for k, v in kw.items():
            a[names.index(k)] = v
        return L.kfac_step(*a)

    assert L.kfac_step(*ok) == INV                 # A_inv aliases A_ema
    assert step_with(ctx=None) == INV
    assert step_with(n=0) == INV
    assert step_with(decay=1.0) == INV
    assert step_with(gamma=-1.0) == INV
    assert step_with(gamma=float("inf")) == INV
    assert step_with(act=None) == INV
    assert step_with(grad_out=np_) == INV
    assert step_with(gW=None) == INV
    assert step_with(out=np_) == INV
    assert step_with(**{"in": 5}) == INV
    # kfac_im2col
    assert L.kfac_im2col(h, lp, 0, None, fake[0], 4) == INV
    assert L.kfac_im2col(h, lp, 0, fake[0], fake[0], 3) == INV                 # ld < N*h*w
    # BatchNorm
    C = (ctypes.c_int32 * 1)(8)
    cp = ctypes.addressof(C)
    assert L.bn_unitwise_precondition(h, 1, 0, cp, fp, fp, 0.0, 1e-6, fp, fp, fp) == INV
    assert L.bn_unitwise_precondition(h, 1, 4, None, fp, fp, 0.0, 1e-6, fp, fp, fp) == INV
    assert L.bn_unitwise_precondition(h, 1, 4, cp, fp, fp, 1.5, 1e-6, fp, fp, fp) == INV
    assert L.bn_unitwise_precondition(h, 1, 4, cp, fp, fp, 0.0, -1.0, fp, fp, fp) == INV
    assert L.bn_unitwise_precondition(h, 1, 4, cp, fp, np_, 0.0, 1e-6, fp, fp, fp) == INV
    Z = (ctypes.c_int32 * 1)(0)
    assert L.bn_unitwise_reduce_nchw(h, 1, 4, cp, ctypes.addressof(Z), fp, fp, fp, fp) == INV
    assert L.bn_unitwise_reduce_nchw(h, 1, 4, cp, None, fp, fp, fp, fp) == INV
    L.kfac_destroy(h)


def test_workspace_too_small_is_reported_before_launch():
    """The 3x3 layer of configuration 2 needs tens of MB of scratch; a 1 MB workspace is refused."""
    L = kfac.lib()
    h = _fake_ctx(1 << 20)
    lay = kfac.kfac_layer(*wl.config_layers(2)[0])
    fake = (ctypes.c_void_p * 1)(0x200000)
    fp = ctypes.addressof(fake)
    st = L.kfac_stats(h, 1, ctypes.addressof(lay), 0, fp, fp, 0.0, 0, fp, fp)
    assert st == kfac.KFAC_ERR_WORKSPACE
    L.kfac_destroy(h)


def test_resnet50_layer_set_matches_planned_histogram():
    layers, bns = wl.resnet50_layers(32)
    dims = sorted([L.dA for L in layers] + [L.dG for L in layers])
    from collections import Counter
    hist = Counter(dims)
    assert hist == Counter({64: 7, 65: 5, 128: 8, 129: 4, 148: 1, 256: 16, 257: 10, 512: 11, 513: 8, 577: 3,
                            1000: 1, 1024: 7, 1025: 7, 1153: 4, 2048: 4, 2049: 3, 2305: 6, 4609: 3})
    assert sum(C for C, _ in bns) == 26560
    tot = sum(sum(wl.flops(L).values()) for L in layers)
    assert abs(tot / 1e12 - 1.396) < 0.01


# ------------------------------------------------------------------ stale statistics: host logic (Sec. 4.3)
def test_next_interval_matches_oracle_exhaustively():
    from oracle import stale
    for s1 in (False, True):
        for s2 in (False, True):
            for d1 in range(1, 40):
                for d2 in range(1, 40):
                    assert kfac.kfac_next_interval(s1, s2, d1, d2) == stale.next_interval(s1, s2, d1, d2)
    assert kfac.kfac_next_interval(True, True, 0, 1) == 0 and kfac.kfac_next_interval(True, True, 1, -3) == 0
    assert kfac.kfac_next_interval(True, True, 2 ** 31 - 1, 2 ** 31 - 1) == 2 ** 31 - 1      # saturates


def test_refresh_state_follows_algorithm_1():
    """Ratio streams (to the last value, to the one before) drive the library's state and the oracle's side by side."""
    import math
    import numpy as np
    from oracle import stale
    rng = np.random.default_rng(11)
    alpha = 0.1
    for trial in range(20):
        st = kfac.kfac_refresh_init(1)
        ref = stale.RefreshState()
        assert (st[0].t_next, st[0].delta, st[0].delta_m1) == (1, 1, 1)
        for t in range(1, 300):
            assert kfac.kfac_refresh_due(st[0], t) == ref.due(t)
            if ref.due(t):
                r1, r2 = rng.choice([0.0, 0.05, 0.0999, 0.1, 0.3, math.inf, math.nan], 2)
                kfac.kfac_refresh_advance(st[0], r1, r2, alpha)
                ref.refreshed(r1 < alpha, r2 < alpha)
                assert (st[0].t_next, st[0].delta, st[0].delta_m1) == (ref.t_next, ref.delta, ref.delta_m1)
    # always similar: Fibonacci refresh steps
    st = kfac.kfac_refresh_init(1)
    steps = []
    for t in range(1, 60):
        if kfac.kfac_refresh_due(st[0], t):
            steps.append(t)
            k = len(steps)
            kfac.kfac_refresh_advance(st[0], 0.0 if k >= 2 else math.inf, 0.0 if k >= 3 else math.inf, alpha)
    assert steps == [1, 2, 3, 5, 8, 13, 21, 34, 55]


def test_staleness_rejects_bad_arguments_without_a_gpu():
    L = kfac.lib()
    h = _fake_ctx()
    fake = (ctypes.c_void_p * 1)(0x200000)
    other = (ctypes.c_void_p * 1)(0x400000)
    null1 = (ctypes.c_void_p * 1)(None)
    fp, op, np_ = ctypes.addressof(fake), ctypes.addressof(other), ctypes.addressof(null1)
    d = (ctypes.c_int32 * 1)(8)
    dp = ctypes.addressof(d)
    out = ctypes.c_void_p(0x600000)
    INV = kfac.KFAC_ERR_INVALID
    assert L.kfac_staleness(None, 1, dp, fp, op, None, out) == INV
    assert L.kfac_staleness(h, 0, dp, fp, op, None, out) == INV
    assert L.kfac_staleness(h, 1, None, fp, op, None, out) == INV
    assert L.kfac_staleness(h, 1, dp, None, op, None, out) == INV
    assert L.kfac_staleness(h, 1, dp, np_, op, None, out) == INV
    assert L.kfac_staleness(h, 1, dp, fp, op, None, None) == INV
    assert L.kfac_staleness(h, 1, dp, fp, fp, None, out) == INV          # X is its own predecessor
    assert L.kfac_staleness(h, 1, dp, fp, op, fp, out) == INV
    z = (ctypes.c_int32 * 1)(0)
    assert L.kfac_staleness(h, 1, ctypes.addressof(z), fp, op, None, out) == INV
    big = (ctypes.c_int32 * 1)(1 << 20)                                    # 2^40 elements: workspace of 1 MB is too small
    assert L.kfac_staleness(h, 1, ctypes.addressof(big), fp, op, None, out) == kfac.KFAC_ERR_WORKSPACE
    L.kfac_destroy(h)


# ------------------------------------------------------------------ symmetric packing (Sec. 5.2): arguments
def test_pack_rejects_bad_arguments_without_a_gpu():
    L = kfac.lib()
    h = _fake_ctx()
    d = (ctypes.c_int32 * 2)(8, 5)
    dp = ctypes.addressof(d)
    assert kfac.kfac_packed_elems([8, 5]) == 36 + 15 and kfac.kfac_packed_elems([4609]) == 4609 * 4610 // 2
    assert L.kfac_packed_elems(0, dp) == 0 and L.kfac_packed_elems(2, None) == 0
    z = (ctypes.c_int32 * 1)(0)
    assert L.kfac_packed_elems(1, ctypes.addressof(z)) == 0
    mats = (ctypes.c_void_p * 2)(0x200000, 0x300000)
    mp = ctypes.addressof(mats)
    buf = ctypes.c_void_p(0x800000)
    INV = kfac.KFAC_ERR_INVALID
    assert L.kfac_pack_upper(None, 2, dp, mp, 0, buf) == INV
    assert L.kfac_pack_upper(h, 0, dp, mp, 0, buf) == INV
    assert L.kfac_pack_upper(h, 2, None, mp, 0, buf) == INV
    assert L.kfac_pack_upper(h, 2, dp, None, 0, buf) == INV
    assert L.kfac_pack_upper(h, 2, dp, mp, 0, None) == INV
    assert L.kfac_pack_upper(h, 2, dp, mp, 5, buf) == INV                      # unknown type
    hole = (ctypes.c_void_p * 2)(0x200000, None)
    assert L.kfac_pack_upper(h, 2, dp, ctypes.addressof(hole), 0, buf) == INV
    assert L.kfac_pack_upper(h, 2, dp, mp, 0, ctypes.c_void_p(0x200010)) == INV  # packed buffer inside a matrix
    assert L.kfac_unpack_upper(h, 2, dp, 0, ctypes.c_void_p(0x300000), mp) == INV
    assert L.kfac_unpack_upper(h, 2, dp, 1, None, mp) == INV
    L.kfac_destroy(h)


# ------------------------------------------------------------------ parameter update (Sec. 6.2, 6.3): host logic, arguments
def test_schedules_match_oracle():
    import math
    import numpy as np
    from oracle import update
    rng = np.random.default_rng(5)
    for _ in range(200):
        eta0, p = float(rng.uniform(1e-4, 1.0)), float(rng.uniform(0.5, 12.0))
        e0 = float(rng.uniform(0, 5))
        e1 = e0 + float(rng.uniform(0.5, 90))
        for e in (0.0, e0, e0 + 1e-9, 0.5 * (e0 + e1), e1 - 1e-9, e1, e1 + 3, float(rng.uniform(0, 100))):
            ref = update.lr_polynomial(eta0, e, e0, e1, p)
            assert math.isclose(kfac.kfac_lr_polynomial(eta0, e, e0, e1, p), ref, rel_tol=1e-13, abs_tol=1e-300)
            m0 = float(rng.uniform(0.0, 1.0))
            assert math.isclose(kfac.kfac_momentum_coupled(m0, eta0, ref), update.momentum_coupled(m0, eta0, ref),
                                rel_tol=1e-15, abs_tol=0.0)
    assert math.isnan(kfac.kfac_lr_polynomial(0.1, 1.0, 5.0, 5.0, 2.0))
    assert math.isnan(kfac.kfac_lr_polynomial(0.1, 1.0, 5.0, 4.0, 2.0))
    assert math.isnan(kfac.kfac_momentum_coupled(0.9, 0.0, 0.1))


def test_update_rejects_bad_arguments_without_a_gpu():
    L = kfac.lib()
    INV = kfac.KFAC_ERR_INVALID
    h = _fake_ctx(1 << 20)
    lays = (kfac.kfac_layer * 2)(kfac.kfac_layer(*wl.fc_layer(2, 64, 32)), kfac.kfac_layer(*wl.fc_layer(2, 16, 8)))
    lp = ctypes.addressof(lays)
    u = (ctypes.c_void_p * 2)(0x200000, 0x300000)
    w = (ctypes.c_void_p * 2)(0x400000, 0x500000)
    wp = (ctypes.c_void_p * 2)(0x600000, 0x700000)
    up, wpt, wpp = ctypes.addressof(u), ctypes.addressof(w), ctypes.addressof(wp)
    call = L.kfac_update_weights
    assert call(None, 2, lp, up, 0.1, 0.9, 1, 1e-9, wpt, wpp) == INV
    assert call(h, 0, lp, up, 0.1, 0.9, 1, 1e-9, wpt, wpp) == INV
    assert call(h, 2, None, up, 0.1, 0.9, 1, 1e-9, wpt, wpp) == INV
    assert call(h, 2, lp, None, 0.1, 0.9, 1, 1e-9, wpt, wpp) == INV
    assert call(h, 2, lp, up, 0.1, 0.9, 1, 1e-9, None, wpp) == INV
    assert call(h, 2, lp, up, 0.1, 0.9, 1, 1e-9, wpt, None) == INV
    assert call(h, 2, lp, up, float("nan"), 0.9, 1, 1e-9, wpt, wpp) == INV
    assert call(h, 2, lp, up, 0.1, float("inf"), 1, 1e-9, wpt, wpp) == INV
    assert call(h, 2, lp, up, 0.1, 0.9, 1, -1.0, wpt, wpp) == INV
    hole = (ctypes.c_void_p * 2)(0x400000, None)
    assert call(h, 2, lp, up, 0.1, 0.9, 1, 1e-9, ctypes.addressof(hole), wpp) == INV
    same = (ctypes.c_void_p * 2)(0x400000 + 64, 0x500000)                          # W_prev inside W
    assert call(h, 2, lp, up, 0.1, 0.9, 1, 1e-9, wpt, ctypes.addressof(same)) == INV
    assert call(h, 2, lp, wpt, 0.1, 0.9, 0, 1e-9, wpt, wpp) == INV                 # U aliases W
    bad = (kfac.kfac_layer * 1)(kfac.kfac_layer(*wl.fc_layer(2, 64, 32)))
    bad[0].c_out = 0
    assert call(h, 1, ctypes.addressof(bad), up, 0.1, 0.9, 1, 1e-9, wpt, wpp) == INV
    L.kfac_destroy(h)


# ------------------------------------------------------------------ whole-layer BatchNorm Fisher (Sec. 4.2): arguments
def test_bn_full_rejects_bad_arguments_without_a_gpu():
    L = kfac.lib()
    INV = kfac.KFAC_ERR_INVALID
    assert kfac.bn_full_workspace_bytes(32, [64, 256]) > 0
    assert kfac.bn_full_workspace_bytes(32, [64, 0]) == 0 and kfac.bn_full_workspace_bytes(0, [64]) == 0
    assert kfac.bn_full_workspace_bytes(32, [40000]) == 0
    assert L.bn_full_workspace_bytes(1, 32, None) == 0
    # the size serves every layer inverted and any one alone, and grows with the layers
    assert kfac.bn_full_workspace_bytes(32, [512, 1024]) >= kfac.bn_full_workspace_bytes(32, [1024])
    h = _fake_ctx(1 << 20)
    C = (ctypes.c_int32 * 2)(8, 4)
    cp = ctypes.addressof(C)
    arrs = [(ctypes.c_void_p * 2)(0x200000 + 0x10000 * k, 0x208000 + 0x10000 * k) for k in range(6)]
    gg, gb, F, Fi, og, ob = [ctypes.addressof(a) for a in arrs]
    call = L.bn_full_precondition
    assert call(None, 2, 32, cp, gg, gb, 0.0, 1e-6, F, None, Fi, None, og, ob) == INV
    assert call(h, 0, 32, cp, gg, gb, 0.0, 1e-6, F, None, Fi, None, og, ob) == INV
    assert call(h, 2, 0, cp, gg, gb, 0.0, 1e-6, F, None, Fi, None, og, ob) == INV
    assert call(h, 2, 32, None, gg, gb, 0.0, 1e-6, F, None, Fi, None, og, ob) == INV
    for k in range(6):
        a = [gg, gb, F, Fi, og, ob]
        a[k] = None
        assert call(h, 2, 32, cp, a[0], a[1], 0.0, 1e-6, a[2], None, a[3], None, a[4], a[5]) == INV
    assert call(h, 2, 32, cp, gg, gb, 1.0, 1e-6, F, None, Fi, None, og, ob) == INV         # decay must stay below 1
    assert call(h, 2, 32, cp, gg, gb, 0.0, -1.0, F, None, Fi, None, og, ob) == INV
    assert call(h, 2, 32, cp, gg, gb, 0.0, 1e-6, F, None, F, None, og, ob) == INV          # inverse in place
    hole = (ctypes.c_void_p * 2)(0x900000, None)
    assert call(h, 2, 32, cp, gg, gb, 0.0, 1e-6, ctypes.addressof(hole), None, Fi, None, og, ob) == INV
    bad = (ctypes.c_int32 * 2)(8, -1)
    assert call(h, 2, 32, ctypes.addressof(bad), gg, gb, 0.0, 1e-6, F, None, Fi, None, og, ob) == INV
    L.kfac_destroy(h)
    # a layer that needs more scratch than the context has is refused before any launch
    h = _fake_ctx(1 << 16)
    big = (ctypes.c_int32 * 1)(1024)
    assert call(h, 1, 32, ctypes.addressof(big), gg, gb, 0.0, 1e-6, F, None, Fi, None, og, ob) == kfac.KFAC_ERR_WORKSPACE
    L.kfac_destroy(h)


# ------------------------------------------------------------------ NHWC -> NCHW conversion (Sec. 5.2): arguments
def test_layout_conversion_rejects_bad_arguments_without_a_gpu():
    L = kfac.lib()
    INV = kfac.KFAC_ERR_INVALID
    h = _fake_ctx(1 << 20)
    lays = (kfac.kfac_layer * 2)(kfac.kfac_layer(*wl.conv_layer(2, 8, 4, 3, 1, 1, 6)), kfac.kfac_layer(*wl.fc_layer(2, 16, 8)))
    lp = ctypes.addressof(lays)
    src = (ctypes.c_void_p * 2)(0x200000, 0x300000)
    dst = (ctypes.c_void_p * 2)(0x400000, 0x500000)
    sp, dp = ctypes.addressof(src), ctypes.addressof(dst)
    call = L.kfac_nhwc_to_nchw
    assert call(None, 2, lp, 0, 0, sp, dp) == INV
    assert call(h, 0, lp, 0, 0, sp, dp) == INV
    assert call(h, 2, None, 0, 0, sp, dp) == INV
    assert call(h, 2, lp, 2, 0, sp, dp) == INV                                   # which is 0 or 1
    assert call(h, 2, lp, 0, 7, sp, dp) == INV                                   # unknown element type
    assert call(h, 2, lp, 0, 0, None, dp) == INV
    assert call(h, 2, lp, 0, 0, sp, None) == INV
    hole = (ctypes.c_void_p * 2)(0x400000, None)
    assert call(h, 2, lp, 0, 0, sp, ctypes.addressof(hole)) == INV               # source without destination
    over = (ctypes.c_void_p * 2)(0x200000 + 256, 0x500000)
    assert call(h, 2, lp, 0, 0, sp, ctypes.addressof(over)) == INV               # in place / overlapping
    none = (ctypes.c_void_p * 2)(None, None)
    assert call(h, 2, lp, 0, 0, ctypes.addressof(none), dp) == kfac.KFAC_OK      # nothing to do
    L.kfac_destroy(h)


def test_workspace_covers_masked_steps():
    """Host-only dry plans: whatever subset of the full ResNet-50 set a fused step inverts, its plan stays
    within kfac_workspace_bytes (the stale-statistics mode changes the mask from step to step)."""
    import numpy as np
    for config in (4, 5):
        layers = wl.config_layers(config)
        bound = kfac.kfac_workspace_bytes(layers)
        assert 0 < kfac.kfac_step_workspace_bytes(layers) <= bound
        rng = np.random.default_rng(config)
        big = [max(L.dA, L.dG) for L in layers]
        masks = [[b >= t for b in big] for t in (512, 1024, 2048, 4096)] + [[b < t for b in big] for t in (512, 2048)]
        masks += [list(rng.random(len(layers)) < rng.random()) for _ in range(120)]
        worst = max(kfac.kfac_step_workspace_bytes(layers, kfac.KFAC_F32, m) for m in masks)
        assert worst <= bound, (config, worst, bound)
    opts = kfac.options(streams=1, pipeline_phases=0)
    layers = wl.config_layers(4)
    assert 0 < kfac.kfac_step_workspace_bytes(layers, kfac.KFAC_F32, None, opts) <= kfac.kfac_workspace_bytes(layers, kfac.KFAC_F32, opts)


def test_options_are_validated():
    L = kfac.lib()
    h = ctypes.c_void_p()
    o = kfac.options()
    assert o.struct_size == ctypes.sizeof(kfac.kfac_options) and o.streams == 4 and o.fp32_products == kfac.KFAC_PRODUCTS_SPLIT_BF16
    ws = ctypes.c_void_p(0x100000)
    assert L.kfac_create_opt(ctypes.addressof(h), None, ws, 1 << 20, ctypes.addressof(o)) == kfac.KFAC_OK
    L.kfac_destroy(h)
    for field, bad in (("struct_size", 4), ("fp32_products", 7), ("streams", 0), ("streams", 5), ("staging_slots", 1),
                       ("recursion_leaf", 300), ("force_tile", 96), ("chunk_gflop", float("nan"))):
        b = kfac.options(**{field: bad})
        assert L.kfac_create_opt(ctypes.addressof(h), None, ws, 1 << 20, ctypes.addressof(b)) == kfac.KFAC_ERR_INVALID, field
        lay = kfac.kfac_layer(*wl.fc_layer(4, 8, 3))
        assert L.kfac_workspace_bytes_opt(ctypes.addressof(lay), 1, 0, ctypes.addressof(b)) == 0, field
