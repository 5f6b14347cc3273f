"""Float64 CPU oracle for the K-FAC hot path -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Thin ctypes wrapper around ``kfac_oracle.c`` (plain C loops, float64, OpenMP).
Only the tests, ``__graft_entry__.smoke()`` and the benchmark's ``cpu_baseline``
leg may import this package.  It imports nothing from the GPU package and the
GPU package imports nothing from here.

All functions take numpy arrays (any float dtype; promoted to float64) and return
new float64 arrays.  A layer is described by the tuple of ints
``(N, c_in, c_out, k, stride, pad, h_in, w_in, bias)``; a fully-connected layer is
``k=1, stride=1, pad=0, h_in=w_in=1``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kfac_oracle.c")
_LIB = os.path.join(_HERE, "libkfac_oracle.so")

OK, INVALID, NOT_PD = 0, 1, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_out_size.restype = ctypes.c_int
    return _lib


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, allow_not_pd: bool = False) -> int:
    if rc == OK or (allow_not_pd and rc == NOT_PD):
        return rc
    raise ValueError("oracle call failed with status %d" % rc)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def out_size(n_in: int, k: int, stride: int, pad: int) -> int:
    return int(_load().oracle_out_size(int(n_in), int(k), int(stride), int(pad)))


def layer_dims(layer: Sequence[int]) -> Tuple[int, int, int, int]:
    """(dA, dG, h, w) of a layer tuple."""
    N, c_in, c_out, k, s, p, h_in, w_in, bias = [int(v) for v in layer]
    return c_in * k * k + (1 if bias else 0), c_out, out_size(h_in, k, s, p), out_size(w_in, k, s, p)


def im2col(layer: Sequence[int], act) -> np.ndarray:
    N, c_in, c_out, k, s, p, h_in, w_in, bias = [int(v) for v in layer]
    dA, _, h, w = layer_dims(layer)
    a = _f64(act)
    assert a.size == N * c_in * h_in * w_in
    P = np.empty((N, dA, h * w), dtype=np.float64)
    _check(_load().oracle_im2col(N, c_in, k, s, p, h_in, w_in, bias, _p(a), _p(P)))
    return P


def factor_A(layer: Sequence[int], act) -> np.ndarray:
    N, c_in, c_out, k, s, p, h_in, w_in, bias = [int(v) for v in layer]
    dA = layer_dims(layer)[0]
    a = _f64(act)
    assert a.size == N * c_in * h_in * w_in
    A = np.empty((dA, dA), dtype=np.float64)
    _check(_load().oracle_factor_A(N, c_in, k, s, p, h_in, w_in, bias, _p(a), _p(A)))
    return A


def factor_G(layer: Sequence[int], grad_out, spatial_mean: bool = False) -> np.ndarray:
    N, c_in, c_out, k, s, p, h_in, w_in, bias = [int(v) for v in layer]
    _, dG, h, w = layer_dims(layer)
    g = _f64(grad_out)
    assert g.size == N * c_out * h * w
    G = np.empty((dG, dG), dtype=np.float64)
    _check(_load().oracle_factor_G(N, c_out, h * w, int(bool(spatial_mean)), _p(g), _p(G)))
    return G


def factor_A_entries(layer: Sequence[int], act, I, J) -> np.ndarray:
    N, c_in, c_out, k, s, p, h_in, w_in, bias = [int(v) for v in layer]
    a = _f64(act)
    assert a.size == N * c_in * h_in * w_in
    I = np.ascontiguousarray(I, dtype=np.int32)
    J = np.ascontiguousarray(J, dtype=np.int32)
    out = np.empty(I.size, dtype=np.float64)
    _check(_load().oracle_factor_A_entries(N, c_in, k, s, p, h_in, w_in, bias, _p(a),
                                           int(I.size), _p(I), _p(J), _p(out)))
    return out


def factor_G_entries(layer: Sequence[int], grad_out, I, J, spatial_mean: bool = False) -> np.ndarray:
    N, c_in, c_out, k, s, p, h_in, w_in, bias = [int(v) for v in layer]
    _, dG, h, w = layer_dims(layer)
    g = _f64(grad_out)
    assert g.size == N * c_out * h * w
    I = np.ascontiguousarray(I, dtype=np.int32)
    J = np.ascontiguousarray(J, dtype=np.int32)
    out = np.empty(I.size, dtype=np.float64)
    _check(_load().oracle_factor_G_entries(N, c_out, h * w, int(bool(spatial_mean)), _p(g),
                                           int(I.size), _p(I), _p(J), _p(out)))
    return out


def kfac_stats(layer: Sequence[int], act, grad_out, decay: float, g_spatial_mean: bool,
               A_ema: Optional[np.ndarray], G_ema: Optional[np.ndarray]):
    """Returns the updated (A_ema, G_ema); inputs are not modified. Either side may be None."""
    N, c_in, c_out, k, s, p, h_in, w_in, bias = [int(v) for v in layer]
    dA, dG, h, w = layer_dims(layer)
    a = None if act is None else _f64(act)
    g = None if grad_out is None else _f64(grad_out)
    A = None if a is None else (np.zeros((dA, dA)) if A_ema is None else _f64(A_ema).copy().reshape(dA, dA))
    G = None if g is None else (np.zeros((dG, dG)) if G_ema is None else _f64(G_ema).copy().reshape(dG, dG))
    if a is not None:
        assert a.size == N * c_in * h_in * w_in
    if g is not None:
        assert g.size == N * c_out * h * w
    _check(_load().oracle_kfac_stats(N, c_in, c_out, k, s, p, h_in, w_in, bias, _p(a), _p(g),
                                     ctypes.c_double(decay), int(bool(g_spatial_mean)), _p(A), _p(G)))
    return A, G


def pi_damping(A_ema, G_ema, gamma: float) -> Tuple[float, float, float]:
    A, G = _f64(A_ema), _f64(G_ema)
    pi, da, dg = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _check(_load().oracle_pi_damping(A.shape[0], _p(A), G.shape[0], _p(G), ctypes.c_double(gamma),
                                     ctypes.byref(pi), ctypes.byref(da), ctypes.byref(dg)))
    return pi.value, da.value, dg.value


def spd_inverse(X, damp: float) -> Tuple[np.ndarray, int]:
    """((X + damp I)^-1, info); info = 0, or j+1 when pivot j is not positive."""
    Xd = _f64(X)
    n = Xd.shape[0]
    assert Xd.shape == (n, n)
    out = np.full((n, n), np.nan)
    info = ctypes.c_int32(0)
    _check(_load().oracle_spd_inverse(n, _p(Xd), ctypes.c_double(damp), _p(out), ctypes.byref(info)),
           allow_not_pd=True)
    return out, int(info.value)


def kfac_invert(A_ema, G_ema, gamma: float):
    """Returns (A_inv, G_inv, pi, info[2])."""
    A, G = _f64(A_ema), _f64(G_ema)
    dA, dG = A.shape[0], G.shape[0]
    Ai, Gi = np.full((dA, dA), np.nan), np.full((dG, dG), np.nan)
    pi = ctypes.c_double()
    info = np.zeros(2, dtype=np.int32)
    _check(_load().oracle_kfac_invert(dA, dG, _p(A), _p(G), ctypes.c_double(gamma), _p(Ai), _p(Gi),
                                      ctypes.byref(pi), _p(info)), allow_not_pd=True)
    return Ai, Gi, pi.value, info


def kfac_precondition(G_inv, A_inv, grad_W) -> np.ndarray:
    Gi, Ai, W = _f64(G_inv), _f64(A_inv), _f64(grad_W)
    dG, dA = Gi.shape[0], Ai.shape[0]
    assert W.shape == (dG, dA)
    U = np.empty((dG, dA))
    _check(_load().oracle_kfac_precondition(dG, dA, _p(Gi), _p(Ai), _p(W), _p(U)))
    return U


def bn_reduce_nchw(dy, xhat):
    d, x = _f64(dy), _f64(xhat)
    N, C = d.shape[0], d.shape[1]
    HW = int(np.prod(d.shape[2:])) if d.ndim > 2 else 1
    gg, gb = np.empty((N, C)), np.empty((N, C))
    _check(_load().oracle_bn_reduce_nchw(N, C, HW, _p(d), _p(x), _p(gg), _p(gb)))
    return gg, gb


def bn_unitwise_precondition(g_gamma, g_beta, decay: float, lam: float, F_ema=None):
    """Returns (F_ema_new [C,3], out_gamma [C], out_beta [C])."""
    gg, gb = _f64(g_gamma), _f64(g_beta)
    N, C = gg.shape
    F = np.zeros((C, 3)) if F_ema is None else _f64(F_ema).copy().reshape(C, 3)
    og, ob = np.empty(C), np.empty(C)
    _check(_load().oracle_bn_unitwise_precondition(N, C, _p(gg), _p(gb), ctypes.c_double(decay),
                                                   ctypes.c_double(lam), _p(F), _p(og), _p(ob)))
    return F, og, ob
