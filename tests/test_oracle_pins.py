"""Pins for the float64 CPU oracle (CPU only).

Each test ties one oracle function to something outside the oracle: a library
routine it must reduce to (torch conv2d / unfold, numpy eigh / solve / kron),
a closed form, an algebraic invariant, or brute force on tiny inputs.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2002_06015_amd import workloads as wl

RNG = np.random.default_rng(20260615)

SMALL_CONVS = [
    # N, c_in, c_out, k, s, p, h_in, w_in, bias
    (2, 3, 4, 3, 1, 1, 5, 5, 1),
    (3, 2, 3, 3, 2, 1, 6, 5, 1),
    (2, 4, 2, 1, 1, 0, 4, 3, 0),
    (1, 2, 5, 1, 2, 0, 5, 5, 1),
    (2, 1, 2, 7, 2, 3, 9, 11, 1),
    (2, 3, 2, 3, 1, 0, 4, 4, 0),
]


def _rand_act(layer):
    N, c_in, _, _, _, _, h_in, w_in, _ = layer
    return np.maximum(RNG.standard_normal((N, c_in, h_in, w_in)), 0.0)


def _rand_grad(layer):
    N, _, c_out = layer[:3]
    _, _, h, w = oracle.layer_dims(layer)
    return RNG.standard_normal((N, c_out, h, w)) * 1e-3


# ---------------------------------------------------------------- patches (Eq. 10)

@pytest.mark.parametrize("layer", SMALL_CONVS)
def test_im2col_matches_library_unfold(layer):
    """torch's unfold is an independent im2col with (c, ky, kx) row order and zero padding."""
    N, c_in, c_out, k, s, p, h_in, w_in, bias = layer
    act = _rand_act(layer)
    P = oracle.im2col(layer, act)
    ref = torch.nn.functional.unfold(torch.from_numpy(act), kernel_size=k, padding=p, stride=s).numpy()
    d0 = c_in * k * k
    assert P.shape[1] == d0 + bias
    np.testing.assert_array_equal(P[:, :d0, :], ref)
    if bias:
        np.testing.assert_array_equal(P[:, d0, :], 1.0)


@pytest.mark.parametrize("layer", SMALL_CONVS)
def test_im2col_reproduces_convolution(layer):
    """Eq. 10: W * im2col(A) reshaped is the layer output, i.e. a library conv2d."""
    N, c_in, c_out, k, s, p, h_in, w_in, bias = layer
    act = _rand_act(layer)
    W = RNG.standard_normal((c_out, c_in, k, k))
    b = RNG.standard_normal(c_out) if bias else None
    P = oracle.im2col(layer, act)
    Wm = W.reshape(c_out, -1)
    if bias:
        Wm = np.concatenate([Wm, b[:, None]], axis=1)      # bias weight multiplies the ones row (last)
    out = np.einsum("od,ndt->not", Wm, P)
    ref = torch.nn.functional.conv2d(torch.from_numpy(act), torch.from_numpy(W),
                                     None if b is None else torch.from_numpy(b), stride=s, padding=p)
    np.testing.assert_allclose(out.reshape(ref.shape), ref.numpy(), rtol=1e-12, atol=1e-12)


def test_out_size_matches_library():
    for (n_in, k, s, p) in [(224, 7, 2, 3), (56, 3, 1, 1), (56, 1, 2, 0), (7, 3, 1, 1), (5, 3, 2, 0), (6, 3, 2, 1)]:
        ref = torch.nn.functional.conv2d(torch.zeros(1, 1, n_in, n_in), torch.zeros(1, 1, k, k),
                                         stride=s, padding=p).shape[-1]
        assert oracle.out_size(n_in, k, s, p) == ref


# ---------------------------------------------------------------- factors (Eq. 9, 11)

@pytest.mark.parametrize("layer", SMALL_CONVS)
def test_factor_A_brute_force_outer_products(layer):
    """A = 1/(N hw) sum over samples and positions of (patch vector)(patch vector)^T,
    with patch vectors cut out of a zero-padded copy by slicing."""
    N, c_in, c_out, k, s, p, h_in, w_in, bias = layer
    dA, _, h, w = oracle.layer_dims(layer)
    act = _rand_act(layer)
    padded = np.pad(act, ((0, 0), (0, 0), (p, p), (p, p)))
    acc = np.zeros((dA, dA))
    for n in range(N):
        for y in range(h):
            for x in range(w):
                v = padded[n, :, y * s:y * s + k, x * s:x * s + k].reshape(-1)
                if bias:
                    v = np.append(v, 1.0)
                acc += np.outer(v, v)
    acc /= N * h * w
    A = oracle.factor_A(layer, act)
    np.testing.assert_allclose(A, acc, rtol=1e-12, atol=1e-14)
    # spot entries, computed one at a time without forming patches
    I, J = np.meshgrid(np.arange(dA), np.arange(dA), indexing="ij")
    ent = oracle.factor_A_entries(layer, act, I.ravel(), J.ravel()).reshape(dA, dA)
    np.testing.assert_allclose(ent, acc, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("layer", SMALL_CONVS)
def test_factor_G_brute_force_outer_products(layer):
    N, c_in, c_out = layer[:3]
    _, dG, h, w = oracle.layer_dims(layer)
    g = _rand_grad(layer)
    acc = np.zeros((dG, dG))
    for n in range(N):
        for y in range(h):
            for x in range(w):
                acc += np.outer(g[n, :, y, x], g[n, :, y, x])
    acc /= N
    np.testing.assert_allclose(oracle.factor_G(layer, g, False), acc, rtol=1e-12, atol=1e-20)
    np.testing.assert_allclose(oracle.factor_G(layer, g, True), acc / (h * w), rtol=1e-12, atol=1e-20)
    I, J = np.meshgrid(np.arange(dG), np.arange(dG), indexing="ij")
    ent = oracle.factor_G_entries(layer, g, I.ravel(), J.ravel(), True).reshape(dG, dG)
    np.testing.assert_allclose(ent, acc / (h * w), rtol=1e-12, atol=1e-20)


def test_factor_invariants():
    layer = (4, 3, 5, 3, 1, 1, 6, 6, 1)
    dA, dG, h, w = oracle.layer_dims(layer)
    act, g = _rand_act(layer), _rand_grad(layer)
    A, G = oracle.factor_A(layer, act), oracle.factor_G(layer, g)
    P = oracle.im2col(layer, act)
    assert np.array_equal(A, A.T) and np.array_equal(G, G.T)
    assert np.linalg.eigvalsh(A).min() >= -1e-12 * np.trace(A)
    assert np.linalg.eigvalsh(G).min() >= -1e-12 * np.trace(G)
    assert A[-1, -1] == pytest.approx(1.0, abs=1e-15)                     # ones row squared
    np.testing.assert_allclose(A[:-1, -1], P[:, :-1, :].mean(axis=(0, 2)), rtol=1e-12)   # mean patch
    assert np.trace(A) == pytest.approx((P ** 2).sum(axis=1).mean(), rel=1e-12)


def test_pointwise_conv_is_a_gram_matrix():
    """k=1, s=1, p=0: A is X^T X / M of the [N*hw, c] matrix of pixels (textbook Gram matrix)."""
    layer = (3, 6, 4, 1, 1, 0, 5, 4, 0)
    act = _rand_act(layer)
    X = act.transpose(0, 2, 3, 1).reshape(-1, 6)
    np.testing.assert_allclose(oracle.factor_A(layer, act), X.T @ X / X.shape[0], rtol=1e-12)
    g = _rand_grad(layer)
    Y = g.transpose(0, 2, 3, 1).reshape(-1, 4)
    np.testing.assert_allclose(oracle.factor_G(layer, g), Y.T @ Y / 3, rtol=1e-12)


def test_fc_is_conv_with_unit_spatial_size():
    fc = tuple(wl.fc_layer(8, 10, 6))
    a = np.maximum(RNG.standard_normal((8, 10)), 0)
    g = RNG.standard_normal((8, 6))
    ab = np.concatenate([a, np.ones((8, 1))], axis=1)
    np.testing.assert_allclose(oracle.factor_A(fc, a), ab.T @ ab / 8, rtol=1e-12)
    np.testing.assert_allclose(oracle.factor_G(fc, g), g.T @ g / 8, rtol=1e-12)


def test_factor_statistics_of_the_generator():
    """For a = ReLU(N(0,1)): E a^2 = 1/2, E a a' = 1/(2 pi), E a = 1/sqrt(2 pi); G -> sigma^2 hw I."""
    layer = wl.conv_layer(8, 4, 4, 3, 1, 1, 24)
    act, g = wl.make_act(layer, 1), wl.make_grad_out(layer, 1)
    A = oracle.factor_A(tuple(layer), act)
    M = layer.M
    tol = 6.0 / math.sqrt(M)
    # centre tap (ky=kx=1) rows never see padding: index c*9 + 4
    centre = [c * 9 + 4 for c in range(4)]
    for i in centre:
        assert abs(A[i, i] - 0.5) < tol
        assert abs(A[i, -1] - 1 / math.sqrt(2 * math.pi)) < tol
        for j in centre:
            if i != j:
                assert abs(A[i, j] - 1 / (2 * math.pi)) < tol
    G = oracle.factor_G(tuple(layer), g, True)
    np.testing.assert_allclose(np.diag(G), 1e-6, rtol=0.1)
    assert np.abs(G - np.diag(np.diag(G))).max() < 1e-6 * tol
    np.testing.assert_allclose(oracle.factor_G(tuple(layer), g, False), G * layer.h * layer.w, rtol=1e-12)


def test_running_average_is_linear():
    layer = (2, 3, 4, 3, 1, 1, 5, 5, 1)
    a0, a1 = _rand_act(layer), _rand_act(layer)
    g0, g1 = _rand_grad(layer), _rand_grad(layer)
    A0, G0 = oracle.kfac_stats(layer, a0, g0, 0.0, False, None, None)
    np.testing.assert_array_equal(A0, oracle.factor_A(layer, a0))          # decay 0 overwrites
    np.testing.assert_array_equal(G0, oracle.factor_G(layer, g0))
    A1, G1 = oracle.kfac_stats(layer, a1, g1, 0.95, False, A0, G0)
    np.testing.assert_allclose(A1, 0.95 * A0 + 0.05 * oracle.factor_A(layer, a1), rtol=1e-13)
    np.testing.assert_allclose(G1, 0.95 * G0 + 0.05 * oracle.factor_G(layer, g1), rtol=1e-13)
    A2, G2 = oracle.kfac_stats(layer, a1, None, 0.5, False, A0, None)      # skip-G form
    assert G2 is None
    np.testing.assert_allclose(A2, 0.5 * A0 + 0.5 * oracle.factor_A(layer, a1), rtol=1e-13)


# ---------------------------------------------------------------- damping and inverse (Eq. 12)

def _spd(n, cond=50.0):
    Q, _ = np.linalg.qr(RNG.standard_normal((n, n)))
    e = np.geomspace(1.0, 1.0 / cond, n)
    return (Q * e) @ Q.T


def test_pi_damping_split():
    A, G = _spd(7), _spd(4) * 1e-6
    gamma = 1e-3
    pi, da, dg = oracle.pi_damping(A, G, gamma)
    assert pi == pytest.approx(math.sqrt(np.linalg.eigvalsh(A).mean() / np.linalg.eigvalsh(G).mean()), rel=1e-12)
    assert da == pytest.approx(pi * gamma, rel=1e-15) and dg == pytest.approx(gamma / pi, rel=1e-15)
    assert da * dg == pytest.approx(gamma ** 2, rel=1e-14)                 # the two dampings multiply to lambda
    pi2, _, _ = oracle.pi_damping(A * 9.0, G / 9.0, gamma)
    assert pi2 == pytest.approx(9.0 * pi, rel=1e-12)
    assert oracle.pi_damping(np.zeros((3, 3)), G, gamma)[0] == 1.0


@pytest.mark.parametrize("n", [1, 2, 3, 17, 64])
def test_spd_inverse_against_eigendecomposition(n):
    X, damp = _spd(n, 1e4), 3e-3
    Xi, info = oracle.spd_inverse(X, damp)
    assert info == 0
    e, Q = np.linalg.eigh(X)
    np.testing.assert_allclose(Xi, (Q / (e + damp)) @ Q.T, rtol=1e-9, atol=1e-9)
    assert np.abs((X + damp * np.eye(n)) @ Xi - np.eye(n)).max() < 1e-10
    assert np.array_equal(Xi, Xi.T)


def test_spd_inverse_special_cases():
    d = np.array([4.0, 0.5, 2.0])
    Xi, _ = oracle.spd_inverse(np.diag(d), 0.25)
    np.testing.assert_allclose(Xi, np.diag(1.0 / (d + 0.25)), rtol=1e-15)
    # 2x2 closed form (Eq. 17): [[a,b],[c,d]]^-1 = 1/(ad-bc) [[d,-b],[-c,a]]
    a, b, dd = 3.0, 1.2, 2.0
    Xi, _ = oracle.spd_inverse(np.array([[a, b], [b, dd]]), 0.0)
    np.testing.assert_allclose(Xi, np.array([[dd, -b], [-b, a]]) / (a * dd - b * b), rtol=1e-14)


def test_spd_inverse_reports_non_positive_pivot():
    X = np.array([[1.0, 2.0, 0.0], [2.0, 1.0, 0.0], [0.0, 0.0, 1.0]])      # indefinite
    _, info = oracle.spd_inverse(X, 0.0)
    assert info == 2
    v = RNG.standard_normal((5, 2))
    _, info = oracle.spd_inverse(v @ v.T, 0.0)                               # rank 2 < 5, no damping
    assert info > 0
    _, info = oracle.spd_inverse(v @ v.T, 1e-3)                              # damping restores PD
    assert info == 0


def test_kfac_invert_composes_damping_and_inverse():
    A, G = _spd(9), _spd(5) * 1e-5
    Ai, Gi, pi, info = oracle.kfac_invert(A, G, 1e-3)
    assert not info.any()
    tA, tG = np.trace(A) / 9, np.trace(G) / 5
    assert pi == pytest.approx(math.sqrt(tA / tG), rel=1e-12)
    np.testing.assert_allclose(Ai, np.linalg.inv(A + pi * 1e-3 * np.eye(9)), rtol=1e-9)
    np.testing.assert_allclose(Gi, np.linalg.inv(G + 1e-3 / pi * np.eye(5)), rtol=1e-9)


# ---------------------------------------------------------------- preconditioning (Eq. 6, 7, 12)

def test_precondition_is_the_kronecker_solve():
    """vec_rowmajor(G^-1 V A^-1) solves (Gd (x) Ad) u = vec_rowmajor(V)."""
    dG, dA = 5, 7
    Ad, Gd = _spd(dA) + 0.1 * np.eye(dA), _spd(dG) + 0.2 * np.eye(dG)
    V = RNG.standard_normal((dG, dA))
    U = oracle.kfac_precondition(np.linalg.inv(Gd), np.linalg.inv(Ad), V)
    ref = np.linalg.solve(np.kron(Gd, Ad), V.reshape(-1)).reshape(dG, dA)
    np.testing.assert_allclose(U, ref, rtol=1e-10, atol=1e-12)


def test_single_sample_fisher_is_exactly_kronecker():
    """N=1, fully-connected: the empirical Fisher vec(g a^T) vec(g a^T)^T equals G (x) A,
    which fixes the Kronecker order, the vec convention and the bias position; the whole
    chain stats -> invert -> precondition then matches a dense solve with both dampings."""
    fc = tuple(wl.fc_layer(1, 4, 3))
    a = np.maximum(RNG.standard_normal((1, 4)), 0) + 0.1
    g = RNG.standard_normal((1, 3))
    A, G = oracle.kfac_stats(fc, a, g, 0.0, False, None, None)
    ab = np.append(a[0], 1.0)
    gradW = np.outer(g[0], ab)                                  # dW = g a^T, last column = bias grad
    F = np.outer(gradW.reshape(-1), gradW.reshape(-1))
    np.testing.assert_allclose(np.kron(G, A), F, rtol=1e-13, atol=1e-15)
    gamma = 0.3
    Ai, Gi, pi, _ = oracle.kfac_invert(A, G, gamma)
    U = oracle.kfac_precondition(Gi, Ai, gradW)
    Fd = np.kron(G + gamma / pi * np.eye(3), A + gamma * pi * np.eye(5))
    np.testing.assert_allclose(U.reshape(-1), np.linalg.solve(Fd, gradW.reshape(-1)), rtol=1e-10)


def test_precondition_large_damping_limit_and_scale_invariance():
    layer = (4, 2, 3, 3, 1, 1, 4, 4, 1)
    dA, dG, _, _ = oracle.layer_dims(layer)
    A, G = oracle.kfac_stats(layer, _rand_act(layer), _rand_grad(layer), 0.0, False, None, None)
    V = RNG.standard_normal((dG, dA))
    gamma = 1e6
    Ai, Gi, _, _ = oracle.kfac_invert(A, G, gamma)
    np.testing.assert_allclose(oracle.kfac_precondition(Gi, Ai, V), V / gamma ** 2, rtol=1e-4)
    # moving a scalar between the factors changes pi but not the result
    Ai1, Gi1, pi1, _ = oracle.kfac_invert(A, G, 1e-2)
    Ai2, Gi2, pi2, _ = oracle.kfac_invert(A * 7.0, G / 7.0, 1e-2)
    assert pi2 == pytest.approx(7.0 * pi1, rel=1e-12)
    np.testing.assert_allclose(oracle.kfac_precondition(Gi2, Ai2, V), oracle.kfac_precondition(Gi1, Ai1, V),
                               rtol=1e-9)


# ---------------------------------------------------------------- BatchNorm unit-wise (Eq. 15-17)

def test_bn_unitwise_per_channel_solve():
    N, C, lam = 6, 5, 1e-3
    gg, gb = RNG.standard_normal((N, C)), RNG.standard_normal((N, C))
    F, og, ob = oracle.bn_unitwise_precondition(gg, gb, 0.0, lam)
    for i in range(C):
        Fi = np.zeros((2, 2))
        for n in range(N):
            v = np.array([gg[n, i], gb[n, i]])
            Fi += np.outer(v, v) / N
        np.testing.assert_allclose(F[i], [Fi[0, 0], Fi[0, 1], Fi[1, 1]], rtol=1e-13)
        u = np.linalg.solve(Fi + lam * np.eye(2), np.array([gg[:, i].mean(), gb[:, i].mean()]))
        np.testing.assert_allclose([og[i], ob[i]], u, rtol=1e-11)


def test_bn_unitwise_special_cases():
    N, C = 4, 3
    gg = RNG.standard_normal((N, C))
    gb = np.zeros((N, C))                                       # b = 0: diagonal blocks
    F, og, ob = oracle.bn_unitwise_precondition(gg, gb, 0.0, 0.5)
    np.testing.assert_allclose(og, gg.mean(0) / ((gg ** 2).mean(0) + 0.5), rtol=1e-13)
    np.testing.assert_array_equal(ob, 0.0)
    gb = RNG.standard_normal((N, C))
    _, og, ob = oracle.bn_unitwise_precondition(gg, gb, 0.0, 1e9)          # lambda -> inf
    np.testing.assert_allclose(og, gg.mean(0) / 1e9, rtol=1e-6)
    np.testing.assert_allclose(ob, gb.mean(0) / 1e9, rtol=1e-6)
    # running average of the three unique numbers, damping not folded in
    F0, _, _ = oracle.bn_unitwise_precondition(gg, gb, 0.0, 1e-3)
    F1, _, _ = oracle.bn_unitwise_precondition(gg * 2, gb * 2, 0.95, 1e-3, F0)
    np.testing.assert_allclose(F1, 0.95 * F0 + 0.05 * 4 * F0, rtol=1e-13)


def test_bn_per_sample_grads_match_autograd():
    N, C, H, W = 3, 4, 5, 2
    dy, xhat = RNG.standard_normal((N, C, H, W)), RNG.standard_normal((N, C, H, W))
    gg, gb = oracle.bn_reduce_nchw(dy.reshape(N, C, -1), xhat.reshape(N, C, -1))
    for n in range(N):
        gamma = torch.ones(C, dtype=torch.float64, requires_grad=True)
        beta = torch.zeros(C, dtype=torch.float64, requires_grad=True)
        y = gamma[None, :, None, None] * torch.from_numpy(xhat[n:n + 1]) + beta[None, :, None, None]
        (y * torch.from_numpy(dy[n:n + 1])).sum().backward()
        np.testing.assert_allclose(gg[n], gamma.grad.numpy(), rtol=1e-12)
        np.testing.assert_allclose(gb[n], beta.grad.numpy(), rtol=1e-12)


# ---------------------------------------------------------------- facts the paper prints

def test_paper_facts_golden():
    facts = {}
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, val = line.split("=")
                facts[key.strip()] = int(val)
    layers, bns = wl.resnet50_layers(32)
    assert len(layers) + len(bns) == facts["resnet50_layers_total"]
    assert sum(1 for L in layers if L.h_in > 1) == facts["resnet50_conv"] == len(bns)
    c = facts["example_c_out"]
    assert c in [C for C, _ in bns]
    # Sec. 4.2: the unit-wise approximation keeps one 2x2 block per channel instead of the 2c x 2c matrix; the
    # oracle's state holds the three distinct entries of each (symmetric) block
    gg, gb = wl.make_bn_grads(4, c, 3)
    F, og, ob = oracle.bn_unitwise_precondition(gg, gb, 0.0, 1e-6)
    assert F.shape == (c, 3) and og.shape == (c,) and ob.shape == (c,)
    # Sec. 5.2: a symmetric d x d statistic is communicated as d (d + 1) / 2 elements
    from oracle import pack as o_pack
    d = 37
    assert o_pack.pack_upper([np.zeros((d, d), np.float32)]).size == d * (d + 1) // 2


def test_accumulating_micro_batches_gives_the_whole_batch_statistics():
    """Sec. 7.1 (accumulation over steps): with decay (j-1)/j at micro-batch j the running average is the plain
    mean, and the mean of the micro-batch statistics is the statistic of the concatenated batch."""
    layer = wl.conv_layer(4, 6, 9, 3, 1, 1, 8)
    acts = [wl.make_act(layer, 700 + j) for j in range(3)]
    grads = [wl.make_grad_out(layer, 700 + j) for j in range(3)]
    A = G = None
    for j in range(3):
        A, G = oracle.kfac_stats(tuple(layer), acts[j], grads[j], j / (j + 1.0), True, A, G)
    whole = layer._replace(N=12)
    Ar, Gr = oracle.kfac_stats(tuple(whole), np.concatenate(acts), np.concatenate(grads), 0.0, True, None, None)
    assert np.allclose(A, Ar, rtol=1e-12, atol=1e-18) and np.allclose(G, Gr, rtol=1e-12, atol=1e-18)


def test_whole_chain_on_a_small_convolution_is_the_dense_damped_solve():
    """Two mini-batches through stats (running average) -> invert -> precondition on a 3x3 convolution with bias
    and spatially averaged gradients, against the same quantities written out with library routines only:
    patches from torch's unfold, the averages as plain sums, pi from the traces (Sec. 3.3, Eq. 12), and the
    preconditioned gradient as the solution of the dense system (G + gamma/pi I) (x) (A + gamma pi I) u = vec(grad W)."""
    layer = (3, 2, 4, 3, 1, 1, 5, 4, 1)
    N, c_in, c_out, k, s, p, h_in, w_in, _ = layer
    dA, dG, h, w = oracle.layer_dims(layer)
    decay, gamma = 0.8, 0.05
    A = G = None
    A_ref, G_ref = np.zeros((dA, dA)), np.zeros((dG, dG))
    for step in range(2):
        act, grad = _rand_act(layer), _rand_grad(layer) * 1e3
        d = 0.0 if step == 0 else decay
        A, G = oracle.kfac_stats(layer, act, grad, d, True, A, G)
        cols = torch.nn.functional.unfold(torch.from_numpy(act), k, padding=p, stride=s).numpy()   # [N, c_in k^2, h w]
        rows = np.concatenate([cols, np.ones((N, 1, h * w))], axis=1)                            # the bias row
        A_new = sum(rows[n] @ rows[n].T for n in range(N)) / (N * h * w)
        gm = grad.reshape(N, c_out, h * w)
        G_new = sum(gm[n] @ gm[n].T for n in range(N)) / (N * h * w)
        A_ref = d * A_ref + (1 - d) * A_new
        G_ref = d * G_ref + (1 - d) * G_new
    np.testing.assert_allclose(A, A_ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(G, G_ref, rtol=1e-12, atol=1e-14)
    V = RNG.standard_normal((dG, dA))
    Ai, Gi, pi, info = oracle.kfac_invert(A, G, gamma)
    assert not info.any()
    U = oracle.kfac_precondition(Gi, Ai, V)
    pi_ref = math.sqrt((np.trace(A_ref) / dA) / (np.trace(G_ref) / dG))
    assert pi == pytest.approx(pi_ref, rel=1e-12)
    dense = np.kron(G_ref + gamma / pi_ref * np.eye(dG), A_ref + gamma * pi_ref * np.eye(dA))
    np.testing.assert_allclose(U.reshape(-1), np.linalg.solve(dense, V.reshape(-1)), rtol=1e-9, atol=1e-12)
