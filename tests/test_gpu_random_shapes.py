"""GPU parity on seeded random layer shapes: whole groups of layers through the fused step and
through the separate calls, every result element by element against the float64 oracle.

The shapes are drawn so that every path of the statistics is hit by some layer of every group:
kernels 1 / 3 / 5 / 7, strides 1 and 2, with and without padding, non-square images, planes that
are and are not whole 16-byte chunks (in-place contraction, the bf16 four-element tail, the
copying path), 3x3 / stride-1 layers with and without the correlation form, single samples, a
bias row or none, fp32 and bf16 inputs.  The damping is large enough (gamma = 0.05) that the
inverses of these small, often rank-deficient factors are well conditioned, so the inverse and
the preconditioned gradient are compared to the same tolerances as everywhere else."""
import numpy as np
import pytest
import torch

import oracle
from paper_2002_06015_amd import kfac, workloads as wl

pytestmark = pytest.mark.gpu

TOL_FACTOR = 1e-4
TOL_INVERSE = 1e-4
TOL_PRECOND = 1e-3
GAMMA = 0.05


def relerr(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    kfac.lib()
    return torch.device("cuda")


def random_layers(seed, count):
    rng = np.random.default_rng(seed)
    layers = []
    while len(layers) < count:
        k = int(rng.choice([1, 1, 3, 3, 5, 7]))
        stride = int(rng.choice([1, 1, 2]))
        pad = int(rng.integers(0, k // 2 + 1))
        h_in, w_in = int(rng.integers(k, 23)), int(rng.integers(k, 23))
        if rng.random() < 0.25:
            w_in = h_in = int(rng.choice([6, 14, 7, 12, 16]))       # 36 / 196 / 49 / 144 / 256 positions for k = 1
        c_in, c_out = int(rng.integers(1, 70)), int(rng.integers(1, 150))
        if k >= 5:
            c_in = int(rng.integers(1, 9))
        N = int(rng.choice([1, 2, 3, 5, 8, 9]))
        layers.append(wl.Layer(N, c_in, c_out, k, stride, pad, h_in, w_in, int(rng.integers(0, 2))))
    return layers


@pytest.mark.parametrize("in_dtype", [kfac.KFAC_F32, kfac.KFAC_BF16])
@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_layer_groups_match_the_oracle(gpu, seed, in_dtype):
    layers = random_layers(seed, 9)
    n = len(layers)
    tdt = torch.bfloat16 if in_dtype == kfac.KFAC_BF16 else torch.float32
    acts, grads, gws = [], [], []
    for i, L in enumerate(layers):
        a, g = wl.make_act(L, 100 * seed + i), wl.make_grad_out(L, 100 * seed + i)
        if in_dtype == kfac.KFAC_BF16:
            a, g = wl.round_to_bf16(a), wl.round_to_bf16(g)
        acts.append(a)
        grads.append(g)
        gws.append(wl.make_grad_W(L, 100 * seed + i))
    ref = []
    for i, L in enumerate(layers):
        Ar, Gr = oracle.kfac_stats(tuple(L), acts[i], grads[i], 0.0, False, None, None)
        Air, Gir, pir, info = oracle.kfac_invert(Ar, Gr, GAMMA)
        assert not info.any()
        ref.append((Ar, Gr, Air, Gir, pir, oracle.kfac_precondition(Gir, Air, gws[i])))
    d_act = [torch.from_numpy(a).cuda().to(tdt) for a in acts]
    d_grad = [torch.from_numpy(g).cuda().to(tdt) for g in grads]
    d_gw = [torch.from_numpy(g).cuda() for g in gws]
    for fused in (False, True):
        ctx = kfac.Context(layers, in_dtype)
        A = [torch.full((L.dA, L.dA), float("nan"), device="cuda") for L in layers]
        G = [torch.full((L.dG, L.dG), float("nan"), device="cuda") for L in layers]
        Ai = [torch.zeros(L.dA, L.dA, device="cuda") for L in layers]
        Gi = [torch.zeros(L.dG, L.dG, device="cuda") for L in layers]
        U = [torch.zeros(L.dG, L.dA, device="cuda") for L in layers]
        pi = torch.zeros(n, device="cuda")
        info = torch.zeros(2 * n, dtype=torch.int32, device="cuda")
        if fused:
            kfac.kfac_step(ctx, layers, in_dtype, d_act, d_grad, 0.0, False, A, G, None, GAMMA, Ai, Gi, pi, info, d_gw, U)
        else:
            kfac.kfac_stats(ctx, layers, in_dtype, d_act, d_grad, 0.0, False, A, G)
            kfac.kfac_invert(ctx, layers, A, G, GAMMA, Ai, Gi, pi, info)
            kfac.kfac_precondition(ctx, layers, Gi, Ai, d_gw, U)
        torch.cuda.synchronize()
        ctx.close()
        assert not info.cpu().numpy().any()
        for i, L in enumerate(layers):
            Ar, Gr, Air, Gir, pir, Ur = ref[i]
            what = "seed %d layer %d %s fused=%s" % (seed, i, tuple(L), fused)
            hA, hG = host(A[i]), host(G[i])
            assert np.array_equal(hA, hA.T) and np.array_equal(hG, hG.T), what
            assert relerr(hA, Ar) <= TOL_FACTOR, what
            assert relerr(hG, Gr) <= TOL_FACTOR, what
            assert abs(float(pi[i]) - pir) <= 1e-4 * pir, what
            assert relerr(host(Ai[i]), Air) <= TOL_INVERSE, what
            assert relerr(host(Gi[i]), Gir) <= TOL_INVERSE, what
            assert relerr(host(U[i]), Ur) <= TOL_PRECOND, what


def random_pointwise_layers(seed, count):
    """1x1 / stride-1 layers (the ones contracted in place from NHWC tensors) with channel counts that are and are
    not multiples of 4 and 8, images from one pixel to a few hundred, one to 33 samples; two other layers so that
    the conversion inside the call runs beside them."""
    rng = np.random.default_rng(seed)
    layers = []
    while len(layers) < count:
        mult = int(rng.choice([1, 4, 8, 8]))
        c_in, c_out = mult * int(rng.integers(1, 300 // mult)), mult * int(rng.integers(1, 200 // mult))
        h, w = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        N = int(rng.choice([1, 2, 3, 8, 33]))
        layers.append(wl.Layer(N, c_in, c_out, 1, 1, 0, h, w, int(rng.integers(0, 2))))
    layers.append(wl.conv_layer(3, 16, 24, 3, 1, 1, int(rng.integers(4, 15))))
    layers.append(wl.fc_layer(int(rng.integers(1, 40)), 48, 16))
    return layers


@pytest.mark.parametrize("in_dtype", [kfac.KFAC_F32, kfac.KFAC_BF16])
@pytest.mark.parametrize("seed", [21, 22, 23])
def test_random_pointwise_groups_from_nhwc_tensors_match_the_oracle(gpu, seed, in_dtype):
    layers = random_pointwise_layers(seed, 10)
    tdt = torch.bfloat16 if in_dtype == kfac.KFAC_BF16 else torch.float32
    ctx = kfac.Context(layers, in_dtype)
    A = [torch.full((L.dA, L.dA), float("nan"), device="cuda") for L in layers]
    G = [torch.full((L.dG, L.dG), float("nan"), device="cuda") for L in layers]
    Ar, Gr = [None] * len(layers), [None] * len(layers)
    for step in range(2):
        decay = 0.0 if step == 0 else 0.75
        d_act, d_grad = [], []
        for i, L in enumerate(layers):
            a, g = wl.make_act(L, 1000 * seed + 10 * i + step), wl.make_grad_out(L, 1000 * seed + 10 * i + step)
            if in_dtype == kfac.KFAC_BF16:
                a, g = wl.round_to_bf16(a), wl.round_to_bf16(g)
            Ar[i], Gr[i] = oracle.kfac_stats(tuple(L), a, g, decay, False, Ar[i], Gr[i])
            h, w = kfac.kfac_layer_dims(L)[2:]
            a = np.ascontiguousarray(a.reshape(L.N, L.c_in, L.h_in, L.w_in).transpose(0, 2, 3, 1))
            g = np.ascontiguousarray(g.reshape(L.N, L.c_out, h, w).transpose(0, 2, 3, 1))
            d_act.append(torch.from_numpy(a).cuda().to(tdt))
            d_grad.append(torch.from_numpy(g).cuda().to(tdt))
        kfac.kfac_stats(ctx, layers, in_dtype, d_act, d_grad, decay, False, A, G, nhwc=True)
        torch.cuda.synchronize()
        for i, L in enumerate(layers):
            what = "seed %d step %d layer %d %s" % (seed, step, i, tuple(L))
            hA, hG = host(A[i]), host(G[i])
            assert np.array_equal(hA, hA.T) and np.array_equal(hG, hG.T), what
            assert relerr(hA, Ar[i]) <= TOL_FACTOR, what
            assert relerr(hG, Gr[i]) <= TOL_FACTOR, what
    ctx.close()
