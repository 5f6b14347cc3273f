"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(whole layer lists per call).

Configuration 3 is small enough for the oracle to rebuild everything element by element.
For the full ResNet-50 layer set (configurations 4 and 5) the oracle computes sampled
factor entries one by one, and the inverses / preconditioned gradients are checked
through properties that hold at any size, evaluated in float64 on the host:
    (X + damp I) X_inv = I        (sampled columns),   X_inv symmetric,
    U = G_inv dW A_inv            (sampled rows, from the GPU's own inverses),
with pi and the dampings recomputed on the host from the factor traces.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2002_06015_amd import kfac, workloads as wl

pytestmark = pytest.mark.gpu

TOL_FACTOR = 1e-4
TOL_PRECOND = 1e-3


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


def _run_step(layers, config, in_dtype, invert_idx=None, decay=0.0, fused=False):
    n = len(layers)
    tdt = torch.bfloat16 if in_dtype == kfac.KFAC_BF16 else torch.float32
    acts, grads, gws = [], [], []
    for i, L in enumerate(layers):
        s = wl.layer_seed(config, i)
        a, g = wl.make_act(L, s), wl.make_grad_out(L, s)
        if in_dtype == kfac.KFAC_BF16:
            a, g = wl.round_to_bf16(a), wl.round_to_bf16(g)
        acts.append(a)
        grads.append(g)
        gws.append(wl.make_grad_W(L, s))
    d_act = [torch.from_numpy(a).cuda().to(tdt) for a in acts]
    d_grad = [torch.from_numpy(g).cuda().to(tdt) for g in grads]
    d_gw = [torch.from_numpy(g).cuda() for g in gws]
    idx = list(range(n)) if invert_idx is None else list(invert_idx)
    ctx = kfac.Context(layers, in_dtype, extra_layer_lists=[[layers[i] for i in idx]])
    A = [torch.full((L.dA, L.dA), float("nan"), device="cuda") for L in layers]
    G = [torch.full((L.dG, L.dG), float("nan"), device="cuda") for L in layers]
    Ai = [torch.zeros_like(x) for x in A]
    Gi = [torch.zeros_like(x) for x in G]
    U = [torch.zeros(L.dG, L.dA, device="cuda") for L in layers]
    pi = torch.zeros(n, device="cuda")
    info = torch.zeros(2 * n, dtype=torch.int32, device="cuda")
    sel = lambda xs: [xs[i] for i in idx]
    if fused:
        # one call; pi / info are indexed by layer, the preconditioning covers every layer
        mask = [i in idx for i in range(n)]
        kfac.kfac_step(ctx, layers, in_dtype, d_act, d_grad, decay, True, A, G, mask, wl.GAMMA, Ai, Gi, pi, info,
                       d_gw, U)
        torch.cuda.synchronize()
        pi_h = host(pi)[idx]
    else:
        kfac.kfac_stats(ctx, layers, in_dtype, d_act, d_grad, decay, True, A, G)
        kfac.kfac_invert(ctx, sel(layers), sel(A), sel(G), wl.GAMMA, sel(Ai), sel(Gi), pi, info)
        kfac.kfac_precondition(ctx, sel(layers), sel(Gi), sel(Ai), sel(d_gw), sel(U))
        torch.cuda.synchronize()
        pi_h = host(pi)
    ctx.close()
    assert not info.cpu().numpy().any()
    return dict(acts=acts, grads=grads, gws=gws, A=A, G=G, Ai=Ai, Gi=Gi, U=U, pi=pi_h, idx=idx)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("in_dtype", [kfac.KFAC_F32, kfac.KFAC_BF16])
def test_config3_element_by_element(gpu, in_dtype):
    """Largest 3x3 layer (A 4609x4609 through the blocked inversion, G 512x512) and the
    FC layer (A 2049x2049, G 1000x1000), everything rebuilt by the oracle (on the
    bf16-rounded inputs for the bf16 variant)."""
    layers = wl.config_layers(3)
    r = _run_step(layers, 3, in_dtype)
    for i, L in enumerate(layers):
        Ar, Gr = oracle.kfac_stats(tuple(L), r["acts"][i], r["grads"][i], 0.0, True, None, None)
        assert relerr(host(r["A"][i]), Ar) <= TOL_FACTOR
        assert relerr(host(r["G"][i]), Gr) <= TOL_FACTOR
        Air, Gir, pir, _ = oracle.kfac_invert(Ar, Gr, wl.GAMMA)
        assert abs(r["pi"][i] - pir) <= 1e-4 * pir
        assert relerr(host(r["Ai"][i]), Air) <= TOL_PRECOND
        assert relerr(host(r["Gi"][i]), Gir) <= TOL_PRECOND
        Ur = oracle.kfac_precondition(Gir, Air, r["gws"][i])
        assert relerr(host(r["U"][i]), Ur) <= TOL_PRECOND


def _check_sampled(layers, r, rng, check_layers, n_pairs=48, n_cols=24):
    worst = {"A": 0.0, "G": 0.0, "inv": 0.0, "U": 0.0}
    for i in check_layers:
        L = layers[i]
        hA, hG = host(r["A"][i]), host(r["G"][i])
        assert np.array_equal(hA, hA.T) and np.array_equal(hG, hG.T)
        # sampled factor entries (always including the bias corner and a diagonal entry)
        I = np.concatenate([rng.integers(0, L.dA, n_pairs), [L.dA - 1, L.dA - 1, 0]])
        J = np.concatenate([rng.integers(0, L.dA, n_pairs), [L.dA - 1, 0, 0]])
        ref = oracle.factor_A_entries(tuple(L), r["acts"][i], I, J)
        worst["A"] = max(worst["A"], float(np.abs(hA[I, J] - ref).max() / np.abs(hA).max()))
        I = rng.integers(0, L.dG, n_pairs)
        J = np.where(rng.random(n_pairs) < 0.5, I, rng.integers(0, L.dG, n_pairs))
        ref = oracle.factor_G_entries(tuple(L), r["grads"][i], I, J, True)
        worst["G"] = max(worst["G"], float(np.abs(hG[I, J] - ref).max() / np.abs(hG).max()))
        if i not in r["idx"]:
            continue
        # damping recomputed on the host; defining property of the inverses on sampled columns
        pi = np.sqrt((np.trace(hA) / L.dA) / (np.trace(hG) / L.dG))
        assert abs(r["pi"][r["idx"].index(i)] - pi) <= 1e-4 * pi
        for X, Xi, damp in ((hA, host(r["Ai"][i]), pi * wl.GAMMA), (hG, host(r["Gi"][i]), wl.GAMMA / pi)):
            assert np.array_equal(Xi, Xi.T)
            cols = rng.integers(0, X.shape[0], n_cols)
            R = X @ Xi[:, cols] + damp * Xi[:, cols]
            R[cols, np.arange(n_cols)] -= 1.0
            worst["inv"] = max(worst["inv"], float(np.abs(R).max()))
        rows = rng.integers(0, L.dG, min(8, L.dG))
        Uref = host(r["Gi"][i])[rows] @ r["gws"][i].astype(np.float64) @ host(r["Ai"][i])
        worst["U"] = max(worst["U"], relerr(host(r["U"][i])[rows], Uref))
    return worst


@pytest.mark.timeout(600)
@pytest.mark.parametrize("fused", [False, True])
def test_config4_full_resnet50_set_sampled(gpu, fused):
    layers = wl.config_layers(4)
    r = _run_step(layers, 4, kfac.KFAC_F32, fused=fused)
    rng = np.random.default_rng(4)
    worst = _check_sampled(layers, r, rng, range(len(layers)))
    assert worst["A"] <= TOL_FACTOR and worst["G"] <= TOL_FACTOR, worst
    assert worst["inv"] <= 1e-3 and worst["U"] <= TOL_PRECOND, worst


@pytest.mark.timeout(900)
@pytest.mark.parametrize("fused", [False, True])
def test_config5_batch128_stale_subset_sampled(gpu, fused):
    """Batch 128, statistics for every layer, inverses only for the seeded 25 % subset.
    Sampled checks on the subset plus a few of the largest layers."""
    layers = wl.config_layers(5)
    subset = [int(i) for i in wl.stale_subset(len(layers), seed=0)]
    r = _run_step(layers, 5, kfac.KFAC_F32, invert_idx=subset, fused=fused)
    rng = np.random.default_rng(5)
    check = sorted(set(subset) | {0, 2, 46, 53})
    worst = _check_sampled(layers, r, rng, check, n_pairs=24, n_cols=16)
    assert worst["A"] <= TOL_FACTOR and worst["G"] <= TOL_FACTOR, worst
    assert worst["inv"] <= 1e-3 and worst["U"] <= TOL_PRECOND, worst
    # layers outside the subset keep whatever inverse they had (zeros here): untouched
    for i in range(len(layers)):
        if i not in subset:
            assert not bool(r["Ai"][i].any().item())
