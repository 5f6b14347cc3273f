"""GPU parity of the parameter update and the weight rescaling (Sec. 6.2, 6.3) against the oracle.

Tolerance: the kernel takes w' in fp32 with two fused multiply-adds and one subtraction (three
roundings, each at most 2^-24 relative to the largest term), the norm in double; the oracle is
float64 throughout.  With |eta U| and |m v| no larger than |w| this bounds the element error by
about 4 * 2^-24 * max|w| and the norm-wise error by 3e-7; the tests allow 1e-6."""
import numpy as np
import pytest
import torch

from oracle import update
from paper_2002_06015_amd import kfac, workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-6


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    kfac.lib()
    return torch.device("cuda")


def _rel(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref) / max(np.linalg.norm(ref), 1e-300))


# weights per layer: below one chunk, ragged tails of 1..3, exactly one chunk, several chunks + tail, a bias column
LAYERS = [wl.fc_layer(2, 3, 1, bias=0), wl.fc_layer(2, 7, 5), wl.fc_layer(2, 64, 64, bias=0),
          wl.fc_layer(2, 301, 77), wl.conv_layer(2, 13, 29, 3, 1, 1, 6), wl.fc_layer(2, 1000, 37),
          wl.fc_layer(2, 2, 2, bias=0)]


def _state(layers, seed):
    rng = np.random.default_rng(seed)
    W, Wp, U = [], [], []
    for L in layers:
        dA, dG = kfac.kfac_layer_dims(L)[:2]
        w = rng.standard_normal((dG, dA)).astype(np.float32) * np.float32(np.sqrt(2.0 / dA))
        W.append(w)
        Wp.append((w + 0.01 * rng.standard_normal((dG, dA)).astype(np.float32)).astype(np.float32))
        U.append((rng.standard_normal((dG, dA)) * 0.5).astype(np.float32))
    return W, Wp, U


@pytest.mark.parametrize("rescale", [False, True])
def test_update_matches_oracle_over_several_steps(gpu, rescale):
    W, Wp, _ = _state(LAYERS, 3)
    ctx = kfac.Context(LAYERS)
    dW = [torch.from_numpy(x).cuda() for x in W]
    dWp = [torch.from_numpy(x).cuda() for x in Wp]
    rW = [x.astype(np.float64) for x in W]
    rWp = [x.astype(np.float64) for x in Wp]
    rng = np.random.default_rng(17)
    for step in range(4):
        eta = update.lr_polynomial(0.05, step, 0, 10, 3.5)
        m = update.momentum_coupled(0.9, 0.05, eta)
        U = [(rng.standard_normal(w.shape) * 0.5).astype(np.float32) for w in W]
        before = [w.clone() for w in dW]
        kfac.kfac_update_weights(ctx, LAYERS, [torch.from_numpy(u).cuda() for u in U], eta, m, rescale, 1e-9, dW, dWp)
        torch.cuda.synchronize()
        for l, L in enumerate(LAYERS):
            dG = kfac.kfac_layer_dims(L)[1]
            # both sides advance from the same fp32 state, so that errors do not compound across steps
            new, prev = update.update_weights(before[l].cpu().numpy().astype(np.float64), rWp[l], U[l], np.float32(eta),
                                              np.float32(m), dG, rescale)
            assert _rel(dW[l].cpu().numpy(), new) < TOL, (step, l)
            assert torch.equal(dWp[l], before[l]), (step, l)                  # w^(t) kept bit for bit
            if rescale:
                nrm = float(np.linalg.norm(dW[l].cpu().numpy().astype(np.float64)))
                assert abs(nrm - np.sqrt(2.0 * dG)) < 1e-5 * np.sqrt(2.0 * dG)
            rWp[l] = dWp[l].cpu().numpy().astype(np.float64)
    ctx.close()


def test_update_special_cases(gpu):
    """eta = 0 and m = 0 leave the weights alone; m = 0 is plain descent; an all-zero layer stays zero when rescaled."""
    W, Wp, U = _state(LAYERS, 9)
    ctx = kfac.Context(LAYERS)
    dU = [torch.from_numpy(x).cuda() for x in U]
    dW = [torch.from_numpy(x).cuda() for x in W]
    dWp = [torch.from_numpy(x).cuda() for x in Wp]
    kfac.kfac_update_weights(ctx, LAYERS, dU, 0.0, 0.0, False, 1e-9, dW, dWp)
    torch.cuda.synchronize()
    for l in range(len(LAYERS)):
        assert np.array_equal(dW[l].cpu().numpy(), W[l]) and np.array_equal(dWp[l].cpu().numpy(), W[l])
    kfac.kfac_update_weights(ctx, LAYERS, dU, 0.25, 0.0, False, 1e-9, dW, dWp)
    torch.cuda.synchronize()
    for l in range(len(LAYERS)):
        ref = W[l].astype(np.float64) - 0.25 * U[l].astype(np.float64)
        assert np.max(np.abs(dW[l].cpu().numpy() - ref)) <= 2.0 ** -23 * np.max(np.abs(ref))
    zW = [torch.zeros_like(x) for x in dW]
    zP = [torch.zeros_like(x) for x in dW]
    zU = [torch.zeros_like(x) for x in dW]
    kfac.kfac_update_weights(ctx, LAYERS, zU, 0.1, 0.9, True, 1e-9, zW, zP)
    torch.cuda.synchronize()
    assert all(float(x.abs().max()) == 0.0 for x in zW)
    ctx.close()


def test_update_full_resnet50_weight_set(gpu):
    """All 54 layers of the ResNet-50 set in one call, in the launch configuration the bench times."""
    layers, _ = wl.resnet50_layers(32)
    layers = [tuple(L) for L in layers]
    W, Wp, U = _state(layers, 21)
    ctx = kfac.Context(layers)
    dW = [torch.from_numpy(x).cuda() for x in W]
    dWp = [torch.from_numpy(x).cuda() for x in Wp]
    kfac.kfac_update_weights(ctx, layers, [torch.from_numpy(x).cuda() for x in U], 0.02, 0.36, True, 1e-9, dW, dWp)
    torch.cuda.synchronize()
    for l, L in enumerate(layers):
        dG = kfac.kfac_layer_dims(L)[1]
        new, prev = update.update_weights(W[l], Wp[l], U[l], np.float32(0.02), np.float32(0.36), dG, True)
        assert _rel(dW[l].cpu().numpy(), new) < TOL, l
        assert np.array_equal(dWp[l].cpu().numpy(), W[l])
    ctx.close()
