"""Pins for the oracle's layer normalisation + PReLU (the paper's encoder variant, Sec. 4.1) against things
other than itself: the reference routines of a numerical library (PyTorch's CPU layer_norm / prelu and its
reverse-mode derivative, in fp64), closed forms that follow from the definitions, and central finite
differences through a whole model."""
import numpy as np
import pytest

import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")


def _case(n, F, seed):
    rng = np.random.default_rng(seed)
    Z = rng.normal(0.3, 2.0, (n, F))
    gamma = rng.normal(1.0, 0.3, F)
    beta = rng.normal(0.0, 0.5, F)
    g = rng.normal(0.0, 1.0, (n, F))
    return Z, gamma, beta, g


@pytest.mark.parametrize("n,F,slope", [(7, 5, 0.25), (40, 64, 0.1), (3, 256, -0.3), (11, 1, 0.25)])
def test_forward_and_backward_match_library_routines(n, F, slope):
    Z, gamma, beta, g = _case(n, F, seed=F)
    tZ = torch.tensor(Z, dtype=torch.float64, requires_grad=True)
    tg = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    tb = torch.tensor(beta, dtype=torch.float64, requires_grad=True)
    ta = torch.tensor([slope], dtype=torch.float64, requires_grad=True)
    out = torch.nn.functional.prelu(torch.nn.functional.layer_norm(tZ, (F,), tg, tb, eps=oracle.LN_EPS), ta)
    out.backward(torch.tensor(g))
    Hn = oracle.layernorm_prelu_fwd(Z, gamma, beta, slope)
    np.testing.assert_allclose(Hn, out.detach().numpy(), rtol=1e-12, atol=1e-12)
    dZ, dg, db, ds = oracle.layernorm_prelu_bwd(Z, g, gamma, beta, slope)
    np.testing.assert_allclose(dZ, tZ.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(ds, ta.grad.item(), rtol=1e-10, atol=1e-11)


def test_closed_forms():
    Z, _, _, g = _case(50, 32, seed=1)
    ones, zeros = np.ones(32), np.zeros(32)
    # slope 1 makes the activation the identity: rows have mean 0 and variance var/(var+eps)
    Y = oracle.layernorm_prelu_fwd(Z, ones, zeros, 1.0)
    np.testing.assert_allclose(Y.mean(1), 0.0, atol=1e-13)
    var = Z.var(1)
    np.testing.assert_allclose(Y.var(1), var / (var + oracle.LN_EPS), rtol=1e-12)
    # invariance under a positive affine map of the row (exact for eps = 0)
    Y0 = oracle.layernorm_prelu_fwd(Z, ones, zeros, 0.25, eps=0.0)
    Y1 = oracle.layernorm_prelu_fwd(3.7 * Z - 11.0, ones, zeros, 0.25, eps=0.0)
    np.testing.assert_allclose(Y0, Y1, rtol=1e-10, atol=1e-12)
    # slope 0 is ReLU; a negative input is scaled by the slope
    Yr = oracle.layernorm_prelu_fwd(Z, ones, zeros, 0.0)
    np.testing.assert_array_equal(Yr, np.maximum(Y, 0.0))
    Yp = oracle.layernorm_prelu_fwd(Z, ones, zeros, 0.25)
    np.testing.assert_allclose(Yp, np.where(Y > 0, Y, 0.25 * Y), rtol=0, atol=0)
    # the gradient w.r.t. Z is orthogonal to the all-ones vector and, for eps = 0, to the normalised row
    # (the Jacobian of the normalisation projects both directions out)
    dZ, _, _, _ = oracle.layernorm_prelu_bwd(Z, g, ones, zeros, 1.0, eps=0.0)
    np.testing.assert_allclose(dZ.sum(1), 0.0, atol=1e-12)
    np.testing.assert_allclose((dZ * oracle.layernorm_prelu_fwd(Z, ones, zeros, 1.0, eps=0.0)).sum(1), 0.0, atol=1e-11)
    # a forced decision mask replaces Y > 0 and nothing else
    dZa, dga, dba, dsa = oracle.layernorm_prelu_bwd(Z, g, ones, zeros, 0.25)
    dZb, dgb, dbb, dsb = oracle.layernorm_prelu_bwd(Z, g, ones, zeros, 0.25, open_mask=Y > 0)
    assert np.array_equal(dZa, dZb) and np.array_equal(dga, dgb) and dsa == dsb


def test_model_gradients_by_finite_differences():
    """Every parameter of a 3-layer model with normalised, PReLU-activated hidden layers."""
    rowptr, colidx = synth.uniform_graph(60, 150, seed=2)
    rowptr, colidx = rowptr.astype(np.int32), colidx.astype(np.int32)
    dims = [5, 6, 4, 3]
    X, y = synth.features(60, dims[0], seed=3).astype(np.float64), synth.labels(60, dims[-1], seed=4)
    rng = np.random.default_rng(5)
    params = []
    for l, (Ws, Wn, b) in enumerate(synth.sage_params(dims, seed=6)):
        layer = [np.asarray(Ws, np.float64), np.asarray(Wn, np.float64), rng.normal(0, 0.1, dims[l + 1])]
        if l < len(dims) - 2:
            layer += [rng.normal(1.0, 0.2, dims[l + 1]), rng.normal(0.0, 0.2, dims[l + 1]), np.array([0.25])]
        params.append(tuple(layer))
    loss, grads, _, _ = omodel.loss_and_grads(rowptr, colidx, X, y, params)
    flat, gflat = omodel.flatten(params), omodel.flatten(grads)
    assert flat.shape == gflat.shape
    h = 1e-6
    worst = 0.0
    for i in range(flat.size):
        e = np.zeros_like(flat)
        e[i] = h
        lp = omodel.loss_and_grads(rowptr, colidx, X, y, omodel.unflatten(flat + e, params))[0]
        lm = omodel.loss_and_grads(rowptr, colidx, X, y, omodel.unflatten(flat - e, params))[0]
        fd = (lp - lm) / (2 * h)
        worst = max(worst, abs(fd - gflat[i]) / max(abs(fd), abs(gflat[i]), 1e-3))
    assert worst < 1e-6, worst   # a dropped or mis-signed term would show as an error of order one
    # a training step moves every tensor against its gradient
    _, new = omodel.train_step(rowptr, colidx, X, y, params, 0.1)
    np.testing.assert_allclose(omodel.flatten(new), flat - 0.1 * gflat, rtol=1e-12, atol=1e-15)
