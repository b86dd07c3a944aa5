"""Pins for the oracle's link-prediction head (Sec. 4.1: link prediction decoder, mini-batch and negative
sampling; App.: formulation of the MLP decoder) against things other than itself: what the sampling rule
guarantees (every positive is a stored edge, the negative tail differs from the positive one, both draws are
uniform -- checked by their frequencies), a library's index/multiply/activation/loss routines and their
reverse-mode derivatives in fp64, and central finite differences through encoder + decoder."""
import numpy as np
import pytest

import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")


def _local_graph(n, m, seed, K=2):
    rowptr, colidx = synth.uniform_graph(n, m, seed)
    sub = oracle.induced_subgraph(rowptr, colidx, oracle.partition(n, K, seed=seed), 0)
    return sub["rowptr"], sub["colidx"]


def test_edge_batch_properties():
    rp, ci = _local_graph(600, 4000, 3)
    n, nnz = len(rp) - 1, int(rp[-1])
    B = 200_000
    u, v, vn = oracle.edge_batch(rp, ci, seed=11, first_counter=0, B=B)
    edges = set(zip(np.repeat(np.arange(n), np.diff(rp)).tolist(), ci.tolist()))
    assert all((a, b) in edges for a, b in zip(u[:5000].tolist(), v[:5000].tolist()))
    # entry index recovered from (u, v): rows are duplicate-free, so (u, v) names one entry
    pos = {e: k for k, e in enumerate(zip(np.repeat(np.arange(n), np.diff(rp)).tolist(), ci.tolist()))}
    idx = np.fromiter((pos[(a, b)] for a, b in zip(u.tolist(), v.tolist())), dtype=np.int64, count=B)
    counts = np.bincount(idx, minlength=nnz)
    expect = B / nnz
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert abs(chi2 - (nnz - 1)) < 6 * np.sqrt(2 * (nnz - 1))        # uniform over the stored entries
    assert (vn != v).all() and vn.min() >= 0 and vn.max() < n
    # the negative tail is uniform over the n-1 other nodes: its gap to v (mod n) is uniform on 1..n-1
    gap = (vn.astype(np.int64) - v) % n
    cg = np.bincount(gap, minlength=n)[1:]
    chi2 = ((cg - B / (n - 1)) ** 2 / (B / (n - 1))).sum()
    assert cg.min() > 0 and abs(chi2 - (n - 2)) < 6 * np.sqrt(2 * (n - 2))
    # positive and negative draws are independent streams; batches are slices of one counter sequence
    u2, v2, vn2 = oracle.edge_batch(rp, ci, seed=11, first_counter=1000, B=500)
    assert np.array_equal(u2, u[1000:1500]) and np.array_equal(v2, v[1000:1500]) and np.array_equal(vn2, vn[1000:1500])
    u3, _, _ = oracle.edge_batch(rp, ci, seed=12, first_counter=0, B=1000)
    assert not np.array_equal(u3, u[:1000])
    assert abs(np.corrcoef(idx[:50_000], vn[:50_000])[0, 1]) < 0.02


def test_edge_batch_two_nodes_and_empty():
    rp, ci = synth.csr_from_pairs(2, [0], [1])
    u, v, vn = oracle.edge_batch(rp, ci, seed=1, first_counter=0, B=64)
    assert np.array_equal(vn, u) and np.array_equal(u + v, np.ones(64, np.int32))   # the only other node is u itself
    assert set(u.tolist()) == {0, 1}
    assert oracle.edge_batch(rp, ci, 1, 0, 0)[0].shape == (0,)


def test_pair_product_against_library():
    rng = np.random.default_rng(0)
    n, F, B = 50, 7, 300                     # B >> n: every node is hit many times, in several roles
    R = rng.standard_normal((n, F))
    u, v = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    vn = ((v + 1 + rng.integers(0, n - 1, B)) % n).astype(np.int32)
    g = rng.standard_normal((2 * B, F))
    tR = torch.tensor(R, requires_grad=True)
    tu, tv, tn = (torch.tensor(a.astype(np.int64)) for a in (u, v, vn))
    E = torch.cat([tR[tu] * tR[tv], tR[tu] * tR[tn]])
    E.backward(torch.tensor(g))
    np.testing.assert_allclose(oracle.pair_product_fwd(R, u, v, vn), E.detach().numpy(), rtol=1e-14)
    np.testing.assert_allclose(oracle.pair_product_bwd(R, u, v, vn, g), tR.grad.numpy(), rtol=1e-11, atol=1e-12)
    # a self pair (u == v) squares the row: gradient 2 r g
    one = np.array([3], np.int32)
    other = np.array([5], np.int32)
    gg = rng.standard_normal((2, F))
    dR = oracle.pair_product_bwd(R, one, one, other, gg)
    np.testing.assert_allclose(dR[3], 2 * R[3] * gg[0] + R[5] * gg[1], rtol=1e-13)
    assert not dR[np.setdiff1d(np.arange(n), [3, 5])].any()


@pytest.mark.parametrize("slope", [0.25, 0.0, -0.4, 1.0])
def test_prelu_against_library(slope):
    rng = np.random.default_rng(1)
    Z, g = rng.standard_normal((40, 9)), rng.standard_normal((40, 9))
    tZ = torch.tensor(Z, requires_grad=True)
    ta = torch.tensor([slope], dtype=torch.float64, requires_grad=True)
    out = torch.nn.functional.prelu(tZ, ta)
    out.backward(torch.tensor(g))
    np.testing.assert_allclose(oracle.prelu_fwd(Z, slope), out.detach().numpy(), rtol=1e-15)
    dZ, ds = oracle.prelu_bwd(Z, g, slope)
    np.testing.assert_allclose(dZ, tZ.grad.numpy(), rtol=1e-14)
    assert ds == pytest.approx(ta.grad.item(), rel=1e-12)
    # a forced mask replaces the decision
    dZ2, _ = oracle.prelu_bwd(Z, g, slope, open_mask=np.ones_like(Z, dtype=bool))
    np.testing.assert_array_equal(dZ2, g)


def test_bce_against_library_and_closed_forms():
    rng = np.random.default_rng(2)
    z = rng.normal(0, 4, 101)
    z[:3] = [800.0, -800.0, 0.0]             # no overflow at large |z|
    tz = torch.tensor(z, requires_grad=True)
    y = torch.cat([torch.ones(40, dtype=torch.float64), torch.zeros(61, dtype=torch.float64)])
    want = torch.nn.functional.binary_cross_entropy_with_logits(tz, y)
    want.backward()
    loss, dz = oracle.bce_logits(z, 40)
    assert loss == pytest.approx(want.item(), rel=1e-13)
    np.testing.assert_allclose(dz, tz.grad.numpy(), rtol=1e-12, atol=1e-300)
    assert oracle.bce_logits(np.zeros(10), 5)[0] == pytest.approx(np.log(2.0), rel=1e-15)
    l, d = oracle.bce_logits(np.array([50.0, -50.0]), 1)      # confident and right: loss and gradient vanish
    assert l < 1e-20 and np.abs(d).max() < 1e-20
    assert oracle.bce_logits(np.array([-30.0]), 1)[0] == pytest.approx(30.0, rel=1e-12)


def _link_case(encoder):
    rp, ci = _local_graph(160, 700, 5)
    n = len(rp) - 1
    rng = np.random.default_rng(3)
    dims, dec_dims = [6, 8, 5], [5, 7, 1]
    enc = []
    for fi, fo in zip(dims[:-1], dims[1:]):
        W = [0.5 * rng.standard_normal((fi, fo)) for _ in range(2 if encoder == "sage" else 1)]
        enc.append(tuple(W) + (0.1 * rng.standard_normal(fo),))
    dec = [(0.5 * rng.standard_normal((5, 7)), np.array([0.25])), (0.5 * rng.standard_normal((7, 1)),)]
    X = rng.standard_normal((n, dims[0]))
    batch = oracle.edge_batch(rp, ci, seed=9, first_counter=0, B=64)
    return rp, ci, X, batch, enc, dec


@pytest.mark.parametrize("encoder", ["sage", "gcn", "mlp"])
def test_link_step_finite_differences(encoder):
    rp, ci, X, batch, enc, dec = _link_case(encoder)
    loss, ge, gd, z = omodel.link_loss_and_grads(rp, ci, X, batch, enc, dec, encoder)
    assert z.shape == (128,) and np.isfinite(loss)

    def f(enc_, dec_):
        R, _ = omodel.forward(rp, ci, X, enc_, encoder)
        zz, _ = omodel.decoder_forward(R, batch, dec_)
        return oracle.bce_logits(zz, 64, need_grad=False)[0]

    h = 1e-6
    for (l, t, idx) in [(0, 0, (1, 2)), (1, 0, (3, 1)), (0, len(enc[0]) - 1, (4,)), (1, len(enc[1]) - 1, (0,))]:
        def bump(delta):
            e2 = [tuple(np.array(a, dtype=np.float64) for a in layer) for layer in enc]
            e2[l][t][idx] += delta
            return f(e2, dec)
        assert (bump(h) - bump(-h)) / (2 * h) == pytest.approx(ge[l][t][idx], rel=2e-5, abs=1e-9)
    for (k, t, idx) in [(0, 0, (2, 3)), (1, 0, (5, 0)), (0, 1, (0,))]:
        def bump(delta):
            d2 = [tuple(np.array(a, dtype=np.float64) for a in layer) for layer in dec]
            d2[k][t][idx] += delta
            return f(enc, d2)
        assert (bump(h) - bump(-h)) / (2 * h) == pytest.approx(np.asarray(gd[k][t])[idx], rel=2e-5, abs=1e-9)


def test_decoder_against_library_autograd():
    rp, ci, X, batch, enc, dec = _link_case("mlp")
    rng = np.random.default_rng(8)
    R = rng.standard_normal((len(rp) - 1, 5))
    tR = torch.tensor(R, requires_grad=True)
    T0 = torch.tensor(dec[0][0], requires_grad=True)
    a0 = torch.tensor(dec[0][1], requires_grad=True)
    T1 = torch.tensor(dec[1][0], requires_grad=True)
    u, v, vn = (torch.tensor(a.astype(np.int64)) for a in batch)
    E0 = torch.cat([tR[u] * tR[v], tR[u] * tR[vn]])
    z = (torch.nn.functional.prelu(E0 @ T0, a0) @ T1).ravel()
    y = torch.cat([torch.ones(64, dtype=torch.float64), torch.zeros(64, dtype=torch.float64)])
    loss = torch.nn.functional.binary_cross_entropy_with_logits(z, y)
    loss.backward()
    zo, saved = omodel.decoder_forward(R, batch, dec)
    np.testing.assert_allclose(zo, z.detach().numpy(), rtol=1e-12, atol=1e-13)
    lo, dz = oracle.bce_logits(zo, 64)
    assert lo == pytest.approx(loss.item(), rel=1e-13)
    d, ds = oracle.prelu_bwd(saved[0][1], oracle.dense_bwd(saved[1][0], saved[1][1], dz.reshape(-1, 1), dec[1][0], 0,
                                                            need_dbias=False)[2], 0.25)
    dT0, _, dE0 = oracle.dense_bwd(saved[0][0], saved[0][1], d, dec[0][0], 0, need_dbias=False)
    np.testing.assert_allclose(dT0, T0.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert ds == pytest.approx(a0.grad.item(), rel=1e-10)
    np.testing.assert_allclose(oracle.pair_product_bwd(R, *batch, dE0), tR.grad.numpy(), rtol=1e-10, atol=1e-13)
