"""Pins for the oracle's GCN layer and dense (MLP) layer -- the paper's other encoders (Sec. 4.1) -- against
things other than its own loops: facts about the normalised adjacency of Kipf & Welling that follow from its
definition (its top eigenvector and eigenvalue, its spectrum, its form on regular and complete graphs), a
dense matrix built by a different route (a library's sparse matrix algebra), a library's reverse-mode
derivative, the adjoint identity and central finite differences."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")


def _local_graph(n, m, seed, K=2):
    rowptr, colidx = synth.uniform_graph(n, m, seed)
    part = oracle.partition(n, K, seed=seed)
    sub = oracle.induced_subgraph(rowptr, colidx, part, 0)
    return sub["rowptr"], sub["colidx"]


def _ahat(rp, ci):
    """Dt^-1/2 (A + I) Dt^-1/2 through scipy's sparse algebra."""
    n = len(rp) - 1
    A = sp.csr_matrix((np.ones(len(ci)), ci, rp), shape=(n, n)) + sp.identity(n, format="csr")
    d = np.asarray(A.sum(1)).ravel()
    S = sp.diags(d ** -0.5)
    return (S @ A @ S).toarray()


def test_sqrt_degree_vector_is_the_eigenvector_of_eigenvalue_one():
    # Ahat (Dt^1/2 1) = Dt^-1/2 (A + I) 1 = Dt^-1/2 Dt 1 = Dt^1/2 1, for any graph
    rp, ci = _local_graph(500, 2000, 7)
    n = len(rp) - 1
    assert (np.diff(rp) == 0).any()
    x = np.sqrt(np.diff(rp) + 1.0)[:, None] * np.array([[1.0, -2.0, 0.5]])
    np.testing.assert_allclose(oracle.gcn_aggregate(rp, ci, x), x, rtol=1e-13)
    np.testing.assert_allclose(oracle.gcn_aggregate(rp, ci, x, transpose=True), x, rtol=1e-13)
    np.testing.assert_allclose(oracle.gcn_norm(rp), 1.0 / np.sqrt(np.diff(rp) + 1.0), rtol=1e-15)
    # the spectrum lies in (-1, 1]: power iteration from a random vector cannot grow
    v = np.random.default_rng(0).standard_normal((n, 1))
    for _ in range(30):
        w = oracle.gcn_aggregate(rp, ci, v)
        assert np.linalg.norm(w) <= np.linalg.norm(v) * (1 + 1e-12)
        v = w


def test_regular_and_complete_graphs():
    n, F = 12, 4
    H = np.random.default_rng(1).standard_normal((n, F))
    # cycle: every node has degree 2, Ahat H = mean over the closed neighbourhood
    u = np.arange(n)
    rp, ci = synth.csr_from_pairs(n, u, (u + 1) % n)
    want = (H + np.roll(H, 1, 0) + np.roll(H, -1, 0)) / 3.0
    np.testing.assert_allclose(oracle.gcn_aggregate(rp, ci, H), want, rtol=1e-13)
    # complete graph: Ahat = J / n, every row becomes the mean of all rows
    iu, ju = np.triu_indices(n, 1)
    rp, ci = synth.csr_from_pairs(n, iu, ju)
    np.testing.assert_allclose(oracle.gcn_aggregate(rp, ci, H), np.tile(H.mean(0), (n, 1)), rtol=1e-13)
    # a graph without edges: Ahat = I
    rp0 = np.zeros(n + 1, dtype=np.int32)
    np.testing.assert_allclose(oracle.gcn_aggregate(rp0, np.zeros(0, np.int32), H), H, rtol=0)
    # star with 4 leaves, features = node id: centre = (0 + (1+2+3+4)/sqrt(10)) ... written out by hand
    rp_s, ci_s = synth.csr_from_pairs(5, [0, 0, 0, 0], [1, 2, 3, 4])
    x = np.arange(5.0)[:, None]
    out = oracle.gcn_aggregate(rp_s, ci_s, x)
    assert out[0, 0] == pytest.approx(10.0 / np.sqrt(5.0 * 2.0))
    for leaf in range(1, 5):
        assert out[leaf, 0] == pytest.approx(leaf / 2.0)     # centre carries feature 0


def test_aggregate_against_sparse_library_and_adjoint():
    rp, ci = _local_graph(400, 1500, 3)
    n = len(rp) - 1
    rng = np.random.default_rng(0)
    H, G = rng.standard_normal((n, 6)), rng.standard_normal((n, 6))
    A = _ahat(rp, ci)
    np.testing.assert_allclose(oracle.gcn_aggregate(rp, ci, H), A @ H, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.gcn_aggregate(rp, ci, G, transpose=True), A.T @ G, rtol=0, atol=1e-13)
    # <Ahat H, G> = <H, Ahat^T G>, also on a directed (non-symmetric) entry list
    rp_d = np.array([0, 2, 2, 3, 4], dtype=np.int32)
    ci_d = np.array([1, 3, 0, 2], dtype=np.int32)
    Hd, Gd = rng.standard_normal((4, 3)), rng.standard_normal((4, 3))
    lhs = (oracle.gcn_aggregate(rp_d, ci_d, Hd) * Gd).sum()
    rhs = (Hd * oracle.gcn_aggregate(rp_d, ci_d, Gd, transpose=True)).sum()
    assert lhs == pytest.approx(rhs, rel=1e-13)


@pytest.mark.parametrize("act", [oracle.ACT_NONE, oracle.ACT_RELU])
@pytest.mark.parametrize("bias", [True, False])
def test_dense_layer_against_library_autograd(act, bias):
    rng = np.random.default_rng(5)
    n, Fi, Fo = 37, 9, 6
    X, W, b, g = rng.standard_normal((n, Fi)), rng.standard_normal((Fi, Fo)), rng.standard_normal(Fo), rng.standard_normal((n, Fo))
    tX = torch.tensor(X, requires_grad=True)
    tW = torch.tensor(W, requires_grad=True)
    tb = torch.tensor(b, requires_grad=True)
    tz = tX @ tW + (tb if bias else 0.0)
    ty = torch.relu(tz) if act == oracle.ACT_RELU else tz
    ty.backward(torch.tensor(g))
    Z, Y = oracle.dense_fwd(X, W, b if bias else None, act)
    np.testing.assert_allclose(Z, tz.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Y, ty.detach().numpy(), rtol=1e-12, atol=1e-13)
    dW, db, dX = oracle.dense_bwd(X, Z, g, W, act, need_dbias=bias)
    np.testing.assert_allclose(dW, tW.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dX, tX.grad.numpy(), rtol=1e-11, atol=1e-12)
    if bias:
        np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-12)
    else:
        assert db is None


@pytest.mark.parametrize("act", [oracle.ACT_NONE, oracle.ACT_RELU])
def test_gcn_layer_against_library_autograd(act):
    rp, ci = _local_graph(300, 1100, 11)
    n = len(rp) - 1
    rng = np.random.default_rng(2)
    Fi, Fo = 7, 5
    H, W, b, g = rng.standard_normal((n, Fi)), rng.standard_normal((Fi, Fo)), rng.standard_normal(Fo), rng.standard_normal((n, Fo))
    A = torch.tensor(_ahat(rp, ci))
    tH = torch.tensor(H, requires_grad=True)
    tW = torch.tensor(W, requires_grad=True)
    tb = torch.tensor(b, requires_grad=True)
    tz = A @ tH @ tW + tb
    ty = torch.relu(tz) if act == oracle.ACT_RELU else tz
    ty.backward(torch.tensor(g))
    M, Z, Hn = oracle.gcn_layer_fwd(rp, ci, H, W, b, act)
    np.testing.assert_allclose(Hn, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    dW, db, dH = oracle.gcn_layer_bwd(rp, ci, M, Z, g, W, act)
    np.testing.assert_allclose(dW, tW.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dH, tH.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert oracle.gcn_layer_bwd(rp, ci, M, Z, g, W, act, need_dH=False)[2] is None


def test_gcn_layer_finite_differences():
    rp, ci = _local_graph(120, 400, 13)
    n = len(rp) - 1
    rng = np.random.default_rng(3)
    Fi, Fo = 4, 3
    H, W, b, g = rng.standard_normal((n, Fi)), rng.standard_normal((Fi, Fo)), rng.standard_normal(Fo), rng.standard_normal((n, Fo))

    def f(H_, W_, b_):
        return float((oracle.gcn_layer_fwd(rp, ci, H_, W_, b_, oracle.ACT_NONE)[2] * g).sum())

    M, Z, _ = oracle.gcn_layer_fwd(rp, ci, H, W, b, oracle.ACT_NONE)
    dW, db, dH = oracle.gcn_layer_bwd(rp, ci, M, Z, g, W, oracle.ACT_NONE)
    h = 1e-6
    for (i, j) in [(0, 0), (3, 2), (1, 1)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[i, j] += h
        Wm[i, j] -= h
        assert (f(H, Wp, b) - f(H, Wm, b)) / (2 * h) == pytest.approx(dW[i, j], rel=1e-6, abs=1e-8)
    for (v, k) in [(0, 0), (n // 2, 3), (n - 1, 1)]:
        Hp, Hm = H.copy(), H.copy()
        Hp[v, k] += h
        Hm[v, k] -= h
        assert (f(Hp, W, b) - f(Hm, W, b)) / (2 * h) == pytest.approx(dH[v, k], rel=1e-6, abs=1e-8)
    bp, bm = b.copy(), b.copy()
    bp[1] += h
    bm[1] -= h
    assert (f(H, W, bp) - f(H, W, bm)) / (2 * h) == pytest.approx(db[1], rel=1e-6, abs=1e-8)
