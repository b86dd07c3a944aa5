"""Pins for the oracle's GCN layer on a bipartite block of a sampled message-flow graph (Sec. 4.1: GCN trained with
the neighbour sampler), against things other than its own loops: a dense matrix Dt^-1 (A_S + I) assembled by a
library's sparse algebra, its row sums and special cases (rows without sampled neighbours, the uncut
neighbourhood, its relation to the plain mean), the adjoint identity, a library's reverse-mode derivative and
central finite differences of the whole sampled step."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")


def _local_graph(n, m, seed, K=2):
    rowptr, colidx = synth.uniform_graph(n, m, seed)
    part = oracle.partition(n, K, seed=seed)
    sub = oracle.induced_subgraph(rowptr, colidx, part, 0)
    return sub["rowptr"], sub["colidx"]


def _block(seed, fanout=3, n_dst=40):
    rp, ci = _local_graph(900, 4000, seed)
    rng = np.random.default_rng(seed)
    lone = np.flatnonzero(np.diff(rp) == 0)[:1]          # one node without neighbours is always asked
    others = rng.choice(np.setdiff1d(np.arange(len(rp) - 1), lone), n_dst - 1, replace=False)
    dst = rng.permutation(np.concatenate([lone, others])).astype(np.int32)
    brp, bcol = oracle.neighbor_sample(dst, rp, ci, fanout, seed=seed)
    src, cols = oracle.mfg_relabel(dst, bcol)
    return brp, cols, len(src), (rp, ci, dst, src)


def _phat(brp, cols, n_src):
    """Dt^-1 (A_S + [I 0]) as a dense [n_dst, n_src] matrix, through scipy."""
    n_dst = len(brp) - 1
    A = sp.csr_matrix((np.ones(len(cols)), cols, brp), shape=(n_dst, n_src))
    A = A + sp.eye(n_dst, n_src, format="csr")
    d = np.asarray(A.sum(1)).ravel()
    return (sp.diags(1.0 / d) @ A).toarray()


def test_aggregate_against_sparse_library_row_sums_and_adjoint():
    brp, cols, n_src, _ = _block(3)
    n_dst = len(brp) - 1
    assert n_src > n_dst and (np.diff(brp) == 0).any() and np.diff(brp).max() == 3
    rng = np.random.default_rng(0)
    H, G = rng.standard_normal((n_src, 5)), rng.standard_normal((n_dst, 5))
    P = _phat(brp, cols, n_src)
    np.testing.assert_allclose(P.sum(1), 1.0, rtol=1e-14)           # a mean: constants are reproduced
    M = oracle.gcn_block_aggregate(brp, cols, H)
    np.testing.assert_allclose(M, P @ H, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.gcn_block_aggregate(brp, cols, np.ones((n_src, 2))), 1.0, rtol=1e-14)
    T = oracle.gcn_block_aggregate(brp, cols, G, transpose=True, n_src=n_src)
    np.testing.assert_allclose(T, P.T @ G, rtol=1e-12, atol=1e-14)
    assert np.sum(M * G) == pytest.approx(np.sum(H * T), rel=1e-12)   # <P H, G> = <H, P^T G>


def test_special_cases():
    brp, cols, n_src, (rp, ci, dst, src) = _block(5)
    n_dst = len(brp) - 1
    H = np.random.default_rng(1).standard_normal((n_src, 4))
    M = oracle.gcn_block_aggregate(brp, cols, H)
    # a row without sampled neighbours keeps its own features
    lone = np.flatnonzero(np.diff(brp) == 0)
    assert len(lone) > 0
    np.testing.assert_array_equal(M[lone], H[lone])
    # relation to the plain mean over the same block: (h_v + d_v mean_v) / (d_v + 1)
    d = np.diff(brp)[:, None].astype(np.float64)
    np.testing.assert_allclose(M, (H[:n_dst] + d * oracle.mean_aggregate(brp, cols, H)) / (d + 1.0), rtol=1e-12, atol=1e-14)
    # nothing cut, every node asked: the random-walk normalisation of A + I on the whole local graph
    n = len(rp) - 1
    every = np.arange(n, dtype=np.int32)
    frp, fcol = oracle.neighbor_sample(every, rp, ci, 10**6, seed=2)
    fsrc, fcols = oracle.mfg_relabel(every, fcol)
    assert np.array_equal(fsrc, every) and np.array_equal(frp, rp)
    A = sp.csr_matrix((np.ones(len(ci)), ci, rp), shape=(n, n)) + sp.identity(n, format="csr")
    want = sp.diags(1.0 / np.asarray(A.sum(1)).ravel()) @ A
    X = np.random.default_rng(2).standard_normal((n, 3))
    np.testing.assert_allclose(oracle.gcn_block_aggregate(frp, fcols, X), want @ X, rtol=1e-12, atol=1e-14)
    # on a regular graph the row-normalised and the symmetric form coincide
    u = np.arange(12)
    crp, cci = synth.csr_from_pairs(12, u, (u + 1) % 12)
    Xc = np.random.default_rng(3).standard_normal((12, 3))
    np.testing.assert_allclose(oracle.gcn_block_aggregate(crp, cci, Xc), oracle.gcn_aggregate(crp, cci, Xc), rtol=1e-13)


@pytest.mark.parametrize("act", [oracle.ACT_NONE, oracle.ACT_RELU])
def test_block_layer_against_library_autograd(act):
    brp, cols, n_src, _ = _block(7, fanout=4)
    n_dst = len(brp) - 1
    rng = np.random.default_rng(4)
    H, W, b = rng.standard_normal((n_src, 6)), 0.5 * rng.standard_normal((6, 5)), 0.1 * rng.standard_normal(5)
    dHn = rng.standard_normal((n_dst, 5))
    M, Z, Hn = oracle.gcn_block_layer_fwd(brp, cols, H, W, b, act)
    dW, db, dH = oracle.gcn_block_layer_bwd(brp, cols, n_src, M, Z, dHn, W, act)
    P = torch.tensor(_phat(brp, cols, n_src))
    Ht, Wt, bt = (torch.tensor(a, requires_grad=True) for a in (H, W, b))
    Zt = P @ Ht @ Wt + bt
    out = torch.relu(Zt) if act == oracle.ACT_RELU else Zt
    out.backward(torch.tensor(dHn))
    np.testing.assert_allclose(Z, Zt.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Hn, out.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dH, Ht.grad.numpy(), rtol=1e-11, atol=1e-12)
    assert dH.shape == (n_src, 6) and np.abs(dH[n_dst:]).max() > 0
    assert oracle.gcn_block_layer_bwd(brp, cols, n_src, M, Z, dHn, W, act, need_dH=False)[2] is None


def _tiny_sampled_problem():
    rp, ci = _local_graph(300, 1200, 7)
    n = len(rp) - 1
    rng = np.random.default_rng(1)
    dims = [6, 8, 5]
    enc = [(0.5 * rng.standard_normal((a, b)), 0.1 * rng.standard_normal(b)) for a, b in zip(dims[:-1], dims[1:])]
    dec = [(0.5 * rng.standard_normal((5, 7)), np.array([0.25])), (0.5 * rng.standard_normal((7, 1)),)]
    X = rng.standard_normal((n, 6))
    batch = oracle.edge_batch(rp, ci, seed=9, first_counter=0, B=40)
    return rp, ci, X, batch, enc, dec


def test_sampled_gcn_step_finite_differences_and_blocks_shared_with_sage():
    rp, ci, X, batch, enc, dec = _tiny_sampled_problem()
    loss, g_enc, g_dec, _, mfg = omodel.sampled_link_loss_and_grads(rp, ci, X, batch, enc, dec, [3, 2], seed=3, step=0,
                                                                    encoder="gcn")
    # the sampler does not depend on the encoder: same blocks as the SAGE step draws
    sage = [(w, w, b) for w, b in enc]
    mfg_s = omodel.sampled_link_loss_and_grads(rp, ci, X, batch, sage, dec, [3, 2], seed=3, step=0)[4]
    for a, b in zip(mfg[0] + mfg[1] + [mfg[2], mfg[3]], mfg_s[0] + mfg_s[1] + [mfg_s[2], mfg_s[3]]):
        assert np.array_equal(a, b)
    rng = np.random.default_rng(5)

    def loss_at(enc_p, dec_p):
        return omodel.sampled_link_loss_and_grads(rp, ci, X, batch, enc_p, dec_p, [3, 2], seed=3, step=0, encoder="gcn")[0]

    h = 1e-6
    for l in range(2):
        for t in range(2):
            for _ in range(3):
                idx = tuple(rng.integers(0, s) for s in enc[l][t].shape)
                plus = [tuple(np.array(a, copy=True) for a in layer) for layer in enc]
                minus = [tuple(np.array(a, copy=True) for a in layer) for layer in enc]
                plus[l][t][idx] += h
                minus[l][t][idx] -= h
                fd = (loss_at(plus, dec) - loss_at(minus, dec)) / (2 * h)
                assert g_enc[l][t][idx] == pytest.approx(fd, rel=2e-5, abs=1e-8), (l, t, idx)
    assert len(g_enc[0]) == 2 and g_enc[0][0].shape == (6, 8) and len(g_dec) == 2


def test_sampled_gcn_step_with_nothing_cut_is_the_row_normalised_full_graph_step():
    """Fan-outs beyond every degree: the sampled step is the full-graph step of the same layer, evaluated on the
    nodes the batch reaches; compared with a dense library evaluation on the whole local graph."""
    rp, ci, X, batch, enc, dec = _tiny_sampled_problem()
    n = len(rp) - 1
    loss, _, _, z, _ = omodel.sampled_link_loss_and_grads(rp, ci, X, batch, enc, dec, [10**6, 10**6], seed=3, step=0,
                                                          encoder="gcn")
    A = sp.csr_matrix((np.ones(len(ci)), ci, rp), shape=(n, n)) + sp.identity(n, format="csr")
    P = (sp.diags(1.0 / np.asarray(A.sum(1)).ravel()) @ A).toarray()
    H1 = np.maximum(P @ X @ enc[0][0] + enc[0][1], 0.0)
    R = P @ H1 @ enc[1][0] + enc[1][1]
    u, v, vneg = batch
    E0 = np.concatenate([R[u] * R[v], R[u] * R[vneg]])
    Z1 = E0 @ dec[0][0]
    E1 = np.where(Z1 > 0, Z1, 0.25 * Z1)
    want_z = (E1 @ dec[1][0]).ravel()
    np.testing.assert_allclose(np.asarray(z).ravel(), want_z, rtol=1e-10, atol=1e-12)
