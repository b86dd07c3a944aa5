"""Pins for the oracle's aggregation, layer, loss, gradient and averaging code.

Each check compares against something other than the oracle's own loops: an
explicit dense row-normalised adjacency multiplied with numpy, hand-computable
graphs, the expected neighbour mean and the closed-form initial gradient from
the proof of Thm. 1, central finite differences, the adjoint identity.
"""
import numpy as np
import pytest

import oracle
from oracle import model
from paper_2305_09887_amd import synth


def _dense_abar(rowptr, colidx):
    n = len(rowptr) - 1
    A = np.zeros((n, n))
    for v in range(n):
        for e in range(rowptr[v], rowptr[v + 1]):
            A[v, colidx[e]] += 1.0
    deg = A.sum(1, keepdims=True)
    return np.divide(A, deg, out=np.zeros_like(A), where=deg > 0)


def _local_graph(n, m, seed, K=2):
    rowptr, colidx = synth.uniform_graph(n, m, seed)
    part = oracle.partition(n, K, seed=seed)
    sub = oracle.induced_subgraph(rowptr, colidx, part, 0)
    return sub["rowptr"], sub["colidx"]


def test_mean_aggregate_dense_brute_force():
    rp, ci = _local_graph(400, 1500, 3)
    n = len(rp) - 1
    assert (np.diff(rp) == 0).any()          # isolated local nodes are present in the case
    H = np.random.default_rng(0).standard_normal((n, 7))
    Abar = _dense_abar(rp, ci)
    assert np.allclose(oracle.mean_aggregate(rp, ci, H), Abar @ H, rtol=0, atol=1e-13)
    assert np.allclose(oracle.mean_aggregate_T(rp, ci, H), Abar.T @ H, rtol=0, atol=1e-13)


def test_mean_aggregate_ones_star_and_path():
    rp, ci = _local_graph(300, 900, 5)
    n = len(rp) - 1
    out = oracle.mean_aggregate(rp, ci, np.ones((n, 3)))
    deg = np.diff(rp)
    assert np.array_equal(out, np.repeat((deg > 0).astype(float)[:, None], 3, 1))
    # star: centre 0 with leaves 1..4 ; features = node id
    rp_s, ci_s = synth.csr_from_pairs(5, [0, 0, 0, 0], [1, 2, 3, 4])
    x = np.arange(5, dtype=float)[:, None]
    assert np.allclose(oracle.mean_aggregate(rp_s.astype(np.int32), ci_s, x).ravel(), [2.5, 0, 0, 0, 0])
    # path 0-1-2-3
    rp_p, ci_p = synth.csr_from_pairs(4, [0, 1, 2], [1, 2, 3])
    assert np.allclose(oracle.mean_aggregate(rp_p.astype(np.int32), ci_p, x[:4]).ravel(), [1, 1, 2, 2])
    # transposed on the star: leaf i receives G_0/4, centre receives sum of leaf G (each leaf has degree 1)
    g = np.array([8.0, 1, 2, 3, 4])[:, None]
    assert np.allclose(oracle.mean_aggregate_T(rp_s.astype(np.int32), ci_s, g).ravel(), [10, 2, 2, 2, 2])


def test_adjoint_identity_on_asymmetric_csr():
    # a CSR that is NOT symmetric: the transposed operator must still be the adjoint
    rng = np.random.default_rng(1)
    n = 200
    deg = rng.integers(0, 6, n)
    rp = np.zeros(n + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    ci = rng.integers(0, n, rp[-1]).astype(np.int32)
    H, G = rng.standard_normal((n, 5)), rng.standard_normal((n, 5))
    lhs = (oracle.mean_aggregate(rp, ci, H) * G).sum()
    rhs = (H * oracle.mean_aggregate_T(rp, ci, G)).sum()
    assert lhs == pytest.approx(rhs, rel=1e-12)


def test_expected_neighbour_mean_of_thm1_proof():
    """One-hot features on the two-class graph: E[(Abar X)_v | y_v=1] = [1-h, h]
    globally, and [(1-h)b, h(1-b)] / ((1-h)b + h(1-b)) inside a part with class-0 share b."""
    h = 0.8
    n = 40_000
    rowptr, colidx, y = synth.two_class_graph(n, 30, h, seed=2)
    X = np.eye(2)[y]
    rp32 = rowptr.astype(np.int32)
    agg = oracle.mean_aggregate(rp32, colidx, X)
    has = np.diff(rowptr) > 0
    got = agg[(y == 1) & has].mean(0)
    assert np.allclose(got, [1 - h, h], atol=0.01)
    # a partition with class mix beta: put a fraction beta of class 0 and 1-beta of class 1 in part 0
    beta = 0.7
    rng = np.random.default_rng(3)
    part = np.where(y == 0, rng.random(n) >= beta, rng.random(n) < beta).astype(np.int32)
    sub = oracle.induced_subgraph(rowptr, colidx, part, 0)
    yl = y[sub["l2g"]]
    b = float((yl == 0).mean())
    agg = oracle.mean_aggregate(sub["rowptr"], sub["colidx"], np.eye(2)[yl])
    has = np.diff(sub["rowptr"]) > 0
    got = agg[(yl == 1) & has].mean(0)
    want = np.array([(1 - h) * b, h * (1 - b)]) / ((1 - h) * b + h * (1 - b))
    assert np.allclose(got, want, atol=0.015)


def test_closed_form_initial_gradient_of_thm1():
    """z = sigmoid(Abar X W), L2 loss, W = 0:  dL/dW[:, c] = sum_v (1/2 - Y_vc) * 1/4 * (Abar X)_v,
    i.e. -1/8 (Abar X)_v for a node of the positive class (proof of Thm. 1)."""
    rp, ci = _local_graph(500, 2500, 9)
    n = len(rp) - 1
    rng = np.random.default_rng(4)
    X = rng.standard_normal((n, 6))
    Y = (rng.random((n, 1)) < 0.5).astype(float)
    W0 = np.zeros((6, 1))
    M, Z, _ = oracle.sage_layer_fwd(rp, ci, X, np.zeros((6, 1)), W0, np.zeros(1), oracle.ACT_NONE)
    loss, dZ = oracle.sigmoid_l2(Z, Y)
    assert loss == pytest.approx(0.125 * n)                      # (1/2)(1/2)^2 per node
    dWs, dWn, db, _ = oracle.sage_layer_bwd(rp, ci, X, M, Z, dZ, np.zeros((6, 1)), W0,
                                            oracle.ACT_NONE, need_dH=False)
    AX = _dense_abar(rp, ci) @ X
    want = ((0.5 - Y) * 0.25 * AX).sum(0)[:, None]
    assert np.allclose(dWn, want, rtol=1e-12, atol=1e-13)
    one = np.flatnonzero(Y.ravel() == 1)[0]
    # single positive node alone: gradient is exactly -1/8 of its aggregated feature
    Zs = Z.copy()
    _, d1 = oracle.sigmoid_l2(Zs[one:one + 1], Y[one:one + 1])
    assert d1.ravel()[0] == pytest.approx(-0.125)


def test_layer_forward_against_numpy_matmul():
    rp, ci = _local_graph(300, 1200, 12)
    n = len(rp) - 1
    rng = np.random.default_rng(5)
    H = rng.standard_normal((n, 9))
    Ws, Wn, b = rng.standard_normal((9, 4)), rng.standard_normal((9, 4)), rng.standard_normal(4)
    M, Z, Hn = oracle.sage_layer_fwd(rp, ci, H, Ws, Wn, b, oracle.ACT_RELU)
    Abar = _dense_abar(rp, ci)
    assert np.allclose(M, Abar @ H, atol=1e-13)
    assert np.allclose(Z, H @ Ws + (Abar @ H) @ Wn + b, atol=1e-12)
    assert np.array_equal(Hn, np.maximum(Z, 0))
    # transposed-operand mistake would show here: W is [F_in, F_out], not square
    _, Z2, Hn2 = oracle.sage_layer_fwd(rp, ci, H, Ws, Wn, b, oracle.ACT_NONE)
    assert np.array_equal(Z2, Hn2)


def test_softmax_ce_against_textbook_values():
    # uniform logits: loss = log C, gradient = (1/C - onehot)/n
    n, C = 5, 4
    y = np.array([0, 1, 2, 3, 0], dtype=np.int32)
    loss, d = oracle.softmax_ce(np.zeros((n, C)), y)
    assert loss == pytest.approx(np.log(C))
    assert np.allclose(d, (np.full((n, C), 1 / C) - np.eye(C)[y]) / n)
    # shift invariance and a 2-class closed form: CE = log(1+exp(-(z1-z0))) for label 1
    z = np.array([[0.3, 1.7]])
    loss, _ = oracle.softmax_ce(z + 1000.0, np.array([1], dtype=np.int32))
    assert loss == pytest.approx(np.log1p(np.exp(-1.4)))


def _fd_check(loss_fn, params, eps=1e-6):
    """Central differences on every parameter entry (tiny model)."""
    grads = []
    for li, layer in enumerate(params):
        gl = []
        for ti, t in enumerate(layer):
            g = np.zeros_like(t, dtype=np.float64)
            it = np.nditer(t, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                def shifted(delta):
                    p2 = [tuple(np.array(a, dtype=np.float64) for a in l) for l in params]
                    p2[li][ti][idx] += delta
                    return loss_fn(p2)
                g[idx] = (shifted(eps) - shifted(-eps)) / (2 * eps)
            gl.append(g)
        grads.append(tuple(gl))
    return grads


@pytest.mark.parametrize("n_layers", [1, 2, 3])
def test_gradients_against_finite_differences(n_layers):
    rp, ci = _local_graph(60, 260, 20 + n_layers)
    n = len(rp) - 1
    rng = np.random.default_rng(6)
    dims = [5, 4, 3, 3][: n_layers] + [3]
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, 3, n).astype(np.int32)
    params = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in synth.sage_params(dims, 8)]
    loss, grads, _, _ = model.loss_and_grads(rp, ci, X, y, params)

    def loss_fn(p):
        logits, _ = model.forward(rp, ci, X, p)
        return oracle.softmax_ce(logits, y, need_grad=False)[0]

    fd = _fd_check(loss_fn, params)
    for gl, fl in zip(grads, fd):
        for g, f in zip(gl, fl):
            assert np.allclose(g, f, rtol=1e-6, atol=1e-9)


def test_input_gradient_against_finite_differences():
    # dH of a layer (the part that needs the transposed aggregation), on an asymmetric CSR
    rng = np.random.default_rng(7)
    n = 40
    deg = rng.integers(0, 4, n)
    rp = np.zeros(n + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    ci = rng.integers(0, n, rp[-1]).astype(np.int32)
    H = rng.standard_normal((n, 3))
    Ws, Wn, b = rng.standard_normal((3, 2)), rng.standard_normal((3, 2)), rng.standard_normal(2)
    R = rng.standard_normal((n, 2))

    def f(Hx):
        return float((oracle.sage_layer_fwd(rp, ci, Hx, Ws, Wn, b, oracle.ACT_RELU)[2] * R).sum())

    M, Z, _ = oracle.sage_layer_fwd(rp, ci, H, Ws, Wn, b, oracle.ACT_RELU)
    dH = oracle.sage_layer_bwd(rp, ci, H, M, Z, R, Ws, Wn, oracle.ACT_RELU)[3]
    fd = np.zeros_like(H)
    for i in range(n):
        for k in range(3):
            Hp, Hm = H.copy(), H.copy()
            Hp[i, k] += 1e-6
            Hm[i, k] -= 1e-6
            fd[i, k] = (f(Hp) - f(Hm)) / 2e-6
    assert np.allclose(dH, fd, rtol=1e-6, atol=1e-8)


def test_sgd_and_average_closed_forms():
    rng = np.random.default_rng(8)
    W, g = rng.standard_normal(11), rng.standard_normal(11)
    assert np.allclose(oracle.sgd_step(W, g, 1e-3), W - 1e-3 * g, rtol=0, atol=1e-16)
    S = rng.standard_normal((5, 13))
    after, wg = oracle.average(S)
    assert np.allclose(wg, S.mean(0), atol=1e-15)
    assert all(np.array_equal(after[i], after[0]) for i in range(5))
    # equal inputs stay put; M = 1 is the identity
    same = np.repeat(S[:1], 4, 0)
    assert np.allclose(oracle.average(same)[0], same, atol=1e-16)
    assert np.array_equal(oracle.average(S[:1])[0], S[:1])
    # failed trainer (bit 2 cleared): mean over the remaining ones, its buffer untouched
    after, wg = oracle.average(S, active_mask=0b11011)
    assert np.allclose(wg, S[[0, 1, 3, 4]].mean(0), atol=1e-15)
    assert np.array_equal(after[2], S[2])
    assert np.array_equal(after[0], after[4])


def test_random_assignment_gives_similar_trainers():
    """Corollary: with i.i.d. random assignment the trainers' initial losses and gradients
    agree in expectation; with a class-sorted assignment (beta -> 1) they do not."""
    h = 0.8
    rowptr, colidx, y = synth.two_class_graph(20_000, 30, h, seed=4)
    X = np.eye(2)[y]
    W = np.array([[0.7], [-0.4]])

    def local_loss_grad(part, p):
        sub = oracle.induced_subgraph(rowptr, colidx, part, p)
        yl = y[sub["l2g"]]
        keep = yl == 1
        M, Z, _ = oracle.sage_layer_fwd(sub["rowptr"], sub["colidx"], X[sub["l2g"]],
                                        np.zeros((2, 1)), W, np.zeros(1), oracle.ACT_NONE)
        Y = yl[:, None].astype(float)
        nz = np.diff(sub["rowptr"]) > 0
        sel = keep & nz
        loss, dZ = oracle.sigmoid_l2(Z[sel], Y[sel])
        return loss / sel.sum(), (M[sel] * dZ).sum(0) / sel.sum()

    rnd = oracle.partition(20_000, 2, seed=1)
    l0, g0 = local_loss_grad(rnd, 0)
    l1, g1 = local_loss_grad(rnd, 1)
    assert abs(l0 - l1) < 0.03 * l0 and np.linalg.norm(g0 - g1) < 0.08 * np.linalg.norm(g0)
    rng = np.random.default_rng(0)
    beta = 0.9
    srt = np.where(y == 0, rng.random(20_000) >= beta, rng.random(20_000) < beta).astype(np.int32)
    l0, g0 = local_loss_grad(srt, 0)
    l1, g1 = local_loss_grad(srt, 1)
    assert abs(l0 - l1) > 0.10 * l0


def test_tma_schedule_timeline():
    # equal trainers, step 1.0, interval 10: every trainer joins after exactly 10 steps per round
    rounds, final = model.tma_schedule(lambda i, k: 1.0, 3, dt_int=10.0, dt_train=35.0)
    assert rounds == [[10] * 3, [20] * 3, [30] * 3]
    assert final == [36] * 3
    # a slow trainer (1.4x) finishes fewer steps; the fast ones wait for it at each round
    rounds, _ = model.tma_schedule(lambda i, k: 1.4 if i == 2 else 1.0, 3, dt_int=10.5, dt_train=25.0)
    # first aggregation: flag at 10.5; fast cross it after 11 steps (t=11.0), slow after 8 (t=11.2)
    # the second interval starts at 11.2: flag at 21.7; fast need 11 more (22.2), slow 8 more (22.4)
    assert rounds == [[11, 11, 8], [22, 22, 16]]
