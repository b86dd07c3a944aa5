"""The paper's other encoders (Sec. 4.1) on the GPU against the fp64 oracle, through the C ABI: the dense
(MLP) layer and the GCN layer, forward and backward, fp32 to 1e-4 and bf16 storage to 2e-2.  The ReLU decision
is taken in the kernel's precision on both sides (from the kernel's own output), as for the SAGE layer."""
import numpy as np
import pytest

import decisions
import oracle
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_09887_amd import binding
    binding.lib()
    return binding


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    return (t if dtype is None else t.to(dtype)).cuda()


def dev_bf16(a):
    bits = synth.to_bf16_bits(np.asarray(a, dtype=np.float32)).reshape(np.shape(a))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def close(got, want, tol, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, what
    rel = np.linalg.norm((got - want).ravel()) / max(np.linalg.norm(want.ravel()), 1e-300)
    mx = np.abs(got - want).max() / max(np.abs(want).max(), 1e-300)
    assert rel <= tol and mx <= tol, f"{what}: rel fro {rel:.2e}, max abs / max {mx:.2e}"


def padded(B, a, bf16=False):
    a = np.asarray(a, dtype=np.float32)
    t = B._padded(a.shape[0], a.shape[1], torch.bfloat16 if bf16 else torch.float32, "cuda")
    t.copy_(dev_bf16(a) if bf16 else dev(a))
    return t


def local_graph(n_glob, m, seed, K=2, kind="uniform"):
    if kind == "uniform":
        rowptr, colidx = synth.uniform_graph(n_glob, m, seed)
    else:
        rowptr, colidx = synth.chung_lu_graph(n_glob, 2.0 * m / n_glob, 2.1, seed)
    part = oracle.partition(n_glob, K, seed=seed)
    sub = oracle.induced_subgraph(rowptr, colidx, part, 0)
    return sub["rowptr"], sub["colidx"]


def _layer_inputs(n, Fi, Fo, seed):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((n, Fi)).astype(np.float32)
    W = synth.glorot(Fi, Fo, rng).astype(np.float32)
    b = (0.1 * rng.standard_normal(Fo)).astype(np.float32)
    g = (rng.standard_normal((n, Fo)) / max(n, 1)).astype(np.float32)
    return H, W, b, g


DENSE_SHAPES = [(1, 8, 8), (3000, 64, 256), (2501, 256, 47), (1000, 100, 64), (777, 47, 33), (4100, 128, 128),
                (1500, 256, 1), (900, 300, 96), (640, 512, 80)]


@pytest.mark.parametrize("n,Fi,Fo", DENSE_SHAPES)
@pytest.mark.parametrize("act", [0, 1])
def test_dense_layer_fp32(B, n, Fi, Fo, act):
    X, W, b, g = _layer_inputs(n, Fi, Fo, seed=Fi + Fo)
    Xd, gd = padded(B, X), padded(B, g)
    Y = B.tma_dense_fwd(Xd, dev(W), dev(b), act)
    Z, want = oracle.dense_fwd(X, W, b, act)
    close(host(Y), want, 1e-4, "Y")
    # backward from the ORACLE's forward output on both sides (its sign pattern is the ReLU decision)
    Yo = padded(B, want)
    dW, db, dX = B.tma_dense_bwd(Xd, Yo, gd, dev(W), act)
    wW, wb, wX = oracle.dense_bwd(X, Z, g, W, act)
    close(host(dW), wW, 1e-4, "dW")
    close(host(db), wb, 1e-4, "db")
    close(host(dX), wX, 1e-4, "dX")
    # no bias, no input gradient (a decoder layer's first use; the first layer of an encoder)
    Y0 = B.tma_dense_fwd(Xd, dev(W), None, act)
    close(host(Y0), oracle.dense_fwd(X, W, None, act)[1], 1e-4, "Y without bias")
    dW0, db0, dX0 = B.tma_dense_bwd(Xd, Yo, gd, dev(W), act, need_dbias=False, need_dX=False)
    assert db0 is None and dX0 is None and torch.equal(dW0, dW)


@pytest.mark.parametrize("n,Fi,Fo", [(3000, 64, 256), (2501, 256, 47), (4100, 128, 128), (1000, 100, 64)])
def test_dense_layer_bf16(B, n, Fi, Fo):
    X, W, b, g = _layer_inputs(n, Fi, Fo, seed=Fi * 3 + Fo)
    X, g = synth.round_bf16(X), synth.round_bf16(g)
    Xd, gd = padded(B, X, True), padded(B, g, True)
    Y = B.tma_dense_fwd(Xd, dev(W), dev(b), 1)
    Z, want = oracle.dense_fwd(X, W, b, 1)
    close(host(Y), want, 2e-2, "Y")
    dW, db, dX = B.tma_dense_bwd(Xd, padded(B, want, True), gd, dev(W), 1)     # the oracle's output decides the ReLU
    wW, wb, wX = oracle.dense_bwd(X, Z, g, W, 1)
    close(host(dW), wW, 2e-2, "dW")
    close(host(db), wb, 2e-2, "db")
    close(host(dX), wX, 2e-2, "dX")


def test_dense_layer_empty_and_unaligned(B):
    W = dev(np.ones((8, 4), np.float32))
    X0 = torch.empty((0, 8), device="cuda")
    assert B.tma_dense_fwd(X0, W, None, 0).shape == (0, 4)
    dW, db, dX = B.tma_dense_bwd(X0, None, torch.empty((0, 4), device="cuda"), W, 0)
    assert not dW.any() and not db.any() and dX.shape == (0, 8)
    # rows with a leading dimension that is no multiple of 16 bytes take the element-wise path
    n, Fi, Fo = 1234, 100, 47
    X, Wn, b, g = _layer_inputs(n, Fi, Fo, seed=9)
    big = torch.zeros((n, Fi + 3), device="cuda")
    big[:, :Fi] = dev(X)
    Xd = big[:, :Fi]
    Y = B.tma_dense_fwd(Xd, dev(Wn), dev(b), 0)
    close(host(Y), oracle.dense_fwd(X, Wn, b, 0)[1], 1e-4, "Y (unaligned)")
    gbig = torch.zeros((n, Fo + 2), device="cuda")
    gbig[:, :Fo] = dev(g)
    dW, db, dX = B.tma_dense_bwd(Xd, None, gbig[:, :Fo], dev(Wn), 0)
    wW, wb, wX = oracle.dense_bwd(X, oracle.dense_fwd(X, Wn, b, 0)[0], g, Wn, 0)
    close(host(dW), wW, 1e-4, "dW (unaligned)")
    close(host(db), wb, 1e-4, "db (unaligned)")
    close(host(dX), wX, 1e-4, "dX (unaligned)")


def test_gcn_norm(B):
    rp, _ = local_graph(20_000, 100_000, 1)
    s = B.tma_gcn_norm(dev(rp))
    np.testing.assert_allclose(host(s), oracle.gcn_norm(rp), rtol=2e-7)
    assert B.tma_gcn_norm(dev(np.zeros(1, np.int32))).numel() == 0


GCN_SHAPES = [(64, 256), (256, 256), (256, 47), (128, 64), (100, 100), (47, 33), (300, 16), (8, 512), (128, 1)]


@pytest.mark.parametrize("Fi,Fo", GCN_SHAPES)
@pytest.mark.parametrize("act", [0, 1])
def test_gcn_layer_fp32(B, Fi, Fo, act):
    rp, ci = local_graph(12_000, 60_000, Fi + Fo, kind="chung_lu" if Fi % 2 else "uniform")
    n = len(rp) - 1
    assert (np.diff(rp) == 0).any()
    H, W, b, g = _layer_inputs(n, Fi, Fo, seed=Fi * 7 + Fo)
    rpd, cid = dev(rp), dev(ci)
    s = B.tma_gcn_norm(rpd)
    Hd, gd = padded(B, H), padded(B, g)
    Mg, Hn = B.tma_gcn_layer_fwd(rpd, cid, s, Hd, dev(W), dev(b), act)
    M, Z, want = oracle.gcn_layer_fwd(rp, ci, H, W, b, act)
    close(host(Hn), want, 1e-4, "Hnext")
    if B.tma_gcn_layer_aggregates_first(Fi, Fo, B.TMA_F32):
        close(host(Mg), M, 1e-4, "M = Ahat H")
    # backward from the ORACLE's saved state on both sides: its M = Ahat H and its output (whose sign pattern is the
    # ReLU decision), so nothing the forward kernel produced reaches the expected values
    Mo, Ho = dev(M.astype(np.float32)), padded(B, want)
    dW, db, dH = B.tma_gcn_layer_bwd(rpd, cid, s, Hd, Mo, Ho, gd, dev(W), act)
    wW, wb, wH = oracle.gcn_layer_bwd(rp, ci, M, Z, g, W, act)
    close(host(dW), wW, 1e-4, "dW")
    close(host(db), wb, 1e-4, "db")
    close(host(dH), wH, 1e-4, "dH")
    dW2, db2, dH2 = B.tma_gcn_layer_bwd(rpd, cid, s, Hd, Mo, Ho, gd, dev(W), act, need_dH=False)
    assert dH2 is None and torch.equal(dW2, dW) and torch.equal(db2, db)     # run to run: the same bits


@pytest.mark.parametrize("Fi,Fo", [(64, 256), (256, 256), (256, 47), (128, 64), (100, 100)])
def test_gcn_layer_bf16(B, Fi, Fo):
    rp, ci = local_graph(12_000, 60_000, Fi + Fo + 1, kind="chung_lu")
    n = len(rp) - 1
    H, W, b, g = _layer_inputs(n, Fi, Fo, seed=Fi * 5 + Fo)
    H, g = synth.round_bf16(H), synth.round_bf16(g)
    rpd, cid = dev(rp), dev(ci)
    s = B.tma_gcn_norm(rpd)
    Hd, gd = padded(B, H, True), padded(B, g, True)
    Mg, Hn = B.tma_gcn_layer_fwd(rpd, cid, s, Hd, dev(W), dev(b), 1)
    M, Z, want = oracle.gcn_layer_fwd(rp, ci, H, W, b, 1)
    close(host(Hn), want, 2e-2, "Hnext")
    Mo = dev_bf16(M.astype(np.float32)).contiguous()
    dW, db, dH = B.tma_gcn_layer_bwd(rpd, cid, s, Hd, Mo, padded(B, want, True), gd, dev(W), 1)
    wW, wb, wH = oracle.gcn_layer_bwd(rp, ci, M, Z, g, W, 1)
    close(host(dW), wW, 2e-2, "dW")
    close(host(db), wb, 2e-2, "db")
    close(host(dH), wH, 2e-2, "dH")


def test_gcn_layer_directed_entries_and_empty(B):
    # a non-symmetric entry list: the backward takes the transposed CSR
    _directed_case(B, 32, 24)      # transforms first
    _directed_case(B, 24, 40)      # aggregates first
    W, b = dev(np.ones((32, 24), np.float32)), dev(np.zeros(24, np.float32))
    Fi, Fo = 32, 24
    # no nodes at all
    rp0 = dev(np.zeros(1, np.int32))
    ci0 = torch.empty(0, dtype=torch.int32, device="cuda")
    s0 = torch.empty(0, device="cuda")
    H0 = torch.empty((0, Fi), device="cuda")
    assert B.tma_gcn_layer_fwd(rp0, ci0, s0, H0, W, b, 1)[1].shape == (0, Fo)
    dW, db, dH = B.tma_gcn_layer_bwd(rp0, ci0, s0, H0, H0, torch.empty((0, Fo), device="cuda"),
                                     torch.empty((0, Fo), device="cuda"), W, 1)
    assert not dW.any() and not db.any() and dH.shape == (0, Fi)


def _directed_case(B, Fi, Fo):
    rng = np.random.default_rng(4)
    n, nnz = 3000, 9000
    u, v = rng.integers(0, n, nnz), rng.integers(0, n, nnz)
    order = np.lexsort((v, u))
    rp = np.zeros(n + 1, np.int32)
    np.add.at(rp, u + 1, 1)
    rp = np.cumsum(rp).astype(np.int32)
    ci = v[order].astype(np.int32)
    order_t = np.lexsort((u, v))
    rpt = np.zeros(n + 1, np.int32)
    np.add.at(rpt, v + 1, 1)
    rpt = np.cumsum(rpt).astype(np.int32)
    cit = u[order_t].astype(np.int32)
    H, W, b, g = _layer_inputs(n, Fi, Fo, seed=2)
    s = B.tma_gcn_norm(dev(rp))
    Hd, gd = padded(B, H), padded(B, g)
    Mg, Hn = B.tma_gcn_layer_fwd(dev(rp), dev(ci), s, Hd, dev(W), dev(b), 0)
    M, Z, want = oracle.gcn_layer_fwd(rp, ci, H, W, b, 0)
    close(host(Hn), want, 1e-4, "Hnext (directed)")
    dW, db, dH = B.tma_gcn_layer_bwd(dev(rpt), dev(cit), s, Hd, Mg, None, gd, dev(W), 0)
    wW, wb, wH = oracle.gcn_layer_bwd(rp, ci, M, Z, g, W, 0)
    close(host(dW), wW, 1e-4, "dW (directed)")
    close(host(dH), wH, 1e-4, "dH (directed)")
    close(host(db), wb, 1e-4, "db (directed)")


def test_row_padding_is_never_multiplied(B):
    """Rows padded to 16 bytes may hold anything (NaN here) in the padding: a reduction length that is no
    multiple of the k-slab must not pull it into the products (0 * NaN would poison the row)."""
    rp, ci = local_graph(6000, 30_000, 77)
    n = len(rp) - 1
    Fi, Fo = 100, 16                       # bf16 rows of 100 are padded to 104; 100 is no multiple of 32
    H, W, b, g = _layer_inputs(n, Fi, Fo, seed=5)
    H = synth.round_bf16(H)
    buf = torch.full((n, 104), float("nan"), dtype=torch.bfloat16, device="cuda")
    buf[:, :Fi] = dev_bf16(H)
    Hd = buf[:, :Fi]
    Y = B.tma_dense_fwd(Hd, dev(W), dev(b), 0)
    close(host(Y), oracle.dense_fwd(H, W, b, 0)[1], 2e-2, "dense Y")
    # the SAGE layer in its transform-first form runs the same kind of product
    rng = np.random.default_rng(1)
    Wn = synth.glorot(Fi, Fo, rng).astype(np.float32)
    inv = dev((1.0 / np.maximum(np.diff(rp), 1) * (np.diff(rp) > 0)).astype(np.float32))
    assert not B.lib().tma_sage_layer_aggregates_first(Fi, Fo, B.TMA_BF16)
    _, Hn = B.tma_sage_layer_fwd(dev(rp), dev(ci), inv, Hd, dev(W), dev(Wn), dev(b), 0)
    want = oracle.sage_layer_fwd(rp, ci, H, W, Wn, b, 0)[2]
    close(host(Hn), want, 2e-2, "SAGE Hnext")
    s = B.tma_gcn_norm(dev(rp))
    Hg = B.tma_gcn_layer_fwd(dev(rp), dev(ci), s, Hd, dev(W), dev(b), 0)[1]
    close(host(Hg), oracle.gcn_layer_fwd(rp, ci, H, W, b, 0)[2], 2e-2, "GCN Hnext")


@pytest.mark.parametrize("Fi,Fo", [(64, 13), (256, 47), (32, 6), (96, 3)])
def test_weights_with_ragged_rows_end_where_the_matrix_ends(B, Fi, Fo):
    """Weight rows that are no multiple of four elements are read in 16-byte groups from 4-byte-aligned addresses,
    and the group that would run past the end of the matrix is fetched earlier and moved back in registers.
    Whatever follows (or precedes) the matrix in memory, NaN here, must not reach a product: forward and input
    gradient of the transform-first SAGE layer, forward of the dense layer."""
    rp, ci = local_graph(5000, 25_000, 31)
    n = len(rp) - 1
    H, Ws, b, g = _layer_inputs(n, Fi, Fo, seed=9)
    Wn = synth.glorot(Fi, Fo, np.random.default_rng(2)).astype(np.float32)

    def carved(W):      # the matrix at an address that is only 4-byte aligned, NaN on both sides
        buf = torch.full((Fi * Fo + 16,), float("nan"), dtype=torch.float32, device="cuda")
        view = buf[5:5 + Fi * Fo].view(Fi, Fo)
        view.copy_(dev(W))
        return view

    dWs, dWn = carved(Ws), carved(Wn)
    Hd = padded(B, H)
    assert not B.lib().tma_sage_layer_aggregates_first(Fi, Fo, B.TMA_F32)
    inv = dev((1.0 / np.maximum(np.diff(rp), 1) * (np.diff(rp) > 0)).astype(np.float32))
    _, Hn = B.tma_sage_layer_fwd(dev(rp), dev(ci), inv, Hd, dWs, dWn, dev(b), 1)
    M_o, Z_o, Hn_o = oracle.sage_layer_fwd(rp, ci, H, Ws, Wn, b, 1)
    close(host(Hn), Hn_o, 1e-4, "SAGE Hnext")
    Hn32 = Hn_o.astype(np.float32)
    want = oracle.sage_layer_bwd(rp, ci, H, M_o.astype(np.float32), Hn32, g, Ws, Wn, 1)
    got = B.tma_sage_layer_bwd(dev(rp), dev(ci), inv, Hd, padded(B, M_o), padded(B, Hn32), padded(B, g), dWs, dWn, 1)
    for a, w, name in zip(got, want, ("dW_self", "dW_neigh", "dbias", "dH")):
        close(host(a), w, 1e-4, name)
    Y = B.tma_dense_fwd(Hd, dWs, dev(b), 0)
    close(host(Y), oracle.dense_fwd(H, Ws, b, 0)[1], 1e-4, "dense Y")


@pytest.mark.parametrize("encoder", ["gcn", "mlp"])
@pytest.mark.parametrize("norm_act", [False, True])
@pytest.mark.parametrize("optimizer", ["sgd", "adam"])
def test_training_steps_with_other_encoders(B, encoder, norm_act, optimizer):
    """Three steps of a 3-layer model (64-96-64-16) on the tiny configuration's part 0: losses, every gradient
    and the weights after each step against the oracle's trainer."""
    from oracle import model as omodel
    from paper_2305_09887_amd.trainer import LocalTrainer
    N, K, dims = 20_000, 4, [64, 96, 64, 16]
    rowptr, colidx = synth.uniform_graph(N, 100_000, seed=1)
    X, y = synth.features(N, dims[0], seed=2), synth.labels(N, dims[-1], seed=3)
    rng = np.random.default_rng(7)
    params = []
    for l, (Ws, _, b) in enumerate(synth.sage_params(dims, seed=5)):
        layer = [Ws, b]
        if norm_act and l < len(dims) - 2:
            layer += [rng.normal(1.0, 0.1, dims[l + 1]).astype(np.float32),
                      rng.normal(0.0, 0.1, dims[l + 1]).astype(np.float32), np.array([0.25], dtype=np.float32)]
        params.append(tuple(layer))
    sub = oracle.induced_subgraph(rowptr, colidx, oracle.partition(N, K, seed=4), 0)
    Xo, yo = X[sub["l2g"]], y[sub["l2g"]]
    tr = LocalTrainer(dev(sub["rowptr"]), dev(sub["colidx"]), dev(sub["inv_deg"], torch.float32), dev(Xo), dev(yo),
                      dims, params=params, norm_act=norm_act, optimizer=optimizer, encoder=encoder)
    p_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in params]
    assert tr.n_params == omodel.flatten(p_o).size
    lr = 0.05 if optimizer == "sgd" else 0.01
    state, losses = None, []
    rp, ci = sub["rowptr"], sub["colidx"]
    for step in range(3):
        loss_g = tr.step(lr).item()
        t = {}
        if optimizer == "sgd":
            loss_o, p_new = omodel.train_step(rp, ci, Xo, yo, p_o, lr, encoder=encoder, trace=t)
            grads_o = t["grads"]
        else:
            loss_o, grads_o, _, _ = omodel.loss_and_grads(rp, ci, Xo, yo, p_o, encoder=encoder, trace=t)
            _, p_new, state = omodel.train_step_adam(rp, ci, Xo, yo, p_o, lr, state, step + 1, encoder=encoder)
        D = decisions.differing(t["pre"], [host(tr.H[1]), host(tr.H[2]), None], f"step {step}")
        bounds = decisions.encoder_bounds(encoder, rp, ci, p_o, t["saved"], t["ups"], D)
        assert abs(loss_g - loss_o) <= 1e-4 * abs(loss_o), f"loss at step {step}"
        for l in range(3):
            for i, (g, w, bd) in enumerate(zip(tr.grads[l], grads_o[l], bounds[l])):
                decisions.close(host(g).ravel(), np.asarray(w).ravel(), 1e-4, f"step {step} layer {l} gradient {i}",
                                extra=bd)
        p_o = p_new
        if decisions.any_differs(D):     # a decision next to zero fell the other way: go on from the oracle's state
            tr.load_params(p_o)
            if optimizer == "adam":
                tr.adam_m.copy_(dev(state[0].astype(np.float32)))
                tr.adam_v.copy_(dev(state[1].astype(np.float32)))
        else:
            close(host(tr.W), omodel.flatten(p_o), 1e-4, f"weights after step {step}")
        losses.append(loss_g)
    assert losses[2] < losses[0]
