"""Sampled message-flow graphs (Sec. 4.1: GraphSAGE-style neighbour sampling) on the GPU against the oracle,
through the C ABI: the sampled blocks and the relabelled node lists bit for bit, the SAGE layer on a bipartite
block forward and backward to 1e-4 (fp32) / 2e-2 (bf16)."""
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


def local_graph(n_glob, m, seed, K=2, kind="chung_lu"):
    if kind == "uniform":
        rowptr, colidx = synth.uniform_graph(n_glob, m, seed)
    else:
        rowptr, colidx = synth.chung_lu_graph(n_glob, 2.0 * m / n_glob, 2.1, seed)
    sub = oracle.induced_subgraph(rowptr, colidx, oracle.partition(n_glob, K, seed=seed), 0)
    return sub["rowptr"], sub["colidx"]


@pytest.mark.parametrize("kind,fanout,n_dst", [("chung_lu", 5, 4000), ("chung_lu", 25, 9000), ("uniform", 2, 1),
                                               ("chung_lu", 10**6, 3000), ("uniform", 3, 0), ("chung_lu", 1, 12_000)])
def test_neighbor_sample_bit_exact(B, kind, fanout, n_dst):
    rp, ci = local_graph(40_000, 400_000, 9, kind=kind)
    n = len(rp) - 1
    deg = np.diff(rp)
    assert kind == "uniform" or deg.max() > 2048 or deg.max() > 64     # rows ranked from LDS, maybe beyond
    rng = np.random.default_rng(fanout)
    dst = rng.permutation(n)[:n_dst].astype(np.int32)
    if n_dst > 10:
        dst[:5] = np.argsort(-deg)[:5]                                  # the hubs are asked for
    brp, bcol, brow = B.tma_neighbor_sample(dev(dst) if n_dst else torch.empty(0, dtype=torch.int32, device="cuda"),
                                            n_dst, int(rp[-1]), dev(rp), dev(ci), fanout, seed=1234 + fanout)
    wrp, wcol = oracle.neighbor_sample(dst, rp, ci, fanout, 1234 + fanout)
    assert np.array_equal(brp.cpu().numpy(), wrp)
    total = int(wrp[-1])
    assert np.array_equal(bcol.cpu().numpy()[:total], wcol)
    assert np.array_equal(brow.cpu().numpy()[:total], np.repeat(np.arange(n_dst, dtype=np.int32), np.diff(wrp)))


def test_neighbor_sample_rows_beyond_the_lds_segment(B):
    # a star: the centre has 5000 neighbours, far more than the keys a wavefront keeps in LDS
    m = 5000
    rp, ci = synth.csr_from_pairs(m + 1, np.zeros(m, dtype=np.int64), np.arange(1, m + 1))
    rp, ci = rp.astype(np.int32), ci.astype(np.int32)
    dst = np.array([7, 0, 4000], dtype=np.int32)
    # fan-outs for which the kernel's first cut of the keys (about 2 * fanout + 32 of them) holds the wanted ones,
    # lands near the 512 keys the LDS segment holds (either side of it over the seeds), is far above it, or is not
    # tried at all
    for fanout, seed in ([(10, 5), (100, 6)] + [(f, s) for f in (232, 240, 248) for s in (7, 8, 9)]
                         + [(1000, 7), (4999, 5), (5000, 5)]):
        brp, bcol, _ = B.tma_neighbor_sample(dev(dst), 3, int(rp[-1]), dev(rp), dev(ci), fanout, seed=seed)
        wrp, wcol = oracle.neighbor_sample(dst, rp, ci, fanout, seed)
        assert np.array_equal(brp.cpu().numpy(), wrp) and np.array_equal(bcol.cpu().numpy()[:wrp[-1]], wcol), (fanout, seed)


@pytest.mark.parametrize("n_dst,cap_dst,fanout", [(700, 2000, 5), (0, 300, 3), (1500, 1500, 10**6), (1, 4000, 1)])
def test_sampling_a_level_with_its_size_on_the_device(B, n_dst, cap_dst, fanout):
    """tma_neighbor_sample_dev + tma_mfg_relabel_dev + tma_gather_rows_dev: the launches are sized for cap_dst rows,
    the row count is read on the device; against the oracle, with the buffers' contents past the counts checked."""
    rp, ci = local_graph(40_000, 400_000, 9)
    n = len(rp) - 1
    rng = np.random.default_rng(n_dst + fanout % 7)
    perm = rng.permutation(n).astype(np.int32)
    if n_dst > 10:                                               # the hubs are asked for
        hubs = np.argsort(-np.diff(rp))[:3].astype(np.int32)
        perm = np.concatenate([hubs, perm[~np.isin(perm, hubs)]])
    dst = perm[:cap_dst].copy()                                  # (the entries past n_dst are stale ids)
    d_n = dev(np.array([n_dst, 77], np.int32))
    nnz = int(rp[-1])
    brp, bcol, brow = B.tma_neighbor_sample_dev(dev(dst), cap_dst, d_n[0:1], nnz, dev(rp), dev(ci), fanout, seed=4321)
    wrp, wcol = oracle.neighbor_sample(dst[:n_dst], rp, ci, fanout, 4321)
    total = int(wrp[-1])
    got = brp.cpu().numpy()
    assert got.shape == (cap_dst + 1,) and np.array_equal(got[:n_dst + 1], wrp) and (got[n_dst:] == total).all()
    assert np.array_equal(bcol.cpu().numpy()[:total], wcol)
    assert np.array_equal(brow.cpu().numpy()[:total], np.repeat(np.arange(n_dst, dtype=np.int32), np.diff(wrp)))
    # node list and positions
    max_items = bcol.numel()
    cols = bcol.clone()
    cols[total:] = -7
    src = torch.full((min(n, cap_dst + max_items),), -5, dtype=torch.int32, device="cuda")
    n_src = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.tma_mfg_relabel_dev(n, dev(dst), cap_dst, d_n[0:1], cols, max_items, d_items=brp[cap_dst:cap_dst + 1], src_out=src,
                          n_src_out=n_src)
    wsrc, wcols = oracle.mfg_relabel(dst[:n_dst], wcol)
    assert int(n_src) == len(wsrc)
    assert np.array_equal(src.cpu().numpy()[:len(wsrc)], wsrc) and (src.cpu().numpy()[len(wsrc):] == -5).all()
    assert np.array_equal(cols.cpu().numpy()[:total], wcols) and (cols.cpu().numpy()[total:] == -7).all()
    # the rows of the node list, gathered with the count on the device
    X = torch.randn(n, 24, device="cuda")
    out = torch.full((src.numel(), 24), 3.0, device="cuda")
    B.tma_gather_rows_dev(src, n_src, X, out)
    assert torch.equal(out[:len(wsrc)], X[torch.as_tensor(wsrc, device="cuda").long()]) and (out[len(wsrc):] == 3.0).all()
    # a batch's distinct nodes: no dst nodes at all
    ids = rng.integers(0, n, 500).astype(np.int32)
    cbuf = dev(ids)
    usrc, un = B.tma_mfg_relabel_dev(n, None, 0, None, cbuf, 500)
    wsrc0, wcols0 = oracle.mfg_relabel(np.zeros(0, np.int32), ids)
    assert int(un) == len(wsrc0) and np.array_equal(usrc.cpu().numpy()[:len(wsrc0)], wsrc0)
    assert np.array_equal(cbuf.cpu().numpy(), wcols0)


@pytest.mark.parametrize("n_dst,n_items", [(300, 5000), (0, 9000), (1, 1), (2000, 0), (50, 40_000)])
def test_mfg_relabel_bit_exact(B, n_dst, n_items):
    n = 20_000
    rng = np.random.default_rng(n_dst + n_items)
    dst = rng.permutation(n)[:n_dst].astype(np.int32)
    cols = rng.integers(0, n, n_items).astype(np.int32)
    if n_dst and n_items:
        cols[::7] = dst[rng.integers(0, n_dst, len(cols[::7]))]          # dst nodes occur as neighbours too
    cap = n_items + 100
    cbuf = torch.full((max(cap, 1),), -7, dtype=torch.int32, device="cuda")
    cbuf[:n_items] = dev(cols)
    d_items = dev(np.array([n_items], np.int32))
    src, n_src = B.tma_mfg_relabel(n, dev(dst) if n_dst else None, n_dst, cbuf, cap, d_items=d_items)
    wsrc, wcols = oracle.mfg_relabel(dst, cols)
    assert n_src == len(wsrc)
    assert np.array_equal(src.cpu().numpy()[:n_src], wsrc)
    assert np.array_equal(cbuf.cpu().numpy()[:n_items], wcols)
    assert (cbuf.cpu().numpy()[n_items:] == -7).all()                      # entries past the device count are left alone


def _block_case(F_in, F_out, fanout, seed):
    rp, ci = local_graph(30_000, 200_000, seed)
    n = len(rp) - 1
    rng = np.random.default_rng(seed)
    dst = rng.permutation(n)[:3000].astype(np.int32)
    brp, bcol = oracle.neighbor_sample(dst, rp, ci, fanout, seed)
    src, cols = oracle.mfg_relabel(dst, bcol)
    H = rng.standard_normal((len(src), F_in)).astype(np.float32)
    Ws, Wn = synth.glorot(F_in, F_out, rng).astype(np.float32), synth.glorot(F_in, F_out, rng).astype(np.float32)
    b = (0.1 * rng.standard_normal(F_out)).astype(np.float32)
    g = (rng.standard_normal((len(dst), F_out)) / len(dst)).astype(np.float32)
    return brp, cols, len(dst), len(src), H, Ws, Wn, b, g


@pytest.mark.parametrize("F_in,F_out,fanout,bf16", [(64, 96, 5, False), (128, 256, 10, False), (256, 47, 3, False),
                                                    (100, 64, 25, False), (128, 128, 10, True)])
@pytest.mark.parametrize("act", [0, 1])
def test_sage_layer_on_a_sampled_block(B, F_in, F_out, fanout, bf16, act):
    brp, cols, n_dst, n_src, H, Ws, Wn, b, g = _block_case(F_in, F_out, fanout, seed=F_in + F_out)
    tol = 2e-2 if bf16 else 1e-4
    if bf16:
        H, g = synth.round_bf16(H), synth.round_bf16(g)
    dt = torch.bfloat16 if bf16 else torch.float32
    put = (lambda a: dev_bf16(a)) if bf16 else (lambda a: dev(a))
    Hd = B._padded(n_src + 5, F_in, dt, "cuda")            # buffers larger than the block, as a trainer keeps them
    Hd[:n_src] = put(H)
    gd = B._padded(n_dst + 5, F_out, dt, "cuda")
    gd[:n_dst] = put(g)
    Md = torch.empty((n_dst + 5, F_in), dtype=dt, device="cuda")
    Hn = B._padded(n_dst + 5, F_out, dt, "cuda")
    rpd, cid = dev(brp), dev(cols)
    rows = dev(np.repeat(np.arange(n_dst, dtype=np.int32), np.diff(brp)))
    inv = B.tma_block_inv_deg(rpd, n_dst)
    np.testing.assert_array_equal(inv.cpu().numpy()[:n_dst],
                                  np.where(np.diff(brp) > 0, 1.0 / np.maximum(np.diff(brp), 1), 0).astype(np.float32))
    B.tma_sage_block_fwd(n_dst, n_src, rpd, cid, inv, Hd, dev(Ws), dev(Wn), dev(b), act, Md, Hn)
    M, Z, want = oracle.sage_layer_fwd(brp, cols, H, Ws, Wn, b, act)
    close(host(Md[:n_dst]), M, tol, "M")
    close(host(Hn[:n_dst]), want, tol, "Hnext")
    dWs, dWn, db = (torch.empty((F_in, F_out), device="cuda"), torch.empty((F_in, F_out), device="cuda"),
                    torch.empty(F_out, device="cuda"))
    dH = torch.full_like(Hd, float("nan"))
    # the backward pass is given the oracle's layer output (rounded to the storage format: signs survive), so both
    # sides take the ReLU decisions of the oracle's own Z
    Hn[:n_dst] = put(want)
    B.tma_sage_block_bwd(n_dst, n_src, len(cols) + 17, rpd, cid, rows, inv, Hd, Md, Hn, gd, dev(Ws), dev(Wn), act, dWs, dWn,
                         db, dH_out=dH)
    wWs, wWn, wb, wH = oracle.sage_layer_bwd(brp, cols, H, M, Z, g, Ws, Wn, act)
    close(host(dWs), wWs, tol, "dW_self")
    close(host(dWn), wWn, tol, "dW_neigh")
    close(host(db), wb, tol, "dbias")
    close(host(dH[:n_src]), wH, tol, "dH over all source rows")
    assert torch.isnan(dH[n_src:]).all()                    # rows past the block are not touched
    dH2 = torch.empty_like(Hd)
    B.tma_sage_block_bwd(n_dst, n_src, len(cols) + 17, rpd, cid, rows, inv, Hd, Md, Hn, gd, dev(Ws), dev(Wn), act, dWs, dWn,
                         db, dH_out=dH2)
    assert torch.equal(dH2[:n_src], dH[:n_src])             # fixed summation order: the same bits
    B.tma_sage_block_bwd(n_dst, n_src, len(cols), rpd, cid, rows, inv, Hd, Md, Hn, gd, dev(Ws), dev(Wn), act, dWs, dWn, db,
                         dH_out=None)                       # a first layer: no input gradient
    close(host(dWs), wWs, tol, "dW_self without dH")


@pytest.mark.parametrize("F_in,F_out,fanout,bf16", [(64, 96, 5, False), (128, 256, 10, False), (256, 47, 3, False),
                                                    (100, 64, 25, False), (128, 128, 10, True)])
@pytest.mark.parametrize("act", [0, 1])
def test_gcn_layer_on_a_sampled_block(B, F_in, F_out, fanout, bf16, act):
    """The GCN layer in its block form (mean over the sampled neighbours and the node itself): aggregate, output,
    and every gradient against the oracle; rows of the buffers past the block stay untouched."""
    brp, cols, n_dst, n_src, H, W, _, b, g = _block_case(F_in, F_out, fanout, seed=F_in + F_out + 1)
    tol = 2e-2 if bf16 else 1e-4
    if bf16:
        H, g = synth.round_bf16(H), synth.round_bf16(g)
    dt = torch.bfloat16 if bf16 else torch.float32
    put = (lambda a: dev_bf16(a)) if bf16 else (lambda a: dev(a))
    Hd = B._padded(n_src + 5, F_in, dt, "cuda")
    Hd[:n_src] = put(H)
    gd = B._padded(n_dst + 5, F_out, dt, "cuda")
    gd[:n_dst] = put(g)
    Md = torch.empty((n_dst + 5, F_in), dtype=dt, device="cuda")
    Hn = B._padded(n_dst + 5, F_out, dt, "cuda")
    rpd, cid = dev(brp), dev(cols)
    rows = dev(np.repeat(np.arange(n_dst, dtype=np.int32), np.diff(brp)))
    c = B.tma_gcn_block_norm(rpd, n_dst)
    np.testing.assert_array_equal(c.cpu().numpy()[:n_dst], (1.0 / (np.diff(brp) + 1.0)).astype(np.float32))
    B.tma_gcn_block_fwd(n_dst, n_src, rpd, cid, c, Hd, dev(W), dev(b), act, Md, Hn)
    M, Z, want = oracle.gcn_block_layer_fwd(brp, cols, H, W, b, act)
    close(host(Md[:n_dst]), M, tol, "M")
    close(host(Hn[:n_dst]), want, tol, "Hnext")
    dW, db = torch.empty((F_in, F_out), device="cuda"), torch.empty(F_out, device="cuda")
    dH = torch.full((n_src + 5, F_in), float("nan"), dtype=dt, device="cuda")
    # the saved aggregate and the layer output that the backward pass reads are the oracle's, in the storage format:
    # both sides then differentiate the same function at the same point, with the oracle's ReLU decisions
    Md[:n_dst] = put(M)
    Hn[:n_dst] = put(want)
    Ms = synth.round_bf16(M.astype(np.float32)) if bf16 else M
    B.tma_gcn_block_bwd(n_dst, n_src, len(cols) + 17, rpd, cid, rows, c, Md, Hn, gd, dev(W), act, dW, db, dH_out=dH)
    wW, wb, wH = oracle.gcn_block_layer_bwd(brp, cols, n_src, Ms, Z, g, W, act)
    close(host(dW), wW, tol, "dW")
    close(host(db), wb, tol, "dbias")
    close(host(dH[:n_src]), wH, tol, "dH over all source rows")
    assert torch.isnan(dH[n_src:]).all()
    dH2 = torch.empty_like(dH)
    B.tma_gcn_block_bwd(n_dst, n_src, len(cols) + 17, rpd, cid, rows, c, Md, Hn, gd, dev(W), act, dW, db, dH_out=dH2)
    assert torch.equal(dH2[:n_src], dH[:n_src])             # fixed summation order: the same bits
    B.tma_gcn_block_bwd(n_dst, n_src, len(cols), rpd, cid, rows, c, Md, Hn, gd, dev(W), act, dW, db, dH_out=None)
    close(host(dW), wW, tol, "dW without dH")


def test_gcn_block_degenerate_shapes(B):
    """No destination rows; a block without any entry (every row keeps its own features)."""
    F_in, F_out = 24, 8
    rng = np.random.default_rng(3)
    W, b = dev(synth.glorot(F_in, F_out, rng).astype(np.float32)), dev(np.zeros(F_out, np.float32))
    H = rng.standard_normal((7, F_in)).astype(np.float32)
    Hd, Md, Hn = dev(H), torch.empty((7, F_in), device="cuda"), torch.empty((7, F_out), device="cuda")
    rp0 = dev(np.zeros(8, dtype=np.int32))
    none = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.tma_gcn_block_fwd(0, 7, rp0, none, torch.ones(1, device="cuda"), Hd, W, b, 0, Md, Hn)     # nothing to do
    c = B.tma_gcn_block_norm(rp0, 7)
    assert bool((c == 1.0).all())
    B.tma_gcn_block_fwd(7, 7, rp0, none, c, Hd, W, b, 0, Md, Hn)
    assert torch.equal(Md, Hd)
    close(host(Hn), H.astype(np.float64) @ host(W), 1e-4, "a block without entries is the dense layer")
    dW, db, dH = torch.empty((F_in, F_out), device="cuda"), torch.empty(F_out, device="cuda"), torch.empty((7, F_in), device="cuda")
    g = rng.standard_normal((7, F_out)).astype(np.float32)
    B.tma_gcn_block_bwd(7, 7, 0, rp0, none, none, c, Md, Hn, dev(g), W, 0, dW, db, dH_out=dH)
    close(host(dH), g.astype(np.float64) @ host(W).T, 1e-4, "dH")
    close(host(dW), H.astype(np.float64).T @ g, 1e-4, "dW")
    torch.cuda.synchronize()


@pytest.mark.parametrize("fanouts,Bn,norm_act,encoder", [([5, 5], 512, False, "sage"), ([10, 25], 300, False, "sage"),
                                                         ([10**6, 10**6], 200, False, "sage"), ([1, 2], 1000, False, "sage"),
                                                         ([5, 10], 400, True, "sage"), ([5, 5], 512, False, "gcn"),
                                                         ([10, 25], 300, False, "gcn"), ([10**6, 10**6], 200, False, "gcn"),
                                                         ([5, 10], 400, True, "gcn")])
def test_sampled_link_prediction_training_steps(B, fanouts, Bn, norm_act, encoder):
    """Three steps of link prediction on sampled message-flow graphs (2-layer SAGE or GCN 64-96-32, decoder 32-48-1)
    on the tiny configuration's part 0: batch, node lists and blocks bit for bit; loss, logits, every gradient and
    the weights after each SGD step against the oracle."""
    from oracle import model as omodel
    from paper_2305_09887_amd.trainer import SampledLinkTrainer
    N, K, dims, dec_dims = 20_000, 4, [64, 96, 32], [32, 48, 1]
    rowptr, colidx = synth.chung_lu_graph(N, 12, 2.1, seed=1)
    X = synth.features(N, dims[0], seed=2)
    rng = np.random.default_rng(7)
    enc = []
    for l, layer in enumerate(synth.sage_params(dims, seed=5)):
        layer = list(layer) if encoder == "sage" else [layer[0], layer[2]]
        if norm_act and l < len(dims) - 2:      # the paper's encoder variant: layer normalisation + PReLU
            layer += [rng.normal(1.0, 0.1, dims[l + 1]).astype(np.float32),
                      rng.normal(0.0, 0.1, dims[l + 1]).astype(np.float32), np.array([0.25], dtype=np.float32)]
        enc.append(tuple(layer))
    dec = [(synth.glorot(32, 48, rng).astype(np.float32), np.array([0.25], np.float32)),
           (synth.glorot(48, 1, rng).astype(np.float32),)]
    sub = oracle.induced_subgraph(rowptr, colidx, oracle.partition(N, K, seed=4), 0)
    rp, ci = sub["rowptr"], sub["colidx"]
    Xo = X[sub["l2g"]]
    tr = SampledLinkTrainer(dev(rp), dev(ci), int(rp[-1]), dev(Xo), dims, dec_dims, fanouts, Bn, batch_seed=99,
                            params=enc, decoder_params=dec, norm_act=norm_act, encoder=encoder)
    e_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in enc]
    d_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in dec]
    assert tr.n_params == omodel.flatten(e_o + d_o).size
    lr, losses = 0.5, []
    for step in range(3):
        loss_g = tr.step(lr).item()
        batch = oracle.edge_batch(rp, ci, 99, step * Bn, Bn)
        t = {}
        loss_o, ge, gd, z, (rps, cis, inputs, seeds) = omodel.sampled_link_loss_and_grads(
            rp, ci, Xo, batch, e_o, d_o, fanouts, 99, step, trace=t, encoder=encoder)
        assert tr.count[2] == len(seeds) and np.array_equal(tr.nodes[2].cpu().numpy()[:len(seeds)], seeds)
        for got, want in zip(tr.batch, batch):
            assert np.array_equal(got.cpu().numpy(), np.searchsorted(seeds, want))
        for l in range(2):
            n_dst = len(rps[l]) - 1
            assert tr.count[l + 1] == n_dst
            assert np.array_equal(tr.blk_rowptr[l].cpu().numpy()[:n_dst + 1], rps[l])
            assert np.array_equal(tr.blk_col[l].cpu().numpy()[:rps[l][-1]], cis[l])
        assert tr.count[0] == len(inputs) and np.array_equal(tr.nodes[0].cpu().numpy()[:len(inputs)], inputs)
        D = decisions.differing(t["pre"], [host(tr.H[1][:tr.count[1]]), None], f"step {step} encoder")
        Dd = decisions.differing(t["dec_pre"], [host(tr.E[1]), None], f"step {step} decoder")
        db, q_top = decisions.decoder_bounds(d_o, t["dsaved"], t["dec_ups"], Dd, t["R"], t["batch_pos"])
        eb = decisions.encoder_bounds(encoder, rps, cis, e_o, t["saved"], t["ups"], D, q_top)
        assert abs(loss_g - loss_o) <= 1e-4 * abs(loss_o), f"loss at step {step}"
        close(host(tr.Zd[2]).ravel(), z, 1e-4, f"logits at step {step}")
        for l in range(2):
            for i, (g, w, bd) in enumerate(zip(tr.grads[l], ge[l], eb[l])):
                decisions.close(host(g).ravel(), np.asarray(w).ravel(), 1e-4, f"step {step} encoder layer {l} gradient {i}",
                                extra=bd)
            for i, (g, w, bd) in enumerate(zip(tr.dec_grads[l], gd[l], db[l])):
                decisions.close(host(g).ravel(), np.asarray(w).ravel(), 1e-4, f"step {step} decoder layer {l} gradient {i}",
                                extra=bd)
        e_o = [tuple(oracle.sgd_step(w, g, lr).reshape(np.shape(w)) for w, g in zip(pl, gl)) for pl, gl in zip(e_o, ge)]
        d_o = [tuple(oracle.sgd_step(w, g, lr).reshape(np.shape(w)) for w, g in zip(pl, gl)) for pl, gl in zip(d_o, gd)]
        decisions.close(host(tr.W), omodel.flatten(e_o + d_o), 1e-4, f"weights after step {step}",
                        extra=lr * (decisions.total(eb) + decisions.total(db)))
        if decisions.any_differs(D, Dd):
            tr.load_params(e_o, d_o)
        losses.append(loss_g)
    assert np.isfinite(losses).all()      # (every step sees another batch: the loss need not fall step by step)


@pytest.mark.parametrize("encoder", ["sage", "gcn"])
def test_sampling_one_step_ahead_on_a_second_stream_changes_nothing(B, encoder):
    """With enable_prefetch() every step trains on the batch that was sampled, on a second stream and into a second
    set of buffers, while the step before it trained: the same batches, blocks and bits as sampling inside the step.
    Also when the caller drives the sampling itself and swaps the feature table between steps."""
    from paper_2305_09887_amd.trainer import SampledLinkTrainer
    N, K, dims, dec_dims, fanouts, Bn = 20_000, 4, [64, 96, 32], [32, 48, 1], [5, 10], 400
    rowptr, colidx = synth.chung_lu_graph(N, 12, 2.1, seed=1)
    X = synth.features(N, dims[0], seed=2)
    rng = np.random.default_rng(7)
    enc = [tuple(l) if encoder == "sage" else (l[0], l[2]) for l in synth.sage_params(dims, seed=5)]
    dec = [(synth.glorot(32, 48, rng).astype(np.float32), np.array([0.25], np.float32)),
           (synth.glorot(48, 1, rng).astype(np.float32),)]
    sub = oracle.induced_subgraph(rowptr, colidx, oracle.partition(N, K, seed=4), 0)
    rp, ci, Xd = dev(sub["rowptr"]), dev(sub["colidx"]), dev(X[sub["l2g"]])
    X2 = Xd.clone()                                       # a second table with the same values at another address

    def make(**kw):
        return SampledLinkTrainer(rp, ci, int(sub["rowptr"][-1]), Xd, dims, dec_dims, fanouts, Bn, batch_seed=99,
                                  params=enc, decoder_params=dec, encoder=encoder, **kw)

    # the plain one fetches every level's size as soon as it exists; the others leave the sizes on the device while
    # they sample (capacity-sized launches) and wait once
    plain, ahead, driven = make(device_counts=False), make(), make()
    ahead.enable_prefetch(background=True)                # a worker thread makes the sampling calls
    driven.enable_prefetch(auto=False)
    for step in range(5):
        lp = plain.step(0.5).item()
        la = ahead.step(0.5).item()
        if step == 0:
            driven.prefetch_sample()
        ld = driven.step(0.5).item()
        driven.set_data(X2 if step % 2 == 0 else Xd)      # the next batch reads the other table
        driven.prefetch_sample()
        for other, l in ((ahead, la), (driven, ld)):
            assert l == lp, f"loss at step {step}"
            assert other.count == plain.count
            for a, b in zip(other.batch, plain.batch):
                assert torch.equal(a, b)
            for l_ in range(3):
                assert torch.equal(other.nodes[l_][:plain.count[l_]], plain.nodes[l_][:plain.count[l_]])
            for l_ in range(2):
                n_dst = plain.count[l_ + 1]
                e = int(plain.blk_rowptr[l_][n_dst])
                assert torch.equal(other.blk_rowptr[l_][:n_dst + 1], plain.blk_rowptr[l_][:n_dst + 1])
                assert torch.equal(other.blk_col[l_][:e], plain.blk_col[l_][:e])
            assert torch.equal(other.W, plain.W), f"weights after step {step}"
    ahead.disable_prefetch()
    assert ahead.step(0.5).item() == plain.step(0.5).item() and torch.equal(ahead.W, plain.W)
    torch.cuda.synchronize()


@pytest.mark.parametrize("encoder", ["sage", "gcn"])
def test_sampled_link_prediction_bf16_storage(B, encoder):
    """The sampled link-prediction step with bf16 feature / activation storage (bf16 MFMA products, fp32
    accumulation and parameters): one step against the oracle at the bf16 tolerance; structure bit for bit."""
    from oracle import model as omodel
    from paper_2305_09887_amd.trainer import SampledLinkTrainer
    N, K, dims, dec_dims, fanouts, Bn = 20_000, 4, [64, 96, 32], [32, 48, 1], [5, 10], 600
    rowptr, colidx = synth.chung_lu_graph(N, 12, 2.1, seed=1)
    X = synth.round_bf16(synth.features(N, dims[0], seed=2))
    rng = np.random.default_rng(7)
    enc = [tuple(l) if encoder == "sage" else (l[0], l[2]) for l in synth.sage_params(dims, seed=5)]
    dec = [(synth.glorot(32, 48, rng).astype(np.float32), np.array([0.25], np.float32)),
           (synth.glorot(48, 1, rng).astype(np.float32),)]
    sub = oracle.induced_subgraph(rowptr, colidx, oracle.partition(N, K, seed=4), 0)
    rp, ci = sub["rowptr"], sub["colidx"]
    Xo = X[sub["l2g"]]
    tr = SampledLinkTrainer(dev(rp), dev(ci), int(rp[-1]), dev_bf16(Xo).contiguous(), dims, dec_dims, fanouts, Bn,
                            batch_seed=3, params=enc, decoder_params=dec, encoder=encoder)
    loss_g = tr.step(0.1).item()
    e_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in enc]
    d_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in dec]
    batch = oracle.edge_batch(rp, ci, 3, 0, Bn)
    t = {}
    loss_o, ge, gd, z, (rps, cis, inputs, seeds) = omodel.sampled_link_loss_and_grads(
        rp, ci, Xo, batch, e_o, d_o, fanouts, 3, 0, decisions="bf16", trace=t, encoder=encoder)    # decisions of the as-stored pass
    assert tr.count == [len(inputs), len(rps[0]) - 1, len(seeds)]
    assert np.array_equal(tr.nodes[0].cpu().numpy()[:len(inputs)], inputs)
    kw = decisions.STORED
    D = decisions.differing(t["pre"], [host(tr.H[1][:tr.count[1]]), None], "encoder", **kw)
    Dd = decisions.differing(t["dec_pre"], [host(tr.E[1]), None], "decoder", **kw)
    db, q_top = decisions.decoder_bounds(d_o, t["dsaved"], t["dec_ups"], Dd, t["R"], t["batch_pos"])
    eb = decisions.encoder_bounds(encoder, rps, cis, e_o, t["saved"], t["ups"], D, q_top)
    print(f"differing decisions: encoder {int(D[0].sum())} of {D[0].size}, decoder {int(Dd[0].sum())} of {Dd[0].size}")
    assert abs(loss_g - loss_o) <= 2e-2 * abs(loss_o)
    close(host(tr.Zd[2]).ravel(), z, 2e-2, "logits")
    for l in range(2):
        for i, (g, w, bd) in enumerate(zip(tr.grads[l], ge[l], eb[l])):
            decisions.close(host(g).ravel(), np.asarray(w).ravel(), 2e-2, f"encoder layer {l} gradient {i}", extra=bd)
        for i, (g, w, bd) in enumerate(zip(tr.dec_grads[l], gd[l], db[l])):
            decisions.close(host(g).ravel(), np.asarray(w).ravel(), 2e-2, f"decoder layer {l} gradient {i}", extra=bd)
