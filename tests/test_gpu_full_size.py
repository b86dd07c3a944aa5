"""Parity at the benchmark's full size: configs[1] (1M-node Chung-Lu graph, K = 8, part 0, 128-256-47 model),
through the same calls and launch configuration bench.py times.

The oracle finishes this size in seconds, so everything is compared in full: partition ids and the local CSR
bit for bit, logits, loss, every gradient and the updated weights to the fp32 tolerance."""
import numpy as np
import pytest

import decisions
import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4


def _close(got, want, what, tol=TOL, extra=0.0):
    decisions.close(got, want, tol, what, extra=extra)


def test_configs1_whole_path_against_oracle():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_09887_amd import binding as B
    from paper_2305_09887_amd.trainer import LocalTrainer
    N, K, p, dims, lr = 1_000_000, 8, 0, [128, 256, 47], 1e-3
    rowptr, colidx = synth.chung_lu_graph(N, 20, 2.1, seed=11)
    X, y = synth.features(N, dims[0], seed=12), synth.labels(N, dims[-1], seed=13)
    params = synth.sage_params(dims, seed=15)
    d = lambda a: torch.as_tensor(a).cuda()

    part = B.tma_partition(N, K, seed=14)
    sub = B.tma_induced_subgraph(d(rowptr), d(colidx), part, p)
    part_o = oracle.partition(N, K, seed=14)
    sub_o = oracle.induced_subgraph(rowptr, colidx, part_o, p)
    assert np.array_equal(part.cpu().numpy(), part_o)
    for k in ("g2l", "l2g", "rowptr", "colidx"):
        assert np.array_equal(sub[k].cpu().numpy(), sub_o[k]), k
    assert np.array_equal(sub["inv_deg"].cpu().numpy(), sub_o["inv_deg"].astype(np.float32))
    deg = np.diff(sub_o["rowptr"])
    assert deg.max() > 64 and (deg == 0).mean() > 0.2        # hub rows and many isolated nodes are in the case

    Xl = B.tma_gather_rows(sub["l2g"], d(X))
    yl = B.tma_gather_rows(sub["l2g"], d(y))
    assert np.array_equal(Xl.cpu().numpy(), X[sub_o["l2g"]]) and np.array_equal(yl.cpu().numpy(), y[sub_o["l2g"]])

    tr = LocalTrainer(sub["rowptr"], sub["colidx"], sub["inv_deg"], Xl, yl, dims, params=params)
    loss_g = tr.step(lr).item()

    p_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in params]
    Xo, yo = X[sub_o["l2g"]], y[sub_o["l2g"]]
    # the oracle takes its own ReLU decisions; where the GPU's differ they must sit next to zero, and what those
    # few terms can change is added to the tolerance (decisions.py)
    t = {}
    loss_o, grads_o, logits_o, saved = omodel.loss_and_grads(sub_o["rowptr"], sub_o["colidx"], Xo, yo, p_o, trace=t)
    D = decisions.differing(t["pre"], [tr.H[1].cpu().numpy(), None], "configs[1] SAGE step")
    bounds = decisions.encoder_bounds("sage", sub_o["rowptr"], sub_o["colidx"], p_o, saved, t["ups"], D)
    print(f"differing ReLU decisions: {int(D[0].sum())} of {D[0].size}; allowed change per tensor {bounds}")
    assert abs(loss_g - loss_o) <= TOL * abs(loss_o)
    _close(tr.M[0].cpu().numpy(), saved[0][1], "M layer 0")
    _close(tr.H[1].cpu().numpy(), saved[1][0], "H layer 1")
    _close(tr.H[2].cpu().numpy(), logits_o, "logits")
    for l in range(2):
        for g, w, bd, name in zip(tr.grads[l], grads_o[l], bounds[l], ("dW_self", "dW_neigh", "dbias")):
            _close(g.cpu().numpy(), w, f"layer {l} {name}", extra=bd)
    new_o = [tuple(oracle.sgd_step(w, g, lr).reshape(np.shape(w)) for w, g in zip(pl, gl)) for pl, gl in zip(p_o, grads_o)]
    _close(tr.W.cpu().numpy(), omodel.flatten(new_o), "weights after the step", tol=1e-6, extra=lr * decisions.total(bounds))


@pytest.fixture(scope="module")
def configs1_part0():
    """The quoted workload's graph, features and part 0 (oracle side), shared by the tests below."""
    N, K = 1_000_000, 8
    rowptr, colidx = synth.chung_lu_graph(N, 20, 2.1, seed=11)
    X = synth.features(N, 128, seed=12)
    sub_o = oracle.induced_subgraph(rowptr, colidx, oracle.partition(N, K, seed=14), 0)
    return sub_o, X[sub_o["l2g"]], synth.labels(N, 47, seed=13)[sub_o["l2g"]]


def test_configs1_gcn_step_against_oracle(configs1_part0):
    """The GCN encoder (Sec. 4.1) at the same size and launch configuration as `bench.py --encoder gcn`:
    layer 0 (128 -> 256) aggregates first, layer 1 (256 -> 47) transforms first."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_09887_amd import binding as B
    from paper_2305_09887_amd.trainer import LocalTrainer
    sub_o, Xo, yo = configs1_part0
    dims, lr = [128, 256, 47], 1e-3
    params = [(Ws, b) for Ws, _, b in synth.sage_params(dims, seed=15)]
    d = lambda a, dt=None: (torch.as_tensor(a) if dt is None else torch.as_tensor(a).to(dt)).cuda()
    assert B.tma_gcn_layer_aggregates_first(128, 256, B.TMA_F32) and not B.tma_gcn_layer_aggregates_first(256, 47, B.TMA_F32)
    tr = LocalTrainer(d(sub_o["rowptr"]), d(sub_o["colidx"]), d(sub_o["inv_deg"], torch.float32), d(Xo), d(yo), dims,
                      params=params, encoder="gcn")
    loss_g = tr.step(lr).item()
    p_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in params]
    t = {}
    loss_o, grads_o, logits_o, saved = omodel.loss_and_grads(sub_o["rowptr"], sub_o["colidx"], Xo, yo, p_o,
                                                             encoder="gcn", trace=t)
    D = decisions.differing(t["pre"], [tr.H[1].cpu().numpy(), None], "configs[1] GCN step")
    bounds = decisions.encoder_bounds("gcn", sub_o["rowptr"], sub_o["colidx"], p_o, saved, t["ups"], D)
    assert abs(loss_g - loss_o) <= TOL * abs(loss_o)
    _close(tr.M[0].cpu().numpy(), saved[0][1], "Ahat H of layer 0")
    _close(tr.H[2].cpu().numpy(), logits_o, "logits")
    for l in range(2):
        for g, w, bd, name in zip(tr.grads[l], grads_o[l], bounds[l], ("dW", "dbias")):
            _close(g.cpu().numpy(), w, f"layer {l} {name}", extra=bd)
    new_o = [tuple(oracle.sgd_step(w, g, lr).reshape(np.shape(w)) for w, g in zip(pl, gl)) for pl, gl in zip(p_o, grads_o)]
    _close(tr.W.cpu().numpy(), omodel.flatten(new_o), "weights after the step", tol=1e-6, extra=lr * decisions.total(bounds))


def test_configs1_link_prediction_step_against_oracle(configs1_part0):
    """The link-prediction task at the size and launch configuration of `bench.py --task link`: SAGE 128-256-256,
    decoder 256-256-1, 65,536 positives and as many negatives; the batch bit for bit, logits, loss, every gradient."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_09887_amd.trainer import LocalTrainer
    sub_o, Xo, _ = configs1_part0
    rp, ci = sub_o["rowptr"], sub_o["colidx"]
    dims, dec_dims, Bn, lr = [128, 256, 256], [256, 256, 1], 65_536, 1e-3
    enc = synth.sage_params(dims, seed=15)
    rng = np.random.default_rng(16)
    dec = [(synth.glorot(256, 256, rng).astype(np.float32), np.array([0.25], np.float32)),
           (synth.glorot(256, 1, rng).astype(np.float32),)]
    d = lambda a, dt=None: (torch.as_tensor(a) if dt is None else torch.as_tensor(a).to(dt)).cuda()
    tr = LocalTrainer(d(rp), d(ci), d(sub_o["inv_deg"], torch.float32), d(Xo), None, dims, params=enc,
                      decoder_dims=dec_dims, batch_size=Bn, batch_seed=15, nnz=int(rp[-1]))
    tr.load_params(enc, dec)
    loss_g = tr.step(lr).item()
    batch = oracle.edge_batch(rp, ci, 15, 0, Bn)
    for got, want in zip(tr.batch, batch):
        assert np.array_equal(got.cpu().numpy(), want)
    counts = np.bincount(np.concatenate([batch[0], batch[0], batch[1], batch[2]]), minlength=len(rp) - 1)
    assert counts.max() > 256 and (counts == 0).mean() > 0.2      # long and empty per-node term lists are in the case
    e_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in enc]
    d_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in dec]
    t = {}
    loss_o, ge, gd, z = omodel.link_loss_and_grads(rp, ci, Xo, batch, e_o, d_o, "sage", trace=t)
    D = decisions.differing(t["pre"], [tr.H[1].cpu().numpy(), None], "encoder")
    Dd = decisions.differing(t["dec_pre"], [tr.E[1].cpu().numpy(), None], "decoder")
    db, q_top = decisions.decoder_bounds(d_o, t["dsaved"], t["dec_ups"], Dd, t["R"], t["batch_pos"])
    eb = decisions.encoder_bounds("sage", rp, ci, e_o, t["saved"], t["ups"], D, q_top)
    assert abs(loss_g - loss_o) <= TOL * abs(loss_o)
    _close(tr.Zd[2].cpu().numpy().ravel(), z, "logits")
    for l in range(2):
        for g, w, bd, name in zip(tr.grads[l], ge[l], eb[l], ("dW_self", "dW_neigh", "dbias")):
            _close(g.cpu().numpy(), w, f"encoder layer {l} {name}", extra=bd)
        for g, w, bd, name in zip(tr.dec_grads[l], gd[l], db[l], ("dTheta", "dslope")):
            _close(g.cpu().numpy().ravel(), np.asarray(w).ravel(), f"decoder layer {l} {name}", extra=bd)


@pytest.mark.parametrize("encoder,device_counts", [("sage", True), ("sage", False), ("gcn", True)])
def test_configs1_sampled_link_prediction_step_against_oracle(configs1_part0, encoder, device_counts):
    """Link prediction on sampled message-flow graphs at the size and launch configuration of
    `bench.py --task link-sampled [--encoder gcn] [--level-sizes host]`: 1,024 positives, fan-outs 10 / 25, encoder
    128-256-256, decoder 256-256-1; node lists and blocks bit for bit, logits, loss and every gradient."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_09887_amd.trainer import SampledLinkTrainer
    sub_o, Xo, _ = configs1_part0
    rp, ci = sub_o["rowptr"], sub_o["colidx"]
    nnz = int(rp[-1])
    dims, dec_dims, fanouts, Bn = [128, 256, 256], [256, 256, 1], [10, 25], 1024
    enc = [tuple(l) if encoder == "sage" else (l[0], l[2]) for l in synth.sage_params(dims, seed=15)]
    rng = np.random.default_rng(16)
    dec = [(synth.glorot(256, 256, rng).astype(np.float32), np.array([0.25], np.float32)),
           (synth.glorot(256, 1, rng).astype(np.float32),)]
    d = lambda a: torch.as_tensor(a).cuda()
    tr = SampledLinkTrainer(d(rp), d(ci), nnz, d(Xo), dims, dec_dims, fanouts, Bn, batch_seed=15, params=enc,
                            decoder_params=dec, nnz_cap=nnz + nnz // 4 + 4096, encoder=encoder,
                            device_counts=device_counts)
    loss_g = tr.step(1e-3).item()
    batch = oracle.edge_batch(rp, ci, 15, 0, Bn)
    e_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in enc]
    d_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in dec]
    t = {}
    loss_o, ge, gd, z, (rps, cis, inputs, seeds) = omodel.sampled_link_loss_and_grads(
        rp, ci, Xo, batch, e_o, d_o, fanouts, 15, 0, trace=t, encoder=encoder)
    assert tr.count == [len(inputs), len(rps[0]) - 1, len(seeds)]
    assert len(inputs) > 20_000 and np.diff(rps[0]).max() == 10 and np.diff(rps[1]).max() == 25   # the fan-outs bind
    assert np.array_equal(tr.nodes[0].cpu().numpy()[:len(inputs)], inputs)
    assert np.array_equal(tr.nodes[2].cpu().numpy()[:len(seeds)], seeds)
    for l in range(2):
        n_dst = len(rps[l]) - 1
        assert np.array_equal(tr.blk_rowptr[l].cpu().numpy()[:n_dst + 1], rps[l])
        assert np.array_equal(tr.blk_col[l].cpu().numpy()[:rps[l][-1]], cis[l])
    D = decisions.differing(t["pre"], [tr.H[1].cpu().numpy(), None], "encoder")
    Dd = decisions.differing(t["dec_pre"], [tr.E[1].cpu().numpy(), None], "decoder")
    db, q_top = decisions.decoder_bounds(d_o, t["dsaved"], t["dec_ups"], Dd, t["R"], t["batch_pos"])
    eb = decisions.encoder_bounds(encoder, rps, cis, e_o, t["saved"], t["ups"], D, q_top)
    assert abs(loss_g - loss_o) <= TOL * abs(loss_o)
    _close(tr.Zd[2].cpu().numpy().ravel(), z, "logits")
    for l in range(2):
        for i, (g, w, bd) in enumerate(zip(tr.grads[l], ge[l], eb[l])):
            _close(g.cpu().numpy().ravel(), np.asarray(w).ravel(), f"encoder layer {l} gradient {i}", extra=bd)
        for i, (g, w, bd) in enumerate(zip(tr.dec_grads[l], gd[l], db[l])):
            _close(g.cpu().numpy().ravel(), np.asarray(w).ravel(), f"decoder layer {l} gradient {i}", extra=bd)
