"""One whole step (assignment, extraction without a host wait, row gathers, training pass, averaging) captured as
a HIP graph: every replay must reproduce the eager step bit for bit, with the program's own eager work and
synchronisations between the replays.  The eager step itself is checked against the oracle once."""
import numpy as np
import pytest

import decisions
import oracle
from oracle import model as omodel
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


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a)).cuda()


def test_captured_step_replays_bit_identically(B):
    from paper_2305_09887_amd.trainer import LocalTrainer
    N, K, p, dims, lr = 60_000, 4, 1, [64, 96, 16], 0.05
    rowptr, colidx = synth.chung_lu_graph(N, 12, 2.1, seed=31)
    X, y = synth.features(N, dims[0], seed=32), synth.labels(N, dims[-1], seed=33)
    params = synth.sage_params(dims, seed=34)
    d_rowptr, d_colidx, d_X, d_y = dev(rowptr), dev(colidx), dev(X), dev(y)

    part = torch.empty(N, dtype=torch.int32, device="cuda")
    B.tma_partition(N, K, 35, out=part)
    first = B.tma_induced_subgraph(d_rowptr, d_colidx, part, p)
    torch.cuda.synchronize()
    n_loc, nnz_loc = first["n_loc"], first["nnz_loc"]
    cap, cap_nnz = n_loc + 1000, nnz_loc + 10_000

    gs = torch.cuda.Stream()
    with torch.cuda.stream(gs):
        Xl = torch.empty((n_loc, dims[0]), dtype=torch.float32, device="cuda")
        yl = torch.empty(n_loc, dtype=torch.int32, device="cuda")
        tr = LocalTrainer(first["rowptr"], first["colidx"], first["inv_deg"], Xl, yl, dims, params=params, stream=gs)
        W0 = tr.W.clone()
        peers = [tr.W.clone() + 0.01 * (k + 1) for k in range(K - 1)]
        peers0 = [w.clone() for w in peers]
        W_all = [tr.W] + peers
        ptrs = torch.tensor([t.data_ptr() for t in W_all], dtype=torch.int64, device="cuda")
        W_global = torch.empty_like(tr.W)
        held = B.tma_induced_subgraph_async(d_rowptr, d_colidx, part, p, cap, cap_nnz)

        def reset():
            tr.W.copy_(W0)
            for w, w0 in zip(peers, peers0):
                w.copy_(w0)
            for t in (part, held["l2g"], held["rowptr"], held["colidx"], Xl, yl, W_global):
                t.fill_(0)      # whatever the step consumes must come from the step itself
            held["inv_deg"].fill_(0)

        def step():
            B.tma_partition(N, K, 35, out=part)
            B.tma_induced_subgraph_async(d_rowptr, d_colidx, part, p, cap, cap_nnz, out=held)
            B.tma_gather_rows(held["l2g"][:n_loc], d_X, out=Xl)
            B.tma_gather_rows(held["l2g"][:n_loc], d_y, out=yl)
            tr.set_graph(held["rowptr"][:n_loc + 1], held["colidx"][:nnz_loc], held["inv_deg"][:n_loc], nnz=nnz_loc)
            tr.step(lr)
            B.tma_average(W_all, W_global_out=W_global, ptr_table=ptrs)

        reset()
        step()
        gs.synchronize()
        assert held["sizes"].cpu().tolist() == [n_loc, nnz_loc]
        eager = dict(W=tr.W.clone(), G=W_global.clone(), dW=tr.dW.clone(), loss=tr.loss.clone(),
                     peers=[w.clone() for w in peers])

    # the eager step against the oracle (one SGD step, then the mean over the K vectors)
    part_o = oracle.partition(N, K, seed=35)
    sub_o = oracle.induced_subgraph(rowptr, colidx, part_o, p)
    p_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in params]
    t = {}
    loss_o, p_new = omodel.train_step(sub_o["rowptr"], sub_o["colidx"], X[sub_o["l2g"]], y[sub_o["l2g"]], p_o, lr, trace=t)
    D = decisions.differing(t["pre"], [tr.H[1].cpu().numpy(), None], "captured step")
    bounds = decisions.encoder_bounds("sage", sub_o["rowptr"], sub_o["colidx"], p_o, t["saved"], t["ups"], D)
    assert abs(float(eager["loss"]) - loss_o) <= 1e-4 * abs(loss_o)
    mean_o = (omodel.flatten(p_new) + sum(w0.cpu().numpy().astype(np.float64) for w0 in peers0)) / K
    decisions.close(eager["G"].cpu().numpy(), mean_o, 1e-4, "averaged weights", extra=lr * decisions.total(bounds) / K)
    assert torch.equal(eager["W"], eager["G"]) and all(torch.equal(w, eager["G"]) for w in eager["peers"])

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(gs):
        reset()
    gs.synchronize()
    with torch.cuda.graph(graph, stream=gs):
        step()
    for replay in range(4):
        with torch.cuda.stream(gs):
            reset()
            # eager work of the program's own between the replays: another part's extraction, a reduction
            other = B.tma_induced_subgraph(d_rowptr, d_colidx, first["g2l"].clamp(min=0) % K, (p + 1) % K)
            assert other["n_loc"] > 0 and float(d_X.sum()) == float(d_X.sum())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert held["sizes"].cpu().tolist() == [n_loc, nnz_loc], f"replay {replay}"
        assert torch.equal(tr.dW, eager["dW"]), f"replay {replay}: gradients differ from the eager step"
        assert torch.equal(tr.loss, eager["loss"]), f"replay {replay}: loss"
        assert torch.equal(tr.W, eager["W"]) and torch.equal(W_global, eager["G"]), f"replay {replay}: weights"
        assert all(torch.equal(w, e) for w, e in zip(peers, eager["peers"])), f"replay {replay}: peers"
