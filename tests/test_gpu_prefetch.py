"""The next step's partition + extraction on a second stream while the current step trains: the same weights, bit
for bit, as the same steps run one after the other on one stream (every kernel is deterministic), with another
assignment seed, hence another subgraph of another size, at every step."""
import numpy as np
import pytest

from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _run(prefetch: bool, steps: int):
    from paper_2305_09887_amd import binding as B
    from paper_2305_09887_amd.trainer import LocalTrainer, SubgraphPrefetcher
    N, K, p, dims = 20_000, 4, 0, [64, 64, 16]
    rowptr, colidx = synth.uniform_graph(N, 100_000, seed=1)
    d = lambda a: torch.as_tensor(a).cuda()
    d_rp, d_ci = d(rowptr), d(colidx)
    d_X, d_y = d(synth.features(N, dims[0], seed=2)), d(synth.labels(N, dims[-1], seed=3))
    cap, cap_nnz = N // K + N // 16, int(rowptr[-1]) // (K * K) * 2 + 4096
    pf = SubgraphPrefetcher(d_rp, d_ci, N, K, p, cap, cap_nnz, tables=(d_X, d_y)) if prefetch else None
    part = torch.empty(N, dtype=torch.int32, device="cuda")
    W = torch.as_tensor(np.concatenate([np.asarray(t, np.float32).ravel() for l in synth.sage_params(dims, seed=5)
                                        for t in l])).cuda()
    nxt, trained, sizes, loss = None, None, [], None
    for t in range(steps):
        if pf is None:
            B.tma_partition(N, K, 100 + t, out=part)
            s = B.tma_induced_subgraph(d_rp, d_ci, part, p, cap_n_loc=cap, cap_nnz_loc=cap_nnz)
        else:
            if nxt is None:
                nxt = pf.start(100 + t)
            s, (Xl, yl), ready = nxt
            torch.cuda.current_stream().wait_event(ready)
        sizes.append((s["n_loc"], s["nnz_loc"]))
        if pf is None:
            Xl, yl = B.tma_gather_rows(s["l2g"], d_X), B.tma_gather_rows(s["l2g"], d_y)
        # the trainer's buffers are sized for one node count: a new one per step, carrying the weights over
        tr = LocalTrainer(s["rowptr"], s["colidx"], s["inv_deg"], Xl, yl, dims)
        assert tr.W.numel() == W.numel()
        tr.W.copy_(W)
        loss = tr.step(0.05)
        W = tr.W
        if pf is not None:
            done = torch.cuda.Event()
            done.record()
            nxt = pf.start(100 + t + 1, after=trained)
            trained = done
    torch.cuda.synchronize()
    return W.cpu().numpy().copy(), float(loss.item()), sizes


def test_prefetched_extraction_gives_the_same_weights():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    W_seq, loss_seq, sizes_seq = _run(False, 6)
    W_pre, loss_pre, sizes_pre = _run(True, 6)
    assert sizes_seq == sizes_pre and len(set(sizes_seq)) > 1      # the subgraph changes from step to step
    assert np.isfinite(W_seq).all() and loss_seq == loss_pre
    assert np.array_equal(W_seq, W_pre)
