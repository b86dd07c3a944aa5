"""One trainer's share at the largest configured size (12.5 M local nodes, bf16 features, width 256): every
activation matrix holds 3.2e9 elements, so row * leading-dimension products pass 2^31 and byte offsets pass 2^32
inside every kernel.  The oracle cannot run 12.5 M rows in a test; it computes SAMPLED rows one by one instead:
for a set S of rows (first, last, and random ones on both sides of the 2^31-element line) the sub-problem
"S plus its neighbours" is extracted, relabelled and given to the oracle, whose rows for S are compared with the
GPU's rows for S.  The weight gradient, a sum over all rows, is checked with an upstream gradient that is nonzero
on S only: the kernel still walks all 12.5 M rows, the oracle needs S alone.

The graph is a symmetric circulant-style graph built on the GPU in closed form (edge {v, v+o} present when
v mod p = 0, for a few (o, p)): degrees 0..8, no host generation time."""
import numpy as np
import pytest

import decisions
import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

N = 12_500_000
F = 256
OFFSETS = [(1, 2), (7_919, 3), (1_000_003, 5), (6_250_001, 1)]   # (offset, period)


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if torch.cuda.get_device_properties(0).total_memory < 100 * 2**30:
        pytest.skip("needs about 60 GB of device memory")
    from paper_2305_09887_amd import binding
    binding.lib()
    return binding


def _graph(n, offsets=None, wide_rowptr=False):
    """Symmetric CSR on the GPU: row v holds v+o (if v % p == 0) and v-o (if (v-o) % p == 0) for each (o, p)."""
    v = torch.arange(n, device="cuda", dtype=torch.int64)
    cols, keep = [], []
    for o, p in (offsets or OFFSETS):
        cols.append((v + o) % n); keep.append(v % p == 0)
        w = (v - o) % n
        cols.append(w); keep.append(w % p == 0)
    cols, keep = torch.stack(cols, 1), torch.stack(keep, 1)
    deg = keep.sum(1)
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    rowptr[1:] = torch.cumsum(deg, 0)
    colidx = cols[keep].to(torch.int32)                        # row-major order = CSR order
    inv_deg = torch.where(deg > 0, 1.0 / deg.clamp(min=1).float(), torch.zeros((), device="cuda"))
    return (rowptr if wide_rowptr else rowptr.to(torch.int32)), colidx, inv_deg.float(), deg


def _sample_rows(n, _deg, k=600):
    rng = np.random.default_rng(5)
    line = 2**31 // F                                          # first row whose elements lie past 2^31
    S = np.concatenate([[0, 1, n - 2, n - 1, line - 1, line, line + 1],
                        rng.integers(0, line, k // 3), rng.integers(line, n, k - k // 3)])
    return np.unique(S).astype(np.int64)


def _sub_problem(S, rowptr, colidx):
    """Rows S with their neighbour lists, relabelled onto U = S u N(S).  Returns (U, rowptr_sub, colidx_sub, pos of S in U)."""
    rp = rowptr.cpu().numpy().astype(np.int64)
    lists = [colidx[rp[v]:rp[v + 1]].cpu().numpy().astype(np.int64) for v in S]
    U = np.unique(np.concatenate([S] + lists))
    pos = {int(u): i for i, u in enumerate(U)}
    sub_rp = np.zeros(len(U) + 1, dtype=np.int32)
    rows = {int(v): l for v, l in zip(S, lists)}
    for i, u in enumerate(U):
        sub_rp[i + 1] = sub_rp[i] + (len(rows[int(u)]) if int(u) in rows else 0)
    sub_ci = np.array([pos[int(c)] for u in U if int(u) in rows for c in rows[int(u)]], dtype=np.int32)
    return U, sub_rp, sub_ci, np.array([pos[int(v)] for v in S])


def _rows(t, idx):
    return t[torch.as_tensor(idx, device="cuda")].float().cpu().numpy().astype(np.float64)


def _close(got, want, tol, what):
    rel = np.linalg.norm((got - want).ravel()) / max(np.linalg.norm(want.ravel()), 1e-300)
    mx = np.abs(got - want).max() / max(np.abs(want).max(), 1e-300)
    assert rel <= tol and mx <= tol, f"{what}: rel fro {rel:.2e}, max abs / max {mx:.2e}"


def test_layer_forward_and_backward_at_12_5_million_rows(B):
    rowptr, colidx, inv_deg, deg = _graph(N)
    assert int(rowptr[-1]) == colidx.numel() and colidx.numel() > 3 * N
    S = _sample_rows(N, deg)
    U, sub_rp, sub_ci, s_in_u = _sub_problem(S, rowptr, colidx)

    torch.manual_seed(1)
    H = torch.empty((N, F), dtype=torch.bfloat16, device="cuda")
    for a in range(0, N, 2_500_000):                           # filled in slices: no fp32 copy of the whole matrix
        H[a:a + 2_500_000] = torch.randn((min(2_500_000, N - a), F), device="cuda").to(torch.bfloat16)
    assert H.numel() > 2**31
    params = synth.sage_params([F, F], seed=3)[0]
    Ws, Wn, b = (torch.as_tensor(p).cuda() for p in params)

    # forward: M = Abar H, H' = relu(H Ws + M Wn + b); rows of S against the oracle on the sub-problem
    M, Hn = B.tma_sage_layer_fwd(rowptr, colidx, inv_deg, H, Ws, Wn, b, B.TMA_ACT_RELU)
    Hu = _rows(H, U)
    M_o, Z_o, Hn_o = oracle.sage_layer_fwd(sub_rp, sub_ci, Hu, params[0], params[1], params[2], oracle.ACT_RELU)
    _close(_rows(M, S), M_o[s_in_u], 2e-2, "M on sampled rows")
    _close(_rows(Hn, S), Hn_o[s_in_u], 2e-2, "H' on sampled rows")

    # backward with an upstream gradient that lives on S only
    dHn = torch.zeros((N, F), dtype=torch.bfloat16, device="cuda")
    g = synth.round_bf16(np.random.default_rng(2).normal(0, 1, (len(S), F)).astype(np.float32))
    bits = synth.to_bf16_bits(g).reshape(g.shape)
    dHn[torch.as_tensor(S, device="cuda")] = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    dWs, dWn, db, dH = B.tma_sage_layer_bwd(rowptr, colidx, inv_deg, H, M, Hn, dHn, Ws, Wn, B.TMA_ACT_RELU, need_dH=True)
    torch.cuda.synchronize()
    # the oracle's sub-problem for backward: rows of U with the oracle's own H, M and Z; dZ is nonzero on S only, so
    # graph rows outside S are not needed.  The ReLU decision is taken in the path's precision by the oracle's
    # as-stored pass (bf16 M and H', bf16 weight operands); the GPU's sign pattern on S is only compared with it.
    p64 = [tuple(np.asarray(t, dtype=np.float64) for t in params)]
    _, pre = omodel.forward_as_stored(sub_rp, sub_ci, Hu, p64, "sage", "bf16", final_relu=True)
    D = np.zeros(pre[0].shape, dtype=bool)
    D[s_in_u] = decisions.check(_rows(Hn, S) > 0, pre[0][s_in_u], "ReLU on the sampled rows", **decisions.STORED)
    dHn_u = np.zeros((len(U), F))
    dHn_u[s_in_u] = g
    (bWs, bWn, bb), = decisions.encoder_bounds("sage", sub_rp, sub_ci, p64, [(Hu, M_o, Z_o, oracle.ACT_RELU)], [dHn_u], [D])
    dWs_o, dWn_o, db_o, dH_o = oracle.sage_layer_bwd(sub_rp, sub_ci, Hu, M_o, pre[0], dHn_u, params[0], params[1],
                                                     oracle.ACT_RELU, need_dH=True)
    decisions.close(dWs.cpu().numpy(), dWs_o, 2e-2, "dW_self", extra=bWs)
    decisions.close(dWn.cpu().numpy(), dWn_o, 2e-2, "dW_neigh", extra=bWn)
    decisions.close(db.cpu().numpy(), db_o, 2e-2, "dbias", extra=bb)
    # dH_v = dZ_v Ws^T + sum_{u in N(v)} inv_deg[u] dZ_u Wn^T (the graph is symmetric).  dZ lives on S, so dH is
    # nonzero on S u N(S) = U, and the oracle's scatter over the sampled rows' lists gives exactly those rows
    spec = np.linalg.norm(np.asarray(params[0], np.float64), 2) + np.linalg.norm(np.asarray(params[1], np.float64), 2)
    decisions.close(_rows(dH, U), dH_o, 2e-2, "dH on S and its neighbours", extra=bb * spec)
    far = np.setdiff1d(np.random.default_rng(9).integers(0, N, 2000), U)
    assert not _rows(dH, far).any()                            # untouched rows are exact zeros


def test_row_wise_kernels_at_12_5_million_rows(B):
    """Normalisation + PReLU and the loss on matrices of more than 2^31 elements.  Sampled rows against the oracle;
    the column sums of the normalisation's backward pass with an upstream gradient that lives on the sample."""
    S = _sample_rows(N, None)
    idx = torch.as_tensor(S, device="cuda")
    torch.manual_seed(4)
    Z = torch.empty((N, F), dtype=torch.bfloat16, device="cuda")
    for a in range(0, N, 2_500_000):
        Z[a:a + 2_500_000] = (torch.randn((min(2_500_000, N - a), F), device="cuda") * 1.5 + 0.2).to(torch.bfloat16)
    rng = np.random.default_rng(6)
    gamma, beta = rng.normal(1, 0.2, F).astype(np.float32), rng.normal(0, 0.3, F).astype(np.float32)
    d = lambda a: torch.as_tensor(a).cuda()
    slope = torch.tensor([0.25], device="cuda")
    H = B.tma_layernorm_prelu_fwd(Z, d(gamma), d(beta), slope)
    Zs = _rows(Z, S)
    _close(_rows(H, S), oracle.layernorm_prelu_fwd(Zs, gamma, beta, 0.25), 2e-2, "H' on sampled rows")
    g = synth.round_bf16(rng.normal(0, 1, (len(S), F)).astype(np.float32))
    dH = torch.zeros((N, F), dtype=torch.bfloat16, device="cuda")
    dH[idx] = torch.from_numpy(synth.to_bf16_bits(g).reshape(g.shape).view(np.int16)).cuda().view(torch.bfloat16)
    dZ, dga, dbe, dsl = B.tma_layernorm_prelu_bwd(Z, dH, d(gamma), d(beta), slope, dZ_out=dH)
    wZ, wga, wbe, wsl = oracle.layernorm_prelu_bwd(Zs, g, gamma, beta, 0.25)
    # both sides normalise the same bf16 Z (the kernel in fp32): its decisions may differ only next to zero
    D = decisions.check(_rows(H, S) > 0, decisions.prelu_pre(oracle.layernorm_prelu_fwd(Zs, gamma, beta, 0.25), 0.25),
                        "PReLU on the sampled rows")
    bZ, bga, bbe, bsl = decisions.ln_prelu_bounds(Zs, g, gamma, beta, 0.25, D)
    decisions.close(_rows(dZ, S), wZ, 2e-2, "dZ on sampled rows", extra=bZ)
    decisions.close(dga.cpu().numpy(), wga, 2e-2, "dgamma", extra=bga)
    decisions.close(dbe.cpu().numpy(), wbe, 2e-2, "dbeta", extra=bbe)
    assert abs(dsl.item() - wsl) <= 2e-2 * abs(wsl) + bsl
    del Z, H, dH, dZ
    # loss: equal logits in every row give log(C) exactly and (1/C - onehot)/n as gradient
    C = 47
    logits = B._padded(N, C, torch.float32, "cuda")
    logits.fill_(0.375)
    labels = (torch.arange(N, device="cuda") % C).to(torch.int32)
    loss, dl = B.tma_softmax_ce(logits, labels)
    assert abs(loss.item() - np.log(C)) <= 1e-5
    got = _rows(dl, S)
    want = np.full((len(S), C), 1.0 / C) - np.eye(C)[S % C]
    _close(got * N, want, 1e-4, "dlogits on sampled rows")


def test_partition_and_extraction_at_100_million_nodes(B):
    """The global side of the same configuration: 100 M nodes, about 400 M CSR entries, K = 8.  Partition ids and
    every array of the extracted part are compared bit for bit with the oracle run on the downloaded graph."""
    n, K, p = 100_000_000, 8, 0
    rowptr, colidx, _, _ = _graph(n, offsets=[(1, 2), (104_729, 3), (15_485_863, 5), (50_000_017, 1)], wide_rowptr=True)
    assert colidx.numel() > 4 * n and int(rowptr[-1]) == colidx.numel()
    part = B.tma_partition(n, K, seed=77)
    part_o = oracle.partition(n, K, seed=77)
    assert np.array_equal(part.cpu().numpy(), part_o)
    sub = B.tma_induced_subgraph(rowptr, colidx, part, p)
    torch.cuda.synchronize()
    want = oracle.induced_subgraph(rowptr.cpu().numpy(), colidx.cpu().numpy(), part_o, p)
    assert sub["n_loc"] == len(want["l2g"]) and sub["nnz_loc"] == len(want["colidx"])
    assert abs(sub["n_loc"] / n - 1 / K) < 1e-3 and abs(sub["nnz_loc"] / colidx.numel() - 1 / K**2) < 1e-3
    for key in ("g2l", "l2g", "rowptr", "colidx"):
        assert np.array_equal(sub[key].cpu().numpy(), want[key]), key
    assert np.array_equal(sub["inv_deg"].cpu().numpy(), want["inv_deg"].astype(np.float32))
