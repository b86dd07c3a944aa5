"""Sampled message-flow graphs (Sec. 4.1: GraphSAGE-style neighbour sampling) on the GPU against the oracle,
through the C ABI: the sampled blocks and the relabelled node lists bit for bit, the SAGE layer on a bipartite
block forward and backward to 1e-4 (fp32) / 2e-2 (bf16)."""
import numpy as np
import pytest

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
    # a star: the centre has 5000 neighbours, more than the keys a wavefront keeps in LDS
    m = 5000
    rp, ci = synth.csr_from_pairs(m + 1, np.zeros(m, dtype=np.int64), np.arange(1, m + 1))
    rp, ci = rp.astype(np.int32), ci.astype(np.int32)
    dst = np.array([7, 0, 4000], dtype=np.int32)
    for fanout in (10, 4999, 5000):
        brp, bcol, _ = B.tma_neighbor_sample(dev(dst), 3, int(rp[-1]), dev(rp), dev(ci), fanout, seed=5)
        wrp, wcol = oracle.neighbor_sample(dst, rp, ci, fanout, 5)
        assert np.array_equal(brp.cpu().numpy(), wrp) and np.array_equal(bcol.cpu().numpy()[:wrp[-1]], wcol)


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
    B.tma_sage_block_bwd(n_dst, n_src, len(cols) + 17, rpd, cid, rows, inv, Hd, Md, Hn, gd, dev(Ws), dev(Wn), act, dWs, dWn,
                         db, dH_out=dH)
    Zs = np.where(host(Hn[:n_dst]) > 0, 1.0, -1.0) if act == 1 else Z
    wWs, wWn, wb, wH = oracle.sage_layer_bwd(brp, cols, H, M, Zs, g, Ws, Wn, act)
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
