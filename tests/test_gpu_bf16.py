"""bf16 storage path (features, activations and their gradients in bf16; weights, weight gradients and
accumulation in fp32) against the fp64 oracle fed with the same bf16-rounded inputs.  Tolerance 2e-2."""
import numpy as np
import pytest

import decisions
import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 2e-2


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
    """fp32 array holding bf16-representable values -> bf16 GPU tensor with the same values."""
    bits = synth.to_bf16_bits(np.asarray(a, dtype=np.float32)).reshape(np.shape(a))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def host(t):
    return t.float().cpu().numpy()


def close(got, want, what, tol=TOL):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, what
    rel = np.linalg.norm((got - want).ravel()) / max(np.linalg.norm(want.ravel()), 1e-300)
    mx = np.abs(got - want).max() / max(np.abs(want).max(), 1e-300)
    assert rel <= tol and mx <= tol, f"{what}: rel fro {rel:.2e}, max abs / max {mx:.2e}"


def _sub(n, m, seed):
    rowptr, colidx = synth.uniform_graph(n, m, seed)
    return oracle.induced_subgraph(rowptr, colidx, oracle.partition(n, 2, seed=seed), 0)


@pytest.mark.parametrize("F", [100, 128, 8, 6])
def test_mean_aggregate_bf16(B, F):
    sub = _sub(6000, 30_000, F)
    n = len(sub["l2g"])
    H = synth.round_bf16(synth.features(n, F, seed=1))
    got = B.tma_mean_aggregate(dev(sub["rowptr"]), dev(sub["colidx"]), dev(sub["inv_deg"], torch.float32), dev_bf16(H))
    assert got.dtype == torch.bfloat16
    close(host(got), oracle.mean_aggregate(sub["rowptr"], sub["colidx"], H), f"M F={F}")


@pytest.mark.parametrize("F,ld,bf16", [(100, 128, True), (100, 104, True), (47, 48, False), (5, 8, False), (33, 40, True)])
def test_mean_aggregate_of_a_ragged_width_in_padded_rows(B, F, ld, bf16):
    """A row width that is no multiple of 16 bytes (the SuperTMA configuration's 100 bf16 features) in rows padded to
    whole 16-byte pieces: the vector path walks the last piece too, so it may overwrite the padding elements of the
    output up to that piece -- and nothing beyond it, and the valid columns are the oracle's."""
    sub = _sub(6000, 30_000, F + ld)
    n = len(sub["l2g"])
    H = synth.features(n, F, seed=1)
    H = synth.round_bf16(H) if bf16 else H
    dt = torch.bfloat16 if bf16 else torch.float32
    per16 = 8 if bf16 else 4
    piece_end = (F + per16 - 1) // per16 * per16
    Hd = torch.full((n, ld), 3.0, dtype=dt, device="cuda")            # finite padding, as a caller's zero-fill would be
    Hd[:, :F] = dev_bf16(H) if bf16 else dev(H)
    out = torch.full((n, ld), -7.0, dtype=dt, device="cuda")
    got = B.tma_mean_aggregate(dev(sub["rowptr"]), dev(sub["colidx"]), dev(sub["inv_deg"], torch.float32), Hd[:, :F],
                               out=out[:, :F])
    close(host(got), oracle.mean_aggregate(sub["rowptr"], sub["colidx"], H), f"M F={F} ld={ld}", tol=TOL if bf16 else 1e-4)
    assert torch.all(out[:, piece_end:] == -7.0)                       # nothing past the last whole piece is touched
    if B.lib() is not None and ld * (2 if bf16 else 4) % 16 == 0:
        # the name of the kernel that ran: the streaming kernel, not the element-wise fallback
        B.tma_profile_begin(None)
        B.tma_mean_aggregate(dev(sub["rowptr"]), dev(sub["colidx"]), dev(sub["inv_deg"], torch.float32), Hd[:, :F],
                             out=out[:, :F])
        assert all("generic" not in k for k in B.tma_profile_end())


def test_sage_layer_bf16_with_100_features_in_padded_rows(B):
    """The first layer of the SuperTMA configuration (100 -> 256, bf16) with H and the saved aggregate M in rows of
    128 elements: forward and backward against the oracle, M's valid columns included."""
    sub = _sub(5000, 40_000, 77)
    rp, ci, inv = sub["rowptr"], sub["colidx"], sub["inv_deg"]
    n, F_in, F_out, ld = len(sub["l2g"]), 100, 256, 128
    H = synth.round_bf16(synth.features(n, F_in, seed=1))
    (Ws, Wn, b), = synth.sage_params([F_in, F_out], seed=2)
    M_o, Z_o, Hn_o = oracle.sage_layer_fwd(rp, ci, H, Ws, Wn, b, oracle.ACT_RELU)
    d_rp, d_ci, d_inv = dev(rp), dev(ci), dev(inv, torch.float32)
    Hd = torch.zeros((n, ld), dtype=torch.bfloat16, device="cuda")
    Hd[:, :F_in] = dev_bf16(H)
    Md = torch.zeros((n, ld), dtype=torch.bfloat16, device="cuda")
    M_g, Hn_g = B.tma_sage_layer_fwd(d_rp, d_ci, d_inv, Hd[:, :F_in], dev(Ws), dev(Wn), dev(b), oracle.ACT_RELU,
                                     M_out=Md[:, :F_in])
    close(host(M_g), M_o, "M")
    close(host(Hn_g), Hn_o, "Hnext")
    dHn = synth.round_bf16(np.random.default_rng(3).standard_normal((n, F_out)).astype(np.float32))
    Mb, Hnb = synth.round_bf16(M_o.astype(np.float32)), synth.round_bf16(Hn_o.astype(np.float32))
    Md[:, :F_in] = dev_bf16(Mb)
    want = oracle.sage_layer_bwd(rp, ci, H, Mb, Hnb, dHn, Ws, Wn, oracle.ACT_RELU, need_dH=False)
    got = B.tma_sage_layer_bwd(d_rp, d_ci, d_inv, Hd[:, :F_in], Md[:, :F_in], dev_bf16(Hnb), dev_bf16(dHn), dev(Ws),
                               dev(Wn), oracle.ACT_RELU, need_dH=False)
    for g, w, name in zip(got[:3], want[:3], ("dW_self", "dW_neigh", "dbias")):
        close(host(g), w, name)


@pytest.mark.parametrize("n_glob,m,F_in,F_out,act", [(4000, 20_000, 100, 256, "relu"), (3000, 12_000, 256, 47, "none"),
                                                     (1200, 5000, 30, 10, "relu")])
def test_sage_layer_bf16(B, n_glob, m, F_in, F_out, act):
    sub = _sub(n_glob, m, F_in + F_out)
    rp, ci, inv = sub["rowptr"], sub["colidx"], sub["inv_deg"]
    n = len(sub["l2g"])
    H = synth.round_bf16(synth.features(n, F_in, seed=1))
    (Ws, Wn, b), = synth.sage_params([F_in, F_out], seed=2)
    a = oracle.ACT_RELU if act == "relu" else oracle.ACT_NONE
    M_o, Z_o, Hn_o = oracle.sage_layer_fwd(rp, ci, H, Ws, Wn, b, a)
    d_rp, d_ci, d_inv = dev(rp), dev(ci), dev(inv, torch.float32)
    M_g, Hn_g = B.tma_sage_layer_fwd(d_rp, d_ci, d_inv, dev_bf16(H), dev(Ws), dev(Wn), dev(b), a)
    assert M_g.dtype == torch.bfloat16 and Hn_g.dtype == torch.bfloat16
    if B.tma_sage_layer_aggregates_first(F_in, F_out, B.TMA_BF16):     # otherwise M_out is scratch
        close(host(M_g), M_o, "M")
    close(host(Hn_g), Hn_o, "Hnext")

    rng = np.random.default_rng(3)
    dHn = synth.round_bf16(rng.standard_normal((n, F_out)).astype(np.float32))
    Mb, Hnb = synth.round_bf16(M_o.astype(np.float32)), synth.round_bf16(Hn_o.astype(np.float32))
    want = oracle.sage_layer_bwd(rp, ci, H, Mb, Hnb if a == oracle.ACT_RELU else Z_o, dHn, Ws, Wn, a)
    got = B.tma_sage_layer_bwd(d_rp, d_ci, d_inv, dev_bf16(H), dev_bf16(Mb), dev_bf16(Hnb), dev_bf16(dHn), dev(Ws),
                               dev(Wn), a)
    for g, w, name in zip(got, want, ("dW_self", "dW_neigh", "dbias", "dH")):
        assert g.dtype == (torch.bfloat16 if name == "dH" else torch.float32)
        close(host(g), w, name)


@pytest.mark.parametrize("n_glob,m,F_in,F_out,act", [(9000, 40_000, 128, 256, "relu"), (4000, 20_000, 100, 256, "relu"),
                                                     (5000, 20_000, 64, 48, "none"), (70_000, 300_000, 32, 320, "relu"),
                                                     (3000, 12_000, 256, 47, "none"), (1200, 5000, 30, 10, "relu")])
def test_sage_layer_bf16_with_prepared_weights(B, n_glob, m, F_in, F_out, act):
    """tma_sage_prepare_weights_bf16 + tma_sage_layer_fwd_prepared: the weight operand narrowed once instead of in
    every tile.  The prepared array against the definition (bf16 round-to-nearest-even of the transposed, stacked
    weights, taken on the host), the layer against the oracle and bit for bit against tma_sage_layer_fwd; widths for
    every tile shape, one layer that transforms first and one whose rows have no groups of four (both run as
    without the array)."""
    sub = _sub(n_glob, m, F_in + F_out)
    rp, ci, inv = sub["rowptr"], sub["colidx"], sub["inv_deg"]
    n = len(sub["l2g"])
    H = synth.round_bf16(synth.features(n, F_in, seed=1))
    (Ws, Wn, b), = synth.sage_params([F_in, F_out], seed=2)
    a = oracle.ACT_RELU if act == "relu" else oracle.ACT_NONE
    d_rp, d_ci, d_inv, d_H = dev(rp), dev(ci), dev(inv, torch.float32), dev_bf16(H)
    d_Ws, d_Wn, d_b = dev(Ws), dev(Wn), dev(b)
    Wt = B.tma_sage_prepare_weights_bf16(d_Ws, d_Wn)
    assert Wt.numel() * 2 == B.tma_sage_weights_bf16_bytes(F_in, F_out) and Wt.numel() * 2 % 256 == 0
    want_bits = synth.to_bf16_bits(np.ascontiguousarray(np.concatenate([Ws, Wn], axis=0).T.astype(np.float32)))
    assert np.array_equal(Wt.cpu().numpy()[:2 * F_in * F_out].view(np.uint16), want_bits.ravel())
    M_p, Hn_p = B.tma_sage_layer_fwd(d_rp, d_ci, d_inv, d_H, d_Ws, d_Wn, d_b, a, Wt=Wt)
    M_g, Hn_g = B.tma_sage_layer_fwd(d_rp, d_ci, d_inv, d_H, d_Ws, d_Wn, d_b, a)
    assert torch.equal(Hn_p.view(torch.int16), Hn_g.view(torch.int16))
    M_o, _, Hn_o = oracle.sage_layer_fwd(rp, ci, H, Ws, Wn, b, a)
    if B.tma_sage_layer_aggregates_first(F_in, F_out, B.TMA_BF16):
        assert torch.equal(M_p.view(torch.int16), M_g.view(torch.int16))
        close(host(M_p), M_o, "M")
    close(host(Hn_p), Hn_o, "Hnext")


def test_losses_and_gather_bf16(B):
    rng = np.random.default_rng(5)
    z = synth.round_bf16((3 * rng.standard_normal((3000, 47))).astype(np.float32))
    y = rng.integers(0, 47, 3000).astype(np.int32)
    loss_o, d_o = oracle.softmax_ce(z, y)
    loss, d = B.tma_softmax_ce(dev_bf16(z), dev(y))
    assert abs(loss.item() - loss_o) <= 1e-3 * abs(loss_o)
    close(host(d), d_o, "dlogits")
    idx = np.sort(rng.choice(3000, 777, replace=False)).astype(np.int32)
    got = B.tma_gather_rows(dev(idx), dev_bf16(z))
    assert np.array_equal(host(got), z[idx])


def test_three_layer_supertma_training_step_bf16(B):
    """Shape of the SuperTMA configuration, scaled down: planted communities as super-nodes, K = 16,
    100-d bf16 features with community-dependent means, 3-layer model (hidden 256)."""
    from paper_2305_09887_amd.trainer import LocalTrainer
    nb, bs, K, dims = 160, 100, 16, [100, 256, 256, 47]
    rowptr, colidx, block = synth.sbm_graph(nb, bs, 36_000, 4_000, seed=21)
    N = nb * bs
    X = synth.round_bf16(synth.community_features(block, nb, dims[0], seed=22))
    y = (block % dims[-1]).astype(np.int32)
    params = synth.sage_params(dims, seed=25)
    part = B.tma_partition(N, K, seed=24, cluster=dev(block), n_clusters=nb)
    part_o = oracle.partition(N, K, seed=24, cluster=block)
    assert np.array_equal(part.cpu().numpy(), part_o)
    p = int(np.bincount(part_o, minlength=K).argmax())
    sub = B.tma_induced_subgraph(dev(rowptr), dev(colidx), part, p)
    so = oracle.induced_subgraph(rowptr, colidx, part_o, p)
    assert np.array_equal(sub["colidx"].cpu().numpy(), so["colidx"]) and sub["n_loc"] >= 2 * bs
    Xl = B.tma_gather_rows(sub["l2g"], dev_bf16(X))
    yl = B.tma_gather_rows(sub["l2g"], dev(y))
    tr = LocalTrainer(sub["rowptr"], sub["colidx"], sub["inv_deg"], Xl, yl, dims, params=params)
    loss_g = tr.step(0.01).item()
    p_o = [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in params]
    # activation decisions in the path's precision: the oracle's as-stored pass (bf16 storage of M and H', bf16 weight
    # operands) decides, its fp64 pass gives the expected values; the GPU's sign patterns are only compared
    t = {}
    loss_o, grads_o, logits_o, saved = omodel.loss_and_grads(so["rowptr"], so["colidx"], X[so["l2g"]], y[so["l2g"]], p_o,
                                                              decisions="bf16", trace=t)
    D = decisions.differing(t["pre"], [host(tr.H[1]), host(tr.H[2]), None], "SuperTMA bf16 step", **decisions.STORED)
    bounds = decisions.encoder_bounds("sage", so["rowptr"], so["colidx"], p_o, saved, t["ups"], D)
    print("differing decisions per layer:", [int(d.sum()) for d in D[:2]], "of", D[0].size, "; allowed change", bounds)
    assert abs(loss_g - loss_o) <= TOL * abs(loss_o)
    close(host(tr.H[3]), logits_o, "logits")
    for l in range(3):
        for g, w, bd, name in zip(tr.grads[l], grads_o[l], bounds[l], ("dW_self", "dW_neigh", "dbias")):
            print(f"layer {l} {name}: rel fro err {np.linalg.norm(host(g) - w) / np.linalg.norm(w):.2e}, "
                  f"allowed change / norm {bd / np.linalg.norm(w):.2e}")
            decisions.close(host(g), w, TOL, f"layer {l} {name}", extra=bd)
