"""The tolerance helper of the whole-step parity tests, checked on the CPU against the oracle itself: decisions are
flipped ON THE ORACLE'S SIDE at a few entries and the change of every gradient must stay under the bound the helper
derives for those entries (and the bound must not be vacuous).  Also the near-zero asserts and the bf16 rounding of
the as-stored pass."""
import numpy as np
import pytest

import decisions
import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth

torch = pytest.importorskip("torch")


def _f64(params):
    return [tuple(np.asarray(t, dtype=np.float64) for t in l) for l in params]


def _params(encoder, dims, norm_act, seed=5):
    rng = np.random.default_rng(seed)
    out = []
    for l, (Ws, Wn, b) in enumerate(synth.sage_params(dims, seed=seed)):
        layer = [Ws, Wn, b] if encoder == "sage" else [Ws, b]
        if norm_act and l < len(dims) - 2:
            layer += [rng.normal(1.0, 0.2, dims[l + 1]), rng.normal(0.0, 0.2, dims[l + 1]), np.array([0.25])]
        out.append(tuple(layer))
    return _f64(out)


def _random_flips(pre_list, rng, k=3):
    D = []
    for pre in pre_list:
        if pre is None:
            D.append(None)
            continue
        d = np.zeros(pre.shape, dtype=bool)
        d[rng.integers(0, pre.shape[0], k), rng.integers(0, pre.shape[1], k)] = True
        D.append(d)
    return D


def _flipped(pre_list, D):
    return [None if p is None else (p > 0) ^ d for p, d in zip(pre_list, D)]


@pytest.mark.parametrize("encoder,norm_act", [("sage", False), ("sage", True), ("gcn", False), ("gcn", True),
                                              ("mlp", False)])
def test_bounds_cover_flipped_decisions_node_task(encoder, norm_act):
    rng = np.random.default_rng(3)
    rowptr, colidx = synth.uniform_graph(300, 900, seed=2)
    dims = [12, 20, 16, 5]
    X, y = synth.features(300, dims[0], seed=3), synth.labels(300, dims[-1], seed=4)
    params = _params(encoder, dims, norm_act)
    tr = {}
    _, g0, _, saved = omodel.loss_and_grads(rowptr, colidx, X, y, params, encoder=encoder, trace=tr)
    for trial in range(4):
        D = _random_flips(tr["pre"], rng)
        _, g1, _, _ = omodel.loss_and_grads(rowptr, colidx, X, y, params, _flipped(tr["pre"], D), encoder)
        bounds = decisions.encoder_bounds(encoder, rowptr, colidx, params, saved, tr["ups"], D)
        worst = 0.0
        for l in range(3):
            assert len(bounds[l]) == len(g0[l])
            for a, b, bd in zip(g0[l], g1[l], bounds[l]):
                change = np.linalg.norm(np.ravel(np.asarray(b) - np.asarray(a)))
                assert change <= bd * (1 + 1e-9) + 1e-15, (l, change, bd)
                worst = max(worst, change / max(bd, 1e-300))
        assert worst > 0.02          # not vacuous: some tensor's change reaches a few percent of its bound


def test_bounds_cover_flipped_decisions_sampled_link_task():
    rng = np.random.default_rng(8)
    rowptr, colidx = synth.chung_lu_graph(600, 8, 2.1, seed=1)
    dims, fanouts, Bn = [10, 14, 8], [3, 4], 40
    X = synth.features(600, dims[0], seed=2)
    enc = _params("sage", dims, True)
    dec = _f64([(synth.glorot(8, 9, rng), np.array([0.25])), (synth.glorot(9, 6, rng), np.array([0.1])),
                (synth.glorot(6, 1, rng),)])
    batch = oracle.edge_batch(rowptr, colidx, 7, 0, Bn)
    tr = {}
    _, ge0, gd0, _, (rps, cis, _, _) = omodel.sampled_link_loss_and_grads(rowptr, colidx, X, batch, enc, dec, fanouts,
                                                                           7, 0, trace=tr)
    for trial in range(4):
        D, Dd = _random_flips(tr["pre"], rng), _random_flips(tr["dec_pre"], rng)
        _, ge1, gd1, _, _ = omodel.sampled_link_loss_and_grads(rowptr, colidx, X, batch, enc, dec, fanouts, 7, 0,
                                                               _flipped(tr["pre"], D), _flipped(tr["dec_pre"], Dd))
        db, q_top = decisions.decoder_bounds(dec, tr["dsaved"], tr["dec_ups"], Dd, tr["R"], tr["batch_pos"])
        eb = decisions.encoder_bounds("sage", rps, cis, enc, tr["saved"], tr["ups"], D, q_top)
        for g0, g1, bounds in ((ge0, ge1, eb), (gd0, gd1, db)):
            for l in range(len(g0)):
                assert len(bounds[l]) == len(g0[l])
                for a, b, bd in zip(g0[l], g1[l], bounds[l]):
                    change = np.linalg.norm(np.ravel(np.asarray(b) - np.asarray(a)))
                    assert change <= bd * (1 + 1e-9) + 1e-15, (l, change, bd)


def test_full_graph_link_task_bounds():
    rng = np.random.default_rng(9)
    rowptr, colidx = synth.uniform_graph(200, 700, seed=5)
    dims, Bn = [10, 12, 8], 64
    X = synth.features(200, dims[0], seed=2)
    enc = _params("gcn", dims, False)
    dec = _f64([(synth.glorot(8, 9, rng), np.array([0.25])), (synth.glorot(9, 1, rng),)])
    batch = oracle.edge_batch(rowptr, colidx, 7, 0, Bn)
    tr = {}
    _, ge0, gd0, _ = omodel.link_loss_and_grads(rowptr, colidx, X, batch, enc, dec, "gcn", trace=tr)
    D, Dd = _random_flips(tr["pre"], rng), _random_flips(tr["dec_pre"], rng)
    _, ge1, gd1, _ = omodel.link_loss_and_grads(rowptr, colidx, X, batch, enc, dec, "gcn", _flipped(tr["pre"], D),
                                                _flipped(tr["dec_pre"], Dd))
    db, q_top = decisions.decoder_bounds(dec, tr["dsaved"], tr["dec_ups"], Dd, tr["R"], tr["batch_pos"])
    eb = decisions.encoder_bounds("gcn", rowptr, colidx, enc, tr["saved"], tr["ups"], D, q_top)
    for g0, g1, bounds in ((ge0, ge1, eb), (gd0, gd1, db)):
        for l in range(len(g0)):
            for a, b, bd in zip(g0[l], g1[l], bounds[l]):
                assert np.linalg.norm(np.ravel(np.asarray(b) - np.asarray(a))) <= bd * (1 + 1e-9) + 1e-15


def test_check_rejects_a_wrong_sign_away_from_zero_and_accepts_one_next_to_it():
    rng = np.random.default_rng(0)
    pre = rng.standard_normal((500, 64))
    pre[3, 5] = 1e-9
    ok = pre > 0
    assert not decisions.check(ok, pre, "same").any()
    flipped = ok.copy()
    flipped[3, 5] = False                                   # within rounding distance of zero: either side is fine
    D = decisions.check(flipped, pre, "near zero")
    assert D.sum() == 1 and D[3, 5]
    wrong = ok.copy()
    wrong[10, 10] = not wrong[10, 10]                       # |pre| ~ 1: a wrong mask
    with pytest.raises(AssertionError, match="not near zero"):
        decisions.check(wrong, pre, "wrong")
    crowded = np.full((100, 100), 1e-12)
    crowded[0, 0] = 1.0
    with pytest.raises(AssertionError, match="rms of zero"):
        decisions.check(crowded > 0, crowded, "crowded")


def test_round_bf16_against_a_library_and_by_hand():
    x = (np.random.default_rng(1).standard_normal(200_000) * 37.0).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_bf16(x), want)
    # 8 significant bits, ties to even: 1 + 2^-8 -> 1, 1 + 3 * 2^-8 -> 1 + 2^-6, exact values unchanged
    assert np.array_equal(oracle.round_bf16([1 + 2**-8, 1 + 3 * 2**-8, -1 - 2**-8, 0.0, 0.375, 256.0 + 1.0]),
                          [1.0, 1 + 2**-6, -1.0, 0.0, 0.375, 256.0])


def test_as_stored_pass_equals_the_plain_pass_when_nothing_needs_rounding():
    """With inputs, weights and every intermediate exactly representable (small integers, identity-like weights) the
    as-stored pass must reproduce the fp64 pass: it only rounds, it does not compute anything else."""
    rowptr = np.array([0, 2, 4, 6, 8], dtype=np.int32)                  # a 4-cycle: every mean is a half-integer
    colidx = np.array([1, 3, 0, 2, 1, 3, 0, 2], dtype=np.int32)
    X = np.array([[2, -4], [6, 8], [-2, 4], [10, -8]], dtype=np.float64)
    params = [(np.eye(2), 2 * np.eye(2), np.array([1.0, -1.0])), (np.eye(2), np.eye(2), np.zeros(2))]
    out, saved = omodel.forward(rowptr, colidx, X, params)
    out_s, pre = omodel.forward_as_stored(rowptr, colidx, X, params, "sage", "bf16")
    assert np.array_equal(out, out_s) and np.array_equal(pre[0], saved[0][2]) and pre[1] is None
    # and it does round: a weight with more than 8 significant bits moves the result by about 2^-9 of it
    params[0] = (np.eye(2) * (1 + 2**-10), 2 * np.eye(2), np.array([1.0, -1.0]))
    out2, _ = omodel.forward(rowptr, colidx, X, params)
    out2_s, _ = omodel.forward_as_stored(rowptr, colidx, X, params, "sage", "bf16")
    assert np.array_equal(out2_s, out_s) and not np.array_equal(out2, out)


@pytest.mark.parametrize("encoder", ["sage", "gcn"])
def test_as_stored_pass_in_both_layer_forms_follows_the_plain_pass(encoder):
    """Aggregate-first and transform-first are the same function (linearity); with fp32 storage the as-stored pass
    stays within fp32 rounding of the fp64 pass in either form, with bf16 storage within a few 2^-9."""
    rp, ci = synth.uniform_graph(200, 600, seed=1)
    X = synth.features(200, 6, seed=2)
    P = _params(encoder, [6, 8, 4], False, seed=3)
    out, saved = omodel.forward(rp, ci, X, P, encoder)
    for forms in ([True, True], [False, False], None):
        a, pre = omodel.forward_as_stored(rp, ci, X, P, encoder, "f32", forms)
        assert np.abs(a - out).max() <= 1e-6 * np.abs(out).max()
        assert np.abs(pre[0] - saved[0][2]).max() <= 1e-6 * np.abs(saved[0][2]).max() and pre[1] is None
        b, _ = omodel.forward_as_stored(rp, ci, X, P, encoder, "bf16", forms)
        assert 1e-4 < np.abs(b - out).max() / np.abs(out).max() <= 3e-2
