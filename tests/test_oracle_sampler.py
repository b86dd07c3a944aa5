"""Pins for the oracle's fan-out neighbour sampler and message-flow graph (Sec. 4.1: the GraphSAGE sampler caps
the neighbours a node aggregates) against what the rule guarantees and against brute force: kept neighbours are a
duplicate-free subset of the row in row order, min(degree, fanout) of them; every neighbour of a large row is kept
with probability fanout / degree (frequencies over many seeds); a full fan-out reproduces the induced subgraph of
the reached nodes; the sampled step equals the full-graph step when nothing is cut."""
import numpy as np
import pytest

import oracle
from oracle import model as omodel
from paper_2305_09887_amd import synth


def _local_graph(n, m, seed, K=2, kind="uniform"):
    rowptr, colidx = (synth.uniform_graph(n, m, seed) if kind == "uniform"
                      else synth.chung_lu_graph(n, 2.0 * m / n, 2.1, seed))
    sub = oracle.induced_subgraph(rowptr, colidx, oracle.partition(n, K, seed=seed), 0)
    return sub["rowptr"], sub["colidx"]


def test_sample_is_an_ordered_subset_of_the_right_size():
    rp, ci = _local_graph(3000, 30_000, 3, kind="chung_lu")
    n = len(rp) - 1
    dst = np.random.default_rng(0).permutation(n)[:1500].astype(np.int32)
    f = 5
    brp, bcol = oracle.neighbor_sample(dst, rp, ci, f, seed=42)
    deg = np.diff(rp)[dst]
    assert np.array_equal(np.diff(brp), np.minimum(deg, f)) and (deg > f).any() and (deg < f).any()
    for i, w in enumerate(dst[:400]):
        row = ci[rp[w]:rp[w + 1]].tolist()
        kept = bcol[brp[i]:brp[i + 1]].tolist()
        assert len(set(kept)) == len(kept)
        it = iter(row)
        assert all(any(k == r for r in it) for k in kept)        # a subsequence of the row
    # deterministic in the seed, different for another seed
    assert np.array_equal(oracle.neighbor_sample(dst, rp, ci, f, 42)[1], bcol)
    assert not np.array_equal(oracle.neighbor_sample(dst, rp, ci, f, 43)[1], bcol)
    # the choice of a row does not depend on which other rows are asked for
    one = oracle.neighbor_sample(dst[7:8], rp, ci, f, 42)[1]
    assert np.array_equal(one, bcol[brp[7]:brp[8]])


def test_every_neighbour_is_kept_with_probability_fanout_over_degree():
    rp, ci = synth.csr_from_pairs(41, np.zeros(40, dtype=np.int64), np.arange(1, 41))     # a star: node 0 has 40 neighbours
    f, trials = 8, 6000
    counts = np.zeros(41)
    pair = 0
    for s in range(trials):
        kept = oracle.neighbor_sample(np.array([0], np.int32), rp, ci, f, seed=s)[1]
        assert len(kept) == f
        counts[kept] += 1
        pair += int(1 in kept and 2 in kept)
    p = f / 40
    sd = np.sqrt(trials * p * (1 - p))
    assert np.abs(counts[1:] - trials * p).max() < 5 * sd
    want_pair = trials * (f * (f - 1)) / (40 * 39)                # without replacement: pairs are negatively correlated
    assert abs(pair - want_pair) < 5 * np.sqrt(want_pair)


def test_relabel_and_full_fanout_reproduce_the_reached_subgraph():
    rp, ci = _local_graph(2000, 9000, 5)
    n = len(rp) - 1
    seeds = np.array([3, 17, 200, 999], dtype=np.int32)
    brp, bcol = oracle.neighbor_sample(seeds, rp, ci, 10**6, seed=1)
    src, cols = oracle.mfg_relabel(seeds, bcol)
    assert np.array_equal(src[:4], seeds) and np.all(np.diff(src[4:]) > 0) and len(set(src.tolist())) == len(src)
    assert np.array_equal(src[cols], bcol)
    for i, w in enumerate(seeds):
        assert np.array_equal(src[cols[brp[i]:brp[i + 1]]], ci[rp[w]:rp[w + 1]])
    # a dst node that is also somebody's neighbour keeps its dst position
    two = np.array([int(ci[rp[seeds[1]]]), int(seeds[1])], dtype=np.int32) if rp[seeds[1] + 1] > rp[seeds[1]] else None
    if two is not None:
        b2 = oracle.neighbor_sample(two, rp, ci, 10**6, seed=1)
        s2, c2 = oracle.mfg_relabel(two, b2[1])
        assert np.array_equal(s2[:2], two) and 0 in c2.tolist()


def test_sampled_step_equals_the_full_graph_step_when_nothing_is_cut():
    rp, ci = _local_graph(300, 1200, 7)
    n = len(rp) - 1
    rng = np.random.default_rng(1)
    dims = [6, 8, 5]
    enc = [(0.5 * rng.standard_normal((a, b)), 0.5 * rng.standard_normal((a, b)), 0.1 * rng.standard_normal(b))
           for a, b in zip(dims[:-1], dims[1:])]
    dec = [(0.5 * rng.standard_normal((5, 7)), np.array([0.25])), (0.5 * rng.standard_normal((7, 1)),)]
    X = rng.standard_normal((n, 6))
    batch = oracle.edge_batch(rp, ci, seed=9, first_counter=0, B=40)
    full = omodel.link_loss_and_grads(rp, ci, X, batch, enc, dec, "sage")
    samp = omodel.sampled_link_loss_and_grads(rp, ci, X, batch, enc, dec, [10**6, 10**6], seed=3, step=0)
    assert samp[0] == pytest.approx(full[0], rel=1e-12)
    np.testing.assert_allclose(samp[3], full[3], rtol=1e-10, atol=1e-12)
    for l in range(2):
        for a, b in zip(samp[1][l], full[1][l]):
            np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-12)
        for a, b in zip(samp[2][l], full[2][l]):
            np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-12)
    rps, cis, inputs, seeds = samp[4]
    assert len(inputs) < n and len(seeds) <= 120
    # with a real cut the blocks shrink and the loss changes
    cut = omodel.sampled_link_loss_and_grads(rp, ci, X, batch, enc, dec, [2, 2], seed=3, step=0)
    assert np.diff(cut[4][0][1]).max() <= 2 and cut[0] != pytest.approx(full[0], rel=1e-6)
    again = omodel.sampled_link_loss_and_grads(rp, ci, X, batch, enc, dec, [2, 2], seed=3, step=1)
    assert again[0] != cut[0]                                       # another step draws other neighbours
