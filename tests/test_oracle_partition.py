"""Pins for the oracle's random assignment and induced-subgraph extraction.

None of these checks re-types the oracle's own formula: they compare against a
published generator test vector, the invariants of a partition function, the
kept-edge ratio the paper prints, and a brute-force edge filter written as a
Python set comprehension straight from the definition in the Preliminaries.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2305_09887_amd import synth


def _read_cols(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_mix64_published_vector(golden_dir):
    want = [int(r[0]) for r in _read_cols(os.path.join(golden_dir, "splitmix64_seed1234567.txt"))]
    got = [oracle.mix64(1234567, i) for i in range(len(want))]
    assert got == want


def test_partition_range_determinism_and_seed():
    n, K = 50_000, 7
    a = oracle.partition(n, K, seed=4)
    b = oracle.partition(n, K, seed=4)
    c = oracle.partition(n, K, seed=5)
    assert a.min() >= 0 and a.max() < K
    assert np.array_equal(a, b)
    assert (a != c).mean() > 0.5


@pytest.mark.parametrize("K", [2, 3, 8, 23])
def test_partition_sizes_binomial_and_chi2(K):
    n = 200_000
    part = oracle.partition(n, K, seed=11)
    counts = np.bincount(part, minlength=K)
    assert counts.sum() == n
    sigma = np.sqrt(n * (1 / K) * (1 - 1 / K))
    assert np.all(np.abs(counts - n / K) < 5 * sigma)
    chi2 = ((counts - n / K) ** 2 / (n / K)).sum()
    # chi-square with K-1 dof: mean K-1, sd sqrt(2(K-1)); 6 sd is far in the tail
    assert chi2 < (K - 1) + 6 * np.sqrt(2 * (K - 1)) + 6


def test_partition_independence_of_neighbouring_ids():
    # consecutive ids must not be correlated: joint counts of (part[v], part[v+1]) ~ uniform on K^2
    n, K = 400_000, 4
    part = oracle.partition(n, K, seed=3)
    joint = np.bincount(part[:-1] * K + part[1:], minlength=K * K)
    exp = (n - 1) / K ** 2
    assert np.all(np.abs(joint - exp) < 6 * np.sqrt(exp))


def test_supertma_nodes_share_cluster_part_and_reductions():
    n, K = 30_000, 5
    rng = np.random.default_rng(0)
    cluster = rng.integers(0, 300, n).astype(np.int32)
    part = oracle.partition(n, K, seed=9, cluster=cluster)
    for c in range(300):
        assert np.unique(part[cluster == c]).size == 1
    # every super-node is a single node  ==>  RandomTMA bit for bit (Sec. 3.2.2, last sentence)
    ident = np.arange(n, dtype=np.int32)
    assert np.array_equal(oracle.partition(n, K, seed=9, cluster=ident), oracle.partition(n, K, seed=9))
    # the part of a super-node equals the part RandomTMA gives to the node with that id
    per_cluster = oracle.partition(300, K, seed=9)
    assert np.array_equal(part, per_cluster[cluster])


def _brute_force_induced(rowptr, colidx, part, p):
    """Definition, literally: V = alpha^-1(p); E = {(u,v) in E : u,v in V} (global ids)."""
    n = len(rowptr) - 1
    V = {v for v in range(n) if part[v] == p}
    E = {(v, int(colidx[e])) for v in range(n) for e in range(rowptr[v], rowptr[v + 1])
         if v in V and int(colidx[e]) in V}
    return V, E


@pytest.mark.parametrize("seed,K", [(1, 2), (2, 3), (3, 4)])
def test_induced_subgraph_matches_brute_force(seed, K):
    rowptr, colidx = synth.uniform_graph(300, 1200, seed)
    part = oracle.partition(300, K, seed=seed + 100)
    seen_nodes = set()
    for p in range(K):
        sub = oracle.induced_subgraph(rowptr, colidx, part, p)
        V, E = _brute_force_induced(rowptr, colidx, part, p)
        l2g = sub["l2g"]
        assert set(l2g.tolist()) == V
        assert np.all(np.diff(l2g) > 0)                      # local id = rank by global id
        got = {(int(l2g[i]), int(l2g[sub["colidx"][e]]))
               for i in range(len(l2g)) for e in range(sub["rowptr"][i], sub["rowptr"][i + 1])}
        assert got == E
        assert sub["rowptr"][-1] == len(E)                   # no duplicates were produced
        # neighbour order of the input row is kept (rows are sorted on input)
        for i in range(len(l2g)):
            row = sub["colidx"][sub["rowptr"][i]:sub["rowptr"][i + 1]]
            assert np.all(np.diff(row) > 0)
        # g2l is the inverse of l2g and -1 elsewhere
        g2l = sub["g2l"]
        assert np.array_equal(g2l[l2g], np.arange(len(l2g)))
        assert np.all(g2l[part != p] == -1)
        deg = np.diff(sub["rowptr"])
        want_inv = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)
        assert np.array_equal(sub["inv_deg"], want_inv)
        assert not (seen_nodes & V)
        seen_nodes |= V
    assert seen_nodes == set(range(300))                     # parts are disjoint and cover V


def test_induced_subgraph_k1_is_identity_and_symmetry_kept():
    rowptr, colidx = synth.uniform_graph(500, 3000, 7)
    part = np.zeros(500, dtype=np.int32)
    sub = oracle.induced_subgraph(rowptr, colidx, part, 0)
    assert np.array_equal(sub["rowptr"], rowptr) and np.array_equal(sub["colidx"], colidx)
    part = oracle.partition(500, 3, seed=1)
    sub = oracle.induced_subgraph(rowptr, colidx, part, 1)
    n = len(sub["l2g"])
    ent = {(i, int(j)) for i in range(n) for j in sub["colidx"][sub["rowptr"][i]:sub["rowptr"][i + 1]]}
    assert all((j, i) in ent for (i, j) in ent)


def test_kept_edge_ratio_matches_printed_values(golden_dir):
    """Sum over trainers of kept edges / all edges = 1/M; paper prints 0.33, 0.20, 0.04."""
    rowptr, colidx = synth.chung_lu_graph(60_000, 20, 2.1, seed=5)
    nnz = int(rowptr[-1])
    src = np.repeat(np.arange(60_000), np.diff(rowptr))
    for M_str, r_str in _read_cols(os.path.join(golden_dir, "kept_edge_ratio.txt")):
        M, r_print = int(M_str), float(r_str)
        part = oracle.partition(60_000, M, seed=77)
        kept = sum(int(oracle.induced_subgraph(rowptr, colidx, part, p)["rowptr"][-1]) for p in range(M))
        # independent count of the same quantity straight from the edge list
        assert kept == int((part[src] == part[colidx]).sum())
        r = kept / nnz
        assert abs(r - 1.0 / M) < 5 * np.sqrt((1 / M) * (1 - 1 / M) / (nnz / 2)) + 2e-3
        assert round(r, 2) == pytest.approx(r_print, abs=0.0051)


def test_supertma_kept_fraction_on_planted_communities():
    """Communities as super-nodes, intra fraction q: kept = q + (1-q)/K by the same 1/K argument."""
    rowptr, colidx, block = synth.sbm_graph(240, 100, 54_000, 6_000, seed=21)
    n = 240 * 100
    src = np.repeat(np.arange(n), np.diff(rowptr))
    q = float((block[src] == block[colidx]).mean())
    K = 16
    part = oracle.partition(n, K, seed=24, cluster=block)
    kept = sum(int(oracle.induced_subgraph(rowptr, colidx, part, p)["rowptr"][-1]) for p in range(K))
    assert abs(kept / rowptr[-1] - (q + (1 - q) / K)) < 0.01
