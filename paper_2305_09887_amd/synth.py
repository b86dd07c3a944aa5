"""Seeded synthetic inputs: graphs, features, labels and initial weights.

This module only *draws inputs*.  It holds none of the method's arithmetic (no
partitioning, no sub-graph extraction, no aggregation, no model code) and it is
the single piece shared by the CPU oracle's tests and the HIP path's tests and
benchmark.  Everything is numpy on the host and a pure function of its seed.

The graph families stand in for the workloads the paper trains on (a social
network, two citation graphs and an e-commerce graph, Table 1 of the paper):
none of those datasets is available here, so the generators reproduce their
shape only -- node/edge counts, a heavy-tailed degree distribution, clustered
communities, feature widths.

All graphs are returned as a CSR pair (rowptr int64 [n+1], colidx int32 [nnz])
of a *simple* undirected graph in the sense of the paper's preliminaries: both
directions of every edge are stored, there are no self-loops and no parallel
edges, and every row is sorted by neighbour id.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "csr_from_pairs", "uniform_graph", "chung_lu_graph", "sbm_graph",
    "two_class_graph", "features", "labels", "glorot", "sage_params",
    "to_bf16_bits", "from_bf16_bits", "round_bf16",
]


# --------------------------------------------------------------------------
# CSR assembly
# --------------------------------------------------------------------------
def _distinct_pair_keys(n: int, u: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Unordered pairs -> sorted unique int64 keys lo*n+hi, self-loops dropped."""
    u = u.astype(np.int64, copy=False)
    v = v.astype(np.int64, copy=False)
    keep = u != v
    lo = np.minimum(u, v)[keep]
    hi = np.maximum(u, v)[keep]
    return np.unique(lo * n + hi)


def _csr_from_keys(n: int, keys: np.ndarray):
    lo = keys // n
    hi = keys - lo * n
    src = np.concatenate([lo, hi])
    dst = np.concatenate([hi, lo])
    order = np.argsort(src * n + dst, kind="stable")
    src = src[order]
    colidx = dst[order].astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(src, minlength=n), out=rowptr[1:])
    return rowptr, colidx


def csr_from_pairs(n: int, u, v):
    """Symmetric sorted CSR of the simple graph on n nodes with edges {u_i,v_i}."""
    return _csr_from_keys(n, _distinct_pair_keys(n, np.asarray(u), np.asarray(v)))


# --------------------------------------------------------------------------
# Graph families
# --------------------------------------------------------------------------
def uniform_graph(n: int, m: int, seed: int):
    """Exactly m distinct undirected edges, endpoints uniform over n nodes."""
    rng = np.random.default_rng(seed)
    keys = np.empty(0, dtype=np.int64)
    while keys.size < m:
        need = m - keys.size
        draw = need + need // 8 + 16
        new = _distinct_pair_keys(n, rng.integers(0, n, draw), rng.integers(0, n, draw))
        new = np.setdiff1d(new, keys, assume_unique=True)
        if new.size > need:  # drop a uniformly random surplus, not the largest keys
            new = new[np.sort(rng.permutation(new.size)[:need])]
        keys = np.union1d(keys, new)
    return _csr_from_keys(n, keys)


def chung_lu_weights(n: int, total: float, gamma: float) -> np.ndarray:
    """Expected degrees w_i ~ (i+i0)^(-1/(gamma-1)), sum = total, max = sqrt(total)."""
    expo = 1.0 / (gamma - 1.0)
    cap = np.sqrt(total)
    i = np.arange(n, dtype=np.float64)

    def w_of(i0):
        raw = (i + i0) ** (-expo)
        return raw * (total / raw.sum())

    lo, hi = 1e-3, float(n)
    for _ in range(80):  # bisection on the shift i0 so that max weight == cap
        mid = 0.5 * (lo + hi)
        if w_of(mid)[0] > cap:
            lo = mid
        else:
            hi = mid
    return w_of(hi)


def chung_lu_graph(n: int, avg_degree: float, gamma: float, seed: int):
    """Chung-Lu power-law graph: n*avg_degree/2 endpoint pairs drawn ~ w (x) w.

    Self-loops and repeated pairs are dropped, so the realised number of CSR
    entries is a little below n*avg_degree; callers report rowptr[-1].  Node ids
    are shuffled so that degree does not correlate with id.
    """
    rng = np.random.default_rng(seed)
    total = float(n) * avg_degree
    w = chung_lu_weights(n, total, gamma)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    m = int(round(total / 2))
    perm = rng.permutation(n)
    u = perm[np.minimum(np.searchsorted(cdf, rng.random(m), side="right"), n - 1)]
    v = perm[np.minimum(np.searchsorted(cdf, rng.random(m), side="right"), n - 1)]
    return csr_from_pairs(n, u, v)


def sbm_graph(n_blocks: int, block_size: int, n_intra: int, n_inter: int, seed: int):
    """Planted-community graph.  Returns (rowptr, colidx, block_of_node int32).

    n_intra pairs are drawn inside a uniformly chosen block, n_inter pairs
    between two uniformly chosen nodes of different blocks (same-block draws are
    dropped); duplicates are dropped.  block_of_node[v] = v // block_size.
    """
    rng = np.random.default_rng(seed)
    n = n_blocks * block_size
    b = rng.integers(0, n_blocks, n_intra)
    u_in = b * block_size + rng.integers(0, block_size, n_intra)
    v_in = b * block_size + rng.integers(0, block_size, n_intra)
    u_out = rng.integers(0, n, n_inter)
    v_out = rng.integers(0, n, n_inter)
    cross = (u_out // block_size) != (v_out // block_size)
    u = np.concatenate([u_in, u_out[cross]])
    v = np.concatenate([v_in, v_out[cross]])
    rowptr, colidx = csr_from_pairs(n, u, v)
    block = (np.arange(n, dtype=np.int64) // block_size).astype(np.int32)
    return rowptr, colidx, block


def two_class_graph(n: int, avg_degree: float, h: float, seed: int):
    """Two equally sized classes; an edge joins same-class nodes with probability h.

    This is the compatibility-matrix graph model of the paper's Lemma 1.
    Returns (rowptr, colidx, y int32) with y[v] = 0 for v < n/2 else 1.
    """
    rng = np.random.default_rng(seed)
    half = n // 2
    y = (np.arange(n) >= half).astype(np.int32)
    m = int(round(n * avg_degree / 2))
    u = rng.integers(0, n, m)
    same = rng.random(m) < h
    cls_v = np.where(same, y[u], 1 - y[u])
    v = cls_v * half + rng.integers(0, half, m)
    rowptr, colidx = csr_from_pairs(n, u, v)
    return rowptr, colidx, y


# --------------------------------------------------------------------------
# Dense inputs
# --------------------------------------------------------------------------
def features(n: int, f: int, seed: int) -> np.ndarray:
    """fp32 node features ~ N(0,1), row-major [n, f]."""
    return np.random.default_rng(seed).standard_normal((n, f), dtype=np.float32)


def community_features(block: np.ndarray, n_blocks: int, f: int, seed: int) -> np.ndarray:
    """x_v = mu_{block(v)} + N(0,1) with mu_c ~ N(0,I); fp32 [n, f]."""
    rng = np.random.default_rng(seed)
    mu = rng.standard_normal((n_blocks, f), dtype=np.float32)
    x = rng.standard_normal((block.shape[0], f), dtype=np.float32)
    x += mu[block]
    return x


def labels(n: int, c: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).integers(0, c, n).astype(np.int32)


def glorot(f_in: int, f_out: int, rng) -> np.ndarray:
    a = np.sqrt(6.0 / (f_in + f_out))
    return rng.uniform(-a, a, (f_in, f_out)).astype(np.float32)


def sage_params(dims, seed: int, bias_scale: float = 0.1):
    """Initial weights of an L-layer mean-SAGE model, dims = [F0, F1, ..., FL].

    Returns a list of (W_self [F_in,F_out], W_neigh [F_in,F_out], b [F_out]) in
    fp32.  Biases are small non-zero values so that a parity test would notice
    a dropped bias term.
    """
    rng = np.random.default_rng(seed)
    out = []
    for f_in, f_out in zip(dims[:-1], dims[1:]):
        w_self = glorot(f_in, f_out, rng)
        w_neigh = glorot(f_in, f_out, rng)
        b = (bias_scale * rng.standard_normal(f_out)).astype(np.float32)
        out.append((w_self, w_neigh, b))
    return out


# --------------------------------------------------------------------------
# bf16 storage helpers (format conversion only)
# --------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array whose values are exactly representable in bf16."""
    return from_bf16_bits(to_bf16_bits(x)).reshape(np.shape(x))
