"""Seeded synthetic inputs at the sizes that are too slow to draw with numpy on the host: the same graph
families as ``synth`` (same recipes, another random stream), drawn with torch on whatever device the caller
names, usually the GPU that is about to consume them.

Like ``synth`` this module only *draws inputs*: it holds none of the method's arithmetic (no partitioning, no
extraction, no aggregation, no model code), and both the oracle's and the HIP path's tests may use it.  Graphs
come back as the CSR pair (rowptr int64 [n+1], colidx int32 [nnz]) of a simple undirected graph: both directions
stored, no self-loops, no parallel edges, rows sorted by neighbour id.
"""
from __future__ import annotations

import math

import torch

__all__ = ["csr_from_pairs", "chung_lu_graph", "chung_lu_share", "sbm_graph", "community_features"]


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def csr_from_pairs(n: int, u: torch.Tensor, v: torch.Tensor):
    """Symmetric sorted CSR of the simple graph on n nodes with edges {u_i, v_i} (self-loops and repeats dropped)."""
    u, v = u.to(torch.int64), v.to(torch.int64)
    keep = u != v
    lo, hi = torch.minimum(u, v)[keep], torch.maximum(u, v)[keep]
    del u, v, keep
    keys = torch.unique(lo * n + hi)                    # sorted, distinct unordered pairs
    del lo, hi
    lo = torch.div(keys, n, rounding_mode="floor")
    hi = keys - lo * n
    del keys
    both = torch.cat([lo * n + hi, hi * n + lo])        # directed entries as row * n + col
    del lo, hi
    both, _ = torch.sort(both)
    src = torch.div(both, n, rounding_mode="floor")
    colidx = (both - src * n).to(torch.int32)
    del both
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=src.device)
    rowptr[1:] = torch.cumsum(torch.bincount(src, minlength=n), 0)
    return rowptr, colidx


def _shift_for_cap(n: int, total: float, expo: float, device) -> tuple[float, float]:
    """(i0, sum of (i + i0)^-expo over i < n) such that the largest expected degree equals sqrt(total)."""
    cap = math.sqrt(total)

    def raw_sum(i0):
        s = 0.0
        for a in range(0, n, 1 << 26):
            i = torch.arange(a, min(n, a + (1 << 26)), dtype=torch.float64, device=device)
            s += float(((i + i0) ** (-expo)).sum())
        return s

    lo, hi = 1e-3, float(n)
    for _ in range(60):                                  # bisection on the shift, as in synth.chung_lu_weights
        mid = 0.5 * (lo + hi)
        if mid ** (-expo) * total / raw_sum(mid) > cap:
            lo = mid
        else:
            hi = mid
    return hi, raw_sum(hi)


def _cdf(weights: torch.Tensor) -> torch.Tensor:
    """Running sum of the weights, taken on the host in one fixed order and sent back: a floating-point prefix sum
    on the GPU may associate differently from run to run, and a cdf that differs in its last bits sends a few of
    the draws to a neighbouring node, so that one seed would no longer name one graph."""
    import numpy as np
    return torch.from_numpy(np.cumsum(weights.cpu().numpy(), dtype=np.float64)).to(weights.device)


def _draw(cdf: torch.Tensor, m: int, g: torch.Generator, chunk: int = 1 << 26) -> torch.Tensor:
    """m indices drawn with probabilities proportional to the increments of cdf."""
    out = torch.empty(m, dtype=torch.int64, device=cdf.device)
    top = cdf.numel() - 1
    for a in range(0, m, chunk):
        b = min(m, a + chunk)
        r = torch.rand(b - a, generator=g, device=cdf.device, dtype=torch.float64) * cdf[-1]
        out[a:b] = torch.searchsorted(cdf, r, right=True).clamp_(max=top)
    return out


def chung_lu_graph(n: int, avg_degree: float, gamma: float, seed: int, device="cuda"):
    """Chung-Lu power-law graph as in synth.chung_lu_graph: expected degrees w_i ~ (i + i0)^(-1/(gamma-1)) with
    sum n*avg_degree and largest value sqrt(sum); n*avg_degree/2 endpoint pairs drawn ~ w (x) w, self-loops and
    repeats dropped; node ids shuffled.  The realised entry count is rowptr[-1]."""
    g = _gen(seed, device)
    total = float(n) * avg_degree
    expo = 1.0 / (gamma - 1.0)
    i0, _ = _shift_for_cap(n, total, expo, device)
    cdf = _cdf((torch.arange(n, dtype=torch.float64, device=device) + i0) ** (-expo))
    perm = torch.randperm(n, generator=g, device=device)
    m = int(round(total / 2))
    u = perm[_draw(cdf, m, g)]
    v = perm[_draw(cdf, m, g)]
    del cdf, perm
    return csr_from_pairs(n, u, v)


def chung_lu_share(n_global: int, total_global: float, gamma: float, n_local: int, seed: int, device="cuda"):
    """One part's share of a Chung-Lu graph too large to draw whole.  A Chung-Lu graph restricted to a node subset
    is Chung-Lu on that subset with the same weights and the GLOBAL weight sum; a random part holds a uniformly
    random subset of the global weight ranks.  So: n_local distinct ranks out of n_global, their weights under
    the global normalisation (sum total_global, cap sqrt(total_global)), and as many pairs as fall with both ends
    into the subset, total_global/2 * (local weight share)^2, drawn ~ w (x) w over the local nodes.
    Local node i stands for the i-th smallest global id of the part; ids carry no degree information.
    Returns (rowptr, colidx) over the n_local local nodes."""
    g = _gen(seed, device)
    expo = 1.0 / (gamma - 1.0)
    i0, raw_sum = _shift_for_cap(n_global, total_global, expo, device)
    ranks = torch.randperm(n_global, generator=g, device=device)[:n_local].to(torch.float64)
    w = (ranks + i0) ** (-expo) * (total_global / raw_sum)
    del ranks
    share = float(w.sum()) / total_global
    m = int(round(total_global / 2 * share * share))
    cdf = _cdf(w)
    del w
    u, v = _draw(cdf, m, g), _draw(cdf, m, g)
    del cdf
    return csr_from_pairs(n_local, u, v)


def sbm_graph(n_blocks: int, block_size: int, n_intra: int, n_inter: int, seed: int, device="cuda"):
    """Planted-community graph as in synth.sbm_graph.  Returns (rowptr, colidx, block_of_node int32)."""
    g = _gen(seed, device)
    n = n_blocks * block_size
    ri = lambda hi, k: torch.randint(0, hi, (k,), generator=g, device=device, dtype=torch.int64)
    b = ri(n_blocks, n_intra)
    u_in, v_in = b * block_size + ri(block_size, n_intra), b * block_size + ri(block_size, n_intra)
    u_out, v_out = ri(n, n_inter), ri(n, n_inter)
    cross = torch.div(u_out, block_size, rounding_mode="floor") != torch.div(v_out, block_size, rounding_mode="floor")
    rowptr, colidx = csr_from_pairs(n, torch.cat([u_in, u_out[cross]]), torch.cat([v_in, v_out[cross]]))
    block = torch.div(torch.arange(n, device=device), block_size, rounding_mode="floor").to(torch.int32)
    return rowptr, colidx, block


def community_features(block: torch.Tensor, n_blocks: int, f: int, seed: int, dtype=torch.float32, rows: int = 1 << 20):
    """x_v = mu_{block(v)} + N(0,1) with mu_c ~ N(0,I), stored as `dtype` [n, f]; drawn in slices of `rows` rows."""
    dev = block.device
    g = _gen(seed, dev)
    mu = torch.randn((n_blocks, f), generator=g, device=dev)
    n = block.numel()
    x = torch.empty((n, f), dtype=dtype, device=dev)
    for a in range(0, n, rows):
        b = min(n, a + rows)
        x[a:b] = (torch.randn((b - a, f), generator=g, device=dev) + mu[block[a:b].long()]).to(dtype)
    return x
