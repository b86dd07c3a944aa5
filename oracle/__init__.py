"""CPU oracle (fp64, plain C) -- TEST INFRASTRUCTURE ONLY.

Thin numpy front-end over ``tma_oracle.c``.  Nothing here is imported by the
product package; only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg use it.  It never imports the HIP binding.

Every function converts its floating-point arguments to fp64 and returns fp64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tma_oracle.c")
_LIB = os.path.join(_HERE, "libtma_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_mix64.restype = C.c_uint64
        _lib.orc_mix64.argtypes = [C.c_uint64, C.c_uint64]
        _lib.orc_softmax_ce.restype = C.c_double
        _lib.orc_sigmoid_l2.restype = C.c_double
        _lib.orc_bce_logits.restype = C.c_double
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


# ---------------------------------------------------------------- partition
def mix64(seed: int, idx: int) -> int:
    return int(lib().orc_mix64(C.c_uint64(seed), C.c_uint64(idx)))


def partition(n_nodes: int, K: int, seed: int, cluster=None) -> np.ndarray:
    """part[v] in [0,K): RandomTMA (cluster None) or SuperTMA (Sec. 3.2.2)."""
    part = np.empty(n_nodes, dtype=np.int32)
    cl = None if cluster is None else _i32(cluster)
    lib().orc_partition(C.c_int64(n_nodes), _p(cl), C.c_int32(K), C.c_uint64(seed), _p(part))
    return part


# ---------------------------------------------------------- induced subgraph
def induced_subgraph(rowptr, colidx, part, p: int):
    """Node-induced subgraph of partition p (Preliminaries).

    Returns dict(g2l, l2g, rowptr, colidx, inv_deg) in the canonical local
    numbering (rank by global id, neighbour order kept).
    """
    rowptr, colidx, part = _i64(rowptr), _i32(colidx), _i32(part)
    n = rowptr.shape[0] - 1
    n_loc, nnz_loc = C.c_int64(0), C.c_int64(0)
    lib().orc_induced_count(C.c_int64(n), _p(rowptr), _p(colidx), _p(part), C.c_int32(p),
                            C.byref(n_loc), C.byref(nnz_loc))
    n_loc, nnz_loc = n_loc.value, nnz_loc.value
    g2l = np.empty(n, dtype=np.int32)
    l2g = np.empty(n_loc, dtype=np.int32)
    rp = np.empty(n_loc + 1, dtype=np.int32)
    ci = np.empty(nnz_loc, dtype=np.int32)
    inv = np.empty(n_loc, dtype=np.float64)
    lib().orc_induced_fill(C.c_int64(n), _p(rowptr), _p(colidx), _p(part), C.c_int32(p),
                           _p(g2l), _p(l2g), _p(rp), _p(ci), _p(inv))
    return dict(g2l=g2l, l2g=l2g, rowptr=rp, colidx=ci, inv_deg=inv)


# --------------------------------------------- the benchmark's all-cores timing leg
def set_threads(n: int) -> None:
    """Row loops of the aggregation and of the SAGE layer on n threads (timing only; tests keep the default 1)."""
    lib().orc_set_threads(C.c_int(int(n)))


def hardware_threads() -> int:
    return int(lib().orc_hardware_threads())


# ------------------------------------------------------- storage formats
def round_bf16(a) -> np.ndarray:
    """Nearest bfloat16 value (8 significant bits, ties to even) of every entry, returned as fp64.

    Written from the format's definition: x = m * 2^e with 1/2 <= |m| < 1, and m is rounded to a multiple of
    2^-8.  Normal range only (no subnormals, no overflow): the test data stays far inside it."""
    m, e = np.frexp(np.asarray(a, dtype=np.float64))
    return np.ldexp(np.rint(np.ldexp(m, 8)), e - 8)


# -------------------------------------------------------------- aggregation
def mean_aggregate(rowptr, colidx, H) -> np.ndarray:
    """M = Abar H.  On a bipartite block (fewer graph rows than rows of H) M has one row per graph row."""
    rowptr, colidx, H = _i32(rowptr), _i32(colidx), _f64(H)
    n, F = rowptr.shape[0] - 1, H.shape[1]
    assert n <= H.shape[0]
    M = np.empty((n, F))
    lib().orc_mean_aggregate(C.c_int64(n), _p(rowptr), _p(colidx), _p(H), C.c_int64(F), _p(M))
    return M


def mean_aggregate_T(rowptr, colidx, G) -> np.ndarray:
    rowptr, colidx, G = _i32(rowptr), _i32(colidx), _f64(G)
    n, F = G.shape
    out = np.empty_like(G)
    lib().orc_mean_aggregate_T(C.c_int64(n), _p(rowptr), _p(colidx), _p(G), C.c_int64(F), _p(out))
    return out


# -------------------------------------------------------------------- layer
ACT_NONE, ACT_RELU = 0, 1


def sage_layer_fwd(rowptr, colidx, H, W_self, W_neigh, bias, act: int):
    """Returns (M, Z, Hnext) of one mean-SAGE layer."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    H, W_self, W_neigh, bias = _f64(H), _f64(W_self), _f64(W_neigh), _f64(bias)
    n, F_in = rowptr.shape[0] - 1, H.shape[1]      # a bipartite block has fewer rows than H: its first n rows are the dst nodes
    F_out = W_self.shape[1]
    assert W_self.shape == (F_in, F_out) and W_neigh.shape == (F_in, F_out) and bias.shape == (F_out,)
    assert n <= H.shape[0]
    M = np.empty((n, F_in))
    Z = np.empty((n, F_out))
    Hn = np.empty((n, F_out))
    lib().orc_sage_layer_fwd(C.c_int64(n), _p(rowptr), _p(colidx), _p(H), C.c_int64(F_in),
                             _p(W_self), _p(W_neigh), _p(bias), C.c_int64(F_out), C.c_int(act),
                             _p(M), _p(Z), _p(Hn))
    return M, Z, Hn


def sage_layer_bwd(rowptr, colidx, H, M, Z, dHnext, W_self, W_neigh, act: int, need_dH=True):
    """Returns (dW_self, dW_neigh, dbias, dH or None).  On a bipartite block (H has more rows than the graph:
    the first n are the destination nodes) dH covers all rows of H."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    H, M, Z, dHnext = _f64(H), _f64(M), _f64(Z), _f64(dHnext)
    W_self, W_neigh = _f64(W_self), _f64(W_neigh)
    n, F_in = M.shape
    F_out = W_self.shape[1]
    dWs = np.empty((F_in, F_out))
    dWn = np.empty((F_in, F_out))
    db = np.empty(F_out)
    dH = np.zeros((H.shape[0], F_in)) if need_dH else None     # rows past n only receive scattered terms
    sM = np.empty((n, F_in))
    sZ = np.empty((n, F_out))
    lib().orc_sage_layer_bwd(C.c_int64(n), _p(rowptr), _p(colidx), _p(H), _p(M), _p(Z), _p(dHnext),
                             _p(W_self), _p(W_neigh), C.c_int64(F_in), C.c_int64(F_out), C.c_int(act),
                             _p(dWs), _p(dWn), _p(db), _p(dH), _p(sM), _p(sZ))
    return dWs, dWn, db, dH


# --------------------------------------------- GCN and MLP encoders (Sec. 4.1)
def gcn_norm(rowptr) -> np.ndarray:
    """s_v = (d_v + 1)^-1/2 over the local degrees."""
    rowptr = _i32(rowptr)
    n = rowptr.shape[0] - 1
    s = np.empty(n)
    lib().orc_gcn_norm(C.c_int64(n), _p(rowptr), _p(s))
    return s


def gcn_aggregate(rowptr, colidx, H, transpose: bool = False) -> np.ndarray:
    """Ahat H (or Ahat^T H), Ahat = Dt^-1/2 (A + I) Dt^-1/2."""
    rowptr, colidx, H = _i32(rowptr), _i32(colidx), _f64(H)
    n, F = H.shape
    M = np.empty_like(H)
    fn = lib().orc_gcn_aggregate_T if transpose else lib().orc_gcn_aggregate
    fn(C.c_int64(n), _p(rowptr), _p(colidx), _p(H), C.c_int64(F), _p(M))
    return M


def dense_fwd(X, W, bias, act: int):
    """Returns (Z, Y): Z = X W + b (bias may be None), Y = act(Z)."""
    X, W = _f64(X), _f64(W)
    b = None if bias is None else _f64(bias)
    n, F_in = X.shape
    F_out = W.shape[1]
    assert W.shape == (F_in, F_out) and (b is None or b.shape == (F_out,))
    Z = np.empty((n, F_out))
    Y = np.empty((n, F_out))
    lib().orc_dense_fwd(C.c_int64(n), _p(X), C.c_int64(F_in), _p(W), _p(b), C.c_int64(F_out), C.c_int(act),
                        _p(Z), _p(Y))
    return Z, Y


def dense_bwd(X, Z, dY, W, act: int, need_dbias=True, need_dX=True):
    """Returns (dW, dbias or None, dX or None)."""
    X, Z, dY, W = _f64(X), _f64(Z), _f64(dY), _f64(W)
    n, F_in = X.shape
    F_out = W.shape[1]
    dW = np.empty((F_in, F_out))
    db = np.empty(F_out) if need_dbias else None
    dX = np.empty((n, F_in)) if need_dX else None
    sZ = np.empty((n, F_out))
    lib().orc_dense_bwd(C.c_int64(n), _p(X), _p(Z), _p(dY), _p(W), C.c_int64(F_in), C.c_int64(F_out), C.c_int(act),
                        _p(dW), _p(db), _p(dX), _p(sZ))
    return dW, db, dX


def gcn_layer_fwd(rowptr, colidx, H, W, bias, act: int):
    """Returns (M, Z, Hnext) of one GCN layer: M = Ahat H, Z = M W + b."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    H, W, bias = _f64(H), _f64(W), _f64(bias)
    n, F_in = H.shape
    F_out = W.shape[1]
    assert W.shape == (F_in, F_out) and bias.shape == (F_out,)
    M = np.empty((n, F_in))
    Z = np.empty((n, F_out))
    Hn = np.empty((n, F_out))
    lib().orc_gcn_layer_fwd(C.c_int64(n), _p(rowptr), _p(colidx), _p(H), C.c_int64(F_in), _p(W), _p(bias),
                            C.c_int64(F_out), C.c_int(act), _p(M), _p(Z), _p(Hn))
    return M, Z, Hn


def gcn_layer_bwd(rowptr, colidx, M, Z, dHnext, W, act: int, need_dH=True):
    """Returns (dW, dbias, dH or None)."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    M, Z, dHnext, W = _f64(M), _f64(Z), _f64(dHnext), _f64(W)
    n, F_in = M.shape
    F_out = W.shape[1]
    dW = np.empty((F_in, F_out))
    db = np.empty(F_out)
    dH = np.empty((n, F_in)) if need_dH else None
    sM = np.empty((n, F_in))
    sZ = np.empty((n, F_out))
    lib().orc_gcn_layer_bwd(C.c_int64(n), _p(rowptr), _p(colidx), _p(M), _p(Z), _p(dHnext), _p(W),
                            C.c_int64(F_in), C.c_int64(F_out), C.c_int(act), _p(dW), _p(db), _p(dH), _p(sM), _p(sZ))
    return dW, db, dH


def gcn_block_aggregate(rowptr, colidx, H, transpose: bool = False, n_src: int | None = None) -> np.ndarray:
    """Row-normalised aggregation with the self-loop on a bipartite block: M = Dt^-1 (A_S + I) H over the block's
    rows (H has a row per source node, the first rows being the block's own nodes); with ``transpose`` the
    adjoint, from one row per block row to n_src rows."""
    rowptr, colidx, H = _i32(rowptr), _i32(colidx), _f64(H)
    n_dst, F = rowptr.shape[0] - 1, H.shape[1]
    if transpose:
        assert H.shape[0] == n_dst and n_src is not None and n_src >= n_dst
        out = np.empty((n_src, F))
        lib().orc_gcn_block_aggregate_T(C.c_int64(n_dst), C.c_int64(n_src), _p(rowptr), _p(colidx), _p(H),
                                        C.c_int64(F), _p(out))
        return out
    assert n_dst <= H.shape[0]
    M = np.empty((n_dst, F))
    lib().orc_gcn_block_aggregate(C.c_int64(n_dst), _p(rowptr), _p(colidx), _p(H), C.c_int64(F), _p(M))
    return M


def gcn_block_layer_fwd(rowptr, colidx, H, W, bias, act: int):
    """Returns (M, Z, Hnext) of one GCN layer on a bipartite block: M = Dt^-1 (A_S + I) H, Z = M W + b."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    H, W, bias = _f64(H), _f64(W), _f64(bias)
    n_dst, F_in = rowptr.shape[0] - 1, H.shape[1]
    F_out = W.shape[1]
    assert W.shape == (F_in, F_out) and bias.shape == (F_out,) and n_dst <= H.shape[0]
    M = np.empty((n_dst, F_in))
    Z = np.empty((n_dst, F_out))
    Hn = np.empty((n_dst, F_out))
    lib().orc_gcn_block_layer_fwd(C.c_int64(n_dst), _p(rowptr), _p(colidx), _p(H), C.c_int64(F_in), _p(W), _p(bias),
                                  C.c_int64(F_out), C.c_int(act), _p(M), _p(Z), _p(Hn))
    return M, Z, Hn


def gcn_block_layer_bwd(rowptr, colidx, n_src: int, M, Z, dHnext, W, act: int, need_dH=True):
    """Returns (dW, dbias, dH [n_src, F_in] or None)."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    M, Z, dHnext, W = _f64(M), _f64(Z), _f64(dHnext), _f64(W)
    n_dst, F_in = M.shape
    F_out = W.shape[1]
    assert n_dst == rowptr.shape[0] - 1 and n_src >= n_dst
    dW = np.empty((F_in, F_out))
    db = np.empty(F_out)
    dH = np.empty((n_src, F_in)) if need_dH else None
    sM = np.empty((n_dst, F_in))
    sZ = np.empty((n_dst, F_out))
    lib().orc_gcn_block_layer_bwd(C.c_int64(n_dst), C.c_int64(n_src), _p(rowptr), _p(colidx), _p(M), _p(Z),
                                  _p(dHnext), _p(W), C.c_int64(F_in), C.c_int64(F_out), C.c_int(act), _p(dW), _p(db),
                                  _p(dH), _p(sM), _p(sZ))
    return dW, db, dH


# ------------------------------------------------------ normalisation + activation
LN_EPS = 1e-5


def layernorm_prelu_fwd(Z, gamma, beta, slope: float, eps: float = LN_EPS) -> np.ndarray:
    """H' = PReLU_slope(LayerNorm_{gamma,beta}(Z)) over the feature axis of every row."""
    Z, gamma, beta = _f64(Z), _f64(gamma), _f64(beta)
    n, F = Z.shape
    assert gamma.shape == (F,) and beta.shape == (F,)
    Hn = np.empty((n, F))
    lib().orc_layernorm_prelu_fwd(C.c_int64(n), C.c_int64(F), _p(Z), _p(gamma), _p(beta), C.c_double(slope),
                                  C.c_double(eps), _p(Hn))
    return Hn


def layernorm_prelu_bwd(Z, dHn, gamma, beta, slope: float, eps: float = LN_EPS, open_mask=None):
    """Returns (dZ, dgamma, dbeta, dslope).  open_mask (bool [n,F]) overrides the decision Y > 0."""
    Z, dHn, gamma, beta = _f64(Z), _f64(dHn), _f64(gamma), _f64(beta)
    n, F = Z.shape
    dZ = np.empty((n, F))
    dg = np.empty(F)
    db = np.empty(F)
    ds = C.c_double(0.0)
    om = None if open_mask is None else np.ascontiguousarray(np.asarray(open_mask).astype(np.uint8))
    zh = np.empty(F)
    dzh = np.empty(F)
    lib().orc_layernorm_prelu_bwd(C.c_int64(n), C.c_int64(F), _p(Z), _p(dHn), _p(gamma), _p(beta), C.c_double(slope),
                                  C.c_double(eps), _p(om), _p(dZ), _p(dg), _p(db), C.byref(ds), _p(zh), _p(dzh))
    return dZ, dg, db, float(ds.value)


# ------------------------------------------------------------------- losses
def softmax_ce(logits, labels, need_grad=True):
    logits, labels = _f64(logits), _i32(labels)
    n, Cc = logits.shape
    d = np.empty_like(logits) if need_grad else None
    loss = lib().orc_softmax_ce(C.c_int64(n), C.c_int64(Cc), _p(logits), _p(labels), _p(d))
    return float(loss), d


def sigmoid_l2(G, Y, need_grad=True):
    G, Y = _f64(G), _f64(Y)
    n, Cc = G.shape
    d = np.empty_like(G) if need_grad else None
    loss = lib().orc_sigmoid_l2(C.c_int64(n), C.c_int64(Cc), _p(G), _p(Y), _p(d))
    return float(loss), d


# ------------------------------------------------------ optimizer / averaging
def sgd_step(W, dW, lr: float) -> np.ndarray:
    W = _f64(W).copy()
    dW = _f64(dW)
    lib().orc_sgd_step(C.c_int64(W.size), _p(W), _p(dW), C.c_double(lr))
    return W


def adam_step(W, dW, m, v, lr: float, t: int, b1: float = 0.9, b2: float = 0.999, eps: float = 1e-8):
    """One Adam update; returns new (W, m, v).  t = 1 for the first step."""
    W, m, v = _f64(W).copy(), _f64(m).copy(), _f64(v).copy()
    dW = _f64(dW)
    lib().orc_adam_step(C.c_int64(W.size), _p(W), _p(dW), _p(m), _p(v), C.c_double(lr), C.c_double(b1),
                        C.c_double(b2), C.c_double(eps), C.c_int64(t))
    return W, m, v


def average(W_stack, active_mask: int | None = None):
    """phi = mean over active trainers.  W_stack [M, P] -> (W_after [M,P], W_global [P])."""
    W = _f64(W_stack).copy()
    M, P = W.shape
    if active_mask is None:
        active_mask = (1 << M) - 1
    Wg = np.zeros(P)
    lib().orc_average(C.c_int32(M), C.c_int64(P), C.c_uint64(active_mask), _p(W), _p(Wg))
    return W, Wg


# ------------------------------------------------ link-prediction head (Sec. 4.1, App.)
def edge_batch(rowptr, colidx, seed: int, first_counter: int, B: int):
    """B positive edges (u, v) and one negative tail v' each, from the counter-based spec; int32 arrays."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.shape[0] - 1
    assert B == 0 or (rowptr[-1] > 0 and n > 1)
    u, v, vn = (np.empty(B, dtype=np.int32) for _ in range(3))
    lib().orc_edge_batch(C.c_int64(n), _p(rowptr), _p(colidx), C.c_uint64(seed), C.c_uint64(first_counter),
                         C.c_int64(B), _p(u), _p(v), _p(vn))
    return u, v, vn


def pair_product_fwd(R, u, v, vneg) -> np.ndarray:
    """E0 [2B, F]: r_u (.) r_v for the positives, then r_u (.) r_v' for the negatives."""
    R, u, v, vneg = _f64(R), _i32(u), _i32(v), _i32(vneg)
    B, F = u.shape[0], R.shape[1]
    E0 = np.empty((2 * B, F))
    lib().orc_pair_product_fwd(C.c_int64(B), C.c_int64(F), _p(R), _p(u), _p(v), _p(vneg), _p(E0))
    return E0


def pair_product_bwd(R, u, v, vneg, dE0) -> np.ndarray:
    R, u, v, vneg, dE0 = _f64(R), _i32(u), _i32(v), _i32(vneg), _f64(dE0)
    n, F = R.shape
    dR = np.empty((n, F))
    lib().orc_pair_product_bwd(C.c_int64(n), C.c_int64(u.shape[0]), C.c_int64(F), _p(R), _p(u), _p(v), _p(vneg),
                               _p(dE0), _p(dR))
    return dR


def prelu_fwd(Z, slope: float) -> np.ndarray:
    Z = _f64(Z)
    Y = np.empty_like(Z)
    lib().orc_prelu_fwd(C.c_int64(Z.size), _p(Z), C.c_double(slope), _p(Y))
    return Y


def prelu_bwd(Z, dY, slope: float, open_mask=None):
    """Returns (dZ, dslope)."""
    Z, dY = _f64(Z), _f64(dY)
    dZ = np.empty_like(Z)
    ds = C.c_double(0.0)
    om = None if open_mask is None else np.ascontiguousarray(np.asarray(open_mask).astype(np.uint8))
    lib().orc_prelu_bwd(C.c_int64(Z.size), _p(Z), _p(dY), C.c_double(slope), _p(om), _p(dZ), C.byref(ds))
    return dZ, float(ds.value)


def bce_logits(z, n_pos: int, need_grad=True):
    """Mean binary cross-entropy of logits z; the first n_pos are positives.  Returns (loss, dz)."""
    z = _f64(z).ravel()
    dz = np.empty_like(z) if need_grad else None
    loss = lib().orc_bce_logits(C.c_int64(z.size), C.c_int64(n_pos), _p(z), _p(dz))
    return float(loss), dz


# ------------------------------------------------ sampled message-flow graphs (Sec. 4.1)
def neighbor_sample(dst, rowptr, colidx, fanout: int, seed: int):
    """Block CSR over the local ids: per dst node all its neighbours, or a uniform `fanout`-subset of them."""
    dst, rowptr, colidx = _i32(dst), _i32(rowptr), _i32(colidx)
    n_dst = dst.shape[0]
    brp = np.empty(n_dst + 1, dtype=np.int32)
    bci = np.empty(max(n_dst * fanout, 1), dtype=np.int32)
    lib().orc_neighbor_sample(C.c_int64(n_dst), _p(dst), _p(rowptr), _p(colidx), C.c_int32(fanout), C.c_uint64(seed),
                              _p(brp), _p(bci))
    return brp, bci[:brp[-1]].copy()


def mfg_relabel(dst, blk_col):
    """Source node list of a block: the dst nodes first, in their order, then the other sampled nodes in
    ascending id order; and the block's columns as positions in that list.  Returns (src, blk_col_positions)."""
    dst, blk_col = _i32(dst), _i32(blk_col)
    new = np.setdiff1d(blk_col, dst)                   # sorted, unique
    src = np.concatenate([dst, new]).astype(np.int32)
    pos = {int(g): i for i, g in enumerate(src.tolist())}
    return src, np.fromiter((pos[int(c)] for c in blk_col.tolist()), dtype=np.int32, count=blk_col.shape[0])
