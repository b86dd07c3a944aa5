"""Activation decisions near zero in whole-step parity tests (test helper; everything here is computed from the
ORACLE's values: nothing the GPU produced enters an oracle call).

ReLU' and PReLU' are yes/no decisions taken from a floating-point value.  A pre-activation within rounding
distance of zero can fall on different sides in the kernel's arithmetic and in the oracle's fp64, and one such
decision switches a whole term of a weight-gradient sum on or off (chain rule in the proof of Thm. 1: the factor
dz/dg).  The tests therefore
  1. let the oracle take its own decisions,
  2. build, from the oracle's deciding values alone, the near-zero set N = {|pre| <= eps * rms(pre)}, assert that
     it holds at most a tiny share of the entries and that every entry on which the GPU's sign pattern differs
     from the oracle's lies in N (anywhere else a differing sign is a wrong result), and
  3. add to the tolerance of every gradient an upper bound of what the differing decisions D (a subset of N) can
     change, computed here from the oracle's activations, upstream gradients and weights.  With D empty, the usual
     case at test sizes, the tolerance is the plain one.

The bound (per gradient tensor, in the Frobenius norm, which also bounds the largest entry): a flipped decision
at entry (v, o) of a ReLU layer changes dZ[v, o] by |dH'[v, o]|; with r_v the 2-norm of row v's change of dZ,
    |d dW_self|_F <= sum_v |H_v| r_v,   |d dW_neigh|_F <= sum_v |M_v| r_v,   |d dbias| <= sum_v r_v,
and the change of dH = dZ W_self^T + Abar^T (dZ W_neigh^T) has row norms
    q_v <= r_v |W_self|_2   and   q_u <= r_v |W_neigh|_2 / deg(v)  for every neighbour u of v,
which arrive at the layer below as a change of its dH'.  Layer normalisation + PReLU: the decision scales the
gradient by 1 or by the slope a, so an entry changes by |1 - a| |dH'|, and the normalisation's Jacobian has
2-norm at most max|gamma| / sigma_v.  GCN and dense layers, bipartite blocks and the link decoder follow the same
pattern with their own operators.
"""
from __future__ import annotations

from collections import defaultdict

import numpy as np

EPS_F32 = 8e-6      # fp32 accumulation of a few hundred products: a few 1e-7 of the value's scale, with margin
EPS_STORED = 2e-2   # decisions taken in the oracle's as-stored pass: what is left is accumulation order plus the
#                     rare bf16 rounding tie upstream that moves an operand by one unit in the last place (2^-8 of
#                     it); with few terms per sum (a 32-wide decoder input) one large term's unit is 6e-3 of the rms
STORED = dict(eps=EPS_STORED, near_share=3e-2, flip_share=2e-4)   # check() arguments for such tests
LN_EPS = 1e-5


def check(gpu_open, pre, what, eps=EPS_F32, near_share=1e-5, flip_share=None, floor=8):
    """Asserts of step 2.  gpu_open: the GPU's decision (its stored activation > 0); pre: the oracle's deciding
    value.  Returns D, the boolean array of differing decisions."""
    pre = np.asarray(pre, dtype=np.float64)
    gpu_open = np.asarray(gpu_open, dtype=bool)
    assert gpu_open.shape == pre.shape, f"{what}: shape {gpu_open.shape} vs {pre.shape}"
    if pre.size == 0:
        return np.zeros(pre.shape, dtype=bool)
    rms = float(np.sqrt(np.mean(pre * pre)))
    near = np.abs(pre) <= eps * rms
    D = gpu_open != (pre > 0)
    outside = int((D & ~near).sum())
    assert outside == 0, f"{what}: {outside} activation decisions differ where the pre-activation is not near zero"
    assert near.sum() <= max(floor, near_share * pre.size), \
        f"{what}: {int(near.sum())} of {pre.size} pre-activations within {eps:g} rms of zero"
    if flip_share is not None:
        assert D.sum() <= max(floor, flip_share * pre.size), f"{what}: {int(D.sum())} of {pre.size} decisions differ"
    return D


def _row_dict(D, ups, q):
    """Per row with a differing decision: 2-norm over its differing entries of |upstream gradient| (+ the row's
    own incoming change, which may add to the upstream value the flipped term carries)."""
    out = {}
    if D is None:
        return out
    for v in np.unique(np.nonzero(D)[0]):
        cols = np.nonzero(D[v])[0]
        out[int(v)] = float(np.linalg.norm(np.abs(ups[v, cols]) + q.get(int(v), 0.0)))
    return out


def _spec(W):
    return float(np.linalg.norm(np.asarray(W, dtype=np.float64), 2))


def _through_activation(act_kind, layer_tail, Z, ups, D, q):
    """(r, extra parameter bounds): r[v] bounds the 2-norm of row v's change of dL/dZ given the incoming change q
    of dL/dH' and the differing decisions D.  act_kind: "relu", "ln_prelu" or "none"."""
    flips = _row_dict(D, ups, q)
    rows = set(q) | set(flips)
    r, extra = {}, ()
    if act_kind == "none":
        return dict(q), extra
    if act_kind == "relu":
        for v in rows:
            r[v] = q.get(v, 0.0) + flips.get(v, 0.0)
        return r, extra
    gamma, beta, slope = (np.asarray(t, dtype=np.float64).ravel() for t in layer_tail)
    a = float(slope[0])
    dgamma = dbeta = dslope = 0.0
    for v in rows:
        z = Z[v]
        sig = np.sqrt(z.var() + LN_EPS)
        zh = (z - z.mean()) / sig
        y = gamma * zh + beta
        dy = max(1.0, abs(a)) * q.get(v, 0.0) + abs(1.0 - a) * flips.get(v, 0.0)
        dgamma += np.abs(zh).max() * dy
        dbeta += dy
        dslope += q.get(v, 0.0) * np.linalg.norm(y)
        if D is not None and D[v].any():
            cols = np.nonzero(D[v])[0]
            dslope += float(((np.abs(ups[v, cols]) + q.get(v, 0.0)) * np.abs(y[cols])).sum())
        r[v] = dy * np.abs(gamma).max() / sig
    return r, (dgamma, dbeta, dslope)


def encoder_bounds(encoder, rowptr, colidx, params, saved, ups, D, q_top=None):
    """Frobenius bounds of the change of every encoder gradient: bounds[l] is a tuple aligned with the oracle's
    grads[l].  rowptr/colidx: the graph, or per-layer lists of bipartite blocks.  D[l]: differing decisions of the
    activation after layer l (None where there is none).  q_top: incoming change of dL/d(output) per row."""
    nl = 3 if encoder == "sage" else 2
    per_layer = isinstance(rowptr, (list, tuple))
    q = dict(q_top or {})
    bounds = [None] * len(params)
    for l in range(len(params) - 1, -1, -1):
        rp, ci = (rowptr[l], colidx[l]) if per_layer else (rowptr, colidx)
        H, M, Z, act = saved[l]
        kind = "ln_prelu" if act == "ln_prelu" else ("relu" if act == 1 else "none")
        r, extra = _through_activation(kind, params[l][nl:nl + 3], Z, ups[l], D[l] if D is not None else None, q)
        rows = np.array(sorted(r), dtype=np.int64)
        rv = np.array([r[int(v)] for v in rows])
        nH = np.linalg.norm(np.asarray(H)[rows], axis=1) if len(rows) else np.zeros(0)
        nM = np.linalg.norm(np.asarray(M)[rows], axis=1) if len(rows) else np.zeros(0)
        if encoder == "sage":
            lin = (float(nH @ rv), float(nM @ rv), float(rv.sum()))
        elif encoder == "gcn":
            lin = (float(nM @ rv), float(rv.sum()))
        else:
            lin = (float(nH @ rv), float(rv.sum()))
        bounds[l] = lin + tuple(extra)
        nq = defaultdict(float)
        if l > 0:
            deg = np.diff(rp)
            if encoder == "sage":
                ws, wn = _spec(params[l][0]), _spec(params[l][1])
                for v, x in zip(rows, rv):
                    nq[int(v)] += x * ws
                    for u in ci[rp[v]:rp[v + 1]]:
                        nq[int(u)] += x * wn / deg[v]
            elif encoder == "gcn" and per_layer:      # on a block: the mean over the sampled neighbours and the node
                w = _spec(params[l][0])
                for v, x in zip(rows, rv):
                    c = x * w / (deg[v] + 1.0)
                    nq[int(v)] += c
                    for u in ci[rp[v]:rp[v + 1]]:
                        nq[int(u)] += c
            elif encoder == "gcn":
                w = _spec(params[l][0])
                s = 1.0 / np.sqrt(deg + 1.0)
                for v, x in zip(rows, rv):
                    nq[int(v)] += x * w * s[v] * s[v]
                    for u in ci[rp[v]:rp[v + 1]]:
                        nq[int(u)] += x * w * s[v] * s[u]
            else:
                w = _spec(params[l][0])
                for v, x in zip(rows, rv):
                    nq[int(v)] += x * w
        q = dict(nq)
    return bounds


def decoder_bounds(dec_params, dsaved, dec_ups, D_dec, R, batch_pos):
    """(bounds per decoder layer aligned with the oracle's dec_grads, q_top for encoder_bounds): the decoder's
    PReLU decisions D_dec[k] (None for the last layer) and what they change."""
    K = len(dec_params)
    q = {}
    bounds = [None] * K
    for k in range(K - 1, -1, -1):
        E, Z = dsaved[k]
        extra = ()
        if k < K - 1:
            a = float(np.asarray(dec_params[k][1]).ravel()[0])
            D = D_dec[k] if D_dec is not None else None
            flips = _row_dict(D, dec_ups[k], q)
            r, ds = {}, 0.0
            for v in set(q) | set(flips):
                r[v] = max(1.0, abs(a)) * q.get(v, 0.0) + abs(1.0 - a) * flips.get(v, 0.0)
                ds += q.get(v, 0.0) * np.linalg.norm(Z[v])
                if D is not None and D[v].any():
                    cols = np.nonzero(D[v])[0]
                    ds += float(((np.abs(dec_ups[k][v, cols]) + q.get(v, 0.0)) * np.abs(Z[v, cols])).sum())
            extra = (ds,)
        else:
            r = dict(q)
        bounds[k] = (float(sum(np.linalg.norm(E[v]) * x for v, x in r.items())),) + extra
        w = _spec(dec_params[k][0])
        q = {v: x * w for v, x in r.items()}
    # through the pair products: row i < B is (u_i, v_i), row B + i is (u_i, v'_i)
    u, v, vneg = (np.asarray(t) for t in batch_pos)
    Bn = len(u)
    top = defaultdict(float)
    R = np.asarray(R)
    for i, x in q.items():
        a, b = (u[i], v[i]) if i < Bn else (u[i - Bn], vneg[i - Bn])
        top[int(a)] += x * np.abs(R[b]).max()
        top[int(b)] += x * np.abs(R[a]).max()
    return bounds, dict(top)


def close(got, want, tol, what, extra=0.0):
    """Relative Frobenius error and largest error relative to the largest magnitude, both <= tol, after `extra`
    (an absolute Frobenius bound of an allowed change) is taken off."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if want.size == 0:
        return
    fro = max(np.linalg.norm(want.ravel()), 1e-300)
    scale = max(np.abs(want).max(), 1e-300)
    err = np.linalg.norm((got - want).ravel())
    mx = np.abs(got - want).max()
    assert err <= tol * fro + extra and mx <= tol * scale + extra, \
        f"{what}: rel fro {err / fro:.2e}, max abs / max {mx / scale:.2e} (tol {tol:g}, allowed change {extra:.2e})"


def total(bounds):
    """Sum over all tensors: a bound for the flat gradient vector."""
    return float(sum(x for layer in bounds if layer is not None for x in layer))


def differing(pre_list, gpu_acts, what, **kw):
    """check() for every activation of a model: pre_list from the oracle's trace ("pre" or "dec_pre"), gpu_acts the
    GPU's stored activations (anything np.asarray takes; entries past the oracle's shape are padding).  Returns the
    list D for encoder_bounds / decoder_bounds."""
    D = []
    for l, pre in enumerate(pre_list):
        if pre is None:
            D.append(None)
            continue
        act = np.asarray(gpu_acts[l])[:pre.shape[0], :pre.shape[1]]
        D.append(check(act > 0, pre, f"{what}, activation {l}", **kw))
    return D


def any_differs(*lists):
    return any(d is not None and d.any() for D in lists for d in D)


def prelu_pre(out, slope):
    """The deciding value behind the oracle's PReLU output: the output itself where open, output / slope elsewhere."""
    out = np.asarray(out, dtype=np.float64)
    return np.where(out > 0, out, out / slope)


def ln_prelu_bounds(Z, upstream, gamma, beta, slope, D):
    """Allowed change of (dZ, dgamma, dbeta, dslope) of one normalisation + PReLU backward call for the differing
    decisions D (Frobenius / absolute bounds)."""
    r, extra = _through_activation("ln_prelu", (gamma, beta, [slope]), np.asarray(Z, dtype=np.float64),
                                   np.asarray(upstream, dtype=np.float64), D, {})
    return (float(sum(r.values())),) + tuple(extra)
