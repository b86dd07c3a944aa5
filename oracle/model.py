"""Oracle compositions: the L-layer local trainer step and the TMA loops.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Built from the layer
functions of the C oracle, in fp64, in the order the paper's Alg. 2 gives for
one trainer iteration: forward on the local subgraph, loss, backward, optimizer
step; and, for several trainers, Alg. 1's aggregate-and-overwrite.
"""
from __future__ import annotations

import numpy as np

from . import (ACT_NONE, ACT_RELU, adam_step, average, bce_logits, dense_bwd, dense_fwd, gcn_aggregate,
               gcn_block_aggregate, gcn_block_layer_bwd, gcn_block_layer_fwd, gcn_layer_bwd,
               gcn_layer_fwd, gcn_norm, layernorm_prelu_bwd, layernorm_prelu_fwd, mean_aggregate,
               mfg_relabel, mix64, neighbor_sample, pair_product_bwd, pair_product_fwd, prelu_bwd,
               prelu_fwd, round_bf16, sage_layer_bwd, sage_layer_fwd, sgd_step, softmax_ce)

ACT_LN_PRELU = "ln_prelu"   # a layer whose parameter tuple ends with (gamma, beta, slope)


def _layer_fwd(encoder, rowptr, colidx, H, lin, act, block=False):
    """(M, Z, Hnext) of one layer of the chosen encoder (Sec. 4.1): "sage" (W_self, W_neigh, b),
    "gcn" (W, b) or the graph-agnostic "mlp" (W, b), whose M is its input.  ``block``: the graph is one bipartite
    block of a sampled message-flow graph (GCN then takes its row-normalised form)."""
    if encoder == "sage":
        return sage_layer_fwd(rowptr, colidx, H, lin[0], lin[1], lin[2], act)
    if encoder == "gcn" and block:
        return gcn_block_layer_fwd(rowptr, colidx, H, lin[0], lin[1], act)
    if encoder == "gcn":
        return gcn_layer_fwd(rowptr, colidx, H, lin[0], lin[1], act)
    if encoder == "mlp":
        Z, Hn = dense_fwd(H, lin[0], lin[1], act)
        return H, Z, Hn
    raise ValueError(encoder)


def _layer_bwd(encoder, rowptr, colidx, H, M, Z, d, lin, act, need_dH, block=False):
    """(gradients of the linear parameters, dH)."""
    if encoder == "sage":
        dWs, dWn, db, dH = sage_layer_bwd(rowptr, colidx, H, M, Z, d, lin[0], lin[1], act, need_dH=need_dH)
        return (dWs, dWn, db), dH
    if encoder == "gcn" and block:
        dW, db, dH = gcn_block_layer_bwd(rowptr, colidx, H.shape[0], M, Z, d, lin[0], act, need_dH=need_dH)
        return (dW, db), dH
    if encoder == "gcn":
        dW, db, dH = gcn_layer_bwd(rowptr, colidx, M, Z, d, lin[0], act, need_dH=need_dH)
        return (dW, db), dH
    dW, db, dH = dense_bwd(H, Z, d, lin[0], act, need_dX=need_dH)
    return (dW, db), dH


def n_linear(encoder):
    return 3 if encoder == "sage" else 2


def forward(rowptr, colidx, X, params, encoder="sage"):
    """Identity on the last layer; between layers ReLU, or, for a layer that carries (gamma, beta, slope)
    after its linear parameters, layer normalisation followed by PReLU (the paper's encoder variant,
    Sec. 4.1).  Returns (logits, saved)."""
    H = np.asarray(X, dtype=np.float64)
    saved = []
    L = len(params)
    nl = n_linear(encoder)
    per_layer = isinstance(rowptr, (list, tuple))     # one bipartite block per layer (a sampled message-flow graph)
    graphs = (rowptr, colidx)
    for l, layer in enumerate(params):
        rowptr, colidx = (graphs[0][l], graphs[1][l]) if per_layer else graphs
        lin = layer[:nl]
        if len(layer) == nl + 3:
            M, Z, _ = _layer_fwd(encoder, rowptr, colidx, H, lin, ACT_NONE, per_layer)
            Hn = layernorm_prelu_fwd(Z, layer[nl], layer[nl + 1], float(np.asarray(layer[nl + 2]).ravel()[0]))
            saved.append((H, M, Z, ACT_LN_PRELU))
        else:
            act = ACT_RELU if l < L - 1 else ACT_NONE
            M, Z, Hn = _layer_fwd(encoder, rowptr, colidx, H, lin, act, per_layer)
            saved.append((H, M, Z, act))
        H = Hn
    return H, saved


def _store(a, storage):
    if storage == "bf16":
        return round_bf16(a)
    if storage == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    raise ValueError(storage)


def forward_as_stored(rowptr, colidx, X, params, encoder="sage", storage="bf16", transform_first=None,
                      final_relu=False):
    """The forward pass again, with every tensor that a reduced-precision path keeps in memory rounded to that
    storage format where it is stored: the aggregate M, a normalised layer's pre-activation Z, every layer's
    output, and the weight matrices as operands of the products (biases, gamma, beta and slopes stay as given;
    sums are still taken in fp64).  This build's reading of where a bf16 path rounds; the paper fixes no precision.

    Used for one thing only: an activation's open/closed decision is a yes/no taken from a floating-point value,
    and for a pre-activation within rounding distance of zero it depends on the precision it is taken in.  A test
    of a reduced-precision path takes the decisions of THIS pass (the path's precision) for the fp64 backward pass.
    ``transform_first[l]`` (optional) says that layer l is evaluated in its other algebraic form, the product
    first and the aggregation on its narrower result (the same function by linearity): what is stored, and so
    rounded, is then Y = H [W_self | W_neigh] (for GCN: S H W) instead of the aggregate.
    ``final_relu``: the last layer has a ReLU too (a single hidden layer looked at on its own).
    Returns (output of the last layer, pre) with pre[l] the value whose sign decides the activation after layer l
    (None for the last layer): Z for ReLU, the normalised and scaled value for layer normalisation + PReLU."""
    H = _store(X, storage)
    L, nl = len(params), n_linear(encoder)
    per_layer = isinstance(rowptr, (list, tuple))
    graphs = (rowptr, colidx)
    pre = []
    for l, layer in enumerate(params):
        rp, ci = (graphs[0][l], graphs[1][l]) if per_layer else graphs
        n_dst = len(rp) - 1
        W = [_store(w, storage) for w in layer[:nl - 1]]
        b = np.asarray(layer[nl - 1], dtype=np.float64)
        tf = transform_first is not None and bool(transform_first[l])
        if encoder == "sage" and tf:
            Ys = _store(dense_fwd(H[:n_dst], W[0], None, ACT_NONE)[0], storage)
            Yn = _store(dense_fwd(H, W[1], None, ACT_NONE)[0], storage)
            Z = Ys + mean_aggregate(rp, ci, Yn) + b
        elif encoder == "sage":
            M = _store(mean_aggregate(rp, ci, H), storage)
            Z, _ = dense_fwd(np.concatenate([H[:n_dst], M], axis=1), np.concatenate(W, axis=0), b, ACT_NONE)
        elif encoder == "gcn" and per_layer:
            if tf:
                raise ValueError("the GCN layer on a block is evaluated aggregate-first only")
            Z, _ = dense_fwd(_store(gcn_block_aggregate(rp, ci, H), storage), W[0], b, ACT_NONE)
        elif encoder == "gcn" and tf:
            s_norm = gcn_norm(rp)[:, None]
            Y = _store(s_norm * dense_fwd(H, W[0], None, ACT_NONE)[0], storage)
            Z = gcn_aggregate(rp, ci, Y / s_norm) + b            # S (A + I) Y: the aggregate applies S on both sides
        elif encoder == "gcn":
            Z, _ = dense_fwd(_store(gcn_aggregate(rp, ci, H), storage), W[0], b, ACT_NONE)
        else:
            Z, _ = dense_fwd(H, W[0], b, ACT_NONE)
        if len(layer) == nl + 3:
            slope = float(np.asarray(layer[nl + 2]).ravel()[0])
            Hn = layernorm_prelu_fwd(_store(Z, storage), layer[nl], layer[nl + 1], slope)
            pre.append(np.where(Hn > 0, Hn, Hn / slope))
        elif l < L - 1 or final_relu:
            pre.append(Z)
            Hn = np.maximum(Z, 0.0)
        else:
            pre.append(None)
            Hn = Z
        H = _store(Hn, storage)
    return H, pre


def decoder_as_stored(R, batch, dec_params, storage="bf16"):
    """The decoder's forward pass with stored tensors rounded like forward_as_stored (pair products, every layer's
    output, the weight matrices as operands).  Returns (logits, pre): pre[k] = the value whose sign decides the
    PReLU after decoder layer k (None for the last)."""
    u, v, vneg = batch
    E = _store(pair_product_fwd(_store(R, storage), u, v, vneg), storage)
    pre = []
    for k, layer in enumerate(dec_params):
        Z, _ = dense_fwd(E, _store(layer[0], storage), None, ACT_NONE)
        Z = _store(Z, storage)
        if k < len(dec_params) - 1:
            pre.append(Z)
            E = _store(prelu_fwd(Z, float(np.asarray(layer[1]).ravel()[0])), storage)
        else:
            pre.append(None)
    return Z.ravel(), pre


def backward(rowptr, colidx, params, saved, d, relu_open=None, encoder="sage", need_dX=False, ups_out=None):
    """Chain rule from d = d(loss)/d(output of the last layer) down to the parameters (and, with need_dX,
    to the input features).  Returns (grads, dX or None).  ``ups_out`` (a list) receives, per layer, the
    gradient with respect to that layer's output as it arrives from above."""
    nl = n_linear(encoder)
    grads = [None] * len(params)
    per_layer = isinstance(rowptr, (list, tuple))
    graphs = (rowptr, colidx)
    if ups_out is not None:
        ups_out[:] = [None] * len(params)
    for l in range(len(params) - 1, -1, -1):
        rowptr, colidx = (graphs[0][l], graphs[1][l]) if per_layer else graphs
        H, M, Z, act = saved[l]
        lin = params[l][:nl]
        if ups_out is not None:
            ups_out[l] = d
        forced = relu_open[l] if relu_open is not None else None
        need_dH = l > 0 or need_dX
        if act == ACT_LN_PRELU:
            gamma, beta = params[l][nl], params[l][nl + 1]
            slope = float(np.asarray(params[l][nl + 2]).ravel()[0])
            dZ, dg, dbeta, ds = layernorm_prelu_bwd(Z, d, gamma, beta, slope, open_mask=forced)
            glin, dH = _layer_bwd(encoder, rowptr, colidx, H, M, Z, dZ, lin, ACT_NONE, need_dH, per_layer)
            grads[l] = glin + (dg, dbeta, np.array([ds]))
        else:
            if forced is not None and act == ACT_RELU:
                Z = np.where(np.asarray(forced), 1.0, -1.0)   # only the sign of Z is used by the backward pass
            glin, dH = _layer_bwd(encoder, rowptr, colidx, H, M, Z, d, lin, act, need_dH, per_layer)
            grads[l] = glin
        d = dH
    return grads, d


def decision_values(params, saved, encoder="sage"):
    """pre[l] = the value whose sign decides the activation after layer l in the fp64 pass that produced ``saved``
    (None for a layer without activation): Z for ReLU, gamma (.) Zhat + beta for layer normalisation + PReLU."""
    nl = n_linear(encoder)
    pre = []
    for layer, (_, _, Z, act) in zip(params, saved):
        if act == ACT_LN_PRELU:
            slope = float(np.asarray(layer[nl + 2]).ravel()[0])
            Hn = layernorm_prelu_fwd(Z, layer[nl], layer[nl + 1], slope)
            pre.append(np.where(Hn > 0, Hn, Hn / slope))
        else:
            pre.append(Z if act == ACT_RELU else None)
    return pre


def _open_masks(pre):
    return [None if p is None else p > 0 for p in pre]


def loss_and_grads(rowptr, colidx, X, y, params, relu_open=None, encoder="sage", decisions=None, trace=None,
                   transform_first=None):
    """Mean softmax-CE over all local nodes and d(loss)/d(params).

    Activation decisions: by default those of this fp64 pass.  ``decisions`` = "bf16" takes them from
    forward_as_stored instead (the precision of a path that stores activations and multiplies weights in
    that format); ``relu_open[l]`` (boolean [n, F_{l+1}]) fixes them outright.  The arithmetic is unchanged.
    ``trace`` (a dict) receives what a test needs to reason about decisions near zero: "pre" (the deciding
    values, per layer), "ups" (the gradient arriving at every layer's output), "saved".
    """
    logits, saved = forward(rowptr, colidx, X, params, encoder)
    loss, d = softmax_ce(logits, y)
    pre = decision_values(params, saved, encoder)
    if decisions is not None:
        _, pre = forward_as_stored(rowptr, colidx, X, params, encoder, decisions, transform_first)
        relu_open = _open_masks(pre)
    ups = []
    grads, _ = backward(rowptr, colidx, params, saved, d, relu_open, encoder, ups_out=ups)
    if trace is not None:
        trace.update(pre=pre, ups=ups, saved=saved)
    return loss, grads, logits, saved


def decoder_forward(R, batch, dec_params):
    """MLP link decoder (App., formulation of the MLP decoder): e0 = r_u (.) r_v, e_{k+1} = PReLU(e_k Theta_k)
    on the hidden layers, the last layer's single column is the logit.  dec_params: (Theta_k, slope_k) per
    hidden layer, (Theta_K,) for the last.  Returns (logits [2B], saved)."""
    u, v, vneg = batch
    E = pair_product_fwd(R, u, v, vneg)
    saved = []
    for k, layer in enumerate(dec_params):
        Z, _ = dense_fwd(E, layer[0], None, ACT_NONE)
        saved.append((E, Z))
        E = prelu_fwd(Z, float(np.asarray(layer[1]).ravel()[0])) if k < len(dec_params) - 1 else Z
    return E.ravel(), saved


def decoder_backward(dsaved, dec_params, dz, dec_open=None, ups_out=None):
    """Chain rule through the decoder from dz = d(loss)/d(logits).  Returns (dec_grads, d(loss)/d(E0)).
    ``ups_out`` receives, per hidden layer, the gradient arriving at its PReLU's output."""
    d = dz.reshape(-1, 1)
    K = len(dec_params)
    dec_grads = [None] * K
    if ups_out is not None:
        ups_out[:] = [None] * K
    for k in range(K - 1, -1, -1):
        E, Z = dsaved[k]
        extra = ()
        if k < K - 1:
            if ups_out is not None:
                ups_out[k] = d
            forced = dec_open[k] if dec_open is not None else None
            d, ds = prelu_bwd(Z, d, float(np.asarray(dec_params[k][1]).ravel()[0]), open_mask=forced)
            extra = (np.array([ds]),)
        dTheta, _, dE = dense_bwd(E, Z, d, dec_params[k][0], ACT_NONE, need_dbias=False)
        dec_grads[k] = (dTheta,) + extra
        d = dE
    return dec_grads, d


def _link_tail(graphs, X_in, batch_pos, enc_params, dec_params, encoder, relu_open, dec_open, decisions, trace,
               transform_first=None):
    """Encoder -> pair products -> decoder -> loss -> all gradients, on whatever graph(s) the encoder runs on."""
    R, saved = forward(graphs[0], graphs[1], X_in, enc_params, encoder)
    z, dsaved = decoder_forward(R, batch_pos, dec_params)
    loss, dz = bce_logits(z, len(batch_pos[0]))
    pre = decision_values(enc_params, saved, encoder)
    dec_pre = [Z if k < len(dec_params) - 1 else None for k, (_, Z) in enumerate(dsaved)]
    if decisions is not None:
        R_s, pre = forward_as_stored(graphs[0], graphs[1], X_in, enc_params, encoder, decisions, transform_first)
        _, dec_pre = decoder_as_stored(R_s, batch_pos, dec_params, decisions)
        relu_open, dec_open = _open_masks(pre), _open_masks(dec_pre)
    dec_ups, ups = [], []
    dec_grads, dE0 = decoder_backward(dsaved, dec_params, dz, dec_open, dec_ups)
    dR = pair_product_bwd(R, batch_pos[0], batch_pos[1], batch_pos[2], dE0)
    enc_grads, _ = backward(graphs[0], graphs[1], enc_params, saved, dR, relu_open, encoder, ups_out=ups)
    if trace is not None:
        trace.update(pre=pre, ups=ups, saved=saved, dec_pre=dec_pre, dec_ups=dec_ups, dsaved=dsaved, R=R,
                     batch_pos=batch_pos)
    return loss, enc_grads, dec_grads, z


def link_loss_and_grads(rowptr, colidx, X, batch, enc_params, dec_params, encoder="sage", relu_open=None,
                        dec_open=None, decisions=None, trace=None, transform_first=None):
    """Link-prediction step (Sec. 4.1): encoder on the whole local subgraph, pair products of the batch's
    positive and negative edges, MLP decoder, mean binary cross-entropy on the logits; gradients of both
    parameter sets.  ``relu_open`` / ``decisions`` / ``trace`` as in loss_and_grads; ``dec_open[k]`` fixes the
    decisions of the decoder's PReLU k.  Returns (loss, enc_grads, dec_grads, logits)."""
    return _link_tail((rowptr, colidx), X, batch, enc_params, dec_params, encoder, relu_open, dec_open, decisions,
                      trace, transform_first)


def layer_seed(seed: int, step: int, layer: int) -> int:
    """Seed of the neighbour sampler for one step and one layer (this build's convention: at most 64 layers)."""
    return mix64(seed, step * 64 + layer)


def sample_mfg(rowptr, colidx, seeds, fanouts, seed: int, step: int):
    """Message-flow graph of a mini-batch (Sec. 4.1: GraphSAGE sampler): starting from the batch's nodes `seeds`
    (the dst nodes of the last layer), every layer l = L-1 .. 0 samples up to fanouts[l] neighbours per dst node;
    its source nodes (dst first, then the new ones in ascending id) are the dst nodes of the layer below.
    Returns (block rowptrs, block colidx in source positions, input node ids), lists indexed by layer."""
    L = len(fanouts)
    rps, cis = [None] * L, [None] * L
    dst = np.asarray(seeds, dtype=np.int32)
    for l in range(L - 1, -1, -1):
        brp, bcol = neighbor_sample(dst, rowptr, colidx, fanouts[l], layer_seed(seed, step, l))
        src, cols = mfg_relabel(dst, bcol)
        rps[l], cis[l] = brp, cols
        dst = src
    return rps, cis, dst


def sampled_link_loss_and_grads(rowptr, colidx, X, batch, enc_params, dec_params, fanouts, seed, step,
                                relu_open=None, dec_open=None, decisions=None, trace=None, encoder="sage"):
    """The link-prediction step on the sampled message-flow graph of its batch (SAGE or GCN encoder): the encoder
    runs on the bipartite blocks only, from the features of the sampled input nodes up to the embeddings of the
    batch's nodes.  Returns (loss, enc_grads, dec_grads, logits, (rps, cis, input_nodes, seeds))."""
    u, v, vneg = batch
    seeds = np.unique(np.concatenate([u, v, vneg])).astype(np.int32)
    rps, cis, inputs = sample_mfg(rowptr, colidx, seeds, fanouts, seed, step)
    pos = tuple(np.searchsorted(seeds, a).astype(np.int32) for a in (u, v, vneg))
    loss, enc_grads, dec_grads, z = _link_tail((rps, cis), np.asarray(X)[inputs], pos, enc_params, dec_params,
                                               encoder, relu_open, dec_open, decisions, trace)
    return loss, enc_grads, dec_grads, z, (rps, cis, inputs, seeds)


def train_step(rowptr, colidx, X, y, params, lr, relu_open=None, encoder="sage", decisions=None, trace=None):
    """One Alg. 2 iteration on the full local subgraph; returns (loss, new params)."""
    loss, grads, _, _ = loss_and_grads(rowptr, colidx, X, y, params, relu_open, encoder, decisions, trace)
    if trace is not None:
        trace["grads"] = grads
    new = [tuple(sgd_step(w, g, lr).reshape(np.shape(w)) for w, g in zip(pl, gl))
           for pl, gl in zip(params, grads)]
    return loss, new


def train_step_adam(rowptr, colidx, X, y, params, lr, state, t, relu_open=None, encoder="sage", trace=None):
    """One Alg. 2 iteration with Adam.  state = (m, v) flat vectors (None before the first step), t = 1, 2, ...
    Returns (loss, new params, new state); the state belongs to the trainer and is never averaged."""
    loss, grads, _, _ = loss_and_grads(rowptr, colidx, X, y, params, relu_open, encoder, trace=trace)
    w, g = flatten(params), flatten(grads)
    m, v = (np.zeros_like(w), np.zeros_like(w)) if state is None else state
    w, m, v = adam_step(w, g, m, v, lr, t)
    return loss, unflatten(w, params), (m, v)


def flatten(params) -> np.ndarray:
    """Flat parameter vector, layer by layer: W_self, W_neigh, b (then gamma, beta, slope where present)."""
    return np.concatenate([np.asarray(t, dtype=np.float64).ravel() for layer in params for t in layer])


def unflatten(flat, like):
    out, o = [], 0
    for layer in like:
        cur = []
        for t in layer:
            sz = int(np.prod(np.shape(t)))
            cur.append(np.asarray(flat[o:o + sz]).reshape(np.shape(t)))
            o += sz
        out.append(tuple(cur))
    return out


def aggregate(params_per_trainer, active_mask=None):
    """Alg. 1 aggregation line + Alg. 2 overwrite, on structured parameters."""
    stack = np.stack([flatten(p) for p in params_per_trainer])
    after, w_global = average(stack, active_mask)
    return [unflatten(after[i], params_per_trainer[i]) for i in range(len(params_per_trainer))], w_global


def tma_schedule(step_time, n_trainers: int, dt_int: float, dt_train: float):
    """Idealised timeline of Alg. 1 (server) and Alg. 2 (trainers).

    ``step_time(i, k)`` is the duration of trainer i's k-th optimizer call.
    The server raises the aggregation flag once ``now - T_agg >= dt_int``; a
    trainer sees the flag only after finishing the step it is in, then blocks
    until the averaged weights come back, which happens when the slowest
    trainer has delivered.  Reading taken where the listing is silent: T_agg is
    reset to the time the broadcast completes (otherwise every poll after the
    first interval would aggregate).  The stop flag is raised once
    ``now - T_start > dt_train``; a trainer checks it at the top of its loop.

    Returns (rounds, final_steps): rounds[r][i] = steps trainer i had finished
    when round r's weights were collected.
    """
    t = [0.0] * n_trainers
    steps = [0] * n_trainers
    t_agg = 0.0
    rounds = []
    while t_agg + dt_int <= dt_train:
        t_flag = t_agg + dt_int
        for i in range(n_trainers):
            while True:
                t[i] += step_time(i, steps[i])
                steps[i] += 1
                if t[i] >= t_flag:
                    break
        t_agg = max(t)
        t = [t_agg] * n_trainers
        rounds.append(list(steps))
    for i in range(n_trainers):
        while t[i] <= dt_train:
            t[i] += step_time(i, steps[i])
            steps[i] += 1
    return rounds, steps
