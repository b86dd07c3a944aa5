"""Oracle compositions: the L-layer local trainer step and the TMA loops.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Built from the layer
functions of the C oracle, in fp64, in the order the paper's Alg. 2 gives for
one trainer iteration: forward on the local subgraph, loss, backward, optimizer
step; and, for several trainers, Alg. 1's aggregate-and-overwrite.
"""
from __future__ import annotations

import numpy as np

from . import (ACT_NONE, ACT_RELU, adam_step, average, bce_logits, dense_bwd, dense_fwd, gcn_layer_bwd, gcn_layer_fwd,
               layernorm_prelu_bwd, layernorm_prelu_fwd, mfg_relabel, mix64, neighbor_sample, pair_product_bwd,
               pair_product_fwd, prelu_bwd, prelu_fwd, sage_layer_bwd, sage_layer_fwd, sgd_step, softmax_ce)

ACT_LN_PRELU = "ln_prelu"   # a layer whose parameter tuple ends with (gamma, beta, slope)


def _layer_fwd(encoder, rowptr, colidx, H, lin, act):
    """(M, Z, Hnext) of one layer of the chosen encoder (Sec. 4.1): "sage" (W_self, W_neigh, b),
    "gcn" (W, b) or the graph-agnostic "mlp" (W, b), whose M is its input."""
    if encoder == "sage":
        return sage_layer_fwd(rowptr, colidx, H, lin[0], lin[1], lin[2], act)
    if encoder == "gcn":
        return gcn_layer_fwd(rowptr, colidx, H, lin[0], lin[1], act)
    if encoder == "mlp":
        Z, Hn = dense_fwd(H, lin[0], lin[1], act)
        return H, Z, Hn
    raise ValueError(encoder)


def _layer_bwd(encoder, rowptr, colidx, H, M, Z, d, lin, act, need_dH):
    """(gradients of the linear parameters, dH)."""
    if encoder == "sage":
        dWs, dWn, db, dH = sage_layer_bwd(rowptr, colidx, H, M, Z, d, lin[0], lin[1], act, need_dH=need_dH)
        return (dWs, dWn, db), dH
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
            M, Z, _ = _layer_fwd(encoder, rowptr, colidx, H, lin, ACT_NONE)
            Hn = layernorm_prelu_fwd(Z, layer[nl], layer[nl + 1], float(np.asarray(layer[nl + 2]).ravel()[0]))
            saved.append((H, M, Z, ACT_LN_PRELU))
        else:
            act = ACT_RELU if l < L - 1 else ACT_NONE
            M, Z, Hn = _layer_fwd(encoder, rowptr, colidx, H, lin, act)
            saved.append((H, M, Z, act))
        H = Hn
    return H, saved


def backward(rowptr, colidx, params, saved, d, relu_open=None, encoder="sage", need_dX=False):
    """Chain rule from d = d(loss)/d(output of the last layer) down to the parameters (and, with need_dX,
    to the input features).  Returns (grads, dX or None)."""
    nl = n_linear(encoder)
    grads = [None] * len(params)
    per_layer = isinstance(rowptr, (list, tuple))
    graphs = (rowptr, colidx)
    for l in range(len(params) - 1, -1, -1):
        rowptr, colidx = (graphs[0][l], graphs[1][l]) if per_layer else graphs
        H, M, Z, act = saved[l]
        lin = params[l][:nl]
        forced = relu_open[l] if relu_open is not None else None
        need_dH = l > 0 or need_dX
        if act == ACT_LN_PRELU:
            gamma, beta = params[l][nl], params[l][nl + 1]
            slope = float(np.asarray(params[l][nl + 2]).ravel()[0])
            dZ, dg, dbeta, ds = layernorm_prelu_bwd(Z, d, gamma, beta, slope, open_mask=forced)
            glin, dH = _layer_bwd(encoder, rowptr, colidx, H, M, Z, dZ, lin, ACT_NONE, need_dH)
            grads[l] = glin + (dg, dbeta, np.array([ds]))
        else:
            if forced is not None and act == ACT_RELU:
                Z = np.where(np.asarray(forced), 1.0, -1.0)   # only the sign of Z is used by the backward pass
            glin, dH = _layer_bwd(encoder, rowptr, colidx, H, M, Z, d, lin, act, need_dH)
            grads[l] = glin
        d = dH
    return grads, d


def loss_and_grads(rowptr, colidx, X, y, params, relu_open=None, encoder="sage"):
    """Mean softmax-CE over all local nodes and d(loss)/d(params).

    ``relu_open[l]`` (optional, boolean [n, F_{l+1}]) fixes where layer l's ReLU (or PReLU) is open instead
    of deciding it from this fp64 forward pass.  ReLU' is a yes/no decision taken from a floating-point
    value; a pre-activation within rounding distance of zero can fall on different sides in fp32 and
    fp64, which changes one whole term of a weight-gradient sum.  A parity test therefore hands the
    decision taken in the kernel's precision to both sides; the arithmetic is unchanged.
    """
    logits, saved = forward(rowptr, colidx, X, params, encoder)
    loss, d = softmax_ce(logits, y)
    grads, _ = backward(rowptr, colidx, params, saved, d, relu_open, encoder)
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


def link_loss_and_grads(rowptr, colidx, X, batch, enc_params, dec_params, encoder="sage", relu_open=None,
                        dec_open=None):
    """Link-prediction step (Sec. 4.1): encoder on the whole local subgraph, pair products of the batch's
    positive and negative edges, MLP decoder, mean binary cross-entropy on the logits; gradients of both
    parameter sets.  ``relu_open`` as in loss_and_grads; ``dec_open[k]`` the same for the decoder's PReLU k.
    Returns (loss, enc_grads, dec_grads, logits)."""
    R, saved = forward(rowptr, colidx, X, enc_params, encoder)
    z, dsaved = decoder_forward(R, batch, dec_params)
    loss, dz = bce_logits(z, len(batch[0]))
    d = dz.reshape(-1, 1)
    K = len(dec_params)
    dec_grads = [None] * K
    for k in range(K - 1, -1, -1):
        E, Z = dsaved[k]
        extra = ()
        if k < K - 1:
            forced = dec_open[k] if dec_open is not None else None
            d, ds = prelu_bwd(Z, d, float(np.asarray(dec_params[k][1]).ravel()[0]), open_mask=forced)
            extra = (np.array([ds]),)
        dTheta, _, dE = dense_bwd(E, Z, d, dec_params[k][0], ACT_NONE, need_dbias=False)
        dec_grads[k] = (dTheta,) + extra
        d = dE
    dR = pair_product_bwd(R, batch[0], batch[1], batch[2], d)
    enc_grads, _ = backward(rowptr, colidx, enc_params, saved, dR, relu_open, encoder)
    return loss, enc_grads, dec_grads, z


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
                                relu_open=None, dec_open=None):
    """The link-prediction step on the sampled message-flow graph of its batch (SAGE encoder): the encoder runs on
    the bipartite blocks only, from the features of the sampled input nodes up to the embeddings of the batch's
    nodes.  Returns (loss, enc_grads, dec_grads, logits, (rps, cis, input_nodes, seeds))."""
    u, v, vneg = batch
    seeds = np.unique(np.concatenate([u, v, vneg])).astype(np.int32)
    rps, cis, inputs = sample_mfg(rowptr, colidx, seeds, fanouts, seed, step)
    R, saved = forward(rps, cis, np.asarray(X)[inputs], enc_params, "sage")
    pos = tuple(np.searchsorted(seeds, a).astype(np.int32) for a in (u, v, vneg))
    z, dsaved = decoder_forward(R, pos, dec_params)
    loss, dz = bce_logits(z, len(u))
    d = dz.reshape(-1, 1)
    K = len(dec_params)
    dec_grads = [None] * K
    for k in range(K - 1, -1, -1):
        E, Z = dsaved[k]
        extra = ()
        if k < K - 1:
            forced = dec_open[k] if dec_open is not None else None
            d, ds = prelu_bwd(Z, d, float(np.asarray(dec_params[k][1]).ravel()[0]), open_mask=forced)
            extra = (np.array([ds]),)
        dTheta, _, dE = dense_bwd(E, Z, d, dec_params[k][0], ACT_NONE, need_dbias=False)
        dec_grads[k] = (dTheta,) + extra
        d = dE
    dR = pair_product_bwd(R, pos[0], pos[1], pos[2], d)
    enc_grads, _ = backward(rps, cis, enc_params, saved, dR, relu_open, "sage")
    return loss, enc_grads, dec_grads, z, (rps, cis, inputs, seeds)


def train_step(rowptr, colidx, X, y, params, lr, relu_open=None, encoder="sage"):
    """One Alg. 2 iteration on the full local subgraph; returns (loss, new params)."""
    loss, grads, _, _ = loss_and_grads(rowptr, colidx, X, y, params, relu_open, encoder)
    new = [tuple(sgd_step(w, g, lr).reshape(np.shape(w)) for w, g in zip(pl, gl))
           for pl, gl in zip(params, grads)]
    return loss, new


def train_step_adam(rowptr, colidx, X, y, params, lr, state, t, relu_open=None, encoder="sage"):
    """One Alg. 2 iteration with Adam.  state = (m, v) flat vectors (None before the first step), t = 1, 2, ...
    Returns (loss, new params, new state); the state belongs to the trainer and is never averaged."""
    loss, grads, _, _ = loss_and_grads(rowptr, colidx, X, y, params, relu_open, encoder)
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
