"""Oracle compositions: the L-layer local trainer step and the TMA loops.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Built from the layer
functions of the C oracle, in fp64, in the order the paper's Alg. 2 gives for
one trainer iteration: forward on the local subgraph, loss, backward, optimizer
step; and, for several trainers, Alg. 1's aggregate-and-overwrite.
"""
from __future__ import annotations

import numpy as np

from . import (ACT_NONE, ACT_RELU, adam_step, average, layernorm_prelu_bwd, layernorm_prelu_fwd,
               sage_layer_bwd, sage_layer_fwd, sgd_step, softmax_ce)

ACT_LN_PRELU = "ln_prelu"   # a layer whose parameter tuple is (W_self, W_neigh, b, gamma, beta, slope)


def forward(rowptr, colidx, X, params):
    """Identity on the last layer; between layers ReLU, or, for a layer that carries (gamma, beta, slope),
    layer normalisation followed by PReLU (the paper's encoder variant, Sec. 4.1).  Returns (logits, saved)."""
    H = np.asarray(X, dtype=np.float64)
    saved = []
    L = len(params)
    for l, layer in enumerate(params):
        Ws, Wn, b = layer[:3]
        if len(layer) == 6:
            M, Z, _ = sage_layer_fwd(rowptr, colidx, H, Ws, Wn, b, ACT_NONE)
            Hn = layernorm_prelu_fwd(Z, layer[3], layer[4], float(np.asarray(layer[5]).ravel()[0]))
            saved.append((H, M, Z, ACT_LN_PRELU))
        else:
            act = ACT_RELU if l < L - 1 else ACT_NONE
            M, Z, Hn = sage_layer_fwd(rowptr, colidx, H, Ws, Wn, b, act)
            saved.append((H, M, Z, act))
        H = Hn
    return H, saved


def loss_and_grads(rowptr, colidx, X, y, params, relu_open=None):
    """Mean softmax-CE over all local nodes and d(loss)/d(params).

    ``relu_open[l]`` (optional, boolean [n, F_{l+1}]) fixes where layer l's ReLU (or PReLU) is open instead
    of deciding it from this fp64 forward pass.  ReLU' is a yes/no decision taken from a floating-point
    value; a pre-activation within rounding distance of zero can fall on different sides in fp32 and
    fp64, which changes one whole term of a weight-gradient sum.  A parity test therefore hands the
    decision taken in the kernel's precision to both sides; the arithmetic is unchanged.
    """
    logits, saved = forward(rowptr, colidx, X, params)
    loss, d = softmax_ce(logits, y)
    grads = [None] * len(params)
    for l in range(len(params) - 1, -1, -1):
        H, M, Z, act = saved[l]
        Ws, Wn = params[l][0], params[l][1]
        forced = relu_open[l] if relu_open is not None else None
        if act == ACT_LN_PRELU:
            gamma, beta, slope = params[l][3], params[l][4], float(np.asarray(params[l][5]).ravel()[0])
            dZ, dg, dbeta, ds = layernorm_prelu_bwd(Z, d, gamma, beta, slope, open_mask=forced)
            dWs, dWn, db, dH = sage_layer_bwd(rowptr, colidx, H, M, Z, dZ, Ws, Wn, ACT_NONE, need_dH=l > 0)
            grads[l] = (dWs, dWn, db, dg, dbeta, np.array([ds]))
        else:
            if forced is not None and act == ACT_RELU:
                Z = np.where(np.asarray(forced), 1.0, -1.0)   # only the sign of Z is used by the backward pass
            dWs, dWn, db, dH = sage_layer_bwd(rowptr, colidx, H, M, Z, d, Ws, Wn, act, need_dH=l > 0)
            grads[l] = (dWs, dWn, db)
        d = dH
    return loss, grads, logits, saved


def train_step(rowptr, colidx, X, y, params, lr, relu_open=None):
    """One Alg. 2 iteration on the full local subgraph; returns (loss, new params)."""
    loss, grads, _, _ = loss_and_grads(rowptr, colidx, X, y, params, relu_open)
    new = [tuple(sgd_step(w, g, lr).reshape(np.shape(w)) for w, g in zip(pl, gl))
           for pl, gl in zip(params, grads)]
    return loss, new


def train_step_adam(rowptr, colidx, X, y, params, lr, state, t, relu_open=None):
    """One Alg. 2 iteration with Adam.  state = (m, v) flat vectors (None before the first step), t = 1, 2, ...
    Returns (loss, new params, new state); the state belongs to the trainer and is never averaged."""
    loss, grads, _, _ = loss_and_grads(rowptr, colidx, X, y, params, relu_open)
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
