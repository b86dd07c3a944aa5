"""One TMA trainer's local training loop (Alg. 2 of the paper) on one HIP stream.

Sequencing and buffer ownership only: every numerical step is a call into the
C ABI (``binding``).  All buffers are allocated once in ``__init__``; ``step``
allocates nothing, so several trainers can be time-sliced on their own streams
without touching the allocator.
"""
from __future__ import annotations

import torch

from . import binding as B


class LocalTrainer:
    """Full-batch L-layer mean-aggregation GraphSAGE on a local induced subgraph.

    ``dims`` = [F_0, F_1, ..., F_L]; between layers ReLU, or with ``norm_act`` layer
    normalisation followed by PReLU (the paper's encoder variant, Sec. 4.1); identity on
    the last; mean softmax cross-entropy over all local nodes; plain SGD, or Adam with trainer-local moments.
    Parameters live in one flat fp32 vector ``W`` (layer by layer: W_self,
    W_neigh, bias, and with ``norm_act`` gamma, beta, slope of the hidden layers),
    gradients in ``dW`` with the same layout, so that the optimizer step and the
    averaging operator are single launches.
    """

    def __init__(self, rowptr, colidx, inv_deg, X, labels, dims, params=None, stream=None,
                 rowptr_T=None, colidx_T=None, norm_act=False, optimizer="sgd"):
        self.norm_act = bool(norm_act)
        if optimizer not in ("sgd", "adam"):
            raise B.TmaError("LocalTrainer: optimizer must be 'sgd' or 'adam'")
        self.optimizer = optimizer
        self.rowptr, self.colidx, self.inv_deg = rowptr, colidx, inv_deg
        # transposed graph for the backward gather; the same CSR for a symmetric graph
        self.rowptr_T = rowptr if rowptr_T is None else rowptr_T
        self.colidx_T = colidx if colidx_T is None else colidx_T
        self.X, self.labels = X, labels
        self.dims = list(dims)
        self.L = len(dims) - 1
        self.n = X.shape[0]
        self.dtype = X.dtype
        dev = X.device
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        if X.shape[1] != dims[0]:
            raise B.TmaError("LocalTrainer: X width differs from dims[0]")

        self.n_params = sum(2 * fi * fo + fo for fi, fo in zip(dims[:-1], dims[1:]))
        if self.norm_act:
            self.n_params += sum(2 * fo + 1 for fo in dims[1:-1])
        self.W = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        self.dW = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        self.layers, self.grads = self._views(self.W), self._views(self.dW)
        if optimizer == "adam":   # moment estimates: this trainer's own state, never averaged
            self.adam_m = torch.zeros_like(self.W)
            self.adam_v = torch.zeros_like(self.W)
        if params is not None:
            self.load_params(params)

        n = max(self.n, 1)
        # activations and their gradients share one row pitch per layer, padded to 16 bytes so that a
        # width such as 47 still takes the library's vector paths
        self.H = [X] + [B._padded(self.n, f, self.dtype, dev) for f in dims[1:]]
        self.M = [torch.empty((n, f), dtype=self.dtype, device=dev)[: self.n] for f in dims[:-1]]
        # gradient w.r.t. H[l] for l = 1..L (index l); dH[L] is d(loss)/d(logits)
        self.dH = [None] + [B._padded(self.n, f, self.dtype, dev) for f in dims[1:]]
        # pre-activations of the normalised layers (index l + 1 = output of layer l), kept for backward
        self.Z = [None] + [B._padded(self.n, f, self.dtype, dev) if self.norm_act and l < self.L - 1 else None
                           for l, f in enumerate(dims[1:])]
        dt = B._feat_dtype(X)
        ws_bytes = max(B.tma_sage_layer_bwd_workspace_bytes(self.n, fi, fo, dt, l > 0)
                       for l, (fi, fo) in enumerate(zip(dims[:-1], dims[1:])))
        ws_bytes = max(ws_bytes, B.tma_loss_workspace_bytes(self.n, dims[-1]))
        if self.norm_act and self.L > 1:
            ws_bytes = max(ws_bytes, max(B.tma_layernorm_prelu_bwd_workspace_bytes(self.n, f) for f in dims[1:-1]))
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.steps_done = 0

    def set_graph(self, rowptr, colidx, inv_deg, rowptr_T=None, colidx_T=None):
        """Point the trainer at a freshly extracted subgraph with the same node count."""
        if rowptr.numel() != self.n + 1 or inv_deg.numel() != self.n:
            raise B.TmaError("LocalTrainer.set_graph: node count differs from the allocated buffers")
        self.rowptr, self.colidx, self.inv_deg = rowptr, colidx, inv_deg
        self.rowptr_T = rowptr if rowptr_T is None else rowptr_T
        self.colidx_T = colidx if colidx_T is None else colidx_T

    def _views(self, flat):
        out, o = [], 0
        for l, (fi, fo) in enumerate(zip(self.dims[:-1], self.dims[1:])):
            ws = flat[o:o + fi * fo].view(fi, fo); o += fi * fo
            wn = flat[o:o + fi * fo].view(fi, fo); o += fi * fo
            b = flat[o:o + fo]; o += fo
            layer = [ws, wn, b]
            if self.norm_act and l < self.L - 1:
                layer += [flat[o:o + fo], flat[o + fo:o + 2 * fo], flat[o + 2 * fo:o + 2 * fo + 1]]
                o += 2 * fo + 1
            out.append(tuple(layer))
        return out

    def load_params(self, params):
        """params: per layer (W_self, W_neigh, bias) or, for a normalised layer, (..., gamma, beta, slope)."""
        with torch.cuda.stream(self.stream):
            for mine, given in zip(self.layers, params):
                if len(mine) != len(given):
                    raise B.TmaError("LocalTrainer.load_params: layer has a different number of tensors")
                for dst, src in zip(mine, given):
                    dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))

    def forward(self):
        for l in range(self.L):
            ws, wn, b = self.layers[l][:3]
            if self.norm_act and l < self.L - 1:
                gamma, beta, slope = self.layers[l][3:]
                B.tma_sage_layer_fwd(self.rowptr, self.colidx, self.inv_deg, self.H[l], ws, wn, b, B.TMA_ACT_NONE,
                                     M_out=self.M[l], Hnext_out=self.Z[l + 1], stream=self.stream)
                B.tma_layernorm_prelu_fwd(self.Z[l + 1], gamma, beta, slope, out=self.H[l + 1], stream=self.stream)
                continue
            act = B.TMA_ACT_RELU if l < self.L - 1 else B.TMA_ACT_NONE
            B.tma_sage_layer_fwd(self.rowptr, self.colidx, self.inv_deg, self.H[l], ws, wn, b, act,
                                 M_out=self.M[l], Hnext_out=self.H[l + 1], stream=self.stream)
        return self.H[self.L]

    def backward(self):
        B.tma_softmax_ce(self.H[self.L], self.labels, loss_out=self.loss, dlogits_out=self.dH[self.L],
                         ws=self.ws, stream=self.stream)
        for l in range(self.L - 1, -1, -1):
            ws, wn = self.layers[l][:2]
            dws, dwn, db = self.grads[l][:3]
            act = B.TMA_ACT_RELU if l < self.L - 1 else B.TMA_ACT_NONE
            out_act = self.H[l + 1]
            if self.norm_act and l < self.L - 1:
                gamma, beta, slope = self.layers[l][3:]
                dgamma, dbeta, dslope = self.grads[l][3:]
                # dL/dZ replaces dL/dH' in place; the layer below then runs without an activation of its own
                B.tma_layernorm_prelu_bwd(self.Z[l + 1], self.dH[l + 1], gamma, beta, slope, dZ_out=self.dH[l + 1],
                                          dgamma=dgamma, dbeta=dbeta, dslope=dslope, ws=self.ws, stream=self.stream)
                act, out_act = B.TMA_ACT_NONE, self.Z[l + 1]
            B.tma_sage_layer_bwd(self.rowptr_T, self.colidx_T, self.inv_deg, self.H[l], self.M[l], out_act,
                                 self.dH[l + 1], ws, wn, act, dW_self=dws, dW_neigh=dwn, dbias=db,
                                 dH_out=self.dH[l], need_dH=l > 0, ws=self.ws, stream=self.stream)

    def step(self, lr: float):
        """One iteration of Alg. 2's loop body on the full local subgraph."""
        self.forward()
        self.backward()
        if self.optimizer == "adam":
            B.tma_adam_step(self.W, self.dW, self.adam_m, self.adam_v, lr, self.steps_done + 1, stream=self.stream)
        else:
            B.tma_sgd_step(self.W, self.dW, lr, stream=self.stream)
        self.steps_done += 1
        return self.loss
