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
    """Full-batch L-layer encoder on a local induced subgraph: mean-aggregation GraphSAGE (default), GCN or the
    graph-agnostic MLP (``encoder`` = "sage" | "gcn" | "mlp"; the paper's encoder choices, Sec. 4.1).

    ``dims`` = [F_0, F_1, ..., F_L]; between layers ReLU, or with ``norm_act`` layer
    normalisation followed by PReLU (the paper's encoder variant, Sec. 4.1); identity on
    the last; mean softmax cross-entropy over all local nodes; plain SGD, or Adam with trainer-local moments.
    Parameters live in one flat fp32 vector ``W`` (layer by layer: W_self,
    W_neigh, bias -- W, bias for GCN and MLP -- and with ``norm_act`` gamma, beta, slope of the hidden layers),
    gradients in ``dW`` with the same layout, so that the optimizer step and the
    averaging operator are single launches.
    """

    def __init__(self, rowptr, colidx, inv_deg, X, labels, dims, params=None, stream=None,
                 rowptr_T=None, colidx_T=None, norm_act=False, optimizer="sgd", encoder="sage"):
        self.norm_act = bool(norm_act)
        if encoder not in ("sage", "gcn", "mlp"):
            raise B.TmaError("LocalTrainer: encoder must be 'sage', 'gcn' or 'mlp'")
        self.encoder = encoder
        self.n_lin = 3 if encoder == "sage" else 2     # tensors of a layer's linear part
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

        n_w = 2 if encoder == "sage" else 1
        self.n_params = sum(n_w * fi * fo + fo for fi, fo in zip(dims[:-1], dims[1:]))
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
        self.M = ([torch.empty((n, f), dtype=self.dtype, device=dev)[: self.n] for f in dims[:-1]]
                  if encoder != "mlp" else None)
        # gradient w.r.t. H[l] for l = 1..L (index l); dH[L] is d(loss)/d(logits)
        self.dH = [None] + [B._padded(self.n, f, self.dtype, dev) for f in dims[1:]]
        # pre-activations of the normalised layers (index l + 1 = output of layer l), kept for backward
        self.Z = [None] + [B._padded(self.n, f, self.dtype, dev) if self.norm_act and l < self.L - 1 else None
                           for l, f in enumerate(dims[1:])]
        dt = B._feat_dtype(X)
        pairs = list(zip(dims[:-1], dims[1:]))
        if encoder == "sage":
            ws_bytes = max(B.tma_sage_layer_bwd_workspace_bytes(self.n, fi, fo, dt, l > 0)
                           for l, (fi, fo) in enumerate(pairs))
        elif encoder == "gcn":
            ws_bytes = max(B.tma_gcn_layer_bwd_workspace_bytes(self.n, fi, fo, dt, l > 0)
                           for l, (fi, fo) in enumerate(pairs))
            self.s_norm = torch.empty(self.n, dtype=torch.float32, device=dev)
            with torch.cuda.stream(self.stream):
                B.tma_gcn_norm(rowptr, out=self.s_norm, stream=self.stream)
        else:
            ws_bytes = max(B.tma_dense_bwd_workspace_bytes(self.n, fi, fo) for fi, fo in pairs)
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
        if self.encoder == "gcn":
            B.tma_gcn_norm(rowptr, out=self.s_norm, stream=self.stream)

    def _views(self, flat):
        out, o = [], 0
        for l, (fi, fo) in enumerate(zip(self.dims[:-1], self.dims[1:])):
            layer = []
            for _ in range(self.n_lin - 1):
                layer.append(flat[o:o + fi * fo].view(fi, fo)); o += fi * fo
            layer.append(flat[o:o + fo]); o += fo
            if self.norm_act and l < self.L - 1:
                layer += [flat[o:o + fo], flat[o + fo:o + 2 * fo], flat[o + 2 * fo:o + 2 * fo + 1]]
                o += 2 * fo + 1
            out.append(tuple(layer))
        return out

    def load_params(self, params):
        """params: per layer (W_self, W_neigh, bias) -- (W, bias) for GCN and MLP -- or, for a normalised layer,
        (..., gamma, beta, slope)."""
        with torch.cuda.stream(self.stream):
            for mine, given in zip(self.layers, params):
                if len(mine) != len(given):
                    raise B.TmaError("LocalTrainer.load_params: layer has a different number of tensors")
                for dst, src in zip(mine, given):
                    dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))

    def _layer_fwd(self, l, act, out):
        lin = self.layers[l][:self.n_lin]
        if self.encoder == "sage":
            B.tma_sage_layer_fwd(self.rowptr, self.colidx, self.inv_deg, self.H[l], lin[0], lin[1], lin[2], act,
                                 M_out=self.M[l], Hnext_out=out, stream=self.stream)
        elif self.encoder == "gcn":
            B.tma_gcn_layer_fwd(self.rowptr, self.colidx, self.s_norm, self.H[l], lin[0], lin[1], act,
                                M_out=self.M[l], Hnext_out=out, stream=self.stream)
        else:
            B.tma_dense_fwd(self.H[l], lin[0], lin[1], act, Y_out=out, stream=self.stream)

    def _layer_bwd(self, l, act, out_act):
        lin, g = self.layers[l][:self.n_lin], self.grads[l][:self.n_lin]
        if self.encoder == "sage":
            B.tma_sage_layer_bwd(self.rowptr_T, self.colidx_T, self.inv_deg, self.H[l], self.M[l], out_act,
                                 self.dH[l + 1], lin[0], lin[1], act, dW_self=g[0], dW_neigh=g[1], dbias=g[2],
                                 dH_out=self.dH[l], need_dH=l > 0, ws=self.ws, stream=self.stream)
        elif self.encoder == "gcn":
            B.tma_gcn_layer_bwd(self.rowptr_T, self.colidx_T, self.s_norm, self.H[l], self.M[l], out_act,
                                self.dH[l + 1], lin[0], act, dW=g[0], dbias=g[1], dH_out=self.dH[l], need_dH=l > 0, ws=self.ws,
                                stream=self.stream)
        else:
            B.tma_dense_bwd(self.H[l], out_act, self.dH[l + 1], lin[0], act, dW=g[0], dbias=g[1], dX_out=self.dH[l],
                            need_dX=l > 0, ws=self.ws, stream=self.stream)

    def forward(self):
        for l in range(self.L):
            if self.norm_act and l < self.L - 1:
                gamma, beta, slope = self.layers[l][self.n_lin:]
                self._layer_fwd(l, B.TMA_ACT_NONE, self.Z[l + 1])
                B.tma_layernorm_prelu_fwd(self.Z[l + 1], gamma, beta, slope, out=self.H[l + 1], stream=self.stream)
                continue
            self._layer_fwd(l, B.TMA_ACT_RELU if l < self.L - 1 else B.TMA_ACT_NONE, self.H[l + 1])
        return self.H[self.L]

    def backward(self):
        B.tma_softmax_ce(self.H[self.L], self.labels, loss_out=self.loss, dlogits_out=self.dH[self.L],
                         ws=self.ws, stream=self.stream)
        for l in range(self.L - 1, -1, -1):
            act = B.TMA_ACT_RELU if l < self.L - 1 else B.TMA_ACT_NONE
            out_act = self.H[l + 1]
            if self.norm_act and l < self.L - 1:
                gamma, beta, slope = self.layers[l][self.n_lin:]
                dgamma, dbeta, dslope = self.grads[l][self.n_lin:]
                # dL/dZ replaces dL/dH' in place; the layer below then runs without an activation of its own
                B.tma_layernorm_prelu_bwd(self.Z[l + 1], self.dH[l + 1], gamma, beta, slope, dZ_out=self.dH[l + 1],
                                          dgamma=dgamma, dbeta=dbeta, dslope=dslope, ws=self.ws, stream=self.stream)
                act, out_act = B.TMA_ACT_NONE, self.Z[l + 1]
            self._layer_bwd(l, act, out_act)

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
