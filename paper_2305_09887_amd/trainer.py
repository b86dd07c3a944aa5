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

    With ``decoder_dims`` = [F_L, D_1, ..., 1] the task is link prediction (Sec. 4.1; App., formulation of the MLP
    decoder) instead of node classification: each step draws ``batch_size`` positive local edges and one
    random-tail negative each (counter-based, ``batch_seed``), multiplies the encoder's embeddings of the two
    ends, runs the MLP decoder (PReLU between its layers, no bias) and takes the mean binary cross-entropy of its
    logits; ``labels`` is then unused.  The decoder's weights (Theta_k, and a slope per hidden layer) follow the
    encoder's in ``W``, so they are averaged with them.
    """

    def __init__(self, rowptr, colidx, inv_deg, X, labels, dims, params=None, stream=None,
                 rowptr_T=None, colidx_T=None, norm_act=False, optimizer="sgd", encoder="sage",
                 decoder_dims=None, batch_size=0, batch_seed=0, nnz=None):
        self.norm_act = bool(norm_act)
        self.dec_dims = list(decoder_dims) if decoder_dims is not None else None
        if self.dec_dims is not None:
            if self.dec_dims[0] != dims[-1] or self.dec_dims[-1] != 1 or len(self.dec_dims) < 2 or batch_size < 1:
                raise B.TmaError("LocalTrainer: decoder_dims must run from dims[-1] to 1, with a batch size")
            if nnz is None:
                raise B.TmaError("LocalTrainer: the link task needs the local entry count nnz")
        self.batch_size, self.batch_seed, self.nnz = int(batch_size), int(batch_seed), nnz
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
        if self.dec_dims is not None:
            self.n_params += sum(a * b for a, b in zip(self.dec_dims[:-1], self.dec_dims[1:])) + len(self.dec_dims) - 2
        self.W = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        self.dW = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        (self.layers, self.dec_layers), (self.grads, self.dec_grads) = self._views(self.W), self._views(self.dW)
        if optimizer == "adam":   # moment estimates: this trainer's own state, never averaged
            self.adam_m = torch.zeros_like(self.W)
            self.adam_v = torch.zeros_like(self.W)
        if params is not None:
            self.load_params(params)

        n = max(self.n, 1)
        # activations and their gradients share one row pitch per layer, padded to 16 bytes so that a
        # width such as 47 still takes the library's vector paths
        self.H = [X] + [B._padded(self.n, f, self.dtype, dev) for f in dims[1:]]
        # the saved aggregate of a SAGE layer may have padded rows (16-byte pieces for any width); GCN's is dense
        self.M = ([(B._padded(n, f, self.dtype, dev) if encoder == "sage" else
                    torch.empty((n, f), dtype=self.dtype, device=dev))[: self.n] for f in dims[:-1]]
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
        if self.dec_dims is not None:
            Bn, dd = self.batch_size, self.dec_dims
            self.batch = tuple(torch.empty(Bn, dtype=torch.int32, device=dev) for _ in range(3))   # u, v, v'
            # E[k]: input of decoder layer k (E[0] the pair products); Zd[k]: output of layer k-1 before its PReLU;
            # dE[k]: gradient w.r.t. E[k], and, for k >= 1, w.r.t. Zd[k] once the PReLU's backward has run in place
            self.E = [B._padded(2 * Bn, f, self.dtype, dev) for f in dd[:-1]]
            self.Zd = [None] + [B._padded(2 * Bn, f, self.dtype, dev) for f in dd[1:]]
            self.dE = [B._padded(2 * Bn, f, self.dtype, dev) for f in dd]
            ws_bytes = max(ws_bytes, B.tma_pair_product_bwd_workspace_bytes(self.n, Bn, dd[0], dt),
                           B.tma_prelu_bwd_workspace_bytes(), B.tma_bce_logits_workspace_bytes(),
                           max(B.tma_dense_bwd_workspace_bytes(2 * Bn, a, b) for a, b in zip(dd[:-1], dd[1:])))
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.steps_done = 0

    def set_graph(self, rowptr, colidx, inv_deg, rowptr_T=None, colidx_T=None, nnz=None):
        """Point the trainer at a freshly extracted subgraph with the same node count."""
        if nnz is not None:
            self.nnz = nnz
        if rowptr.numel() != self.n + 1 or inv_deg.numel() != self.n:
            raise B.TmaError("LocalTrainer.set_graph: node count differs from the allocated buffers")
        self.rowptr, self.colidx, self.inv_deg = rowptr, colidx, inv_deg
        self.rowptr_T = rowptr if rowptr_T is None else rowptr_T
        self.colidx_T = colidx if colidx_T is None else colidx_T
        if self.encoder == "gcn":
            B.tma_gcn_norm(rowptr, out=self.s_norm, stream=self.stream)

    def set_data(self, X, labels=None):
        """Point the trainer at other feature rows (and labels) for the same nodes, e.g. the other half of a
        double buffer that a second stream has filled."""
        if X.shape != self.H[0].shape or X.dtype != self.dtype or X.stride() != self.H[0].stride():
            raise B.TmaError("LocalTrainer.set_data: X differs in shape, dtype or row stride from the one it replaces")
        if labels is not None and (self.labels is None or labels.shape != self.labels.shape):
            raise B.TmaError("LocalTrainer.set_data: labels differ in shape from the ones they replace")
        self.X = X
        self.H[0] = X
        if labels is not None:
            self.labels = labels

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
        dec = []
        if self.dec_dims is not None:
            K = len(self.dec_dims) - 1
            for k, (a, b) in enumerate(zip(self.dec_dims[:-1], self.dec_dims[1:])):
                layer = [flat[o:o + a * b].view(a, b)]; o += a * b
                if k < K - 1:
                    layer.append(flat[o:o + 1]); o += 1
                dec.append(tuple(layer))
        return out, dec

    def load_params(self, params, decoder_params=None):
        """params: per layer (W_self, W_neigh, bias) -- (W, bias) for GCN and MLP -- or, for a normalised layer,
        (..., gamma, beta, slope).  decoder_params: per decoder layer (Theta, slope), the last one (Theta,)."""
        pairs = list(zip(self.layers, params))
        if decoder_params is not None:
            pairs += list(zip(self.dec_layers, decoder_params))
        with torch.cuda.stream(self.stream):
            for mine, given in pairs:
                if len(mine) != len(given):
                    raise B.TmaError("LocalTrainer.load_params: layer has a different number of tensors")
                for dst, src in zip(mine, given):
                    dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))

    def _layer_fwd(self, l, act, out):
        lin = self.layers[l][:self.n_lin]
        if self.encoder == "sage":
            Wt = None
            F_in, F_out = lin[0].shape
            if (self.dtype == torch.bfloat16 and F_in % 4 == 0
                    and B.tma_sage_layer_aggregates_first(F_in, F_out, B.TMA_BF16)):
                # bf16 storage: the product takes its weight operand narrowed once per pass, not once per tile
                # (prepared anew every pass: the optimizer, an averaging or a caller may have changed the weights)
                held = getattr(self, "_Wt", None)
                if held is None:
                    held = self._Wt = {}
                if l not in held:
                    held[l] = torch.empty(B.tma_sage_weights_bf16_bytes(F_in, F_out) // 2, dtype=torch.int16,
                                          device=lin[0].device)
                Wt = B.tma_sage_prepare_weights_bf16(lin[0], lin[1], out=held[l], stream=self.stream)
            B.tma_sage_layer_fwd(self.rowptr, self.colidx, self.inv_deg, self.H[l], lin[0], lin[1], lin[2], act,
                                 M_out=self.M[l], Hnext_out=out, stream=self.stream, Wt=Wt)
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

    def time_layers(self, on: bool = True):
        """Bracket every encoder layer's forward and backward with a pair of events on the trainer's stream
        (aggregation, products, normalisation of that layer); `layer_times_ms()` reads them back."""
        self._layer_events = {"fwd": [[] for _ in range(self.L)], "bwd": [[] for _ in range(self.L)]} if on else None

    def _mark(self, which, l):
        ev = getattr(self, "_layer_events", None)
        if ev is None:
            return None
        e = torch.cuda.Event(enable_timing=True)
        e.record(self.stream)
        ev[which][l].append(e)
        return e

    def layer_times_ms(self):
        """{"fwd": [[ms per recorded pass] per layer], "bwd": ...}; waits for the stream."""
        self.stream.synchronize()
        ev = self._layer_events
        return {w: [[a.elapsed_time(b) for a, b in zip(per[0::2], per[1::2])] for per in ev[w]] for w in ("fwd", "bwd")}

    def forward(self):
        for l in range(self.L):
            self._mark("fwd", l)
            if self.norm_act and l < self.L - 1:
                gamma, beta, slope = self.layers[l][self.n_lin:]
                self._layer_fwd(l, B.TMA_ACT_NONE, self.Z[l + 1])
                B.tma_layernorm_prelu_fwd(self.Z[l + 1], gamma, beta, slope, out=self.H[l + 1], stream=self.stream)
            else:
                self._layer_fwd(l, B.TMA_ACT_RELU if l < self.L - 1 else B.TMA_ACT_NONE, self.H[l + 1])
            self._mark("fwd", l)
        return self.H[self.L]

    def _draw_batch(self):
        u, v, vneg = self.batch
        B.tma_edge_batch(self.rowptr, self.colidx, self.nnz, self.batch_seed, self.steps_done * self.batch_size,
                         self.batch_size, u_out=u, v_out=v, vneg_out=vneg, stream=self.stream)

    def _decoder_forward(self, R):
        """Pair products of the batch (indices into the rows of R), decoder layers; the logits end up in Zd[K]."""
        u, v, vneg = self.batch
        B.tma_pair_product_fwd(R, u, v, vneg, E0_out=self.E[0], stream=self.stream)
        K = len(self.dec_dims) - 1
        for k in range(K):
            B.tma_dense_fwd(self.E[k], self.dec_layers[k][0], None, B.TMA_ACT_NONE, Y_out=self.Zd[k + 1],
                            stream=self.stream)
            if k < K - 1:
                B.tma_prelu_fwd(self.Zd[k + 1], self.dec_layers[k][1], out=self.E[k + 1], stream=self.stream)
        return self.Zd[K]

    def _decoder_backward(self, R, dR_out):
        """Loss of the logits and the chain rule down to d(loss)/d(R), written to dR_out."""
        K = len(self.dec_dims) - 1
        u, v, vneg = self.batch
        B.tma_bce_logits(self.Zd[K], self.batch_size, loss_out=self.loss, dz_out=self.dE[K], ws=self.ws,
                         stream=self.stream)
        for k in range(K - 1, -1, -1):
            if k < K - 1:   # through the PReLU that follows layer k, in place
                B.tma_prelu_bwd(self.Zd[k + 1], self.dE[k + 1], self.dec_layers[k][1], dZ_out=self.dE[k + 1],
                                dslope=self.dec_grads[k][1], ws=self.ws, stream=self.stream)
            B.tma_dense_bwd(self.E[k], None, self.dE[k + 1], self.dec_layers[k][0], B.TMA_ACT_NONE,
                            dW=self.dec_grads[k][0], need_dbias=False, dX_out=self.dE[k], ws=self.ws,
                            stream=self.stream)
        B.tma_pair_product_bwd(R, u, v, vneg, self.dE[0], dR_out=dR_out, ws=self.ws, stream=self.stream)

    def backward(self):
        if self.dec_dims is not None:
            self._decoder_backward(self.H[self.L], self.dH[self.L])
        else:
            B.tma_softmax_ce(self.H[self.L], self.labels, loss_out=self.loss, dlogits_out=self.dH[self.L],
                             ws=self.ws, stream=self.stream)
        for l in range(self.L - 1, -1, -1):
            self._mark("bwd", l)
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
            self._mark("bwd", l)

    def _optimizer_step(self, lr: float):
        if self.optimizer == "adam":
            B.tma_adam_step(self.W, self.dW, self.adam_m, self.adam_v, lr, self.steps_done + 1, stream=self.stream)
        else:
            B.tma_sgd_step(self.W, self.dW, lr, stream=self.stream)
        self.steps_done += 1

    def step(self, lr: float):
        """One iteration of Alg. 2's loop body on the full local subgraph."""
        self.forward()
        if self.dec_dims is not None:
            self._draw_batch()
            self._decoder_forward(self.H[self.L])
        self.backward()
        self._optimizer_step(lr)
        return self.loss


class _Mfg:
    """Buffers of one mini-batch's message-flow graph: the batch, the node list of every level, the blocks, the
    gathered input features, and the sampler's own workspace (so that a batch can be sampled on one stream while
    another one trains).  ``ready``: recorded when all of it has been written; ``released``: recorded on the
    training stream after the last pass that read it."""

    def __init__(self, cap, ecap, Bn, F0, n, dtype, dev):
        L = len(cap) - 1
        i32 = lambda k: torch.empty(k, dtype=torch.int32, device=dev)
        self.nodes = [i32(c) for c in cap]
        self.count = [0] * (L + 1)
        self.blk_rowptr = [i32(cap[l + 1] + 1) for l in range(L)]
        self.blk_col = [i32(ecap[l]) for l in range(L)]
        self.blk_row = [i32(ecap[l]) for l in range(L)]
        self.blk_inv_deg = [torch.empty(cap[l + 1], dtype=torch.float32, device=dev) for l in range(L)]
        self.H0 = torch.empty((cap[0], F0), dtype=dtype, device=dev)
        self.bcat = i32(3 * Bn)                       # u | v | v': node ids when drawn, then positions in level L
        self.batch = (self.bcat[:Bn], self.bcat[Bn:2 * Bn], self.bcat[2 * Bn:])
        ws_bytes = max(max(B.tma_neighbor_sample_workspace_bytes(cap[l + 1]) for l in range(L)),
                       B.tma_mfg_relabel_workspace_bytes(n))
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        # level sizes as the sampler leaves them on the device, and where they are copied for the host
        self.d_count = i32(L + 1)
        self.h_count = torch.empty(L + 1, dtype=torch.int32, pin_memory=True)
        self.counted = None          # recorded after that copy; None once the sizes are in `count`
        self.step = -1
        self.ready = self.released = None

    def resolve(self):
        """Wait (the only wait of a batch) until the level sizes have arrived on the host."""
        if self.counted is not None:
            self.counted.synchronize()
            self.count[:] = self.h_count.tolist()
            self.counted = None


class SampledLinkTrainer(LocalTrainer):
    """Link prediction on the sampled message-flow graph of each mini-batch (Sec. 4.1: random positive edges, one
    random-tail negative each, a GraphSAGE-style sampler that caps the neighbours per node and layer, MLP decoder).

    Per step: draw the batch, list its distinct nodes, and for layer l = L-1 .. 0 sample up to ``fanouts[l]``
    neighbours of every node of the level above and list the nodes reached; gather the features of the lowest
    level; run the mean-aggregation SAGE layers on the bipartite blocks, the decoder and the loss; go back the same
    way.  Only the sampled neighbourhood is touched.  Hidden layers use ReLU, or with ``norm_act`` layer
    normalisation followed by PReLU.  All buffers are sized once for the largest possible level
    (3 * batch_size nodes at the top, times 1 + fanout per layer, capped by the local node count).  The level sizes
    of a batch stay on the device while it is sampled (launches sized for the capacities) and come back with one
    copy, waited for once before the training pass is enqueued; ``device_counts=False`` fetches each level's size as
    soon as it exists instead (one wait per level, launches of the exact sizes).  The neighbour sampler's seed for step t and layer l is
    SplitMix64(batch_seed, 64 t + l).  ``encoder``: "sage" (W_self, W_neigh, b per layer) or "gcn" (W, b per layer;
    on a block the layer averages over the sampled neighbours and the node itself).

    A batch and its message-flow graph depend on the graph, the seeds and the step number only, never on the
    model: after ``enable_prefetch()`` every ``step`` trains on the batch that was sampled while the step before
    it trained (a second stream, a second set of buffers), and then starts the sampling of the next one, so the
    sampler's kernels and its waits for the level sizes fall beside the training kernels.  Same batches, same
    arithmetic, same bits as without it.
    """

    def __init__(self, rowptr, colidx, nnz, X, dims, decoder_dims, fanouts, batch_size, batch_seed=0, params=None,
                 decoder_params=None, stream=None, optimizer="sgd", norm_act=False, nnz_cap=None, encoder="sage",
                 device_counts=True):
        self.device_counts = bool(device_counts)
        if len(fanouts) != len(dims) - 1:
            raise B.TmaError("SampledLinkTrainer: one fan-out per layer")
        if colidx.numel() < nnz or (nnz_cap is not None and nnz_cap < nnz):
            raise B.TmaError("SampledLinkTrainer: nnz entries must be there in colidx, and nnz_cap >= nnz")
        if encoder not in ("sage", "gcn"):
            raise B.TmaError("SampledLinkTrainer: encoder must be 'sage' or 'gcn'")
        self.norm_act, self.encoder, self.n_lin = bool(norm_act), encoder, 3 if encoder == "sage" else 2
        if optimizer not in ("sgd", "adam"):
            raise B.TmaError("SampledLinkTrainer: optimizer must be 'sgd' or 'adam'")
        self.optimizer = optimizer
        self.dec_dims = list(decoder_dims)
        if self.dec_dims[0] != dims[-1] or self.dec_dims[-1] != 1 or batch_size < 1:
            raise B.TmaError("SampledLinkTrainer: decoder_dims must run from dims[-1] to 1, with a batch size")
        self.rowptr, self.colidx, self.nnz, self.X = rowptr, colidx, int(nnz), X
        # the block buffers are sized for graphs of up to this many entries (set_graph may bring a larger graph)
        self.nnz_cap = int(nnz if nnz_cap is None else nnz_cap)
        self.dims, self.L, self.n, self.dtype = list(dims), len(dims) - 1, X.shape[0], X.dtype
        self.fanouts = [int(f) for f in fanouts]
        self.batch_size, self.batch_seed = int(batch_size), int(batch_seed)
        dev, L, Bn = X.device, self.L, self.batch_size
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        if X.shape[1] != dims[0] or not X.is_contiguous():
            raise B.TmaError("SampledLinkTrainer: X must be a dense [n, dims[0]] table")

        self.n_params = sum((self.n_lin - 1) * fi * fo + fo for fi, fo in zip(dims[:-1], dims[1:]))
        if self.norm_act:
            self.n_params += sum(2 * fo + 1 for fo in dims[1:-1])
        self.n_params += sum(a * b for a, b in zip(self.dec_dims[:-1], self.dec_dims[1:])) + len(self.dec_dims) - 2
        self.W = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        self.dW = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        (self.layers, self.dec_layers), (self.grads, self.dec_grads) = self._views(self.W), self._views(self.dW)
        if optimizer == "adam":
            self.adam_m, self.adam_v = torch.zeros_like(self.W), torch.zeros_like(self.W)
        if params is not None:
            self.load_params(params, decoder_params)

        # capacities: nodes of level l (the input rows of layer l; level L = the batch's nodes), entries of block l
        cap = [0] * (L + 1)
        cap[L] = max(min(self.n, 3 * Bn), 1)
        for l in range(L - 1, -1, -1):
            cap[l] = max(min(self.n, cap[l + 1] * (1 + self.fanouts[l])), 1)
        self.cap = cap
        self.ecap = [max(min(cap[l + 1] * self.fanouts[l], self.nnz_cap), 1) for l in range(L)]
        self._mfgs = [_Mfg(cap, self.ecap, Bn, dims[0], self.n, self.dtype, dev)]
        self._side = self._pending = self._inputs_ready = self._worker = None
        self._auto = True
        self.H = [None] + [B._padded(cap[l], dims[l], self.dtype, dev) for l in range(1, L + 1)]
        self._bind(self._mfgs[0])
        self.M = [torch.empty((cap[l + 1], dims[l]), dtype=self.dtype, device=dev) for l in range(L)]
        self.dH = [None] + [B._padded(cap[l], dims[l], self.dtype, dev) for l in range(1, L + 1)]
        # pre-activations of the normalised hidden layers (index l + 1 = output of layer l), kept for the backward
        self.Z = [None] + [B._padded(cap[l], dims[l], self.dtype, dev) if self.norm_act and l < L else None
                           for l in range(1, L + 1)]
        dd, dt = self.dec_dims, B._feat_dtype(X)
        self.E = [B._padded(2 * Bn, f, self.dtype, dev) for f in dd[:-1]]
        self.Zd = [None] + [B._padded(2 * Bn, f, self.dtype, dev) for f in dd[1:]]
        self.dE = [B._padded(2 * Bn, f, self.dtype, dev) for f in dd]
        ws_bytes = max(          # the training pass's workspace (the sampler's is part of each batch's buffers)
            max((B.tma_sage_block_bwd_workspace_bytes if encoder == "sage" else B.tma_gcn_block_bwd_workspace_bytes)(
                cap[l + 1], cap[l], self.ecap[l], dims[l], dims[l + 1], dt, l > 0) for l in range(L)),
            B.tma_pair_product_bwd_workspace_bytes(cap[L], Bn, dd[0], dt), B.tma_prelu_bwd_workspace_bytes(),
            B.tma_bce_logits_workspace_bytes(),
            max(B.tma_dense_bwd_workspace_bytes(2 * Bn, a, b) for a, b in zip(dd[:-1], dd[1:])))
        if self.norm_act and L > 1:
            ws_bytes = max(ws_bytes, max(B.tma_layernorm_prelu_bwd_workspace_bytes(cap[l], dims[l]) for l in range(1, L)))
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.steps_done = 0

    def _bind(self, mfg):
        """The batch the training pass works on."""
        self._cur = mfg
        self.nodes, self.count, self.blk_rowptr, self.blk_col = mfg.nodes, mfg.count, mfg.blk_rowptr, mfg.blk_col
        self.blk_row, self.blk_inv_deg, self.bcat, self.batch = mfg.blk_row, mfg.blk_inv_deg, mfg.bcat, mfg.batch
        self.H[0] = mfg.H0

    def set_graph(self, rowptr, colidx, nnz, ready=None):
        """Point the trainer at another local graph over the same nodes, with at most the entry count given at
        construction.  ``ready``: an event after which its arrays may be read (for sampling on the second stream)."""
        if rowptr.numel() != self.n + 1 or nnz > self.nnz_cap:
            raise B.TmaError("SampledLinkTrainer.set_graph: node count or entry count beyond the allocated buffers")
        self.rowptr, self.colidx, self.nnz = rowptr, colidx, int(nnz)
        self._inputs_ready = ready

    def set_data(self, X, labels=None):
        """Point the trainer at another feature table over the same nodes."""
        if X.shape != self.X.shape or X.dtype != self.dtype or not X.is_contiguous():
            raise B.TmaError("SampledLinkTrainer.set_data: X differs in shape or dtype from the one it replaces")
        self.X = X

    def sample(self, mfg=None, step=None, stream=None):
        """The batch of step ``step`` (default: the next one) and its message-flow graph: node lists, blocks, input
        features, written to ``mfg`` (default: the buffers the training pass reads) on ``stream``."""
        mfg = self._cur if mfg is None else mfg
        t = self.steps_done if step is None else int(step)
        L, Bn, st = self.L, self.batch_size, self.stream if stream is None else stream
        u, v, vneg = mfg.batch
        B.tma_edge_batch(self.rowptr, self.colidx, self.nnz, self.batch_seed, t * Bn, Bn, u_out=u, v_out=v, vneg_out=vneg,
                         stream=st)
        if self.device_counts:
            return self._sample_levels_on_device(mfg, t, st)
        _, mfg.count[L] = B.tma_mfg_relabel(self.n, None, 0, mfg.bcat, 3 * Bn, src_out=mfg.nodes[L], ws=mfg.ws, stream=st)
        for l in range(L - 1, -1, -1):
            n_dst = mfg.count[l + 1]
            B.tma_neighbor_sample(mfg.nodes[l + 1], n_dst, self.nnz, self.rowptr, self.colidx, self.fanouts[l],
                                  B.tma_mix64(self.batch_seed, 64 * t + l), blk_rowptr_out=mfg.blk_rowptr[l],
                                  blk_col_out=mfg.blk_col[l], blk_row_out=mfg.blk_row[l], ws=mfg.ws, stream=st)
            _, mfg.count[l] = B.tma_mfg_relabel(self.n, mfg.nodes[l + 1], n_dst, mfg.blk_col[l], self.ecap[l],
                                                d_items=mfg.blk_rowptr[l][n_dst:n_dst + 1], src_out=mfg.nodes[l],
                                                ws=mfg.ws, stream=st)
            if self.encoder == "sage":
                B.tma_block_inv_deg(mfg.blk_rowptr[l], n_dst, out=mfg.blk_inv_deg[l], stream=st)
            else:
                B.tma_gcn_block_norm(mfg.blk_rowptr[l], n_dst, out=mfg.blk_inv_deg[l], stream=st)
        B.tma_gather_rows(mfg.nodes[0][:mfg.count[0]], self.X, out=mfg.H0[:mfg.count[0]], stream=st)
        mfg.step = t

    def _sample_levels_on_device(self, mfg, t, st):
        """The levels of batch t with their sizes left on the device: nothing here waits for the GPU."""
        L, Bn, dc = self.L, self.batch_size, mfg.d_count
        B.tma_mfg_relabel_dev(self.n, None, 0, None, mfg.bcat, 3 * Bn, src_out=mfg.nodes[L], n_src_out=dc[L:L + 1],
                              ws=mfg.ws, stream=st)
        for l in range(L - 1, -1, -1):
            cap_dst, d_n_dst = self.cap[l + 1], dc[l + 1:l + 2]
            B.tma_neighbor_sample_dev(mfg.nodes[l + 1], cap_dst, d_n_dst, self.nnz, self.rowptr, self.colidx,
                                      self.fanouts[l], B.tma_mix64(self.batch_seed, 64 * t + l),
                                      blk_rowptr_out=mfg.blk_rowptr[l], blk_col_out=mfg.blk_col[l],
                                      blk_row_out=mfg.blk_row[l], ws=mfg.ws, stream=st)
            # (the rows past the level's size have no entries: the element at the capacity holds the entry count)
            B.tma_mfg_relabel_dev(self.n, mfg.nodes[l + 1], cap_dst, d_n_dst, mfg.blk_col[l], self.ecap[l],
                                  d_items=mfg.blk_rowptr[l][cap_dst:cap_dst + 1], src_out=mfg.nodes[l],
                                  n_src_out=dc[l:l + 1], ws=mfg.ws, stream=st)
            if self.encoder == "sage":
                B.tma_block_inv_deg(mfg.blk_rowptr[l], cap_dst, out=mfg.blk_inv_deg[l], stream=st)
            else:
                B.tma_gcn_block_norm(mfg.blk_rowptr[l], cap_dst, out=mfg.blk_inv_deg[l], stream=st)
        B.tma_gather_rows_dev(mfg.nodes[0], dc[0:1], self.X, mfg.H0, stream=st)
        with torch.cuda.stream(st):
            mfg.h_count.copy_(dc, non_blocking=True)
            mfg.counted = torch.cuda.Event()
            mfg.counted.record(st)
        mfg.step = t

    def enable_prefetch(self, stream=None, auto=True, background=False):
        """From now on ``step`` trains on a batch sampled ahead on a second stream (``stream``, or a new one of
        default priority) into a second set of buffers; see the class description.  ``auto``: every step starts
        the sampling of the next one itself; otherwise the caller does, with prefetch_sample(), once the graph and
        features of the next step are known (set_graph / set_data).  ``background``: the sampling calls, with
        their waits for the level sizes, are made by a worker thread, so that the calling thread goes straight on
        to enqueue the next training pass (the library's calls release the interpreter lock)."""
        self._drain()
        self._side = stream if stream is not None else torch.cuda.Stream(device=self.W.device)
        self._auto, self._pending = bool(auto), None
        if background and self._worker is None:
            from concurrent.futures import ThreadPoolExecutor
            self._worker = ThreadPoolExecutor(max_workers=1, thread_name_prefix="tma-sampler")
        elif not background and self._worker is not None:
            self._worker.shutdown(wait=True)
            self._worker = None
        if len(self._mfgs) < 2:
            self._mfgs.append(_Mfg(self.cap, self.ecap, self.batch_size, self.dims[0], self.n, self.dtype, self.W.device))

    def _drain(self):
        """Wait for a sampling that a worker thread is still making."""
        if self._pending is not None and hasattr(self._pending, "result"):
            self._pending = self._pending.result()

    def disable_prefetch(self):
        """Back to sampling inside ``step`` on the training stream (waits for a sampling that is under way)."""
        self._drain()
        if self._side is not None:
            self._side.synchronize()
        if self._worker is not None:
            self._worker.shutdown(wait=True)
        self._side = self._pending = self._worker = None

    def prefetch_sample(self, prepare=None):
        """Start sampling the next step's batch on the second stream, from the graph and feature table the trainer
        points at (after the event given with set_graph, if any).  The level sizes are waited for here, or by the
        worker thread, while the training stream works through what has been enqueued.  ``prepare``: called first,
        in the thread that samples (e.g. the next step's extraction followed by set_graph / set_data)."""
        if self._side is None:
            raise B.TmaError("SampledLinkTrainer.prefetch_sample: call enable_prefetch() first")
        self._drain()
        t = self.steps_done
        mfg, side = self._mfgs[t % 2], self._side

        def work():
            if prepare is not None:
                prepare()
            with torch.cuda.stream(side):
                if mfg.released is not None:        # the training pass that last read these buffers
                    side.wait_event(mfg.released)
                if self._inputs_ready is not None:
                    side.wait_event(self._inputs_ready)
                self.sample(mfg, t, side)
                mfg.ready = torch.cuda.Event()
                mfg.ready.record(side)
            return mfg

        self._pending = self._worker.submit(work) if self._worker is not None else work()

    def _block_fwd(self, l, act, out):
        block_fwd = B.tma_sage_block_fwd if self.encoder == "sage" else B.tma_gcn_block_fwd
        block_fwd(self.count[l + 1], self.count[l], self.blk_rowptr[l], self.blk_col[l], self.blk_inv_deg[l], self.H[l],
                  *self.layers[l][:self.n_lin], act, self.M[l], out, stream=self.stream)

    def forward(self):
        for l in range(self.L):
            n_dst = self.count[l + 1]
            if self.norm_act and l < self.L - 1:
                gamma, beta, slope = self.layers[l][self.n_lin:]
                self._block_fwd(l, B.TMA_ACT_NONE, self.Z[l + 1])
                B.tma_layernorm_prelu_fwd(self.Z[l + 1][:n_dst], gamma, beta, slope, out=self.H[l + 1][:n_dst],
                                          stream=self.stream)
                continue
            self._block_fwd(l, B.TMA_ACT_RELU if l < self.L - 1 else B.TMA_ACT_NONE, self.H[l + 1])
        return self.H[self.L][:self.count[self.L]]

    def backward(self):
        n_top = self.count[self.L]
        self._decoder_backward(self.H[self.L][:n_top], self.dH[self.L][:n_top])
        for l in range(self.L - 1, -1, -1):
            act = B.TMA_ACT_RELU if l < self.L - 1 else B.TMA_ACT_NONE
            out_act, n_dst = self.H[l + 1], self.count[l + 1]
            if self.norm_act and l < self.L - 1:
                gamma, beta, slope = self.layers[l][self.n_lin:]
                dgamma, dbeta, dslope = self.grads[l][self.n_lin:]
                # dL/dZ replaces dL/dH' in place; the layer below then runs without an activation of its own
                B.tma_layernorm_prelu_bwd(self.Z[l + 1][:n_dst], self.dH[l + 1][:n_dst], gamma, beta, slope,
                                          dZ_out=self.dH[l + 1][:n_dst], dgamma=dgamma, dbeta=dbeta, dslope=dslope,
                                          ws=self.ws, stream=self.stream)
                act, out_act = B.TMA_ACT_NONE, self.Z[l + 1]
            block = (n_dst, self.count[l], self.ecap[l], self.blk_rowptr[l], self.blk_col[l], self.blk_row[l],
                     self.blk_inv_deg[l])
            dH_out = self.dH[l] if l > 0 else None
            if self.encoder == "sage":
                ws_, wn = self.layers[l][:2]
                dws, dwn, db = self.grads[l][:3]
                B.tma_sage_block_bwd(*block, self.H[l], self.M[l], out_act, self.dH[l + 1], ws_, wn, act, dws, dwn, db,
                                     dH_out=dH_out, ws=self.ws, stream=self.stream)
            else:
                dw, db = self.grads[l][:2]
                B.tma_gcn_block_bwd(*block, self.M[l], out_act, self.dH[l + 1], self.layers[l][0], act, dw, db,
                                    dH_out=dH_out, ws=self.ws, stream=self.stream)

    def step(self, lr: float):
        """One iteration of Alg. 2's loop body on the sampled neighbourhood of one mini-batch."""
        if self._side is None:
            self.sample()
            self._cur.resolve()
        else:
            self._drain()
            if self._pending is None or self._pending.step != self.steps_done:
                self.prefetch_sample()             # nothing sampled ahead (first step, or the step count was set)
                self._drain()
            mfg, self._pending = self._pending, None
            mfg.resolve()
            self.stream.wait_event(mfg.ready)
            self._bind(mfg)
        R = self.forward()
        self._decoder_forward(R)
        self.backward()
        self._optimizer_step(lr)
        if self._side is not None:
            self._cur.released = torch.cuda.Event()
            self._cur.released.record(self.stream)
            if self._auto:
                self.prefetch_sample()
        return self.loss


class SubgraphPrefetcher:
    """Partition + induced-subgraph extraction + row gathers of the NEXT step on a stream of its own while the
    current step trains (Alg. 1: a trainer's part, its subgraph and its feature rows depend on the assignment seed
    only, not on the model).

    ``start(seed)`` launches them on the extraction stream, waits on the host for the two sizes (the library's
    extraction call returns them) and hands back ``(subgraph dict, gathered tables, event)``; the consumer's stream
    waits for the event before its first kernel that reads any of it.  The host therefore never stalls the training
    stream for the sizes: they arrive while the previous step is still running.  ``tables``: global per-node arrays
    whose local rows are gathered into one of two buffers each (capacity cap_n_loc rows), alternating between
    calls.  ``after``: an event the work must wait for before it may write, namely the end of the last training
    step that read what this call overwrites or may be handed again by the allocator (the step before the one now
    running).  Host logic only.
    """

    def __init__(self, rowptr, colidx, n_nodes: int, K: int, p: int, cap_n_loc=None, cap_nnz_loc=None, cluster=None,
                 n_clusters: int = 0, tables=()):
        self.rowptr, self.colidx, self.n_nodes, self.K, self.p = rowptr, colidx, int(n_nodes), int(K), int(p)
        self.cap_n_loc, self.cap_nnz_loc = cap_n_loc, cap_nnz_loc
        self.cluster, self.n_clusters = cluster, n_clusters
        dev = rowptr.device
        self.stream = torch.cuda.Stream(device=dev)        # default priority
        self.part = torch.empty(self.n_nodes, dtype=torch.int32, device=dev)
        self.tables = list(tables)
        if self.tables and cap_n_loc is None:
            raise B.TmaError("SubgraphPrefetcher: gathering tables needs cap_n_loc")
        self.slot = 0
        self.buffers = [[torch.empty((int(cap_n_loc),) + tuple(t.shape[1:]), dtype=t.dtype, device=dev) for t in self.tables]
                        for _ in range(2)]

    def start(self, seed: int, after=None):
        with torch.cuda.stream(self.stream):
            if after is not None:
                self.stream.wait_event(after)
            B.tma_partition(self.n_nodes, self.K, seed, cluster=self.cluster, n_clusters=self.n_clusters, out=self.part)
            sub = B.tma_induced_subgraph(self.rowptr, self.colidx, self.part, self.p, cap_n_loc=self.cap_n_loc,
                                         cap_nnz_loc=self.cap_nnz_loc)
            gathered = [B.tma_gather_rows(sub["l2g"], t, out=buf[:sub["n_loc"]])
                        for t, buf in zip(self.tables, self.buffers[self.slot])]
            self.slot ^= 1
            done = torch.cuda.Event()
            done.record(self.stream)
        return sub, gathered, done
