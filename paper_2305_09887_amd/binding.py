"""ctypes binding of libtma: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and
streams, nothing else); every computation happens in the library's kernels.
The library is loaded on first use; if it has not been built the call raises --
there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("TMA_LIBRARY_PATH") or os.path.join(_PKG, "libtma.so")   # (a build elsewhere: set TMA_LIBRARY_PATH)

TMA_F32, TMA_BF16 = 0, 1
TMA_ACT_NONE, TMA_ACT_RELU = 0, 1

EXPORTS = (
    "tma_version", "tma_last_error", "tma_partition", "tma_mix64",
    "tma_induced_subgraph_workspace_bytes", "tma_induced_subgraph_count", "tma_induced_subgraph_fill",
    "tma_induced_subgraph", "tma_induced_subgraph_async", "tma_random_subgraph_async",
    "tma_mean_aggregate", "tma_sage_layer_aggregates_first", "tma_sage_layer_fwd",
    "tma_sage_layer_bwd_workspace_bytes", "tma_sage_layer_bwd",
    "tma_layernorm_prelu_fwd", "tma_layernorm_prelu_bwd_workspace_bytes", "tma_layernorm_prelu_bwd",
    "tma_layernorm_prelu_bwd_static_max_f", "tma_layernorm_prelu_bwd_static",
    "tma_dense_fwd", "tma_dense_bwd_workspace_bytes", "tma_dense_bwd",
    "tma_gcn_norm", "tma_gcn_layer_aggregates_first", "tma_gcn_layer_fwd",
    "tma_gcn_layer_bwd_workspace_bytes", "tma_gcn_layer_bwd",
    "tma_edge_batch", "tma_pair_product_fwd", "tma_pair_product_bwd_workspace_bytes", "tma_pair_product_bwd",
    "tma_prelu_fwd", "tma_prelu_bwd_workspace_bytes", "tma_prelu_bwd", "tma_bce_logits_workspace_bytes",
    "tma_bce_logits",
    "tma_neighbor_sample_workspace_bytes", "tma_neighbor_sample", "tma_mfg_relabel_workspace_bytes", "tma_mfg_relabel",
    "tma_neighbor_sample_dev", "tma_mfg_relabel_dev", "tma_gather_rows_dev",
    "tma_sage_weights_bf16_bytes", "tma_sage_prepare_weights_bf16", "tma_sage_layer_fwd_prepared",
    "tma_block_inv_deg", "tma_sage_block_fwd", "tma_sage_block_bwd_workspace_bytes", "tma_sage_block_bwd",
    "tma_gcn_block_norm", "tma_gcn_block_fwd", "tma_gcn_block_bwd_workspace_bytes", "tma_gcn_block_bwd",
    "tma_loss_workspace_bytes", "tma_softmax_ce", "tma_sigmoid_l2", "tma_sgd_step", "tma_adam_step", "tma_average",
    "tma_gather_rows", "tma_profile_begin", "tma_profile_end", "tma_profile_count", "tma_profile_entry",
    "tma_profile_sequence_count", "tma_profile_sequence_entry",
)


class TmaError(RuntimeError):
    pass


_lib = None


def lib() -> C.CDLL:
    """The loaded C library (raises if libtma.so is missing)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise TmaError(f"{_LIB_PATH} not found: build it with `python -m paper_2305_09887_amd.build` "
                           "(there is no CPU fallback)")
        L = C.CDLL(_LIB_PATH)
        L.tma_last_error.restype = C.c_char_p
        for name in ("tma_induced_subgraph_workspace_bytes", "tma_sage_layer_bwd_workspace_bytes",
                     "tma_loss_workspace_bytes", "tma_layernorm_prelu_bwd_workspace_bytes",
                     "tma_dense_bwd_workspace_bytes", "tma_gcn_layer_bwd_workspace_bytes",
                     "tma_pair_product_bwd_workspace_bytes", "tma_prelu_bwd_workspace_bytes",
                     "tma_bce_logits_workspace_bytes", "tma_neighbor_sample_workspace_bytes",
                     "tma_mfg_relabel_workspace_bytes", "tma_sage_block_bwd_workspace_bytes",
                     "tma_gcn_block_bwd_workspace_bytes", "tma_sage_weights_bf16_bytes"):
            getattr(L, name).restype = C.c_size_t
        L.tma_mix64.restype = C.c_uint64
        L.tma_mix64.argtypes = [C.c_uint64, C.c_uint64]
        _lib = L
    return _lib


def tma_mix64(seed: int, unit: int) -> int:
    """SplitMix64(seed, unit), the library's generator, on the host (no GPU work)."""
    m = (1 << 64) - 1
    return int(lib().tma_mix64(seed & m, unit & m))


def _check(rc: int):
    if rc != 0:
        raise TmaError(f"libtma error {rc}: {lib().tma_last_error().decode()}")


def _stream(stream=None) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _ptr(t, dtype=None, name="tensor") -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise TmaError(f"{name}: expected a CUDA/HIP tensor")
    if dtype is not None and t.dtype != dtype:
        raise TmaError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TmaError(f"{name}: expected a contiguous tensor")
    return C.c_void_p(t.data_ptr())


def _feat_dtype(t) -> int:
    if t.dtype == torch.float32:
        return TMA_F32
    if t.dtype == torch.bfloat16:
        return TMA_BF16
    raise TmaError(f"unsupported feature dtype {t.dtype}")


def _rows_ld(t, name):
    """2-D row-major tensor, possibly with padded rows: returns (rows, cols, ld)."""
    if t.dim() != 2 or t.stride(1) != 1:
        raise TmaError(f"{name}: expected a 2-D tensor with unit inner stride")
    return t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _padded(n: int, cols: int, dtype, device) -> torch.Tensor:
    """[n, cols] view of a buffer whose rows are padded to a multiple of 16 bytes (vector-path friendly)."""
    per16 = 16 // torch.empty(0, dtype=dtype).element_size()
    ld = (cols + per16 - 1) // per16 * per16
    return torch.empty((max(n, 1), ld), dtype=dtype, device=device)[:n, :cols]


def _same_ld(a, b, what):
    if a is None or b is None:
        return
    if a.stride(0) != b.stride(0) and a.shape[0] > 1:
        raise TmaError(f"{what}: tensors must share one leading dimension")


def _record(t: torch.Tensor, stream) -> torch.Tensor:
    """A temporary allocated here (on torch's current stream) but used by kernels on `stream`: tell the caching
    allocator, so that the memory is not handed out again while those kernels run."""
    if stream is not None and t.is_cuda and stream != torch.cuda.current_stream(t.device):
        t.record_stream(stream)
    return t


def _workspace(nbytes: int, device, stream=None) -> torch.Tensor:
    return _record(torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device), stream)


def tma_version() -> int:
    return lib().tma_version()


# ---------------------------------------------------------------------------
def tma_partition(n_nodes: int, K: int, seed: int, cluster=None, n_clusters: int = 0, out=None, stream=None):
    """part[v] in [0,K): RandomTMA (cluster None) or SuperTMA (cluster = int32 super-node ids)."""
    dev = cluster.device if cluster is not None else torch.device("cuda", torch.cuda.current_device())
    if out is None:
        out = torch.empty(n_nodes, dtype=torch.int32, device=dev)
    if out.numel() != n_nodes or (cluster is not None and cluster.numel() != n_nodes):
        raise TmaError("tma_partition: part_out / cluster must have n_nodes elements")
    if cluster is not None and n_clusters <= 0:
        raise TmaError("tma_partition: n_clusters must be given with cluster")
    _check(lib().tma_partition(C.c_int64(n_nodes), _ptr(cluster, torch.int32, "cluster"), C.c_int64(n_clusters),
                               C.c_int32(K), C.c_uint64(seed), _ptr(out, torch.int32, "part_out"), _stream(stream)))
    return out


def tma_induced_subgraph(rowptr, colidx, part, p: int, cap_n_loc: int | None = None, cap_nnz_loc: int | None = None,
                         stream=None):
    """The extraction.  Returns dict(g2l, l2g, rowptr, colidx, inv_deg, n_loc, nnz_loc).  With both capacities
    given every buffer is allocated up front and the library makes both passes in one call; otherwise the
    entry list is allocated between the passes, at its exact size."""
    n = rowptr.numel() - 1
    if part.numel() != n:
        raise TmaError("tma_induced_subgraph: part must have one entry per node")
    dev = rowptr.device
    if colidx.numel() == 0:      # edgeless graph: the library wants a non-NULL pointer, never read
        colidx = torch.zeros(1, dtype=torch.int32, device=dev)
    cap = n if cap_n_loc is None else min(int(cap_n_loc), n)
    L = lib()
    ws_bytes = L.tma_induced_subgraph_workspace_bytes(C.c_int64(n), C.c_int64(cap))
    ws = _workspace(ws_bytes, dev, stream)
    g2l = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    l2g = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    rp = torch.empty(cap + 1, dtype=torch.int32, device=dev)
    n_loc, nnz_loc = C.c_int64(0), C.c_int64(0)
    if cap_nnz_loc is not None:
        ci = torch.empty(max(int(cap_nnz_loc), 1), dtype=torch.int32, device=dev)
        inv = torch.empty(max(cap, 1), dtype=torch.float32, device=dev)
        _check(L.tma_induced_subgraph(
            C.c_int64(n), _ptr(rowptr, torch.int64, "rowptr"), _ptr(colidx, torch.int32, "colidx"),
            _ptr(part, torch.int32, "part"), C.c_int32(p), _ptr(g2l), _ptr(l2g), _ptr(rp), _ptr(ci), _ptr(inv),
            C.c_int64(cap), C.c_int64(int(cap_nnz_loc)), C.byref(n_loc), C.byref(nnz_loc), _ptr(ws),
            C.c_size_t(ws.numel()), _stream(stream)))
        n_loc, nnz_loc = n_loc.value, nnz_loc.value
    else:
        _check(L.tma_induced_subgraph_count(
            C.c_int64(n), _ptr(rowptr, torch.int64, "rowptr"), _ptr(colidx, torch.int32, "colidx"),
            _ptr(part, torch.int32, "part"), C.c_int32(p), _ptr(g2l), _ptr(l2g), _ptr(rp), C.c_int64(cap),
            C.byref(n_loc), C.byref(nnz_loc), _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
        n_loc, nnz_loc = n_loc.value, nnz_loc.value
        ci = torch.empty(max(nnz_loc, 1), dtype=torch.int32, device=dev)
        inv = torch.empty(max(n_loc, 1), dtype=torch.float32, device=dev)
        _check(L.tma_induced_subgraph_fill(
            C.c_int64(n), _ptr(colidx), _ptr(g2l), C.c_int64(n_loc), _ptr(rp), _ptr(ci), _ptr(inv), C.c_int64(cap),
            _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return dict(g2l=g2l[:n], l2g=l2g[:n_loc], rowptr=rp[:n_loc + 1], colidx=ci[:nnz_loc], inv_deg=inv[:n_loc],
                n_loc=n_loc, nnz_loc=nnz_loc)


def tma_induced_subgraph_async(rowptr, colidx, part, p: int, cap_n_loc: int, cap_nnz_loc: int, out=None, stream=None,
                               rule=None):
    """The extraction without a host wait.  Returns dict(g2l, l2g, rowptr, colidx, inv_deg, sizes, ws): the buffers
    at their capacities and sizes = device int64 [|V^(p)|, kept entries].  Pass a previous result as `out` to
    write into the same buffers again (fixed addresses, as a captured graph needs).  rule = (K, seed) with part
    None: RandomTMA's assignment is recomputed inside the extraction (tma_random_subgraph_async)."""
    n = rowptr.numel() - 1
    if (part is None) == (rule is None):
        raise TmaError("tma_induced_subgraph_async: give either part or rule=(K, seed)")
    if part is not None and part.numel() != n:
        raise TmaError("tma_induced_subgraph_async: part must have one entry per node")
    dev = rowptr.device
    if colidx.numel() == 0:
        colidx = torch.zeros(1, dtype=torch.int32, device=dev)
    cap, cap_nnz = min(int(cap_n_loc), n), int(cap_nnz_loc)
    L = lib()
    ws_bytes = L.tma_induced_subgraph_workspace_bytes(C.c_int64(n), C.c_int64(cap))
    if out is None:
        i32 = lambda k: torch.empty(max(k, 1), dtype=torch.int32, device=dev)
        out = dict(g2l=i32(n), l2g=i32(cap), rowptr=i32(cap + 1), colidx=i32(cap_nnz),
                   inv_deg=torch.empty(max(cap, 1), dtype=torch.float32, device=dev),
                   sizes=torch.zeros(2, dtype=torch.int64, device=dev),
                   ws=torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev))
    if (out["g2l"].numel() < n or out["l2g"].numel() < cap or out["rowptr"].numel() < cap + 1
            or out["colidx"].numel() < cap_nnz or out["inv_deg"].numel() < cap or out["ws"].numel() < ws_bytes):
        raise TmaError("tma_induced_subgraph_async: `out` holds buffers below the capacities")
    tail = (_ptr(out["g2l"], torch.int32), _ptr(out["l2g"], torch.int32), _ptr(out["rowptr"], torch.int32),
            _ptr(out["colidx"], torch.int32), _ptr(out["inv_deg"], torch.float32), C.c_int64(cap), C.c_int64(cap_nnz),
            _ptr(out["sizes"], torch.int64), _ptr(out["ws"]), C.c_size_t(out["ws"].numel()), _stream(stream))
    head = (C.c_int64(n), _ptr(rowptr, torch.int64, "rowptr"), _ptr(colidx, torch.int32, "colidx"))
    if rule is None:
        _check(L.tma_induced_subgraph_async(*head, _ptr(part, torch.int32, "part"), C.c_int32(p), *tail))
    else:
        _check(L.tma_random_subgraph_async(*head, C.c_int32(int(rule[0])), C.c_uint64(int(rule[1]) & ((1 << 64) - 1)),
                                           C.c_int32(p), *tail))
    return out


def tma_random_subgraph_async(rowptr, colidx, K: int, seed: int, p: int, cap_n_loc: int, cap_nnz_loc: int, out=None,
                              stream=None):
    """RandomTMA's assignment fused into the extraction: tma_induced_subgraph_async without a part array."""
    return tma_induced_subgraph_async(rowptr, colidx, None, p, cap_n_loc, cap_nnz_loc, out=out, stream=stream,
                                      rule=(K, seed))


def tma_mean_aggregate(rowptr, colidx, inv_deg, H, out=None, stream=None):
    n, F, ldh = _rows_ld(H, "H")
    if rowptr.numel() != n + 1 or inv_deg.numel() != n:
        raise TmaError("tma_mean_aggregate: graph and feature row counts differ")
    if out is None:
        out = torch.empty((n, F), dtype=H.dtype, device=H.device)
    _, Fo, ldm = _rows_ld(out, "M_out")
    if out.shape[0] != n or Fo != F or out.dtype != H.dtype:
        raise TmaError("tma_mean_aggregate: M_out shape/dtype mismatch")
    _check(lib().tma_mean_aggregate(C.c_int64(n), _ptr(rowptr, torch.int32), _ptr(colidx, torch.int32),
                                    _ptr(inv_deg, torch.float32), C.c_void_p(H.data_ptr()), C.c_int64(ldh),
                                    C.c_int32(F), C.c_int32(_feat_dtype(H)), C.c_void_p(out.data_ptr()),
                                    C.c_int64(ldm), _stream(stream)))
    return out


def tma_sage_layer_aggregates_first(F_in: int, F_out: int, dtype: int) -> bool:
    """True if the layer computes M = Abar H first (M_out holds it); False if it transforms first."""
    return bool(lib().tma_sage_layer_aggregates_first(C.c_int32(F_in), C.c_int32(F_out), C.c_int32(dtype)))


def tma_sage_weights_bf16_bytes(F_in: int, F_out: int) -> int:
    return int(lib().tma_sage_weights_bf16_bytes(C.c_int32(F_in), C.c_int32(F_out)))


def tma_sage_prepare_weights_bf16(W_self, W_neigh, out=None, stream=None):
    """The layer's weights narrowed to bf16 with the output feature as the row ([F_out, 2 F_in], int16 bits), for
    tma_sage_layer_fwd(..., Wt=...); to be called again whenever the weights have changed."""
    F_in, F_out = W_self.shape
    if tuple(W_neigh.shape) != (F_in, F_out):
        raise TmaError("tma_sage_prepare_weights_bf16: weight shapes differ")
    if out is None:
        out = torch.empty(tma_sage_weights_bf16_bytes(F_in, F_out) // 2, dtype=torch.int16, device=W_self.device)
    if out.numel() * out.element_size() < 2 * F_in * F_out * 2:
        raise TmaError("tma_sage_prepare_weights_bf16: out too small")
    _check(lib().tma_sage_prepare_weights_bf16(_ptr(W_self, torch.float32, "W_self"), _ptr(W_neigh, torch.float32, "W_neigh"),
                                               C.c_int32(F_in), C.c_int32(F_out), _ptr(out), _stream(stream)))
    return out


def tma_sage_layer_fwd(rowptr, colidx, inv_deg, H, W_self, W_neigh, bias, act: int, M_out=None, Hnext_out=None,
                       stream=None, Wt=None):
    """Returns (M, Hnext).  Wt: the weights as tma_sage_prepare_weights_bf16 leaves them (bf16 storage only; the
    call then goes through tma_sage_layer_fwd_prepared and returns the same bits)."""
    n, F_in, ldh = _rows_ld(H, "H")
    F_out = W_self.shape[1]
    if tuple(W_self.shape) != (F_in, F_out) or tuple(W_neigh.shape) != (F_in, F_out) or bias.numel() != F_out:
        raise TmaError("tma_sage_layer_fwd: weight shapes do not match H")
    if rowptr.numel() != n + 1 or inv_deg.numel() != n:
        raise TmaError("tma_sage_layer_fwd: graph and feature row counts differ")
    if M_out is None:
        M_out = _padded(n, F_in, H.dtype, H.device)
    if Hnext_out is None:
        Hnext_out = _padded(n, F_out, H.dtype, H.device)
    if tuple(M_out.shape) != (n, F_in) or tuple(Hnext_out.shape) != (n, F_out) or M_out.dtype != H.dtype:
        raise TmaError("tma_sage_layer_fwd: output shapes")
    _, _, ld_next = _rows_ld(Hnext_out, "Hnext_out")
    _, _, ldm = _rows_ld(M_out, "M_out")
    args = (C.c_int64(n), _ptr(rowptr, torch.int32), _ptr(colidx, torch.int32), _ptr(inv_deg, torch.float32),
            C.c_void_p(H.data_ptr()), C.c_int64(ldh), C.c_int32(F_in), _ptr(W_self, torch.float32, "W_self"),
            _ptr(W_neigh, torch.float32, "W_neigh"), _ptr(bias, torch.float32, "bias"), C.c_int32(F_out),
            C.c_int32(act), C.c_int32(_feat_dtype(H)), C.c_void_p(M_out.data_ptr()), C.c_int64(ldm),
            C.c_void_p(Hnext_out.data_ptr()), C.c_int64(ld_next))
    if Wt is not None:
        if Wt.numel() * Wt.element_size() < 2 * F_in * F_out * 2:
            raise TmaError("tma_sage_layer_fwd: Wt too small for these widths")
        _check(lib().tma_sage_layer_fwd_prepared(*args, _ptr(Wt), _stream(stream)))
    else:
        _check(lib().tma_sage_layer_fwd(*args, _stream(stream)))
    return M_out, Hnext_out


def tma_sage_layer_bwd_workspace_bytes(n: int, F_in: int, F_out: int, dtype: int, need_dH: bool) -> int:
    return int(lib().tma_sage_layer_bwd_workspace_bytes(C.c_int64(n), C.c_int32(F_in), C.c_int32(F_out),
                                                        C.c_int32(dtype), C.c_int32(1 if need_dH else 0)))


def tma_sage_layer_bwd(rowptr_T, colidx_T, inv_deg, H, M, Hnext, dHnext, W_self, W_neigh, act: int,
                       dW_self=None, dW_neigh=None, dbias=None, dH_out=None, need_dH=True, ws=None, stream=None):
    """Returns (dW_self, dW_neigh, dbias, dH or None)."""
    n, F_in, ldh = _rows_ld(H, "H")
    F_out = W_self.shape[1]
    dev = H.device
    if tuple(M.shape) != (n, F_in) or tuple(dHnext.shape) != (n, F_out) or M.dtype != H.dtype:
        raise TmaError("tma_sage_layer_bwd: M / dHnext shapes")
    _, _, ldm = _rows_ld(M, "M")
    if act == TMA_ACT_RELU and (Hnext is None or tuple(Hnext.shape) != (n, F_out)):
        raise TmaError("tma_sage_layer_bwd: Hnext is required with ReLU")
    if need_dH and (rowptr_T.numel() != n + 1 or inv_deg.numel() != n):
        raise TmaError("tma_sage_layer_bwd: graph and feature row counts differ")
    if dW_self is None:
        dW_self = torch.empty((F_in, F_out), dtype=torch.float32, device=dev)
    if dW_neigh is None:
        dW_neigh = torch.empty((F_in, F_out), dtype=torch.float32, device=dev)
    if dbias is None:
        dbias = torch.empty(F_out, dtype=torch.float32, device=dev)
    if need_dH and dH_out is None:
        dH_out = torch.empty((max(n, 1), ldh), dtype=H.dtype, device=dev)[:n, :F_in]
    if not need_dH:
        dH_out = None
    if dH_out is not None:
        if tuple(dH_out.shape) != (n, F_in) or _rows_ld(dH_out, "dH_out")[2] != ldh:
            raise TmaError("tma_sage_layer_bwd: dH_out must have the shape and leading dimension of H")
    _, _, ld_next = _rows_ld(dHnext, "dHnext")
    if act == TMA_ACT_RELU:
        _same_ld(Hnext, dHnext, "tma_sage_layer_bwd: Hnext / dHnext")
    dt = _feat_dtype(H)
    need = tma_sage_layer_bwd_workspace_bytes(n, F_in, F_out, dt, need_dH)
    if ws is None:
        ws = _workspace(need, dev, stream)
    _check(lib().tma_sage_layer_bwd(
        C.c_int64(n), _ptr(rowptr_T, torch.int32), _ptr(colidx_T, torch.int32), _ptr(inv_deg, torch.float32),
        C.c_void_p(H.data_ptr()), C.c_int64(ldh), C.c_void_p(M.data_ptr()), C.c_int64(ldm),
        C.c_void_p(Hnext.data_ptr() if Hnext is not None else 0), C.c_void_p(dHnext.data_ptr()), C.c_int64(ld_next),
        _ptr(W_self, torch.float32), _ptr(W_neigh, torch.float32),
        C.c_int32(F_in), C.c_int32(F_out), C.c_int32(act), C.c_int32(dt),
        _ptr(dW_self, torch.float32, "dW_self"), _ptr(dW_neigh, torch.float32, "dW_neigh"),
        _ptr(dbias, torch.float32, "dbias"), C.c_void_p(dH_out.data_ptr() if dH_out is not None else 0), _ptr(ws),
        C.c_size_t(ws.numel()), _stream(stream)))
    return dW_self, dW_neigh, dbias, dH_out


# --------------------------------------------------------------------------- other encoders (Sec. 4.1)
def tma_dense_fwd(X, W, bias, act: int, Y_out=None, stream=None):
    """Y = act(X W + b); bias may be None."""
    n, F_in, ldx = _rows_ld(X, "X")
    F_out = W.shape[1]
    if tuple(W.shape) != (F_in, F_out) or (bias is not None and bias.numel() != F_out):
        raise TmaError("tma_dense_fwd: weight shapes do not match X")
    if Y_out is None:
        Y_out = _padded(n, F_out, X.dtype, X.device)
    if tuple(Y_out.shape) != (n, F_out) or Y_out.dtype != X.dtype:
        raise TmaError("tma_dense_fwd: output shape/dtype")
    _, _, ldy = _rows_ld(Y_out, "Y_out")
    _check(lib().tma_dense_fwd(
        C.c_int64(n), C.c_void_p(X.data_ptr()), C.c_int64(ldx), C.c_int32(F_in), _ptr(W, torch.float32, "W"),
        _ptr(bias, torch.float32, "bias"), C.c_int32(F_out), C.c_int32(act), C.c_int32(_feat_dtype(X)),
        C.c_void_p(Y_out.data_ptr()), C.c_int64(ldy), _stream(stream)))
    return Y_out


def tma_dense_bwd_workspace_bytes(n: int, F_in: int, F_out: int) -> int:
    return int(lib().tma_dense_bwd_workspace_bytes(C.c_int64(n), C.c_int32(F_in), C.c_int32(F_out)))


def tma_dense_bwd(X, Y, dY, W, act: int, dW=None, dbias=None, dX_out=None, need_dbias=True, need_dX=True, ws=None,
                  stream=None):
    """Returns (dW, dbias or None, dX or None)."""
    n, F_in, ldx = _rows_ld(X, "X")
    F_out = W.shape[1]
    dev = X.device
    if tuple(dY.shape) != (n, F_out) or dY.dtype != X.dtype:
        raise TmaError("tma_dense_bwd: dY shape/dtype")
    if act == TMA_ACT_RELU and (Y is None or tuple(Y.shape) != (n, F_out)):
        raise TmaError("tma_dense_bwd: Y is required with ReLU")
    if dW is None:
        dW = torch.empty((F_in, F_out), dtype=torch.float32, device=dev)
    if need_dbias and dbias is None:
        dbias = torch.empty(F_out, dtype=torch.float32, device=dev)
    if not need_dbias:
        dbias = None
    if need_dX and dX_out is None:
        dX_out = _padded(n, F_in, X.dtype, dev)
    if not need_dX:
        dX_out = None
    ld_dx = _rows_ld(dX_out, "dX_out")[2] if dX_out is not None else F_in
    if dX_out is not None and tuple(dX_out.shape) != (n, F_in):
        raise TmaError("tma_dense_bwd: dX_out shape")
    _, _, ldy = _rows_ld(dY, "dY")
    if act == TMA_ACT_RELU:
        _same_ld(Y, dY, "tma_dense_bwd: Y / dY")
    if ws is None:
        ws = _workspace(tma_dense_bwd_workspace_bytes(n, F_in, F_out), dev, stream)
    _check(lib().tma_dense_bwd(
        C.c_int64(n), C.c_void_p(X.data_ptr()), C.c_int64(ldx), C.c_void_p(Y.data_ptr() if Y is not None else 0),
        C.c_void_p(dY.data_ptr()), C.c_int64(ldy), _ptr(W, torch.float32, "W"), C.c_int32(F_in), C.c_int32(F_out),
        C.c_int32(act), C.c_int32(_feat_dtype(X)), _ptr(dW, torch.float32, "dW"), _ptr(dbias, torch.float32, "dbias"),
        C.c_void_p(dX_out.data_ptr() if dX_out is not None else 0), C.c_int64(ld_dx), _ptr(ws),
        C.c_size_t(ws.numel()), _stream(stream)))
    return dW, dbias, dX_out


def tma_gcn_norm(rowptr, out=None, stream=None):
    """s_v = (d_v + 1)^-1/2 from the local rowptr (int32 [n+1])."""
    n = rowptr.numel() - 1
    if out is None:
        out = torch.empty(max(n, 0), dtype=torch.float32, device=rowptr.device)
    if out.numel() != n:
        raise TmaError("tma_gcn_norm: out must have n entries")
    _check(lib().tma_gcn_norm(C.c_int64(n), _ptr(rowptr, torch.int32, "rowptr"), _ptr(out, torch.float32, "out"),
                              _stream(stream)))
    return out


def tma_gcn_layer_aggregates_first(F_in: int, F_out: int, dtype: int) -> bool:
    return bool(lib().tma_gcn_layer_aggregates_first(C.c_int32(F_in), C.c_int32(F_out), C.c_int32(dtype)))


def tma_gcn_layer_fwd(rowptr, colidx, s_norm, H, W, bias, act: int, M_out=None, Hnext_out=None, stream=None):
    """Hnext = act(Ahat H W + b).  Returns (M, Hnext); M is Ahat H when the layer aggregates first."""
    n, F_in, ldh = _rows_ld(H, "H")
    F_out = W.shape[1]
    if tuple(W.shape) != (F_in, F_out) or bias.numel() != F_out:
        raise TmaError("tma_gcn_layer_fwd: weight shapes do not match H")
    if rowptr.numel() != n + 1 or s_norm.numel() != n:
        raise TmaError("tma_gcn_layer_fwd: graph and feature row counts differ")
    if M_out is None:
        M_out = torch.empty((n, F_in), dtype=H.dtype, device=H.device)
    if Hnext_out is None:
        Hnext_out = _padded(n, F_out, H.dtype, H.device)
    if tuple(M_out.shape) != (n, F_in) or tuple(Hnext_out.shape) != (n, F_out) or Hnext_out.dtype != H.dtype:
        raise TmaError("tma_gcn_layer_fwd: output shape/dtype")
    _, _, ld_next = _rows_ld(Hnext_out, "Hnext_out")
    _check(lib().tma_gcn_layer_fwd(
        C.c_int64(n), _ptr(rowptr, torch.int32), _ptr(colidx, torch.int32), _ptr(s_norm, torch.float32, "s_norm"),
        C.c_void_p(H.data_ptr()), C.c_int64(ldh), C.c_int32(F_in), _ptr(W, torch.float32, "W"),
        _ptr(bias, torch.float32, "bias"), C.c_int32(F_out), C.c_int32(act), C.c_int32(_feat_dtype(H)),
        _ptr(M_out, H.dtype, "M_out"), C.c_void_p(Hnext_out.data_ptr()), C.c_int64(ld_next), _stream(stream)))
    return M_out, Hnext_out


def tma_gcn_layer_bwd_workspace_bytes(n: int, F_in: int, F_out: int, dtype: int, need_dH: bool) -> int:
    return int(lib().tma_gcn_layer_bwd_workspace_bytes(C.c_int64(n), C.c_int32(F_in), C.c_int32(F_out),
                                                       C.c_int32(dtype), C.c_int32(1 if need_dH else 0)))


def tma_gcn_layer_bwd(rowptr_T, colidx_T, s_norm, H, M, Hnext, dHnext, W, act: int, dW=None, dbias=None, dH_out=None,
                      need_dH=True, ws=None, stream=None):
    """Returns (dW, dbias, dH or None).  M: what the forward left in M_out."""
    n, F_in, ldh = _rows_ld(H, "H")
    F_out = W.shape[1]
    dev = H.device
    if tuple(dHnext.shape) != (n, F_out) or dHnext.dtype != H.dtype or tuple(M.shape) != (n, F_in):
        raise TmaError("tma_gcn_layer_bwd: M / dHnext shape or dtype")
    if act == TMA_ACT_RELU and (Hnext is None or tuple(Hnext.shape) != (n, F_out)):
        raise TmaError("tma_gcn_layer_bwd: Hnext is required with ReLU")
    if rowptr_T.numel() != n + 1 or s_norm.numel() != n:
        raise TmaError("tma_gcn_layer_bwd: graph and feature row counts differ")
    if dW is None:
        dW = torch.empty((F_in, F_out), dtype=torch.float32, device=dev)
    if dbias is None:
        dbias = torch.empty(F_out, dtype=torch.float32, device=dev)
    if need_dH and dH_out is None:
        dH_out = torch.empty((max(n, 1), ldh), dtype=H.dtype, device=dev)[:n, :F_in]
    if not need_dH:
        dH_out = None
    if dH_out is not None:
        if tuple(dH_out.shape) != (n, F_in) or _rows_ld(dH_out, "dH_out")[2] != ldh:
            raise TmaError("tma_gcn_layer_bwd: dH_out must have the shape and leading dimension of H")
    _, _, ld_next = _rows_ld(dHnext, "dHnext")
    if act == TMA_ACT_RELU:
        _same_ld(Hnext, dHnext, "tma_gcn_layer_bwd: Hnext / dHnext")
    dt = _feat_dtype(H)
    if ws is None:
        ws = _workspace(tma_gcn_layer_bwd_workspace_bytes(n, F_in, F_out, dt, need_dH), dev, stream)
    _check(lib().tma_gcn_layer_bwd(
        C.c_int64(n), _ptr(rowptr_T, torch.int32), _ptr(colidx_T, torch.int32), _ptr(s_norm, torch.float32, "s_norm"),
        C.c_void_p(H.data_ptr()), C.c_int64(ldh), _ptr(M, H.dtype, "M"),
        C.c_void_p(Hnext.data_ptr() if Hnext is not None else 0),
        C.c_void_p(dHnext.data_ptr()), C.c_int64(ld_next), _ptr(W, torch.float32, "W"), C.c_int32(F_in),
        C.c_int32(F_out), C.c_int32(act), C.c_int32(dt), _ptr(dW, torch.float32, "dW"),
        _ptr(dbias, torch.float32, "dbias"), C.c_void_p(dH_out.data_ptr() if dH_out is not None else 0), _ptr(ws),
        C.c_size_t(ws.numel()), _stream(stream)))
    return dW, dbias, dH_out


# --------------------------------------------------------------------------- link-prediction head (Sec. 4.1, App.)
def tma_edge_batch(rowptr, colidx, nnz: int, seed: int, first_counter: int, B: int, u_out=None, v_out=None,
                   vneg_out=None, stream=None):
    """B positive edges (u, v) of the local CSR and one negative tail v' each; int32 device tensors."""
    n = rowptr.numel() - 1
    dev = rowptr.device
    if colidx.numel() < nnz:
        raise TmaError("tma_edge_batch: colidx holds fewer than nnz entries")
    outs = []
    for t in (u_out, v_out, vneg_out):
        if t is None:
            t = torch.empty(B, dtype=torch.int32, device=dev)
        if t.numel() != B:
            raise TmaError("tma_edge_batch: outputs need B entries")
        outs.append(t)
    _check(lib().tma_edge_batch(
        C.c_int64(n), C.c_int64(nnz), _ptr(rowptr, torch.int32, "rowptr"), _ptr(colidx, torch.int32, "colidx"),
        C.c_uint64(seed), C.c_uint64(first_counter), C.c_int64(B), _ptr(outs[0], torch.int32), _ptr(outs[1], torch.int32),
        _ptr(outs[2], torch.int32), _stream(stream)))
    return tuple(outs)


def tma_pair_product_fwd(R, u, v, vneg, E0_out=None, stream=None):
    """E0 [2B, F]: r_u (.) r_v for the positives, then r_u (.) r_v' for the negatives."""
    n, F, ldr = _rows_ld(R, "R")
    Bn = u.numel()
    if v.numel() != Bn or vneg.numel() != Bn:
        raise TmaError("tma_pair_product_fwd: u, v, vneg need the same length")
    if E0_out is None:
        E0_out = _padded(2 * Bn, F, R.dtype, R.device)
    if tuple(E0_out.shape) != (2 * Bn, F) or E0_out.dtype != R.dtype:
        raise TmaError("tma_pair_product_fwd: E0_out shape/dtype")
    _, _, lde = _rows_ld(E0_out, "E0_out")
    _check(lib().tma_pair_product_fwd(
        C.c_int64(Bn), C.c_int32(F), C.c_void_p(R.data_ptr()), C.c_int64(ldr), C.c_int32(_feat_dtype(R)),
        _ptr(u, torch.int32, "u"), _ptr(v, torch.int32, "v"), _ptr(vneg, torch.int32, "vneg"),
        C.c_void_p(E0_out.data_ptr()), C.c_int64(lde), _stream(stream)))
    return E0_out


def tma_pair_product_bwd_workspace_bytes(n: int, Bn: int, F: int, dtype: int) -> int:
    return int(lib().tma_pair_product_bwd_workspace_bytes(C.c_int64(n), C.c_int64(Bn), C.c_int32(F), C.c_int32(dtype)))


def tma_pair_product_bwd(R, u, v, vneg, dE0, dR_out=None, ws=None, stream=None):
    """dR [n, F]: gradient of the pair products w.r.t. the embeddings (zero rows outside the batch)."""
    n, F, ldr = _rows_ld(R, "R")
    Bn = u.numel()
    if tuple(dE0.shape) != (2 * Bn, F) or dE0.dtype != R.dtype:
        raise TmaError("tma_pair_product_bwd: dE0 shape/dtype")
    if dR_out is None:
        dR_out = _padded(n, F, R.dtype, R.device)
    if tuple(dR_out.shape) != (n, F) or dR_out.dtype != R.dtype:
        raise TmaError("tma_pair_product_bwd: dR_out shape/dtype")
    _, _, lde = _rows_ld(dE0, "dE0")
    _, _, ld_dr = _rows_ld(dR_out, "dR_out")
    dt = _feat_dtype(R)
    if ws is None:
        ws = _workspace(tma_pair_product_bwd_workspace_bytes(n, Bn, F, dt), R.device, stream)
    _check(lib().tma_pair_product_bwd(
        C.c_int64(n), C.c_int64(Bn), C.c_int32(F), C.c_void_p(R.data_ptr()), C.c_int64(ldr), C.c_int32(dt),
        _ptr(u, torch.int32, "u"), _ptr(v, torch.int32, "v"), _ptr(vneg, torch.int32, "vneg"),
        C.c_void_p(dE0.data_ptr()), C.c_int64(lde), C.c_void_p(dR_out.data_ptr()), C.c_int64(ld_dr), _ptr(ws),
        C.c_size_t(ws.numel()), _stream(stream)))
    return dR_out


def tma_prelu_fwd(Z, slope, out=None, stream=None):
    """Y = PReLU_slope(Z); slope is a 1-element fp32 device tensor."""
    n, F, ldz = _rows_ld(Z, "Z")
    if out is None:
        out = _padded(n, F, Z.dtype, Z.device)
    if tuple(out.shape) != (n, F) or out.dtype != Z.dtype or slope.numel() != 1:
        raise TmaError("tma_prelu_fwd: out shape/dtype or slope")
    _, _, ldy = _rows_ld(out, "out")
    _check(lib().tma_prelu_fwd(C.c_int64(n), C.c_int32(F), C.c_void_p(Z.data_ptr()), C.c_int64(ldz),
                               _ptr(slope, torch.float32, "slope"), C.c_int32(_feat_dtype(Z)),
                               C.c_void_p(out.data_ptr()), C.c_int64(ldy), _stream(stream)))
    return out


def tma_prelu_bwd_workspace_bytes() -> int:
    return int(lib().tma_prelu_bwd_workspace_bytes())


def tma_prelu_bwd(Z, dY, slope, dZ_out=None, dslope=None, ws=None, stream=None):
    """Returns (dZ, dslope).  dZ_out may be dY itself."""
    n, F, ldz = _rows_ld(Z, "Z")
    if tuple(dY.shape) != (n, F) or dY.dtype != Z.dtype or slope.numel() != 1:
        raise TmaError("tma_prelu_bwd: dY shape/dtype or slope")
    if dZ_out is None:
        dZ_out = _padded(n, F, Z.dtype, Z.device)
    if dslope is None:
        dslope = torch.empty(1, dtype=torch.float32, device=Z.device)
    if tuple(dZ_out.shape) != (n, F) or dZ_out.dtype != Z.dtype or dslope.numel() != 1:
        raise TmaError("tma_prelu_bwd: output shape/dtype")
    _, _, ldd = _rows_ld(dY, "dY")
    _, _, ld_dz = _rows_ld(dZ_out, "dZ_out")
    if ws is None:
        ws = _workspace(tma_prelu_bwd_workspace_bytes(), Z.device, stream)
    _check(lib().tma_prelu_bwd(
        C.c_int64(n), C.c_int32(F), C.c_void_p(Z.data_ptr()), C.c_int64(ldz), C.c_void_p(dY.data_ptr()), C.c_int64(ldd),
        _ptr(slope, torch.float32, "slope"), C.c_int32(_feat_dtype(Z)), C.c_void_p(dZ_out.data_ptr()), C.c_int64(ld_dz),
        _ptr(dslope, torch.float32, "dslope"), _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return dZ_out, dslope


def tma_bce_logits_workspace_bytes() -> int:
    return int(lib().tma_bce_logits_workspace_bytes())


def tma_bce_logits(z, n_pos: int, loss_out=None, dz_out=None, need_grad=True, ws=None, stream=None):
    """Mean binary cross-entropy of the logits z [count, 1] (first n_pos positives).  Returns (loss, dz or None)."""
    count, one, ldz = _rows_ld(z, "z")
    if one != 1:
        raise TmaError("tma_bce_logits: z must have one column")
    if loss_out is None:
        loss_out = torch.empty(1, dtype=torch.float32, device=z.device)
    if need_grad and dz_out is None:
        dz_out = _padded(count, 1, z.dtype, z.device)
    if not need_grad:
        dz_out = None
    ld_dz = _rows_ld(dz_out, "dz_out")[2] if dz_out is not None else 1
    if dz_out is not None and (tuple(dz_out.shape) != (count, 1) or dz_out.dtype != z.dtype):
        raise TmaError("tma_bce_logits: dz_out shape/dtype")
    if ws is None:
        ws = _workspace(tma_bce_logits_workspace_bytes(), z.device, stream)
    _check(lib().tma_bce_logits(
        C.c_int64(count), C.c_int64(n_pos), C.c_void_p(z.data_ptr()), C.c_int64(ldz), C.c_int32(_feat_dtype(z)),
        _ptr(loss_out, torch.float32, "loss_out"), C.c_void_p(dz_out.data_ptr() if dz_out is not None else 0),
        C.c_int64(ld_dz), _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return loss_out, dz_out


# --------------------------------------------------------------------------- sampled message-flow graphs (Sec. 4.1)
def tma_neighbor_sample_workspace_bytes(n_dst: int) -> int:
    return int(lib().tma_neighbor_sample_workspace_bytes(C.c_int64(n_dst)))


def tma_neighbor_sample(dst, n_dst: int, nnz: int, rowptr, colidx, fanout: int, seed: int, blk_rowptr_out=None,
                        blk_col_out=None, blk_row_out=None, ws=None, stream=None):
    """Block over the first n_dst entries of dst: returns (blk_rowptr [n_dst+1], blk_col, blk_row); the number of
    kept entries stays on the device in blk_rowptr[n_dst]."""
    dev = rowptr.device
    cap = max(min(n_dst * fanout, nnz), 1)
    if blk_rowptr_out is None:
        blk_rowptr_out = torch.empty(n_dst + 1, dtype=torch.int32, device=dev)
    if blk_col_out is None:
        blk_col_out = torch.empty(cap, dtype=torch.int32, device=dev)
    if blk_row_out is None:
        blk_row_out = torch.empty(cap, dtype=torch.int32, device=dev)
    if blk_rowptr_out.numel() < n_dst + 1 or dst.numel() < n_dst or colidx.numel() < nnz:
        raise TmaError("tma_neighbor_sample: dst / blk_rowptr_out / colidx too short")
    if ws is None:
        ws = _workspace(tma_neighbor_sample_workspace_bytes(n_dst), dev, stream)
    _check(lib().tma_neighbor_sample(
        C.c_int64(n_dst), _ptr(dst, torch.int32, "dst"), C.c_int64(nnz), _ptr(rowptr, torch.int32, "rowptr"),
        _ptr(colidx, torch.int32, "colidx"), C.c_int32(fanout), C.c_uint64(seed), _ptr(blk_rowptr_out, torch.int32),
        _ptr(blk_col_out, torch.int32), _ptr(blk_row_out, torch.int32), C.c_int64(min(blk_col_out.numel(), blk_row_out.numel())),
        _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return blk_rowptr_out, blk_col_out, blk_row_out


def tma_mfg_relabel_workspace_bytes(n: int) -> int:
    return int(lib().tma_mfg_relabel_workspace_bytes(C.c_int64(n)))


def tma_mfg_relabel(n: int, dst, n_dst: int, cols, max_items: int, d_items=None, src_out=None, ws=None, stream=None):
    """cols[:count] becomes positions in the node list src = dst[:n_dst] + the other nodes of cols (ascending).
    d_items: 1-element int32 device tensor (view) with the count, or None for max_items.  Returns (src, n_src)."""
    dev = cols.device
    if src_out is None:
        src_out = torch.empty(max(min(n, n_dst + max_items), 1), dtype=torch.int32, device=dev)
    if ws is None:
        ws = _workspace(tma_mfg_relabel_workspace_bytes(n), dev, stream)
    n_src = C.c_int64(0)
    _check(lib().tma_mfg_relabel(
        C.c_int64(n), C.c_int64(n_dst), _ptr(dst, torch.int32, "dst") if n_dst > 0 else C.c_void_p(0), C.c_int64(max_items),
        C.c_void_p(d_items.data_ptr() if d_items is not None else 0), _ptr(cols, torch.int32, "cols"),
        _ptr(src_out, torch.int32, "src_out"), C.c_int64(src_out.numel()), C.byref(n_src), _ptr(ws), C.c_size_t(ws.numel()),
        _stream(stream)))
    return src_out, int(n_src.value)


def tma_neighbor_sample_dev(dst, cap_dst: int, d_n_dst, nnz: int, rowptr, colidx, fanout: int, seed: int,
                            blk_rowptr_out=None, blk_col_out=None, blk_row_out=None, ws=None, stream=None):
    """tma_neighbor_sample with the number of dst nodes in d_n_dst (1-element int32 device tensor or view); launches
    and buffers are those of cap_dst rows.  blk_rowptr[*d_n_dst .. cap_dst] all hold the number of kept entries."""
    dev = rowptr.device
    cap = max(min(cap_dst * fanout, nnz), 1)
    if blk_rowptr_out is None:
        blk_rowptr_out = torch.empty(cap_dst + 1, dtype=torch.int32, device=dev)
    if blk_col_out is None:
        blk_col_out = torch.empty(cap, dtype=torch.int32, device=dev)
    if blk_row_out is None:
        blk_row_out = torch.empty(cap, dtype=torch.int32, device=dev)
    if blk_rowptr_out.numel() < cap_dst + 1 or dst.numel() < cap_dst or colidx.numel() < nnz or d_n_dst.numel() < 1:
        raise TmaError("tma_neighbor_sample_dev: dst / blk_rowptr_out / colidx / d_n_dst too short")
    if ws is None:
        ws = _workspace(tma_neighbor_sample_workspace_bytes(cap_dst), dev, stream)
    _check(lib().tma_neighbor_sample_dev(
        C.c_int64(cap_dst), _ptr(d_n_dst, torch.int32, "d_n_dst"), _ptr(dst, torch.int32, "dst"), C.c_int64(nnz),
        _ptr(rowptr, torch.int32, "rowptr"), _ptr(colidx, torch.int32, "colidx"), C.c_int32(fanout), C.c_uint64(seed),
        _ptr(blk_rowptr_out, torch.int32), _ptr(blk_col_out, torch.int32), _ptr(blk_row_out, torch.int32),
        C.c_int64(min(blk_col_out.numel(), blk_row_out.numel())), _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return blk_rowptr_out, blk_col_out, blk_row_out


def tma_mfg_relabel_dev(n: int, dst, cap_dst: int, d_n_dst, cols, max_items: int, d_items=None, src_out=None,
                        n_src_out=None, ws=None, stream=None):
    """tma_mfg_relabel without the wait: the number of dst nodes is read from d_n_dst (None with cap_dst = 0) and the
    length of the node list is written to n_src_out (1-element int32 device tensors or views).  Returns
    (src, n_src_out)."""
    dev = cols.device
    if src_out is None:
        src_out = torch.empty(max(min(n, cap_dst + max_items), 1), dtype=torch.int32, device=dev)
    if n_src_out is None:
        n_src_out = torch.empty(1, dtype=torch.int32, device=dev)
    if ws is None:
        ws = _workspace(tma_mfg_relabel_workspace_bytes(n), dev, stream)
    _check(lib().tma_mfg_relabel_dev(
        C.c_int64(n), C.c_int64(cap_dst), _ptr(d_n_dst, torch.int32, "d_n_dst") if cap_dst > 0 else C.c_void_p(0),
        _ptr(dst, torch.int32, "dst") if cap_dst > 0 else C.c_void_p(0), C.c_int64(max_items),
        C.c_void_p(d_items.data_ptr() if d_items is not None else 0), _ptr(cols, torch.int32, "cols"),
        _ptr(src_out, torch.int32, "src_out"), C.c_int64(src_out.numel()), _ptr(n_src_out, torch.int32, "n_src_out"),
        _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return src_out, n_src_out


def tma_block_inv_deg(blk_rowptr, n_dst: int, out=None, stream=None):
    if out is None:
        out = torch.empty(max(n_dst, 1), dtype=torch.float32, device=blk_rowptr.device)
    _check(lib().tma_block_inv_deg(C.c_int64(n_dst), _ptr(blk_rowptr, torch.int32, "blk_rowptr"),
                                   _ptr(out, torch.float32, "out"), _stream(stream)))
    return out


def tma_sage_block_fwd(n_dst: int, n_src: int, blk_rowptr, blk_col, inv_deg, H, W_self, W_neigh, bias, act: int,
                       M_out, Hnext_out, stream=None):
    """Layer on a bipartite block; H, M_out, Hnext_out are buffers with at least n_src / n_dst / n_dst rows."""
    _, F_in, ldh = _rows_ld(H, "H")
    F_out = W_self.shape[1]
    if H.shape[0] < n_src or M_out.shape[0] < n_dst or Hnext_out.shape[0] < n_dst:
        raise TmaError("tma_sage_block_fwd: a buffer has too few rows")
    if tuple(W_self.shape) != (F_in, F_out) or tuple(W_neigh.shape) != (F_in, F_out) or bias.numel() != F_out:
        raise TmaError("tma_sage_block_fwd: weight shapes do not match H")
    if M_out.shape[1] != F_in or Hnext_out.shape[1] != F_out or not M_out.is_contiguous():
        raise TmaError("tma_sage_block_fwd: M_out must be a dense [rows, F_in] buffer, Hnext_out [rows, F_out]")
    _, _, ld_next = _rows_ld(Hnext_out, "Hnext_out")
    _check(lib().tma_sage_block_fwd(
        C.c_int64(n_dst), C.c_int64(n_src), _ptr(blk_rowptr, torch.int32), _ptr(blk_col, torch.int32),
        _ptr(inv_deg, torch.float32), C.c_void_p(H.data_ptr()), C.c_int64(ldh), C.c_int32(F_in),
        _ptr(W_self, torch.float32, "W_self"), _ptr(W_neigh, torch.float32, "W_neigh"), _ptr(bias, torch.float32, "bias"),
        C.c_int32(F_out), C.c_int32(act), C.c_int32(_feat_dtype(H)), C.c_void_p(M_out.data_ptr()),
        C.c_void_p(Hnext_out.data_ptr()), C.c_int64(ld_next), _stream(stream)))
    return M_out, Hnext_out


def tma_sage_block_bwd_workspace_bytes(n_dst: int, n_src: int, max_entries: int, F_in: int, F_out: int, dtype: int,
                                       need_dH: bool) -> int:
    return int(lib().tma_sage_block_bwd_workspace_bytes(C.c_int64(n_dst), C.c_int64(n_src), C.c_int64(max_entries),
                                                        C.c_int32(F_in), C.c_int32(F_out), C.c_int32(dtype),
                                                        C.c_int32(1 if need_dH else 0)))


def tma_sage_block_bwd(n_dst: int, n_src: int, max_entries: int, blk_rowptr, blk_col, blk_row, inv_deg, H, M, Hnext,
                       dHnext, W_self, W_neigh, act: int, dW_self, dW_neigh, dbias, dH_out=None, ws=None, stream=None):
    """Backward on a bipartite block; dH_out (buffer with the leading dimension of H, at least n_src rows) or None."""
    _, F_in, ldh = _rows_ld(H, "H")
    F_out = W_self.shape[1]
    _, _, ld_next = _rows_ld(dHnext, "dHnext")
    if act == TMA_ACT_RELU:
        _same_ld(Hnext, dHnext, "tma_sage_block_bwd: Hnext / dHnext")
    if dH_out is not None and (dH_out.shape[0] < n_src or _rows_ld(dH_out, "dH_out")[2] != ldh):
        raise TmaError("tma_sage_block_bwd: dH_out needs n_src rows and the leading dimension of H")
    dt = _feat_dtype(H)
    if ws is None:
        ws = _workspace(tma_sage_block_bwd_workspace_bytes(n_dst, n_src, max_entries, F_in, F_out, dt, dH_out is not None),
                        H.device, stream)
    _check(lib().tma_sage_block_bwd(
        C.c_int64(n_dst), C.c_int64(n_src), C.c_int64(max_entries), _ptr(blk_rowptr, torch.int32),
        _ptr(blk_col, torch.int32), _ptr(blk_row, torch.int32), _ptr(inv_deg, torch.float32), C.c_void_p(H.data_ptr()),
        C.c_int64(ldh), C.c_void_p(M.data_ptr()), C.c_void_p(Hnext.data_ptr() if Hnext is not None else 0),
        C.c_void_p(dHnext.data_ptr()), C.c_int64(ld_next), _ptr(W_self, torch.float32), _ptr(W_neigh, torch.float32),
        C.c_int32(F_in), C.c_int32(F_out), C.c_int32(act), C.c_int32(dt), _ptr(dW_self, torch.float32, "dW_self"),
        _ptr(dW_neigh, torch.float32, "dW_neigh"), _ptr(dbias, torch.float32, "dbias"),
        C.c_void_p(dH_out.data_ptr() if dH_out is not None else 0), _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return dH_out


def tma_gcn_block_norm(blk_rowptr, n_dst: int, out=None, stream=None):
    """c_v = 1 / (|S(v)| + 1) for the block's first n_dst rows."""
    if out is None:
        out = torch.empty(max(n_dst, 1), dtype=torch.float32, device=blk_rowptr.device)
    if out.numel() < n_dst or blk_rowptr.numel() < n_dst + 1:
        raise TmaError("tma_gcn_block_norm: a buffer has too few elements")
    _check(lib().tma_gcn_block_norm(C.c_int64(n_dst), _ptr(blk_rowptr, torch.int32), _ptr(out, torch.float32),
                                    _stream(stream)))
    return out


def tma_gcn_block_fwd(n_dst: int, n_src: int, blk_rowptr, blk_col, c_norm, H, W, bias, act: int, M_out, Hnext_out,
                      stream=None):
    """GCN layer on a bipartite block; H, M_out, Hnext_out are buffers with at least n_src / n_dst / n_dst rows."""
    _, F_in, ldh = _rows_ld(H, "H")
    F_out = W.shape[1]
    if H.shape[0] < n_src or M_out.shape[0] < n_dst or Hnext_out.shape[0] < n_dst:
        raise TmaError("tma_gcn_block_fwd: a buffer has too few rows")
    if tuple(W.shape) != (F_in, F_out) or bias.numel() != F_out:
        raise TmaError("tma_gcn_block_fwd: weight shapes do not match H")
    if M_out.shape[1] != F_in or Hnext_out.shape[1] != F_out or not M_out.is_contiguous():
        raise TmaError("tma_gcn_block_fwd: M_out must be a dense [rows, F_in] buffer, Hnext_out [rows, F_out]")
    _, _, ld_next = _rows_ld(Hnext_out, "Hnext_out")
    _check(lib().tma_gcn_block_fwd(
        C.c_int64(n_dst), C.c_int64(n_src), _ptr(blk_rowptr, torch.int32), _ptr(blk_col, torch.int32),
        _ptr(c_norm, torch.float32), C.c_void_p(H.data_ptr()), C.c_int64(ldh), C.c_int32(F_in),
        _ptr(W, torch.float32, "W"), _ptr(bias, torch.float32, "bias"), C.c_int32(F_out), C.c_int32(act),
        C.c_int32(_feat_dtype(H)), C.c_void_p(M_out.data_ptr()), C.c_void_p(Hnext_out.data_ptr()), C.c_int64(ld_next),
        _stream(stream)))
    return M_out, Hnext_out


def tma_gcn_block_bwd_workspace_bytes(n_dst: int, n_src: int, max_entries: int, F_in: int, F_out: int, dtype: int,
                                      need_dH: bool) -> int:
    return int(lib().tma_gcn_block_bwd_workspace_bytes(C.c_int64(n_dst), C.c_int64(n_src), C.c_int64(max_entries),
                                                       C.c_int32(F_in), C.c_int32(F_out), C.c_int32(dtype),
                                                       C.c_int32(1 if need_dH else 0)))


def tma_gcn_block_bwd(n_dst: int, n_src: int, max_entries: int, blk_rowptr, blk_col, blk_row, c_norm, M, Hnext, dHnext,
                      W, act: int, dW, dbias, dH_out=None, ws=None, stream=None):
    """Backward of the GCN layer on a bipartite block; dH_out (buffer with at least n_src rows of F_in) or None."""
    F_in, F_out = W.shape
    _, _, ld_next = _rows_ld(dHnext, "dHnext")
    if act == TMA_ACT_RELU:
        _same_ld(Hnext, dHnext, "tma_gcn_block_bwd: Hnext / dHnext")
    if M.shape[0] < n_dst or M.shape[1] != F_in or not M.is_contiguous():
        raise TmaError("tma_gcn_block_bwd: M must be the dense [rows, F_in] buffer of the forward pass")
    ldh = 0
    if dH_out is not None:
        rows, Fh, ldh = _rows_ld(dH_out, "dH_out")
        if rows < n_src or Fh != F_in or dH_out.dtype != M.dtype:
            raise TmaError("tma_gcn_block_bwd: dH_out needs n_src rows of F_in elements in the features' dtype")
    dt = _feat_dtype(M)
    if ws is None:
        ws = _workspace(tma_gcn_block_bwd_workspace_bytes(n_dst, n_src, max_entries, F_in, F_out, dt, dH_out is not None),
                        M.device, stream)
    _check(lib().tma_gcn_block_bwd(
        C.c_int64(n_dst), C.c_int64(n_src), C.c_int64(max_entries), _ptr(blk_rowptr, torch.int32),
        _ptr(blk_col, torch.int32), _ptr(blk_row, torch.int32), _ptr(c_norm, torch.float32), C.c_void_p(M.data_ptr()),
        C.c_void_p(Hnext.data_ptr() if Hnext is not None else 0), C.c_void_p(dHnext.data_ptr()), C.c_int64(ld_next),
        _ptr(W, torch.float32, "W"), C.c_int32(F_in), C.c_int32(F_out), C.c_int32(act), C.c_int32(dt),
        _ptr(dW, torch.float32, "dW"), _ptr(dbias, torch.float32, "dbias"),
        C.c_void_p(dH_out.data_ptr() if dH_out is not None else 0), C.c_int64(ldh), _ptr(ws), C.c_size_t(ws.numel()),
        _stream(stream)))
    return dH_out


def tma_loss_workspace_bytes(n: int, Cc: int) -> int:
    return int(lib().tma_loss_workspace_bytes(C.c_int64(n), C.c_int32(Cc)))


LN_EPS = 1e-5


def tma_layernorm_prelu_fwd(Z, gamma, beta, slope, eps: float = LN_EPS, out=None, stream=None):
    """H' = PReLU_slope(LayerNorm_{gamma,beta}(Z)); slope is a 1-element fp32 device tensor."""
    n, F, ldz = _rows_ld(Z, "Z")
    if gamma.numel() != F or beta.numel() != F or slope.numel() != 1:
        raise TmaError("tma_layernorm_prelu_fwd: gamma / beta need F entries, slope one")
    if out is None:
        out = _padded(n, F, Z.dtype, Z.device)
    if tuple(out.shape) != (n, F) or out.dtype != Z.dtype:
        raise TmaError("tma_layernorm_prelu_fwd: out shape/dtype mismatch")
    _, _, ldo = _rows_ld(out, "out")
    _check(lib().tma_layernorm_prelu_fwd(
        C.c_int64(n), C.c_int32(F), C.c_void_p(Z.data_ptr()), C.c_int64(ldz), _ptr(gamma, torch.float32, "gamma"),
        _ptr(beta, torch.float32, "beta"), _ptr(slope, torch.float32, "slope"), C.c_float(eps),
        C.c_int32(_feat_dtype(Z)), C.c_void_p(out.data_ptr()), C.c_int64(ldo), _stream(stream)))
    return out


def tma_layernorm_prelu_bwd_workspace_bytes(n: int, F: int) -> int:
    return lib().tma_layernorm_prelu_bwd_workspace_bytes(C.c_int64(n), C.c_int32(F))


def tma_layernorm_prelu_bwd(Z, dHnext, gamma, beta, slope, eps: float = LN_EPS, dZ_out=None, dgamma=None, dbeta=None,
                            dslope=None, ws=None, stream=None):
    """Returns (dZ, dgamma, dbeta, dslope).  dZ_out may be dHnext itself (overwritten in place)."""
    n, F, ldz = _rows_ld(Z, "Z")
    dev = Z.device
    if tuple(dHnext.shape) != (n, F) or dHnext.dtype != Z.dtype:
        raise TmaError("tma_layernorm_prelu_bwd: dHnext shape/dtype mismatch")
    if gamma.numel() != F or beta.numel() != F or slope.numel() != 1:
        raise TmaError("tma_layernorm_prelu_bwd: gamma / beta need F entries, slope one")
    if dZ_out is None:
        dZ_out = _padded(n, F, Z.dtype, dev)
    if tuple(dZ_out.shape) != (n, F) or dZ_out.dtype != Z.dtype:
        raise TmaError("tma_layernorm_prelu_bwd: dZ_out shape/dtype mismatch")
    dgamma = torch.empty(F, dtype=torch.float32, device=dev) if dgamma is None else dgamma
    dbeta = torch.empty(F, dtype=torch.float32, device=dev) if dbeta is None else dbeta
    dslope = torch.empty(1, dtype=torch.float32, device=dev) if dslope is None else dslope
    if dgamma.numel() != F or dbeta.numel() != F or dslope.numel() != 1:
        raise TmaError("tma_layernorm_prelu_bwd: gradient output sizes")
    if ws is None:
        ws = _workspace(tma_layernorm_prelu_bwd_workspace_bytes(n, F), dev, stream)
    _, _, ldd = _rows_ld(dHnext, "dHnext")
    _, _, ldo = _rows_ld(dZ_out, "dZ_out")
    _check(lib().tma_layernorm_prelu_bwd(
        C.c_int64(n), C.c_int32(F), C.c_void_p(Z.data_ptr()), C.c_int64(ldz), C.c_void_p(dHnext.data_ptr()),
        C.c_int64(ldd), _ptr(gamma, torch.float32, "gamma"), _ptr(beta, torch.float32, "beta"),
        _ptr(slope, torch.float32, "slope"), C.c_float(eps), C.c_int32(_feat_dtype(Z)),
        C.c_void_p(dZ_out.data_ptr()), C.c_int64(ldo), _ptr(dgamma, torch.float32), _ptr(dbeta, torch.float32),
        _ptr(dslope, torch.float32), _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return dZ_out, dgamma, dbeta, dslope


def tma_layernorm_prelu_bwd_static_max_f() -> int:
    return int(lib().tma_layernorm_prelu_bwd_static_max_f())


def tma_layernorm_prelu_bwd_static(Z, dHnext, gamma, beta, slope, dZ_out, dgamma, dbeta, dslope, eps: float = LN_EPS,
                                   stream=None):
    """The backward pass through the library's own scratch array: no workspace, and every output is the caller's
    (this wrapper allocates nothing either).  Returns (dZ_out, dgamma, dbeta, dslope)."""
    n, F, ldz = _rows_ld(Z, "Z")
    if tuple(dHnext.shape) != (n, F) or dHnext.dtype != Z.dtype:
        raise TmaError("tma_layernorm_prelu_bwd_static: dHnext shape/dtype mismatch")
    if tuple(dZ_out.shape) != (n, F) or dZ_out.dtype != Z.dtype:
        raise TmaError("tma_layernorm_prelu_bwd_static: dZ_out shape/dtype mismatch")
    if gamma.numel() != F or beta.numel() != F or slope.numel() != 1:
        raise TmaError("tma_layernorm_prelu_bwd_static: gamma / beta need F entries, slope one")
    if dgamma.numel() != F or dbeta.numel() != F or dslope.numel() != 1:
        raise TmaError("tma_layernorm_prelu_bwd_static: gradient output sizes")
    _, _, ldd = _rows_ld(dHnext, "dHnext")
    _, _, ldo = _rows_ld(dZ_out, "dZ_out")
    _check(lib().tma_layernorm_prelu_bwd_static(
        C.c_int64(n), C.c_int32(F), C.c_void_p(Z.data_ptr()), C.c_int64(ldz), C.c_void_p(dHnext.data_ptr()),
        C.c_int64(ldd), _ptr(gamma, torch.float32, "gamma"), _ptr(beta, torch.float32, "beta"),
        _ptr(slope, torch.float32, "slope"), C.c_float(eps), C.c_int32(_feat_dtype(Z)),
        C.c_void_p(dZ_out.data_ptr()), C.c_int64(ldo), _ptr(dgamma, torch.float32), _ptr(dbeta, torch.float32),
        _ptr(dslope, torch.float32), _stream(stream)))
    return dZ_out, dgamma, dbeta, dslope


def tma_softmax_ce(logits, labels, loss_out=None, dlogits_out=None, need_grad=True, ws=None, stream=None):
    """Returns (loss [1] fp32 device tensor, dlogits or None)."""
    n, Cc, ldz = _rows_ld(logits, "logits")
    dev = logits.device
    if labels.numel() != n:
        raise TmaError("tma_softmax_ce: labels must have one entry per row")
    if loss_out is None:
        loss_out = torch.empty(1, dtype=torch.float32, device=dev)
    if need_grad and dlogits_out is None:
        dlogits_out = torch.empty((max(n, 1), ldz), dtype=logits.dtype, device=dev)[:n, :Cc]
    if need_grad and (tuple(dlogits_out.shape) != (n, Cc) or _rows_ld(dlogits_out, "dlogits_out")[2] != ldz):
        raise TmaError("tma_softmax_ce: dlogits_out must have the shape and leading dimension of logits")
    if ws is None:
        ws = _workspace(tma_loss_workspace_bytes(n, Cc), dev, stream)
    _check(lib().tma_softmax_ce(C.c_int64(n), C.c_int32(Cc), C.c_void_p(logits.data_ptr()), C.c_int64(ldz),
                                C.c_int32(_feat_dtype(logits)), _ptr(labels, torch.int32, "labels"),
                                _ptr(loss_out, torch.float32),
                                C.c_void_p(dlogits_out.data_ptr() if need_grad else 0),
                                _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return loss_out, (dlogits_out if need_grad else None)


def tma_sigmoid_l2(G, Y, loss_out=None, dG_out=None, need_grad=True, ws=None, stream=None):
    n, Cc, ldg = _rows_ld(G, "G")
    dev = G.device
    if tuple(Y.shape) != (n, Cc):
        raise TmaError("tma_sigmoid_l2: Y shape")
    if loss_out is None:
        loss_out = torch.empty(1, dtype=torch.float32, device=dev)
    if need_grad and dG_out is None:
        dG_out = torch.empty((max(n, 1), ldg), dtype=G.dtype, device=dev)[:n, :Cc]
    if need_grad and (tuple(dG_out.shape) != (n, Cc) or _rows_ld(dG_out, "dG_out")[2] != ldg):
        raise TmaError("tma_sigmoid_l2: dG_out must have the shape and leading dimension of G")
    if ws is None:
        ws = _workspace(tma_loss_workspace_bytes(n, Cc), dev, stream)
    _check(lib().tma_sigmoid_l2(C.c_int64(n), C.c_int32(Cc), C.c_void_p(G.data_ptr()), C.c_int64(ldg),
                                C.c_int32(_feat_dtype(G)), _ptr(Y, torch.float32, "Y"),
                                _ptr(loss_out, torch.float32), C.c_void_p(dG_out.data_ptr() if need_grad else 0),
                                _ptr(ws), C.c_size_t(ws.numel()), _stream(stream)))
    return loss_out, (dG_out if need_grad else None)


def tma_sgd_step(W, dW, lr: float, stream=None):
    if W.numel() != dW.numel():
        raise TmaError("tma_sgd_step: W and dW differ in size")
    _check(lib().tma_sgd_step(C.c_int64(W.numel()), _ptr(W, torch.float32, "W"), _ptr(dW, torch.float32, "dW"),
                              C.c_float(lr), _stream(stream)))
    return W


def tma_adam_step(W, dW, m, v, lr: float, step: int, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                  stream=None):
    if not (W.numel() == dW.numel() == m.numel() == v.numel()):
        raise TmaError("tma_adam_step: W, dW, m, v must have the same length")
    _check(lib().tma_adam_step(C.c_int64(W.numel()), _ptr(W, torch.float32, "W"), _ptr(dW, torch.float32, "dW"),
                               _ptr(m, torch.float32, "m"), _ptr(v, torch.float32, "v"), C.c_double(lr),
                               C.c_double(beta1), C.c_double(beta2), C.c_double(eps), C.c_int64(step), _stream(stream)))
    return W


def tma_average(W_list, active_mask: int | None = None, W_global_out=None, ptr_table=None, stream=None):
    """Mean of the active trainers' flat fp32 parameter vectors, written back into each of them.

    ``ptr_table`` (int64 device tensor holding the data pointers) can be passed
    to avoid rebuilding it on every call.
    """
    M = len(W_list)
    n = W_list[0].numel()
    for w in W_list:
        if w.numel() != n or w.dtype != torch.float32 or not w.is_cuda or not w.is_contiguous():
            raise TmaError("tma_average: every W must be a contiguous fp32 GPU tensor of the same size")
    if active_mask is None:
        active_mask = (1 << M) - 1
    if ptr_table is None:
        ptr_table = _record(torch.tensor([w.data_ptr() for w in W_list], dtype=torch.int64, device=W_list[0].device),
                            stream)
    if W_global_out is not None and W_global_out.numel() != n:
        raise TmaError("tma_average: W_global_out size")
    _check(lib().tma_average(_ptr(ptr_table, torch.int64), C.c_int32(M), C.c_uint64(active_mask), C.c_int64(n),
                             _ptr(W_global_out, torch.float32), _stream(stream)))
    return W_global_out


def tma_gather_rows(l2g, src, out=None, stream=None):
    """out[i] = src[l2g[i]] for a 1-D or 2-D row-major table (features, labels)."""
    n_loc = l2g.numel()
    if src.dim() == 1:
        row_bytes, src_ld = src.element_size(), src.element_size()
        shape = (n_loc,)
    else:
        _, cols, ld = _rows_ld(src, "src")
        row_bytes, src_ld = cols * src.element_size(), ld * src.element_size()
        shape = (n_loc, cols)
    if out is None:
        out = torch.empty(shape, dtype=src.dtype, device=src.device)
    if tuple(out.shape) != shape or out.dtype != src.dtype:
        raise TmaError("tma_gather_rows: out must have the gathered shape and the table's dtype")
    dst_ld = row_bytes
    if not out.is_contiguous():      # rows with a pitch of their own (a padded layout)
        if out.dim() != 2 or out.stride(1) != 1 or out.stride(0) < shape[1]:
            raise TmaError("tma_gather_rows: out must be row-major (contiguous, or rows with a larger pitch)")
        dst_ld = out.stride(0) * out.element_size()
    _check(lib().tma_gather_rows(C.c_int64(n_loc), _ptr(l2g, torch.int32, "l2g"), C.c_void_p(src.data_ptr()),
                                 C.c_int64(src_ld), C.c_int64(row_bytes), C.c_void_p(out.data_ptr()),
                                 C.c_int64(dst_ld), _stream(stream)))
    return out


def tma_gather_rows_dev(l2g, d_n_rows, src, out, stream=None):
    """out[i] = src[l2g[i]] for i < min(*d_n_rows, rows of out): the row count is read on the device (1-element
    int32 tensor or view); the launch is sized for all rows of ``out`` (a 2-D row-major buffer)."""
    cap = out.shape[0]
    _, cols, ld = _rows_ld(src, "src")
    row_bytes, src_ld = cols * src.element_size(), ld * src.element_size()
    if out.dim() != 2 or out.shape[1] != cols or out.dtype != src.dtype or out.stride(1) != 1 or l2g.numel() < cap:
        raise TmaError("tma_gather_rows_dev: out must be a row-major [cap, cols] buffer of the table's dtype, l2g as long")
    _check(lib().tma_gather_rows_dev(C.c_int64(cap), _ptr(d_n_rows, torch.int32, "d_n_rows"), _ptr(l2g, torch.int32, "l2g"),
                                     C.c_void_p(src.data_ptr()), C.c_int64(src_ld), C.c_int64(row_bytes),
                                     C.c_void_p(out.data_ptr()), C.c_int64(out.stride(0) * out.element_size()),
                                     _stream(stream)))
    return out


def tma_profile_begin(kernel_filter: str | None = None):
    _check(lib().tma_profile_begin(None if not kernel_filter else kernel_filter.encode()))


def tma_profile_sequence() -> list:
    """Names of the timed launches of the window that the last tma_profile_end closed, in launch order."""
    L = lib()
    out = []
    for i in range(L.tma_profile_sequence_count()):
        name = C.c_char_p()
        _check(L.tma_profile_sequence_entry(C.c_int(i), C.byref(name)))
        out.append(name.value.decode())
    return out


def tma_profile_end() -> dict:
    """Stops the event timing and returns {kernel name: (launches, total_ms)}."""
    L = lib()
    _check(L.tma_profile_end())
    out = {}
    for i in range(L.tma_profile_count()):
        name, cnt, ms = C.c_char_p(), C.c_int64(0), C.c_double(0.0)
        _check(L.tma_profile_entry(C.c_int(i), C.byref(name), C.byref(cnt), C.byref(ms)))
        out[name.value.decode()] = (cnt.value, ms.value)
    return out
