/*
 * libtma -- C ABI of the MI355X (gfx950) hot path of one TMA trainer:
 * random partition assignment, node-induced subgraph extraction, mean
 * aggregation GraphSAGE layer forward/backward, loss, SGD step and on-device
 * parameter averaging ("Randomized Partitions Improve Model Aggregation",
 * RandomTMA / SuperTMA; arXiv 2305.09887).
 *
 * Conventions (all entry points)
 *   - Return value: TMA_OK (0) or a negative tma_status.  No exceptions, no
 *     exit().  tma_last_error() returns a thread-local message for the last
 *     failing call on this thread.
 *   - Pointers are DEVICE pointers unless their name starts with h_.
 *   - The caller owns every buffer and the stream.  The library allocates and
 *     frees no device memory; scratch space is passed in as (ws, ws_bytes) and
 *     sized with the matching *_workspace_bytes query.  Work is enqueued on
 *     `stream` only (a hipStream_t passed as void*; NULL = the default stream)
 *     and the call returns without waiting, except tma_induced_subgraph_count
 *     which must hand two sizes back to the host.
 *   - Matrices are row-major with an explicit leading dimension in ELEMENTS.
 *   - Indices: local graphs int32 rowptr/colidx; the global graph has an int64
 *     rowptr (more than 2^31 entries are allowed) and int32 colidx.
 *   - dtype selects the storage type of features/activations (tma_dtype).
 *     Weights, weight gradients, losses and averaging are always fp32.
 *   - Arguments are validated on the host (NULL where not allowed, negative or
 *     inconsistent sizes, misaligned workspace); the contents of index arrays
 *     are a precondition and are not scanned: 0 <= colidx < n, rowptr
 *     non-decreasing, part ids in [0,K).
 */
#ifndef TMA_H
#define TMA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *tma_stream_t; /* hipStream_t */

typedef enum {
    TMA_OK = 0,
    TMA_ERR_INVALID_ARG = -1,
    TMA_ERR_BAD_SHAPE = -2,
    TMA_ERR_WORKSPACE_TOO_SMALL = -3,
    TMA_ERR_UNSUPPORTED_DTYPE = -4,
    TMA_ERR_HIP = -5
} tma_status;

typedef enum { TMA_F32 = 0, TMA_BF16 = 1 } tma_dtype;
typedef enum { TMA_ACT_NONE = 0, TMA_ACT_RELU = 1 } tma_act;

/* Library version as major*10000 + minor*100 + patch. */
int tma_version(void);

/* Message of the last error raised on the calling thread ("" if none). */
const char *tma_last_error(void);

/* ------------------------------------------------------------------------
 * Random assignment (paper Sec. 3.2.2).
 *   cluster == NULL : RandomTMA -- each node is assigned independently and
 *                     uniformly to one of K partitions.
 *   cluster != NULL : SuperTMA  -- each super-node (mini-cluster id in
 *                     [0, n_clusters)) is assigned that way and a node
 *                     inherits the partition of cluster[v].  With one node
 *                     per super-node (cluster[v] = v) the result equals
 *                     RandomTMA's, as the paper notes for N = |V|.
 * The paper fixes no generator; this library's is
 *     part = floor( SplitMix64(seed, unit) * K / 2^64 ),
 * SplitMix64(seed, unit) = output number unit+1 of the SplitMix64 stream
 * seeded with `seed`.  Pure function of (seed, unit id, K).
 *   part_out [n_nodes] int32, written.   1 <= K <= 2^30.
 * ---------------------------------------------------------------------- */
int tma_partition(int64_t n_nodes, const int32_t *cluster, int64_t n_clusters,
                  int32_t K, uint64_t seed, int32_t *part_out, tma_stream_t stream);

/* The generator itself, on the host: SplitMix64(seed, unit) as defined above (the paper asks for random,
 * independent assignment, Sec. 3.2.2, and names no generator).  For callers that derive one seed from another
 * with the library's own rule, e.g. the neighbour sampler's seed of step t and layer l,
 * tma_mix64(batch_seed, 64 t + l).  Pure function; no GPU work. */
uint64_t tma_mix64(uint64_t seed, uint64_t unit);

/* ------------------------------------------------------------------------
 * Node-induced subgraph of partition p (paper, Preliminaries):
 *   V^(p) = { v : part[v] = p },  E^(p) = { (u,v) in E : u, v in V^(p) }.
 * Canonical output: local id = rank of the global id within V^(p); the
 * neighbours of a row keep their input order.  Two calls:
 *
 * _count  writes g2l_out [n_nodes] (local id, or -1 outside the part),
 *         l2g_out [cap_n_loc], rowptr_loc_out [cap_n_loc + 1]; then WAITS for
 *         the stream and stores |V^(p)| and the number of kept CSR entries in
 *         *h_n_loc / *h_nnz_loc (host memory).  If |V^(p)| > cap_n_loc nothing
 *         is written past the capacity, the sizes are still reported and the
 *         call returns TMA_ERR_BAD_SHAPE (retry with larger buffers).  More
 *         than 2^31-1 kept entries also give TMA_ERR_BAD_SHAPE.
 * _fill   writes colidx_loc_out [nnz_loc] and inv_deg_out [n_loc]
 *         (1/local degree in fp32, 0 for a node without local neighbours);
 *         asynchronous.  It takes the g2l and rowptr_loc that _count wrote and
 *         the SAME workspace and cap_n_loc, untouched since that call: _count
 *         leaves there a membership bitmap and every local row's bounds in the
 *         global CSR, which is why _fill needs neither rowptr, part nor l2g.
 * Workspace: tma_induced_subgraph_workspace_bytes(n_nodes, cap_n_loc) bytes
 * (about n_nodes/8 + 32 * cap_n_loc), 256-byte aligned, shared by the two
 * calls of one extraction.
 * ---------------------------------------------------------------------- */
size_t tma_induced_subgraph_workspace_bytes(int64_t n_nodes, int64_t cap_n_loc);

int tma_induced_subgraph_count(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                               const int32_t *part, int32_t p,
                               int32_t *g2l_out, int32_t *l2g_out, int32_t *rowptr_loc_out,
                               int64_t cap_n_loc, int64_t *h_n_loc, int64_t *h_nnz_loc,
                               void *ws, size_t ws_bytes, tma_stream_t stream);

/* Both calls in one, for a caller that brings buffers of a capacity it chose
 * (colidx_loc_out [cap_nnz_loc], inv_deg_out [cap_n_loc], the others as for
 * _count): no return to the caller between the host wait and the second
 * pass.  TMA_ERR_BAD_SHAPE, with the sizes reported, if either capacity is
 * too small (nothing is then written to colidx_loc_out / inv_deg_out). */
int tma_induced_subgraph(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                         const int32_t *part, int32_t p,
                         int32_t *g2l_out, int32_t *l2g_out, int32_t *rowptr_loc_out,
                         int32_t *colidx_loc_out, float *inv_deg_out,
                         int64_t cap_n_loc, int64_t cap_nnz_loc,
                         int64_t *h_n_loc, int64_t *h_nnz_loc,
                         void *ws, size_t ws_bytes, tma_stream_t stream);

/* The same extraction with no host wait, for callers that keep the sizes on
 * the device (a step replayed as a HIP graph, a loop that never blocks): both
 * passes are enqueued over as many rows as the capacity allows and the second
 * pass reads the node count from device memory.  d_sizes_out [2] int64
 * (device) receives |V^(p)| and the kept entries of the first
 * min(|V^(p)|, cap_n_loc) rows; the caller reads it when it wants to (e.g. an
 * asynchronous copy) and must check both against its capacities: rows past
 * cap_n_loc are dropped, and a row whose entries would end past cap_nnz_loc
 * gets its inv_deg but no entries -- nothing is ever written out of bounds.
 * Within the capacities all five outputs equal those of
 * tma_induced_subgraph bit for bit; elements past the actual sizes are left
 * untouched.  Same workspace as above.  Nothing here clears memory with a
 * memset, so the call may be captured into a graph. */
int tma_induced_subgraph_async(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                               const int32_t *part, int32_t p,
                               int32_t *g2l_out, int32_t *l2g_out, int32_t *rowptr_loc_out,
                               int32_t *colidx_loc_out, float *inv_deg_out,
                               int64_t cap_n_loc, int64_t cap_nnz_loc, int64_t *d_sizes_out,
                               void *ws, size_t ws_bytes, tma_stream_t stream);

/* RandomTMA's assignment (Sec. 3.2.2) fused into the extraction: the outputs of
 * tma_partition(n_nodes, NULL, 0, K, seed, part) followed by
 * tma_induced_subgraph_async(..., part, p, ...), bit for bit, without a part
 * array.  Node v belongs to the part iff floor(SplitMix64(seed, v) * K / 2^64)
 * = p, so membership of a neighbour is recomputed (a few integer multiplies)
 * where the general form looks it up; on graphs whose membership bitmap
 * outgrows the L2 those look-ups, not the entries, bound the extraction.
 * Arguments, capacities, workspace and error behaviour as for
 * tma_induced_subgraph_async; 1 <= K <= 2^30, 0 <= p < K.  (Super-node
 * assignments go through tma_partition and the general form.) */
int tma_random_subgraph_async(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                              int32_t K, uint64_t seed, int32_t p,
                              int32_t *g2l_out, int32_t *l2g_out, int32_t *rowptr_loc_out,
                              int32_t *colidx_loc_out, float *inv_deg_out,
                              int64_t cap_n_loc, int64_t cap_nnz_loc, int64_t *d_sizes_out,
                              void *ws, size_t ws_bytes, tma_stream_t stream);

int tma_induced_subgraph_fill(int64_t n_nodes, const int32_t *colidx,
                              const int32_t *g2l, int64_t n_loc, const int32_t *rowptr_loc,
                              int32_t *colidx_loc_out, float *inv_deg_out,
                              int64_t cap_n_loc, const void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Mean aggregation with the row-normalised adjacency (paper Thm. 1 and the
 * first equation of its proof), over the local neighbourhood:
 *     M_v = inv_deg[v] * sum_{u in N'(v)} H_u        (0 for an isolated node)
 * H, M_out: [n, F] of `dtype`, leading dimensions ldh / ldm.  fp32 accumulation
 * in neighbour order.  Also exported on its own because it is the HBM-bound
 * kernel of the path.  With 16-byte aligned pointers and pitches a row is
 * handled in 16-byte pieces; if F is no multiple of such a piece and both
 * pitches leave room for the last whole piece, the padding elements of M_out
 * inside that piece are overwritten.
 * ---------------------------------------------------------------------- */
int tma_mean_aggregate(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                       const float *inv_deg, const void *H, int64_t ldh, int32_t F,
                       int32_t dtype, void *M_out, int64_t ldm, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * One mean-aggregation GraphSAGE layer, forward:
 *     M = Abar H,   Z = H W_self + M W_neigh + 1 b^T,   H' = act(Z)
 * (the paper names the encoder, Sec. 4.1, and writes its aggregation as
 * Abar X W in Thm. 1; self and neighbour terms have separate weights, the
 * neighbour mean excludes the node itself).
 *   H       [n, F_in]  dtype, ld = ldh
 *   W_self, W_neigh [F_in, F_out] fp32 row-major, dense;  bias [F_out] fp32
 *   M_out   [n, F_in]  dtype, leading dimension ldm >= F_in, 16-byte aligned: the layer's saved state.  It holds
 *           M = Abar H when the layer aggregates first (tma_sage_layer_aggregates_first() = 1).  When
 *           F_out is at most about half of F_in the layer transforms first -- Y = H [W_self | W_neigh],
 *           H' = act(Y_self + Abar Y_neigh + b), the same function by linearity with a much narrower
 *           gather -- and uses M_out as scratch; backward then ignores M.
 *   Hnext_out [n, F_out] dtype, leading dimension ld_next >= F_out; padding
 *           columns are either left alone or set to zero.  With TMA_ACT_RELU the sign pattern of
 *           H' equals that of Z, so H' is all that backward needs.
 * The 16-byte vector paths need 16-byte aligned pointers and leading
 * dimensions that are multiples of 16 bytes (pad rows for widths such as
 * 47, or 100 in bf16); anything else takes a slower element-wise path with
 * the same result.  A row width that is no multiple of 16 bytes still takes
 * the vector path of the aggregation when ldh and ldm leave room for the last
 * whole 16-byte piece (100 bf16 elements with ld >= 104): the padding elements
 * of M_out up to that piece are then overwritten (with sums of H's padding).
 * No workspace.
 * ---------------------------------------------------------------------- */
/* 1 if a layer of these widths aggregates first (M_out = Abar H), 0 if it transforms first. */
int tma_sage_layer_aggregates_first(int32_t F_in, int32_t F_out, int32_t dtype);

int tma_sage_layer_fwd(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                       const float *inv_deg,
                       const void *H, int64_t ldh, int32_t F_in,
                       const float *W_self, const float *W_neigh, const float *bias,
                       int32_t F_out, int32_t act, int32_t dtype,
                       void *M_out, int64_t ldm, void *Hnext_out, int64_t ld_next, tma_stream_t stream);

/* The same layer (Thm. 1: Abar X W; Sec. 4.1: GraphSAGE) for bf16 storage with the weight operand prepared once
 * instead of narrowed from fp32 inside every tile of the product.
 * tma_sage_prepare_weights_bf16 writes Wt_out[o * 2 F_in + k] = bf16(k < F_in ? W_self[k][o] : W_neigh[k - F_in][o])
 * (round to nearest even, the rounding the product applies itself), tma_sage_weights_bf16_bytes(F_in, F_out) bytes,
 * 16-byte aligned, caller-owned; call it again whenever the weights have changed.
 * tma_sage_layer_fwd_prepared takes the arguments of tma_sage_layer_fwd plus that array (dtype must be TMA_BF16)
 * and returns the same bits; a layer that transforms first, or operands without 8-byte aligned groups of four,
 * run as in tma_sage_layer_fwd (W_self / W_neigh must therefore be valid too). */
size_t tma_sage_weights_bf16_bytes(int32_t F_in, int32_t F_out);

int tma_sage_prepare_weights_bf16(const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out,
                                  void *Wt_out, tma_stream_t stream);

int tma_sage_layer_fwd_prepared(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                                const float *inv_deg,
                                const void *H, int64_t ldh, int32_t F_in,
                                const float *W_self, const float *W_neigh, const float *bias,
                                int32_t F_out, int32_t act, int32_t dtype,
                                void *M_out, int64_t ldm, void *Hnext_out, int64_t ld_next,
                                const void *Wt_bf16, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Backward of the layer (chain rule as in the proof of Thm. 1, which writes
 * the one-layer case dL/dw = dL/dz * dz/dg * dg/dw):
 *     dZ = dHnext (.) act'(Z)                  (act' from the sign of Hnext)
 *     dW_self = H^T dZ,  dW_neigh = M^T dZ,  dbias = column sums of dZ
 *     dH = dZ W_self^T + Abar^T (dZ W_neigh^T)
 *   H, M, ldm as in forward;  Hnext [n, F_out] the forward output (read only
 *            when act = TMA_ACT_RELU);  dHnext [n, F_out] dtype; both with
 *            leading dimension ld_next (padding columns are ignored)
 *   rowptr_T/colidx_T : CSR of the TRANSPOSED local graph.  For a symmetric
 *            graph (every configuration of a simple undirected graph) pass
 *            rowptr/colidx again.  inv_deg is that of the forward graph.
 *   dW_self, dW_neigh [F_in, F_out], dbias [F_out] fp32: OVERWRITTEN.
 *   dH_out [n, F_in] dtype with the leading dimension of H (ldh), or NULL to
 *            skip the input gradient (first layer).
 * Workspace: tma_sage_layer_bwd_workspace_bytes(n, F_in, F_out, dtype,
 * dH_out != NULL), 256-byte aligned.  Results are deterministic (fixed
 * reduction order, no floating-point atomics).
 * ---------------------------------------------------------------------- */
size_t tma_sage_layer_bwd_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out,
                                          int32_t dtype, int32_t need_dH);

int tma_sage_layer_bwd(int64_t n, const int32_t *rowptr_T, const int32_t *colidx_T,
                       const float *inv_deg,
                       const void *H, int64_t ldh, const void *M, int64_t ldm, const void *Hnext,
                       const void *dHnext, int64_t ld_next,
                       const float *W_self, const float *W_neigh,
                       int32_t F_in, int32_t F_out, int32_t act, int32_t dtype,
                       float *dW_self, float *dW_neigh, float *dbias, void *dH_out,
                       void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Normalisation and activation of the paper's encoders (Sec. 4.1, paragraph on
 * GNN encoders: PReLU as the non-linearity, Layer Normalization before it),
 * applied to a layer's pre-activation Z (run the layer with TMA_ACT_NONE):
 *     Zh = (Z - mean_f Z) / sqrt(var_f Z + eps)     per node, biased variance
 *     Y  = gamma (.) Zh + beta                      gamma, beta [F] fp32
 *     H' = Y where Y > 0, slope * Y elsewhere       slope: ONE fp32 value (device)
 * _fwd writes H' [n, F] (leading dimension ld_out); Z is kept by the caller for
 * backward.  _bwd takes dL/dH' and writes dZ_out [n, F] = dL/dZ (pass it to
 * tma_sage_layer_bwd as dHnext with TMA_ACT_NONE; dZ_out may alias dHnext),
 * dgamma [F], dbeta [F], dslope [1] (overwritten, fixed summation order).
 * Z, dHnext, H', dZ of `dtype`; rows of at most 1024 elements; 16-byte
 * aligned pointers and leading dimensions take the vector path.
 * Workspace (_bwd): tma_layernorm_prelu_bwd_workspace_bytes(n, F), 256-byte
 * aligned.
 * ---------------------------------------------------------------------- */
int tma_layernorm_prelu_fwd(int64_t n, int32_t F, const void *Z, int64_t ldz,
                            const float *gamma, const float *beta, const float *slope, float eps,
                            int32_t dtype, void *Hnext_out, int64_t ld_out, tma_stream_t stream);

size_t tma_layernorm_prelu_bwd_workspace_bytes(int64_t n, int32_t F);

int tma_layernorm_prelu_bwd(int64_t n, int32_t F, const void *Z, int64_t ldz,
                            const void *dHnext, int64_t ld_d,
                            const float *gamma, const float *beta, const float *slope, float eps,
                            int32_t dtype, void *dZ_out, int64_t ld_dz,
                            float *dgamma, float *dbeta, float *dslope,
                            void *ws, size_t ws_bytes, tma_stream_t stream);

/* tma_layernorm_prelu_bwd for callers that cannot allocate or carry a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without (ws, ws_bytes), same kernels, same
 * results bit for bit.  The per-block partial sums go to an array that the library itself holds in device memory
 * (4.2 MB per GPU, from load until the process ends), sized for rows of at most
 * tma_layernorm_prelu_bwd_static_max_f() = 256 elements; a larger F returns TMA_ERR_BAD_SHAPE and launches
 * nothing.  The call allocates and frees nothing.  All calls on one GPU share that array: calls that may overlap
 * on one GPU (different streams without an ordering between them) race on it and must use the workspace form;
 * nothing in it has to be cleared between calls (every slot that is read is written first, in the same call). */
int32_t tma_layernorm_prelu_bwd_static_max_f(void);

int tma_layernorm_prelu_bwd_static(int64_t n, int32_t F, const void *Z, int64_t ldz,
                                   const void *dHnext, int64_t ld_d,
                                   const float *gamma, const float *beta, const float *slope, float eps,
                                   int32_t dtype, void *dZ_out, int64_t ld_dz,
                                   float *dgamma, float *dbeta, float *dslope, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * The paper's other encoders (Sec. 4.1, paragraph on GNN encoders).
 *
 * Dense layer -- a layer of the graph-agnostic MLP encoder and, without bias,
 * of the link decoder (App., formulation of the MLP decoder):
 *     Y = act(X W + 1 b^T)
 *     dZ = dY (.) act'(Y);  dW = X^T dZ;  dbias = 1^T dZ;  dX = dZ W^T
 *   X [n, F_in] dtype, ldx;  W [F_in, F_out] fp32 row-major;  bias [F_out] fp32
 *   or NULL;  Y, dY [n, F_out] dtype, ldy;  act as for the SAGE layer (Y is
 *   read by the backward only with TMA_ACT_RELU).
 *   dW [F_in, F_out] fp32 OVERWRITTEN; dbias [F_out] fp32 or NULL; dX_out
 *   [n, F_in] dtype with leading dimension ld_dx, or NULL to skip it.
 * All pointers device memory; n = 0 is a no-op forward and writes zero
 * gradients backward.  Workspace of the backward:
 * tma_dense_bwd_workspace_bytes(n, F_in, F_out), 256-byte aligned.
 * Deterministic (fixed reduction order).
 * ---------------------------------------------------------------------- */
int tma_dense_fwd(int64_t n, const void *X, int64_t ldx, int32_t F_in,
                  const float *W, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                  void *Y_out, int64_t ldy, tma_stream_t stream);

size_t tma_dense_bwd_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out);

int tma_dense_bwd(int64_t n, const void *X, int64_t ldx, const void *Y, const void *dY, int64_t ldy,
                  const float *W, int32_t F_in, int32_t F_out, int32_t act, int32_t dtype,
                  float *dW, float *dbias, void *dX_out, int64_t ld_dx,
                  void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * GCN layer (the graph convolution of Kipf & Welling, which the paper cites
 * for its GCN encoder) on the local subgraph:
 *     Ahat = S (A + I) S,  S = diag(s),  s_v = (d_v + 1)^-1/2, d_v = local degree
 *     Hnext = act(Ahat H W + 1 b^T)
 *     dZ = dHnext (.) act'(Hnext);  dW = (Ahat H)^T dZ;  dbias = 1^T dZ;
 *     dH = Ahat^T dZ W^T
 * tma_gcn_norm writes s [n] fp32 from the local rowptr (once per extraction).
 *   rowptr/colidx, H, ldh, act, dtype, Hnext, dHnext, ld_next: as for the SAGE
 *   layer;  W [F_in, F_out], bias [F_out] fp32.  The backward takes the CSR
 *   of the TRANSPOSED local graph (the same arrays for a symmetric graph).
 *   dW [F_in, F_out], dbias [F_out] fp32 OVERWRITTEN;  dH_out [n, F_in] dtype
 *   with leading dimension ldh, or NULL.
 * The gather runs on the narrower side: the layer aggregates first (M_out =
 * Ahat H, kept for the backward) unless F_out padded to 16 bytes is smaller
 * than F_in; then it multiplies first and M_out is scratch; tma_gcn_layer_aggregates_first
 * tells which.  M_out / M: [n, F_in] dtype, dense, 16-byte aligned, never
 * aliasing H; the backward reads M only in the aggregate-first form and H only
 * in the other (the unused one may be NULL).
 * Backward workspace (256-byte aligned): tma_gcn_layer_bwd_workspace_bytes(n,
 * F_in, F_out, dtype, dH_out != NULL).  Deterministic.
 * ---------------------------------------------------------------------- */
int tma_gcn_norm(int64_t n, const int32_t *rowptr, float *s_out, tma_stream_t stream);

int tma_gcn_layer_aggregates_first(int32_t F_in, int32_t F_out, int32_t dtype);

int tma_gcn_layer_fwd(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *s_norm,
                      const void *H, int64_t ldh, int32_t F_in,
                      const float *W, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                      void *M_out, void *Hnext_out, int64_t ld_next, tma_stream_t stream);

size_t tma_gcn_layer_bwd_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out, int32_t dtype,
                                         int32_t need_dH);

int tma_gcn_layer_bwd(int64_t n, const int32_t *rowptr_T, const int32_t *colidx_T, const float *s_norm,
                      const void *H, int64_t ldh, const void *M, const void *Hnext, const void *dHnext,
                      int64_t ld_next,
                      const float *W, int32_t F_in, int32_t F_out, int32_t act, int32_t dtype,
                      float *dW, float *dbias, void *dH_out,
                      void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Link-prediction head (Sec. 4.1, paragraphs on the link prediction decoder
 * and on mini-batch and negative sampling; App., formulation of the MLP
 * decoder).  All pointers device memory unless stated; every call is ordered
 * on `stream`, allocates nothing, and is deterministic.
 *
 * tma_edge_batch: B positive edges drawn uniformly with replacement from the
 * local CSR entries and one negative tail per positive, uniform over the local
 * nodes other than the positive tail.  Counter-based: sample i uses counter
 * c = first_counter + i of the SplitMix64 stream of tma_partition,
 *     e = floor(z(2c) * nnz / 2^64),  u = row of entry e,  v = colidx[e],
 *     r = floor(z(2c+1) * (n-1) / 2^64),  v' = r + (r >= v).
 *   n, nnz : local node and entry counts (host values; B > 0 needs n >= 2 and
 *            nnz >= 1);  rowptr [n+1], colidx [nnz] int32
 *   u_out, v_out, vneg_out [B] int32.
 *
 * tma_pair_product_fwd: decoder input E0 [2B, F] (leading dimension lde):
 * row i = r_u(i) (.) r_v(i), row B+i = r_u(i) (.) r_v'(i), from the embeddings
 * R [n, F] dtype (leading dimension ldr).
 *
 * tma_pair_product_bwd: dR [n, F] (leading dimension ld_dr) = gradient of E0
 * w.r.t. R given dE0 [2B, F]; rows of nodes outside the batch are zero.  A
 * node's terms are summed in a fixed order (no floating-point atomics).
 * Workspace: tma_pair_product_bwd_workspace_bytes(n, B, F, dtype), 256-byte
 * aligned.
 *
 * tma_prelu_fwd / _bwd: Y = Z > 0 ? Z : a Z with one learnable slope a
 * (slope: 1 fp32 value in device memory); dZ = dY (Z > 0 ? 1 : a), dslope_out
 * [1] fp32 = sum of dY Z over Z <= 0 (OVERWRITTEN).  dZ_out may alias dY.
 * Workspace of the backward: tma_prelu_bwd_workspace_bytes(), 16-byte aligned.
 *
 * tma_bce_logits: mean binary cross-entropy of `count` logits z[i * ldz]
 * (dtype), the first n_pos being positives; loss_out [1] fp32 OVERWRITTEN;
 * dz_out[i * ld_dz] = (sigmoid(z_i) - y_i) / count, or NULL.  The paper calls
 * the decoder's output the link probability and names no loss: this build
 * treats the last layer's scalar as a logit.  Workspace:
 * tma_bce_logits_workspace_bytes(), 16-byte aligned.
 * ---------------------------------------------------------------------- */
int tma_edge_batch(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                   uint64_t seed, uint64_t first_counter, int64_t B,
                   int32_t *u_out, int32_t *v_out, int32_t *vneg_out, tma_stream_t stream);

int tma_pair_product_fwd(int64_t B, int32_t F, const void *R, int64_t ldr, int32_t dtype,
                         const int32_t *u, const int32_t *v, const int32_t *vneg,
                         void *E0_out, int64_t lde, tma_stream_t stream);

size_t tma_pair_product_bwd_workspace_bytes(int64_t n, int64_t B, int32_t F, int32_t dtype);

int tma_pair_product_bwd(int64_t n, int64_t B, int32_t F, const void *R, int64_t ldr, int32_t dtype,
                         const int32_t *u, const int32_t *v, const int32_t *vneg,
                         const void *dE0, int64_t lde, void *dR_out, int64_t ld_dr,
                         void *ws, size_t ws_bytes, tma_stream_t stream);

int tma_prelu_fwd(int64_t n, int32_t F, const void *Z, int64_t ldz, const float *slope, int32_t dtype,
                  void *Y_out, int64_t ldy, tma_stream_t stream);

size_t tma_prelu_bwd_workspace_bytes(void);

int tma_prelu_bwd(int64_t n, int32_t F, const void *Z, int64_t ldz, const void *dY, int64_t ldd,
                  const float *slope, int32_t dtype, void *dZ_out, int64_t ld_dz, float *dslope_out,
                  void *ws, size_t ws_bytes, tma_stream_t stream);

size_t tma_bce_logits_workspace_bytes(void);

int tma_bce_logits(int64_t count, int64_t n_pos, const void *z, int64_t ldz, int32_t dtype,
                   float *loss_out, void *dz_out, int64_t ld_dz,
                   void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Sampled message-flow graphs (Sec. 4.1, paragraph on mini-batch and negative
 * sampling: a GraphSAGE-style sampler caps the neighbours a node aggregates, so
 * a step runs the encoder on the sampled neighbourhood of its batch only).
 * All pointers device memory unless stated; ordered on `stream`; no allocation;
 * deterministic.
 *
 * tma_neighbor_sample: for each of the n_dst DISTINCT local nodes dst[i], all its local
 * neighbours if it has at most `fanout`, else a uniform subset of exactly
 * `fanout` of them: entry e of the local CSR gets the key SplitMix64(seed, e)
 * (the stream of tma_partition) and the row keeps the `fanout` smallest
 * (key, e), in row order.  `seed` is the caller's per step and layer.
 *   nnz            local entry count (host value); rowptr [n+1], colidx [nnz]
 *   blk_rowptr_out [n_dst+1]; blk_col_out, blk_row_out [cap_entries]: kept
 *                  neighbours (local ids) and the row i each belongs to;
 *                  cap_entries >= min(n_dst * fanout, nnz), which distinct
 *                  nodes cannot exceed (nothing is written past it).  The
 *                  number of kept entries is blk_rowptr_out[n_dst] (stays on
 *                  the device).
 * Workspace: tma_neighbor_sample_workspace_bytes(n_dst), 256-byte aligned.
 *
 * tma_mfg_relabel: node list of a block.  src_out = the n_dst nodes of dst, in
 * their order, followed by the other nodes that occur in cols, in ascending
 * id; cols (max_items entries, of which the first *d_items count when d_items
 * is not NULL) is overwritten with positions in src_out.  *h_n_src (HOST)
 * receives the length of src_out: the call waits for the stream.  n = number
 * of local nodes (ids < n); cap_src >= min(n, n_dst + max_items).  With
 * n_dst = 0 this is "sorted unique ids + positions" (the nodes of a batch).
 * Workspace: tma_mfg_relabel_workspace_bytes(n), 256-byte aligned.
 *
 * tma_neighbor_sample_dev / tma_mfg_relabel_dev: the same two steps for a caller
 * that lets the level sizes stay on the device while it samples (no wait for
 * the stream between the levels of a batch; the sizes are read back once, after
 * the last level).  cap_dst is the capacity the launches are sized for and
 * *d_n_dst (device, <= cap_dst) the number of dst nodes.  The sampler gives the
 * rows from *d_n_dst up to cap_dst no entries: blk_rowptr_out has cap_dst + 1
 * elements, its elements [*d_n_dst .. cap_dst] all hold the number of kept
 * entries (so &blk_rowptr_out[cap_dst] serves as d_items of the relabelling),
 * workspace and cap_entries are those of cap_dst rows.  The relabelling writes
 * the length of src_out to *d_n_src_out (device) and returns without waiting;
 * cap_src >= min(n, cap_dst + max_items); with cap_dst = 0, d_n_dst may be NULL.
 * The first *d_n_dst rows / *d_n_src_out nodes and all entries are, bit for
 * bit, what the host-count forms produce.
 *
 * tma_block_inv_deg: inv_deg_out[i] = 1 / (entries of block row i), 0 for an
 * empty row.
 *
 * tma_sage_block_fwd / _bwd: the mean-aggregation GraphSAGE layer of
 * tma_sage_layer_fwd / _bwd on a bipartite block: n_dst output rows; H has
 * n_src >= n_dst rows whose first n_dst are the dst nodes themselves; blk_col
 * holds positions in [0, n_src).  M_out [n_dst, F_in] always receives Abar H
 * (the block form always aggregates first).  The backward writes dH_out for
 * all n_src rows (leading dimension ldh; NULL to skip) and builds the block's
 * transpose itself (it needs blk_row and max_entries >= the entry count).
 * Workspace: tma_sage_block_bwd_workspace_bytes(n_dst, n_src, max_entries,
 * F_in, F_out, dtype, dH_out != NULL), 256-byte aligned.
 * ---------------------------------------------------------------------- */
size_t tma_neighbor_sample_workspace_bytes(int64_t n_dst);

int tma_neighbor_sample(int64_t n_dst, const int32_t *dst, int64_t nnz, const int32_t *rowptr,
                        const int32_t *colidx, int32_t fanout, uint64_t seed,
                        int32_t *blk_rowptr_out, int32_t *blk_col_out, int32_t *blk_row_out,
                        int64_t cap_entries, void *ws, size_t ws_bytes, tma_stream_t stream);

size_t tma_mfg_relabel_workspace_bytes(int64_t n);

int tma_mfg_relabel(int64_t n, int64_t n_dst, const int32_t *dst, int64_t max_items,
                    const int32_t *d_items, int32_t *cols_inout, int32_t *src_out, int64_t cap_src,
                    int64_t *h_n_src, void *ws, size_t ws_bytes, tma_stream_t stream);

int tma_neighbor_sample_dev(int64_t cap_dst, const int32_t *d_n_dst, const int32_t *dst, int64_t nnz,
                            const int32_t *rowptr, const int32_t *colidx, int32_t fanout, uint64_t seed,
                            int32_t *blk_rowptr_out, int32_t *blk_col_out, int32_t *blk_row_out,
                            int64_t cap_entries, void *ws, size_t ws_bytes, tma_stream_t stream);

int tma_mfg_relabel_dev(int64_t n, int64_t cap_dst, const int32_t *d_n_dst, const int32_t *dst,
                        int64_t max_items, const int32_t *d_items, int32_t *cols_inout, int32_t *src_out,
                        int64_t cap_src, int32_t *d_n_src_out, void *ws, size_t ws_bytes, tma_stream_t stream);

int tma_block_inv_deg(int64_t n_dst, const int32_t *blk_rowptr, float *inv_deg_out, tma_stream_t stream);

int tma_sage_block_fwd(int64_t n_dst, int64_t n_src, const int32_t *blk_rowptr, const int32_t *blk_col,
                       const float *inv_deg, const void *H, int64_t ldh, int32_t F_in,
                       const float *W_self, const float *W_neigh, const float *bias,
                       int32_t F_out, int32_t act, int32_t dtype,
                       void *M_out, void *Hnext_out, int64_t ld_next, tma_stream_t stream);

size_t tma_sage_block_bwd_workspace_bytes(int64_t n_dst, int64_t n_src, int64_t max_entries,
                                          int32_t F_in, int32_t F_out, int32_t dtype, int32_t need_dH);

int tma_sage_block_bwd(int64_t n_dst, int64_t n_src, int64_t max_entries,
                       const int32_t *blk_rowptr, const int32_t *blk_col, const int32_t *blk_row,
                       const float *inv_deg, const void *H, int64_t ldh, const void *M,
                       const void *Hnext, const void *dHnext, int64_t ld_next,
                       const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out,
                       int32_t act, int32_t dtype,
                       float *dW_self, float *dW_neigh, float *dbias, void *dH_out,
                       void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * GCN layer on a bipartite block of a sampled message-flow graph (Sec. 4.1:
 * the GCN encoder trained with the neighbour sampler).  The symmetric
 * normalisation of tma_gcn_layer_* needs a degree for the source side, which
 * a sampled block does not define; on a block the layer is taken in its
 * row-normalised form with the self-loop,
 *     m_v = ( h_v + sum_{u in S(v)} h_u ) / ( |S(v)| + 1 ),  Z = M W + 1 b^T,
 *     H' = act(Z),
 * the mean over the sampled neighbourhood and the node itself.  Blocks, node
 * order (the n_dst destination nodes are the first sources) and buffers as
 * for tma_sage_block_*.
 *   tma_gcn_block_norm: c_out [n_dst] fp32 = 1 / (|S(v)| + 1).
 *   tma_gcn_block_fwd:  M_out [n_dst, F_in] dense (16-byte aligned, kept for
 *     the backward pass), Hnext_out [n_dst, F_out] with leading dimension
 *     ld_next; W [F_in, F_out] and bias fp32.
 *   tma_gcn_block_bwd:  dW = M^T dZ, dbias = 1^T dZ with dZ = dHnext (.)
 *     act'(Hnext); dH_out [n_src, F_in] (leading dimension ldh; NULL = not
 *     wanted) = (A_S + I)^T diag(c) dZ W^T.  blk_row [max_entries]: the dst row
 *     of every block entry, as tma_neighbor_sample wrote it.
 * Workspace of the backward pass: tma_gcn_block_bwd_workspace_bytes(n_dst,
 * n_src, max_entries, F_in, F_out, dtype, dH_out != NULL), 256-byte aligned.
 * ---------------------------------------------------------------------- */
int tma_gcn_block_norm(int64_t n_dst, const int32_t *blk_rowptr, float *c_out, tma_stream_t stream);

int tma_gcn_block_fwd(int64_t n_dst, int64_t n_src, const int32_t *blk_rowptr, const int32_t *blk_col,
                      const float *c_norm, const void *H, int64_t ldh, int32_t F_in,
                      const float *W, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                      void *M_out, void *Hnext_out, int64_t ld_next, tma_stream_t stream);

size_t tma_gcn_block_bwd_workspace_bytes(int64_t n_dst, int64_t n_src, int64_t max_entries,
                                         int32_t F_in, int32_t F_out, int32_t dtype, int32_t need_dH);

int tma_gcn_block_bwd(int64_t n_dst, int64_t n_src, int64_t max_entries,
                      const int32_t *blk_rowptr, const int32_t *blk_col, const int32_t *blk_row,
                      const float *c_norm, const void *M, const void *Hnext, const void *dHnext,
                      int64_t ld_next, const float *W, int32_t F_in, int32_t F_out,
                      int32_t act, int32_t dtype, float *dW, float *dbias,
                      void *dH_out, int64_t ldh, void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Losses on the last layer's output.
 * tma_softmax_ce: mean softmax cross-entropy over the n local nodes (reading
 *   taken for workloads with class labels); loss_out[0] fp32 (device),
 *   dlogits_out = (softmax - onehot)/n in `dtype`, [n, C] with the leading
 *   dimension of the logits (ld); may be NULL.
 * tma_sigmoid_l2: the loss of Thm. 1, L = 1/2 sum (y - sigmoid(g))^2 over all
 *   nodes and outputs; dG = (z - y) z (1 - z), laid out like G (ld).
 *   Y fp32 dense [n, C].
 * Workspace: tma_loss_workspace_bytes(n, C) bytes, 256-byte aligned.
 * ---------------------------------------------------------------------- */
size_t tma_loss_workspace_bytes(int64_t n, int32_t C);

int tma_softmax_ce(int64_t n, int32_t C, const void *logits, int64_t ld, int32_t dtype,
                   const int32_t *labels, float *loss_out, void *dlogits_out,
                   void *ws, size_t ws_bytes, tma_stream_t stream);

int tma_sigmoid_l2(int64_t n, int32_t C, const void *G, int64_t ld, int32_t dtype,
                   const float *Y, float *loss_out, void *dG_out,
                   void *ws, size_t ws_bytes, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Optimizer step of Alg. 2 (the paper does not name the optimizer; plain SGD
 * is the reading taken): W <- W - lr * dW over a flat fp32 vector.
 * ---------------------------------------------------------------------- */
int tma_sgd_step(int64_t n_params, float *W, const float *dW, float lr, tma_stream_t stream);

/* Adam (Kingma & Ba) as a second choice for the same call, with bias correction:
 *     m <- beta1 m + (1-beta1) dW,  v <- beta2 v + (1-beta2) dW^2,
 *     W <- W - lr (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps),   step = 1, 2, ...
 * The scalars are doubles so that 1-beta and the bias corrections are formed exactly before they are
 * narrowed.  m, v [n_params] fp32 are the trainer's own state (zero before the first step); the
 * aggregation operator averages parameters only (Sec. 3.1), never this state. */
int tma_adam_step(int64_t n_params, float *W, const float *dW, float *m, float *v,
                  double lr, double beta1, double beta2, double eps, int64_t step, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Aggregation operator phi of Alg. 1 = arithmetic mean of the trainers'
 * parameters (Sec. 3.1), followed by the overwrite of Alg. 2: every ACTIVE
 * trainer's vector is replaced by the mean.  Trainers whose bit in
 * active_mask is clear are skipped and left untouched (the paper's failure
 * experiment continues with the remaining trainers).
 *   W_ptrs : DEVICE array of n_trainers device pointers, each [n_params] fp32
 *   n_trainers in [1, 64]
 *   W_global_out : [n_params] fp32 or NULL
 * Sum in trainer-index order in fp32, then one multiply by 1/|active|.
 * The caller orders this call after the trainers' last steps (events).
 * ---------------------------------------------------------------------- */
int tma_average(float *const *W_ptrs, int32_t n_trainers, uint64_t active_mask,
                int64_t n_params, float *W_global_out, tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Gather of the local rows of a row-major table (a trainer "loads" its part
 * of the feature matrix and of the label vector, Alg. 2, set-up line):
 *     dst[i, :] = src[l2g[i], :]     for i in [0, n_loc)
 * Rows are row_bytes long; src_ld_bytes / dst_ld_bytes are the row pitches.
 * Any element type: 16-byte copies when pointers, pitches and row_bytes are
 * multiples of 16, 4-byte copies when multiples of 4, else byte copies.
 * ---------------------------------------------------------------------- */
int tma_gather_rows(int64_t n_loc, const int32_t *l2g, const void *src, int64_t src_ld_bytes,
                    int64_t row_bytes, void *dst, int64_t dst_ld_bytes, tma_stream_t stream);

/* The same with the row count on the device: rows [0, min(*d_n_rows, cap_rows)) are copied, the launch is sized for
 * cap_rows and nothing else is written (for the input rows of a sampled batch whose size has not come back yet). */
int tma_gather_rows_dev(int64_t cap_rows, const int32_t *d_n_rows, const int32_t *l2g, const void *src,
                        int64_t src_ld_bytes, int64_t row_bytes, void *dst, int64_t dst_ld_bytes,
                        tma_stream_t stream);

/* ------------------------------------------------------------------------
 * Measurement aid (not part of the method): per-kernel durations from HIP
 * events recorded on the launch stream around every kernel launch of this
 * library between _begin and _end.  kernel_filter NULL or "" times every
 * kernel; otherwise only the kernel with exactly that name.  _end waits for
 * the recorded events, then _count/_entry read the totals per kernel name
 * (name_out stays valid until the next _begin).  Host-side state only.
 * ---------------------------------------------------------------------- */
int tma_profile_begin(const char *kernel_filter);
int tma_profile_end(void);
int tma_profile_count(void);
int tma_profile_entry(int index, const char **name_out, int64_t *launches_out, double *total_ms_out);
/* The timed launches of the window that the last _end closed, in launch order (the same names; a profiler's
 * dispatch list of the same run can be matched against it one to one). */
int tma_profile_sequence_count(void);
int tma_profile_sequence_entry(int index, const char **name_out);

#ifdef __cplusplus
}
#endif
#endif /* TMA_H */
