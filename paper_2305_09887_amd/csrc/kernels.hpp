// Internal launch interface between the translation units of libtma.
#pragma once

#include "common.hpp"

namespace tma {

// Row gather-reduce over a CSR:  out_v = scale_v * sum_{u in row v} in_u  (+ out_v when accumulate).
// scale_v = inv_deg[v] when inv_deg != nullptr, else 1.  fp32 accumulation in neighbour order.
// in_rows: rows of `in` when it is not an n-row matrix (the ids of colidx index it); 0 = n rows.
int launch_spmm(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                int64_t ld_in, int32_t F, int32_t dtype, void *out, int64_t ld_out, bool accumulate,
                hipStream_t stream, int64_t in_rows = 0);

// Same gather with the layer epilogue fused: out_v = act(scale_v * sum + [out_v] + self_v + bias), or, with
// scale_all, out_v = act(scale_v * (sum + [out_v] + self_v) + bias) (the GCN form, self inside the normalisation).
// edge_scale (may be NULL): neighbour u enters the sum as edge_scale[u] * in_u and self_v as edge_scale[v] * self_v.
int launch_spmm_combine(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                        int64_t ld_in, int32_t F, int32_t dtype, void *out, int64_t ld_out, bool accumulate,
                        const void *self, int64_t ld_self, const float *bias, int32_t F_valid, bool relu,
                        bool scale_all, const float *edge_scale, hipStream_t stream, int64_t in_rows = 0);

// dst_v = inv_deg[v] * g_v (.) [h_v > 0]  (mask only with relu); columns F..F_pad-1 of dst are zeroed.
int launch_scale_mask_rows(int64_t n, int32_t F, int32_t F_pad, const void *g, const void *h, int64_t ld,
                           const float *inv_deg, bool relu, int32_t dtype, void *dst, int64_t ld_dst,
                           hipStream_t stream);

// Z = [H | M] [W_self ; W_neigh] + b ;  Hnext = act(Z)      (M: [n, F_in] with leading dimension ldm)
int launch_sage_gemm_fwd(int64_t n, const void *H, int64_t ldh, const void *M, int64_t ldm, int32_t F_in, const float *W_self,
                         const float *W_neigh, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                         void *Hnext, int64_t ld_next, hipStream_t stream, const void *Wt_bf16 = nullptr);
// bf16 copy of [W_self ; W_neigh] with the output feature as the row: Wt[o][k], k < 2 F_in (row pitch 2 F_in)
size_t sage_weights_bf16_bytes(int32_t F_in, int32_t F_out);
int launch_sage_prepare_weights_bf16(const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out, void *Wt_out,
                                     hipStream_t stream);

// [dH_self | inv_deg * dM] = dZ [W_self^T | W_neigh^T],  dZ = dHnext (.) act'(Hnext)
int launch_sage_gemm_bwd_data(int64_t n, const void *dHnext, const void *Hnext, int64_t ld_next,
                              const float *inv_deg, const float *W_self, const float *W_neigh, int32_t F_in,
                              int32_t F_out, int32_t act, int32_t dtype, void *dH_self_out, int64_t ldh,
                              void *dM_scaled_out, hipStream_t stream);

// [dW_self ; dW_neigh] = [H | M]^T dZ,  dbias = 1^T dZ   (split over nodes, two-stage fixed-order reduction)
size_t sage_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out);
int launch_sage_gemm_bwd_weight(int64_t n, const void *H, int64_t ldh, const void *M, int64_t ldm, const void *dHnext,
                                const void *Hnext, int64_t ld_next, int32_t F_in, int32_t F_out, int32_t act,
                                int32_t dtype,
                                float *dW_self, float *dW_neigh, float *dbias, void *ws, size_t ws_bytes,
                                hipStream_t stream);

// Transform-before-aggregate form of the layer (chosen when two padded output widths fit into F_in):
//   forward   [Y_self | Y_neigh] = H [W_self | W_neigh];  Hnext = act(Y_self + Abar Y_neigh + b)  (launch_spmm_combine)
//   backward  dYn = Abar^T dZ (gather of inv_deg-scaled dZ);  [dW_self | dW_neigh] = H^T [dZ | dYn];  db = 1^T dZ;
//             dH = [dZ | dYn] [W_self | W_neigh]^T
// Ys, Yn, dYn: [n, Fp] blocks with leading dimension ldy, Fp = F_out padded to 16 bytes.
int launch_sage_tf_gemm_fwd(int64_t n, const void *H, int64_t ldh, int32_t F_in, const float *W_self,
                            const float *W_neigh, int32_t F_out, int32_t dtype, void *Ys, void *Yn, int64_t ldy,
                            hipStream_t stream);
size_t sage_tf_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out, int32_t dtype);
int launch_sage_tf_gemm_bwd_weight(int64_t n, const void *H, int64_t ldh, const void *dHnext, const void *Hnext,
                                   int64_t ld_next, const void *dYn, int64_t ldy, int32_t F_in, int32_t F_out,
                                   int32_t act, int32_t dtype, float *dW_self, float *dW_neigh, float *dbias, void *ws,
                                   size_t ws_bytes, hipStream_t stream);
int launch_sage_tf_gemm_bwd_data(int64_t n, const void *dHnext, const void *Hnext, int64_t ld_next, const void *dYn,
                                 int64_t ldy, const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out,
                                 int32_t act, int32_t dtype, void *dH, int64_t ldh, hipStream_t stream);

// Second stage of a split weight-gradient product, fixed order: partial is [n_splits][halves * F][N] and
// colsum_partial [n_splits][N]; rows [0, F) go to dW_first, rows [F, 2F) (halves = 2) to dW_second, the
// column sums to dbias (skipped when NULL).  n_splits = 0 writes zeros.
int launch_reduce_splits(const float *partial, const float *colsum_partial, int n_splits, int32_t F, int32_t N,
                         int halves, float *dW_first, float *dW_second, float *dbias, hipStream_t stream);

// Single-operand transforms (dense layer; GCN products).  row_scale (may be NULL) multiplies output row v by
// row_scale[v]; bias may be NULL.
//   fwd:        Y = act(X W + b)  or  diag(row_scale) (X W); N_out >= F_out columns are written (at most F_out
//               rounded up to 8, only without bias), zeros past F_out
//   bwd data:   dX = [diag(row_scale)] dZ W^T,   dZ = dY (.) act'(Y)
//   bwd weight: dW = X^T dZ,  dbias = 1^T dZ (skipped when NULL)
int launch_dense_gemm_fwd(int64_t n, const void *X, int64_t ldx, int32_t F_in, const float *W, const float *bias,
                          const float *row_scale, int32_t F_out, int32_t N_out, int32_t act, int32_t dtype, void *Y,
                          int64_t ldy, hipStream_t s);
int launch_dense_gemm_bwd_data(int64_t n, const void *dY, const void *Y, int64_t ld, const float *W, int32_t F_in,
                               int32_t F_out, int32_t act, int32_t dtype, const float *row_scale, void *dX,
                               int64_t ldx, hipStream_t s);
size_t dense_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out);
int launch_dense_gemm_bwd_weight(int64_t n, const void *X, int64_t ldx, const void *dY, const void *Y, int64_t ld,
                                 int32_t F_in, int32_t F_out, int32_t act, int32_t dtype, float *dW, float *dbias,
                                 void *ws, size_t ws_bytes, hipStream_t s);

// prefix_out[i] = values[0] + ... + values[i-1] for i <= n (n + 1 outputs).  ws: exclusive_scan_i32_workspace_bytes(n).
size_t exclusive_scan_i32_workspace_bytes(int64_t n);
int launch_exclusive_scan_i32(int64_t n, const int32_t *values, int32_t *prefix_out, void *ws, hipStream_t s);

// out[j] = sum over b < nb of partial[b * width + j], j < F, in a fixed order (nb = 0 writes zeros).
int launch_sum_partials(int nb, int width, int F, const float *partial, float *out, hipStream_t stream);

// sorted[range r] = unsorted[range r] in ascending order, for the n ranges of rowptr (distinct numbers per range).
// queue: n int32 of scratch; counter: one int32 that is zero on entry.
int launch_sort_lists(int64_t n, const int32_t *rowptr, const int32_t *unsorted, int32_t *sorted, int32_t *queue,
                      int32_t *counter, hipStream_t s);

}  // namespace tma
