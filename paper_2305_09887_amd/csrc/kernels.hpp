// Internal launch interface between the translation units of libtma.
#pragma once

#include "common.hpp"

namespace tma {

// Row gather-reduce over a CSR:  out_v = scale_v * sum_{u in row v} in_u  (+ out_v when accumulate).
// scale_v = inv_deg[v] when inv_deg != nullptr, else 1.  fp32 accumulation in neighbour order.
int launch_spmm(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                int64_t ld_in, int32_t F, int32_t dtype, void *out, int64_t ld_out, bool accumulate,
                hipStream_t stream);

// Z = [H | M] [W_self ; W_neigh] + b ;  Hnext = act(Z)
int launch_sage_gemm_fwd(int64_t n, const void *H, int64_t ldh, const void *M, int32_t F_in, const float *W_self,
                         const float *W_neigh, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                         void *Hnext, int64_t ld_next, hipStream_t stream);

// [dH_self | inv_deg * dM] = dZ [W_self^T | W_neigh^T],  dZ = dHnext (.) act'(Hnext)
int launch_sage_gemm_bwd_data(int64_t n, const void *dHnext, const void *Hnext, int64_t ld_next,
                              const float *inv_deg, const float *W_self, const float *W_neigh, int32_t F_in,
                              int32_t F_out, int32_t act, int32_t dtype, void *dH_self_out, int64_t ldh,
                              void *dM_scaled_out, hipStream_t stream);

// [dW_self ; dW_neigh] = [H | M]^T dZ,  dbias = 1^T dZ   (split over nodes, two-stage fixed-order reduction)
size_t sage_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out);
int launch_sage_gemm_bwd_weight(int64_t n, const void *H, int64_t ldh, const void *M, const void *dHnext,
                                const void *Hnext, int64_t ld_next, int32_t F_in, int32_t F_out, int32_t act,
                                int32_t dtype,
                                float *dW_self, float *dW_neigh, float *dbias, void *ws, size_t ws_bytes,
                                hipStream_t stream);

}  // namespace tma
