// Entry points of one mean-aggregation GraphSAGE layer (forward / backward).
// Sequencing only: aggregation kernel, then the MFMA transform; all on the
// caller's stream, no allocation, no synchronisation.
#include "kernels.hpp"

namespace tma {

static size_t elem_size(int32_t dtype) { return dtype == TMA_BF16 ? 2 : 4; }

struct BwdWorkspace {
    size_t dm_bytes;      // D^-1 dM  [n, F_in]
    size_t weight_bytes;  // split partials
    size_t total() const { return dm_bytes + weight_bytes; }
};

// Order of the two halves of a layer.  Aggregating first costs a gather of F_in-wide rows, transforming
// first a gather of F_out-wide rows; the products cost the same either way.  The transform-first form is
// taken when its two padded output blocks fit into the [n, F_in] buffer the caller provides for saved
// state (M_out), i.e. when F_out is at most about half of F_in (the last layer of the models here).
static int pad_cols(int32_t F_out, int32_t dtype) { return int(round_up(size_t(F_out), dtype == TMA_BF16 ? 8 : 4)); }
static bool aggregates_first(int32_t F_in, int32_t F_out, int32_t dtype) { return 2 * pad_cols(F_out, dtype) > F_in; }

static BwdWorkspace plan_bwd(int64_t n, int32_t F_in, int32_t F_out, int32_t dtype, bool need_dH)
{
    BwdWorkspace w;
    const size_t rows = size_t(n > 0 ? n : 1);
    if (aggregates_first(F_in, F_out, dtype)) {
        w.dm_bytes = need_dH ? round_up(rows * size_t(F_in) * elem_size(dtype), 256) : 0;
        w.weight_bytes = sage_gemm_bwd_weight_workspace_bytes(n, F_in, F_out);
    } else {  // scaled dZ and dYn, [n, Fp] each
        w.dm_bytes = 2 * round_up(rows * size_t(pad_cols(F_out, dtype)) * elem_size(dtype), 256);
        w.weight_bytes = sage_tf_gemm_bwd_weight_workspace_bytes(n, F_in, F_out, dtype);
    }
    return w;
}

// Wt_bf16 (may be NULL): the weights as tma_sage_prepare_weights_bf16 leaves them, for the bf16 aggregate-first form
static int sage_layer_fwd(const char *fn, int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg,
                          const void *H, int64_t ldh, int32_t F_in, const float *W_self, const float *W_neigh,
                          const float *bias, int32_t F_out, int32_t act, int32_t dtype, void *M_out, int64_t ldm,
                          void *Hnext_out, int64_t ld_next, const void *Wt_bf16, tma_stream_t stream)
{
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n outside [0, 2^31)", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n == 0) return TMA_OK;
    TMA_REQUIRE(rowptr && inv_deg && H && W_self && W_neigh && bias && M_out && Hnext_out, TMA_ERR_INVALID_ARG,
                "%s: NULL argument", fn);
    TMA_REQUIRE(ldh >= F_in && ldm >= F_in && ld_next >= F_out, TMA_ERR_BAD_SHAPE,
                "%s: ldh < F_in, ldm < F_in or ld_next < F_out", fn);
    hipStream_t s = as_stream(stream);
    if (aggregates_first(F_in, F_out, dtype)) {
        if (int rc = launch_spmm(n, rowptr, colidx, inv_deg, H, ldh, F_in, dtype, M_out, ldm, false, s)) return rc;
        return launch_sage_gemm_fwd(n, H, ldh, M_out, ldm, F_in, W_self, W_neigh, bias, F_out, act, dtype, Hnext_out,
                                    ld_next, s, Wt_bf16);
    }
    // transform first: [Y_self | Y_neigh] = H [W_self | W_neigh] into the M_out buffer, then
    // Hnext = act(Y_self + Abar Y_neigh + b) by the gather kernel.  Needs ld_next >= the padded width.
    const int Fp = pad_cols(F_out, dtype);
    char *scratch = static_cast<char *>(M_out);
    void *Ys = scratch;
    void *Yn = scratch + size_t(n) * size_t(Fp) * elem_size(dtype);
    TMA_REQUIRE(aligned(M_out, 16), TMA_ERR_INVALID_ARG, "%s: M_out must be 16-byte aligned", fn);
    if (int rc = launch_sage_tf_gemm_fwd(n, H, ldh, F_in, W_self, W_neigh, F_out, dtype, Ys, Yn, Fp, s)) return rc;
    if (ld_next >= Fp)   // whole padded rows (vector path); the padding columns of Hnext receive zeros
        return launch_spmm_combine(n, rowptr, colidx, inv_deg, Yn, Fp, Fp, dtype, Hnext_out, ld_next, false, Ys, Fp,
                                   bias, F_out, act == TMA_ACT_RELU, false, nullptr, s);
    return launch_spmm_combine(n, rowptr, colidx, inv_deg, Yn, Fp, F_out, dtype, Hnext_out, ld_next, false, Ys, Fp,
                               bias, F_out, act == TMA_ACT_RELU, false, nullptr, s);
}

}  // namespace tma

extern "C" int tma_sage_layer_fwd(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg,
                                  const void *H, int64_t ldh, int32_t F_in, const float *W_self,
                                  const float *W_neigh, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                                  void *M_out, int64_t ldm, void *Hnext_out, int64_t ld_next, tma_stream_t stream)
{
    return tma::sage_layer_fwd("tma_sage_layer_fwd", n, rowptr, colidx, inv_deg, H, ldh, F_in, W_self, W_neigh, bias, F_out,
                               act, dtype, M_out, ldm, Hnext_out, ld_next, nullptr, stream);
}

extern "C" size_t tma_sage_weights_bf16_bytes(int32_t F_in, int32_t F_out)
{
    if (F_in < 1 || F_out < 1) return 0;
    return tma::sage_weights_bf16_bytes(F_in, F_out);
}

extern "C" int tma_sage_prepare_weights_bf16(const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out,
                                             void *Wt_out, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_sage_prepare_weights_bf16";
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(W_self && W_neigh && Wt_out && aligned(Wt_out, 16), TMA_ERR_INVALID_ARG,
                "%s: NULL argument, or Wt_out not 16-byte aligned", fn);
    return launch_sage_prepare_weights_bf16(W_self, W_neigh, F_in, F_out, Wt_out, as_stream(stream));
}

extern "C" int tma_sage_layer_fwd_prepared(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg,
                                           const void *H, int64_t ldh, int32_t F_in, const float *W_self,
                                           const float *W_neigh, const float *bias, int32_t F_out, int32_t act,
                                           int32_t dtype, void *M_out, int64_t ldm, void *Hnext_out, int64_t ld_next,
                                           const void *Wt_bf16, tma_stream_t stream)
{
    const char *fn = "tma_sage_layer_fwd_prepared";
    TMA_REQUIRE(dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: prepared weights belong to bf16 storage (dtype %d)", fn,
                dtype);
    TMA_REQUIRE(Wt_bf16 && tma::aligned(Wt_bf16, 16), TMA_ERR_INVALID_ARG, "%s: Wt_bf16 is NULL or not 16-byte aligned", fn);
    return tma::sage_layer_fwd(fn, n, rowptr, colidx, inv_deg, H, ldh, F_in, W_self, W_neigh, bias, F_out, act, dtype,
                               M_out, ldm, Hnext_out, ld_next, Wt_bf16, stream);
}

extern "C" int tma_sage_layer_aggregates_first(int32_t F_in, int32_t F_out, int32_t dtype)
{
    return tma::aggregates_first(F_in, F_out, dtype) ? 1 : 0;
}

extern "C" size_t tma_sage_layer_bwd_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out, int32_t dtype,
                                                     int32_t need_dH)
{
    if (n < 0 || F_in < 1 || F_out < 1) return 0;
    return tma::plan_bwd(n, F_in, F_out, dtype, need_dH != 0).total();
}

extern "C" int tma_sage_layer_bwd(int64_t n, const int32_t *rowptr_T, const int32_t *colidx_T, const float *inv_deg,
                                  const void *H, int64_t ldh, const void *M, int64_t ldm, const void *Hnext,
                                  const void *dHnext, int64_t ld_next, const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out, int32_t act,
                                  int32_t dtype, float *dW_self, float *dW_neigh, float *dbias, void *dH_out, void *ws,
                                  size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_sage_layer_bwd";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n outside [0, 2^31)", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(dW_self && dW_neigh && dbias, TMA_ERR_INVALID_ARG, "%s: gradient output is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    const bool need_dH = dH_out != nullptr;
    const BwdWorkspace w = plan_bwd(n, F_in, F_out, dtype, need_dH);
    TMA_REQUIRE(ws_bytes >= w.total(), TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, ws_bytes,
                w.total());
    const bool agg_first = aggregates_first(F_in, F_out, dtype);
    if (n > 0) {
        TMA_REQUIRE(H && (M || !agg_first) && dHnext && W_self && W_neigh, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
        TMA_REQUIRE(act == TMA_ACT_NONE || Hnext, TMA_ERR_INVALID_ARG, "%s: Hnext is required with ReLU", fn);
        TMA_REQUIRE(!need_dH || (rowptr_T && inv_deg), TMA_ERR_INVALID_ARG, "%s: graph is NULL", fn);
        TMA_REQUIRE(ldh >= F_in && ld_next >= F_out && (!agg_first || ldm >= F_in), TMA_ERR_BAD_SHAPE,
                    "%s: ldh < F_in, ldm < F_in or ld_next < F_out", fn);
    }
    hipStream_t s = as_stream(stream);
    char *base = static_cast<char *>(ws);
    void *dMs = base;
    void *wws = base + w.dm_bytes;

    if (!agg_first) {
        // transform-first form: dYn = Abar^T dZ as a gather of the inv_deg-scaled, masked dZ over the transposed
        // graph; then the two products with [dZ | dYn]
        TMA_REQUIRE(n == 0 || (rowptr_T && inv_deg), TMA_ERR_INVALID_ARG, "%s: graph is NULL", fn);
        const int Fp = pad_cols(F_out, dtype);
        void *dZs = base;
        void *dYn = base + w.dm_bytes / 2;
        if (int rc = launch_scale_mask_rows(n, F_out, Fp, dHnext, Hnext, ld_next, inv_deg, act == TMA_ACT_RELU, dtype,
                                            dZs, Fp, s))
            return rc;
        if (int rc = launch_spmm(n, rowptr_T, colidx_T, nullptr, dZs, Fp, Fp, dtype, dYn, Fp, false, s)) return rc;
        if (int rc = launch_sage_tf_gemm_bwd_weight(n, H, ldh, dHnext, Hnext, ld_next, dYn, Fp, F_in, F_out, act, dtype,
                                                    dW_self, dW_neigh, dbias, wws, w.weight_bytes, s))
            return rc;
        if (!need_dH || n == 0) return TMA_OK;
        return launch_sage_tf_gemm_bwd_data(n, dHnext, Hnext, ld_next, dYn, Fp, W_self, W_neigh, F_in, F_out, act,
                                            dtype, dH_out, ldh, s);
    }
    if (int rc = launch_sage_gemm_bwd_weight(n, H, ldh, M, ldm, dHnext, Hnext, ld_next, F_in, F_out, act, dtype, dW_self,
                                             dW_neigh, dbias, wws, w.weight_bytes, s))
        return rc;
    if (!need_dH || n == 0) return TMA_OK;
    // dH = dZ W_self^T  (written by the transform)  +  A^T (D^-1 dZ W_neigh^T)  (gathered on top of it)
    if (int rc = launch_sage_gemm_bwd_data(n, dHnext, Hnext, ld_next, inv_deg, W_self, W_neigh, F_in, F_out, act, dtype,
                                           dH_out, ldh, dMs, s))
        return rc;
    return launch_spmm(n, rowptr_T, colidx_T, nullptr, dMs, F_in, F_in, dtype, dH_out, ldh, true, s);
}
