// Single-operand transforms on the matrix cores: the dense layer Y = act(X W + b)
// of the graph-agnostic MLP encoder and of the link decoder, and the products of
// the GCN layer (paper Sec. 4.1, paragraphs on GNN encoders and on the link
// prediction decoder; App., formulation of the MLP decoder):
//   forward   Y = act(X W + b)            or   Y = diag(s) (X W)      (GCN, before the aggregation)
//   backward  dX = dZ W^T                 or   dX = diag(s) (dZ W^T)
//             dW = X^T dZ,  db = 1^T dZ,       dZ = dY (.) act'(Y)
// Same kernel template as the GraphSAGE transforms; the operand views that
// present concatenations there are used here with the first part only.
#include "gemm_core.hpp"

namespace tma {

template <typename T, bool kRowScale>
struct DenseEpilogue {  // out = act(acc + b)  or  row_scale[row] * acc
    static constexpr bool kColAux = true, kRowAux = kRowScale;
    T *out;
    int64_t ld;
    const float *bias;       // may be NULL
    const float *row_scale;  // read only with kRowScale
    bool relu;
    __device__ __forceinline__ float col_aux(int col) const { return bias ? bias[col] : 0.0f; }
    __device__ __forceinline__ float row_aux(int64_t row) const { return kRowScale ? row_scale[row] : 0.0f; }
    __device__ __forceinline__ float value(float v, float caux, float raux, int) const
    {
        v += caux;
        if (kRowScale) v *= raux;
        if (relu) v = v > 0.0f ? v : 0.0f;
        return v;
    }
    __device__ __forceinline__ void store(int64_t row, int col, float v, int) const { narrow1(out + row * ld + col, v); }
    static constexpr bool kPairs = sizeof(T) == 2;
    __device__ __forceinline__ bool pairs_ok() const { return ld % 2 == 0 && word_aligned(out); }
    __device__ __forceinline__ T *at(int64_t row, int col) const { return out + row * ld + col; }
};

static int pad8(int32_t F) { return int(round_up(size_t(F), 8)); }

// ---- forward ----------------------------------------------------------------
// N_out >= F_out columns are written; those past F_out receive zeros (the weight view is zero there)
template <typename T, bool kRowScale>
static int dense_fwd_typed(int64_t n, const T *X, int64_t ldx, int32_t F_in, const float *W, const float *bias,
                           const float *row_scale, int32_t F_out, int32_t N_out, bool relu, T *Y, int64_t ldy,
                           hipStream_t s)
{
    DenseEpilogue<T, kRowScale> e{Y, ldy, bias, row_scale, relu};
    const int64_t K = F_in, kps = int64_t(round_up(size_t(K), 32));
    // a group of four along k must not reach into row padding, nor a group of four columns past F_out
    const bool va = vec4_ok(X, ldx) && F_in % 4 == 0;
    const bool vb = F_out % 4 == 0 && aligned(W, 16);
    const char *name = kname<T>("gemm_dense_fwd", "gemm_dense_fwd_generic", "gemm_dense_fwd_bf16",
                                "gemm_dense_fwd_bf16_generic", va);
#define TMA_DENSE_FWD(VA_, VB_)                                                               \
    do {                                                                                      \
        CatRows<T, VA_> a{X, ldx, X, ldx, F_in, n, F_in};                                          \
        SideWeights<VB_> b{W, W, F_in, F_out, pad8(F_out)};                                   \
        launch_by_width<T, 32, false>(name, a, b, e, n, N_out, K, kps, 1, nullptr, s);        \
    } while (0)
    // (va: F_in is a multiple of four, so W holds at least four elements and may be read in unaligned groups)
    if (va && vb) TMA_DENSE_FWD(true, kAligned4);
    else if (va) TMA_DENSE_FWD(true, kUnaligned4);
    else TMA_DENSE_FWD(false, kElementwise);
#undef TMA_DENSE_FWD
    return check_launch("dense gemm fwd");
}

int launch_dense_gemm_fwd(int64_t n, const void *X, int64_t ldx, int32_t F_in, const float *W, const float *bias,
                          const float *row_scale, int32_t F_out, int32_t N_out, int32_t act, int32_t dtype, void *Y,
                          int64_t ldy, hipStream_t s)
{
    if (n == 0 || F_out == 0) return TMA_OK;
    if (N_out < F_out || N_out > pad8(F_out) || (bias && N_out != F_out))
        return fail(TMA_ERR_BAD_SHAPE, "dense gemm fwd: %d output columns for F_out = %d", N_out, F_out);
    const bool relu = act == TMA_ACT_RELU;
    if (dtype == TMA_F32) {
        const float *x = static_cast<const float *>(X);
        float *y = static_cast<float *>(Y);
        return row_scale ? dense_fwd_typed<float, true>(n, x, ldx, F_in, W, bias, row_scale, F_out, N_out, relu, y, ldy, s)
                         : dense_fwd_typed<float, false>(n, x, ldx, F_in, W, bias, row_scale, F_out, N_out, relu, y, ldy, s);
    }
    if (dtype == TMA_BF16) {
        const uint16_t *x = static_cast<const uint16_t *>(X);
        uint16_t *y = static_cast<uint16_t *>(Y);
        return row_scale ? dense_fwd_typed<uint16_t, true>(n, x, ldx, F_in, W, bias, row_scale, F_out, N_out, relu, y, ldy, s)
                         : dense_fwd_typed<uint16_t, false>(n, x, ldx, F_in, W, bias, row_scale, F_out, N_out, relu, y, ldy, s);
    }
    return fail(TMA_ERR_UNSUPPORTED_DTYPE, "dense gemm fwd: dtype %d", dtype);
}

// ---- backward: data ---------------------------------------------------------
template <typename T, bool kRowScale, bool kRelu>
static int dense_bwd_data_typed(int64_t n, const T *g, const T *h, int64_t ld, const float *W, int32_t F_in,
                                int32_t F_out, const float *row_scale, T *dX, int64_t ldx, hipStream_t s)
{
    DenseEpilogue<T, kRowScale> e{dX, ldx, nullptr, row_scale, false};
    const int64_t K = F_out, kps = int64_t(round_up(size_t(K), 32));
    const bool va = vec4_ok(g, ld) && (!kRelu || vec4_ok(h, ld));
    const bool vb = vec4_ok(W, F_out);
    const char *name = kname<T>("gemm_dense_bwd_data", "gemm_dense_bwd_data_generic", "gemm_dense_bwd_data_bf16",
                                "gemm_dense_bwd_data_bf16_generic", va);
#define TMA_DENSE_BD(VA_, VB_)                                                                \
    do {                                                                                      \
        MaskedGrad<true, T, VA_, kRelu> a{g, h, F_out, ld, n};                                \
        CatWeightsT<VB_> b{W, W, F_in, F_out};                                                \
        launch_by_width<T, 32, false>(name, a, b, e, n, F_in, K, kps, 1, nullptr, s);         \
    } while (0)
    if (va && vb) TMA_DENSE_BD(true, true);
    else if (va) TMA_DENSE_BD(true, false);
    else TMA_DENSE_BD(false, false);
#undef TMA_DENSE_BD
    return check_launch("dense gemm bwd data");
}

template <typename T>
static int dense_bwd_data_any(int64_t n, const void *dY, const void *Y, int64_t ld, const float *W, int32_t F_in,
                              int32_t F_out, bool relu, const float *row_scale, void *dX, int64_t ldx, hipStream_t s)
{
    const T *g = static_cast<const T *>(dY);
    const T *h = static_cast<const T *>(Y);
    T *d = static_cast<T *>(dX);
    if (row_scale)
        return relu ? dense_bwd_data_typed<T, true, true>(n, g, h, ld, W, F_in, F_out, row_scale, d, ldx, s)
                    : dense_bwd_data_typed<T, true, false>(n, g, h, ld, W, F_in, F_out, row_scale, d, ldx, s);
    return relu ? dense_bwd_data_typed<T, false, true>(n, g, h, ld, W, F_in, F_out, row_scale, d, ldx, s)
                : dense_bwd_data_typed<T, false, false>(n, g, h, ld, W, F_in, F_out, row_scale, d, ldx, s);
}

int launch_dense_gemm_bwd_data(int64_t n, const void *dY, const void *Y, int64_t ld, const float *W, int32_t F_in,
                               int32_t F_out, int32_t act, int32_t dtype, const float *row_scale, void *dX,
                               int64_t ldx, hipStream_t s)
{
    if (n == 0 || F_in == 0) return TMA_OK;
    const bool relu = act == TMA_ACT_RELU;
    if (dtype == TMA_F32) return dense_bwd_data_any<float>(n, dY, Y, ld, W, F_in, F_out, relu, row_scale, dX, ldx, s);
    if (dtype == TMA_BF16)
        return dense_bwd_data_any<uint16_t>(n, dY, Y, ld, W, F_in, F_out, relu, row_scale, dX, ldx, s);
    return fail(TMA_ERR_UNSUPPORTED_DTYPE, "dense gemm bwd data: dtype %d", dtype);
}

// ---- backward: weights ------------------------------------------------------
static WeightSplit plan_dense_weight_split(int64_t n, int32_t F_in, int32_t F_out)
{
    const int bn = F_out <= 64 ? 64 : (F_out <= 96 ? 96 : 128);
    const int64_t tiles = ceil_div(int64_t(F_in), 128) * ceil_div(F_out, bn);
    int64_t want = ceil_div(512, tiles > 0 ? tiles : 1);
    const int64_t max_useful = ceil_div(n > 0 ? n : 1, 128);
    if (want > max_useful) want = max_useful;
    if (want < 1) want = 1;
    WeightSplit w;
    w.k_per_split = int64_t(round_up(size_t(ceil_div(n > 0 ? n : 1, want)), 32));
    w.n_splits = int(ceil_div(n > 0 ? n : 1, w.k_per_split));
    w.partial_bytes = round_up(size_t(w.n_splits) * size_t(F_in) * size_t(F_out) * 4, 256);
    w.colsum_bytes = round_up(size_t(w.n_splits) * size_t(F_out) * 4, 256);
    return w;
}

size_t dense_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out)
{
    const WeightSplit w = plan_dense_weight_split(n, F_in, F_out);
    return w.partial_bytes + w.colsum_bytes;
}

template <typename T, bool kRelu>
static int dense_bwd_weight_typed(int64_t n, const T *X, int64_t ldx, const T *g, const T *h, int64_t ld, int32_t F_in,
                                  int32_t F_out, const WeightSplit &w, float *partial, float *colsum, hipStream_t s)
{
    SplitEpilogue e{partial, int64_t(F_in), F_out};
    const bool v = vec4_ok(X, ldx) && F_in % 4 == 0 && vec4_ok(g, ld) && (!kRelu || vec4_ok(h, ld));
    const char *name = kname<T>("gemm_dense_bwd_weight", "gemm_dense_bwd_weight_generic", "gemm_dense_bwd_weight_bf16",
                                "gemm_dense_bwd_weight_bf16_generic", v);
    if (v) {
        CatRowsT<T, true> a{X, ldx, X, ldx, F_in, n};
        MaskedGrad<false, T, true, kRelu> b{g, h, F_out, ld, n};
        launch_by_width<T, 32, true>(name, a, b, e, int64_t(F_in), F_out, n, w.k_per_split, w.n_splits, colsum, s);
    } else {
        CatRowsT<T, false> a{X, ldx, X, ldx, F_in, n};
        MaskedGrad<false, T, false, kRelu> b{g, h, F_out, ld, n};
        launch_by_width<T, 32, true>(name, a, b, e, int64_t(F_in), F_out, n, w.k_per_split, w.n_splits, colsum, s);
    }
    return check_launch("dense gemm bwd weight");
}

int launch_dense_gemm_bwd_weight(int64_t n, const void *X, int64_t ldx, const void *dY, const void *Y, int64_t ld,
                                 int32_t F_in, int32_t F_out, int32_t act, int32_t dtype, float *dW, float *dbias,
                                 void *ws, size_t ws_bytes, hipStream_t s)
{
    if (dtype != TMA_F32 && dtype != TMA_BF16)
        return fail(TMA_ERR_UNSUPPORTED_DTYPE, "dense gemm bwd weight: dtype %d", dtype);
    if (F_out == 0 || F_in == 0) return TMA_OK;
    const WeightSplit w = plan_dense_weight_split(n, F_in, F_out);
    if (ws_bytes < w.partial_bytes + w.colsum_bytes)
        return fail(TMA_ERR_WORKSPACE_TOO_SMALL, "dense gemm bwd weight: workspace %zu < %zu", ws_bytes,
                    w.partial_bytes + w.colsum_bytes);
    float *partial = static_cast<float *>(ws);
    float *colsum = reinterpret_cast<float *>(static_cast<char *>(ws) + w.partial_bytes);
    const bool relu = act == TMA_ACT_RELU;
    // without rows there is nothing to multiply (the operands may be NULL); the second stage writes zeros
    if (n > 0) {
        int rc;
        if (dtype == TMA_F32) {
            const float *x = static_cast<const float *>(X), *g = static_cast<const float *>(dY),
                        *h = static_cast<const float *>(Y);
            rc = relu ? dense_bwd_weight_typed<float, true>(n, x, ldx, g, h, ld, F_in, F_out, w, partial, colsum, s)
                      : dense_bwd_weight_typed<float, false>(n, x, ldx, g, h, ld, F_in, F_out, w, partial, colsum, s);
        } else {
            const uint16_t *x = static_cast<const uint16_t *>(X), *g = static_cast<const uint16_t *>(dY),
                           *h = static_cast<const uint16_t *>(Y);
            rc = relu ? dense_bwd_weight_typed<uint16_t, true>(n, x, ldx, g, h, ld, F_in, F_out, w, partial, colsum, s)
                      : dense_bwd_weight_typed<uint16_t, false>(n, x, ldx, g, h, ld, F_in, F_out, w, partial, colsum, s);
        }
        if (rc) return rc;
    }
    return launch_reduce_splits(partial, colsum, n > 0 ? w.n_splits : 0, F_in, F_out, 1, dW, nullptr, dbias, s);
}

}  // namespace tma
