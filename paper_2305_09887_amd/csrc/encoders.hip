// Entry points of the paper's other encoders (Sec. 4.1, paragraph on GNN
// encoders): the graph convolution of Kipf & Welling on the local subgraph and
// the dense layer of the graph-agnostic MLP encoder (also a layer of the link
// decoder).  Sequencing plus two small row-wise kernels; the products run in the
// matrix-core template, the aggregation in the streaming gather.
//
// GCN layer:   Ahat = S (A + I) S,  S = diag((d_v + 1)^-1/2).  The gather runs on the narrower side.
// Transform first (F_out < F_in):
//   forward   Y = S (H W)                               (product, rows scaled in its epilogue)
//             H' = act(S (A + I) Y + b)                 (gather: sum of neighbour rows + own row, scaled)
//   backward  dZ = dH' (.) act'(H'),  db = 1^T dZ,  Q = S dZ        (one row-wise pass)
//             G = S (A + I)^T Q  = Ahat^T dZ            (gather over the transposed graph)
//             dW = H^T G,   dH = G W^T                  (products)
// Aggregate first (F_out >= F_in):
//   forward   M = S (A + I) S H                         (gather with a weight per neighbour), H' = act(M W + b)
//   backward  dW = M^T dZ, db = 1^T dZ                  (mask applied while loading; no gather for a first layer)
//             dH = S (A + I)^T (S dZ W^T)               (product with scaled rows, then the gather)
#include "kernels.hpp"

namespace tma {

static size_t elem_size(int32_t dtype) { return dtype == TMA_BF16 ? 2 : 4; }
static int pad_cols(int32_t F, int32_t dtype) { return int(round_up(size_t(F), dtype == TMA_BF16 ? 8 : 4)); }

__device__ __forceinline__ float load1(const float *p) { return *p; }
__device__ __forceinline__ float load1(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store1(float *p, float v) { *p = v; }
__device__ __forceinline__ void store1(uint16_t *p, float v) { *p = f32_to_bf16(v); }

__global__ __launch_bounds__(256) void gcn_norm_kernel(int64_t n, const int32_t *__restrict__ rowptr,
                                                       float *__restrict__ s)
{
    const int64_t v = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (v < n) s[v] = 1.0f / sqrtf(float(rowptr[v + 1] - rowptr[v]) + 1.0f);
}

// dst_v = s_v * (g_v (.) [h_v > 0]) on rows of F elements (columns F .. F_pad-1 of dst are zeroed), and the
// column sums of the unscaled masked rows, one partial row of F_pad sums per block.  A row is cut into units
// (16-byte chunks with kVec, single elements otherwise); `tpr` threads share a row, 256 / tpr rows run side by
// side.  kVec needs F == F_pad.
template <typename T, bool kVec>
__global__ __launch_bounds__(256) void scale_mask_colsum_kernel(int64_t n, int F, int F_pad, const T *__restrict__ g,
                                                                const T *__restrict__ h, int64_t ld,
                                                                const float *__restrict__ s, int relu,
                                                                T *__restrict__ dst, int64_t ld_dst,
                                                                float *__restrict__ partial, int64_t rows_per_block,
                                                                int tpr)
{
    constexpr int E = kVec ? Chunk<T>::kElems : 1;
    __shared__ float red[256 * E];
    const int units = F_pad / E;
    const int rp = 256 / tpr;
    const int sub = threadIdx.x % tpr, rl = threadIdx.x / tpr;
    const bool live = rl < rp;
    const int64_t r0 = int64_t(blockIdx.x) * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block) < n ? (r0 + rows_per_block) : n;
    for (int u0 = 0; u0 < units; u0 += tpr) {
        const int u = u0 + sub;
        float cs[E];
#pragma unroll
        for (int i = 0; i < E; ++i) cs[i] = 0.0f;
        if (live && u < units) {
            for (int64_t v = r0 + rl; v < r1; v += rp) {
                const float sv = s[v];
                float x[E];
                if constexpr (kVec) {
                    Chunk<T>::load(g + v * ld + u * E, x);
                    if (relu) {
                        float y[E];
                        Chunk<T>::load(h + v * ld + u * E, y);
#pragma unroll
                        for (int i = 0; i < E; ++i) x[i] = y[i] > 0.0f ? x[i] : 0.0f;
                    }
                } else {
                    x[0] = 0.0f;
                    if (u < F) {
                        x[0] = load1(g + v * ld + u);
                        if (relu && !(load1(h + v * ld + u) > 0.0f)) x[0] = 0.0f;
                    }
                }
                float out[E];
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    cs[i] += x[i];
                    out[i] = x[i] * sv;
                }
                if constexpr (kVec) Chunk<T>::store(dst + v * ld_dst + u * E, out);
                else store1(dst + v * ld_dst + u, out[0]);
            }
        }
#pragma unroll
        for (int i = 0; i < E; ++i) red[threadIdx.x * E + i] = cs[i];
        __syncthreads();
        if (rl == 0 && u < units) {
#pragma unroll
            for (int i = 0; i < E; ++i) {
                float t = 0.0f;
                for (int q = 0; q < rp; ++q) t += red[(q * tpr + sub) * E + i];   // fixed order
                partial[int64_t(blockIdx.x) * F_pad + u * E + i] = t;
            }
        }
        __syncthreads();
    }
}

// out[j] = sum over b < nb of partial[b][j], j < F (rows of `width` floats), fixed order: 16 columns per
// block, 16 slices of the blocks each, combined in slice order.
__global__ __launch_bounds__(256) void sum_partials_kernel(int nb, int width, int F, const float *__restrict__ partial,
                                                           float *__restrict__ out)
{
    __shared__ float part[16][16];
    const int c = threadIdx.x % 16, slice = threadIdx.x / 16;
    const int j = blockIdx.x * 16 + c;
    const int per = (nb + 15) / 16;
    const int b0 = slice * per;
    const int b1 = (b0 + per) < nb ? (b0 + per) : nb;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    if (j < F) {
        int b = b0;
        for (; b + 3 < b1; b += 4) {
            s0 += partial[int64_t(b) * width + j];
            s1 += partial[int64_t(b + 1) * width + j];
            s2 += partial[int64_t(b + 2) * width + j];
            s3 += partial[int64_t(b + 3) * width + j];
        }
        for (; b < b1; ++b) s0 += partial[int64_t(b) * width + j];
    }
    part[slice][c] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (slice == 0 && j < F) {
        float t = 0.0f;
        for (int k = 0; k < 16; ++k) t += part[k][c];
        out[j] = t;
    }
}

int launch_sum_partials(int nb, int width, int F, const float *partial, float *out, hipStream_t stream)
{
    if (F <= 0) return TMA_OK;
    TMA_TIMED("sum_partials", stream);
    hipLaunchKernelGGL(sum_partials_kernel, dim3(unsigned(ceil_div(F, 16))), dim3(256), 0, stream, nb, width, F, partial,
                       out);
    return check_launch("sum_partials");
}

constexpr int kColsumMaxBlocks = 1024;

struct ColsumPlan {
    bool vec;
    int tpr;
    int64_t blocks, rows_per_block;
};

static ColsumPlan plan_colsum(int64_t n, int F, int F_pad, size_t elem, bool vec_ok)
{
    ColsumPlan p;
    const int E = int(16 / elem);
    p.vec = vec_ok && F == F_pad && F % E == 0;
    const int units = p.vec ? F_pad / E : F_pad;
    p.tpr = units < 256 ? (units > 0 ? units : 1) : 256;
    const int rp = 256 / p.tpr;
    int64_t blocks = ceil_div(n > 0 ? n : 1, int64_t(rp) * 8);
    if (blocks > kColsumMaxBlocks) blocks = kColsumMaxBlocks;
    p.rows_per_block = ceil_div(n > 0 ? n : 1, blocks);
    p.blocks = ceil_div(n > 0 ? n : 1, p.rows_per_block);
    return p;
}

// Order of the two halves of the layer.  Aggregating first gathers F_in-wide rows and needs no gather at all
// in the backward of a first layer, nor a pass over dZ of its own; transforming first gathers F_out-wide rows.
// The layer transforms first only when the padded F_out is smaller than F_in, which also makes the caller's
// [n, F_in] state buffer large enough for either form.
static bool gcn_aggregates_first(int32_t F_in, int32_t F_out, int32_t dtype) { return pad_cols(F_out, dtype) >= F_in; }

struct GcnBwdWorkspace {
    size_t grad_bytes;     // transform first: Q and G, [n, Fp] each; aggregate first: S (dZ W^T), [n, F_in]
    size_t colsum_bytes;   // per-block column sums (transform first)
    size_t weight_bytes;   // split partials of dW
    size_t total() const { return grad_bytes + colsum_bytes + weight_bytes; }
};

static GcnBwdWorkspace plan_gcn_bwd(int64_t n, int32_t F_in, int32_t F_out, int32_t dtype, bool need_dH)
{
    GcnBwdWorkspace w;
    const size_t rows = size_t(n > 0 ? n : 1);
    if (gcn_aggregates_first(F_in, F_out, dtype)) {
        w.grad_bytes = need_dH ? round_up(rows * size_t(F_in) * elem_size(dtype), 256) : 0;
        w.colsum_bytes = 0;
    } else {
        const int Fp = pad_cols(F_out, dtype);
        w.grad_bytes = 2 * round_up(rows * size_t(Fp) * elem_size(dtype), 256);
        w.colsum_bytes = round_up(size_t(kColsumMaxBlocks) * size_t(Fp) * 4, 256);
    }
    w.weight_bytes = dense_gemm_bwd_weight_workspace_bytes(n, F_in, F_out);
    return w;
}

template <typename T>
static int scale_mask_colsum(int64_t n, int F, int Fp, const T *g, const T *h, int64_t ld, const float *s, bool relu,
                             T *dst, float *partial, float *dbias, hipStream_t stream)
{
    const bool vec_ok = aligned(g, 16) && (size_t(ld) * sizeof(T)) % 16 == 0 && (!relu || aligned(h, 16)) && aligned(dst, 16);
    const ColsumPlan p = plan_colsum(n, F, Fp, sizeof(T), vec_ok);
    if (n > 0) {
        TMA_TIMED("scale_mask_colsum", stream);
        if (p.vec)
            hipLaunchKernelGGL((scale_mask_colsum_kernel<T, true>), dim3(unsigned(p.blocks)), dim3(256), 0, stream, n, F,
                               Fp, g, h, ld, s, relu ? 1 : 0, dst, int64_t(Fp), partial, p.rows_per_block, p.tpr);
        else
            hipLaunchKernelGGL((scale_mask_colsum_kernel<T, false>), dim3(unsigned(p.blocks)), dim3(256), 0, stream, n, F,
                               Fp, g, h, ld, s, relu ? 1 : 0, dst, int64_t(Fp), partial, p.rows_per_block, p.tpr);
        if (int rc = check_launch("scale_mask_colsum")) return rc;
    }
    return launch_sum_partials(n > 0 ? int(p.blocks) : 0, Fp, F, partial, dbias, stream);
}

}  // namespace tma

extern "C" int tma_gcn_norm(int64_t n, const int32_t *rowptr, float *s_out, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_gcn_norm";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n outside [0, 2^31)", fn);
    if (n == 0) return TMA_OK;
    TMA_REQUIRE(rowptr && s_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    hipStream_t s = as_stream(stream);
    TMA_TIMED("gcn_norm", s);
    hipLaunchKernelGGL(gcn_norm_kernel, dim3(unsigned(ceil_div(n, 256))), dim3(256), 0, s, n, rowptr, s_out);
    return check_launch(fn);
}

extern "C" int tma_gcn_layer_aggregates_first(int32_t F_in, int32_t F_out, int32_t dtype)
{
    return tma::gcn_aggregates_first(F_in, F_out, dtype) ? 1 : 0;
}

extern "C" int tma_gcn_layer_fwd(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *s_norm,
                                 const void *H, int64_t ldh, int32_t F_in, const float *W, const float *bias,
                                 int32_t F_out, int32_t act, int32_t dtype, void *M_out, void *Hnext_out,
                                 int64_t ld_next, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_gcn_layer_fwd";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n outside [0, 2^31)", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n == 0) return TMA_OK;
    TMA_REQUIRE(rowptr && s_norm && H && W && bias && M_out && Hnext_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    TMA_REQUIRE(ldh >= F_in && ld_next >= F_out, TMA_ERR_BAD_SHAPE, "%s: ldh < F_in or ld_next < F_out", fn);
    TMA_REQUIRE(aligned(M_out, 16), TMA_ERR_INVALID_ARG, "%s: M_out must be 16-byte aligned", fn);
    TMA_REQUIRE(H != M_out, TMA_ERR_INVALID_ARG, "%s: M_out must not alias H", fn);
    hipStream_t s = as_stream(stream);
    if (gcn_aggregates_first(F_in, F_out, dtype)) {
        // M = S (A + I) S H in one pass over H: neighbours and the own row weighted by s, the sum scaled by s_v
        if (int rc = launch_spmm_combine(n, rowptr, colidx, s_norm, H, ldh, F_in, dtype, M_out, F_in, false, H, ldh,
                                         nullptr, F_in, false, true, s_norm, s))
            return rc;
        return launch_dense_gemm_fwd(n, M_out, F_in, F_in, W, bias, nullptr, F_out, F_out, act, dtype, Hnext_out, ld_next,
                                     s);
    }
    const int Fp = pad_cols(F_out, dtype);   // Fp < F_in: Y = S (H W) fits into the state buffer as [n, Fp]
    if (int rc = launch_dense_gemm_fwd(n, H, ldh, F_in, W, nullptr, s_norm, F_out, Fp, TMA_ACT_NONE, dtype, M_out, Fp, s))
        return rc;
    // whole padded rows when the output has room for them (vector path); its padding columns receive zeros
    const int F_rows = ld_next >= Fp ? Fp : F_out;
    return launch_spmm_combine(n, rowptr, colidx, s_norm, M_out, Fp, F_rows, dtype, Hnext_out, ld_next, false, M_out, Fp,
                               bias, F_out, act == TMA_ACT_RELU, true, nullptr, s);
}

extern "C" size_t tma_gcn_layer_bwd_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out, int32_t dtype,
                                                    int32_t need_dH)
{
    if (n < 0 || F_in < 1 || F_out < 1) return 0;
    return tma::plan_gcn_bwd(n, F_in, F_out, dtype, need_dH != 0).total();
}

extern "C" int tma_gcn_layer_bwd(int64_t n, const int32_t *rowptr_T, const int32_t *colidx_T, const float *s_norm,
                                 const void *H, int64_t ldh, const void *M, const void *Hnext, const void *dHnext,
                                 int64_t ld_next, const float *W, int32_t F_in, int32_t F_out, int32_t act,
                                 int32_t dtype, float *dW, float *dbias, void *dH_out, void *ws, size_t ws_bytes,
                                 tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_gcn_layer_bwd";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n outside [0, 2^31)", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(dW && dbias, TMA_ERR_INVALID_ARG, "%s: gradient output is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    const bool need_dH = dH_out != nullptr;
    const bool agg_first = gcn_aggregates_first(F_in, F_out, dtype);
    const GcnBwdWorkspace w = plan_gcn_bwd(n, F_in, F_out, dtype, need_dH);
    TMA_REQUIRE(ws_bytes >= w.total(), TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, ws_bytes,
                w.total());
    if (n > 0) {
        TMA_REQUIRE(s_norm && dHnext && W && (agg_first ? M != nullptr : H != nullptr), TMA_ERR_INVALID_ARG,
                    "%s: NULL argument", fn);
        TMA_REQUIRE(act == TMA_ACT_NONE || Hnext, TMA_ERR_INVALID_ARG, "%s: Hnext is required with ReLU", fn);
        TMA_REQUIRE((agg_first && !need_dH) || rowptr_T, TMA_ERR_INVALID_ARG, "%s: graph is NULL", fn);
        TMA_REQUIRE(ldh >= F_in && ld_next >= F_out, TMA_ERR_BAD_SHAPE, "%s: ldh < F_in or ld_next < F_out", fn);
    }
    hipStream_t s = as_stream(stream);
    char *base = static_cast<char *>(ws);
    void *wws = base + w.grad_bytes + w.colsum_bytes;
    int rc;
    if (agg_first) {
        // dW = M^T dZ, db = 1^T dZ;  dH = S (A + I)^T (S dZ W^T): product with its rows scaled, then the gather
        if ((rc = launch_dense_gemm_bwd_weight(n, M, F_in, dHnext, Hnext, ld_next, F_in, F_out, act, dtype, dW, dbias, wws,
                                               w.weight_bytes, s)))
            return rc;
        if (!need_dH || n == 0) return TMA_OK;
        void *P = base;
        if ((rc = launch_dense_gemm_bwd_data(n, dHnext, Hnext, ld_next, W, F_in, F_out, act, dtype, s_norm, P, F_in, s)))
            return rc;
        return launch_spmm_combine(n, rowptr_T, colidx_T, s_norm, P, F_in, F_in, dtype, dH_out, ldh, false, P, F_in,
                                   nullptr, F_in, false, true, nullptr, s);
    }
    const int Fp = pad_cols(F_out, dtype);
    void *Q = base;
    void *G = base + w.grad_bytes / 2;
    float *colsum = reinterpret_cast<float *>(base + w.grad_bytes);
    const bool relu = act == TMA_ACT_RELU;
    if (dtype == TMA_F32)
        rc = scale_mask_colsum<float>(n, F_out, Fp, static_cast<const float *>(dHnext), static_cast<const float *>(Hnext),
                                      ld_next, s_norm, relu, static_cast<float *>(Q), colsum, dbias, s);
    else
        rc = scale_mask_colsum<uint16_t>(n, F_out, Fp, static_cast<const uint16_t *>(dHnext),
                                         static_cast<const uint16_t *>(Hnext), ld_next, s_norm, relu,
                                         static_cast<uint16_t *>(Q), colsum, dbias, s);
    if (rc) return rc;
    if ((rc = launch_spmm_combine(n, rowptr_T, colidx_T, s_norm, Q, Fp, Fp, dtype, G, Fp, false, Q, Fp, nullptr, Fp, false,
                                  true, nullptr, s)))
        return rc;
    if ((rc = launch_dense_gemm_bwd_weight(n, H, ldh, G, nullptr, Fp, F_in, F_out, TMA_ACT_NONE, dtype, dW, nullptr, wws,
                                           w.weight_bytes, s)))
        return rc;
    if (!need_dH || n == 0) return TMA_OK;
    return launch_dense_gemm_bwd_data(n, G, nullptr, Fp, W, F_in, F_out, TMA_ACT_NONE, dtype, nullptr, dH_out, ldh, s);
}

extern "C" int tma_dense_fwd(int64_t n, const void *X, int64_t ldx, int32_t F_in, const float *W, const float *bias,
                             int32_t F_out, int32_t act, int32_t dtype, void *Y_out, int64_t ldy, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_dense_fwd";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n outside [0, 2^31)", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n == 0) return TMA_OK;
    TMA_REQUIRE(X && W && Y_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    TMA_REQUIRE(ldx >= F_in && ldy >= F_out, TMA_ERR_BAD_SHAPE, "%s: ldx < F_in or ldy < F_out", fn);
    return launch_dense_gemm_fwd(n, X, ldx, F_in, W, bias, nullptr, F_out, F_out, act, dtype, Y_out, ldy,
                                 as_stream(stream));
}

extern "C" size_t tma_dense_bwd_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out)
{
    if (n < 0 || F_in < 1 || F_out < 1) return 0;
    return tma::dense_gemm_bwd_weight_workspace_bytes(n, F_in, F_out);
}

extern "C" int tma_dense_bwd(int64_t n, const void *X, int64_t ldx, const void *Y, const void *dY, int64_t ldy,
                             const float *W, int32_t F_in, int32_t F_out, int32_t act, int32_t dtype, float *dW,
                             float *dbias, void *dX_out, int64_t ld_dx, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_dense_bwd";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n outside [0, 2^31)", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(dW, TMA_ERR_INVALID_ARG, "%s: dW is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    if (n > 0) {
        TMA_REQUIRE(X && dY && W, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
        TMA_REQUIRE(act == TMA_ACT_NONE || Y, TMA_ERR_INVALID_ARG, "%s: Y is required with ReLU", fn);
        TMA_REQUIRE(ldx >= F_in && ldy >= F_out && (!dX_out || ld_dx >= F_in), TMA_ERR_BAD_SHAPE,
                    "%s: leading dimension smaller than the row", fn);
    }
    hipStream_t s = as_stream(stream);
    if (int rc = launch_dense_gemm_bwd_weight(n, X, ldx, dY, Y, ldy, F_in, F_out, act, dtype, dW, dbias, ws, ws_bytes, s))
        return rc;
    if (!dX_out || n == 0) return TMA_OK;
    return launch_dense_gemm_bwd_data(n, dY, Y, ldy, W, F_in, F_out, act, dtype, nullptr, dX_out, ld_dx, s);
}
