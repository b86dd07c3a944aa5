// Dense per-layer transform of the mean-aggregation GraphSAGE layer and its
// gradients, on the matrix cores (the only MFMA-bound part of the path):
//   forward   Z = [H | M] [W_self ; W_neigh] + b,  H' = act(Z)
//   backward  [dH_self | D^-1 dM] = dZ [W_self^T | W_neigh^T]
//             [dW_self ; dW_neigh] = [H | M]^T dZ,   db = 1^T dZ
// with dZ = dH' (.) act'(Z) formed while loading (chain rule as in the proof of
// the paper's Thm. 1).
//
// The products run in the tile kernel template of gemm_core.hpp (fp32 storage: fp32 MFMA, so the 1e-4 parity
// bound holds without any reduced-precision pass; bf16 storage: bf16 MFMA with fp32 accumulation); this file
// holds the operand / epilogue combinations of the GraphSAGE layer, the split planning of the weight gradient
// and its fixed-order second stage.
#include "gemm_core.hpp"

namespace tma {

// Second stage of the split reduction, fixed order.  A block owns 16 groups of four
// consecutive outputs; its 16 lanes-by-split slices each add up 1/16 of the splits (all
// their 16-byte loads in flight together), then the slices are combined in slice order
// through LDS.
constexpr int kRedCols = 16;    // float4 columns per block
constexpr int kRedSlices = 16;  // split slices per block

__global__ __launch_bounds__(256) void reduce_splits_kernel(const float *__restrict__ partial,
                                                            const float *__restrict__ colsum_partial, int n_splits,
                                                            int F, int N, int halves, float *__restrict__ dW_self,
                                                            float *__restrict__ dW_neigh, float *__restrict__ dbias)
{
    __shared__ float4 part[kRedSlices][kRedCols];
    const int64_t total = int64_t(halves) * F * N;      // weight-gradient entries; then N bias entries
    const int64_t total_all = total + N;
    const int col = threadIdx.x % kRedCols, q = threadIdx.x / kRedCols;
    const int64_t e0 = (int64_t(blockIdx.x) * kRedCols + col) * 4;
    const int per = (n_splits + kRedSlices - 1) / kRedSlices;
    const int s_begin = q * per, s_end = (s_begin + per < n_splits) ? s_begin + per : n_splits;
    float4 s = zero4();
    if (e0 < total_all) {
        const bool vec = (e0 + 3 < total) && (total % 4 == 0);
        if (vec) {
#pragma unroll 8
            for (int sp = s_begin; sp < s_end; ++sp) {
                const float4 v = *reinterpret_cast<const float4 *>(partial + int64_t(sp) * total + e0);
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            }
        } else {
            float t[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int sp = s_begin; sp < s_end; ++sp)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int64_t e = e0 + c;
                    if (e < total) t[c] += partial[int64_t(sp) * total + e];
                    else if (e < total_all) t[c] += colsum_partial[int64_t(sp) * N + (e - total)];
                }
            s = make_float4(t[0], t[1], t[2], t[3]);
        }
    }
    part[q][col] = s;
    __syncthreads();
    if (q == 0 && e0 < total_all) {
        float r[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int w = 0; w < kRedSlices; ++w) {
            const float4 v = part[w][col];
            r[0] += v.x; r[1] += v.y; r[2] += v.z; r[3] += v.w;
        }
        const int64_t half = int64_t(F) * N;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t e = e0 + c;
            if (e < half) dW_self[e] = r[c];
            else if (e < total) dW_neigh[e - half] = r[c];
            else if (e < total_all && dbias) dbias[e - total] = r[c];
        }
    }
}

// Split reduction for the transform-first form: partial is [splits][F][2*Fp]; column c of the left half
// goes to dW_self[:, c], of the right half to dW_neigh[:, c]; the column sums of the left half are dbias.
__global__ __launch_bounds__(256) void reduce_splits_halves_kernel(const float *__restrict__ partial,
                                                                   const float *__restrict__ colsum_partial,
                                                                   int n_splits, int F, int Fo, int Fp,
                                                                   float *__restrict__ dW_self,
                                                                   float *__restrict__ dW_neigh,
                                                                   float *__restrict__ dbias)
{
    __shared__ float part[kRedSlices][kRedCols];
    const int N = 2 * Fp;
    const int64_t total = int64_t(F) * N;
    const int64_t total_all = total + N;
    const int col = threadIdx.x % kRedCols, q = threadIdx.x / kRedCols;
    const int64_t e = int64_t(blockIdx.x) * kRedCols + col;
    const int per = (n_splits + kRedSlices - 1) / kRedSlices;
    const int s_begin = q * per, s_end = (s_begin + per < n_splits) ? s_begin + per : n_splits;
    float s = 0.0f;
    if (e < total) {
#pragma unroll 8
        for (int sp = s_begin; sp < s_end; ++sp) s += partial[int64_t(sp) * total + e];
    } else if (e < total_all) {
        for (int sp = s_begin; sp < s_end; ++sp) s += colsum_partial[int64_t(sp) * N + (e - total)];
    }
    part[q][col] = s;
    __syncthreads();
    if (q == 0 && e < total_all) {
        float r = 0.0f;
#pragma unroll
        for (int w = 0; w < kRedSlices; ++w) r += part[w][col];
        if (e < total) {
            const int64_t m = e / N;
            const int c = int(e - m * N);
            const bool second = c >= Fp;
            const int cc = c - (second ? Fp : 0);
            if (cc < Fo) (second ? dW_neigh : dW_self)[m * Fo + cc] = r;
        } else {
            const int c = int(e - total);
            if (c < Fo) dbias[c] = r;
        }
    }
}

int launch_reduce_splits(const float *partial, const float *colsum_partial, int n_splits, int32_t F, int32_t N,
                         int halves, float *dW_first, float *dW_second, float *dbias, hipStream_t stream)
{
    const int64_t total_all = int64_t(halves) * F * N + N;
    TMA_TIMED("reduce_splits", stream);
    hipLaunchKernelGGL(reduce_splits_kernel, dim3(unsigned(ceil_div(total_all, 4 * kRedCols))), dim3(256), 0, stream,
                       partial, colsum_partial, n_splits, F, N, halves, dW_first, dW_second, dbias);
    return check_launch("split reduce");
}

#ifndef TMA_GEMM_WIDE_BF16
#define TMA_GEMM_WIDE_BF16 1
#endif
constexpr bool kWideBf16 = TMA_GEMM_WIDE_BF16 != 0;
#ifndef TMA_GEMM_WIDE_BWD_DATA
#define TMA_GEMM_WIDE_BWD_DATA 1
#endif
constexpr bool kWideBwdData = TMA_GEMM_WIDE_BWD_DATA != 0;

// ---- forward ----------------------------------------------------------------
template <typename T, bool VA, class AL, class BL>
static void fwd_launch(const AL &a, const BL &b, const FwdEpilogue<T> &e, int64_t n, int F_out, int64_t K, int64_t kps,
                       hipStream_t s)
{
    if (F_out <= 64 || few_tiles(n, F_out))
        launch_gemm<128, 64, 32, 4, 1, false, T>(kname<T>("gemm_fwd_128x64", "gemm_fwd_128x64_generic", "gemm_fwd_128x64_bf16", "gemm_fwd_128x64_bf16_generic", VA),
                                              a, b, e, n, F_out, K, kps, 1, nullptr, s);
    else if constexpr (kWideBf16 && sizeof(T) == 2 && VA) {
        // bf16 storage: the product is bound by streaming [H | M]; a tile as wide as the output reads it once
        if (F_out > 128 && F_out <= 256)
            launch_gemm<128, 256, 32, 2, 4, false, T>("gemm_fwd_128x256_bf16", a, b, e, n, F_out, K, kps, 1, nullptr, s);
        else
            launch_gemm<128, 128, 32, 2, 2, false, T>("gemm_fwd_128x128_bf16", a, b, e, n, F_out, K, kps, 1, nullptr, s);
    } else
        launch_gemm<128, 128, (sizeof(T) == 2 ? 32 : 16), 2, 2, false, T>(kname<T>("gemm_fwd_128x128", "gemm_fwd_128x128_generic", "gemm_fwd_128x128_bf16", "gemm_fwd_128x128_bf16_generic", VA),
                                               a, b, e, n, F_out, K, kps, 1, nullptr, s);
}

template <typename T, bool VA, bool VB>
static void fwd_dispatch(int64_t n, const T *H, int64_t ldh, const T *M, int64_t ldm, int F_in, const float *W_self,
                         const float *W_neigh, const FwdEpilogue<T> &e, int F_out, hipStream_t s)
{
    CatRows<T, VA> a{H, ldh, M, ldm, F_in, n, 2 * F_in};
    const int64_t K = 2 * int64_t(F_in);
    const int64_t kps = int64_t(round_up(size_t(K), 32));
    CatWeights<VB> b{W_self, W_neigh, F_in, F_out};
    fwd_launch<T, VA>(a, b, e, n, F_out, K, kps, s);
}

// bf16 storage with the weights prepared as Wt[o][k] (bf16): both operands are rows of packed bf16, contiguous
// along k, and go into LDS as loaded -- no conversion, no 2-byte fragment reads of a [k][n] weight tile.
static void fwd_prepared(int64_t n, const uint16_t *H, int64_t ldh, const uint16_t *M, int64_t ldm, int F_in,
                         const uint16_t *Wt, const FwdEpilogue<uint16_t> &e, int F_out, hipStream_t s)
{
    CatRows<uint16_t, true> a{H, ldh, M, ldm, F_in, n, 2 * F_in};
    CatRows<uint16_t, true> b{Wt, 2 * int64_t(F_in), Wt, 2 * int64_t(F_in), 2 * F_in, F_out, 2 * F_in};
    const int64_t K = 2 * int64_t(F_in);
    fwd_launch<uint16_t, true>(a, b, e, n, F_out, K, int64_t(round_up(size_t(K), 32)), s);
}

__global__ __launch_bounds__(256) void narrow_transpose_weights_kernel(const float *__restrict__ Ws,
                                                                       const float *__restrict__ Wn, int F, int N,
                                                                       uint16_t *__restrict__ Wt)
{
    const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;   // over [2F][N]: coalesced reads
    if (idx >= 2 * int64_t(F) * N) return;
    const int k = int(idx / N), o = int(idx - int64_t(k) * N);
    const float v = k < F ? Ws[int64_t(k) * N + o] : Wn[int64_t(k - F) * N + o];
    Wt[int64_t(o) * 2 * F + k] = f32_to_bf16(v);
}

size_t sage_weights_bf16_bytes(int32_t F_in, int32_t F_out)
{
    return round_up(2 * size_t(F_in) * size_t(F_out) * sizeof(uint16_t), 256);
}

int launch_sage_prepare_weights_bf16(const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out, void *Wt_out,
                                     hipStream_t stream)
{
    const int64_t total = 2 * int64_t(F_in) * F_out;
    TMA_TIMED("prepare_weights_bf16", stream);
    hipLaunchKernelGGL(narrow_transpose_weights_kernel, dim3(unsigned(ceil_div(total, 256))), dim3(256), 0, stream, W_self,
                       W_neigh, F_in, F_out, static_cast<uint16_t *>(Wt_out));
    return check_launch("prepare weights");
}

template <typename T>
static int fwd_typed(int64_t n, const T *H, int64_t ldh, const T *M, int64_t ldm, int32_t F_in, const float *W_self,
                     const float *W_neigh, const float *bias, int32_t F_out, int32_t act, T *Hnext, int64_t ld_next,
                     hipStream_t stream)
{
    FwdEpilogue<T> e{Hnext, ld_next, bias, act == TMA_ACT_RELU};
    const bool va = vec4_ok(H, ldh) && vec4_ok(M, ldm) && F_in % 4 == 0;
    const bool vb = vec4_ok(W_self, F_out) && vec4_ok(W_neigh, F_out);
    if (va && vb) fwd_dispatch<T, true, true>(n, H, ldh, M, ldm, F_in, W_self, W_neigh, e, F_out, stream);
    else if (va) fwd_dispatch<T, true, false>(n, H, ldh, M, ldm, F_in, W_self, W_neigh, e, F_out, stream);
    else if (vb) fwd_dispatch<T, false, true>(n, H, ldh, M, ldm, F_in, W_self, W_neigh, e, F_out, stream);
    else fwd_dispatch<T, false, false>(n, H, ldh, M, ldm, F_in, W_self, W_neigh, e, F_out, stream);
    return check_launch("sage gemm fwd");
}

int launch_sage_gemm_fwd(int64_t n, const void *H, int64_t ldh, const void *M, int64_t ldm, int32_t F_in, const float *W_self,
                         const float *W_neigh, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                         void *Hnext, int64_t ld_next, hipStream_t stream, const void *Wt_bf16)
{
    if (n == 0 || F_out == 0) return TMA_OK;
    if (Wt_bf16 && dtype == TMA_BF16) {
        const uint16_t *h = static_cast<const uint16_t *>(H), *m = static_cast<const uint16_t *>(M);
        // the packed path needs groups of four bf16 at 8-byte aligned addresses in both operands
        if (vec4_ok(h, ldh) && vec4_ok(m, ldm) && F_in % 4 == 0 && aligned(Wt_bf16, 8)) {
            FwdEpilogue<uint16_t> e{static_cast<uint16_t *>(Hnext), ld_next, bias, act == TMA_ACT_RELU};
            fwd_prepared(n, h, ldh, m, ldm, F_in, static_cast<const uint16_t *>(Wt_bf16), e, F_out, stream);
            return check_launch("sage gemm fwd");
        }
    }
    if (dtype == TMA_F32)
        return fwd_typed<float>(n, static_cast<const float *>(H), ldh, static_cast<const float *>(M), ldm, F_in, W_self,
                                W_neigh, bias, F_out, act, static_cast<float *>(Hnext), ld_next, stream);
    if (dtype == TMA_BF16)
        return fwd_typed<uint16_t>(n, static_cast<const uint16_t *>(H), ldh, static_cast<const uint16_t *>(M), ldm, F_in,
                                   W_self, W_neigh, bias, F_out, act, static_cast<uint16_t *>(Hnext), ld_next, stream);
    return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm fwd: dtype %d", dtype);
}

// ---- backward: data ---------------------------------------------------------
template <typename T, bool VA, bool VB, bool kRelu>
static void bwd_data_dispatch(int64_t n, const T *g, const T *h, int64_t ld_next, const float *W_self,
                              const float *W_neigh, int F_in, int F_out, const BwdDataEpilogue<T> &e, hipStream_t s)
{
    MaskedGrad<true, T, VA, kRelu> a{g, h, F_out, ld_next, n};
    CatWeightsT<VB> b{W_self, W_neigh, F_in, F_out};
    const int N = 2 * F_in;
    const int64_t K = F_out;
    const char *name = kname<T>("gemm_bwd_data_128x128", "gemm_bwd_data_128x128_generic", "gemm_bwd_data_128x128_bf16",
                                "gemm_bwd_data_128x128_bf16_generic", VA);
    if (few_tiles(n, N)) {
        const char *narrow = kname<T>("gemm_bwd_data_128x64", "gemm_bwd_data_128x64_generic", "gemm_bwd_data_128x64_bf16",
                                      "gemm_bwd_data_128x64_bf16_generic", VA);
        launch_gemm<128, 64, 32, 4, 1, false, T>(narrow, a, b, e, n, N, K, int64_t(round_up(size_t(K), 32)), 1, nullptr, s);
    } else if (kWideBwdData && sizeof(T) == 2 && VA && N >= 256 && K > 48) {
        if constexpr (kWideBwdData && sizeof(T) == 2 && VA)   // bf16 storage: half as many passes over the gradient rows
            launch_gemm<128, 256, 32, 2, 4, false, T>("gemm_bwd_data_128x256_bf16", a, b, e, n, N, K,
                                                      int64_t(round_up(size_t(K), 32)), 1, nullptr, s);
    } else if (K <= 48) {  // short reduction: 16-wide slabs waste less of the last one
        const int64_t kps = int64_t(round_up(size_t(K), 16));
        launch_gemm<128, 128, 16, 2, 2, false, T>(name, a, b, e, n, N, K, kps, 1, nullptr, s);
    } else {
        const int64_t kps = int64_t(round_up(size_t(K), 32));
        launch_gemm<128, 128, 32, 2, 2, false, T>(name, a, b, e, n, N, K, kps, 1, nullptr, s);
    }
}

template <typename T>
static int bwd_data_typed(int64_t n, const T *g, const T *h, int64_t ld_next, const float *inv_deg,
                          const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out, int32_t act,
                          T *dH_self_out, int64_t ldh, T *dM_scaled_out, hipStream_t stream)
{
    const bool relu = act == TMA_ACT_RELU;
    BwdDataEpilogue<T> e{dH_self_out, ldh, dM_scaled_out, inv_deg, F_in};
    const bool va = vec4_ok(g, ld_next) && (!relu || vec4_ok(h, ld_next));
    const bool vb = vec4_ok(W_self, F_out) && vec4_ok(W_neigh, F_out);
#define TMA_BWD_DATA(VA_, VB_)                                                                                    \
    (relu ? bwd_data_dispatch<T, VA_, VB_, true>(n, g, h, ld_next, W_self, W_neigh, F_in, F_out, e, stream)       \
          : bwd_data_dispatch<T, VA_, VB_, false>(n, g, h, ld_next, W_self, W_neigh, F_in, F_out, e, stream))
    if (va && vb) TMA_BWD_DATA(true, true);
    else if (va) TMA_BWD_DATA(true, false);
    else if (vb) TMA_BWD_DATA(false, true);
    else TMA_BWD_DATA(false, false);
#undef TMA_BWD_DATA
    return check_launch("sage gemm bwd data");
}

int launch_sage_gemm_bwd_data(int64_t n, const void *dHnext, const void *Hnext, int64_t ld_next,
                              const float *inv_deg, const float *W_self, const float *W_neigh, int32_t F_in,
                              int32_t F_out, int32_t act, int32_t dtype, void *dH_self_out, int64_t ldh,
                              void *dM_scaled_out, hipStream_t stream)
{
    if (n == 0 || F_in == 0) return TMA_OK;
    if (dtype == TMA_F32)
        return bwd_data_typed<float>(n, static_cast<const float *>(dHnext), static_cast<const float *>(Hnext), ld_next,
                                     inv_deg, W_self, W_neigh, F_in, F_out, act, static_cast<float *>(dH_self_out),
                                     ldh, static_cast<float *>(dM_scaled_out), stream);
    if (dtype == TMA_BF16)
        return bwd_data_typed<uint16_t>(n, static_cast<const uint16_t *>(dHnext), static_cast<const uint16_t *>(Hnext),
                                        ld_next, inv_deg, W_self, W_neigh, F_in, F_out, act,
                                        static_cast<uint16_t *>(dH_self_out), ldh,
                                        static_cast<uint16_t *>(dM_scaled_out), stream);
    return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm bwd: dtype %d", dtype);
}

// ---- backward: weights ------------------------------------------------------

// wide: 256 x 256 tiles (bf16 storage with F_out > 128: the product is bound by streaming its two operands, which
// 128 x 128 tiles read two and four times: 54 GB instead of 16 GB per launch on a 12.5 M-row part); fewer tiles then
// need more splits to fill the chip, capped so that the partial results stay under a quarter of the operands'
// bytes.  Below some 4e5 rows that cap leaves too few work items and the narrow tiles are faster (95 vs 109 us at
// 125 k rows), above it the wide ones are (2 M rows: 1.17 -> 0.73 ms for 128 -> 256, 2.47 -> 1.42 ms for 256 -> 256).
static bool wide_weight_tiles(int64_t n, int32_t F_in, int32_t F_out, int elem_bytes)
{
    return kWideBf16 && elem_bytes == 2 && F_out > 128 && F_out <= 256 && F_in >= 128 && n >= 400000;
}

static WeightSplit plan_weight_split(int64_t n, int32_t F_in, int32_t F_out, bool wide = false)
{
    const int bn = wide ? 256 : (F_out <= 64 ? 64 : 128);
    const int64_t tiles = ceil_div(2 * int64_t(F_in), wide ? 256 : 128) * ceil_div(F_out, bn);
    int64_t want = ceil_div(512, tiles > 0 ? tiles : 1);
    const int64_t max_useful = ceil_div(n > 0 ? n : 1, 128);
    if (want > max_useful) want = max_useful;
    if (wide) {
        const int64_t cap = (n > 0 ? n : 1) * (2 * int64_t(F_in) + F_out) * 2 / 4 / (2 * int64_t(F_in) * F_out * 4);
        if (want > cap) want = cap;
    }
    if (want < 1) want = 1;
    WeightSplit w;
    w.k_per_split = int64_t(round_up(size_t(ceil_div(n > 0 ? n : 1, want)), 32));
    w.n_splits = int(ceil_div(n > 0 ? n : 1, w.k_per_split));
    w.partial_bytes = round_up(size_t(w.n_splits) * 2 * size_t(F_in) * size_t(F_out) * 4, 256);
    w.colsum_bytes = round_up(size_t(w.n_splits) * size_t(F_out) * 4, 256);
    return w;
}

size_t sage_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out)
{
    const WeightSplit w = plan_weight_split(n, F_in, F_out);
    size_t bytes = w.partial_bytes + w.colsum_bytes;
    if (wide_weight_tiles(n, F_in, F_out, 2)) {   // the query does not know the storage type: room for either plan
        const WeightSplit v = plan_weight_split(n, F_in, F_out, true);
        if (v.partial_bytes + v.colsum_bytes > bytes) bytes = v.partial_bytes + v.colsum_bytes;
    }
    return bytes;
}

template <typename T, bool VA, bool VB, bool kRelu>
static void bwd_weight_dispatch(int64_t n, const T *H, int64_t ldh, const T *M, int64_t ldm, const T *g, const T *h,
                                int64_t ld_next, int F_in, int F_out, const WeightSplit &w, const SplitEpilogue &e,
                                float *colsum, hipStream_t s)
{
    constexpr bool V = VA && VB;
    CatRowsT<T, VA> a{H, ldh, M, ldm, F_in, n};
    MaskedGrad<false, T, VB, kRelu> b{g, h, F_out, ld_next, n};
    const int64_t Mtot = 2 * int64_t(F_in);
    if (F_out <= 64)
        launch_gemm<128, 64, 32, 4, 1, true, T>(kname<T>("gemm_bwd_weight_128x64", "gemm_bwd_weight_128x64_generic", "gemm_bwd_weight_128x64_bf16", "gemm_bwd_weight_128x64_bf16_generic", V),
                                             a, b, e, Mtot, F_out, n, w.k_per_split, w.n_splits, colsum, s);
    else if constexpr (kWideBf16 && sizeof(T) == 2 && V) {
        if (wide_weight_tiles(n, F_in, F_out, 2))
            launch_gemm<256, 256, 32, 4, 2, true, T>("gemm_bwd_weight_256x256_bf16", a, b, e, Mtot, F_out, n, w.k_per_split,
                                                     w.n_splits, colsum, s);
        else
            launch_gemm<128, 128, 32, 2, 2, true, T>("gemm_bwd_weight_128x128_bf16", a, b, e, Mtot, F_out, n, w.k_per_split,
                                                     w.n_splits, colsum, s);
    } else
        launch_gemm<128, 128, (sizeof(T) == 2 ? 32 : 16), 2, 2, true, T>(kname<T>("gemm_bwd_weight_128x128", "gemm_bwd_weight_128x128_generic", "gemm_bwd_weight_128x128_bf16", "gemm_bwd_weight_128x128_bf16_generic", V),
                                              a, b, e, Mtot, F_out, n, w.k_per_split, w.n_splits, colsum, s);
}

template <typename T>
static int bwd_weight_typed(int64_t n, const T *H, int64_t ldh, const T *M, int64_t ldm, const T *g, const T *h, int64_t ld_next,
                            int32_t F_in, int32_t F_out, int32_t act, const WeightSplit &w, const SplitEpilogue &e,
                            float *colsum, hipStream_t stream)
{
    const bool relu = act == TMA_ACT_RELU;
    const bool va = vec4_ok(H, ldh) && vec4_ok(M, ldm) && F_in % 4 == 0;
    const bool vb = vec4_ok(g, ld_next) && (!relu || vec4_ok(h, ld_next));
#define TMA_BWD_WEIGHT(VA_, VB_)                                                                                           \
    (relu ? bwd_weight_dispatch<T, VA_, VB_, true>(n, H, ldh, M, ldm, g, h, ld_next, F_in, F_out, w, e, colsum, stream)         \
          : bwd_weight_dispatch<T, VA_, VB_, false>(n, H, ldh, M, ldm, g, h, ld_next, F_in, F_out, w, e, colsum, stream))
    if (va && vb) TMA_BWD_WEIGHT(true, true);
    else if (va) TMA_BWD_WEIGHT(true, false);
    else if (vb) TMA_BWD_WEIGHT(false, true);
    else TMA_BWD_WEIGHT(false, false);
#undef TMA_BWD_WEIGHT
    return check_launch("sage gemm bwd weight");
}

int launch_sage_gemm_bwd_weight(int64_t n, const void *H, int64_t ldh, const void *M, int64_t ldm, const void *dHnext,
                                const void *Hnext, int64_t ld_next, int32_t F_in, int32_t F_out, int32_t act,
                                int32_t dtype, float *dW_self, float *dW_neigh, float *dbias, void *ws, size_t ws_bytes,
                                hipStream_t stream)
{
    if (dtype != TMA_F32 && dtype != TMA_BF16) return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm bwd: dtype %d", dtype);
    if (F_out == 0) return TMA_OK;
    const bool relu_ = act == TMA_ACT_RELU;
    const bool all_vec = dtype == TMA_BF16 && vec4_ok(static_cast<const uint16_t *>(H), ldh) &&
                         vec4_ok(static_cast<const uint16_t *>(M), ldm) && F_in % 4 == 0 &&
                         vec4_ok(static_cast<const uint16_t *>(dHnext), ld_next) &&
                         (!relu_ || vec4_ok(static_cast<const uint16_t *>(Hnext), ld_next));
    const WeightSplit w = plan_weight_split(n, F_in, F_out, all_vec && wide_weight_tiles(n, F_in, F_out, 2));
    if (ws_bytes < w.partial_bytes + w.colsum_bytes)
        return fail(TMA_ERR_WORKSPACE_TOO_SMALL, "sage gemm bwd weight: workspace %zu < %zu", ws_bytes,
                    w.partial_bytes + w.colsum_bytes);
    float *partial = static_cast<float *>(ws);
    float *colsum = reinterpret_cast<float *>(static_cast<char *>(ws) + w.partial_bytes);
    const int64_t Mtot = 2 * int64_t(F_in);
    SplitEpilogue e{partial, Mtot, F_out};
    // An empty node set leaves nothing to multiply: the operands may then be NULL, and the kernel's clamped
    // loads would have no valid row to fall back to.  The second stage alone writes the zero gradients.
    const bool have_rows = F_in > 0 && n > 0;
    if (have_rows) {
        int rc;
        if (dtype == TMA_F32)
            rc = bwd_weight_typed<float>(n, static_cast<const float *>(H), ldh, static_cast<const float *>(M), ldm,
                                         static_cast<const float *>(dHnext), static_cast<const float *>(Hnext), ld_next,
                                         F_in, F_out, act, w, e, colsum, stream);
        else
            rc = bwd_weight_typed<uint16_t>(n, static_cast<const uint16_t *>(H), ldh, static_cast<const uint16_t *>(M), ldm,
                                            static_cast<const uint16_t *>(dHnext),
                                            static_cast<const uint16_t *>(Hnext), ld_next, F_in, F_out, act, w, e,
                                            colsum, stream);
        if (rc) return rc;
    }
    return launch_reduce_splits(partial, colsum, have_rows ? w.n_splits : 0, F_in, F_out, 2, dW_self, dW_neigh, dbias,
                                stream);
}

// ---- transform-before-aggregate form -----------------------------------------
static int pad_cols(int32_t F_out, int32_t dtype) { return int(round_up(size_t(F_out), dtype == TMA_BF16 ? 8 : 4)); }


template <typename T>
static int tf_fwd_typed(int64_t n, const T *H, int64_t ldh, int32_t F_in, const float *W_self, const float *W_neigh,
                        int32_t F_out, int Fp, T *Ys, T *Yn, int64_t ldy, hipStream_t s)
{
    HalvesEpilogue<T> e{Ys, Yn, ldy, Fp};
    const int64_t K = F_in, kps = int64_t(round_up(size_t(K), 32));
    const bool va = vec4_ok(H, ldh);
    const bool vb = F_out % 4 == 0 && aligned(W_self, 16) && aligned(W_neigh, 16);
    TMA_REQUIRE(vb || int64_t(F_in) * F_out >= 4, TMA_ERR_INVALID_ARG, "sage gemm tf fwd: weight matrix below four elements");
    const char *name = kname<T>("gemm_tf_fwd", "gemm_tf_fwd_generic", "gemm_tf_fwd_bf16", "gemm_tf_fwd_bf16_generic", va);
#define TMA_TF_FWD(VA_, VB_)                                                                      \
    do {                                                                                          \
        CatRows<T, VA_> a{H, ldh, H, ldh, F_in, n, F_in};                                                   \
        SideWeights<VB_> b{W_self, W_neigh, F_in, F_out, Fp};                                     \
        launch_by_width<T, 32, false>(name, a, b, e, n, 2 * Fp, K, kps, 1, nullptr, s);              \
    } while (0)
    // weights whose rows are not multiples of four: 16-byte loads from 4-byte-aligned addresses
    // (the form is only chosen for F_in >= 8, so the matrices hold at least four elements)
    if (va && vb) TMA_TF_FWD(true, kAligned4);
    else if (va) TMA_TF_FWD(true, kUnaligned4);
    else if (vb) TMA_TF_FWD(false, kAligned4);
    else TMA_TF_FWD(false, kUnaligned4);
#undef TMA_TF_FWD
    return check_launch("sage gemm tf fwd");
}

int launch_sage_tf_gemm_fwd(int64_t n, const void *H, int64_t ldh, int32_t F_in, const float *W_self,
                            const float *W_neigh, int32_t F_out, int32_t dtype, void *Ys, void *Yn, int64_t ldy,
                            hipStream_t stream)
{
    if (n == 0) return TMA_OK;
    const int Fp = pad_cols(F_out, dtype);
    if (dtype == TMA_F32)
        return tf_fwd_typed<float>(n, static_cast<const float *>(H), ldh, F_in, W_self, W_neigh, F_out, Fp,
                                   static_cast<float *>(Ys), static_cast<float *>(Yn), ldy, stream);
    if (dtype == TMA_BF16)
        return tf_fwd_typed<uint16_t>(n, static_cast<const uint16_t *>(H), ldh, F_in, W_self, W_neigh, F_out, Fp,
                                      static_cast<uint16_t *>(Ys), static_cast<uint16_t *>(Yn), ldy, stream);
    return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm tf fwd: dtype %d", dtype);
}

static WeightSplit plan_tf_weight_split(int64_t n, int32_t F_in, int Fp)
{
    const int N = 2 * Fp;
    const int bn = N <= 64 ? 64 : (N <= 96 ? 96 : 128);
    const int64_t tiles = ceil_div(int64_t(F_in), 128) * ceil_div(N, bn);
    int64_t want = ceil_div(512, tiles > 0 ? tiles : 1);
    const int64_t max_useful = ceil_div(n > 0 ? n : 1, 128);
    if (want > max_useful) want = max_useful;
    if (want < 1) want = 1;
    WeightSplit w;
    w.k_per_split = int64_t(round_up(size_t(ceil_div(n > 0 ? n : 1, want)), 32));
    w.n_splits = int(ceil_div(n > 0 ? n : 1, w.k_per_split));
    w.partial_bytes = round_up(size_t(w.n_splits) * size_t(F_in) * size_t(N) * 4, 256);
    w.colsum_bytes = round_up(size_t(w.n_splits) * size_t(N) * 4, 256);
    return w;
}

size_t sage_tf_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out, int32_t dtype)
{
    const WeightSplit w = plan_tf_weight_split(n, F_in, pad_cols(F_out, dtype));
    return w.partial_bytes + w.colsum_bytes;
}

template <typename T>
static int tf_bwd_weight_typed(int64_t n, const T *H, int64_t ldh, const T *g, const T *h, int64_t ld_next,
                               const T *dYn, int64_t ldy, int32_t F_in, int32_t F_out, int Fp, bool relu,
                               const WeightSplit &w, float *partial, float *colsum, hipStream_t s)
{
    SplitEpilogue e{partial, int64_t(F_in), 2 * Fp};
    const bool va = vec4_ok(H, ldh);
    const bool vb = vec4_ok(g, ld_next) && (!relu || vec4_ok(h, ld_next)) && vec4_ok(dYn, ldy);
    const char *name = kname<T>("gemm_tf_bwd_weight", "gemm_tf_bwd_weight_generic", "gemm_tf_bwd_weight_bf16",
                                "gemm_tf_bwd_weight_bf16_generic", va && vb);
#define TMA_TF_BW(VA_, VB_, R_)                                                                                       \
    do {                                                                                                              \
        CatRowsT<T, VA_> a{H, ldh, H, ldh, F_in, n};                                                                       \
        SideGrad<false, T, VB_, R_> b{g, h, dYn, F_out, Fp, ld_next, ldy, n};                                         \
        launch_by_width<T, (sizeof(T) == 2 ? 32 : 16), true>(name, a, b, e, int64_t(F_in), 2 * Fp, n, w.k_per_split, w.n_splits, colsum, s);     \
    } while (0)
#define TMA_TF_BW2(VA_, VB_)         \
    do {                             \
        if (relu) TMA_TF_BW(VA_, VB_, true); \
        else TMA_TF_BW(VA_, VB_, false);     \
    } while (0)
    if (va && vb) TMA_TF_BW2(true, true);
    else if (va) TMA_TF_BW2(true, false);
    else if (vb) TMA_TF_BW2(false, true);
    else TMA_TF_BW2(false, false);
#undef TMA_TF_BW2
#undef TMA_TF_BW
    return check_launch("sage gemm tf bwd weight");
}

int launch_sage_tf_gemm_bwd_weight(int64_t n, const void *H, int64_t ldh, const void *dHnext, const void *Hnext,
                                   int64_t ld_next, const void *dYn, int64_t ldy, int32_t F_in, int32_t F_out,
                                   int32_t act, int32_t dtype, float *dW_self, float *dW_neigh, float *dbias, void *ws,
                                   size_t ws_bytes, hipStream_t stream)
{
    if (dtype != TMA_F32 && dtype != TMA_BF16) return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm tf bwd: dtype %d", dtype);
    const int Fp = pad_cols(F_out, dtype);
    const WeightSplit w = plan_tf_weight_split(n, F_in, Fp);
    if (ws_bytes < w.partial_bytes + w.colsum_bytes)
        return fail(TMA_ERR_WORKSPACE_TOO_SMALL, "sage gemm tf bwd weight: workspace %zu < %zu", ws_bytes,
                    w.partial_bytes + w.colsum_bytes);
    float *partial = static_cast<float *>(ws);
    float *colsum = reinterpret_cast<float *>(static_cast<char *>(ws) + w.partial_bytes);
    const bool relu = act == TMA_ACT_RELU;
    int rc = TMA_OK;
    if (n == 0) {
        // no rows: nothing to multiply (operands may be NULL); the second stage writes the zero gradients
    } else if (dtype == TMA_F32)
        rc = tf_bwd_weight_typed<float>(n, static_cast<const float *>(H), ldh, static_cast<const float *>(dHnext),
                                        static_cast<const float *>(Hnext), ld_next, static_cast<const float *>(dYn),
                                        ldy, F_in, F_out, Fp, relu, w, partial, colsum, stream);
    else
        rc = tf_bwd_weight_typed<uint16_t>(n, static_cast<const uint16_t *>(H), ldh,
                                           static_cast<const uint16_t *>(dHnext),
                                           static_cast<const uint16_t *>(Hnext), ld_next,
                                           static_cast<const uint16_t *>(dYn), ldy, F_in, F_out, Fp, relu, w, partial,
                                           colsum, stream);
    if (rc) return rc;
    const int64_t total_all = int64_t(F_in) * 2 * Fp + 2 * Fp;
    TMA_TIMED("reduce_splits_halves", stream);
    hipLaunchKernelGGL(reduce_splits_halves_kernel, dim3(unsigned(ceil_div(total_all, kRedCols))), dim3(256), 0, stream,
                       partial, colsum, n > 0 ? w.n_splits : 0, F_in, F_out, Fp, dW_self, dW_neigh, dbias);
    return check_launch("sage gemm tf bwd weight reduce");
}

template <typename T>
static int tf_bwd_data_typed(int64_t n, const T *g, const T *h, int64_t ld_next, const T *dYn, int64_t ldy,
                             const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out, int Fp, bool relu,
                             T *dH, int64_t ldh, hipStream_t s)
{
    RowsEpilogue<T> e{dH, ldh};
    const int64_t K = 2 * int64_t(Fp), kps = int64_t(round_up(size_t(K), 32));
    const bool va = vec4_ok(g, ld_next) && (!relu || vec4_ok(h, ld_next)) && vec4_ok(dYn, ldy);
    const bool vb = F_out % 4 == 0 && aligned(W_self, 16) && aligned(W_neigh, 16);
    TMA_REQUIRE(vb || int64_t(F_in) * F_out >= 4, TMA_ERR_INVALID_ARG, "sage gemm tf bwd data: weight matrix below four elements");
    const char *name = kname<T>("gemm_tf_bwd_data", "gemm_tf_bwd_data_generic", "gemm_tf_bwd_data_bf16",
                                "gemm_tf_bwd_data_bf16_generic", va);
#define TMA_TF_BD(VA_, VB_, R_)                                                                        \
    do {                                                                                               \
        SideGrad<true, T, VA_, R_> a{g, h, dYn, F_out, Fp, ld_next, ldy, n};                           \
        SideWeightsT<VB_> b{W_self, W_neigh, F_in, F_out, Fp};                                         \
        launch_gemm<128, 128, (sizeof(T) == 2 ? 32 : 16), 2, 2, false, T>(name, a, b, e, n, F_in, K, kps, 1, nullptr, s);         \
    } while (0)
#define TMA_TF_BD2(VA_, VB_)                 \
    do {                                     \
        if (relu) TMA_TF_BD(VA_, VB_, true); \
        else TMA_TF_BD(VA_, VB_, false);     \
    } while (0)
    if (va && vb) TMA_TF_BD2(true, kAligned4);
    else if (va) TMA_TF_BD2(true, kUnaligned4);
    else if (vb) TMA_TF_BD2(false, kAligned4);
    else TMA_TF_BD2(false, kUnaligned4);
#undef TMA_TF_BD2
#undef TMA_TF_BD
    return check_launch("sage gemm tf bwd data");
}

int launch_sage_tf_gemm_bwd_data(int64_t n, const void *dHnext, const void *Hnext, int64_t ld_next, const void *dYn,
                                 int64_t ldy, const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out,
                                 int32_t act, int32_t dtype, void *dH, int64_t ldh, hipStream_t stream)
{
    if (n == 0) return TMA_OK;
    const int Fp = pad_cols(F_out, dtype);
    const bool relu = act == TMA_ACT_RELU;
    if (dtype == TMA_F32)
        return tf_bwd_data_typed<float>(n, static_cast<const float *>(dHnext), static_cast<const float *>(Hnext),
                                        ld_next, static_cast<const float *>(dYn), ldy, W_self, W_neigh, F_in, F_out, Fp,
                                        relu, static_cast<float *>(dH), ldh, stream);
    if (dtype == TMA_BF16)
        return tf_bwd_data_typed<uint16_t>(n, static_cast<const uint16_t *>(dHnext),
                                           static_cast<const uint16_t *>(Hnext), ld_next,
                                           static_cast<const uint16_t *>(dYn), ldy, W_self, W_neigh, F_in, F_out, Fp,
                                           relu, static_cast<uint16_t *>(dH), ldh, stream);
    return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm tf bwd data: dtype %d", dtype);
}

}  // namespace tma
