// Losses on the last layer's output, the SGD step and the parameter
// averaging operator.  All small, streaming or latency-bound kernels.
#include "common.hpp"

#include <cmath>

namespace tma {

__device__ __forceinline__ float ld(const float *p) { return *p; }
__device__ __forceinline__ float ld(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st(float *p, float v) { *p = v; }
__device__ __forceinline__ void st(uint16_t *p, float v) { *p = f32_to_bf16(v); }

// Sum of one float per thread over a 256-thread block, fixed order.
__device__ __forceinline__ float block_sum_256(float v)
{
    __shared__ float wave_part[256 / kWave];
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) wave_part[threadIdx.x / kWave] = v;
    __syncthreads();
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < 256 / kWave; ++w) s += wave_part[w];
    __syncthreads();
    return s;
}

// Sixteen lanes per node (coalesced row reads): log-sum-exp, loss term,
// gradient (softmax - onehot)/n.  kRegs > 0: the row (C <= 16 * kRegs) is read once and kept in
// registers, one exp per element; kRegs = 0: any C, the row is read three times (it stays in L1).
// A block walks over several groups of 16 rows so that the number of partial loss sums stays small.
constexpr int kCeLanes = 16;
constexpr int kCeRows = 256 / kCeLanes;
constexpr int kCeMaxBlocks = 2048;

template <typename T, int kRegs>
__global__ __launch_bounds__(256) void softmax_ce_kernel(int64_t n, int C, const T *__restrict__ logits, int64_t ld_in,
                                                         const int32_t *__restrict__ labels,
                                                         T *__restrict__ dlogits, float *__restrict__ block_loss)
{
    const int sub = threadIdx.x % kCeLanes;
    const float inv_n = 1.0f / float(n);
    float term = 0.0f;
    for (int64_t v0 = int64_t(blockIdx.x) * kCeRows; v0 < n; v0 += int64_t(gridDim.x) * kCeRows) {
        const int64_t v = v0 + threadIdx.x / kCeLanes;
        const bool live = v < n;
        const T *z = logits + (live ? v : 0) * ld_in;
        if constexpr (kRegs > 0) {
            float zr[kRegs];
            float mx = -INFINITY;
#pragma unroll
            for (int k = 0; k < kRegs; ++k) {
                const int c = sub + k * kCeLanes;
                zr[k] = (live && c < C) ? ld(z + c) : -INFINITY;
                mx = fmaxf(mx, zr[k]);
            }
#pragma unroll
            for (int d = kCeLanes / 2; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, kWave));
            float ex[kRegs];
            float se = 0.0f;
#pragma unroll
            for (int k = 0; k < kRegs; ++k) {
                ex[k] = (live && sub + k * kCeLanes < C) ? expf(zr[k] - mx) : 0.0f;
                se += ex[k];
            }
#pragma unroll
            for (int d = kCeLanes / 2; d >= 1; d >>= 1) se += __shfl_xor(se, d, kWave);
            if (live) {
                const int y = labels[v];
                const float lse = mx + logf(se);
                const float inv_se = 1.0f / se;
#pragma unroll
                for (int k = 0; k < kRegs; ++k) {
                    const int c = sub + k * kCeLanes;
                    if (c == y) term += lse - zr[k];
                    if (dlogits && c < C) st(dlogits + v * ld_in + c, (ex[k] * inv_se - (c == y ? 1.0f : 0.0f)) * inv_n);
                }
            }
        } else {
            float mx = -INFINITY;
            if (live)
                for (int c = sub; c < C; c += kCeLanes) mx = fmaxf(mx, ld(z + c));
#pragma unroll
            for (int d = kCeLanes / 2; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, kWave));
            float se = 0.0f;
            if (live)
                for (int c = sub; c < C; c += kCeLanes) se += expf(ld(z + c) - mx);
#pragma unroll
            for (int d = kCeLanes / 2; d >= 1; d >>= 1) se += __shfl_xor(se, d, kWave);
            if (live) {
                const float lse = mx + logf(se);
                const int y = labels[v];
                if (sub == 0) term += lse - ld(z + y);
                if (dlogits)
                    for (int c = sub; c < C; c += kCeLanes)
                        st(dlogits + v * ld_in + c, (expf(ld(z + c) - lse) - (c == y ? 1.0f : 0.0f)) * inv_n);
            }
        }
    }
    const float s = block_sum_256(term);
    if (threadIdx.x == 0) block_loss[blockIdx.x] = s;
}

// z = sigmoid(g); L = 1/2 sum (y - z)^2 ; dL/dg = (z - y) z (1 - z)   (loss of the paper's Thm. 1)
template <typename T>
__global__ __launch_bounds__(256) void sigmoid_l2_kernel(int64_t n, int C, const T *__restrict__ G, int64_t ld_in,
                                                         const float *__restrict__ Y, T *__restrict__ dG,
                                                         float *__restrict__ block_loss)
{
    const int64_t total = n * C;
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    float term = 0.0f;
    if (i < total) {
        const int64_t v = i / C;
        const int c = int(i - v * C);
        const float z = 1.0f / (1.0f + expf(-ld(G + v * ld_in + c)));
        const float r = z - Y[i];
        term = 0.5f * r * r;
        if (dG) st(dG + v * ld_in + c, r * z * (1.0f - z));
    }
    const float s = block_sum_256(term);
    if (threadIdx.x == 0) block_loss[blockIdx.x] = s;
}

// Single block: fixed-order sum of the per-block terms, times `scale`.
__global__ __launch_bounds__(256) void finish_loss_kernel(int64_t nb, const float *__restrict__ block_loss,
                                                          float scale, float *__restrict__ loss_out)
{
    float s = 0.0f;
    for (int64_t i = threadIdx.x; i < nb; i += 256) s += block_loss[i];
    s = block_sum_256(s);
    if (threadIdx.x == 0) *loss_out = s * scale;
}

__global__ __launch_bounds__(256) void sgd_kernel(int64_t n, float *__restrict__ W, const float *__restrict__ dW, float lr)
{
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride) W[i] -= lr * dW[i];
}

// Adam with bias correction; 1 - b, c1 = 1 - b1^t and c2 = 1 - b2^t are formed on the host in double precision
// (1 - 0.999 taken in fp32 is already off by 1e-5).
__global__ __launch_bounds__(256) void adam_kernel(int64_t n, float *__restrict__ W, const float *__restrict__ dW,
                                                   float *__restrict__ m, float *__restrict__ v, float lr, float b1,
                                                   float omb1, float b2, float omb2, float eps, float inv_c1,
                                                   float inv_c2)
{
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride) {
        const float g = dW[i];
        const float mi = b1 * m[i] + omb1 * g;
        const float vi = b2 * v[i] + omb2 * g * g;
        m[i] = mi;
        v[i] = vi;
        W[i] -= lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
    }
}

// Mean over the active trainers in index order, written back to each of them.
__global__ __launch_bounds__(256) void average_kernel(float *const *__restrict__ W_ptrs, int n_trainers,
                                                      uint64_t active, float inv_count, int64_t n,
                                                      float *__restrict__ W_global)
{
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t j = int64_t(blockIdx.x) * 256 + threadIdx.x; j < n; j += stride) {
        float s = 0.0f;
        for (int i = 0; i < n_trainers; ++i)
            if ((active >> i) & 1ull) s += W_ptrs[i][j];
        s *= inv_count;
        if (W_global) W_global[j] = s;
        for (int i = 0; i < n_trainers; ++i)
            if ((active >> i) & 1ull) W_ptrs[i][j] = s;
    }
}

static int check_loss_args(const char *fn, int64_t n, int32_t C, const void *in, int64_t ldi, int32_t dtype,
                           const float *loss_out, const void *ws, size_t ws_bytes)
{
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX && C >= 1, TMA_ERR_INVALID_ARG, "%s: bad n or C", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(loss_out, TMA_ERR_INVALID_ARG, "%s: loss_out is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    TMA_REQUIRE(ws_bytes >= tma_loss_workspace_bytes(n, C), TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace too small", fn);
    TMA_REQUIRE(n == 0 || (in && ldi >= C), TMA_ERR_INVALID_ARG, "%s: input NULL or ld < C", fn);
    return TMA_OK;
}

}  // namespace tma

extern "C" size_t tma_loss_workspace_bytes(int64_t n, int32_t C)
{
    if (n < 0 || C < 1) return 0;
    // one partial sum per block: the element-wise loss runs one thread per (node, output),
    // the softmax loss sixteen lanes per node
    const int64_t items = n * int64_t(C);
    int64_t blocks = tma::ceil_div(items > 0 ? items : 1, 256);
    const int64_t ce_blocks = tma::ceil_div(n > 0 ? n : 1, tma::kCeRows);
    if (ce_blocks > blocks) blocks = ce_blocks;
    return tma::round_up(size_t(blocks) * 4, 256);
}

extern "C" int tma_softmax_ce(int64_t n, int32_t C, const void *logits, int64_t ldz, int32_t dtype,
                              const int32_t *labels, float *loss_out, void *dlogits_out, void *ws, size_t ws_bytes,
                              tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_softmax_ce";
    if (int rc = check_loss_args(fn, n, C, logits, ldz, dtype, loss_out, ws, ws_bytes)) return rc;
    TMA_REQUIRE(n == 0 || labels, TMA_ERR_INVALID_ARG, "%s: labels is NULL", fn);
    hipStream_t s = as_stream(stream);
    float *block_loss = static_cast<float *>(ws);
    int64_t nb = n > 0 ? ceil_div(n, kCeRows) : 0;
    if (nb > kCeMaxBlocks) nb = kCeMaxBlocks;
    if (nb > 0) {
        TMA_TIMED("softmax_ce", s);
#define TMA_CE(T, R)                                                                                              \
    hipLaunchKernelGGL((softmax_ce_kernel<T, R>), dim3(unsigned(nb)), dim3(256), 0, s, n, C,                      \
                       static_cast<const T *>(logits), ldz, labels, static_cast<T *>(dlogits_out), block_loss)
        if (dtype == TMA_F32) {
            if (C <= 2 * kCeLanes) TMA_CE(float, 2);
            else if (C <= 4 * kCeLanes) TMA_CE(float, 4);
            else TMA_CE(float, 0);
        } else {
            if (C <= 2 * kCeLanes) TMA_CE(uint16_t, 2);
            else if (C <= 4 * kCeLanes) TMA_CE(uint16_t, 4);
            else TMA_CE(uint16_t, 0);
        }
#undef TMA_CE
    }
    TMA_TIMED("finish_loss", s);
    hipLaunchKernelGGL(finish_loss_kernel, dim3(1), dim3(256), 0, s, nb, block_loss, n > 0 ? 1.0f / float(n) : 0.0f,
                       loss_out);
    return check_launch(fn);
}

extern "C" int tma_sigmoid_l2(int64_t n, int32_t C, const void *G, int64_t ldg, int32_t dtype, const float *Y,
                              float *loss_out, void *dG_out, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_sigmoid_l2";
    if (int rc = check_loss_args(fn, n, C, G, ldg, dtype, loss_out, ws, ws_bytes)) return rc;
    TMA_REQUIRE(n == 0 || Y, TMA_ERR_INVALID_ARG, "%s: Y is NULL", fn);
    hipStream_t s = as_stream(stream);
    float *block_loss = static_cast<float *>(ws);
    const int64_t nb = n > 0 ? ceil_div(n * C, 256) : 0;
    if (nb > 0) {
        TMA_TIMED("sigmoid_l2", s);
        if (dtype == TMA_F32)
            hipLaunchKernelGGL(sigmoid_l2_kernel<float>, dim3(unsigned(nb)), dim3(256), 0, s, n, C,
                               static_cast<const float *>(G), ldg, Y, static_cast<float *>(dG_out), block_loss);
        else
            hipLaunchKernelGGL(sigmoid_l2_kernel<uint16_t>, dim3(unsigned(nb)), dim3(256), 0, s, n, C,
                               static_cast<const uint16_t *>(G), ldg, Y, static_cast<uint16_t *>(dG_out), block_loss);
    }
    TMA_TIMED("finish_loss", s);
    hipLaunchKernelGGL(finish_loss_kernel, dim3(1), dim3(256), 0, s, nb, block_loss, 1.0f, loss_out);
    return check_launch(fn);
}

extern "C" int tma_sgd_step(int64_t n_params, float *W, const float *dW, float lr, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_sgd_step";
    TMA_REQUIRE(n_params >= 0, TMA_ERR_INVALID_ARG, "%s: n_params < 0", fn);
    if (n_params == 0) return TMA_OK;
    TMA_REQUIRE(W && dW, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    int64_t blocks = ceil_div(n_params, 256);
    if (blocks > 4096) blocks = 4096;
    TMA_TIMED("sgd", as_stream(stream));
    hipLaunchKernelGGL(sgd_kernel, dim3(unsigned(blocks)), dim3(256), 0, as_stream(stream), n_params, W, dW, lr);
    return check_launch(fn);
}

extern "C" int tma_adam_step(int64_t n_params, float *W, const float *dW, float *m, float *v, double lr, double beta1,
                             double beta2, double eps, int64_t step, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_adam_step";
    TMA_REQUIRE(n_params >= 0, TMA_ERR_INVALID_ARG, "%s: n_params < 0", fn);
    TMA_REQUIRE(step >= 1, TMA_ERR_INVALID_ARG, "%s: step counts from 1", fn);
    TMA_REQUIRE(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0 && eps >= 0.0, TMA_ERR_INVALID_ARG,
                "%s: need 0 <= beta < 1 and eps >= 0", fn);
    if (n_params == 0) return TMA_OK;
    TMA_REQUIRE(W && dW && m && v, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    const double c1 = 1.0 - pow(beta1, double(step)), c2 = 1.0 - pow(beta2, double(step));
    int64_t blocks = ceil_div(n_params, 256);
    if (blocks > 4096) blocks = 4096;
    TMA_TIMED("adam", as_stream(stream));
    hipLaunchKernelGGL(adam_kernel, dim3(unsigned(blocks)), dim3(256), 0, as_stream(stream), n_params, W, dW, m, v,
                       float(lr), float(beta1), float(1.0 - beta1), float(beta2), float(1.0 - beta2), float(eps),
                       float(1.0 / c1), float(1.0 / c2));
    return check_launch(fn);
}

extern "C" int tma_average(float *const *W_ptrs, int32_t n_trainers, uint64_t active_mask, int64_t n_params,
                           float *W_global_out, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_average";
    TMA_REQUIRE(n_trainers >= 1 && n_trainers <= 64, TMA_ERR_INVALID_ARG, "%s: n_trainers=%d outside [1,64]", fn,
                n_trainers);
    TMA_REQUIRE(n_params >= 0, TMA_ERR_INVALID_ARG, "%s: n_params < 0", fn);
    if (n_trainers < 64) active_mask &= (1ull << n_trainers) - 1ull;
    const int count = __builtin_popcountll(active_mask);
    TMA_REQUIRE(count >= 1, TMA_ERR_INVALID_ARG, "%s: no active trainer", fn);
    if (n_params == 0) return TMA_OK;
    TMA_REQUIRE(W_ptrs, TMA_ERR_INVALID_ARG, "%s: W_ptrs is NULL", fn);
    int64_t blocks = ceil_div(n_params, 256);
    if (blocks > 4096) blocks = 4096;
    TMA_TIMED("average", as_stream(stream));
    hipLaunchKernelGGL(average_kernel, dim3(unsigned(blocks)), dim3(256), 0, as_stream(stream), W_ptrs, n_trainers,
                       active_mask, 1.0f / float(count), n_params, W_global_out);
    return check_launch(fn);
}
