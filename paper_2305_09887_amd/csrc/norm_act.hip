// Layer normalisation followed by PReLU (the non-linearity of the paper's encoders, Sec. 4.1: PReLU
// with Layer Normalization before the activation), forward and backward, on a layer's pre-activation
// Z [n, F]:
//     Zh = (Z - mean_f Z) / sqrt(var_f Z + eps),  Y = gamma (.) Zh + beta,  H' = Y > 0 ? Y : slope * Y.
// Row-wise, HBM bound: forward reads Z and writes H' (2 n F s bytes), backward reads Z and dH' and writes
// dZ (3 n F s).  G lanes share a row (one 16-byte chunk per lane and pass, G a power of two so that the
// row reductions are xor-shuffles); a lane keeps its columns for all rows it visits, so gamma, beta and
// the partial sums of dgamma / dbeta live in registers.  The column sums are finished in two fixed-order
// stages (inside the block through LDS, across blocks by a second kernel): no atomics, bit-reproducible.
#include "kernels.hpp"

#include <mutex>
#include <type_traits>

namespace tma {

constexpr int kNormThreads = 256;
constexpr int kNormMaxBlocks = 2048;
constexpr int kNormMaxPerLane = 16;   // elements a lane holds: rows of up to 64 * 16 = 1024 elements

// How a lane's elements map to columns.  V: CPL chunks of E elements, chunk index sub + c*G.
// Otherwise one element per step, column sub + c*G (any F, any alignment).
template <typename T, bool V, int CPL>
struct RowMap {
    static constexpr int E = V ? Chunk<T>::kElems : 1;
    static constexpr int PER = CPL * E;
    static __device__ __forceinline__ int col(int sub, int G, int c, int i) { return (sub + c * G) * E + i; }
    static __device__ __forceinline__ void load(const T *row, int sub, int G, int F, float (&x)[PER])
    {
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            if constexpr (V) {
                float v[E];
                if (col(sub, G, c, 0) < F) Chunk<T>::load(row + col(sub, G, c, 0), v);
#pragma unroll
                for (int i = 0; i < E; ++i) x[c * E + i] = col(sub, G, c, 0) < F ? v[i] : 0.0f;
            } else {
                const int f = col(sub, G, c, 0);
                x[c] = 0.0f;
                if (f < F) {
                    if constexpr (sizeof(T) == 4) x[c] = reinterpret_cast<const float *>(row)[f];
                    else x[c] = bf16_to_f32(reinterpret_cast<const uint16_t *>(row)[f]);
                }
            }
        }
    }
    static __device__ __forceinline__ void store(T *row, int sub, int G, int F, const float (&x)[PER])
    {
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            if constexpr (V) {
                float v[E];
#pragma unroll
                for (int i = 0; i < E; ++i) v[i] = x[c * E + i];
                if (col(sub, G, c, 0) < F) Chunk<T>::store(row + col(sub, G, c, 0), v);
            } else {
                const int f = col(sub, G, c, 0);
                if (f < F) {
                    if constexpr (sizeof(T) == 4) reinterpret_cast<float *>(row)[f] = x[c];
                    else reinterpret_cast<uint16_t *>(row)[f] = f32_to_bf16(x[c]);
                }
            }
        }
    }
    static __device__ __forceinline__ void load_f32(const float *vec, int sub, int G, int F, float (&x)[PER])
    {
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int i = 0; i < E; ++i) x[c * E + i] = col(sub, G, c, i) < F ? vec[col(sub, G, c, i)] : 0.0f;
    }
};

__device__ __forceinline__ float group_sum(float v, int G)
{
    for (int d = G / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

// mean and 1/sqrt(var + eps) of the row spread over the group's registers (two passes, as the definition reads)
template <int PER>
__device__ __forceinline__ void row_stats(const float (&x)[PER], const bool (&in)[PER], int G, int F, float eps, float &mu,
                                          float &rstd)
{
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < PER; ++k) s += in[k] ? x[k] : 0.0f;
    mu = group_sum(s, G) / float(F);
    float q = 0.0f;
#pragma unroll
    for (int k = 0; k < PER; ++k) q += in[k] ? (x[k] - mu) * (x[k] - mu) : 0.0f;
    rstd = 1.0f / sqrtf(group_sum(q, G) / float(F) + eps);
}

template <typename T, bool V, int CPL>
__global__ __launch_bounds__(kNormThreads) void ln_prelu_fwd_kernel(int64_t n, int F, const T *__restrict__ Z, int64_t ldz,
                                                                    const float *__restrict__ gamma,
                                                                    const float *__restrict__ beta,
                                                                    const float *__restrict__ slope_p, float eps,
                                                                    T *__restrict__ out, int64_t ld_out, int G)
{
    using Map = RowMap<T, V, CPL>;
    constexpr int PER = Map::PER;
    const int sub = threadIdx.x % G;
    const int rows_per_block = kNormThreads / G;
    const float slope = *slope_p;
    float ga[PER], be[PER];
    bool in[PER];
    Map::load_f32(gamma, sub, G, F, ga);
    Map::load_f32(beta, sub, G, F, be);
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < Map::E; ++i) in[c * Map::E + i] = Map::col(sub, G, c, i) < F;

    for (int64_t v = int64_t(blockIdx.x) * rows_per_block + threadIdx.x / G; v < n;
         v += int64_t(gridDim.x) * rows_per_block) {
        float x[PER];
        Map::load(Z + v * ldz, sub, G, F, x);
        float mu, rstd;
        row_stats<PER>(x, in, G, F, eps, mu, rstd);
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const float y = ga[k] * ((x[k] - mu) * rstd) + be[k];
            x[k] = y > 0.0f ? y : slope * y;
        }
        Map::store(out + v * ld_out, sub, G, F, x);
    }
}

// partial layout per block: [0,F) dgamma, [F,2F) dbeta, [2F] dslope
template <typename T, bool V, int CPL>
__global__ __launch_bounds__(kNormThreads) void ln_prelu_bwd_kernel(int64_t n, int F, const T *__restrict__ Z, int64_t ldz,
                                                                    const T *dHn, int64_t ld_d,   // may alias dZ
                                                                    const float *__restrict__ gamma,
                                                                    const float *__restrict__ beta,
                                                                    const float *__restrict__ slope_p, float eps,
                                                                    T *dZ, int64_t ld_dz,
                                                                    float *__restrict__ partial, int G)
{
    using Map = RowMap<T, V, CPL>;
    constexpr int PER = Map::PER;
    __shared__ float red[2 * kNormThreads * PER];   // [row group][the group's columns] x {dgamma, dbeta}
    __shared__ float red_slope[kNormThreads / kWave];
    const int sub = threadIdx.x % G;
    const int grp = threadIdx.x / G;
    const int rows_per_block = kNormThreads / G;
    const float slope = *slope_p;
    float ga[PER], be[PER], dga[PER], dbe[PER];
    bool in[PER];
    Map::load_f32(gamma, sub, G, F, ga);
    Map::load_f32(beta, sub, G, F, be);
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < Map::E; ++i) in[c * Map::E + i] = Map::col(sub, G, c, i) < F;
#pragma unroll
    for (int k = 0; k < PER; ++k) dga[k] = dbe[k] = 0.0f;
    float dsl = 0.0f;

    for (int64_t v = int64_t(blockIdx.x) * rows_per_block + grp; v < n; v += int64_t(gridDim.x) * rows_per_block) {
        float x[PER], g[PER];
        Map::load(Z + v * ldz, sub, G, F, x);
        Map::load(dHn + v * ld_d, sub, G, F, g);
        float mu, rstd;
        row_stats<PER>(x, in, G, F, eps, mu, rstd);
        float m1 = 0.0f, m2 = 0.0f;
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const float zh = (x[k] - mu) * rstd;
            const float y = ga[k] * zh + be[k];
            const bool open = y > 0.0f;
            const float dy = in[k] ? (open ? g[k] : slope * g[k]) : 0.0f;
            if (in[k] && !open) dsl += g[k] * y;
            dga[k] += dy * zh;
            dbe[k] += dy;
            const float dzh = dy * ga[k];
            m1 += dzh;
            m2 += dzh * zh;
            x[k] = zh;
            g[k] = dzh;
        }
        m1 = group_sum(m1, G) / float(F);
        m2 = group_sum(m2, G) / float(F);
#pragma unroll
        for (int k = 0; k < PER; ++k) x[k] = (g[k] - m1 - x[k] * m2) * rstd;
        Map::store(dZ + v * ld_dz, sub, G, F, x);
    }

    // block stage: the row groups' partial column sums are added in group order
    const int width = G * PER;   // columns covered by one group (including positions past F)
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        red[(grp * width + sub * PER + k) * 2 + 0] = dga[k];
        red[(grp * width + sub * PER + k) * 2 + 1] = dbe[k];
    }
    for (int d = kWave / 2; d >= 1; d >>= 1) dsl += __shfl_xor(dsl, d, kWave);
    if (threadIdx.x % kWave == 0) red_slope[threadIdx.x / kWave] = dsl;
    __syncthreads();
    float *mine = partial + int64_t(blockIdx.x) * (2 * F + 1);
    if (grp == 0) {
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int i = 0; i < Map::E; ++i) {
                const int k = c * Map::E + i;
                const int f = Map::col(sub, G, c, i);
                if (f < F) {
                    float sg = 0.0f, sb = 0.0f;
                    for (int r = 0; r < rows_per_block; ++r) {
                        sg += red[(r * width + sub * PER + k) * 2 + 0];
                        sb += red[(r * width + sub * PER + k) * 2 + 1];
                    }
                    mine[f] = sg;
                    mine[F + f] = sb;
                }
            }
    }
    if (threadIdx.x == 0) {
        float s = 0.0f;
        for (int w = 0; w < kNormThreads / kWave; ++w) s += red_slope[w];
        mine[2 * F] = s;
    }
}

// second stage: a block owns 16 columns of the per-block partial sums; its 16 slices each add up 1/16 of
// the blocks (four loads in flight), then the slices are combined in slice order through LDS
constexpr int kFinCols = 16;
constexpr int kFinSlices = 16;

__global__ __launch_bounds__(256) void ln_prelu_finish_kernel(int nb, int F, const float *__restrict__ partial,
                                                              float *__restrict__ dgamma, float *__restrict__ dbeta,
                                                              float *__restrict__ dslope)
{
    __shared__ float part[kFinSlices][kFinCols];
    const int width = 2 * F + 1;
    const int c = threadIdx.x % kFinCols;
    const int slice = threadIdx.x / kFinCols;
    const int j = blockIdx.x * kFinCols + c;
    const int per = (nb + kFinSlices - 1) / kFinSlices;
    const int b0 = slice * per;
    const int b1 = (b0 + per) < nb ? (b0 + per) : nb;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    if (j < width) {
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
    if (slice == 0 && j < width) {
        float s = 0.0f;
        for (int k = 0; k < kFinSlices; ++k) s += part[k][c];
        if (j < F) dgamma[j] = s;
        else if (j < 2 * F) dbeta[j - F] = s;
        else *dslope = s;
    }
}

struct NormPlan {
    bool vec;
    int G, cpl;
    int64_t blocks;
};

static bool plan_norm(int64_t n, int F, size_t elem, bool vec_ok, NormPlan &p)
{
    const int E = int(16 / elem);
    p.vec = vec_ok && F % E == 0;
    const int units = p.vec ? F / E : F;          // chunks or elements per row
    int G = 4;
    while (G < units && G < kWave) G *= 2;
    p.G = G;
    p.cpl = int(ceil_div(units, G));
    const int per = p.cpl * (p.vec ? E : 1);
    if (per > kNormMaxPerLane) return false;
    const int rows_per_block = kNormThreads / G;
    p.blocks = ceil_div(n > 0 ? n : 1, rows_per_block);
    if (p.blocks > kNormMaxBlocks) p.blocks = kNormMaxBlocks;
    return true;
}

// rounds the chunk count up to an instantiated value (1, 2, 4 chunks; 16 single elements)
template <typename T, typename Launch>
static int dispatch_norm(const NormPlan &p, const char *fn, Launch &&launch)
{
    if (p.vec) {
        if (p.cpl == 1) launch(std::integral_constant<bool, true>{}, std::integral_constant<int, 1>{});
        else if (p.cpl == 2) launch(std::integral_constant<bool, true>{}, std::integral_constant<int, 2>{});
        else if (p.cpl * Chunk<T>::kElems <= kNormMaxPerLane && p.cpl <= 4)
            launch(std::integral_constant<bool, true>{}, std::integral_constant<int, 16 / Chunk<T>::kElems>{});
        else return fail(TMA_ERR_BAD_SHAPE, "%s: rows too long", fn);
    } else {
        launch(std::integral_constant<bool, false>{}, std::integral_constant<int, kNormMaxPerLane>{});
    }
    return check_launch(fn);
}

}  // namespace tma

static int check_norm_args(const char *fn, int64_t n, int32_t F, const void *Z, int64_t ldz, const float *gamma,
                           const float *beta, const float *slope, float eps, int32_t dtype)
{
    using namespace tma;
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX && F >= 1, TMA_ERR_INVALID_ARG, "%s: bad n or F", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(eps >= 0.0f, TMA_ERR_INVALID_ARG, "%s: eps < 0", fn);
    TMA_REQUIRE(gamma && beta && slope, TMA_ERR_INVALID_ARG, "%s: gamma / beta / slope is NULL", fn);
    TMA_REQUIRE(n == 0 || (Z && ldz >= F), TMA_ERR_INVALID_ARG, "%s: Z is NULL or ldz < F", fn);
    return TMA_OK;
}

extern "C" int tma_layernorm_prelu_fwd(int64_t n, int32_t F, const void *Z, int64_t ldz, const float *gamma,
                                       const float *beta, const float *slope, float eps, int32_t dtype,
                                       void *Hnext_out, int64_t ld_out, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_layernorm_prelu_fwd";
    if (int rc = check_norm_args(fn, n, F, Z, ldz, gamma, beta, slope, eps, dtype)) return rc;
    if (n == 0) return TMA_OK;
    TMA_REQUIRE(Hnext_out && ld_out >= F, TMA_ERR_INVALID_ARG, "%s: Hnext_out is NULL or ld_out < F", fn);
    const size_t elem = dtype == TMA_BF16 ? 2 : 4;
    const bool vec_ok = aligned(Z, 16) && aligned(Hnext_out, 16) && (size_t(ldz) * elem) % 16 == 0 &&
                        (size_t(ld_out) * elem) % 16 == 0;
    NormPlan p;
    TMA_REQUIRE(plan_norm(n, F, elem, vec_ok, p), TMA_ERR_BAD_SHAPE, "%s: F = %d is beyond %d elements per row", fn, F,
                kWave * kNormMaxPerLane);
    hipStream_t s = as_stream(stream);
    TMA_TIMED(dtype == TMA_BF16 ? "ln_prelu_fwd_bf16" : "ln_prelu_fwd_f32", s);
    auto go = [&](auto t) {
        using T = decltype(t);
        return dispatch_norm<T>(p, fn, [&](auto vtag, auto ctag) {
            hipLaunchKernelGGL((ln_prelu_fwd_kernel<T, decltype(vtag)::value, decltype(ctag)::value>),
                               dim3(unsigned(p.blocks)), dim3(kNormThreads), 0, s, n, F, static_cast<const T *>(Z), ldz,
                               gamma, beta, slope, eps, static_cast<T *>(Hnext_out), ld_out, p.G);
        });
    };
    return dtype == TMA_BF16 ? go(uint16_t{}) : go(float{});
}

extern "C" size_t tma_layernorm_prelu_bwd_workspace_bytes(int64_t n, int32_t F)
{
    if (n < 0 || F < 1) return 0;
    return tma::round_up(size_t(tma::kNormMaxBlocks) * (2 * size_t(F) + 1) * 4, 256);
}

namespace tma {

// Both backward entry points: argument checks that do not concern the scratch space, then the two launches.
// `partial` holds kNormMaxBlocks * (2 F + 1) floats; every slot that the second kernel reads has been written by
// the first one in the same call, so the buffer needs no clearing.
static int ln_prelu_bwd_run(const char *fn, int64_t n, int32_t F, const void *Z, int64_t ldz, const void *dHnext,
                            int64_t ld_d, const float *gamma, const float *beta, const float *slope, float eps,
                            int32_t dtype, void *dZ_out, int64_t ld_dz, float *dgamma, float *dbeta, float *dslope,
                            float *partial, hipStream_t s)
{
    TMA_REQUIRE(n == 0 || (dHnext && dZ_out && ld_d >= F && ld_dz >= F), TMA_ERR_INVALID_ARG,
                "%s: dHnext / dZ_out NULL or leading dimension < F", fn);
    const size_t elem = dtype == TMA_BF16 ? 2 : 4;
    const bool vec_ok = aligned(Z, 16) && aligned(dHnext, 16) && aligned(dZ_out, 16) && (size_t(ldz) * elem) % 16 == 0 &&
                        (size_t(ld_d) * elem) % 16 == 0 && (size_t(ld_dz) * elem) % 16 == 0;
    NormPlan p;
    TMA_REQUIRE(plan_norm(n, F, elem, vec_ok, p), TMA_ERR_BAD_SHAPE, "%s: F = %d is beyond %d elements per row", fn, F,
                kWave * kNormMaxPerLane);
    const int nb = n > 0 ? int(p.blocks) : 0;
    if (n > 0) {
        TMA_TIMED(dtype == TMA_BF16 ? "ln_prelu_bwd_bf16" : "ln_prelu_bwd_f32", s);
        auto go = [&](auto t) {
            using T = decltype(t);
            return dispatch_norm<T>(p, fn, [&](auto vtag, auto ctag) {
                hipLaunchKernelGGL((ln_prelu_bwd_kernel<T, decltype(vtag)::value, decltype(ctag)::value>),
                                   dim3(unsigned(p.blocks)), dim3(kNormThreads), 0, s, n, F, static_cast<const T *>(Z),
                                   ldz, static_cast<const T *>(dHnext), ld_d, gamma, beta, slope, eps,
                                   static_cast<T *>(dZ_out), ld_dz, partial, p.G);
            });
        };
        if (int rc = dtype == TMA_BF16 ? go(uint16_t{}) : go(float{})) return rc;
    }
    TMA_TIMED("ln_prelu_finish", s);
    hipLaunchKernelGGL(ln_prelu_finish_kernel, dim3(unsigned(ceil_div(2 * F + 1, kFinCols))), dim3(256), 0, s, nb, F, partial,
                       dgamma, dbeta, dslope);
    return check_launch(fn);
}

// Library-owned scratch of tma_layernorm_prelu_bwd_static: the per-block partial sums for rows of up to
// kStaticNormMaxF elements (2048 * 513 floats = 4.2 MB per GPU, held until the process ends).
constexpr int kStaticNormMaxF = 256;
constexpr size_t kStaticNormFloats = size_t(kNormMaxBlocks) * (2 * size_t(kStaticNormMaxF) + 1);

}  // namespace tma

static __device__ __align__(256) float scratch[tma::kStaticNormFloats];

namespace tma {

// Device address of `scratch` on the current device.  In host code the array's name is only a handle for
// hipGetSymbolAddress; each GPU holds its own copy at its own address, looked up once per device.
static int static_norm_scratch(const char *fn, float **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static float *ptr[kMaxDevices] = {};
    int dev = -1;
    TMA_HIP_TRY(hipGetDevice(&dev), fn);
    TMA_REQUIRE(dev >= 0 && dev < kMaxDevices, TMA_ERR_HIP, "%s: device index %d", fn, dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        TMA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), fn);
        TMA_REQUIRE(p != nullptr, TMA_ERR_HIP, "%s: no device address for the static scratch array", fn);
        ptr[dev] = static_cast<float *>(p);
    }
    *out = ptr[dev];
    return TMA_OK;
}

}  // namespace tma

extern "C" int tma_layernorm_prelu_bwd(int64_t n, int32_t F, const void *Z, int64_t ldz, const void *dHnext,
                                       int64_t ld_d, const float *gamma, const float *beta, const float *slope,
                                       float eps, int32_t dtype, void *dZ_out, int64_t ld_dz, float *dgamma,
                                       float *dbeta, float *dslope, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_layernorm_prelu_bwd";
    if (int rc = check_norm_args(fn, n, F, Z, ldz, gamma, beta, slope, eps, dtype)) return rc;
    TMA_REQUIRE(dgamma && dbeta && dslope, TMA_ERR_INVALID_ARG, "%s: gradient output is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    TMA_REQUIRE(ws_bytes >= tma_layernorm_prelu_bwd_workspace_bytes(n, F), TMA_ERR_WORKSPACE_TOO_SMALL,
                "%s: workspace too small", fn);
    return ln_prelu_bwd_run(fn, n, F, Z, ldz, dHnext, ld_d, gamma, beta, slope, eps, dtype, dZ_out, ld_dz, dgamma, dbeta,
                            dslope, static_cast<float *>(ws), as_stream(stream));
}

extern "C" int32_t tma_layernorm_prelu_bwd_static_max_f(void) { return tma::kStaticNormMaxF; }

extern "C" int tma_layernorm_prelu_bwd_static(int64_t n, int32_t F, const void *Z, int64_t ldz, const void *dHnext,
                                              int64_t ld_d, const float *gamma, const float *beta, const float *slope,
                                              float eps, int32_t dtype, void *dZ_out, int64_t ld_dz, float *dgamma,
                                              float *dbeta, float *dslope, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_layernorm_prelu_bwd_static";
    if (int rc = check_norm_args(fn, n, F, Z, ldz, gamma, beta, slope, eps, dtype)) return rc;
    TMA_REQUIRE(dgamma && dbeta && dslope, TMA_ERR_INVALID_ARG, "%s: gradient output is NULL", fn);
    TMA_REQUIRE(F <= kStaticNormMaxF, TMA_ERR_BAD_SHAPE,
                "%s: F = %d is beyond the %d elements per row that the library's own scratch array is sized for "
                "(use tma_layernorm_prelu_bwd with a workspace)", fn, F, kStaticNormMaxF);
    float *partial = nullptr;
    if (int rc = static_norm_scratch(fn, &partial)) return rc;
    return ln_prelu_bwd_run(fn, n, F, Z, ldz, dHnext, ld_d, gamma, beta, slope, eps, dtype, dZ_out, ld_dz, dgamma, dbeta,
                            dslope, partial, as_stream(stream));
}
