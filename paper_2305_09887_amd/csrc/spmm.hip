// Mean aggregation  M = Abar H  (paper Thm. 1, first equation of its proof) and
// the plain row gather-sum used by the backward pass.  HBM/gather bound: the
// flops (2 per gathered element) are negligible.
//
// Mapping.  A feature row is cut into 16-byte chunks; G lanes (a power of two,
// the smallest that covers the row, at most the 64-lane wavefront) own one row
// and each lane keeps its chunk(s) of the running sum in registers, so every
// neighbour row is fetched with one coalesced 16-byte load per lane.  The G
// lanes read up to G neighbour ids with one coalesced load and pass them round
// by cross-lane shuffle.  Local graphs under random assignment are very sparse
// (mean local degree 2-5) with a power-law tail, so rows are binned by degree
// inside the block: a row of more than kHubDegree entries is deferred and then
// summed by all groups of the workgroup together, each taking every NG-th run
// of G neighbours, with a fixed-order combine through LDS.  The result of a
// row depends only on its own neighbour list, never on scheduling.
#include "kernels.hpp"

namespace tma {

constexpr int kSpmmThreads = 256;
constexpr int kRowsPerGroup = 4;   // rows a lane group walks through per block
constexpr int kHubDegree = 48;     // rows longer than this are summed by the whole workgroup

template <typename T>
struct Chunk;

template <>
struct Chunk<float> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void load(const float *p, float (&v)[4])
    {
        const float4 x = *reinterpret_cast<const float4 *>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&v)[4])
    {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};

template <>
struct Chunk<uint16_t> {  // bf16 storage
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void load(const uint16_t *p, float (&v)[8])
    {
        const uint4 x = *reinterpret_cast<const uint4 *>(p);
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void store(uint16_t *p, const float (&v)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = uint32_t(f32_to_bf16(v[2 * i])) | (uint32_t(f32_to_bf16(v[2 * i + 1])) << 16);
        *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

__device__ __forceinline__ float load_elem(const float *p) { return *p; }
__device__ __forceinline__ float load_elem(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store_elem(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(uint16_t *p, float v) { *p = f32_to_bf16(v); }

// U neighbour rows (entries j .. j+U-1 of the run whose ids sit in `mine`) fetched together, then added in order.
template <typename T, int G, int CPL, int U>
__device__ __forceinline__ void gather_batch(const T *__restrict__ in, int64_t ld, int32_t mine, int j, int sub,
                                             int n_chunks, float (&acc)[CPL][Chunk<T>::kElems])
{
    constexpr int E = Chunk<T>::kElems;
    float v[U][CPL][E];
#pragma unroll
    for (int q = 0; q < U; ++q) {
        const T *row = in + int64_t(__shfl(mine, j + q, G)) * ld;
#pragma unroll
        for (int c = 0; c < CPL; ++c)
            if (sub + c * G < n_chunks) Chunk<T>::load(row + (sub + c * G) * E, v[q][c]);
    }
#pragma unroll
    for (int q = 0; q < U; ++q)
#pragma unroll
        for (int c = 0; c < CPL; ++c)
            if (sub + c * G < n_chunks)
#pragma unroll
                for (int i = 0; i < E; ++i) acc[c][i] += v[q][c][i];
}

// Adds the rows colidx[e] for e = beg, beg+1, ... in runs of G entries that start
// `run_stride` entries apart.  Every lane of the group gets the same trip counts.
// kDeep: up to 16 rows in flight per lane (long rows are latency bound: a 500-entry
// row walked four loads at a time sets the kernel's tail).
template <typename T, int G, int CPL, bool kDeep>
__device__ __forceinline__ void gather_sum(const T *__restrict__ in, int64_t ld, const int32_t *__restrict__ colidx,
                                           int32_t beg, int32_t end, int32_t run_stride, int sub, int n_chunks,
                                           float (&acc)[CPL][Chunk<T>::kElems])
{
    for (int32_t e0 = beg; e0 < end; e0 += run_stride) {
        const int cnt = (end - e0) < G ? (end - e0) : G;
        const int32_t mine = sub < cnt ? colidx[e0 + sub] : 0;
        int j = 0;
        if constexpr (kDeep && CPL == 1 && G >= 16)
            for (; j + 16 <= cnt; j += 16) gather_batch<T, G, CPL, 16>(in, ld, mine, j, sub, n_chunks, acc);
        for (; j + 4 <= cnt; j += 4) gather_batch<T, G, CPL, 4>(in, ld, mine, j, sub, n_chunks, acc);
        for (; j < cnt; ++j) gather_batch<T, G, CPL, 1>(in, ld, mine, j, sub, n_chunks, acc);
    }
}

// What happens to a finished row sum s_v:
//   out_v = act( scale_v * s_v  [+ out_v]  [+ self_v]  [+ bias] )
// scale_v = inv_deg[v] (mean) or 1; "+ out_v" accumulates onto what is there (backward: on top of
// dZ W_self^T); "+ self_v + bias" and the activation turn the gather into the layer output when the
// transform ran before the aggregation.
template <typename T>
struct SpmmOut {
    T *out;
    int64_t ld_out;
    const float *inv_deg;
    int accumulate;
    const T *self;
    int64_t ld_self;
    const float *bias;
    int F;  // valid elements of a row (bias is not applied to padding)
    int relu;
};

template <typename T, int G, int CPL>
__device__ __forceinline__ void finish_row(int64_t v, const SpmmOut<T> &o, int sub, int n_chunks,
                                           float (&acc)[CPL][Chunk<T>::kElems])
{
    constexpr int E = Chunk<T>::kElems;
    const float scale = o.inv_deg ? o.inv_deg[v] : 1.0f;
#pragma unroll
    for (int c = 0; c < CPL; ++c)
        if (sub + c * G < n_chunks) {
            const int f0 = (sub + c * G) * E;
            T *dst = o.out + v * o.ld_out + f0;
            float r[E];
#pragma unroll
            for (int i = 0; i < E; ++i) r[i] = acc[c][i] * scale;
            if (o.accumulate) {
                float old[E];
                Chunk<T>::load(dst, old);
#pragma unroll
                for (int i = 0; i < E; ++i) r[i] += old[i];
            }
            if (o.self) {
                float sv[E];
                Chunk<T>::load(o.self + v * o.ld_self + f0, sv);
#pragma unroll
                for (int i = 0; i < E; ++i) r[i] += sv[i];
            }
            if (o.bias) {
#pragma unroll
                for (int i = 0; i < E; ++i) r[i] += (f0 + i < o.F) ? o.bias[f0 + i] : 0.0f;
            }
            if (o.relu) {
#pragma unroll
                for (int i = 0; i < E; ++i) r[i] = r[i] > 0.0f ? r[i] : 0.0f;
            }
            Chunk<T>::store(dst, r);
        }
}

// Adds the rows colidx[e], e in [beg, end), into the accumulators of up to four consecutive
// CSR rows at once: entry e belongs to row r when bound[r] <= e < bound[r+1].  The entries
// of consecutive rows are contiguous in colidx, so the group walks them as one list with
// four independent 16-byte loads in flight, and steers each loaded chunk to its row by
// predication (adding 0 elsewhere).  At a mean local degree of 2-5 this is what keeps
// enough bytes in flight; walking the rows one after the other leaves the lanes waiting.
template <typename T, int G, int R, int U>
__device__ __forceinline__ void gather_rows_batch(const T *__restrict__ in, int64_t ld, int32_t mine, int j, int32_t e_first,
                                                  const int32_t (&bound)[R + 1], int sub, bool own,
                                                  float (&acc)[R][Chunk<T>::kElems])
{
    constexpr int E = Chunk<T>::kElems;
    float v[U][E];
#pragma unroll
    for (int q = 0; q < U; ++q) {
        const T *row = in + int64_t(__shfl(mine, j + q, G)) * ld;
        if (own) Chunk<T>::load(row + sub * E, v[q]);
    }
#pragma unroll
    for (int q = 0; q < U; ++q) {
        const int32_t e = e_first + q;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool hit = e >= bound[r] && e < bound[r + 1];
            if (own)
#pragma unroll
                for (int i = 0; i < E; ++i) acc[r][i] += hit ? v[q][i] : 0.0f;
        }
    }
}

template <typename T, int G, int R>
__device__ __forceinline__ void gather_sum_rows(const T *__restrict__ in, int64_t ld,
                                                const int32_t *__restrict__ colidx, const int32_t (&bound)[R + 1],
                                                int sub, int n_chunks, float (&acc)[R][Chunk<T>::kElems])
{
    const bool own = sub < n_chunks;
    const int32_t end = bound[R];
    for (int32_t e0 = bound[0]; e0 < end; e0 += G) {
        const int cnt = (end - e0) < G ? (end - e0) : G;
        const int32_t mine = sub < cnt ? colidx[e0 + sub] : 0;
        int j = 0;
        if constexpr (G >= 8)
            for (; j + 8 <= cnt; j += 8) gather_rows_batch<T, G, R, 8>(in, ld, mine, j, e0 + j, bound, sub, own, acc);
        for (; j + 4 <= cnt; j += 4) gather_rows_batch<T, G, R, 4>(in, ld, mine, j, e0 + j, bound, sub, own, acc);
        for (; j < cnt; ++j) gather_rows_batch<T, G, R, 1>(in, ld, mine, j, e0 + j, bound, sub, own, acc);
    }
}

template <typename T, int G, int CPL>
__global__ __launch_bounds__(kSpmmThreads) void spmm_rows_kernel(int64_t n, const int32_t *__restrict__ rowptr,
                                                                 const int32_t *__restrict__ colidx,
                                                                 const T *__restrict__ in, int64_t ld_in,
                                                                 SpmmOut<T> o, int n_chunks)
{
    constexpr int E = Chunk<T>::kElems;
    constexpr int NG = kSpmmThreads / G;
    constexpr int R = kRowsPerGroup;
    constexpr int RPB = NG * R;
    __shared__ int32_t hub_rows[RPB];
    __shared__ int32_t hub_count;
    __shared__ float partial[NG][G * CPL * E];

    const int sub = threadIdx.x % G;
    const int grp = threadIdx.x / G;
    if (threadIdx.x == 0) hub_count = 0;
    __syncthreads();

    // the group owns R consecutive rows v0 .. v0+R-1
    const int64_t base = int64_t(blockIdx.x) * RPB;
    const int64_t v0 = base + int64_t(grp) * R;
    int32_t bound[R + 1];
#pragma unroll
    for (int r = 0; r <= R; ++r) bound[r] = rowptr[(v0 + r) < n ? (v0 + r) : n];
    bool any_hub = false;
#pragma unroll
    for (int r = 0; r < R; ++r) any_hub = any_hub || (bound[r + 1] - bound[r] > kHubDegree);

    if (CPL == 1 && !any_hub) {
        float acc[R][E];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int k = 0; k < E; ++k) acc[r][k] = 0.0f;
        gather_sum_rows<T, G, R>(in, ld_in, colidx, bound, sub, n_chunks, acc);
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (v0 + r < n) {
                float one[1][E];
#pragma unroll
                for (int k = 0; k < E; ++k) one[0][k] = acc[r][k];
                finish_row<T, G, 1>(v0 + r, o, sub, n_chunks, one);
            }
    } else {
        for (int r = 0; r < R; ++r) {
            const int64_t v = v0 + r;
            if (v >= n) break;
            const int32_t beg = bound[r], end = bound[r + 1];
            if (end - beg > kHubDegree) {
                if (sub == 0) hub_rows[atomicAdd(&hub_count, 1)] = int32_t(v - base);
                continue;
            }
            float acc[CPL][E];
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int k = 0; k < E; ++k) acc[c][k] = 0.0f;
            gather_sum<T, G, CPL, false>(in, ld_in, colidx, beg, end, G, sub, n_chunks, acc);
            finish_row<T, G, CPL>(v, o, sub, n_chunks, acc);
        }
    }
    __syncthreads();

    const int n_hubs = hub_count;
    for (int h = 0; h < n_hubs; ++h) {
        const int64_t v = base + hub_rows[h];
        const int32_t beg = rowptr[v], end = rowptr[v + 1];
        float acc[CPL][E];
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int k = 0; k < E; ++k) acc[c][k] = 0.0f;
        if (beg + grp * G < end) gather_sum<T, G, CPL, true>(in, ld_in, colidx, beg + grp * G, end, NG * G, sub, n_chunks, acc);
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int k = 0; k < E; ++k) partial[grp][(c * G + sub) * E + k] = acc[c][k];
        __syncthreads();
        if (grp == 0) {
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int k = 0; k < E; ++k) {
                    float s = 0.0f;
                    for (int g = 0; g < NG; ++g) s += partial[g][(c * G + sub) * E + k];  // fixed order
                    acc[c][k] = s;
                }
            finish_row<T, G, CPL>(v, o, sub, n_chunks, acc);
        }
        __syncthreads();
    }
}

// Any F, any alignment: one wavefront per row, lane owns elements lane, lane+64, ...
template <typename T>
__global__ __launch_bounds__(kSpmmThreads) void spmm_rows_generic_kernel(int64_t n, const int32_t *__restrict__ rowptr,
                                                                         const int32_t *__restrict__ colidx,
                                                                         const T *__restrict__ in, int64_t ld_in,
                                                                         SpmmOut<T> o, int F)
{
    constexpr int kPer = 8;  // elements per lane per sweep: 512 features per sweep
    const int lane = threadIdx.x % kWave;
    const int64_t v = int64_t(blockIdx.x) * (kSpmmThreads / kWave) + threadIdx.x / kWave;
    if (v >= n) return;
    const int32_t beg = rowptr[v], end = rowptr[v + 1];
    const float scale = o.inv_deg ? o.inv_deg[v] : 1.0f;
    for (int f0 = 0; f0 < F; f0 += kWave * kPer) {
        float acc[kPer];
#pragma unroll
        for (int k = 0; k < kPer; ++k) acc[k] = 0.0f;
        for (int32_t e = beg; e < end; ++e) {
            const T *row = in + int64_t(colidx[e]) * ld_in;
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int f = f0 + k * kWave + lane;
                if (f < F) acc[k] += load_elem(row + f);
            }
        }
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int f = f0 + k * kWave + lane;
            if (f < F) {
                T *dst = o.out + v * o.ld_out + f;
                float r = acc[k] * scale;
                if (o.accumulate) r += load_elem(dst);
                if (o.self) r += load_elem(o.self + v * o.ld_self + f);
                if (o.bias && f < o.F) r += o.bias[f];
                if (o.relu) r = r > 0.0f ? r : 0.0f;
                store_elem(dst, r);
            }
        }
    }
}

template <typename T, int G, int CPL>
static void launch_rows(int64_t n, const int32_t *rowptr, const int32_t *colidx, const T *in, int64_t ld_in,
                        const SpmmOut<T> &o, int n_chunks, hipStream_t s)
{
    constexpr int RPB = (kSpmmThreads / G) * kRowsPerGroup;
    char name[48];
    snprintf(name, sizeof(name), "%s_%s_g%dx%d", o.self ? "spmm_combine" : (o.inv_deg ? "spmm_mean" : "spmm_sum"),
             sizeof(T) == 4 ? "f32" : "bf16", G, CPL);
    TMA_TIMED(name, s);
    hipLaunchKernelGGL((spmm_rows_kernel<T, G, CPL>), dim3(unsigned(ceil_div(n, RPB))), dim3(kSpmmThreads), 0, s, n,
                       rowptr, colidx, in, ld_in, o, n_chunks);
}

template <typename T>
static int launch_typed(int64_t n, const int32_t *rowptr, const int32_t *colidx, const T *in, int64_t ld_in, int32_t F,
                        const SpmmOut<T> &o, hipStream_t s)
{
    const size_t row_bytes = size_t(F) * sizeof(T);
    const bool vec_ok = row_bytes % 16 == 0 && (size_t(ld_in) * sizeof(T)) % 16 == 0 &&
                        (size_t(o.ld_out) * sizeof(T)) % 16 == 0 && aligned(in, 16) && aligned(o.out, 16) &&
                        (!o.self || ((size_t(o.ld_self) * sizeof(T)) % 16 == 0 && aligned(o.self, 16))) &&
                        row_bytes / 16 <= 256;
    if (!vec_ok) {
        TMA_TIMED(o.self ? "spmm_combine_generic" : (o.inv_deg ? "spmm_mean_generic" : "spmm_sum_generic"), s);
        hipLaunchKernelGGL((spmm_rows_generic_kernel<T>), dim3(unsigned(ceil_div(n, kSpmmThreads / kWave))),
                           dim3(kSpmmThreads), 0, s, n, rowptr, colidx, in, ld_in, o, F);
        return check_launch("spmm (generic)");
    }
    const int nc = int(row_bytes / 16);
#define TMA_SPMM_CASE(G, CPL) launch_rows<T, G, CPL>(n, rowptr, colidx, in, ld_in, o, nc, s)
    if (nc <= 4) TMA_SPMM_CASE(4, 1);
    else if (nc <= 8) TMA_SPMM_CASE(8, 1);
    else if (nc <= 16) TMA_SPMM_CASE(16, 1);
    else if (nc <= 32) TMA_SPMM_CASE(32, 1);
    else if (nc <= 64) TMA_SPMM_CASE(64, 1);
    else if (nc <= 128) TMA_SPMM_CASE(64, 2);
    else TMA_SPMM_CASE(64, 4);
#undef TMA_SPMM_CASE
    return check_launch("spmm");
}

template <typename T>
static int spmm_any(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                    int64_t ld_in, int32_t F, void *out, int64_t ld_out, bool accumulate, const void *self,
                    int64_t ld_self, const float *bias, int32_t F_valid, bool relu, hipStream_t stream)
{
    SpmmOut<T> o{static_cast<T *>(out), ld_out, inv_deg, accumulate ? 1 : 0, static_cast<const T *>(self), ld_self,
                 bias, F_valid, relu ? 1 : 0};
    return launch_typed<T>(n, rowptr, colidx, static_cast<const T *>(in), ld_in, F, o, stream);
}

int launch_spmm(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                int64_t ld_in, int32_t F, int32_t dtype, void *out, int64_t ld_out, bool accumulate,
                hipStream_t stream)
{
    return launch_spmm_combine(n, rowptr, colidx, inv_deg, in, ld_in, F, dtype, out, ld_out, accumulate, nullptr, 0,
                               nullptr, F, false, stream);
}

int launch_spmm_combine(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                        int64_t ld_in, int32_t F, int32_t dtype, void *out, int64_t ld_out, bool accumulate,
                        const void *self, int64_t ld_self, const float *bias, int32_t F_valid, bool relu,
                        hipStream_t stream)
{
    if (n == 0 || F == 0) return TMA_OK;
    if (dtype == TMA_F32)
        return spmm_any<float>(n, rowptr, colidx, inv_deg, in, ld_in, F, out, ld_out, accumulate, self, ld_self, bias,
                               F_valid, relu, stream);
    if (dtype == TMA_BF16)
        return spmm_any<uint16_t>(n, rowptr, colidx, inv_deg, in, ld_in, F, out, ld_out, accumulate, self, ld_self,
                                  bias, F_valid, relu, stream);
    return fail(TMA_ERR_UNSUPPORTED_DTYPE, "spmm: dtype %d", dtype);
}

// dst_v = inv_deg[v] * g_v (.) [h_v > 0]   (rows of F elements; padding up to F_pad is zeroed)
template <typename T>
__global__ __launch_bounds__(256) void scale_mask_rows_kernel(int64_t n, int F, int F_pad, const T *__restrict__ g,
                                                              const T *__restrict__ h, int64_t ld,
                                                              const float *__restrict__ inv_deg, int relu,
                                                              T *__restrict__ dst, int64_t ld_dst)
{
    const int64_t total = n * F_pad;
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < total; i += stride) {
        const int64_t v = i / F_pad;
        const int f = int(i - v * F_pad);
        float r = 0.0f;
        if (f < F) {
            r = load_elem(g + v * ld + f) * inv_deg[v];
            if (relu && !(load_elem(h + v * ld + f) > 0.0f)) r = 0.0f;
        }
        store_elem(dst + v * ld_dst + f, r);
    }
}

int launch_scale_mask_rows(int64_t n, int32_t F, int32_t F_pad, const void *g, const void *h, int64_t ld,
                           const float *inv_deg, bool relu, int32_t dtype, void *dst, int64_t ld_dst,
                           hipStream_t stream)
{
    if (n == 0 || F_pad == 0) return TMA_OK;
    int64_t blocks = ceil_div(n * F_pad, 256);
    if (blocks > 256 * 32) blocks = 256 * 32;
    TMA_TIMED("scale_mask_rows", stream);
    if (dtype == TMA_F32)
        hipLaunchKernelGGL(scale_mask_rows_kernel<float>, dim3(unsigned(blocks)), dim3(256), 0, stream, n, F, F_pad,
                           static_cast<const float *>(g), static_cast<const float *>(h), ld, inv_deg, relu ? 1 : 0,
                           static_cast<float *>(dst), ld_dst);
    else
        hipLaunchKernelGGL(scale_mask_rows_kernel<uint16_t>, dim3(unsigned(blocks)), dim3(256), 0, stream, n, F, F_pad,
                           static_cast<const uint16_t *>(g), static_cast<const uint16_t *>(h), ld, inv_deg,
                           relu ? 1 : 0, static_cast<uint16_t *>(dst), ld_dst);
    return check_launch("scale_mask_rows");
}

}  // namespace tma

extern "C" int tma_mean_aggregate(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg,
                                  const void *H, int64_t ldh, int32_t F, int32_t dtype, void *M_out, int64_t ldm,
                                  tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_mean_aggregate";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX && F >= 0, TMA_ERR_INVALID_ARG, "%s: bad n or F", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n == 0 || F == 0) return TMA_OK;
    TMA_REQUIRE(rowptr && inv_deg && H && M_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    TMA_REQUIRE(ldh >= F && ldm >= F, TMA_ERR_BAD_SHAPE, "%s: leading dimension smaller than F", fn);
    TMA_REQUIRE(H != M_out, TMA_ERR_INVALID_ARG, "%s: in-place aggregation is not supported", fn);
    return launch_spmm(n, rowptr, colidx, inv_deg, H, ldh, F, dtype, M_out, ldm, false, as_stream(stream));
}
