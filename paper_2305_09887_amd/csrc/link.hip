// Link-prediction head (paper Sec. 4.1, paragraphs on the link prediction
// decoder and on mini-batch and negative sampling; App., formulation of the MLP
// decoder): the edge mini-batch with one random-tail negative per positive, the
// decoder input e0(u, v) = r_u (.) r_v and its gradient back into the
// embeddings, the decoder's PReLU, and the binary cross-entropy on its logits.
// The decoder's products run in the dense-layer kernels.  Everything here is
// HBM / latency bound row-wise work.
//
// The gradient of the pair products is a scatter (a node receives a term from
// every sample it takes part in).  It is computed without floating-point
// atomics: the 4B terms are written out as rows of a matrix C, an incidence list
// node -> rows of C is built with integer counting, an exclusive scan and a fill,
// each node's list is sorted, and the streaming row gather sums every node's rows
// in that fixed order.
#include "kernels.hpp"

namespace tma {

__device__ __forceinline__ float ld1(const float *p) { return *p; }
__device__ __forceinline__ float ld1(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st1(float *p, float v) { *p = v; }
__device__ __forceinline__ void st1(uint16_t *p, float v) { *p = f32_to_bf16(v); }

// `kVec`: a row is handled in 16-byte chunks (E elements), else element by element
template <typename T, bool kVec>
struct RowUnit {
    static constexpr int E = kVec ? Chunk<T>::kElems : 1;
    static __device__ __forceinline__ void load(const T *p, float (&v)[E])
    {
        if constexpr (kVec) Chunk<T>::load(p, v);
        else v[0] = ld1(p);
    }
    static __device__ __forceinline__ void store(T *p, const float (&v)[E])
    {
        if constexpr (kVec) Chunk<T>::store(p, v);
        else st1(p, v[0]);
    }
};

// ---- mini-batch ---------------------------------------------------------------------------------
// Sample i uses counter c = first_counter + i:  entry e = floor(z(2c) * nnz / 2^64) of the CSR is the positive
// edge (row of e, colidx[e]); the negative tail is r + (r >= v) with r = floor(z(2c+1) * (n-1) / 2^64).
__global__ __launch_bounds__(256) void edge_batch_kernel(int64_t n, int64_t nnz, const int32_t *__restrict__ rowptr,
                                                         const int32_t *__restrict__ colidx, uint64_t seed,
                                                         uint64_t first_counter, int64_t B, int32_t *__restrict__ u,
                                                         int32_t *__restrict__ v, int32_t *__restrict__ vneg)
{
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= B) return;
    const uint64_t c = first_counter + uint64_t(i);
    const int64_t e = int64_t(__umul64hi(splitmix64_at(seed, 2 * c), uint64_t(nnz)));
    int64_t lo = 0, hi = n;   // rowptr[lo] <= e < rowptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= e) lo = mid;
        else hi = mid;
    }
    const int32_t tail = colidx[e];
    const int64_t r = int64_t(__umul64hi(splitmix64_at(seed, 2 * c + 1), uint64_t(n - 1)));
    u[i] = int32_t(lo);
    v[i] = tail;
    vneg[i] = int32_t(r + (r >= tail ? 1 : 0));
}

// ---- pair products ------------------------------------------------------------------------------
// E0[i] = r_u(i) (.) r_v(i),  E0[B + i] = r_u(i) (.) r_v'(i)
template <typename T, bool kVec>
__global__ __launch_bounds__(256) void pair_product_fwd_kernel(int64_t B, int units, const T *__restrict__ R,
                                                               int64_t ldr, const int32_t *__restrict__ u,
                                                               const int32_t *__restrict__ v,
                                                               const int32_t *__restrict__ vneg, T *__restrict__ E0,
                                                               int64_t lde)
{
    constexpr int E = RowUnit<T, kVec>::E;
    const int64_t total = B * units;
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t w = int64_t(blockIdx.x) * 256 + threadIdx.x; w < total; w += stride) {
        const int64_t i = w / units;
        const int f = int(w - i * units) * E;
        float a[E], b[E], c[E], p[E], q[E];
        RowUnit<T, kVec>::load(R + int64_t(u[i]) * ldr + f, a);
        RowUnit<T, kVec>::load(R + int64_t(v[i]) * ldr + f, b);
        RowUnit<T, kVec>::load(R + int64_t(vneg[i]) * ldr + f, c);
#pragma unroll
        for (int k = 0; k < E; ++k) {
            p[k] = a[k] * b[k];
            q[k] = a[k] * c[k];
        }
        RowUnit<T, kVec>::store(E0 + i * lde + f, p);
        RowUnit<T, kVec>::store(E0 + (B + i) * lde + f, q);
    }
}

// The four terms of sample i, rows 4i .. 4i+3 of C [4B, Fc] (columns F .. Fc-1 zero):
//   4i+0 = dE0[i] (.) r_v -> u     4i+1 = dE0[i] (.) r_u -> v     4i+2 = dE0[B+i] (.) r_v' -> u     4i+3 = dE0[B+i] (.) r_u -> v'
template <typename T, bool kVec>
__global__ __launch_bounds__(256) void pair_product_terms_kernel(int64_t B, int units, int F, const T *__restrict__ R,
                                                                 int64_t ldr, const int32_t *__restrict__ u,
                                                                 const int32_t *__restrict__ v,
                                                                 const int32_t *__restrict__ vneg,
                                                                 const T *__restrict__ dE0, int64_t lde,
                                                                 T *__restrict__ C, int64_t Fc)
{
    constexpr int E = RowUnit<T, kVec>::E;
    const int64_t total = B * units;
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t w = int64_t(blockIdx.x) * 256 + threadIdx.x; w < total; w += stride) {
        const int64_t i = w / units;
        const int f = int(w - i * units) * E;
        float t0[E], t1[E], t2[E], t3[E];
        if (kVec || f < F) {
            float a[E], b[E], c[E], gp[E], gn[E];
            RowUnit<T, kVec>::load(R + int64_t(u[i]) * ldr + f, a);
            RowUnit<T, kVec>::load(R + int64_t(v[i]) * ldr + f, b);
            RowUnit<T, kVec>::load(R + int64_t(vneg[i]) * ldr + f, c);
            RowUnit<T, kVec>::load(dE0 + i * lde + f, gp);
            RowUnit<T, kVec>::load(dE0 + (B + i) * lde + f, gn);
#pragma unroll
            for (int k = 0; k < E; ++k) {
                t0[k] = gp[k] * b[k];
                t1[k] = gp[k] * a[k];
                t2[k] = gn[k] * c[k];
                t3[k] = gn[k] * a[k];
            }
        } else {
#pragma unroll
            for (int k = 0; k < E; ++k) t0[k] = t1[k] = t2[k] = t3[k] = 0.0f;
        }
        T *row = C + 4 * i * Fc + f;
        RowUnit<T, kVec>::store(row, t0);
        RowUnit<T, kVec>::store(row + Fc, t1);
        RowUnit<T, kVec>::store(row + 2 * Fc, t2);
        RowUnit<T, kVec>::store(row + 3 * Fc, t3);
    }
}

__device__ __forceinline__ int32_t term_target(int64_t j, const int32_t *u, const int32_t *v, const int32_t *vneg)
{
    const int64_t i = j >> 2;
    const int role = int(j & 3);
    return role == 1 ? v[i] : (role == 3 ? vneg[i] : u[i]);
}

__global__ __launch_bounds__(256) void fill_zero_i32_kernel(int64_t count, int32_t *__restrict__ p)
{
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < count; i += stride) p[i] = 0;
}

__global__ __launch_bounds__(256) void incidence_count_kernel(int64_t B, const int32_t *__restrict__ u,
                                                              const int32_t *__restrict__ v,
                                                              const int32_t *__restrict__ vneg, int32_t *__restrict__ deg)
{
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= B) return;
    atomicAdd(&deg[u[i]], 2);
    atomicAdd(&deg[v[i]], 1);
    atomicAdd(&deg[vneg[i]], 1);
}

// Places term j somewhere inside its node's range (the order inside a range is settled by the sort below).
__global__ __launch_bounds__(256) void incidence_fill_kernel(int64_t B, const int32_t *__restrict__ u,
                                                             const int32_t *__restrict__ v,
                                                             const int32_t *__restrict__ vneg,
                                                             const int32_t *__restrict__ rowptr,
                                                             int32_t *__restrict__ cursor, int32_t *__restrict__ unsorted)
{
    const int64_t j = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (j >= 4 * B) return;
    const int32_t t = term_target(j, u, v, vneg);
    unsorted[rowptr[t] + atomicAdd(&cursor[t], 1)] = int32_t(j);
}

// sorted[range of node] = the node's term numbers in ascending order.  First kernel: a thread sorts a range of
// up to 8 by insertion and queues longer ranges.  Second kernel: a wavefront per queued range ranks its numbers
// (they are distinct: the rank of a number is the count of smaller ones) from a copy in LDS.  The queue's order
// does not matter: every range is sorted independently.
constexpr int kShortList = 8;
constexpr int kRankLds = 2048;     // entries of a range that fit a wavefront's LDS segment

__global__ __launch_bounds__(256) void incidence_sort_short_kernel(int64_t n, const int32_t *__restrict__ rowptr,
                                                                   const int32_t *__restrict__ unsorted,
                                                                   int32_t *__restrict__ sorted,
                                                                   int32_t *__restrict__ long_rows,
                                                                   int32_t *__restrict__ n_long)
{
    const int64_t r = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int lane = threadIdx.x % kWave;
    int32_t beg = 0, len = 0;
    if (r < n) {
        beg = rowptr[r];
        len = rowptr[r + 1] - beg;
    }
    // one queue reservation per wavefront, not per range (the ranges of hub nodes sit next to each other)
    const bool is_long = len > kShortList;
    const uint64_t longs = __ballot(is_long);
    if (longs != 0) {
        const int leader = __ffsll(static_cast<long long>(longs)) - 1;
        int32_t first = 0;
        if (lane == leader) first = atomicAdd(n_long, int32_t(__popcll(longs)));
        first = __shfl(first, leader, kWave);
        if (is_long) long_rows[first + __popcll(longs & ((uint64_t(1) << lane) - 1))] = int32_t(r);
    }
    if (!is_long && len > 0) {
        int32_t a[kShortList];
#pragma unroll
        for (int k = 0; k < kShortList; ++k) a[k] = k < len ? unsorted[beg + k] : INT32_MAX;
#pragma unroll
        for (int k = 1; k < kShortList; ++k)
#pragma unroll
            for (int m = k; m > 0; --m)
                if (a[m] < a[m - 1]) {
                    const int32_t t = a[m];
                    a[m] = a[m - 1];
                    a[m - 1] = t;
                }
#pragma unroll
        for (int k = 0; k < kShortList; ++k)
            if (k < len) sorted[beg + k] = a[k];
    }
}

__global__ __launch_bounds__(256) void incidence_sort_long_kernel(const int32_t *__restrict__ rowptr,
                                                                  const int32_t *__restrict__ unsorted,
                                                                  int32_t *__restrict__ sorted,
                                                                  const int32_t *__restrict__ long_rows,
                                                                  const int32_t *__restrict__ n_long)
{
    __shared__ __attribute__((aligned(16))) int32_t stage[256 / kWave][kRankLds];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int count = *n_long;
    const int waves = gridDim.x * (256 / kWave);
    for (int q = blockIdx.x * (256 / kWave) + wave; q < count; q += waves) {
        const int32_t row = long_rows[q];
        const int32_t beg = rowptr[row], len = rowptr[row + 1] - beg;
        const bool in_lds = len <= kRankLds;
        const int32_t len4 = (len + 3) & ~3;   // padded with the largest number, which is smaller than nothing
        if (in_lds)
            for (int32_t k = lane; k < len4; k += kWave) stage[wave][k] = k < len ? unsorted[beg + k] : INT32_MAX;
        // a wavefront's LDS accesses complete in program order: its own writes above are visible to the reads below
        __builtin_amdgcn_wave_barrier();
        for (int32_t k = lane; k < len; k += kWave) {
            int32_t rank = 0;
            if (in_lds) {
                const int32_t mine = stage[wave][k];
                const int4 *quads = reinterpret_cast<const int4 *>(&stage[wave][0]);
#pragma unroll 4
                for (int32_t m = 0; m < len4 / 4; ++m) {   // four numbers per LDS read, several reads in flight
                    const int4 t = quads[m];
                    rank += (t.x < mine ? 1 : 0) + (t.y < mine ? 1 : 0) + (t.z < mine ? 1 : 0) + (t.w < mine ? 1 : 0);
                }
                sorted[beg + rank] = mine;
            } else {
                const int32_t mine = unsorted[beg + k];
#pragma unroll 8
                for (int32_t m = 0; m < len; ++m) rank += unsorted[beg + m] < mine ? 1 : 0;
                sorted[beg + rank] = mine;
            }
        }
        __builtin_amdgcn_wave_barrier();   // before the segment is overwritten by the next range
    }
}

// sorted[range r] = unsorted[range r] in ascending order for every range of rowptr (n ranges).  queue: n int32
// of scratch; counter: one int32 that is ZERO on entry.
int launch_sort_lists(int64_t n, const int32_t *rowptr, const int32_t *unsorted, int32_t *sorted, int32_t *queue,
                      int32_t *counter, hipStream_t s)
{
    if (n <= 0) return TMA_OK;
    {
        TMA_TIMED("incidence_sort_short", s);
        hipLaunchKernelGGL(incidence_sort_short_kernel, dim3(unsigned(ceil_div(n, 256))), dim3(256), 0, s, n, rowptr,
                           unsorted, sorted, queue, counter);
    }
    TMA_TIMED("incidence_sort_long", s);
    hipLaunchKernelGGL(incidence_sort_long_kernel, dim3(1024), dim3(256), 0, s, rowptr, unsorted, sorted, queue, counter);
    return check_launch("sort lists");
}

// ---- PReLU with one learnable slope ---------------------------------------------------------------
template <typename T, bool kVec>
__global__ __launch_bounds__(256) void prelu_fwd_kernel(int64_t n, int units, const T *__restrict__ Z, int64_t ldz,
                                                        const float *__restrict__ slope, T *__restrict__ Y, int64_t ldy)
{
    constexpr int E = RowUnit<T, kVec>::E;
    const float a = *slope;
    const int64_t total = n * units;
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t w = int64_t(blockIdx.x) * 256 + threadIdx.x; w < total; w += stride) {
        const int64_t i = w / units;
        const int f = int(w - i * units) * E;
        float z[E];
        RowUnit<T, kVec>::load(Z + i * ldz + f, z);
#pragma unroll
        for (int k = 0; k < E; ++k) z[k] = z[k] > 0.0f ? z[k] : a * z[k];
        RowUnit<T, kVec>::store(Y + i * ldy + f, z);
    }
}

constexpr int kPreluMaxBlocks = 1024;

// dZ = dY (.) (Z > 0 ? 1 : a);  partial[block] = sum of dY * Z over the block's entries with Z <= 0
template <typename T, bool kVec>
__global__ __launch_bounds__(256) void prelu_bwd_kernel(int64_t n, int units, const T *__restrict__ Z, int64_t ldz,
                                                        const T *__restrict__ dY, int64_t ldd,
                                                        const float *__restrict__ slope, T *__restrict__ dZ,
                                                        int64_t ld_dz, float *__restrict__ partial)
{
    constexpr int E = RowUnit<T, kVec>::E;
    __shared__ float red[256];
    const float a = *slope;
    const int64_t total = n * units;
    const int64_t stride = int64_t(gridDim.x) * 256;
    float da = 0.0f;
    for (int64_t w = int64_t(blockIdx.x) * 256 + threadIdx.x; w < total; w += stride) {
        const int64_t i = w / units;
        const int f = int(w - i * units) * E;
        float z[E], g[E];
        RowUnit<T, kVec>::load(Z + i * ldz + f, z);
        RowUnit<T, kVec>::load(dY + i * ldd + f, g);
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const bool open = z[k] > 0.0f;
            da += open ? 0.0f : g[k] * z[k];
            g[k] = open ? g[k] : a * g[k];
        }
        RowUnit<T, kVec>::store(dZ + i * ld_dz + f, g);
    }
    red[threadIdx.x] = da;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {   // fixed tree
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// ---- binary cross-entropy on logits ---------------------------------------------------------------
// loss = mean_i softplus(y_i ? -z_i : z_i),  dz_i = (sigmoid(z_i) - y_i) / count;  y_i = [i < n_pos]
template <typename T>
__global__ __launch_bounds__(256) void bce_logits_kernel(int64_t count, int64_t n_pos, const T *__restrict__ z,
                                                         int64_t ldz, T *__restrict__ dz, int64_t ld_dz,
                                                         float *__restrict__ partial)
{
    __shared__ float red[256];
    const float inv = 1.0f / float(count);
    const int64_t stride = int64_t(gridDim.x) * 256;
    float acc = 0.0f;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < count; i += stride) {
        const float x = ld1(z + i * ldz);
        const bool pos = i < n_pos;
        const float t = pos ? -x : x;
        acc += (t > 0.0f ? t + log1pf(expf(-t)) : log1pf(expf(t))) * inv;
        if (dz) {
            const float sg = x >= 0.0f ? 1.0f / (1.0f + expf(-x)) : expf(x) / (1.0f + expf(x));
            st1(dz + i * ld_dz, (sg - (pos ? 1.0f : 0.0f)) * inv);
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// ---- host side ------------------------------------------------------------------------------------
static size_t elem_size(int32_t dtype) { return dtype == TMA_BF16 ? 2 : 4; }
static int pad_cols(int32_t F, int32_t dtype) { return int(round_up(size_t(F), dtype == TMA_BF16 ? 8 : 4)); }
static unsigned capped_blocks(int64_t work) { return unsigned(work < 1 ? 1 : (work > 256 * 64 ? 256 * 64 : work)); }

struct PairBwdWorkspace {
    size_t terms_bytes, deg_bytes, rowptr_bytes, list_bytes, scan_bytes;
    size_t total() const { return terms_bytes + deg_bytes + rowptr_bytes + 2 * list_bytes + scan_bytes; }
};

static PairBwdWorkspace plan_pair_bwd(int64_t n, int64_t B, int32_t F, int32_t dtype)
{
    PairBwdWorkspace w;
    const size_t b = size_t(B > 0 ? B : 1), rows = size_t(n > 0 ? n : 1);
    w.terms_bytes = round_up(4 * b * size_t(pad_cols(F, dtype)) * elem_size(dtype), 256);
    w.deg_bytes = round_up((2 * rows + 1) * 4, 256);    // per-node counts (later the queue of long lists), fill cursors, queue length
    w.rowptr_bytes = round_up((rows + 1) * 4, 256);
    w.list_bytes = round_up(4 * b * 4, 256);            // unsorted and sorted term lists
    w.scan_bytes = exclusive_scan_i32_workspace_bytes(n);
    return w;
}

template <typename T>
static bool rows_vec_ok(const T *p, int64_t ld) { return aligned(p, 16) && (size_t(ld) * sizeof(T)) % 16 == 0; }

}  // namespace tma

extern "C" int tma_edge_batch(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, uint64_t seed,
                              uint64_t first_counter, int64_t B, int32_t *u_out, int32_t *v_out, int32_t *vneg_out,
                              tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_edge_batch";
    TMA_REQUIRE(B >= 0 && n >= 0 && n <= INT32_MAX && nnz >= 0 && nnz <= INT32_MAX, TMA_ERR_INVALID_ARG,
                "%s: negative or oversized argument", fn);
    if (B == 0) return TMA_OK;
    TMA_REQUIRE(n >= 2 && nnz >= 1, TMA_ERR_INVALID_ARG,
                "%s: a batch needs at least one edge and two nodes (n=%lld, nnz=%lld)", fn, (long long)n, (long long)nnz);
    TMA_REQUIRE(rowptr && colidx && u_out && v_out && vneg_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    hipStream_t s = as_stream(stream);
    TMA_TIMED("edge_batch", s);
    hipLaunchKernelGGL(edge_batch_kernel, dim3(unsigned(ceil_div(B, 256))), dim3(256), 0, s, n, nnz, rowptr, colidx, seed,
                       first_counter, B, u_out, v_out, vneg_out);
    return check_launch(fn);
}

extern "C" int tma_pair_product_fwd(int64_t B, int32_t F, const void *R, int64_t ldr, int32_t dtype, const int32_t *u,
                                    const int32_t *v, const int32_t *vneg, void *E0_out, int64_t lde,
                                    tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_pair_product_fwd";
    TMA_REQUIRE(B >= 0 && 2 * B <= INT32_MAX && F >= 1 && F <= (1 << 20), TMA_ERR_BAD_SHAPE, "%s: B or F", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (B == 0) return TMA_OK;
    TMA_REQUIRE(R && u && v && vneg && E0_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    TMA_REQUIRE(ldr >= F && lde >= F, TMA_ERR_BAD_SHAPE, "%s: leading dimension smaller than F", fn);
    hipStream_t s = as_stream(stream);
    TMA_TIMED("pair_product_fwd", s);
    if (dtype == TMA_F32) {
        const float *r = static_cast<const float *>(R);
        float *e = static_cast<float *>(E0_out);
        if (F % 4 == 0 && rows_vec_ok(r, ldr) && rows_vec_ok(e, lde))
            hipLaunchKernelGGL((pair_product_fwd_kernel<float, true>), dim3(capped_blocks(ceil_div(B * (F / 4), 256))),
                               dim3(256), 0, s, B, F / 4, r, ldr, u, v, vneg, e, lde);
        else
            hipLaunchKernelGGL((pair_product_fwd_kernel<float, false>), dim3(capped_blocks(ceil_div(B * F, 256))), dim3(256),
                               0, s, B, F, r, ldr, u, v, vneg, e, lde);
    } else {
        const uint16_t *r = static_cast<const uint16_t *>(R);
        uint16_t *e = static_cast<uint16_t *>(E0_out);
        if (F % 8 == 0 && rows_vec_ok(r, ldr) && rows_vec_ok(e, lde))
            hipLaunchKernelGGL((pair_product_fwd_kernel<uint16_t, true>), dim3(capped_blocks(ceil_div(B * (F / 8), 256))),
                               dim3(256), 0, s, B, F / 8, r, ldr, u, v, vneg, e, lde);
        else
            hipLaunchKernelGGL((pair_product_fwd_kernel<uint16_t, false>), dim3(capped_blocks(ceil_div(B * F, 256))),
                               dim3(256), 0, s, B, F, r, ldr, u, v, vneg, e, lde);
    }
    return check_launch(fn);
}

extern "C" size_t tma_pair_product_bwd_workspace_bytes(int64_t n, int64_t B, int32_t F, int32_t dtype)
{
    if (n < 0 || B < 0 || F < 1) return 0;
    return tma::plan_pair_bwd(n, B, F, dtype).total();
}

extern "C" int tma_pair_product_bwd(int64_t n, int64_t B, int32_t F, const void *R, int64_t ldr, int32_t dtype,
                                    const int32_t *u, const int32_t *v, const int32_t *vneg, const void *dE0,
                                    int64_t lde, void *dR_out, int64_t ld_dr, void *ws, size_t ws_bytes,
                                    tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_pair_product_bwd";
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX && B >= 0 && 4 * B <= INT32_MAX && F >= 1 && F <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: n, B or F", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n == 0) return TMA_OK;
    TMA_REQUIRE(dR_out && ld_dr >= F, TMA_ERR_INVALID_ARG, "%s: dR_out NULL or its leading dimension smaller than F", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    const PairBwdWorkspace w = plan_pair_bwd(n, B, F, dtype);
    TMA_REQUIRE(ws_bytes >= w.total(), TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, ws_bytes,
                w.total());
    if (B > 0) {
        TMA_REQUIRE(R && u && v && vneg && dE0, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
        TMA_REQUIRE(ldr >= F && lde >= F, TMA_ERR_BAD_SHAPE, "%s: leading dimension smaller than F", fn);
    }
    hipStream_t s = as_stream(stream);
    char *base = static_cast<char *>(ws);
    void *terms = base;
    int32_t *deg = reinterpret_cast<int32_t *>(base + w.terms_bytes);
    int32_t *cursor = deg + n;
    int32_t *rowptr = reinterpret_cast<int32_t *>(base + w.terms_bytes + w.deg_bytes);
    int32_t *unsorted = reinterpret_cast<int32_t *>(base + w.terms_bytes + w.deg_bytes + w.rowptr_bytes);
    int32_t *sorted = reinterpret_cast<int32_t *>(base + w.terms_bytes + w.deg_bytes + w.rowptr_bytes + w.list_bytes);
    void *scan_ws = base + w.terms_bytes + w.deg_bytes + w.rowptr_bytes + 2 * w.list_bytes;
    const int Fc = pad_cols(F, dtype);

    {
        TMA_TIMED("incidence_count", s);
        hipLaunchKernelGGL(fill_zero_i32_kernel, dim3(capped_blocks(ceil_div(2 * n + 1, 256))), dim3(256), 0, s, 2 * n + 1,
                           deg);
        if (B > 0)
            hipLaunchKernelGGL(incidence_count_kernel, dim3(unsigned(ceil_div(B, 256))), dim3(256), 0, s, B, u, v, vneg,
                               deg);
    }
    if (int rc = check_launch(fn)) return rc;
    if (int rc = launch_exclusive_scan_i32(n, deg, rowptr, scan_ws, s)) return rc;
    if (B > 0) {
        {
            TMA_TIMED("incidence_fill", s);
            hipLaunchKernelGGL(incidence_fill_kernel, dim3(unsigned(ceil_div(4 * B, 256))), dim3(256), 0, s, B, u, v, vneg,
                               rowptr, cursor, unsorted);
        }
        // the per-node counts are spent once the scan has run: their array takes the queue of long lists
        if (int rc = launch_sort_lists(n, rowptr, unsorted, sorted, deg, deg + 2 * n, s)) return rc;
        TMA_TIMED("pair_product_terms", s);
        if (dtype == TMA_F32) {
            const float *r = static_cast<const float *>(R), *g = static_cast<const float *>(dE0);
            float *c = static_cast<float *>(terms);
            if (F % 4 == 0 && rows_vec_ok(r, ldr) && rows_vec_ok(g, lde))
                hipLaunchKernelGGL((pair_product_terms_kernel<float, true>), dim3(capped_blocks(ceil_div(B * (F / 4), 256))),
                                   dim3(256), 0, s, B, F / 4, F, r, ldr, u, v, vneg, g, lde, c, int64_t(Fc));
            else
                hipLaunchKernelGGL((pair_product_terms_kernel<float, false>), dim3(capped_blocks(ceil_div(B * Fc, 256))),
                                   dim3(256), 0, s, B, Fc, F, r, ldr, u, v, vneg, g, lde, c, int64_t(Fc));
        } else {
            const uint16_t *r = static_cast<const uint16_t *>(R), *g = static_cast<const uint16_t *>(dE0);
            uint16_t *c = static_cast<uint16_t *>(terms);
            if (F % 8 == 0 && rows_vec_ok(r, ldr) && rows_vec_ok(g, lde))
                hipLaunchKernelGGL((pair_product_terms_kernel<uint16_t, true>),
                                   dim3(capped_blocks(ceil_div(B * (F / 8), 256))), dim3(256), 0, s, B, F / 8, F, r, ldr, u,
                                   v, vneg, g, lde, c, int64_t(Fc));
            else
                hipLaunchKernelGGL((pair_product_terms_kernel<uint16_t, false>), dim3(capped_blocks(ceil_div(B * Fc, 256))),
                                   dim3(256), 0, s, B, Fc, F, r, ldr, u, v, vneg, g, lde, c, int64_t(Fc));
        }
        if (int rc = check_launch(fn)) return rc;
    }
    // dR_v = sum of the node's terms, in ascending term order; nodes outside the batch receive zeros
    const int F_rows = ld_dr >= Fc ? Fc : F;
    return launch_spmm(n, rowptr, sorted, nullptr, terms, Fc, F_rows, dtype, dR_out, ld_dr, false, s, B > 0 ? 4 * B : 1);
}

extern "C" int tma_prelu_fwd(int64_t n, int32_t F, const void *Z, int64_t ldz, const float *slope, int32_t dtype,
                             void *Y_out, int64_t ldy, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_prelu_fwd";
    TMA_REQUIRE(n >= 0 && F >= 1 && F <= (1 << 20), TMA_ERR_BAD_SHAPE, "%s: n or F", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n == 0) return TMA_OK;
    TMA_REQUIRE(Z && slope && Y_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    TMA_REQUIRE(ldz >= F && ldy >= F, TMA_ERR_BAD_SHAPE, "%s: leading dimension smaller than F", fn);
    hipStream_t s = as_stream(stream);
    TMA_TIMED("prelu_fwd", s);
    if (dtype == TMA_F32) {
        const float *z = static_cast<const float *>(Z);
        float *y = static_cast<float *>(Y_out);
        if (F % 4 == 0 && rows_vec_ok(z, ldz) && rows_vec_ok(y, ldy))
            hipLaunchKernelGGL((prelu_fwd_kernel<float, true>), dim3(capped_blocks(ceil_div(n * (F / 4), 256))), dim3(256),
                               0, s, n, F / 4, z, ldz, slope, y, ldy);
        else
            hipLaunchKernelGGL((prelu_fwd_kernel<float, false>), dim3(capped_blocks(ceil_div(n * F, 256))), dim3(256), 0, s,
                               n, F, z, ldz, slope, y, ldy);
    } else {
        const uint16_t *z = static_cast<const uint16_t *>(Z);
        uint16_t *y = static_cast<uint16_t *>(Y_out);
        if (F % 8 == 0 && rows_vec_ok(z, ldz) && rows_vec_ok(y, ldy))
            hipLaunchKernelGGL((prelu_fwd_kernel<uint16_t, true>), dim3(capped_blocks(ceil_div(n * (F / 8), 256))),
                               dim3(256), 0, s, n, F / 8, z, ldz, slope, y, ldy);
        else
            hipLaunchKernelGGL((prelu_fwd_kernel<uint16_t, false>), dim3(capped_blocks(ceil_div(n * F, 256))), dim3(256), 0,
                               s, n, F, z, ldz, slope, y, ldy);
    }
    return check_launch(fn);
}

extern "C" size_t tma_prelu_bwd_workspace_bytes(void) { return size_t(tma::kPreluMaxBlocks) * sizeof(float); }

extern "C" int tma_prelu_bwd(int64_t n, int32_t F, const void *Z, int64_t ldz, const void *dY, int64_t ldd,
                             const float *slope, int32_t dtype, void *dZ_out, int64_t ld_dz, float *dslope_out, void *ws,
                             size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_prelu_bwd";
    TMA_REQUIRE(n >= 0 && F >= 1 && F <= (1 << 20), TMA_ERR_BAD_SHAPE, "%s: n or F", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(dslope_out && ws && aligned(ws, 16) && ws_bytes >= tma_prelu_bwd_workspace_bytes(), TMA_ERR_INVALID_ARG,
                "%s: dslope_out / workspace", fn);
    hipStream_t s = as_stream(stream);
    float *partial = static_cast<float *>(ws);
    int blocks = 0;
    if (n > 0) {
        TMA_REQUIRE(Z && dY && slope && dZ_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
        TMA_REQUIRE(ldz >= F && ldd >= F && ld_dz >= F, TMA_ERR_BAD_SHAPE, "%s: leading dimension smaller than F", fn);
        TMA_TIMED("prelu_bwd", s);
#define TMA_PRELU_BWD(T_, V_, UNITS_)                                                                                  \
    do {                                                                                                               \
        int64_t b_ = ceil_div(n * int64_t(UNITS_), 256 * 4);                                                           \
        blocks = int(b_ < 1 ? 1 : (b_ > kPreluMaxBlocks ? kPreluMaxBlocks : b_));                                      \
        hipLaunchKernelGGL((prelu_bwd_kernel<T_, V_>), dim3(unsigned(blocks)), dim3(256), 0, s, n, UNITS_,             \
                           static_cast<const T_ *>(Z), ldz, static_cast<const T_ *>(dY), ldd, slope,                   \
                           static_cast<T_ *>(dZ_out), ld_dz, partial);                                                 \
    } while (0)
        if (dtype == TMA_F32) {
            if (F % 4 == 0 && rows_vec_ok(static_cast<const float *>(Z), ldz) &&
                rows_vec_ok(static_cast<const float *>(dY), ldd) && rows_vec_ok(static_cast<float *>(dZ_out), ld_dz))
                TMA_PRELU_BWD(float, true, F / 4);
            else
                TMA_PRELU_BWD(float, false, F);
        } else {
            if (F % 8 == 0 && rows_vec_ok(static_cast<const uint16_t *>(Z), ldz) &&
                rows_vec_ok(static_cast<const uint16_t *>(dY), ldd) && rows_vec_ok(static_cast<uint16_t *>(dZ_out), ld_dz))
                TMA_PRELU_BWD(uint16_t, true, F / 8);
            else
                TMA_PRELU_BWD(uint16_t, false, F);
        }
#undef TMA_PRELU_BWD
        if (int rc = check_launch(fn)) return rc;
    }
    return launch_sum_partials(blocks, 1, 1, partial, dslope_out, s);
}

extern "C" size_t tma_bce_logits_workspace_bytes(void) { return size_t(tma::kPreluMaxBlocks) * sizeof(float); }

extern "C" int tma_bce_logits(int64_t count, int64_t n_pos, const void *z, int64_t ldz, int32_t dtype, float *loss_out,
                              void *dz_out, int64_t ld_dz, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_bce_logits";
    TMA_REQUIRE(count >= 0 && n_pos >= 0 && n_pos <= count, TMA_ERR_INVALID_ARG, "%s: count / n_pos", fn);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(loss_out && ws && aligned(ws, 16) && ws_bytes >= tma_bce_logits_workspace_bytes(), TMA_ERR_INVALID_ARG,
                "%s: loss_out / workspace", fn);
    hipStream_t s = as_stream(stream);
    float *partial = static_cast<float *>(ws);
    int blocks = 0;
    if (count > 0) {
        TMA_REQUIRE(z && ldz >= 1 && (!dz_out || ld_dz >= 1), TMA_ERR_INVALID_ARG, "%s: NULL logits or bad stride", fn);
        const int64_t b = ceil_div(count, 256 * 2);
        blocks = int(b < 1 ? 1 : (b > kPreluMaxBlocks ? kPreluMaxBlocks : b));
        TMA_TIMED("bce_logits", s);
        if (dtype == TMA_F32)
            hipLaunchKernelGGL(bce_logits_kernel<float>, dim3(unsigned(blocks)), dim3(256), 0, s, count, n_pos,
                               static_cast<const float *>(z), ldz, static_cast<float *>(dz_out), ld_dz, partial);
        else
            hipLaunchKernelGGL(bce_logits_kernel<uint16_t>, dim3(unsigned(blocks)), dim3(256), 0, s, count, n_pos,
                               static_cast<const uint16_t *>(z), ldz, static_cast<uint16_t *>(dz_out), ld_dz, partial);
        if (int rc = check_launch(fn)) return rc;
    }
    return launch_sum_partials(blocks, 1, 1, partial, loss_out, s);
}
