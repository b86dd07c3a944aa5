// Mean aggregation  M = Abar H  (paper Thm. 1, first equation of its proof) and
// the plain row gather-sum used by the backward pass.  HBM/gather bound: the
// flops (2 per gathered element) are negligible.
//
// Mapping.  A feature row is cut into 16-byte chunks; G lanes (one per chunk; any
// G up to the 64-lane wavefront, 64 / G rows share a wavefront) own one row and
// each lane keeps its chunk of the running sum in registers, so every neighbour
// row is fetched with one coalesced 16-byte load per lane.
//
// Local graphs under random assignment are very sparse (mean local degree 2-5)
// with a power-law tail.  Two things follow.  (1) A row is too short to hide a
// memory latency by itself, so a lane group walks through its rows as one
// stream of steps of up to four neighbours and runs that stream as a three-stage
// pipeline: the neighbour ids of step s+2, the feature loads of step s+1 and the
// additions of step s are in flight together, across row boundaries.  (2) A
// group can only pull a few loads per latency, so a long row would become the
// tail of the launch: rows longer than a threshold (a multiple of the mean
// degree) are deferred and then summed by all groups of the workgroup together,
// each taking one contiguous share, with a fixed-order combine through LDS.  The
// result of a row depends only on its own neighbour list, never on scheduling.
//
// Every load in the pipeline is issued unconditionally (an unused slot repeats an
// address that was just fetched): the wait counters are then exact and a wait for
// step s never also waits for the loads of step s+1.
#include "kernels.hpp"

namespace tma {

constexpr int kSpmmThreads = 256;
constexpr int kDies = 8;           // accelerator dies (XCDs) of the chip
constexpr int kRowsPerGroup = 4;   // rows a lane group walks through per block
constexpr int kHubDegree = 48;     // rows longer than this are summed by the whole workgroup

__device__ __forceinline__ float load_elem(const float *p) { return *p; }
__device__ __forceinline__ float load_elem(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store_elem(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(uint16_t *p, float v) { *p = f32_to_bf16(v); }

// U neighbour rows (entries j .. j+U-1 of the run whose ids sit in `mine`) fetched together, then added in order.
template <typename T, int G, int CPL, int U>
__device__ __forceinline__ void gather_batch(const T *__restrict__ in, int64_t ld, int32_t mine, int j, int sub,
                                             int n_chunks, const float *__restrict__ edge_scale,
                                             float (&acc)[CPL][Chunk<T>::kElems])
{
    constexpr int E = Chunk<T>::kElems;
    float v[U][CPL][E];
    float w[U];
#pragma unroll
    for (int q = 0; q < U; ++q) {
        const int32_t id = __shfl(mine, j + q, G);
        w[q] = edge_scale ? edge_scale[id] : 1.0f;
        const T *row = in + int64_t(id) * ld;
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
                for (int i = 0; i < E; ++i) acc[c][i] += edge_scale ? w[q] * v[q][c][i] : v[q][c][i];
}

// Adds the rows colidx[e] for e = beg, beg+1, ... in runs of G entries that start
// `run_stride` entries apart.  Every lane of the group gets the same trip counts.
// kDeep: up to 16 rows in flight per lane (long rows are latency bound: a 500-entry
// row walked four loads at a time sets the kernel's tail).
template <typename T, int G, int CPL, bool kDeep>
__device__ __forceinline__ void gather_sum(const T *__restrict__ in, int64_t ld, const int32_t *__restrict__ colidx,
                                           int32_t beg, int32_t end, int32_t run_stride, int sub, int n_chunks,
                                           const float *__restrict__ edge_scale,
                                           float (&acc)[CPL][Chunk<T>::kElems])
{
    for (int32_t e0 = beg; e0 < end; e0 += run_stride) {
        const int cnt = (end - e0) < G ? (end - e0) : G;
        const int32_t mine = sub < cnt ? colidx[e0 + sub] : 0;
        int j = 0;
        if constexpr (kDeep && CPL == 1 && G >= 16)
            for (; j + 16 <= cnt; j += 16) gather_batch<T, G, CPL, 16>(in, ld, mine, j, sub, n_chunks, edge_scale, acc);
        for (; j + 4 <= cnt; j += 4) gather_batch<T, G, CPL, 4>(in, ld, mine, j, sub, n_chunks, edge_scale, acc);
        for (; j < cnt; ++j) gather_batch<T, G, CPL, 1>(in, ld, mine, j, sub, n_chunks, edge_scale, acc);
    }
}

// What happens to a finished row sum s_v:
//   out_v = act( scale_v * s_v  [+ out_v]  [+ self_v]  [+ bias] )
//   out_v = act( scale_v * (s_v  [+ out_v]  [+ self_v])  [+ bias] )      with scale_all
// With edge_scale the sum is s_v = sum_u edge_scale[u] in_u and self_v stands for edge_scale[v] self_v
// (GCN aggregation S (A + I) S H in one pass over the unscaled H).
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
    int scale_all;  // the scale multiplies the sum with "+ out_v" / "+ self_v" already added (GCN: s_v (sum + self_v))
    const float *edge_scale;  // neighbour u enters the sum as edge_scale[u] * in_u, and self_v as edge_scale[v] * self_v
    int64_t in_rows;          // rows of the gathered matrix (>= 1): filler loads stay below it
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
            for (int i = 0; i < E; ++i) r[i] = o.scale_all ? acc[c][i] : acc[c][i] * scale;
            if (o.accumulate) {
                float old[E];
                Chunk<T>::load(dst, old);
#pragma unroll
                for (int i = 0; i < E; ++i) r[i] += old[i];
            }
            if (o.self) {
                float sv[E];
                Chunk<T>::load(o.self + v * o.ld_self + f0, sv);
                const float ws = o.edge_scale ? o.edge_scale[v] : 1.0f;
#pragma unroll
                for (int i = 0; i < E; ++i) r[i] += ws * sv[i];
            }
            if (o.scale_all) {
#pragma unroll
                for (int i = 0; i < E; ++i) r[i] *= scale;
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

// ---------------------------------------------------------------------------------------------------
// Rows of at most 64 chunks: the streaming kernel.

constexpr int kStreamU = 4;              // neighbours per step
constexpr int kMinDefer = 24;            // rows up to this length are never deferred
constexpr int kDeferFactor = 4;          // ... nor rows up to this multiple of the mean degree
constexpr int kMaxRowsPerBlock = 1024;   // rows of one workgroup (row bounds and deferred-row list sit in LDS)
constexpr int kPartialBytes = 16384;     // LDS for the partial sums of deferred rows

// One step of a group's stream: add the rows ids[lo .. hi) (hi - lo <= kStreamU) to the running sum of
// segment `seg`; `last` closes the segment.  seg < 0: nothing left (the loads of such a step are dummies).
struct Step {
    int32_t lo, hi, seg;
    bool last;
};

template <int U>
__device__ __forceinline__ void issue_ids(const int32_t *__restrict__ ids, int32_t last_entry, const Step &s,
                                          int32_t (&I)[U])
{
    // an unused slot repeats the step's last entry; a step without entries reads any valid entry
    const int32_t filler = s.hi > s.lo ? s.hi - 1 : (s.lo < last_entry ? s.lo : last_entry);
#pragma unroll
    for (int q = 0; q < U; ++q) I[q] = ids[s.lo + q < s.hi ? s.lo + q : filler];
}

// kEdge: every neighbour row comes with a weight edge_scale[id], fetched next to the row
template <typename T, int U, bool kEdge>
__device__ __forceinline__ void issue_gathers(const T *__restrict__ in, int64_t ld, const float *__restrict__ edge_scale,
                                              const Step &s, const int32_t (&I)[U], int32_t &recent, int sub,
                                              uint4 (&V)[U], float (&Wt)[U])
{
    constexpr int E = Chunk<T>::kElems;
#pragma unroll
    for (int q = 0; q < U; ++q) {
        recent = s.lo + q < s.hi ? I[q] : recent;   // unused slot: a row this group fetched a moment ago
        V[q] = *reinterpret_cast<const uint4 *>(in + int64_t(recent) * ld + sub * E);
        if constexpr (kEdge) Wt[q] = edge_scale[recent];
    }
}

template <typename T, int U, bool kEdge>
__device__ __forceinline__ void consume(const Step &s, const uint4 (&V)[U], const float (&Wt)[U],
                                        float (&acc)[Chunk<T>::kElems])
{
    constexpr int E = Chunk<T>::kElems;
#pragma unroll
    for (int q = 0; q < U; ++q) {
        float v[E];
        Chunk<T>::widen(V[q], v);
        const bool used = s.lo + q < s.hi;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += used ? (kEdge ? Wt[q] * v[i] : v[i]) : 0.0f;
    }
}

// What a row's output needs besides the sum, fetched together with the row's last gathers.
struct RowExtra {
    float scale;
    uint4 raw;
};

// Runs the steps that `gen` hands out through the ids -> gathers -> additions pipeline.  `extra(seg, X)`
// issues the loads a closing step needs (or nothing); `emit(seg, acc, X)` takes a finished segment.
template <typename T, bool kEdge, typename Gen, typename Extra, typename Emit>
__device__ __forceinline__ void stream_segments(const T *__restrict__ in, int64_t ld, const int32_t *__restrict__ ids,
                                                const float *__restrict__ edge_scale, int32_t last_entry, int sub,
                                                int32_t recent, Gen &&gen, Extra &&extra, Emit &&emit)
{
    constexpr int E = Chunk<T>::kElems;
    constexpr int U = kStreamU;
    int32_t I0[U], I1[U];
    uint4 V0[U], V1[U];
    float W0[U], W1[U];
    RowExtra X0, X1;
    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.0f;

    Step a = gen();
    issue_ids<U>(ids, last_entry, a, I0);
    Step b = gen();
    issue_ids<U>(ids, last_entry, b, I1);
    issue_gathers<T, U, kEdge>(in, ld, edge_scale, a, I0, recent, sub, V0, W0);
    extra(a.seg, X0);
    // entering a half: step a has its gathers in flight (V0/X0 in the first half), step b its ids (I1)
    auto half = [&](int32_t (&Ia)[U], int32_t (&Ib)[U], uint4 (&Va)[U], uint4 (&Vb)[U], float (&Wa)[U],
                    float (&Wb)[U], RowExtra &Xa, RowExtra &Xb) __attribute__((always_inline)) {
        const Step c = gen();
        issue_ids<U>(ids, last_entry, c, Ia);
        issue_gathers<T, U, kEdge>(in, ld, edge_scale, b, Ib, recent, sub, Vb, Wb);
        extra(b.seg, Xb);
        consume<T, U, kEdge>(a, Va, Wa, acc);
        if (a.last) {
            emit(a.seg, acc, Xa);
#pragma unroll
            for (int i = 0; i < E; ++i) acc[i] = 0.0f;
        }
        a = b;
        b = c;
    };
    while (a.seg >= 0) {
        half(I0, I1, V0, V1, W0, W1, X0, X1);
        if (a.seg < 0) break;
        half(I1, I0, V1, V0, W1, W0, X1, X0);
    }
}

// kExtra: 0 = nothing, 1 = "+ self_v", 2 = "+ out_v" (accumulate).  kScale: multiply by inv_deg[v].
// kEdge: weighted neighbours (and self row), see SpmmOut::edge_scale.
template <typename T, int kExtra, bool kScale, bool kEdge = false>
__global__ __launch_bounds__(kSpmmThreads) void spmm_stream_kernel(int64_t n, const int32_t *__restrict__ rowptr,
                                                                   const int32_t *__restrict__ colidx,
                                                                   const T *__restrict__ in, int64_t ld_in,
                                                                   SpmmOut<T> o, int G, int rows_per_group,
                                                                   int min_defer)
{
    constexpr int E = Chunk<T>::kElems;
    constexpr int U = kStreamU;
    constexpr int kHubsPerPass = kPartialBytes / (kSpmmThreads * E * int(sizeof(float)));
    __shared__ int32_t bounds[kMaxRowsPerBlock + 1];   // rowptr of the workgroup's rows
    __shared__ int32_t deferred[kMaxRowsPerBlock];
    __shared__ int32_t n_deferred;
    __shared__ int32_t total_entries;
    __shared__ float partial[kPartialBytes / sizeof(float)];

    const int lane = threadIdx.x % kWave;
    const int gpw = kWave / G;                       // groups per wavefront
    const int gl = lane / G;
    const bool live = gl < gpw;                      // lanes past the last whole group idle
    const int sub = lane - gl * G;
    const int NG = (kSpmmThreads / kWave) * gpw;
    const int grp = (threadIdx.x / kWave) * gpw + gl;

    const int rows_per_block = NG * rows_per_group;  // <= kMaxRowsPerBlock
    // Workgroups are dealt round-robin to the 8 dies, each with an L2 of its own.  Die d takes the d-th eighth of
    // the row range (the grid is a multiple of 8): rows with neighbouring ids, which on a clustered graph gather
    // from the same few hundred rows, then share one L2 instead of filling all eight with the same lines.
    const int64_t per_die = gridDim.x / kDies;
    const int64_t base = (int64_t(blockIdx.x % kDies) * per_die + blockIdx.x / kDies) * rows_per_block;
    if (base >= n) return;
    const int block_rows = int((n - base) < rows_per_block ? (n - base) : rows_per_block);   // >= 1
    for (int i = threadIdx.x; i <= block_rows; i += kSpmmThreads) bounds[i] = rowptr[base + i];
    if (threadIdx.x == 0) {
        n_deferred = 0;
        total_entries = rowptr[n];
    }
    __syncthreads();
    const int32_t nnz = total_entries;
    const int32_t *ids = nnz > 0 ? colidx : rowptr;   // readable at index 0 even without entries
    const int32_t last_entry = nnz > 0 ? nnz - 1 : 0;
    const int64_t by_mean = int64_t(kDeferFactor) * (int64_t(nnz) / n);
    const int32_t defer_above = by_mean > min_defer ? int32_t(by_mean < INT32_MAX ? by_mean : INT32_MAX) : min_defer;

    // ---- the group's own rows, block-local indices [r, r_end)
    int r = live ? grp * rows_per_group : block_rows;
    const int r_end = (r + rows_per_group) < block_rows ? (r + rows_per_group) : block_rows;
    const int r_first = r < block_rows ? r : 0;
    int32_t e = r < r_end ? bounds[r] : 0;
    bool fresh = true;
    auto next_row_step = [&]() {
        Step s{0, 0, -1, false};
        while (r < r_end) {
            const int32_t end = bounds[r + 1];
            if (fresh && end - e > defer_above) {
                if (sub == 0) deferred[atomicAdd(&n_deferred, 1)] = r;
                ++r;
                e = end;
                continue;
            }
            s.seg = r;
            s.lo = e;
            s.hi = (end - e > U) ? e + U : end;
            s.last = s.hi == end;
            e = s.hi;
            fresh = s.last;
            if (s.last) ++r;
            break;
        }
        return s;
    };
    auto row_extra = [&](int32_t seg, RowExtra &X) {
        const int64_t v = base + (seg >= 0 ? seg : r_first);
        if constexpr (kScale) X.scale = o.inv_deg[v];
        if constexpr (kExtra == 1) X.raw = *reinterpret_cast<const uint4 *>(o.self + v * o.ld_self + sub * E);
        if constexpr (kExtra == 2) X.raw = *reinterpret_cast<const uint4 *>(o.out + v * o.ld_out + sub * E);
    };
    auto finish = [&](int32_t seg, const float (&acc)[E], const RowExtra &X) {
        const int64_t v = base + seg;
        const int f0 = sub * E;
        float res[E];
#pragma unroll
        for (int i = 0; i < E; ++i) res[i] = (kScale && !o.scale_all) ? acc[i] * X.scale : acc[i];
        if constexpr (kExtra != 0) {
            float x[E];
            Chunk<T>::widen(X.raw, x);
#pragma unroll
            for (int i = 0; i < E; ++i) res[i] += (kEdge && kExtra == 1) ? X.scale * x[i] : x[i];
        }
        if (kScale && o.scale_all) {
#pragma unroll
            for (int i = 0; i < E; ++i) res[i] *= X.scale;
        }
        if (o.bias) {
#pragma unroll
            for (int i = 0; i < E; ++i) res[i] += (f0 + i < o.F) ? o.bias[f0 + i] : 0.0f;
        }
        if (o.relu) {
#pragma unroll
            for (int i = 0; i < E; ++i) res[i] = res[i] > 0.0f ? res[i] : 0.0f;
        }
        Chunk<T>::store(o.out + v * o.ld_out + f0, res);
    };
    // a row that exists in the gathered matrix, for the loads of slots that carry nothing yet
    const int32_t filler_row = int32_t((base + r_first) < o.in_rows ? (base + r_first) : o.in_rows - 1);
    stream_segments<T, kEdge>(in, ld_in, ids, o.edge_scale, last_entry, sub, filler_row, next_row_step, row_extra,
                              finish);
    __syncthreads();

    // ---- deferred rows, kHubsPerPass at a time: group g sums the g-th share of each, then a fixed-order combine
    const int n_hubs = n_deferred;
    const int width = G * E;                         // floats of one partial row
    for (int h0 = 0; h0 < n_hubs; h0 += kHubsPerPass) {
        const int h_end = (h0 + kHubsPerPass) < n_hubs ? (h0 + kHubsPerPass) : n_hubs;
        if (live) {
            int h = h0;
            int32_t pos = 0, stop = 0;
            bool open = false;
            auto next_share_step = [&]() {
                Step s{0, 0, -1, false};
                if (h >= h_end) return s;
                if (!open) {
                    const int row = deferred[h];
                    const int32_t beg = bounds[row], end = bounds[row + 1];
                    const int32_t share = int32_t((int64_t(end - beg) + int64_t(NG) * U - 1) / (int64_t(NG) * U)) * U;
                    const int64_t lo = int64_t(beg) + int64_t(grp) * share;
                    pos = lo < end ? int32_t(lo) : end;
                    stop = (lo + share) < end ? int32_t(lo + share) : end;
                    open = true;
                }
                s.seg = h - h0;
                s.lo = pos;
                s.hi = (stop - pos > U) ? pos + U : stop;
                s.last = s.hi == stop;
                pos = s.hi;
                if (s.last) {
                    ++h;
                    open = false;
                }
                return s;
            };
            auto no_extra = [](int32_t, RowExtra &) {};
            auto to_lds = [&](int32_t seg, const float (&acc)[E], const RowExtra &) {
#pragma unroll
                for (int i = 0; i < E; ++i) partial[(seg * NG + grp) * width + sub * E + i] = acc[i];
            };
            stream_segments<T, kEdge>(in, ld_in, ids, o.edge_scale, last_entry, sub, filler_row, next_share_step,
                                      no_extra, to_lds);
        }
        __syncthreads();
        if (live && grp < h_end - h0) {
            const int64_t v = base + deferred[h0 + grp];
            float acc[E];
#pragma unroll
            for (int i = 0; i < E; ++i) acc[i] = 0.0f;
            for (int g = 0; g < NG; ++g)   // fixed order
#pragma unroll
                for (int i = 0; i < E; ++i) acc[i] += partial[(grp * NG + g) * width + sub * E + i];
            float one[1][E];
#pragma unroll
            for (int i = 0; i < E; ++i) one[0][i] = acc[i];
            finish_row<T, 1, 1>(v, o, sub, G, one);
        }
        __syncthreads();
    }
}

// Rows wider than 64 chunks (1 KB): the whole wavefront owns one row, CPL chunks per lane; rows one after
// the other, rows of more than kHubDegree entries by the whole workgroup.
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
    for (int r = 0; r < R; ++r) {
        const int64_t v = v0 + r;
        if (v >= n) break;
        const int32_t beg = rowptr[v], end = rowptr[v + 1];
        if (end - beg > kHubDegree) {
            if (sub == 0) hub_rows[atomicAdd(&hub_count, 1)] = int32_t(v - base);
            continue;
        }
        float acc[CPL][E];
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int k = 0; k < E; ++k) acc[c][k] = 0.0f;
        gather_sum<T, G, CPL, false>(in, ld_in, colidx, beg, end, G, sub, n_chunks, o.edge_scale, acc);
        finish_row<T, G, CPL>(v, o, sub, n_chunks, acc);
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
        if (beg + grp * G < end) gather_sum<T, G, CPL, true>(in, ld_in, colidx, beg + grp * G, end, NG * G, sub, n_chunks, o.edge_scale, acc);
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
            const int32_t u = colidx[e];
            const T *row = in + int64_t(u) * ld_in;
            const float w = o.edge_scale ? o.edge_scale[u] : 1.0f;
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int f = f0 + k * kWave + lane;
                if (f < F) acc[k] += w * load_elem(row + f);
            }
        }
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int f = f0 + k * kWave + lane;
            if (f < F) {
                T *dst = o.out + v * o.ld_out + f;
                float r = o.scale_all ? acc[k] : acc[k] * scale;
                if (o.accumulate) r += load_elem(dst);
                if (o.self) r += (o.edge_scale ? o.edge_scale[v] : 1.0f) * load_elem(o.self + v * o.ld_self + f);
                if (o.scale_all) r *= scale;
                if (o.bias && f < o.F) r += o.bias[f];
                if (o.relu) r = r > 0.0f ? r : 0.0f;
                store_elem(dst, r);
            }
        }
    }
}

template <typename T, int G, int CPL>
static void launch_wide_rows(int64_t n, const int32_t *rowptr, const int32_t *colidx, const T *in, int64_t ld_in,
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

template <typename T, int kExtra, bool kScale, bool kEdge = false>
static void launch_stream(int64_t n, const int32_t *rowptr, const int32_t *colidx, const T *in, int64_t ld_in,
                          const SpmmOut<T> &o, int G, hipStream_t s)
{
    // rows per group: long enough a stream for the pipeline to pay, short enough to leave the chip
    // several workgroups per compute unit
    const int NG = (kSpmmThreads / kWave) * (kWave / G);
    // Rows per lane group: enough blocks to fill the chip six times over, 4 to 8 rows each; a group's pipeline
    // costs two extra steps to fill and drain, so on very long row ranges (millions of rows: every block runs many
    // rounds anyway) 16 rows per group amortise it better (12.5 M rows: -7 %), while on a dense cache-resident
    // graph (mean degree 44, 144 k rows) longer groups only lengthen the tail (+15 %).
    int64_t rpg = ceil_div(n, int64_t(NG) * 256 * 6);
    const int64_t rpg_max = n >= (int64_t(1) << 22) ? 16 : 8;
    rpg = rpg < 4 ? 4 : (rpg > rpg_max ? rpg_max : rpg);
    if (rpg * NG > kMaxRowsPerBlock) rpg = kMaxRowsPerBlock / NG;
    char name[48];
    snprintf(name, sizeof(name), "%s_%s_g%dx1",
             kEdge ? "spmm_weighted" : (kExtra == 1 ? "spmm_combine" : (kScale ? "spmm_mean" : "spmm_sum")),
             sizeof(T) == 4 ? "f32" : "bf16", G);
    TMA_TIMED(name, s);
    hipLaunchKernelGGL((spmm_stream_kernel<T, kExtra, kScale, kEdge>),
                       dim3(unsigned(round_up(size_t(ceil_div(n, rpg * NG)), kDies))), dim3(kSpmmThreads), 0, s, n, rowptr,
                       colidx, in, ld_in, o, G, int(rpg), kMinDefer);
}

template <typename T>
static int launch_typed(int64_t n, const int32_t *rowptr, const int32_t *colidx, const T *in, int64_t ld_in, int32_t F,
                        const SpmmOut<T> &o, hipStream_t s)
{
    // A row is walked in whole 16-byte pieces.  A width that is no multiple of 16 bytes (100 bf16 elements) still
    // takes this path when every pitch leaves room for the last piece: the piece's tail then reads and writes
    // padding elements inside the rows (never memory outside them).
    const size_t row_bytes = round_up(size_t(F) * sizeof(T), 16);
    const bool vec_ok = (size_t(ld_in) * sizeof(T)) % 16 == 0 && size_t(ld_in) * sizeof(T) >= row_bytes &&
                        (size_t(o.ld_out) * sizeof(T)) % 16 == 0 && size_t(o.ld_out) * sizeof(T) >= row_bytes &&
                        aligned(in, 16) && aligned(o.out, 16) &&
                        (!o.self || ((size_t(o.ld_self) * sizeof(T)) % 16 == 0 && aligned(o.self, 16) &&
                                     size_t(o.ld_self) * sizeof(T) >= row_bytes)) &&
                        row_bytes / 16 <= 256 && !(o.self && o.accumulate);
    // the streaming kernel's weighted form takes the self weight from the row scale it already holds
    const bool edge_stream = o.edge_scale && o.self && o.inv_deg == o.edge_scale;
    if (!vec_ok || (o.edge_scale && !edge_stream && row_bytes / 16 <= 64)) {
        TMA_TIMED(o.self ? "spmm_combine_generic" : (o.inv_deg ? "spmm_mean_generic" : "spmm_sum_generic"), s);
        hipLaunchKernelGGL((spmm_rows_generic_kernel<T>), dim3(unsigned(ceil_div(n, kSpmmThreads / kWave))),
                           dim3(kSpmmThreads), 0, s, n, rowptr, colidx, in, ld_in, o, F);
        return check_launch("spmm (generic)");
    }
    const int nc = int(row_bytes / 16);
    if (nc <= 64) {
        const int extra = o.self ? 1 : (o.accumulate ? 2 : 0);
#define TMA_SPMM_STREAM(X, S) launch_stream<T, X, S>(n, rowptr, colidx, in, ld_in, o, nc, s)
        if (o.edge_scale) {
            launch_stream<T, 1, true, true>(n, rowptr, colidx, in, ld_in, o, nc, s);
        } else if (o.inv_deg) {
            if (extra == 0) TMA_SPMM_STREAM(0, true);
            else if (extra == 1) TMA_SPMM_STREAM(1, true);
            else TMA_SPMM_STREAM(2, true);
        } else {
            if (extra == 0) TMA_SPMM_STREAM(0, false);
            else if (extra == 1) TMA_SPMM_STREAM(1, false);
            else TMA_SPMM_STREAM(2, false);
        }
#undef TMA_SPMM_STREAM
    } else if (nc <= 128) {
        launch_wide_rows<T, 64, 2>(n, rowptr, colidx, in, ld_in, o, nc, s);
    } else {
        launch_wide_rows<T, 64, 4>(n, rowptr, colidx, in, ld_in, o, nc, s);
    }
    return check_launch("spmm");
}

template <typename T>
static int spmm_any(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                    int64_t ld_in, int32_t F, void *out, int64_t ld_out, bool accumulate, const void *self,
                    int64_t ld_self, const float *bias, int32_t F_valid, bool relu, bool scale_all,
                    const float *edge_scale, int64_t in_rows, hipStream_t stream)
{
    SpmmOut<T> o{static_cast<T *>(out), ld_out, inv_deg, accumulate ? 1 : 0, static_cast<const T *>(self), ld_self,
                 bias, F_valid, relu ? 1 : 0, (scale_all && inv_deg) ? 1 : 0, edge_scale, in_rows > 0 ? in_rows : n};
    return launch_typed<T>(n, rowptr, colidx, static_cast<const T *>(in), ld_in, F, o, stream);
}

int launch_spmm(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                int64_t ld_in, int32_t F, int32_t dtype, void *out, int64_t ld_out, bool accumulate,
                hipStream_t stream, int64_t in_rows)
{
    return launch_spmm_combine(n, rowptr, colidx, inv_deg, in, ld_in, F, dtype, out, ld_out, accumulate, nullptr, 0,
                               nullptr, F, false, false, nullptr, stream, in_rows);
}

int launch_spmm_combine(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *inv_deg, const void *in,
                        int64_t ld_in, int32_t F, int32_t dtype, void *out, int64_t ld_out, bool accumulate,
                        const void *self, int64_t ld_self, const float *bias, int32_t F_valid, bool relu,
                        bool scale_all, const float *edge_scale, hipStream_t stream, int64_t in_rows)
{
    if (n == 0 || F == 0) return TMA_OK;
    if (dtype == TMA_F32)
        return spmm_any<float>(n, rowptr, colidx, inv_deg, in, ld_in, F, out, ld_out, accumulate, self, ld_self, bias,
                               F_valid, relu, scale_all, edge_scale, in_rows, stream);
    if (dtype == TMA_BF16)
        return spmm_any<uint16_t>(n, rowptr, colidx, inv_deg, in, ld_in, F, out, ld_out, accumulate, self, ld_self,
                                  bias, F_valid, relu, scale_all, edge_scale, in_rows, stream);
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
