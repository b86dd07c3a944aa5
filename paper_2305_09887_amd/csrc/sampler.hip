// Sampled message-flow graphs (paper Sec. 4.1, paragraph on mini-batch and
// negative sampling: a GraphSAGE-style sampler caps the neighbours a node
// aggregates, so a step touches the sampled neighbourhood of its batch only):
//   * fan-out neighbour sampling on the local CSR (a uniform subset per row, by key ranking);
//   * the node list of a block (dst nodes first, the new ones in ascending id) and the
//     relabelling of its columns, with the scan of the subgraph extraction;
//   * the mean-aggregation GraphSAGE layer on such a bipartite block, forward and backward;
//     the backward gathers over the block's transpose, which is built here with integer
//     counting, a scan, a fill and a sort of every list (no floating-point atomics).
// Integer / latency bound work around the layer kernels.
#include "kernels.hpp"

namespace tma {

constexpr int kThreadCopy = 32;     // rows kept whole and no longer than this are copied by their thread
constexpr int kKeyLds = 512;        // keys a wavefront keeps in its LDS segment (4 KB: 2048 measured 15 % slower, fewer wavefronts fit)
constexpr int kLongRowBlocks = 1024;   // workgroups (of four wavefronts) that share the queue of long rows (256: 20 % slower; 4096: no faster)

__device__ __forceinline__ int32_t item_count(const int32_t *d_items, int64_t max_items)
{
    if (!d_items) return int32_t(max_items);
    const int32_t c = *d_items;
    return c < max_items ? c : int32_t(max_items);
}

// ---- neighbour sampling -----------------------------------------------------------------------
// d_n_dst (may be NULL): the number of dst rows when it is only known on the device; n_dst is then the capacity the
// launch is sized for, and the rows from the count up to the capacity are given no entries.
// (also clears the counter of the queue that the fill kernels build)
__global__ __launch_bounds__(256) void sample_count_kernel(int64_t n_dst, const int32_t *__restrict__ d_n_dst,
                                                           const int32_t *__restrict__ dst,
                                                           const int32_t *__restrict__ rowptr, int32_t fanout,
                                                           int32_t *__restrict__ deg, int32_t *__restrict__ n_queued)
{
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i == 0) *n_queued = 0;
    if (i >= n_dst) return;
    if (i >= item_count(d_n_dst, n_dst)) {
        deg[i] = 0;
        return;
    }
    const int32_t w = dst[i];
    const int32_t d = rowptr[w + 1] - rowptr[w];
    deg[i] = d < fanout ? d : fanout;
}

// Rows that are kept whole and short are copied by their thread; the others are queued for a wavefront each
// (one queue reservation per wavefront).
__global__ __launch_bounds__(256) void sample_fill_short_kernel(int64_t n_dst, const int32_t *__restrict__ d_n_dst,
                                                                const int32_t *__restrict__ dst,
                                                                const int32_t *__restrict__ rowptr,
                                                                const int32_t *__restrict__ colidx, int32_t fanout,
                                                                const int32_t *__restrict__ blk_rowptr,
                                                                int32_t *__restrict__ blk_col, int32_t *__restrict__ blk_row,
                                                                int64_t cap, int32_t *__restrict__ queue,
                                                                int32_t *__restrict__ n_queued)
{
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int lane = threadIdx.x % kWave;
    int32_t beg = 0, d = 0;
    if (i < item_count(d_n_dst, n_dst)) {
        const int32_t w = dst[i];
        beg = rowptr[w];
        d = rowptr[w + 1] - beg;
    }
    const bool whole = d <= fanout;
    const bool queued = d > 0 && !(whole && d <= kThreadCopy);
    const uint64_t mask = __ballot(queued);
    if (mask != 0) {
        const int leader = __ffsll(static_cast<long long>(mask)) - 1;
        int32_t first = 0;
        if (lane == leader) first = atomicAdd(n_queued, int32_t(__popcll(mask)));
        first = __shfl(first, leader, kWave);
        if (queued) queue[first + __popcll(mask & ((uint64_t(1) << lane) - 1))] = int32_t(i);
    }
    if (d > 0 && !queued) {
        const int32_t out = blk_rowptr[i];
        for (int32_t k = 0; k < d && out + k < cap; ++k) {   // (cap is only reached with repeated dst nodes)
            blk_col[out + k] = colidx[beg + k];
            blk_row[out + k] = int32_t(i);
        }
    }
}

// The fanout-th smallest of `count` keys (key_at(j), j < count) that fit NC registers per lane (chunk c: key
// c * 64 + lane), found bit by bit from the top: per bit one count over the keys (ballots), no sorting.  On return
// T is that key and `remaining` says how many of the keys equal to T are still needed after all keys below T.
// Lanes past the end hold the all-ones key, which never counts as having a zero bit.
template <int NC, class KeyAt>
__device__ __forceinline__ void threshold_in_registers(int32_t count, int lane, int32_t fanout, KeyAt key_at, uint64_t &T,
                                                       int32_t &remaining)
{
    uint64_t kreg[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) kreg[c] = (c * kWave + lane < count) ? key_at(c * kWave + lane) : ~uint64_t(0);
    T = 0;
    remaining = fanout;
    for (int bit = 63; bit >= 0; --bit) {
        const uint64_t above = bit == 63 ? uint64_t(0) : (~uint64_t(0) << (bit + 1));
        int32_t zeros = 0;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const bool hit = ((kreg[c] ^ T) & above) == 0 && ((kreg[c] >> bit) & 1) == 0;
            zeros += int32_t(__popcll(__ballot(hit)));
        }
        if (zeros < remaining) {   // the threshold has a 1 here; the keys with a 0 are all below it
            remaining -= zeros;
            T |= uint64_t(1) << bit;
        }
    }
}

// The same for any count: up to 16 registers per lane hold the keys, beyond that key_at is asked again for every bit.
template <class KeyAt>
__device__ __forceinline__ void threshold_of(int32_t count, int lane, int32_t fanout, KeyAt key_at, uint64_t &T,
                                             int32_t &remaining)
{
    if (count <= kWave) return threshold_in_registers<1>(count, lane, fanout, key_at, T, remaining);
    if (count <= 2 * kWave) return threshold_in_registers<2>(count, lane, fanout, key_at, T, remaining);
    if (count <= 4 * kWave) return threshold_in_registers<4>(count, lane, fanout, key_at, T, remaining);
    if (count <= 8 * kWave) return threshold_in_registers<8>(count, lane, fanout, key_at, T, remaining);
    if (count <= 16 * kWave) return threshold_in_registers<16>(count, lane, fanout, key_at, T, remaining);
    T = 0;                 // bits of the threshold decided so far (the undecided low bits are 0)
    remaining = fanout;    // the threshold is the remaining-th smallest of the keys that match T's decided bits
    for (int bit = 63; bit >= 0; --bit) {
        const uint64_t above = bit == 63 ? uint64_t(0) : (~uint64_t(0) << (bit + 1));
        int32_t zeros = 0;         // matching keys whose bit `bit` is 0
        for (int32_t base = 0; base < count; base += kWave) {
            const int32_t k = base + lane;
            bool hit = false;
            if (k < count) {
                const uint64_t key = key_at(k);
                hit = ((key ^ T) & above) == 0 && ((key >> bit) & 1) == 0;
            }
            zeros += int32_t(__popcll(__ballot(hit)));
        }
        if (zeros < remaining) {
            remaining -= zeros;
            T |= uint64_t(1) << bit;
        }
    }
}

// A wavefront per queued row.  A row longer than the fan-out keeps the `fanout` entries with the smallest
// (key, entry index), key(e) = SplitMix64(seed, e), in row order: kept are the keys below the fanout-th smallest
// key T and, of the keys equal to T, the first ones in row order that are still needed.
//
// T of a long row is looked for among few keys: the keys are uniform on the 64-bit range, so the fanout-th
// smallest of d lies near fanout / d of the range, and one pass over the row first collects the keys below a
// bound U = (2 fanout + 32) / d of the range (about 2 fanout + 32 of them, in the wavefront's LDS segment).  If at
// least `fanout` and no more than the segment holds were collected, every key up to T is among them and the T and
// `remaining` of the collected keys are those of the row; otherwise (a chance far below one in a million for
// fan-outs up to about 150, and always when the fan-out is a large share of the row) all keys of the row are
// ranked as for a short row, recomputed for every bit once they no longer fit the registers.  Either way the
// result is exact.
__global__ __launch_bounds__(256) void sample_fill_long_kernel(const int32_t *__restrict__ dst,
                                                               const int32_t *__restrict__ rowptr,
                                                               const int32_t *__restrict__ colidx, int32_t fanout,
                                                               uint64_t seed, const int32_t *__restrict__ blk_rowptr,
                                                               int32_t *__restrict__ blk_col, int32_t *__restrict__ blk_row,
                                                               int64_t cap, const int32_t *__restrict__ queue,
                                                               const int32_t *__restrict__ n_queued)
{
    __shared__ uint64_t keys[256 / kWave][kKeyLds];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const uint64_t lower_lanes = (uint64_t(1) << lane) - 1;
    const int count = *n_queued;
    const int waves = gridDim.x * (256 / kWave);
    for (int q = blockIdx.x * (256 / kWave) + wave; q < count; q += waves) {
        const int32_t i = queue[q];
        const int32_t w = dst[i];
        const int32_t beg = rowptr[w], d = rowptr[w + 1] - beg;
        const int32_t out = blk_rowptr[i];
        if (d <= fanout) {
            for (int32_t k = lane; k < d && out + k < cap; k += kWave) {
                blk_col[out + k] = colidx[beg + k];
                blk_row[out + k] = i;
            }
            continue;
        }
        auto fresh_key = [&](int32_t k) { return splitmix64_at(seed, uint64_t(beg + k)); };
        auto held_key = [&](int32_t k) { return keys[wave][k]; };
        // a wavefront's LDS accesses complete in program order: its own writes are visible to its later reads; the
        // wave barriers only keep the compiler from moving the accesses across them

        uint64_t T = 0;
        int32_t remaining = fanout;
        bool found = false;
        const int64_t want = 2 * int64_t(fanout) + 32;
        if (d > 2 * kWave && want < d) {
            const uint64_t U = (~uint64_t(0) / uint64_t(d)) * uint64_t(want);
            int32_t held = 0;
            for (int32_t base = 0; base < d; base += kWave) {
                const int32_t k = base + lane;
                uint64_t key = 0;
                bool low = false;
                if (k < d) {
                    key = fresh_key(k);
                    low = key < U;
                }
                const uint64_t lows = __ballot(low);
                if (low) {
                    const int32_t p = held + int32_t(__popcll(lows & lower_lanes));
                    if (p < kKeyLds) keys[wave][p] = key;
                }
                held += int32_t(__popcll(lows));
            }
            __builtin_amdgcn_wave_barrier();
            if (held >= fanout && held <= kKeyLds) {
                threshold_of(held, lane, fanout, held_key, T, remaining);
                found = true;
            }
            __builtin_amdgcn_wave_barrier();   // before the segment is written again
        }
        if (!found) threshold_of(d, lane, fanout, fresh_key, T, remaining);
        // keys below T: fanout - remaining of them; of the keys equal to T the first `remaining` in row order
        int32_t kept_before = 0, equal_before = 0;
        for (int32_t base = 0; base < d; base += kWave) {
            const int32_t k = base + lane;
            bool below = false, equal = false;
            if (k < d) {
                const uint64_t key = fresh_key(k);
                below = key < T;
                equal = key == T;
            }
            const uint64_t equals = __ballot(equal);
            const bool keep = below || (equal && equal_before + int32_t(__popcll(equals & lower_lanes)) < remaining);
            const uint64_t kept = __ballot(keep);
            if (keep) {
                const int32_t p = out + kept_before + int32_t(__popcll(kept & lower_lanes));
                if (p < cap) {
                    blk_col[p] = colidx[beg + k];
                    blk_row[p] = i;
                }
            }
            kept_before += int32_t(__popcll(kept));
            equal_before += int32_t(__popcll(equals));
        }
        __builtin_amdgcn_wave_barrier();   // before the segment is overwritten by the next row
    }
}

// ---- node list of a block and relabelling -------------------------------------------------------
__global__ __launch_bounds__(256) void fill_i32_kernel(int64_t count, int32_t *__restrict__ p, int32_t value)
{
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < count; i += stride) p[i] = value;
}

__global__ __launch_bounds__(256) void fill2_i32_kernel(int64_t count, int32_t *__restrict__ p, int32_t value,
                                                        int32_t *__restrict__ q, int32_t q_value)
{
    const int64_t stride = int64_t(gridDim.x) * 256;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < count; i += stride) {
        p[i] = value;
        q[i] = q_value;
    }
}

__global__ __launch_bounds__(256) void mark_dst_kernel(int64_t n_dst, const int32_t *__restrict__ d_n_dst,
                                                       const int32_t *__restrict__ dst, int32_t *__restrict__ pos,
                                                       int32_t *__restrict__ src)
{
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= item_count(d_n_dst, n_dst)) return;
    pos[dst[i]] = int32_t(i);
    src[i] = dst[i];
}

__global__ __launch_bounds__(256) void flag_new_kernel(int64_t max_items, const int32_t *__restrict__ d_items,
                                                       const int32_t *__restrict__ cols, const int32_t *__restrict__ pos,
                                                       int32_t *__restrict__ isnew)
{
    const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (e >= item_count(d_items, max_items)) return;
    const int32_t c = cols[e];
    if (pos[c] < 0) isnew[c] = 1;     // several writers, one value
}

// (rank[n] is the number of new nodes; n_src_out, if given, receives the length of the node list)
__global__ __launch_bounds__(256) void assign_new_kernel(int64_t n, int64_t n_dst_cap, const int32_t *__restrict__ d_n_dst,
                                                         const int32_t *__restrict__ isnew,
                                                         const int32_t *__restrict__ rank, int32_t *__restrict__ pos,
                                                         int32_t *__restrict__ src, int32_t *__restrict__ n_src_out)
{
    const int64_t c = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int32_t n_dst = item_count(d_n_dst, n_dst_cap);
    if (c == 0 && n_src_out) *n_src_out = n_dst + rank[n];
    if (c >= n || !isnew[c]) return;
    const int32_t p = n_dst + rank[c];
    pos[c] = p;
    src[p] = int32_t(c);
}

__global__ __launch_bounds__(256) void relabel_kernel(int64_t max_items, const int32_t *__restrict__ d_items,
                                                      int32_t *__restrict__ cols, const int32_t *__restrict__ pos)
{
    const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (e >= item_count(d_items, max_items)) return;
    cols[e] = pos[cols[e]];
}

__global__ __launch_bounds__(256) void block_inv_deg_kernel(int64_t n_dst, const int32_t *__restrict__ blk_rowptr,
                                                            float *__restrict__ inv_deg)
{
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n_dst) return;
    const int32_t d = blk_rowptr[i + 1] - blk_rowptr[i];
    inv_deg[i] = d > 0 ? 1.0f / float(d) : 0.0f;
}

// ---- transpose of a block -----------------------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_count_kernel(int64_t max_items, const int32_t *__restrict__ d_items,
                                                              const int32_t *__restrict__ cols, int32_t *__restrict__ deg)
{
    const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (e >= item_count(d_items, max_items)) return;
    atomicAdd(&deg[cols[e]], 1);
}

__global__ __launch_bounds__(256) void transpose_fill_kernel(int64_t max_items, const int32_t *__restrict__ d_items,
                                                             const int32_t *__restrict__ cols,
                                                             const int32_t *__restrict__ rowptr_T,
                                                             int32_t *__restrict__ cursor, int32_t *__restrict__ unsorted)
{
    const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (e >= item_count(d_items, max_items)) return;
    const int32_t c = cols[e];
    unsorted[rowptr_T[c] + atomicAdd(&cursor[c], 1)] = int32_t(e);
}

// entry numbers -> the dst rows they belong to (ascending entry numbers are ascending rows)
__global__ __launch_bounds__(256) void entries_to_rows_kernel(int64_t max_items, const int32_t *__restrict__ d_items,
                                                              int32_t *__restrict__ list, const int32_t *__restrict__ blk_row)
{
    const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (e >= item_count(d_items, max_items)) return;
    list[e] = blk_row[list[e]];
}

static size_t elem_size(int32_t dtype) { return dtype == TMA_BF16 ? 2 : 4; }
static unsigned blocks_for(int64_t work) { return unsigned(ceil_div(work > 0 ? work : 1, 256)); }
static unsigned capped_blocks(int64_t work)
{
    const int64_t b = ceil_div(work > 0 ? work : 1, 256);
    return unsigned(b > 256 * 64 ? 256 * 64 : b);
}

struct BlockBwdWorkspace {
    size_t dm_bytes;       // inv_deg-scaled dM, [n_dst, F_in]
    size_t deg_bytes;      // per-source counts (then the sort's queue), fill cursors, queue length
    size_t rowptr_bytes;   // transposed rowptr
    size_t list_bytes;     // unsorted and sorted lists, one of each
    size_t scan_bytes;
    size_t weight_bytes;
    size_t total() const { return dm_bytes + deg_bytes + rowptr_bytes + 2 * list_bytes + scan_bytes + weight_bytes; }
};

static BlockBwdWorkspace plan_block_bwd(int64_t n_dst, int64_t n_src, int64_t max_entries, int32_t F_in, int32_t F_out,
                                        int32_t dtype, bool need_dH)
{
    BlockBwdWorkspace w{};
    const size_t rows = size_t(n_dst > 0 ? n_dst : 1), srcs = size_t(n_src > 0 ? n_src : 1);
    const size_t items = size_t(max_entries > 0 ? max_entries : 1);
    if (need_dH) {
        w.dm_bytes = round_up(rows * size_t(F_in) * elem_size(dtype), 256);
        w.deg_bytes = round_up((2 * srcs + 1) * 4, 256);
        w.rowptr_bytes = round_up((srcs + 1) * 4, 256);
        w.list_bytes = round_up(items * 4, 256);
        w.scan_bytes = exclusive_scan_i32_workspace_bytes(n_src);
    }
    w.weight_bytes = sage_gemm_bwd_weight_workspace_bytes(n_dst, F_in, F_out);
    return w;
}

// Transpose of a block: for every source node the dst rows that sampled it, in ascending order (rowptr_T [n_src + 1],
// sorted [entries]); blk_row = the dst row of every entry of the block.  deg: 2 * n_src + 1 int32 of
// scratch, unsorted: max_entries int32 of scratch.
static int transpose_block(const char *fn, int64_t n_dst, int64_t n_src, int64_t max_entries, const int32_t *blk_rowptr,
                           const int32_t *blk_col, const int32_t *blk_row, int32_t *deg, int32_t *rowptr_T, int32_t *unsorted,
                           int32_t *sorted, void *scan_ws, hipStream_t s)
{
    const int32_t *d_items = blk_rowptr ? blk_rowptr + n_dst : nullptr;
    int32_t *cursor = deg + n_src;
    {
        TMA_TIMED("transpose_count", s);
        hipLaunchKernelGGL(fill_i32_kernel, dim3(capped_blocks(2 * n_src + 1)), dim3(256), 0, s, 2 * n_src + 1, deg, 0);
        if (max_entries > 0 && n_dst > 0)
            hipLaunchKernelGGL(transpose_count_kernel, dim3(blocks_for(max_entries)), dim3(256), 0, s, max_entries, d_items,
                               blk_col, deg);
    }
    if (int rc = check_launch(fn)) return rc;
    if (int rc = launch_exclusive_scan_i32(n_src, deg, rowptr_T, scan_ws, s)) return rc;
    if (max_entries > 0 && n_dst > 0) {
        {
            TMA_TIMED("transpose_fill", s);
            hipLaunchKernelGGL(transpose_fill_kernel, dim3(blocks_for(max_entries)), dim3(256), 0, s, max_entries, d_items,
                               blk_col, rowptr_T, cursor, unsorted);
        }
        if (int rc = launch_sort_lists(n_src, rowptr_T, unsorted, sorted, deg, deg + 2 * n_src, s)) return rc;
        TMA_TIMED("transpose_rows", s);
        hipLaunchKernelGGL(entries_to_rows_kernel, dim3(blocks_for(max_entries)), dim3(256), 0, s, max_entries, d_items,
                           sorted, blk_row);
        if (int rc = check_launch(fn)) return rc;
    }
    return TMA_OK;
}

// The same workspace layout with the weight-gradient scratch of the one-matrix (GCN) layer.
static BlockBwdWorkspace plan_gcn_block_bwd(int64_t n_dst, int64_t n_src, int64_t max_entries, int32_t F_in, int32_t F_out,
                                            int32_t dtype, bool need_dH)
{
    BlockBwdWorkspace w = plan_block_bwd(n_dst, n_src, max_entries, F_in, F_out, dtype, need_dH);
    w.weight_bytes = dense_gemm_bwd_weight_workspace_bytes(n_dst, F_in, F_out);
    return w;
}

}  // namespace tma

extern "C" size_t tma_neighbor_sample_workspace_bytes(int64_t n_dst)
{
    if (n_dst < 0) return 0;
    const size_t rows = size_t(n_dst > 0 ? n_dst : 1);
    return tma::round_up((2 * rows + 1) * 4, 256) + tma::exclusive_scan_i32_workspace_bytes(n_dst);
}

namespace tma {

// d_n_dst == NULL: n_dst rows.  Otherwise n_dst is a capacity and the row count is read on the device.
static int neighbor_sample(const char *fn, int64_t n_dst, const int32_t *d_n_dst, const int32_t *dst, int64_t nnz,
                           const int32_t *rowptr, const int32_t *colidx, int32_t fanout, uint64_t seed,
                           int32_t *blk_rowptr_out, int32_t *blk_col_out, int32_t *blk_row_out, int64_t cap_entries,
                           void *ws, size_t ws_bytes, tma_stream_t stream)
{
    TMA_REQUIRE(n_dst >= 0 && n_dst <= INT32_MAX && nnz >= 0 && nnz <= INT32_MAX && fanout >= 1, TMA_ERR_INVALID_ARG,
                "%s: n_dst, nnz or fanout", fn);
    TMA_REQUIRE(blk_rowptr_out && ws && aligned(ws, 256) && ws_bytes >= tma_neighbor_sample_workspace_bytes(n_dst),
                TMA_ERR_INVALID_ARG, "%s: blk_rowptr_out / workspace", fn);
    const int64_t bound = n_dst * int64_t(fanout) < nnz ? n_dst * int64_t(fanout) : nnz;
    TMA_REQUIRE(cap_entries >= bound && cap_entries <= INT32_MAX, TMA_ERR_WORKSPACE_TOO_SMALL,
                "%s: room for %lld entries, up to %lld may be kept", fn, (long long)cap_entries, (long long)bound);
    hipStream_t s = as_stream(stream);
    int32_t *deg = static_cast<int32_t *>(ws);                 // per-row counts, then the queue of rows for a wavefront
    const size_t rows = size_t(n_dst > 0 ? n_dst : 1);
    int32_t *n_queued = deg + 2 * rows;
    void *scan_ws = static_cast<char *>(ws) + round_up((2 * rows + 1) * 4, 256);
    if (n_dst > 0) {
        TMA_REQUIRE(dst && rowptr && (nnz == 0 || (colidx && blk_col_out && blk_row_out)), TMA_ERR_INVALID_ARG,
                    "%s: NULL argument", fn);
        TMA_TIMED("sample_count", s);
        hipLaunchKernelGGL(sample_count_kernel, dim3(blocks_for(n_dst)), dim3(256), 0, s, n_dst, d_n_dst, dst, rowptr, fanout,
                           deg, n_queued);
    }
    if (int rc = check_launch(fn)) return rc;
    if (int rc = launch_exclusive_scan_i32(n_dst, deg, blk_rowptr_out, scan_ws, s)) return rc;
    if (n_dst == 0 || nnz == 0) return TMA_OK;
    int32_t *queue = deg + rows;
    {
        TMA_TIMED("sample_fill_short", s);
        hipLaunchKernelGGL(sample_fill_short_kernel, dim3(blocks_for(n_dst)), dim3(256), 0, s, n_dst, d_n_dst, dst, rowptr,
                           colidx, fanout, blk_rowptr_out, blk_col_out, blk_row_out, cap_entries, queue, n_queued);
    }
    TMA_TIMED("sample_fill_long", s);
    hipLaunchKernelGGL(sample_fill_long_kernel, dim3(kLongRowBlocks), dim3(256), 0, s, dst, rowptr, colidx, fanout, seed,
                       blk_rowptr_out, blk_col_out, blk_row_out, cap_entries, queue, n_queued);
    return check_launch(fn);
}

}  // namespace tma

extern "C" int tma_neighbor_sample(int64_t n_dst, const int32_t *dst, int64_t nnz, const int32_t *rowptr,
                                   const int32_t *colidx, int32_t fanout, uint64_t seed, int32_t *blk_rowptr_out,
                                   int32_t *blk_col_out, int32_t *blk_row_out, int64_t cap_entries, void *ws,
                                   size_t ws_bytes, tma_stream_t stream)
{
    return tma::neighbor_sample("tma_neighbor_sample", n_dst, nullptr, dst, nnz, rowptr, colidx, fanout, seed,
                                blk_rowptr_out, blk_col_out, blk_row_out, cap_entries, ws, ws_bytes, stream);
}

extern "C" int tma_neighbor_sample_dev(int64_t cap_dst, const int32_t *d_n_dst, const int32_t *dst, int64_t nnz,
                                       const int32_t *rowptr, const int32_t *colidx, int32_t fanout, uint64_t seed,
                                       int32_t *blk_rowptr_out, int32_t *blk_col_out, int32_t *blk_row_out,
                                       int64_t cap_entries, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    const char *fn = "tma_neighbor_sample_dev";
    TMA_REQUIRE(d_n_dst, TMA_ERR_INVALID_ARG, "%s: d_n_dst is NULL", fn);
    return tma::neighbor_sample(fn, cap_dst, d_n_dst, dst, nnz, rowptr, colidx, fanout, seed, blk_rowptr_out,
                                blk_col_out, blk_row_out, cap_entries, ws, ws_bytes, stream);
}

extern "C" size_t tma_mfg_relabel_workspace_bytes(int64_t n)
{
    if (n < 0) return 0;
    const size_t rows = size_t(n > 0 ? n : 1);
    return 2 * tma::round_up(rows * 4, 256) + tma::round_up((rows + 1) * 4, 256) + tma::exclusive_scan_i32_workspace_bytes(n);
}

namespace tma {

// d_n_dst == NULL: n_dst dst nodes.  Otherwise n_dst is a capacity and the count is read on the device.
// h_n_src != NULL: the length of the node list is copied to the host (one wait); d_n_src_out != NULL: it is left
// on the device.
static int mfg_relabel(const char *fn, int64_t n, int64_t n_dst, const int32_t *d_n_dst, const int32_t *dst,
                       int64_t max_items, const int32_t *d_items, int32_t *cols_inout, int32_t *src_out, int64_t cap_src,
                       int64_t *h_n_src, int32_t *d_n_src_out, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    TMA_REQUIRE(n >= 0 && n <= INT32_MAX && n_dst >= 0 && n_dst <= n && max_items >= 0 && max_items <= INT32_MAX,
                TMA_ERR_INVALID_ARG, "%s: n, n_dst or max_items", fn);
    TMA_REQUIRE((h_n_src || d_n_src_out) && ws && aligned(ws, 256) && ws_bytes >= tma_mfg_relabel_workspace_bytes(n),
                TMA_ERR_INVALID_ARG, "%s: no place for the node count / workspace", fn);
    const int64_t bound = n_dst + max_items < n ? n_dst + max_items : n;
    TMA_REQUIRE(cap_src >= bound, TMA_ERR_WORKSPACE_TOO_SMALL, "%s: room for %lld source nodes, up to %lld possible", fn,
                (long long)cap_src, (long long)bound);
    if (h_n_src) *h_n_src = n_dst;
    hipStream_t s = as_stream(stream);
    if (n == 0) {
        if (d_n_src_out) {   // (a fill kernel, not a memset: callers may capture this into a graph)
            hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(256), 0, s, int64_t(1), d_n_src_out, 0);
            return check_launch(fn);
        }
        return TMA_OK;
    }
    TMA_REQUIRE((n_dst == 0 || dst) && (max_items == 0 || cols_inout) && (bound == 0 || src_out), TMA_ERR_INVALID_ARG,
                "%s: NULL argument", fn);
    const size_t rows = size_t(n);
    char *base = static_cast<char *>(ws);
    int32_t *pos = reinterpret_cast<int32_t *>(base);
    int32_t *isnew = reinterpret_cast<int32_t *>(base + round_up(rows * 4, 256));
    int32_t *rank = reinterpret_cast<int32_t *>(base + 2 * round_up(rows * 4, 256));
    void *scan_ws = base + 2 * round_up(rows * 4, 256) + round_up((rows + 1) * 4, 256);
    {
        TMA_TIMED("mfg_mark", s);
        hipLaunchKernelGGL(fill2_i32_kernel, dim3(capped_blocks(n)), dim3(256), 0, s, n, pos, -1, isnew, 0);
        if (n_dst > 0)
            hipLaunchKernelGGL(mark_dst_kernel, dim3(blocks_for(n_dst)), dim3(256), 0, s, n_dst, d_n_dst, dst, pos, src_out);
        if (max_items > 0)
            hipLaunchKernelGGL(flag_new_kernel, dim3(blocks_for(max_items)), dim3(256), 0, s, max_items, d_items,
                               cols_inout, pos, isnew);
    }
    if (int rc = check_launch(fn)) return rc;
    if (int rc = launch_exclusive_scan_i32(n, isnew, rank, scan_ws, s)) return rc;
    {
        TMA_TIMED("mfg_relabel", s);
        hipLaunchKernelGGL(assign_new_kernel, dim3(blocks_for(n)), dim3(256), 0, s, n, n_dst, d_n_dst, isnew, rank, pos,
                           src_out, d_n_src_out);
        if (max_items > 0)
            hipLaunchKernelGGL(relabel_kernel, dim3(blocks_for(max_items)), dim3(256), 0, s, max_items, d_items, cols_inout,
                               pos);
    }
    if (int rc = check_launch(fn)) return rc;
    if (h_n_src) {
        int32_t n_new = 0;
        // copy in stream order and wait for it: the caller sizes the next launches with the count
        TMA_HIP_TRY(hipMemcpyWithStream(&n_new, rank + n, sizeof(n_new), hipMemcpyDeviceToHost, s), fn);
        *h_n_src = n_dst + n_new;
    }
    return TMA_OK;
}

}  // namespace tma

extern "C" int tma_mfg_relabel(int64_t n, int64_t n_dst, const int32_t *dst, int64_t max_items, const int32_t *d_items,
                               int32_t *cols_inout, int32_t *src_out, int64_t cap_src, int64_t *h_n_src, void *ws,
                               size_t ws_bytes, tma_stream_t stream)
{
    const char *fn = "tma_mfg_relabel";
    TMA_REQUIRE(h_n_src, TMA_ERR_INVALID_ARG, "%s: h_n_src is NULL", fn);
    return tma::mfg_relabel(fn, n, n_dst, nullptr, dst, max_items, d_items, cols_inout, src_out, cap_src, h_n_src, nullptr,
                            ws, ws_bytes, stream);
}

extern "C" int tma_mfg_relabel_dev(int64_t n, int64_t cap_dst, const int32_t *d_n_dst, const int32_t *dst,
                                   int64_t max_items, const int32_t *d_items, int32_t *cols_inout, int32_t *src_out,
                                   int64_t cap_src, int32_t *d_n_src_out, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    const char *fn = "tma_mfg_relabel_dev";
    TMA_REQUIRE(d_n_src_out && (cap_dst == 0 || d_n_dst), TMA_ERR_INVALID_ARG, "%s: d_n_src_out / d_n_dst is NULL", fn);
    return tma::mfg_relabel(fn, n, cap_dst, cap_dst > 0 ? d_n_dst : nullptr, dst, max_items, d_items, cols_inout, src_out,
                            cap_src, nullptr, d_n_src_out, ws, ws_bytes, stream);
}

extern "C" int tma_block_inv_deg(int64_t n_dst, const int32_t *blk_rowptr, float *inv_deg_out, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_block_inv_deg";
    TMA_REQUIRE(n_dst >= 0 && n_dst <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n_dst", fn);
    if (n_dst == 0) return TMA_OK;
    TMA_REQUIRE(blk_rowptr && inv_deg_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    hipStream_t s = as_stream(stream);
    TMA_TIMED("block_inv_deg", s);
    hipLaunchKernelGGL(block_inv_deg_kernel, dim3(blocks_for(n_dst)), dim3(256), 0, s, n_dst, blk_rowptr, inv_deg_out);
    return check_launch(fn);
}

extern "C" int tma_sage_block_fwd(int64_t n_dst, int64_t n_src, const int32_t *blk_rowptr, const int32_t *blk_col,
                                  const float *inv_deg, const void *H, int64_t ldh, int32_t F_in, const float *W_self,
                                  const float *W_neigh, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                                  void *M_out, void *Hnext_out, int64_t ld_next, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_sage_block_fwd";
    TMA_REQUIRE(n_dst >= 0 && n_dst <= n_src && n_src <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: need 0 <= n_dst <= n_src", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n_dst == 0) return TMA_OK;
    TMA_REQUIRE(blk_rowptr && inv_deg && H && W_self && W_neigh && bias && M_out && Hnext_out, TMA_ERR_INVALID_ARG,
                "%s: NULL argument", fn);
    TMA_REQUIRE(ldh >= F_in && ld_next >= F_out && H != M_out, TMA_ERR_BAD_SHAPE, "%s: leading dimensions / aliasing", fn);
    hipStream_t s = as_stream(stream);
    if (int rc = launch_spmm(n_dst, blk_rowptr, blk_col, inv_deg, H, ldh, F_in, dtype, M_out, F_in, false, s, n_src))
        return rc;
    return launch_sage_gemm_fwd(n_dst, H, ldh, M_out, F_in, F_in, W_self, W_neigh, bias, F_out, act, dtype, Hnext_out, ld_next, s);
}

extern "C" size_t tma_sage_block_bwd_workspace_bytes(int64_t n_dst, int64_t n_src, int64_t max_entries, int32_t F_in,
                                                     int32_t F_out, int32_t dtype, int32_t need_dH)
{
    if (n_dst < 0 || n_src < n_dst || max_entries < 0 || F_in < 1 || F_out < 1) return 0;
    return tma::plan_block_bwd(n_dst, n_src, max_entries, F_in, F_out, dtype, need_dH != 0).total();
}

extern "C" int tma_sage_block_bwd(int64_t n_dst, int64_t n_src, int64_t max_entries, const int32_t *blk_rowptr,
                                  const int32_t *blk_col, const int32_t *blk_row, const float *inv_deg, const void *H,
                                  int64_t ldh, const void *M, const void *Hnext, const void *dHnext, int64_t ld_next,
                                  const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out, int32_t act,
                                  int32_t dtype, float *dW_self, float *dW_neigh, float *dbias, void *dH_out, void *ws,
                                  size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_sage_block_bwd";
    TMA_REQUIRE(n_dst >= 0 && n_dst <= n_src && n_src <= INT32_MAX && max_entries >= 0 && max_entries <= INT32_MAX,
                TMA_ERR_INVALID_ARG, "%s: need 0 <= n_dst <= n_src", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(dW_self && dW_neigh && dbias, TMA_ERR_INVALID_ARG, "%s: gradient output is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    const bool need_dH = dH_out != nullptr;
    const BlockBwdWorkspace w = plan_block_bwd(n_dst, n_src, max_entries, F_in, F_out, dtype, need_dH);
    TMA_REQUIRE(ws_bytes >= w.total(), TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, ws_bytes,
                w.total());
    if (n_dst > 0) {
        TMA_REQUIRE(H && M && dHnext && W_self && W_neigh, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
        TMA_REQUIRE(act == TMA_ACT_NONE || Hnext, TMA_ERR_INVALID_ARG, "%s: Hnext is required with ReLU", fn);
        TMA_REQUIRE(!need_dH || (blk_rowptr && inv_deg && (max_entries == 0 || (blk_col && blk_row))), TMA_ERR_INVALID_ARG,
                    "%s: block is NULL", fn);
        TMA_REQUIRE(ldh >= F_in && ld_next >= F_out, TMA_ERR_BAD_SHAPE, "%s: ldh < F_in or ld_next < F_out", fn);
    }
    hipStream_t s = as_stream(stream);
    char *base = static_cast<char *>(ws);
    void *dMs = base;
    int32_t *deg = reinterpret_cast<int32_t *>(base + w.dm_bytes);
    int32_t *rowptr_T = reinterpret_cast<int32_t *>(base + w.dm_bytes + w.deg_bytes);
    int32_t *unsorted = reinterpret_cast<int32_t *>(base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes);
    int32_t *sorted = reinterpret_cast<int32_t *>(base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes + w.list_bytes);
    void *scan_ws = base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes + 2 * w.list_bytes;
    void *wws = base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes + 2 * w.list_bytes + w.scan_bytes;

    if (int rc = launch_sage_gemm_bwd_weight(n_dst, H, ldh, M, F_in, dHnext, Hnext, ld_next, F_in, F_out, act, dtype, dW_self,
                                             dW_neigh, dbias, wws, w.weight_bytes, s))
        return rc;
    if (!need_dH || n_src == 0) return TMA_OK;
    // dH rows of the dst nodes: dZ W_self^T; D^-1 dZ W_neigh^T goes to the workspace
    if (int rc = launch_sage_gemm_bwd_data(n_dst, dHnext, Hnext, ld_next, inv_deg, W_self, W_neigh, F_in, F_out, act, dtype,
                                           dH_out, ldh, dMs, s))
        return rc;
    if (int rc = transpose_block(fn, n_dst, n_src, max_entries, blk_rowptr, blk_col, blk_row, deg, rowptr_T, unsorted, sorted,
                                 scan_ws, s))
        return rc;
    // dH += A^T (D^-1 dM): on top of the product for the dst rows, plain for the rows that are sources only
    const int64_t n_rows_dm = n_dst > 0 ? n_dst : 1;
    if (int rc = launch_spmm(n_dst, rowptr_T, sorted, nullptr, dMs, F_in, F_in, dtype, dH_out, ldh, true, s, n_rows_dm))
        return rc;
    char *tail = static_cast<char *>(dH_out) + size_t(n_dst) * size_t(ldh) * elem_size(dtype);
    return launch_spmm(n_src - n_dst, rowptr_T + n_dst, sorted, nullptr, dMs, F_in, F_in, dtype, tail, ldh, false, s,
                       n_rows_dm);
}

// ---- GCN layer on a block: m_v = (h_v + sum over the sampled neighbours) / (|S(v)| + 1) ---------------------------
__global__ __launch_bounds__(256) void gcn_block_norm_kernel(int64_t n_dst, const int32_t *__restrict__ blk_rowptr,
                                                             float *__restrict__ out)
{
    const int64_t v = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (v < n_dst) out[v] = 1.0f / float(blk_rowptr[v + 1] - blk_rowptr[v] + 1);
}

extern "C" int tma_gcn_block_norm(int64_t n_dst, const int32_t *blk_rowptr, float *c_out, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_gcn_block_norm";
    TMA_REQUIRE(n_dst >= 0 && n_dst <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n_dst", fn);
    if (n_dst == 0) return TMA_OK;
    TMA_REQUIRE(blk_rowptr && c_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    hipStream_t s = as_stream(stream);
    TMA_TIMED("gcn_block_norm", s);
    hipLaunchKernelGGL(gcn_block_norm_kernel, dim3(blocks_for(n_dst)), dim3(256), 0, s, n_dst, blk_rowptr, c_out);
    return check_launch(fn);
}

extern "C" int tma_gcn_block_fwd(int64_t n_dst, int64_t n_src, const int32_t *blk_rowptr, const int32_t *blk_col,
                                 const float *c_norm, const void *H, int64_t ldh, int32_t F_in, const float *W,
                                 const float *bias, int32_t F_out, int32_t act, int32_t dtype, void *M_out, void *Hnext_out,
                                 int64_t ld_next, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_gcn_block_fwd";
    TMA_REQUIRE(n_dst >= 0 && n_dst <= n_src && n_src <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: need 0 <= n_dst <= n_src", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    if (n_dst == 0) return TMA_OK;
    TMA_REQUIRE(blk_rowptr && c_norm && H && W && bias && M_out && Hnext_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    TMA_REQUIRE(ldh >= F_in && ld_next >= F_out && H != M_out, TMA_ERR_BAD_SHAPE, "%s: leading dimensions / aliasing", fn);
    TMA_REQUIRE(aligned(M_out, 16), TMA_ERR_INVALID_ARG, "%s: M_out must be 16-byte aligned", fn);
    hipStream_t s = as_stream(stream);
    // one pass over the sampled rows: neighbours and the own row summed, the sum scaled by 1 / (|S(v)| + 1)
    if (int rc = launch_spmm_combine(n_dst, blk_rowptr, blk_col, c_norm, H, ldh, F_in, dtype, M_out, F_in, false, H, ldh,
                                     nullptr, F_in, false, true, nullptr, s, n_src))
        return rc;
    return launch_dense_gemm_fwd(n_dst, M_out, F_in, F_in, W, bias, nullptr, F_out, F_out, act, dtype, Hnext_out, ld_next, s);
}

extern "C" size_t tma_gcn_block_bwd_workspace_bytes(int64_t n_dst, int64_t n_src, int64_t max_entries, int32_t F_in,
                                                    int32_t F_out, int32_t dtype, int32_t need_dH)
{
    if (n_dst < 0 || n_src < n_dst || max_entries < 0 || F_in < 1 || F_out < 1) return 0;
    return tma::plan_gcn_block_bwd(n_dst, n_src, max_entries, F_in, F_out, dtype, need_dH != 0).total();
}

extern "C" int tma_gcn_block_bwd(int64_t n_dst, int64_t n_src, int64_t max_entries, const int32_t *blk_rowptr,
                                 const int32_t *blk_col, const int32_t *blk_row, const float *c_norm, const void *M,
                                 const void *Hnext, const void *dHnext, int64_t ld_next, const float *W, int32_t F_in,
                                 int32_t F_out, int32_t act, int32_t dtype, float *dW, float *dbias, void *dH_out,
                                 int64_t ldh, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_gcn_block_bwd";
    TMA_REQUIRE(n_dst >= 0 && n_dst <= n_src && n_src <= INT32_MAX && max_entries >= 0 && max_entries <= INT32_MAX,
                TMA_ERR_INVALID_ARG, "%s: need 0 <= n_dst <= n_src", fn);
    TMA_REQUIRE(F_in >= 1 && F_out >= 1 && F_in <= (1 << 20) && F_out <= (1 << 20), TMA_ERR_BAD_SHAPE,
                "%s: F_in=%d F_out=%d", fn, F_in, F_out);
    TMA_REQUIRE(act == TMA_ACT_NONE || act == TMA_ACT_RELU, TMA_ERR_INVALID_ARG, "%s: act %d", fn, act);
    TMA_REQUIRE(dtype == TMA_F32 || dtype == TMA_BF16, TMA_ERR_UNSUPPORTED_DTYPE, "%s: dtype %d", fn, dtype);
    TMA_REQUIRE(dW && dbias, TMA_ERR_INVALID_ARG, "%s: gradient output is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    const bool need_dH = dH_out != nullptr;
    const BlockBwdWorkspace w = plan_gcn_block_bwd(n_dst, n_src, max_entries, F_in, F_out, dtype, need_dH);
    TMA_REQUIRE(ws_bytes >= w.total(), TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, ws_bytes,
                w.total());
    if (n_dst > 0) {
        TMA_REQUIRE(M && dHnext && W, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
        TMA_REQUIRE(act == TMA_ACT_NONE || Hnext, TMA_ERR_INVALID_ARG, "%s: Hnext is required with ReLU", fn);
        TMA_REQUIRE(!need_dH || (blk_rowptr && c_norm && (max_entries == 0 || (blk_col && blk_row))), TMA_ERR_INVALID_ARG,
                    "%s: block is NULL", fn);
        TMA_REQUIRE(ld_next >= F_out && (!need_dH || ldh >= F_in), TMA_ERR_BAD_SHAPE, "%s: ldh < F_in or ld_next < F_out", fn);
    }
    hipStream_t s = as_stream(stream);
    char *base = static_cast<char *>(ws);
    void *P = base;      // c_v (dZ W^T)_v, one row per dst node
    int32_t *deg = reinterpret_cast<int32_t *>(base + w.dm_bytes);
    int32_t *rowptr_T = reinterpret_cast<int32_t *>(base + w.dm_bytes + w.deg_bytes);
    int32_t *unsorted = reinterpret_cast<int32_t *>(base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes);
    int32_t *sorted = reinterpret_cast<int32_t *>(base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes + w.list_bytes);
    void *scan_ws = base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes + 2 * w.list_bytes;
    void *wws = base + w.dm_bytes + w.deg_bytes + w.rowptr_bytes + 2 * w.list_bytes + w.scan_bytes;

    // dW = M^T dZ, db = 1^T dZ
    if (int rc = launch_dense_gemm_bwd_weight(n_dst, M, F_in, dHnext, Hnext, ld_next, F_in, F_out, act, dtype, dW, dbias,
                                              wws, w.weight_bytes, s))
        return rc;
    if (!need_dH || n_src == 0) return TMA_OK;
    if (int rc = launch_dense_gemm_bwd_data(n_dst, dHnext, Hnext, ld_next, W, F_in, F_out, act, dtype, c_norm, P, F_in, s))
        return rc;
    if (int rc = transpose_block(fn, n_dst, n_src, max_entries, blk_rowptr, blk_col, blk_row, deg, rowptr_T, unsorted, sorted,
                                 scan_ws, s))
        return rc;
    // dH = (A_S + I)^T P: the dst rows take their own row of P on top of the gathered ones, the others gather only
    const int64_t n_rows_p = n_dst > 0 ? n_dst : 1;
    if (int rc = launch_spmm_combine(n_dst, rowptr_T, sorted, nullptr, P, F_in, F_in, dtype, dH_out, ldh, false, P, F_in,
                                     nullptr, F_in, false, false, nullptr, s, n_rows_p))
        return rc;
    char *tail = static_cast<char *>(dH_out) + size_t(n_dst) * size_t(ldh) * elem_size(dtype);
    return launch_spmm(n_src - n_dst, rowptr_T + n_dst, sorted, nullptr, P, F_in, F_in, dtype, tail, ldh, false, s, n_rows_p);
}
