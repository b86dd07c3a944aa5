// Node-induced subgraph of one partition (paper, Preliminaries):
//   V^(p) = alpha^-1(p),  E^(p) = edges of E with both end points in V^(p).
//
// Integer-only, HBM-scan bound.  Two prefix scans (local-node flags, kept
// degrees) done as reduce -> scan-of-block-sums -> apply, which needs no
// inter-block waiting, and an order-preserving compaction that uses wavefront
// ballots over the concatenated entries of sixteen consecutive local rows.
//
// The flag scan also leaves, for the two passes over the local rows, a
// membership bitmap (one bit per global node: 1/32 of the bytes of the id map,
// so the random look-ups per entry stay in cache) and each local row's bounds in
// the global CSR in local order (read coalesced instead of through l2g ->
// rowptr).  Only entries that are kept go on to the id map.
#include "common.hpp"

#include <type_traits>

namespace tma {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;                           // consecutive items per thread
constexpr int kScanTile = kScanThreads * kScanItems;    // items per block
constexpr int kWaveRows = 16;                           // consecutive local rows per wavefront
constexpr int kRowsPerBlock = (256 / kWave) * kWaveRows;

// ---- value sources / sinks of the two scans -------------------------------
struct FlagIn {  // 1 where the node belongs to partition p
    const int32_t *part;
    int32_t p;
    __device__ int32_t load(int64_t i) const { return part[i] == p ? 1 : 0; }
    // eight consecutive items from a 32-byte aligned position: two 16-byte loads
    __device__ bool load8(int64_t first, int32_t (&v)[8]) const
    {
        if ((reinterpret_cast<uintptr_t>(part) & 15) != 0) return false;
        const int4 a = *reinterpret_cast<const int4 *>(part + first);
        const int4 b = *reinterpret_cast<const int4 *>(part + first + 4);
        v[0] = a.x == p; v[1] = a.y == p; v[2] = a.z == p; v[3] = a.w == p;
        v[4] = b.x == p; v[5] = b.y == p; v[6] = b.z == p; v[7] = b.w == p;
        return true;
    }
};
struct RuleIn {  // the same flag, computed: RandomTMA's assignment of node i is a pure function of (seed, i)
    uint64_t seed;
    uint32_t K;
    int32_t p;
    __device__ int32_t load(int64_t i) const
    {
        return int32_t(__umul64hi(splitmix64_at(seed, uint64_t(i)), uint64_t(K))) == p ? 1 : 0;
    }
    __device__ bool load8(int64_t first, int32_t (&v)[8]) const
    {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = load(first + j);
        return true;
    }
};

struct FlagOut {  // local id = exclusive rank; inverse map, row bounds for the first `cap` local nodes; bitmap
    int32_t *g2l;
    int32_t *l2g;
    int64_t cap;
    const int64_t *rowptr;
    int64_t *row_beg;
    int32_t *row_len;
    uint8_t *member;
    __device__ void store(int64_t i, int64_t prefix, int32_t v, int64_t /*n*/) const
    {
        g2l[i] = v ? int32_t(prefix) : -1;
        if (v && prefix < cap) {
            l2g[prefix] = int32_t(i);
            const int64_t b = rowptr[i];
            row_beg[prefix] = b;
            row_len[prefix] = int32_t(rowptr[i + 1] - b);
        }
    }
    // all eight items of a thread at once: the id map goes out as two 16-byte stores
    __device__ bool store8(int64_t first, int64_t prefix, const int32_t (&v)[8]) const
    {
        if ((reinterpret_cast<uintptr_t>(g2l) & 15) != 0) return false;
        int32_t id[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            id[j] = v[j] ? int32_t(prefix) : -1;
            if (v[j] && prefix < cap) {
                l2g[prefix] = int32_t(first + j);
                const int64_t b = rowptr[first + j];
                row_beg[prefix] = b;
                row_len[prefix] = int32_t(rowptr[first + j + 1] - b);
            }
            prefix += v[j];
        }
        *reinterpret_cast<int4 *>(g2l + first) = make_int4(id[0], id[1], id[2], id[3]);
        *reinterpret_cast<int4 *>(g2l + first + 4) = make_int4(id[4], id[5], id[6], id[7]);
        return true;
    }
    // the eight flags of one thread's consecutive items (first item = bit 0) are one byte of the bitmap
    __device__ void store_flags(int64_t first, uint32_t bits, int64_t n) const
    {
        if (first < n) member[first >> 3] = uint8_t(bits);
    }
};
struct DegIn {
    const int32_t *deg;
    __device__ int32_t load(int64_t i) const { return deg[i]; }
    __device__ bool load8(int64_t first, int32_t (&v)[8]) const
    {
        if ((reinterpret_cast<uintptr_t>(deg) & 15) != 0) return false;
        const int4 a = *reinterpret_cast<const int4 *>(deg + first);
        const int4 b = *reinterpret_cast<const int4 *>(deg + first + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        return true;
    }
};
struct DegOut {  // rowptr_loc[i] = exclusive prefix, rowptr_loc[n] = total
    int32_t *rowptr_loc;
    __device__ void store(int64_t i, int64_t prefix, int32_t v, int64_t n) const
    {
        rowptr_loc[i] = int32_t(prefix);
        if (i == n - 1) rowptr_loc[n] = int32_t(prefix + v);
    }
    __device__ void store_flags(int64_t, uint32_t, int64_t) const {}
    __device__ bool store8(int64_t first, int64_t prefix, const int32_t (&v)[8]) const
    {
        if ((reinterpret_cast<uintptr_t>(rowptr_loc) & 15) != 0) return false;
        int32_t x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = int32_t(prefix);
            prefix += v[j];
        }
        *reinterpret_cast<int4 *>(rowptr_loc + first) = make_int4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<int4 *>(rowptr_loc + first + 4) = make_int4(x[4], x[5], x[6], x[7]);
        return true;
    }
};

__device__ __forceinline__ int64_t effective_n(const int64_t *d_n, int64_t cap)
{
    if (!d_n) return cap;
    int64_t n = *d_n;
    return n < cap ? n : cap;
}

// Block-wide exclusive scan of one int per thread (256 threads = 4 wavefronts).
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t &block_total)
{
    __shared__ int32_t wave_sums[kScanThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    int32_t incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int32_t t = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += t;
    }
    if (lane == kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    int32_t offset = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / kWave; ++w) {
        int32_t s = wave_sums[w];
        if (w < wave) offset += s;
        total += s;
    }
    __syncthreads();
    block_total = total;
    return offset + incl - v;
}

template <class In>
__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(const int64_t *d_n, int64_t cap, In in,
                                                                   int64_t *__restrict__ block_sums)
{
    const int64_t n = effective_n(d_n, cap);
    const int64_t base = int64_t(blockIdx.x) * kScanTile + int64_t(threadIdx.x) * kScanItems;
    int32_t c = 0;
    int32_t v[kScanItems];
    if (base + kScanItems <= n && in.load8(base, v)) {
#pragma unroll
        for (int j = 0; j < kScanItems; ++j) c += v[j];
    } else {
#pragma unroll
        for (int j = 0; j < kScanItems; ++j)
            if (base + j < n) c += in.load(base + j);
    }
    int32_t total;
    block_exclusive_scan(c, total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// One block turns the per-block sums into exclusive offsets and stores the
// grand total.  nb is at most a few 10^4 (10^8 nodes / 2048).
__global__ __launch_bounds__(1024) void scan_sums_kernel(int64_t nb, int64_t *__restrict__ block_sums,
                                                         int64_t *__restrict__ total_out, int32_t *first_out)
{
    // first_out: rowptr_loc[0] = 0 also when the partition is empty (the apply kernel then stores nothing)
    if (threadIdx.x == 0 && first_out) *first_out = 0;
    __shared__ int64_t wave_sums[1024 / kWave];
    __shared__ int64_t carry_s;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < nb; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int64_t v = i < nb ? block_sums[i] : 0;
        int64_t incl = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            int64_t t = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += t;
        }
        if (lane == kWave - 1) wave_sums[wave] = incl;
        __syncthreads();
        int64_t offset = carry_s, chunk_total = 0;
        for (int w = 0; w < 1024 / kWave; ++w) {
            int64_t s = wave_sums[w];
            if (w < wave) offset += s;
            chunk_total += s;
        }
        if (i < nb) block_sums[i] = offset + incl - v;
        __syncthreads();
        if (threadIdx.x == 0) carry_s += chunk_total;
        __syncthreads();
    }
    if (threadIdx.x == 0) *total_out = carry_s;
}

// Sum over the workgroup of one 64-bit value per thread, returned to every thread.
__device__ __forceinline__ int64_t block_sum_i64(int64_t v)
{
    __shared__ int64_t wave_sums64[kScanThreads / kWave];
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) wave_sums64[threadIdx.x / kWave] = v;
    __syncthreads();
    int64_t total = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / kWave; ++w) total += wave_sums64[w];
    __syncthreads();
    return total;
}

// Up to this many tiles the apply kernel adds up the tile sums before its own tile by itself (a few loads per
// thread) and no kernel scans them; above it scan_sums_kernel turns them into offsets first.
constexpr int64_t kInlineTiles = 1024;

// block_sums: per-tile sums (total_out != nullptr: this kernel derives its offset from them, and its first
// workgroup stores the grand total to total_out and 0 to first_out, if given) or per-tile exclusive offsets
// (total_out == nullptr).  zero_out[0 .. zero_n) is cleared, one element per workgroup, for a later kernel.
template <class In, class Out>
__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(const int64_t *d_n, int64_t cap, In in, Out out,
                                                                  const int64_t *__restrict__ block_sums,
                                                                  int64_t *__restrict__ total_out,
                                                                  int32_t *__restrict__ first_out,
                                                                  int64_t *__restrict__ zero_out, int64_t zero_n)
{
    if (zero_out && threadIdx.x == 0 && int64_t(blockIdx.x) < zero_n) zero_out[blockIdx.x] = 0;
    int64_t tile_offset;
    if (total_out) {
        int64_t before = 0, all = 0;
        for (int64_t b = threadIdx.x; b < int64_t(gridDim.x); b += kScanThreads) {
            const int64_t v = block_sums[b];
            all += v;
            if (b < int64_t(blockIdx.x)) before += v;
        }
        tile_offset = block_sum_i64(before);
        all = block_sum_i64(all);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            *total_out = all;
            if (first_out) *first_out = 0;
        }
    } else {
        tile_offset = block_sums[blockIdx.x];
    }
    const int64_t n = effective_n(d_n, cap);
    const int64_t base = int64_t(blockIdx.x) * kScanTile + int64_t(threadIdx.x) * kScanItems;
    static_assert(kScanItems == 8, "one thread's flags are one byte of the bitmap");
    int32_t v[kScanItems];
    int32_t c = 0;
    uint32_t bits = 0;
    const bool whole = base + kScanItems <= n;   // all eight items exist: 16-byte loads and stores where aligned
    if (!(whole && in.load8(base, v))) {
#pragma unroll
        for (int j = 0; j < kScanItems; ++j) v[j] = (base + j < n) ? in.load(base + j) : 0;
    }
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        c += v[j];
        bits |= (v[j] != 0 ? 1u : 0u) << j;
    }
    out.store_flags(base, bits, n);
    int32_t total;
    int64_t prefix = tile_offset + block_exclusive_scan(c, total);
    // the last item also closes the output (DegOut writes the total after it): left to the item-wise path
    if (whole && base + kScanItems < n && out.store8(base, prefix, v)) return;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (base + j < n) out.store(base + j, prefix, v[j], n);
        prefix += v[j];
    }
}

// Does global node u belong to the part?  Read from the bitmap that the flag scan leaves (any assignment), or
// recomputed from the assignment rule (RandomTMA: a few integer multiplies instead of a random memory access; on
// graphs whose bitmap outgrows the L2 the look-ups, not the entries, bound the two row passes).
struct BitMember {
    const uint32_t *__restrict__ bits;
    __device__ __forceinline__ int operator()(int32_t u) const
    {
        return int((bits[uint32_t(u) >> 5] >> (uint32_t(u) & 31u)) & 1u);
    }
};
struct RuleMember {
    uint64_t seed;
    uint32_t K;
    int32_t p;
    __device__ __forceinline__ int operator()(int32_t u) const
    {
        return int32_t(__umul64hi(splitmix64_at(seed, uint64_t(uint32_t(u))), uint64_t(K))) == p ? 1 : 0;
    }
};

// The two passes over the local rows walk the entries of kWaveRows consecutive rows as ONE stream per wavefront:
// lane j < kWaveRows holds row j's bounds, a prefix sum over the row lengths gives every stream position its row,
// and the 64 lanes take 64 consecutive stream positions per chunk, kStreamChunks chunks in flight.  All lanes
// carry entries whatever the degree distribution (rows of 2 entries next to rows of 900), every lane has
// several independent index -> bit (-> id) chains in flight, and there is no workgroup barrier on this path.
// Rows longer than kGiantRow are left out of the stream and scanned by the whole workgroup afterwards
// (power-law graphs: a handful of rows hold thousands of entries and would otherwise set the kernel's tail).
constexpr int kGiantRow = 512;
constexpr int kStreamChunks = 4;

struct RowStream {
    int32_t start[kWaveRows];  // wave-uniform: stream position of row j's first entry
    int32_t total;             // wave-uniform: entries in the stream
    int64_t adjust;            // lane j: row_beg[j] - start[j]  (global CSR position = adjust[row] + stream position)
    int32_t first, last;       // lane j: the stream positions [first, last) of row j

    // len: lane j's row length as it enters the stream (0 for lanes >= kWaveRows and for rows left out)
    __device__ __forceinline__ void build(int64_t beg, int32_t len)
    {
        const int lane = threadIdx.x & (kWave - 1);
        int32_t incl = len;
#pragma unroll
        for (int d = 1; d < kWaveRows; d <<= 1) {
            const int32_t t = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += t;
        }
        first = incl - len;
        last = incl;
        adjust = beg - first;
#pragma unroll
        for (int j = 0; j < kWaveRows; ++j) start[j] = __builtin_amdgcn_readlane(first, j);
        total = __builtin_amdgcn_readlane(incl, kWaveRows - 1);
    }
    // row of stream position t < total: the last row that starts at or before t (rows without entries
    // share their start with the row after them and are passed over)
    __device__ __forceinline__ int row_of(int32_t t) const
    {
        int r = 0;
#pragma unroll
        for (int j = 1; j < kWaveRows; ++j) r += t >= start[j] ? 1 : 0;
        return r;
    }
    // bits of a 64-position chunk starting at stream position c that belong to this lane's row
    __device__ __forceinline__ uint64_t own_bits(int32_t c) const
    {
        int32_t lo = first - c, hi = last - c;
        lo = lo < 0 ? 0 : (lo > kWave ? kWave : lo);
        hi = hi < 0 ? 0 : (hi > kWave ? kWave : hi);
        const uint64_t below_hi = hi >= kWave ? ~0ull : ((1ull << hi) - 1ull);
        const uint64_t below_lo = lo >= kWave ? ~0ull : ((1ull << lo) - 1ull);
        return below_hi & ~below_lo;
    }
};

// Kept degree of every local row: entries whose column is local too.
template <class Member>
__global__ __launch_bounds__(256) void row_count_kernel(const int64_t *d_n_loc, int64_t cap,
                                                        const int64_t *__restrict__ row_beg,
                                                        const int32_t *__restrict__ row_len,
                                                        const int32_t *__restrict__ colidx, Member member,
                                                        int32_t *__restrict__ deg,
                                                        int64_t *__restrict__ tile_sums)
{
    // tile_sums (may be NULL): tile_sums[t] (zero on entry) receives the kept degrees of the scan tile t that this workgroup's rows lie in:
    // the first stage of the scan that turns deg into rowptr_loc (integer atomics: the sum has one value)
    static_assert(kScanTile % kRowsPerBlock == 0, "the rows of a workgroup lie within one scan tile");
    __shared__ int32_t giant_rows[kRowsPerBlock];
    __shared__ int32_t giant_count;
    __shared__ int32_t block_kept;
    __shared__ int32_t wave_part[256 / kWave];
    if (threadIdx.x == 0) {
        giant_count = 0;
        block_kept = 0;
    }
    __syncthreads();

    const int64_t n_loc = effective_n(d_n_loc, cap);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t row0 = int64_t(blockIdx.x) * kRowsPerBlock;
    const int64_t i = row0 + wave * kWaveRows + lane;      // this lane's row (lanes < kWaveRows)
    const bool has_row = lane < kWaveRows && i < n_loc;
    int64_t beg = 0;
    int32_t len = 0;
    if (has_row) {
        beg = row_beg[i];
        len = row_len[i];
        if (len > kGiantRow) {
            giant_rows[atomicAdd(&giant_count, 1)] = int32_t(i - row0);
            len = -1;
        }
    }
    const bool in_stream = has_row && len >= 0;
    RowStream st;
    st.build(beg, len > 0 ? len : 0);
    int32_t c = 0;
    for (int32_t c0 = 0; c0 < st.total; c0 += kStreamChunks * kWave) {
        int32_t u[kStreamChunks];
#pragma unroll
        for (int q = 0; q < kStreamChunks; ++q) {
            u[q] = -1;
            if (c0 + q * kWave >= st.total) continue;     // wave-uniform: the chunk lies past the end
            const int32_t t = c0 + q * kWave + lane;
            // every lane takes part in the shuffle (positions past the end ask for row_of(0), a valid lane)
            const int64_t base = __shfl(st.adjust, st.row_of(t < st.total ? t : 0), kWave);
            if (t < st.total) u[q] = colidx[base + t];
        }
#pragma unroll
        for (int q = 0; q < kStreamChunks; ++q) {
            if (c0 + q * kWave >= st.total) continue;
            const bool keep = u[q] >= 0 && member(u[q]) != 0;
            c += __popcll(__ballot(keep) & st.own_bits(c0 + q * kWave));
        }
    }
    if (in_stream) deg[i] = c;
    int32_t wave_kept = c;       // lanes past the rows of the wavefront hold 0
#pragma unroll
    for (int d = kWaveRows / 2; d >= 1; d >>= 1) wave_kept += __shfl_xor(wave_kept, d, kWave);
    if (lane == 0 && wave_kept) atomicAdd(&block_kept, wave_kept);
    __syncthreads();

    const int n_giants = giant_count;
    for (int h = 0; h < n_giants; ++h) {
        const int64_t ih = row0 + giant_rows[h];
        const int64_t end = row_beg[ih] + row_len[ih];
        int32_t ch = 0;
        for (int64_t e = row_beg[ih] + threadIdx.x; e < end; e += 4 * 256) {  // up to four index -> bit chains in flight
            int32_t u[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) u[j] = e + j * 256 < end ? colidx[e + j * 256] : -1;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (u[j] >= 0) ch += member(u[j]);
        }
#pragma unroll
        for (int d = kWave / 2; d >= 1; d >>= 1) ch += __shfl_xor(ch, d, kWave);
        if ((threadIdx.x & (kWave - 1)) == 0) wave_part[threadIdx.x / kWave] = ch;
        __syncthreads();
        if (threadIdx.x == 0) {
            const int32_t kept = wave_part[0] + wave_part[1] + wave_part[2] + wave_part[3];
            deg[ih] = kept;
            block_kept += kept;
        }
        __syncthreads();
    }
    if (tile_sums && threadIdx.x == 0 && block_kept)
        atomicAdd(reinterpret_cast<unsigned long long *>(tile_sums + row0 / kScanTile),
                  static_cast<unsigned long long>(block_kept));
}

// Order-preserving compaction of each local row into colidx_loc, relabelled.
// n_loc rows at most; with d_n_loc the actual count is read from the device (a launch sized by capacity).  A row
// whose entries would end past cap_nnz is skipped: the caller's buffer is then too small and the sizes say so.
// The rows of a wavefront are consecutive, so are their ranges in colidx_loc: the kept entries of the stream go
// to consecutive positions from the first row's offset on, shifted by the kept entries of the giant rows left
// out of the stream before them.
template <class Member>
__global__ __launch_bounds__(256) void row_fill_kernel(int64_t n_loc, const int64_t *__restrict__ d_n_loc,
                                                       int64_t cap_nnz, const int64_t *__restrict__ row_beg,
                                                       const int32_t *__restrict__ row_len,
                                                       const int32_t *__restrict__ colidx, Member member,
                                                       const int32_t *__restrict__ g2l,
                                                       const int32_t *__restrict__ rowptr_loc,
                                                       int32_t *__restrict__ colidx_loc,
                                                       float *__restrict__ inv_deg)
{
    __shared__ int32_t giant_rows[kRowsPerBlock];
    __shared__ int32_t giant_count;
    __shared__ int32_t wave_part[256 / kWave];
    if (threadIdx.x == 0) giant_count = 0;
    __syncthreads();

    if (d_n_loc) {
        const int64_t actual = *d_n_loc;
        n_loc = actual < n_loc ? actual : n_loc;
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t row0 = int64_t(blockIdx.x) * kRowsPerBlock;
    const int64_t i = row0 + wave * kWaveRows + lane;
    int64_t beg = 0;
    int32_t len = 0, out = 0, left_out = 0;
    if (lane < kWaveRows && i < n_loc) {
        beg = row_beg[i];
        len = row_len[i];
        out = rowptr_loc[i];
        const int32_t end = rowptr_loc[i + 1];
        inv_deg[i] = end > out ? 1.0f / float(end - out) : 0.0f;
        // nothing to write: a row without kept entries (most rows of a sparse part) never touches colidx again
        if (int64_t(end) > cap_nnz || end == out) len = 0;
        if (len > kGiantRow) {  // left to the whole workgroup below
            giant_rows[atomicAdd(&giant_count, 1)] = int32_t(i - row0);
            left_out = end - out;
            len = 0;
        }
    }
    RowStream st;
    st.build(beg, len);
    // kept entries of the giant rows before this lane's row, among the rows of the wavefront
    int32_t shift = left_out;
#pragma unroll
    for (int d = 1; d < kWaveRows; d <<= 1) {
        const int32_t t = __shfl_up(shift, d, kWave);
        if (lane >= d) shift += t;
    }
    shift -= left_out;
    int32_t pos = __builtin_amdgcn_readlane(out, 0);     // next free position of the stream's output
    for (int32_t c0 = 0; c0 < st.total; c0 += kStreamChunks * kWave) {
        int32_t u[kStreamChunks], lid[kStreamChunks], extra[kStreamChunks];
        bool keep[kStreamChunks];
#pragma unroll
        for (int q = 0; q < kStreamChunks; ++q) {
            u[q] = -1;
            extra[q] = 0;
            if (c0 + q * kWave >= st.total) continue;          // wave-uniform: the chunk lies past the end
            const int32_t t = c0 + q * kWave + lane;
            const int r = st.row_of(t < st.total ? t : 0);     // every lane takes part in the shuffles
            const int64_t base = __shfl(st.adjust, r, kWave);
            extra[q] = __shfl(shift, r, kWave);
            if (t < st.total) u[q] = colidx[base + t];
        }
#pragma unroll
        for (int q = 0; q < kStreamChunks; ++q) keep[q] = u[q] >= 0 && member(u[q]) != 0;
#pragma unroll
        for (int q = 0; q < kStreamChunks; ++q) lid[q] = keep[q] ? g2l[u[q]] : 0;
#pragma unroll
        for (int q = 0; q < kStreamChunks; ++q) {
            if (c0 + q * kWave >= st.total) continue;
            const uint64_t ballot = __ballot(keep[q]);
            if (keep[q]) colidx_loc[pos + extra[q] + __popcll(ballot & ((1ull << lane) - 1ull))] = lid[q];
            pos += __popcll(ballot);
        }
    }
    __syncthreads();

    // Giant rows: the whole workgroup, 4 consecutive entries per thread and round (1024 per round, order kept: a
    // thread's entries follow those of all lower threads).  The longest row of a power-law graph sets the tail of
    // this kernel, so a round carries as many independent index -> bit -> id chains as the registers allow.
    const int n_hubs = giant_count;
    constexpr int kPerThread = 4;
    for (int h = 0; h < n_hubs; ++h) {
        const int64_t ih = row0 + giant_rows[h];
        const int64_t hbeg = row_beg[ih], hend = hbeg + row_len[ih];
        int32_t hout = rowptr_loc[ih];
        int32_t u_next[kPerThread];
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            const int64_t e = hbeg + int64_t(threadIdx.x) * kPerThread + j;
            u_next[j] = e < hend ? colidx[e] : -1;
        }
        for (int64_t off = 0; off < hend - hbeg; off += 256 * kPerThread) {
            int32_t u[kPerThread], lid[kPerThread];
            bool keep[kPerThread];
            uint64_t ballot[kPerThread];
#pragma unroll
            for (int j = 0; j < kPerThread; ++j) u[j] = u_next[j];
#pragma unroll
            for (int j = 0; j < kPerThread; ++j) {   // next round's entries are fetched during this one
                const int64_t e = hbeg + off + 256 * kPerThread + int64_t(threadIdx.x) * kPerThread + j;
                u_next[j] = e < hend ? colidx[e] : -1;
            }
#pragma unroll
            for (int j = 0; j < kPerThread; ++j) keep[j] = u[j] >= 0 && member(u[j]) != 0;
#pragma unroll
            for (int j = 0; j < kPerThread; ++j) lid[j] = keep[j] ? g2l[u[j]] : 0;
            int32_t wave_kept = 0, below = 0;
#pragma unroll
            for (int j = 0; j < kPerThread; ++j) {
                ballot[j] = __ballot(keep[j]);
                wave_kept += __popcll(ballot[j]);
                below += __popcll(ballot[j] & ((1ull << lane) - 1ull));
            }
            if (lane == 0) wave_part[wave] = wave_kept;
            __syncthreads();
            int32_t before = 0, total = 0;
#pragma unroll
            for (int w = 0; w < 256 / kWave; ++w) {
                const int32_t t = wave_part[w];
                if (w < wave) before += t;
                total += t;
            }
            int32_t pos = hout + before + below;
#pragma unroll
            for (int j = 0; j < kPerThread; ++j) {
                if (keep[j]) colidx_loc[pos++] = lid[j];
            }
            hout += total;
            __syncthreads();
        }
    }
}

struct CountWorkspace {
    int64_t *node_block_sums;  // [nb_nodes]
    int64_t *row_block_sums;   // [nb_rows]
    int64_t *sizes;            // [2] n_loc, nnz_loc
    int32_t *deg;              // [cap_n_loc]
    int64_t *row_beg;          // [cap_n_loc] first entry of the local row in the global CSR
    int32_t *row_len;          // [cap_n_loc] its global degree
    uint32_t *member;          // bit v = node v belongs to the partition
    size_t bytes;
};

static CountWorkspace carve(void *ws, int64_t n_nodes, int64_t cap)
{
    const int64_t nb_nodes = ceil_div(n_nodes > 0 ? n_nodes : 1, kScanTile);
    const int64_t nb_rows = ceil_div(cap > 0 ? cap : 1, kScanTile);
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    CountWorkspace w;
    w.node_block_sums = reinterpret_cast<int64_t *>(p + off);
    off += round_up(size_t(nb_nodes) * 8, 256);
    w.row_block_sums = reinterpret_cast<int64_t *>(p + off);
    off += round_up(size_t(nb_rows) * 8, 256);
    w.sizes = reinterpret_cast<int64_t *>(p + off);
    off += 256;
    w.deg = reinterpret_cast<int32_t *>(p + off);
    off += round_up(size_t(cap > 0 ? cap : 1) * 4, 256);
    w.row_beg = reinterpret_cast<int64_t *>(p + off);
    off += round_up(size_t(cap > 0 ? cap : 1) * 8, 256);
    w.row_len = reinterpret_cast<int32_t *>(p + off);
    off += round_up(size_t(cap > 0 ? cap : 1) * 4, 256);
    w.member = reinterpret_cast<uint32_t *>(p + off);
    off += round_up(size_t(n_nodes > 0 ? n_nodes : 1) / 8 + 8, 256);
    w.bytes = off;
    return w;
}

size_t exclusive_scan_i32_workspace_bytes(int64_t n)
{
    return round_up(size_t(ceil_div(n > 0 ? n : 1, kScanTile) + 1) * sizeof(int64_t), 256);
}

int launch_exclusive_scan_i32(int64_t n, const int32_t *values, int32_t *prefix_out, void *ws, hipStream_t s)
{
    int64_t *block_sums = static_cast<int64_t *>(ws);
    const int64_t nb = n > 0 ? ceil_div(n, kScanTile) : 0;
    int64_t *total = block_sums + (nb > 0 ? nb : 1);
    DegIn in{values};
    DegOut out{prefix_out};
    TMA_TIMED("exclusive_scan", s);
    if (nb > 0)
        hipLaunchKernelGGL(scan_reduce_kernel<DegIn>, dim3(unsigned(nb)), dim3(kScanThreads), 0, s,
                           static_cast<const int64_t *>(nullptr), n, in, block_sums);
    const bool inline_sums = nb > 0 && nb <= kInlineTiles;
    if (!inline_sums) hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(1024), 0, s, nb, block_sums, total, prefix_out);
    if (nb > 0)
        hipLaunchKernelGGL((scan_apply_kernel<DegIn, DegOut>), dim3(unsigned(nb)), dim3(kScanThreads), 0, s,
                           static_cast<const int64_t *>(nullptr), n, in, out, block_sums,
                           inline_sums ? total : nullptr, inline_sums ? prefix_out : nullptr,
                           static_cast<int64_t *>(nullptr), int64_t(0));
    return check_launch("exclusive scan");
}

}  // namespace tma

extern "C" size_t tma_induced_subgraph_workspace_bytes(int64_t n_nodes, int64_t cap_n_loc)
{
    if (n_nodes < 0 || cap_n_loc < 0) return 0;
    return tma::carve(nullptr, n_nodes, cap_n_loc).bytes;
}

namespace tma {

// The counting pass, enqueued on the stream: flags, node ranks, kept degrees, rowptr_loc.  The two totals
// (|V^(p)|, kept entries) end up in sizes[0..1] (device memory); nothing here waits for the GPU.
// kRule: membership comes from RandomTMA's assignment rule (seed, K) instead of a part array.
template <bool kRule>
static int enqueue_count(const char *fn, int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                         const int32_t *part, int32_t p, int32_t K, uint64_t seed, int32_t *g2l_out, int32_t *l2g_out,
                         int32_t *rowptr_loc_out, int64_t cap_n_loc, int64_t *sizes, void *ws, size_t ws_bytes,
                         hipStream_t s)
{
    using In = std::conditional_t<kRule, RuleIn, FlagIn>;
    using Member = std::conditional_t<kRule, RuleMember, BitMember>;
    TMA_REQUIRE(n_nodes >= 0 && n_nodes <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: n_nodes outside [0, 2^31)", fn);
    TMA_REQUIRE(cap_n_loc >= 0 && cap_n_loc <= n_nodes, TMA_ERR_INVALID_ARG,
                "%s: cap_n_loc must lie in [0, n_nodes]", fn);
    TMA_REQUIRE(rowptr_loc_out, TMA_ERR_INVALID_ARG, "%s: rowptr_loc_out is NULL", fn);
    TMA_REQUIRE(n_nodes == 0 || (rowptr && (kRule || part) && g2l_out), TMA_ERR_INVALID_ARG,
                "%s: rowptr / part / g2l_out is NULL", fn);
    TMA_REQUIRE(cap_n_loc == 0 || l2g_out, TMA_ERR_INVALID_ARG, "%s: l2g_out is NULL", fn);
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    CountWorkspace w = carve(ws, n_nodes, cap_n_loc);
    TMA_REQUIRE(ws_bytes >= w.bytes, TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, ws_bytes,
                w.bytes);
    if (!sizes) sizes = w.sizes;

    const unsigned nb_nodes = unsigned(ceil_div(n_nodes > 0 ? n_nodes : 1, kScanTile));
    const unsigned nb_rows = unsigned(ceil_div(cap_n_loc > 0 ? cap_n_loc : 1, kScanTile));
    In fin;
    Member mem;
    if constexpr (kRule) {
        fin = RuleIn{seed, uint32_t(K), p};
        mem = RuleMember{seed, uint32_t(K), p};
    } else {
        fin = FlagIn{part, p};
        mem = BitMember{w.member};
    }
    FlagOut fout{g2l_out, l2g_out, cap_n_loc, rowptr, w.row_beg, w.row_len, reinterpret_cast<uint8_t *>(w.member)};
    // 1. rank local nodes.  Few tiles: the apply kernel adds up the tile sums itself; many: a scan kernel first.
    const bool inline_nodes = nb_nodes <= kInlineTiles, inline_rows = nb_rows <= kInlineTiles;
    {
        TMA_TIMED("scan_reduce_flags", s);
        hipLaunchKernelGGL(scan_reduce_kernel<In>, dim3(nb_nodes), dim3(kScanThreads), 0, s, nullptr, n_nodes,
                           fin, w.node_block_sums);
    }
    if (!inline_nodes) {
        TMA_TIMED("scan_sums", s);
        hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(1024), 0, s, int64_t(nb_nodes), w.node_block_sums,
                           sizes + 0, rowptr_loc_out);
    }
    {   // also clears the tile sums that the kept-degree pass adds to (nb_rows <= nb_nodes)
        TMA_TIMED("scan_apply_flags", s);
        hipLaunchKernelGGL((scan_apply_kernel<In, FlagOut>), dim3(nb_nodes), dim3(kScanThreads), 0, s, nullptr,
                           n_nodes, fin, fout, w.node_block_sums, inline_nodes ? sizes + 0 : nullptr,
                           inline_nodes ? rowptr_loc_out : nullptr, w.row_block_sums, int64_t(nb_rows));
    }
    // 2. kept degree per local row and per scan tile, then rowptr_loc by the second scan
    if (cap_n_loc > 0) {
        const unsigned row_blocks = unsigned(ceil_div(cap_n_loc, kRowsPerBlock));
        TMA_TIMED("row_count", s);
        hipLaunchKernelGGL(row_count_kernel<Member>, dim3(row_blocks), dim3(256), 0, s, sizes + 0, cap_n_loc, w.row_beg,
                           w.row_len, colidx, mem, w.deg, inline_rows ? w.row_block_sums : nullptr);
    }
    DegIn din{w.deg};
    DegOut dout{rowptr_loc_out};
    if (!inline_rows) {   // many tiles: their sums by a pass of its own (one atomic per workgroup would queue up)
        {
            TMA_TIMED("scan_reduce_deg", s);
            hipLaunchKernelGGL(scan_reduce_kernel<DegIn>, dim3(nb_rows), dim3(kScanThreads), 0, s, sizes + 0,
                               cap_n_loc, din, w.row_block_sums);
        }
        TMA_TIMED("scan_sums", s);
        hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(1024), 0, s, int64_t(nb_rows), w.row_block_sums,
                           sizes + 1, static_cast<int32_t *>(nullptr));
    }
    {
        TMA_TIMED("scan_apply_deg", s);
        hipLaunchKernelGGL((scan_apply_kernel<DegIn, DegOut>), dim3(nb_rows), dim3(kScanThreads), 0, s, sizes + 0,
                           cap_n_loc, din, dout, w.row_block_sums, inline_rows ? sizes + 1 : nullptr,
                           static_cast<int32_t *>(nullptr), static_cast<int64_t *>(nullptr), int64_t(0));
    }
    return check_launch(fn);
}

}  // namespace tma

extern "C" int tma_induced_subgraph_count(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                                          const int32_t *part, int32_t p, int32_t *g2l_out, int32_t *l2g_out,
                                          int32_t *rowptr_loc_out, int64_t cap_n_loc, int64_t *h_n_loc,
                                          int64_t *h_nnz_loc, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_induced_subgraph_count";
    TMA_REQUIRE(h_n_loc && h_nnz_loc, TMA_ERR_INVALID_ARG, "%s: h_n_loc / h_nnz_loc is NULL", fn);
    hipStream_t s = as_stream(stream);
    if (int rc = enqueue_count<false>(fn, n_nodes, rowptr, colidx, part, p, 0, 0, g2l_out, l2g_out, rowptr_loc_out,
                                      cap_n_loc, nullptr, ws, ws_bytes, s))
        return rc;
    const CountWorkspace w = carve(ws, n_nodes, cap_n_loc);

    int64_t h_sizes[2] = {0, 0};
    // copy in stream order and wait for it (one call: measurably shorter than an asynchronous copy
    // followed by a stream synchronisation)
    TMA_HIP_TRY(hipMemcpyWithStream(h_sizes, w.sizes, sizeof(h_sizes), hipMemcpyDeviceToHost, s), fn);
    *h_n_loc = h_sizes[0];
    *h_nnz_loc = h_sizes[1];
    TMA_REQUIRE(h_sizes[0] <= cap_n_loc, TMA_ERR_BAD_SHAPE,
                "%s: partition has %lld nodes but cap_n_loc is %lld (nnz reported covers the first cap rows only)",
                fn, (long long)h_sizes[0], (long long)cap_n_loc);
    TMA_REQUIRE(h_sizes[1] <= INT32_MAX, TMA_ERR_BAD_SHAPE, "%s: %lld kept entries do not fit int32 local indexing",
                fn, (long long)h_sizes[1]);
    return TMA_OK;
}

extern "C" int tma_induced_subgraph_fill(int64_t n_nodes, const int32_t *colidx, const int32_t *g2l, int64_t n_loc,
                                         const int32_t *rowptr_loc, int32_t *colidx_loc_out, float *inv_deg_out,
                                         int64_t cap_n_loc, const void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_induced_subgraph_fill";
    TMA_REQUIRE(n_nodes >= 0 && n_nodes <= INT32_MAX && n_loc >= 0 && n_loc <= cap_n_loc && cap_n_loc <= n_nodes,
                TMA_ERR_INVALID_ARG, "%s: need 0 <= n_loc <= cap_n_loc <= n_nodes < 2^31", fn);
    if (n_loc == 0) return TMA_OK;
    TMA_REQUIRE(ws && aligned(ws, 256), TMA_ERR_INVALID_ARG, "%s: workspace NULL or not 256-byte aligned", fn);
    const CountWorkspace w = carve(const_cast<void *>(ws), n_nodes, cap_n_loc);
    TMA_REQUIRE(ws_bytes >= w.bytes, TMA_ERR_WORKSPACE_TOO_SMALL, "%s: workspace %zu < %zu bytes", fn, ws_bytes,
                w.bytes);
    TMA_REQUIRE(g2l && rowptr_loc && inv_deg_out, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    // colidx / colidx_loc_out may be NULL only for a graph without entries; not knowable here without a
    // device read, so they are required whenever there are local rows.
    TMA_REQUIRE(colidx && colidx_loc_out, TMA_ERR_INVALID_ARG, "%s: colidx / colidx_loc_out is NULL", fn);
    const unsigned blocks = unsigned(ceil_div(n_loc, kRowsPerBlock));
    TMA_TIMED("row_fill", as_stream(stream));
    hipLaunchKernelGGL(row_fill_kernel<BitMember>, dim3(blocks), dim3(256), 0, as_stream(stream), n_loc,
                       static_cast<const int64_t *>(nullptr), int64_t(INT64_MAX), w.row_beg, w.row_len,
                       colidx, BitMember{w.member}, g2l, rowptr_loc, colidx_loc_out, inv_deg_out);
    return check_launch(fn);
}

extern "C" int tma_induced_subgraph(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx, const int32_t *part,
                                    int32_t p, int32_t *g2l_out, int32_t *l2g_out, int32_t *rowptr_loc_out,
                                    int32_t *colidx_loc_out, float *inv_deg_out, int64_t cap_n_loc,
                                    int64_t cap_nnz_loc, int64_t *h_n_loc, int64_t *h_nnz_loc, void *ws,
                                    size_t ws_bytes, tma_stream_t stream)
{
    using namespace tma;
    const char *fn = "tma_induced_subgraph";
    TMA_REQUIRE(cap_nnz_loc >= 0, TMA_ERR_INVALID_ARG, "%s: cap_nnz_loc < 0", fn);
    if (int rc = tma_induced_subgraph_count(n_nodes, rowptr, colidx, part, p, g2l_out, l2g_out, rowptr_loc_out,
                                            cap_n_loc, h_n_loc, h_nnz_loc, ws, ws_bytes, stream))
        return rc;
    TMA_REQUIRE(*h_nnz_loc <= cap_nnz_loc, TMA_ERR_BAD_SHAPE,
                "%s: the subgraph keeps %lld entries but cap_nnz_loc is %lld", fn, (long long)*h_nnz_loc,
                (long long)cap_nnz_loc);
    return tma_induced_subgraph_fill(n_nodes, colidx, g2l_out, *h_n_loc, rowptr_loc_out, colidx_loc_out, inv_deg_out,
                                     cap_n_loc, ws, ws_bytes, stream);
}

namespace tma {

template <bool kRule>
static int subgraph_async(const char *fn, int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                          const int32_t *part, int32_t p, int32_t K, uint64_t seed, int32_t *g2l_out, int32_t *l2g_out,
                          int32_t *rowptr_loc_out, int32_t *colidx_loc_out, float *inv_deg_out, int64_t cap_n_loc,
                          int64_t cap_nnz_loc, int64_t *d_sizes_out, void *ws, size_t ws_bytes, tma_stream_t stream)
{
    using Member = std::conditional_t<kRule, RuleMember, BitMember>;
    TMA_REQUIRE(cap_nnz_loc >= 0 && cap_nnz_loc <= INT32_MAX, TMA_ERR_INVALID_ARG, "%s: cap_nnz_loc outside [0, 2^31)", fn);
    TMA_REQUIRE(d_sizes_out, TMA_ERR_INVALID_ARG, "%s: d_sizes_out is NULL", fn);
    TMA_REQUIRE(cap_n_loc == 0 || (colidx && colidx_loc_out && inv_deg_out), TMA_ERR_INVALID_ARG,
                "%s: colidx / colidx_loc_out / inv_deg_out is NULL", fn);
    hipStream_t s = as_stream(stream);
    if (int rc = enqueue_count<kRule>(fn, n_nodes, rowptr, colidx, part, p, K, seed, g2l_out, l2g_out, rowptr_loc_out,
                                      cap_n_loc, d_sizes_out, ws, ws_bytes, s))
        return rc;
    if (cap_n_loc == 0) return TMA_OK;
    const CountWorkspace w = carve(ws, n_nodes, cap_n_loc);
    Member mem;
    if constexpr (kRule)
        mem = RuleMember{seed, uint32_t(K), p};
    else
        mem = BitMember{w.member};
    // the second pass over as many rows as the capacity allows; the kernel reads the actual count
    const unsigned blocks = unsigned(ceil_div(cap_n_loc, kRowsPerBlock));
    TMA_TIMED("row_fill", s);
    hipLaunchKernelGGL(row_fill_kernel<Member>, dim3(blocks), dim3(256), 0, s, cap_n_loc,
                       static_cast<const int64_t *>(d_sizes_out), cap_nnz_loc, w.row_beg, w.row_len, colidx, mem, g2l_out,
                       rowptr_loc_out, colidx_loc_out, inv_deg_out);
    return check_launch(fn);
}

}  // namespace tma

extern "C" int tma_induced_subgraph_async(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx,
                                          const int32_t *part, int32_t p, int32_t *g2l_out, int32_t *l2g_out,
                                          int32_t *rowptr_loc_out, int32_t *colidx_loc_out, float *inv_deg_out,
                                          int64_t cap_n_loc, int64_t cap_nnz_loc, int64_t *d_sizes_out, void *ws,
                                          size_t ws_bytes, tma_stream_t stream)
{
    return tma::subgraph_async<false>("tma_induced_subgraph_async", n_nodes, rowptr, colidx, part, p, 0, 0, g2l_out,
                                      l2g_out, rowptr_loc_out, colidx_loc_out, inv_deg_out, cap_n_loc, cap_nnz_loc,
                                      d_sizes_out, ws, ws_bytes, stream);
}

extern "C" int tma_random_subgraph_async(int64_t n_nodes, const int64_t *rowptr, const int32_t *colidx, int32_t K,
                                         uint64_t seed, int32_t p, int32_t *g2l_out, int32_t *l2g_out,
                                         int32_t *rowptr_loc_out, int32_t *colidx_loc_out, float *inv_deg_out,
                                         int64_t cap_n_loc, int64_t cap_nnz_loc, int64_t *d_sizes_out, void *ws,
                                         size_t ws_bytes, tma_stream_t stream)
{
    const char *fn = "tma_random_subgraph_async";
    TMA_REQUIRE(K >= 1 && K <= (1 << 30), TMA_ERR_INVALID_ARG, "%s: K outside [1, 2^30]", fn);
    TMA_REQUIRE(p >= 0 && p < K, TMA_ERR_INVALID_ARG, "%s: p outside [0, K)", fn);
    return tma::subgraph_async<true>(fn, n_nodes, rowptr, colidx, nullptr, p, K, seed, g2l_out, l2g_out, rowptr_loc_out,
                                     colidx_loc_out, inv_deg_out, cap_n_loc, cap_nnz_loc, d_sizes_out, ws, ws_bytes, stream);
}
