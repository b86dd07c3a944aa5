// Row gather  dst[i,:] = src[l2g[i],:]  -- how a trainer takes its part of the
// feature matrix and the label vector (Alg. 2, set-up line).  Pure data
// movement, HBM bound: row_bytes read + row_bytes written per local node.
#include "common.hpp"

namespace tma {

// W = copy word (uint4: 16 B, uint32_t: 4 B, uint8_t: 1 B).  Consecutive
// threads copy consecutive words of a row; a block walks several rows.
// d_n (may be NULL): the row count when it is only known on the device; n_loc is then the capacity of the launch.
template <typename W>
__global__ __launch_bounds__(256) void gather_rows_kernel(int64_t n_cap, const int32_t *__restrict__ d_n,
                                                          const int32_t *__restrict__ l2g,
                                                          const char *__restrict__ src, int64_t src_ld,
                                                          int32_t words_per_row, int32_t rows_per_block,
                                                          char *__restrict__ dst, int64_t dst_ld)
{
    // a block copies rows_per_block consecutive local rows; thread t starts at word t of that run of rows
    int64_t n_loc = n_cap;
    if (d_n && *d_n < n_loc) n_loc = *d_n;
    const int64_t row0 = int64_t(blockIdx.x) * rows_per_block;
    if (row0 >= n_loc) return;
    const int32_t block_words = rows_per_block * words_per_row;
    for (int32_t t = threadIdx.x; t < block_words; t += 256) {
        const int32_t r = t / words_per_row;
        const int32_t w = t - r * words_per_row;
        const int64_t i = row0 + r;
        if (i < n_loc) {
            const W *s = reinterpret_cast<const W *>(src + int64_t(l2g[i]) * src_ld) + w;
            W *d = reinterpret_cast<W *>(dst + i * dst_ld) + w;
            *d = *s;
        }
    }
}

template <typename W>
static int launch_gather(int64_t n_loc, const int32_t *d_n, const int32_t *l2g, const void *src, int64_t src_ld,
                         int64_t row_bytes, void *dst, int64_t dst_ld, hipStream_t s)
{
    const int64_t words = row_bytes / int64_t(sizeof(W));
    if (words > (1 << 24)) return fail(TMA_ERR_BAD_SHAPE, "tma_gather_rows: rows longer than 2^24 words");
    // about 2048 words (8 per thread) per block
    int64_t rows_per_block = 2048 / words;
    if (rows_per_block < 1) rows_per_block = 1;
    TMA_TIMED(sizeof(W) == 16 ? "gather_rows_w16" : (sizeof(W) == 4 ? "gather_rows_w4" : "gather_rows_w1"), s);
    hipLaunchKernelGGL(gather_rows_kernel<W>, dim3(unsigned(ceil_div(n_loc, rows_per_block))), dim3(256), 0, s, n_loc,
                       d_n, l2g, static_cast<const char *>(src), src_ld, int32_t(words), int32_t(rows_per_block),
                       static_cast<char *>(dst), dst_ld);
    return TMA_OK;
}

static int gather_rows(const char *fn, int64_t n_loc, const int32_t *d_n, const int32_t *l2g, const void *src,
                       int64_t src_ld_bytes, int64_t row_bytes, void *dst, int64_t dst_ld_bytes, tma_stream_t stream)
{
    TMA_REQUIRE(n_loc >= 0 && row_bytes >= 0, TMA_ERR_INVALID_ARG, "%s: negative size", fn);
    if (n_loc == 0 || row_bytes == 0) return TMA_OK;
    TMA_REQUIRE(l2g && src && dst, TMA_ERR_INVALID_ARG, "%s: NULL argument", fn);
    TMA_REQUIRE(src_ld_bytes >= row_bytes && dst_ld_bytes >= row_bytes, TMA_ERR_BAD_SHAPE, "%s: pitch < row_bytes", fn);
    hipStream_t s = as_stream(stream);
    auto mult = [&](int64_t a) {
        return row_bytes % a == 0 && src_ld_bytes % a == 0 && dst_ld_bytes % a == 0 && aligned(src, size_t(a)) &&
               aligned(dst, size_t(a));
    };
    int rc;
    if (mult(16)) rc = launch_gather<uint4>(n_loc, d_n, l2g, src, src_ld_bytes, row_bytes, dst, dst_ld_bytes, s);
    else if (mult(4)) rc = launch_gather<uint32_t>(n_loc, d_n, l2g, src, src_ld_bytes, row_bytes, dst, dst_ld_bytes, s);
    else rc = launch_gather<uint8_t>(n_loc, d_n, l2g, src, src_ld_bytes, row_bytes, dst, dst_ld_bytes, s);
    if (rc) return rc;
    return check_launch(fn);
}

}  // namespace tma

extern "C" int tma_gather_rows(int64_t n_loc, const int32_t *l2g, const void *src, int64_t src_ld_bytes,
                               int64_t row_bytes, void *dst, int64_t dst_ld_bytes, tma_stream_t stream)
{
    return tma::gather_rows("tma_gather_rows", n_loc, nullptr, l2g, src, src_ld_bytes, row_bytes, dst, dst_ld_bytes, stream);
}

extern "C" int tma_gather_rows_dev(int64_t cap_rows, const int32_t *d_n_rows, const int32_t *l2g, const void *src,
                                   int64_t src_ld_bytes, int64_t row_bytes, void *dst, int64_t dst_ld_bytes,
                                   tma_stream_t stream)
{
    const char *fn = "tma_gather_rows_dev";
    TMA_REQUIRE(d_n_rows, TMA_ERR_INVALID_ARG, "%s: d_n_rows is NULL", fn);
    return tma::gather_rows(fn, cap_rows, d_n_rows, l2g, src, src_ld_bytes, row_bytes, dst, dst_ld_bytes, stream);
}
