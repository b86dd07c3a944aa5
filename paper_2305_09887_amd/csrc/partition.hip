// Random node / super-node assignment (paper Sec. 3.2.2): one 64-bit
// counter hash per node, no state, no communication.  HBM-write bound:
// 4 B written per node (+4 B read of the cluster id for SuperTMA).
#include "common.hpp"

namespace tma {

// Four consecutive nodes per thread so that the store is one 16-byte write.
__global__ __launch_bounds__(256) void partition_kernel(int64_t n_nodes,
                                                        const int32_t *__restrict__ cluster,
                                                        uint32_t K, uint64_t seed,
                                                        int32_t *__restrict__ part)
{
    const int64_t stride = int64_t(gridDim.x) * blockDim.x * 4;
    for (int64_t v0 = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x) * 4; v0 < n_nodes; v0 += stride) {
        int32_t out[4];
        if (v0 + 4 <= n_nodes) {
            int4 c = make_int4(0, 0, 0, 0);
            if (cluster) c = *reinterpret_cast<const int4 *>(cluster + v0);
            const int32_t cl[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint64_t unit = cluster ? uint64_t(uint32_t(cl[j])) : uint64_t(v0 + j);
                out[j] = int32_t(__umul64hi(splitmix64_at(seed, unit), uint64_t(K)));
            }
            *reinterpret_cast<int4 *>(part + v0) = make_int4(out[0], out[1], out[2], out[3]);
        } else {
            for (int64_t v = v0; v < n_nodes; ++v) {
                uint64_t unit = cluster ? uint64_t(uint32_t(cluster[v])) : uint64_t(v);
                part[v] = int32_t(__umul64hi(splitmix64_at(seed, unit), uint64_t(K)));
            }
        }
    }
}

}  // namespace tma

extern "C" int tma_partition(int64_t n_nodes, const int32_t *cluster, int64_t n_clusters, int32_t K,
                             uint64_t seed, int32_t *part_out, tma_stream_t stream)
{
    using namespace tma;
    TMA_REQUIRE(n_nodes >= 0, TMA_ERR_INVALID_ARG, "tma_partition: n_nodes < 0");
    TMA_REQUIRE(K >= 1 && K <= (1 << 30), TMA_ERR_INVALID_ARG, "tma_partition: K=%d outside [1, 2^30]", K);
    TMA_REQUIRE(cluster == nullptr || n_clusters >= 1, TMA_ERR_INVALID_ARG,
                "tma_partition: cluster given but n_clusters < 1");
    if (n_nodes == 0) return TMA_OK;
    TMA_REQUIRE(part_out != nullptr, TMA_ERR_INVALID_ARG, "tma_partition: part_out is NULL");
    TMA_REQUIRE(aligned(part_out, 16) && (cluster == nullptr || aligned(cluster, 16)), TMA_ERR_INVALID_ARG,
                "tma_partition: part_out/cluster must be 16-byte aligned");
    int64_t blocks = ceil_div(n_nodes, 256 * 4);
    if (blocks > 256 * 32) blocks = 256 * 32;
    TMA_TIMED("partition", as_stream(stream));
    hipLaunchKernelGGL(partition_kernel, dim3(unsigned(blocks)), dim3(256), 0, as_stream(stream), n_nodes,
                       cluster, uint32_t(K), seed, part_out);
    return check_launch("tma_partition");
}
