// Kernel argument blocks of the search kernels (host fills, device reads).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cagra {

struct SingleParams {
    const uint32_t *graph;
    const float *dataset;
    const float *queries;
    uint32_t *ids_out;
    float *dists_out;
    uint32_t *stats;      // optional [B, 4]
    uint32_t *counter;    // persistent-scheduling query counter (workspace)
    int64_t N, B, ld, ld_queries;
    uint64_t seed;
    int32_t degree, dim, metric;
    int32_t k, itopk, search_width;
    int32_t max_iterations, reset_interval, hash_bits, team_log2;
    // byte offsets into the dynamic LDS block
    int32_t off_query, off_newid, off_newdist, off_parents;
};

hipError_t launch_search_single(const SingleParams &P, int mr, int cr, int grid, size_t smem,
                                hipStream_t stream);

}  // namespace cagra
