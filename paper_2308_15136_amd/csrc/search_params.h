// Kernel argument block of the search kernels (host fills, device reads).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cagra {

struct SearchParams {
    const uint32_t *graph;
    const void *dataset;  // rows of fp32, fp16 or uint8, see the kernel's element type
    const float *queries;
    uint32_t *ids_out;
    float *dists_out;
    uint32_t *stats;      // optional [B, 4]
    uint32_t *counter;    // single mode: persistent-scheduling query counter (workspace)
    // multi mode (workspace): one visited table per query, every worker's final list, and a
    // per-query count of workers that have finished
    uint32_t *tables;     // [B, 2, 1 << hash_bits]: two tables per query, used in turn
    uint32_t *which;      // [B]: which of a query's two tables is in use (0 / 1)
    uint64_t *lists;      // [B, workers, 64 * MR]
    uint32_t *done;       // [B]
    uint32_t *notes;      // [B, workers, 8]: per worker its pass / parent / distance counts and flags
    int64_t N, B, ld, ld_queries;
    uint64_t seed;
    int32_t degree, dim, metric;      // dim: row width the kernels work on, a whole number of 16-byte pieces
    int32_t dim_query;                // elements a query really has (<= dim); the LDS copy is zero beyond them
    int32_t short_rows;               // fp32 rows up to 384 bytes, up to 64 or 129 to 256 candidates per pass: the kernels built for one more wavefront per SIMD
    int32_t k, itopk, search_width;   // multi mode: itopk is the per-worker list length, width is 1
    int32_t workers;                  // multi mode: workgroups per query
    int32_t max_iterations, reset_interval, team_log2;
    int32_t hash_bits;                // multi mode: log2 of each device-memory table
    int32_t table_words;              // single mode: entries of the LDS table (multiple of 64)
    // byte offsets into the dynamic LDS block
    int32_t off_query, off_newid, off_newdist, off_parents;
    // wave teams (several wavefronts per query): a few workgroup-wide words, the publication buffers
    // (2 buffers x waves x pub_cap keys, high words then low words) and their capacity per wavefront
    int32_t off_team, off_pub, pub_cap;
    int32_t workspace_clean;          // multi mode: the caller vouches for a clean workspace, no init launch
};

// One set of launchers per storage type of the dataset (fp32, fp16, uint8).
#define CAGRA_DECLARE_LAUNCHERS(T)                                                                  \
    hipError_t launch_search_single_##T(const SearchParams &P, int mr, int cr, int grid, size_t smem, \
                                        hipStream_t stream);                                        \
    hipError_t launch_search_multi_##T(const SearchParams &P, int mr, int cr, size_t smem, hipStream_t stream); \
    hipError_t launch_search_wide_##T(const SearchParams &P, int mr, int grid, size_t smem, hipStream_t stream); \
    hipError_t launch_search_team_##T(const SearchParams &P, int mr, int waves, int grid, int cus, size_t smem, hipStream_t stream);
CAGRA_DECLARE_LAUNCHERS(f32)
CAGRA_DECLARE_LAUNCHERS(f16)
CAGRA_DECLARE_LAUNCHERS(u8)
#undef CAGRA_DECLARE_LAUNCHERS

void launch_zero_counter(uint32_t *counter, hipStream_t stream);
void launch_multi_init(const SearchParams &P, hipStream_t stream);
hipError_t launch_convert(const float *src, int64_t rows, int dim, int64_t ld_src, int elem, void *dst,
                          int64_t ld_dst, hipStream_t stream);

}  // namespace cagra
