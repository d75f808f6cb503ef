// Host-callable launchers of the build-side kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace cagra {

// Exhaustive search: `scratch` holds block_rows x exact_search_pitch(N) floats.
int64_t exact_search_pitch(int64_t N);
hipError_t launch_exact_search(const float *X, int64_t N, int dim, int64_t ldX, int metric,
                               const float *Q, int64_t B, int64_t ldQ, int k, int exclude_self,
                               int64_t self_offset, uint32_t *ids, float *dists, float *scratch,
                               int64_t block_rows, hipStream_t stream);

// The same for query rows row_begin .. row_end only; with a gate (device) every kernel of it returns at
// once unless *gate != 0.
hipError_t launch_exact_search_gated(const float *X, int64_t N, int dim, int64_t ldX, int metric,
                                     const float *Q, int64_t row_end, int64_t ldQ, int64_t row_begin, int k,
                                     int exclude_self, int64_t self_offset, uint32_t *ids, float *dists,
                                     float *scratch, int64_t block_rows, const uint32_t *gate, hipStream_t stream);
// k smallest (value, column) of every row of a dense block D[rows, pitch]
void launch_row_select(const float *D, int64_t pitch, int64_t rows, int k, uint32_t *ids_out, float *best_d,
                       hipStream_t stream);

// Exhaustive search with an fp16 matrix-core filter in front of the exact arithmetic
// (exact_filter.hip); same results as launch_exact_search.  `extra` holds plan.bytes.
constexpr int kFilterCap = 4096;   // candidates kept per query row
struct FilterPlan {
    int dimP, t;
    int64_t block_rows, stride, n_sample, sample_pitch, n_blocks;
    size_t off_x16, off_nx, off_q16, off_nq, off_max, off_thr_ids, off_thr_d, off_count, off_buf, off_flags, bytes;
};
void launch_fill_u32(uint32_t *p, int64_t n, uint32_t value, hipStream_t stream);   // p[0..n) = value
FilterPlan plan_exact_filter(int64_t N, int dim, int64_t B, int k, bool share_queries);
hipError_t launch_exact_filter(const float *X, int64_t N, int dim, int64_t ldX, int metric, const float *Q,
                               int64_t B, int64_t ldQ, int k, int exclude_self, int64_t self_offset, uint32_t *ids,
                               float *dists, float *plain_scratch, int64_t plain_block_rows, void *extra,
                               const FilterPlan &plan, bool share_queries, uint32_t *blocks_redone /* device, may be null */,
                               hipStream_t stream);

struct OptimizeScratch {
    uint32_t *indeg;      // [N]
    uint32_t *cursor;     // [N]
    uint64_t *offset;     // [N]
    uint64_t *block_sum;  // [ceil(N / 1024)]
    uint64_t *bucket;     // [N * degree]
};

// Reversed graph of the first d entries of every row of g (rows ld entries apart, entries >= N
// skipped): rev[N, d] sources ordered by (rank, source), rev_len[N].  Scratch sized for degree d.
hipError_t launch_reverse(const uint32_t *g, int64_t N, int d, int64_t ld, uint32_t *rev, uint32_t *rev_len,
                          const OptimizeScratch &s, hipStream_t stream);

// knn_dist == nullptr: rank-based reordering; else the distances of the knn entries are the weights
hipError_t launch_optimize(const uint32_t *knn, const float *knn_dist, int64_t N, int d_init, int d, uint32_t *graph,
                           uint32_t *pruned, uint32_t *rev, uint32_t *rev_len,
                           const OptimizeScratch &s, hipStream_t stream);

// NN-descent in synchronous rounds (nn_descent.hip): rounds 0..rounds, sample s, results in
// ids_out / dists_out [N, k]; workspace of nn_descent_workspace_bytes(N, k, s).
size_t nn_descent_workspace_bytes(int64_t N, int k, int s);
int nn_descent_auto_rounds(int64_t N);
hipError_t launch_nn_descent(const float *X, int64_t N, int dim, int64_t ld, int metric, int k, int rounds,
                             int s, uint64_t seed, uint32_t *ids_out, float *dists_out, void *workspace,
                             hipStream_t stream);

}  // namespace cagra
