// Host-callable launchers of the build-side kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cagra {

// Exhaustive search: `scratch` holds block_rows x exact_search_pitch(N) floats.
int64_t exact_search_pitch(int64_t N);
hipError_t launch_exact_search(const float *X, int64_t N, int dim, int64_t ldX, int metric,
                               const float *Q, int64_t B, int64_t ldQ, int k, int exclude_self,
                               int64_t self_offset, uint32_t *ids, float *dists, float *scratch,
                               int64_t block_rows, hipStream_t stream);

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
