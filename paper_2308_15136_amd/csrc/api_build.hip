// C ABI: exhaustive search, graph optimisation and the whole build.  Host-side validation
// and workspace carving only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "../../include/cagra_hip.h"
#include "build_kernels.h"

namespace cagra {

static size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// Rows of the distance block computed per pass: as many as fit in about 8 GiB.
static int64_t exact_block_rows(int64_t N, int64_t B)
{
    const int64_t pitch = exact_search_pitch(N);
    int64_t rows = ((int64_t)8 << 30) / (pitch * 4);
    rows = std::max<int64_t>(128, rows / 128 * 128);
    return std::min<int64_t>(rows, std::max<int64_t>(B, 1));
}

struct Carver {
    unsigned char *p;
    size_t used = 0;
    explicit Carver(void *base) : p(static_cast<unsigned char *>(base)) {}
    template <typename T> T *take(size_t n)
    {
        T *r = p ? reinterpret_cast<T *>(p + used) : nullptr;
        used += up256(n * sizeof(T));
        return r;
    }
};

struct OptimizeCarve {
    OptimizeScratch s;
    uint32_t *pruned, *rev, *rev_len;
    size_t bytes;
};

static OptimizeCarve carve_optimize(void *base, int64_t N, int degree)
{
    Carver c(base);
    OptimizeCarve o;
    o.s.indeg = c.take<uint32_t>(N);
    o.s.cursor = c.take<uint32_t>(N);
    o.s.offset = c.take<uint64_t>(N);
    o.s.block_sum = c.take<uint64_t>((N + 1023) / 1024);
    o.s.bucket = c.take<uint64_t>((size_t)N * degree);
    o.pruned = c.take<uint32_t>((size_t)N * degree);
    o.rev = c.take<uint32_t>((size_t)N * degree);
    o.rev_len = c.take<uint32_t>(N);
    o.bytes = c.used;
    return o;
}

static int check_degrees(int64_t N, int32_t degree, int32_t init_degree)
{
    if (degree < 2 || (degree & 1) || degree > 256) return CAGRA_ERR_BAD_DEGREE;
    if (init_degree < degree || init_degree > 512 || init_degree >= N) return CAGRA_ERR_BAD_DEGREE;
    return CAGRA_OK;
}

// Rows are read in 16-byte pieces: a row is `dim` rounded up to a multiple of 4 floats wide, and the caller vouches that
// the floats beyond `dim` are zero (they add nothing to either distance, in any summation order).
static int32_t pad4(int32_t dim) { return (dim + 3) & ~3; }

static int check_matrix(const float *p, int64_t rows, int32_t dim, int64_t ld)
{
    if (rows < 0 || rows > 0x7FFFFFFFll || dim < 1 || dim > 0x7FFFFFFF - 4 || ld < pad4(dim) || (ld & 3)) return CAGRA_ERR_BAD_SHAPE;
    if (((uintptr_t)p & 15) != 0) return CAGRA_ERR_BAD_SHAPE;
    return CAGRA_OK;
}

}  // namespace cagra

using namespace cagra;

extern "C" {

size_t cagra_exact_search_workspace_bytes(int64_t N, int64_t B, int32_t k)
{
    if (N < 1 || B < 0 || k < 1) return 256;
    // the distance block, and the running distances of a block of rows
    return up256((size_t)exact_block_rows(N, B) * ((size_t)exact_search_pitch(N) + (size_t)k) * sizeof(float));
}

int cagra_exact_search(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                       const float *queries, int64_t B, int64_t ld_queries, int32_t k,
                       int32_t exclude_self, int64_t self_offset, uint32_t *ids_out, float *dists_out,
                       void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!dataset) return CAGRA_ERR_NULL_POINTER;
    if (B > 0 && (!queries || !ids_out)) return CAGRA_ERR_NULL_POINTER;
    if (N < 1) return CAGRA_ERR_BAD_SHAPE;
    int rc = check_matrix(dataset, N, dim, ld);
    if (rc == CAGRA_OK) rc = check_matrix(queries, B, dim, ld_queries);
    if (rc != CAGRA_OK) return rc;
    if (metric != CAGRA_L2 && metric != CAGRA_IP) return CAGRA_ERR_BAD_OPTION;
    if (k < 1 || k > 512 || k > N) return CAGRA_ERR_BAD_TOPK;
    if (exclude_self && (self_offset < 0 || self_offset + B > N)) return CAGRA_ERR_BAD_SHAPE;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 ||
        workspace_bytes < cagra_exact_search_workspace_bytes(N, B, k))
        return CAGRA_ERR_WORKSPACE;
    if (B == 0) return CAGRA_OK;
    dim = pad4(dim);
    hipError_t e = launch_exact_search(dataset, N, dim, ld, (int)metric, queries, B, ld_queries, k,
                                       exclude_self ? 1 : 0, self_offset, ids_out, dists_out,
                                       static_cast<float *>(workspace), exact_block_rows(N, B),
                                       static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

// The algorithm a request resolves to: 1 plain, 2 filtered; 0 for an unusable request.
// (the filtered algorithm keeps a query row in LDS beside its 32 KB sorting buffer: dim <= 8192)
static int resolve_exact_algo(int algo, int64_t N, int dim)
{
    constexpr int kMaxFilteredDim = 8192;
    if (algo == CAGRA_EXACT_AUTO)
        return N >= 131072 && dim <= kMaxFilteredDim ? CAGRA_EXACT_FILTERED : CAGRA_EXACT_PLAIN;
    if (algo == CAGRA_EXACT_PLAIN) return CAGRA_EXACT_PLAIN;
    if (algo == CAGRA_EXACT_FILTERED && N >= 4096 && dim <= kMaxFilteredDim) return CAGRA_EXACT_FILTERED;
    return 0;
}

size_t cagra_exact_search_ex_workspace_bytes(int64_t N, int32_t dim, int64_t B, int32_t k, cagra_exact_algo algo)
{
    const size_t plain = cagra_exact_search_workspace_bytes(N, B, k);
    if (N < 1 || B < 1 || k < 1 || dim < 1 || resolve_exact_algo((int)algo, N, dim) != CAGRA_EXACT_FILTERED) return plain;
    // sized for distinct queries; a call with queries == dataset needs less and accepts this too
    return plain + plan_exact_filter(N, dim, B, k, false).bytes;
}

int cagra_exact_search_ex(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                          const float *queries, int64_t B, int64_t ld_queries, int32_t k,
                          int32_t exclude_self, int64_t self_offset, cagra_exact_algo algo, uint32_t *ids_out,
                          float *dists_out, uint32_t *blocks_redone_out, void *workspace, size_t workspace_bytes,
                          void *hip_stream)
{
    if (N < 1) return CAGRA_ERR_BAD_SHAPE;
    const int resolved = resolve_exact_algo((int)algo, N, dim);
    if (resolved == 0) return CAGRA_ERR_BAD_OPTION;
    if (resolved == CAGRA_EXACT_PLAIN) {
        int rc = cagra_exact_search(dataset, N, dim, ld, metric, queries, B, ld_queries, k, exclude_self, self_offset,
                                    ids_out, dists_out, workspace, workspace_bytes, hip_stream);
        if (rc == CAGRA_OK && blocks_redone_out != nullptr) {
            launch_fill_u32(blocks_redone_out, 1, 0u, static_cast<hipStream_t>(hip_stream));
            if (hipGetLastError() != hipSuccess) rc = CAGRA_ERR_LAUNCH;
        }
        return rc;
    }
    if (!dataset) return CAGRA_ERR_NULL_POINTER;
    if (B > 0 && (!queries || !ids_out)) return CAGRA_ERR_NULL_POINTER;
    int rc = check_matrix(dataset, N, dim, ld);
    if (rc == CAGRA_OK) rc = check_matrix(queries, B, dim, ld_queries);
    if (rc != CAGRA_OK) return rc;
    if (metric != CAGRA_L2 && metric != CAGRA_IP) return CAGRA_ERR_BAD_OPTION;
    if (k < 1 || k > 512 || k > N) return CAGRA_ERR_BAD_TOPK;
    if (exclude_self && (self_offset < 0 || self_offset + B > N)) return CAGRA_ERR_BAD_SHAPE;
    if (B == 0) return CAGRA_OK;
    dim = pad4(dim);
    const bool share = queries == dataset && ld_queries == ld && B <= N;
    const size_t plain = cagra_exact_search_workspace_bytes(N, B, k);
    const FilterPlan pl = plan_exact_filter(N, dim, B, k, share);
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < plain + pl.bytes)
        return CAGRA_ERR_WORKSPACE;
    hipError_t e = launch_exact_filter(dataset, N, dim, ld, (int)metric, queries, B, ld_queries, k,
                                       exclude_self ? 1 : 0, self_offset, ids_out, dists_out,
                                       static_cast<float *>(workspace), exact_block_rows(N, B),
                                       static_cast<unsigned char *>(workspace) + plain, pl, share, blocks_redone_out,
                                       static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

size_t cagra_optimize_workspace_bytes(int64_t N, int32_t init_degree, int32_t degree)
{
    (void)init_degree;
    if (N < 1 || degree < 1) return 256;
    return carve_optimize(nullptr, N, degree).bytes;
}

int cagra_optimize(const uint32_t *knn, int64_t N, int32_t init_degree, int32_t degree,
                   uint32_t *graph_out, uint32_t *pruned_out, uint32_t *reversed_out,
                   uint32_t *reversed_len_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return cagra_optimize_ex(knn, nullptr, N, init_degree, degree, CAGRA_REORDER_RANK, graph_out, pruned_out,
                             reversed_out, reversed_len_out, workspace, workspace_bytes, hip_stream);
}

int cagra_optimize_ex(const uint32_t *knn, const float *knn_dists, int64_t N, int32_t init_degree, int32_t degree,
                      cagra_reorder reorder, uint32_t *graph_out, uint32_t *pruned_out, uint32_t *reversed_out,
                      uint32_t *reversed_len_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!knn || !graph_out) return CAGRA_ERR_NULL_POINTER;
    if (reorder != CAGRA_REORDER_RANK && reorder != CAGRA_REORDER_DISTANCE) return CAGRA_ERR_BAD_OPTION;
    if (reorder == CAGRA_REORDER_DISTANCE && !knn_dists) return CAGRA_ERR_NULL_POINTER;
    if (N < 2 || N > 0x7FFFFFFFll) return CAGRA_ERR_BAD_SHAPE;
    int rc = check_degrees(N, degree, init_degree);
    if (rc != CAGRA_OK) return rc;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 ||
        workspace_bytes < cagra_optimize_workspace_bytes(N, init_degree, degree))
        return CAGRA_ERR_WORKSPACE;
    OptimizeCarve c = carve_optimize(workspace, N, degree);
    hipError_t e = launch_optimize(knn, reorder == CAGRA_REORDER_DISTANCE ? knn_dists : nullptr, N, init_degree,
                                   degree, graph_out, pruned_out ? pruned_out : c.pruned,
                                   reversed_out ? reversed_out : c.rev,
                                   reversed_len_out ? reversed_len_out : c.rev_len, c.s,
                                   static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

size_t cagra_build_workspace_bytes(int64_t N, int32_t dim, int32_t degree, int32_t init_degree)
{
    return cagra_build_ex_workspace_bytes(N, dim, degree, init_degree, nullptr);
}

static int nnd_sample_of(const cagra_build_opts &o, int init_degree)
{
    return o.nnd_sample == 0 ? std::min(32, init_degree) : o.nnd_sample;
}

size_t cagra_build_ex_workspace_bytes(int64_t N, int32_t dim, int32_t degree, int32_t init_degree,
                                      const cagra_build_opts *opts)
{
    cagra_build_opts o = {};
    if (opts) o = *opts;
    if (init_degree == 0) init_degree = 2 * degree;
    if (N < 2 || degree < 1) return 256;
    // the k-NN graph; its distances for NN-descent (which produces them) or the distance-based reordering
    const bool dists = o.initial_graph == 1 || o.reorder == CAGRA_REORDER_DISTANCE;
    const size_t knn = up256((size_t)N * init_degree * sizeof(uint32_t)) * (dists ? 2 : 1);
    // the scratch of the first stage is dead once the k-NN graph exists, so the optimisation reuses its space
    const size_t first = o.initial_graph == 1
                             ? nn_descent_workspace_bytes(N, init_degree, nnd_sample_of(o, init_degree))
                             : cagra_exact_search_ex_workspace_bytes(N, dim, N, init_degree,
                                                                     (cagra_exact_algo)o.exact_algo);
    return knn + std::max(first, cagra_optimize_workspace_bytes(N, init_degree, degree));
}

int cagra_build(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                int32_t degree, int32_t init_degree, uint32_t *graph_out, void *workspace,
                size_t workspace_bytes, void *hip_stream)
{
    return cagra_build_ex(dataset, N, dim, ld, metric, degree, init_degree, nullptr, graph_out, workspace,
                          workspace_bytes, hip_stream);
}

int cagra_build_ex(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                   int32_t degree, int32_t init_degree, const cagra_build_opts *opts, uint32_t *graph_out,
                   void *workspace, size_t workspace_bytes, void *hip_stream)
{
    cagra_build_opts o = {};
    if (opts) o = *opts;
    if (init_degree == 0) init_degree = 2 * degree;
    if (o.reorder != CAGRA_REORDER_RANK && o.reorder != CAGRA_REORDER_DISTANCE) return CAGRA_ERR_BAD_OPTION;
    if (o.initial_graph != 0 && o.initial_graph != 1) return CAGRA_ERR_BAD_OPTION;
    if (o.initial_graph == 0 && resolve_exact_algo(o.exact_algo, N, dim) == 0) return CAGRA_ERR_BAD_OPTION;
    if (!dataset || !graph_out) return CAGRA_ERR_NULL_POINTER;
    if (N < 2) return CAGRA_ERR_BAD_SHAPE;
    int rc = check_matrix(dataset, N, dim, ld);
    if (rc != CAGRA_OK) return rc;
    if (metric != CAGRA_L2 && metric != CAGRA_IP) return CAGRA_ERR_BAD_OPTION;
    rc = check_degrees(N, degree, init_degree);
    if (rc != CAGRA_OK) return rc;
    const int sample = nnd_sample_of(o, init_degree);
    if (o.initial_graph == 1 && (sample < 1 || sample > 64 || sample > init_degree || o.nnd_rounds > 1000))
        return CAGRA_ERR_BAD_OPTION;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 ||
        workspace_bytes < cagra_build_ex_workspace_bytes(N, dim, degree, init_degree, &o))
        return CAGRA_ERR_WORKSPACE;
    dim = pad4(dim);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t knn_bytes = up256((size_t)N * init_degree * sizeof(uint32_t));
    uint32_t *knn = static_cast<uint32_t *>(workspace);
    unsigned char *rest = static_cast<unsigned char *>(workspace) + knn_bytes;
    float *knn_dists = nullptr;
    if (o.initial_graph == 1 || o.reorder == CAGRA_REORDER_DISTANCE) {
        knn_dists = reinterpret_cast<float *>(rest);
        rest += knn_bytes;
    }
    hipError_t e;
    if (o.initial_graph == 1) {
        const int rounds = o.nnd_rounds <= 0 ? nn_descent_auto_rounds(N) : o.nnd_rounds;
        e = launch_nn_descent(dataset, N, dim, ld, (int)metric, init_degree, rounds, sample, o.seed, knn, knn_dists,
                              rest, stream);
    } else if (resolve_exact_algo(o.exact_algo, N, dim) == CAGRA_EXACT_FILTERED) {
        const FilterPlan pl = plan_exact_filter(N, dim, N, init_degree, true);
        e = launch_exact_filter(dataset, N, dim, ld, (int)metric, dataset, N, ld, init_degree, 1, 0, knn, knn_dists,
                                reinterpret_cast<float *>(rest), exact_block_rows(N, N),
                                rest + cagra_exact_search_workspace_bytes(N, N, init_degree), pl, true, nullptr, stream);
    } else {
        e = launch_exact_search(dataset, N, dim, ld, (int)metric, dataset, N, ld, init_degree, 1, 0,
                                knn, knn_dists, reinterpret_cast<float *>(rest), exact_block_rows(N, N), stream);
    }
    if (e != hipSuccess) return CAGRA_ERR_LAUNCH;
    OptimizeCarve c = carve_optimize(rest, N, degree);
    e = launch_optimize(knn, o.reorder == CAGRA_REORDER_DISTANCE ? knn_dists : nullptr, N, init_degree, degree,
                        graph_out, c.pruned, c.rev, c.rev_len, c.s, stream);
    return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

}  // extern "C"
