// Reachability measures of a fixed out-degree graph (Sec. III-A): the 2-hop node count of every
// node on the GPU, the numbers of strongly and weakly connected components on the host (a
// sequential graph traversal; it works on a host copy of the graph).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <new>
#include <vector>

#include "../../include/cagra_hip.h"
#include "device_util.h"

namespace cagra {

constexpr int kTwoHopMaxDegree = 64;
constexpr int kTwoHopSlots = 8192;   // >= 1.9 x (64 + 64 * 64) ids

// One wavefront per node X: X's neighbours and their neighbours go into an LDS set; the count
// is the number of distinct ids other than X.
__global__ void __launch_bounds__(kWave)
two_hop_kernel(const uint32_t *__restrict__ graph, int64_t N, int degree, uint32_t *__restrict__ counts)
{
    __shared__ uint32_t slots[kTwoHopSlots];
    const int lane = lane_id();
    for (int64_t x = blockIdx.x; x < N; x += gridDim.x) {
        for (int i = lane; i < kTwoHopSlots; i += kWave) slots[i] = kInvalidId;
        __syncthreads();
        uint32_t fresh = 0;
        const uint32_t mine = lane < degree ? graph[x * degree + lane] : kInvalidId;   // degree <= 64
        for (int step = -1; step < degree; ++step) {
            // step -1: the neighbours themselves; step i: the row of neighbour i
            uint32_t id = mine;
            if (step >= 0) {
                const uint32_t y = __builtin_amdgcn_readlane(mine, step);
                id = (lane < degree && (int64_t)y < N) ? graph[(int64_t)y * degree + lane] : kInvalidId;
            }
            if ((int64_t)id < N && id != (uint32_t)x) {
                uint32_t s = (id * 2654435761u) >> 19;   // 13 bits
                for (;;) {
                    const uint32_t old = atomicCAS(&slots[s], kInvalidId, id);
                    if (old == kInvalidId) { ++fresh; break; }
                    if (old == id) break;
                    s = (s + 1) & (kTwoHopSlots - 1);
                }
            }
        }
        // sum over the wavefront
        for (int off = 32; off >= 1; off >>= 1) fresh += (uint32_t)__shfl_xor((int)fresh, off, kWave);
        if (lane == 0) counts[x] = fresh;
        __syncthreads();
    }
}

// Strongly connected components by the path-based algorithm (two stacks: the nodes of the
// current search path that may still join an earlier component, and the boundaries between
// candidate components), with the recursion kept in an explicit frame stack.
static int64_t count_strong(const uint32_t *g, int64_t N, int d)
{
    const uint32_t none = 0xFFFFFFFFu;
    std::vector<uint32_t> order(N, none);      // preorder number, none = not reached yet
    std::vector<uint8_t> assigned(N, 0);       // already part of a finished component
    std::vector<uint32_t> open_nodes, boundaries, frame_node;
    std::vector<int32_t> frame_edge;
    uint32_t clock = 0;
    int64_t components = 0;
    for (int64_t root = 0; root < N; ++root) {
        if (order[root] != none) continue;
        frame_node.push_back((uint32_t)root);
        frame_edge.push_back(0);
        order[root] = clock++;
        open_nodes.push_back((uint32_t)root);
        boundaries.push_back((uint32_t)root);
        while (!frame_node.empty()) {
            const uint32_t v = frame_node.back();
            int32_t &e = frame_edge.back();
            if (e < d) {
                const uint32_t w = g[(size_t)v * d + e];
                ++e;
                if (order[w] == none) {
                    order[w] = clock++;
                    open_nodes.push_back(w);
                    boundaries.push_back(w);
                    frame_node.push_back(w);
                    frame_edge.push_back(0);
                } else if (!assigned[w]) {
                    // w is on the current path: everything reached after it collapses into its component
                    while (order[boundaries.back()] > order[w]) boundaries.pop_back();
                }
            } else {
                if (boundaries.back() == v) {
                    boundaries.pop_back();
                    uint32_t w;
                    do {
                        w = open_nodes.back();
                        open_nodes.pop_back();
                        assigned[w] = 1;
                    } while (w != v);
                    ++components;
                }
                frame_node.pop_back();
                frame_edge.pop_back();
            }
        }
    }
    return components;
}

// Weakly connected components: breadth-first labelling over the edges taken in both directions
// (the reversed adjacency is built first as offsets + sources).
static int64_t count_weak(const uint32_t *g, int64_t N, int d)
{
    std::vector<uint64_t> start(N + 1, 0);
    for (int64_t e = 0; e < N * d; ++e) ++start[g[e] + 1];
    for (int64_t v = 0; v < N; ++v) start[v + 1] += start[v];
    std::vector<uint32_t> source(N * (size_t)d);
    std::vector<uint64_t> fill(start.begin(), start.end() - 1);
    for (int64_t v = 0; v < N; ++v)
        for (int i = 0; i < d; ++i) source[fill[g[(size_t)v * d + i]]++] = (uint32_t)v;
    std::vector<uint8_t> seen(N, 0);
    std::vector<uint32_t> queue;
    int64_t components = 0;
    for (int64_t root = 0; root < N; ++root) {
        if (seen[root]) continue;
        ++components;
        seen[root] = 1;
        queue.assign(1, (uint32_t)root);
        while (!queue.empty()) {
            const uint32_t v = queue.back();
            queue.pop_back();
            for (int i = 0; i < d; ++i) {
                const uint32_t w = g[(size_t)v * d + i];
                if (!seen[w]) { seen[w] = 1; queue.push_back(w); }
            }
            for (uint64_t t = start[v]; t < start[v + 1]; ++t) {
                const uint32_t w = source[t];
                if (!seen[w]) { seen[w] = 1; queue.push_back(w); }
            }
        }
    }
    return components;
}

}  // namespace cagra

using namespace cagra;

extern "C" {

int cagra_two_hop_counts(const uint32_t *graph, int64_t N, int32_t degree, uint32_t *counts_out, void *hip_stream)
{
    if (!graph || !counts_out) return CAGRA_ERR_NULL_POINTER;
    if (N < 1 || N > 0x7FFFFFFFll) return CAGRA_ERR_BAD_SHAPE;
    if (degree < 1 || degree > kTwoHopMaxDegree) return CAGRA_ERR_BAD_DEGREE;
    const unsigned grid = (unsigned)(N < 65536 ? N : 65536);
    hipLaunchKernelGGL(two_hop_kernel, dim3(grid), dim3(kWave), 0, static_cast<hipStream_t>(hip_stream), graph, N,
                       (int)degree, counts_out);
    return hipGetLastError() == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

int cagra_count_components(const uint32_t *graph_host, int64_t N, int32_t degree, int64_t *strong_out,
                           int64_t *weak_out)
{
    if (!graph_host || (!strong_out && !weak_out)) return CAGRA_ERR_NULL_POINTER;
    if (N < 1 || N > 0x7FFFFFFFll) return CAGRA_ERR_BAD_SHAPE;
    if (degree < 1) return CAGRA_ERR_BAD_DEGREE;
    for (int64_t e = 0; e < N * degree; ++e)
        if (graph_host[e] >= (uint64_t)N) return CAGRA_ERR_BAD_SHAPE;
    try {
        if (strong_out) *strong_out = count_strong(graph_host, N, degree);
        if (weak_out) *weak_out = count_weak(graph_host, N, degree);
    } catch (const std::bad_alloc &) {
        return CAGRA_ERR_WORKSPACE;
    }
    return CAGRA_OK;
}

}  // extern "C"
