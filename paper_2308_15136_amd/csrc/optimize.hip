// CAGRA graph optimisation for gfx950 (Sec. III-B.2): detour count (Eq. 3) with ranks as edge
// weights (what CAGRA adopts; integer work only) or with the stored distances of the initial
// graph (the distance-based variant the paper compares with), reorder and prune, reversed
// graph, interleaved merge.
#include "device_util.h"
#include "build_kernels.h"

namespace cagra {

// ---- reorder + prune -------------------------------------------------------------------------
// One workgroup (256 threads) per node X.  The initial list of X sits in LDS together with a
// small open-addressing map id -> rank in that list.  For every Z = list[i] the list of Z is
// streamed once; an entry W at rank l of Z that is also entry j of X is a detourable route for
// the edge X -> W iff max(i, l) < j (rank-based), or iff both hops are shorter than the edge,
// max(dist(X, Z), dist(Z, W)) < dist(X, W), when the distance table knn_dist is given.

constexpr int kMaxInit = 512;
constexpr int kMapSize = 2048;   // >= 4 * kMaxInit

__global__ void __launch_bounds__(256)
prune_kernel(const uint32_t *__restrict__ knn, const float *__restrict__ knn_dist, int64_t N, int d_init, int d,
             uint32_t *__restrict__ pruned)
{
    __shared__ uint32_t xlist[kMaxInit];
    __shared__ float xdist[kMaxInit];
    __shared__ uint32_t cnt[kMaxInit];
    __shared__ uint32_t map_key[kMapSize];
    __shared__ uint16_t map_val[kMapSize];
    const int tid = threadIdx.x;
    const int64_t x = blockIdx.x;
    const uint32_t *lx = knn + x * d_init;

    for (int i = tid; i < kMapSize; i += 256) map_key[i] = kInvalidId;
    for (int i = tid; i < d_init; i += 256) {
        xlist[i] = lx[i];
        cnt[i] = 0;
        xdist[i] = knn_dist ? knn_dist[x * d_init + i] : 0.f;
    }
    __syncthreads();
    for (int j = tid; j < d_init; j += 256) {
        uint32_t id = xlist[j];
        uint32_t s = (id * 2654435761u) >> 21;          // 11 bits
        for (;;) {
            uint32_t old = atomicCAS(&map_key[s], kInvalidId, id);
            if (old == kInvalidId || old == id) { map_val[s] = (uint16_t)j; break; }
            s = (s + 1) & (kMapSize - 1);
        }
    }
    __syncthreads();

    const int wave = tid >> 6, lane = tid & 63;
    for (int i = wave; i < d_init; i += 4) {
        const uint32_t *lz = knn + (int64_t)xlist[i] * d_init;
        const float *dz = knn_dist ? knn_dist + (int64_t)xlist[i] * d_init : nullptr;
        for (int l = lane; l < d_init; l += 64) {
            const uint32_t w = lz[l];
            uint32_t s = (w * 2654435761u) >> 21;
            for (;;) {
                const uint32_t key = map_key[s];
                if (key == kInvalidId) break;
                if (key == w) {
                    const int j = map_val[s];
                    const bool detour = dz ? (xdist[i] < xdist[j] && dz[l] < xdist[j]) : (j > i && j > l);
                    if (detour) atomicAdd(&cnt[j], 1u);
                    break;
                }
                s = (s + 1) & (kMapSize - 1);
            }
        }
    }
    __syncthreads();

    // new position of entry j = number of entries with a smaller (count, rank) key
    for (int j = tid; j < d_init; j += 256) {
        const uint32_t cj = cnt[j];
        int pos = 0;
        for (int o = 0; o < d_init; ++o) {
            const uint32_t co = cnt[o];
            pos += (co < cj) || (co == cj && o < j);
        }
        if (pos < d) pruned[x * d + pos] = xlist[j];
    }
}

// ---- reversed graph --------------------------------------------------------------------------
// Edges X -> Y at rank r are bucketed per target Y (count, scan, fill); each bucket keeps its d
// smallest (r, X) keys in order.

__global__ void fill_u32_kernel(uint32_t *p, int64_t n, uint32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// The graph whose edges are reversed is the first d entries of rows that are ld entries apart;
// entries that are not node ids (unused slots) are skipped.
__global__ void indegree_kernel(const uint32_t *__restrict__ g, int64_t N, int d, int64_t ld, uint32_t *indeg)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N * d) return;
    const int64_t x = e / d;
    const uint32_t y = g[x * ld + (e - x * d)];
    if ((int64_t)y < N) atomicAdd(&indeg[y], 1u);
}

// Exclusive scan of uint32 counts into uint64 offsets, three passes over blocks of 1024.
__global__ void __launch_bounds__(256)
scan_block_kernel(const uint32_t *__restrict__ in, int64_t n, uint64_t *__restrict__ out, uint64_t *__restrict__ block_sum)
{
    __shared__ uint64_t part[256];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * 1024 + tid * 4;
    uint64_t v[4], s = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) { v[u] = base + u < n ? in[base + u] : 0; s += v[u]; }
    part[tid] = s;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        uint64_t t = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += t;
        __syncthreads();
    }
    uint64_t run = part[tid] - s;
#pragma unroll
    for (int u = 0; u < 4; ++u) { if (base + u < n) out[base + u] = run; run += v[u]; }
    if (tid == 255) block_sum[blockIdx.x] = part[255];
}

__global__ void __launch_bounds__(256)
scan_sums_kernel(uint64_t *block_sum, int64_t n_blocks)
{
    __shared__ uint64_t part[256];
    __shared__ uint64_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < n_blocks; base += 256) {
        const int64_t i = base + tid;
        const uint64_t v = i < n_blocks ? block_sum[i] : 0;
        part[tid] = v;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            uint64_t t = tid >= off ? part[tid - off] : 0;
            __syncthreads();
            part[tid] += t;
            __syncthreads();
        }
        if (i < n_blocks) block_sum[i] = carry + part[tid] - v;
        __syncthreads();
        if (tid == 255) carry += part[255];
        __syncthreads();
    }
}

__global__ void scan_add_kernel(uint64_t *out, int64_t n, const uint64_t *__restrict__ block_sum)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] += block_sum[i >> 10];
}

__global__ void bucket_fill_kernel(const uint32_t *__restrict__ g, int64_t N, int d, int64_t ld,
                                   const uint64_t *__restrict__ offset, uint32_t *cursor,
                                   uint64_t *__restrict__ bucket)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N * d) return;
    const uint32_t x = (uint32_t)(e / d), r = (uint32_t)(e - (int64_t)x * d);
    const uint32_t y = g[(int64_t)x * ld + r];
    if ((int64_t)y >= N) return;
    const uint32_t pos = atomicAdd(&cursor[y], 1u);
    bucket[offset[y] + pos] = ((uint64_t)r << 32) | x;
}

// One wavefront per target node: the d smallest keys of its bucket, ascending.
constexpr int kRevPool = 1024;   // >= max degree (256) + 512

__global__ void __launch_bounds__(64)
reverse_select_kernel(const uint64_t *__restrict__ bucket, const uint64_t *__restrict__ offset,
                      const uint32_t *__restrict__ indeg, int64_t N, int d,
                      uint32_t *__restrict__ rev, uint32_t *__restrict__ rev_len)
{
    __shared__ uint64_t pool[kRevPool];
    __shared__ int count;
    const int lane = threadIdx.x;
    const int64_t y = blockIdx.x;
    const uint64_t *src = bucket + offset[y];
    const int64_t n_in = indeg[y];
    if (lane == 0) count = 0;
    uint64_t tau = ~0ull;
    __syncthreads();
    auto sort_pool = [&]() {
        for (int k = 2; k <= kRevPool; k <<= 1)
            for (int j = k >> 1; j >= 1; j >>= 1) {
                __syncthreads();
                for (int i = lane; i < kRevPool / 2; i += 64) {
                    int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                    int hi = lo | j;
                    uint64_t a = pool[lo], b = pool[hi];
                    bool asc = (lo & k) == 0;
                    if ((a > b) == asc) { pool[lo] = b; pool[hi] = a; }
                }
            }
        __syncthreads();
    };
    for (int64_t base = 0; base < n_in; base += 512) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t i = base + u * 64 + lane;
            if (i < n_in) {
                const uint64_t key = src[i];
                if (key < tau) pool[atomicAdd(&count, 1)] = key;
            }
        }
        __syncthreads();
        const int n = count;
        __syncthreads();   // everyone has read the count before the next round appends to it
        if (n > kRevPool - 512 && base + 512 < n_in) {
            for (int i = n + lane; i < kRevPool; i += 64) pool[i] = ~0ull;
            sort_pool();
            if (lane == 0) count = n < d ? n : d;
            if (n >= d) tau = pool[d - 1];
            __syncthreads();
        }
    }
    const int n = count;
    for (int i = n + lane; i < kRevPool; i += 64) pool[i] = ~0ull;
    sort_pool();
    const int keep = n < d ? n : d;
    for (int i = lane; i < d; i += 64) rev[y * d + i] = i < keep ? (uint32_t)pool[i] : kInvalidId;
    if (lane == 0) rev_len[y] = (uint32_t)keep;
}

// ---- merge -----------------------------------------------------------------------------------
// Even slots from the pruned list, odd slots from the reversed list while it lasts (at most
// d/2), duplicates skipped on both sides.  One thread per node; the row being written is the
// "taken" set.
__global__ void merge_kernel(const uint32_t *__restrict__ pruned, const uint32_t *__restrict__ rev,
                             const uint32_t *__restrict__ rev_len, int64_t N, int d,
                             uint32_t *__restrict__ graph)
{
    const int64_t y = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (y >= N) return;
    const uint32_t *p = pruned + y * d, *r = rev + y * d;
    uint32_t *out = graph + y * d;
    const int nr = (int)rev_len[y];
    int ip = 0, ir = 0, nrev = 0;
    for (int slot = 0; slot < d; ++slot) {
        bool done = false;
        if ((slot & 1) && nrev < d / 2) {
            for (; ir < nr; ++ir) {
                const uint32_t c = r[ir];
                bool dup = false;
                for (int t = 0; t < slot; ++t) dup |= (out[t] == c);
                if (!dup) break;
            }
            if (ir < nr) { out[slot] = r[ir++]; ++nrev; done = true; }
        }
        if (!done) {
            for (;; ++ip) {
                const uint32_t c = p[ip];
                bool dup = false;
                for (int t = 0; t < slot; ++t) dup |= (out[t] == c);
                if (!dup) break;
            }
            out[slot] = p[ip++];
        }
    }
}

static unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// Reversed graph of the first d entries of every row of g (rows ld apart): rev[N, d], rev_len[N].
hipError_t launch_reverse(const uint32_t *g, int64_t N, int d, int64_t ld, uint32_t *rev, uint32_t *rev_len,
                          const OptimizeScratch &s, hipStream_t stream)
{
    const int64_t n_edges = N * d;
    const int64_t n_blocks = (N + 1023) / 1024;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(N, 256)), dim3(256), 0, stream, s.indeg, N, 0u);
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(N, 256)), dim3(256), 0, stream, s.cursor, N, 0u);
    hipLaunchKernelGGL(indegree_kernel, dim3(blocks_for(n_edges, 256)), dim3(256), 0, stream, g, N, d, ld, s.indeg);
    hipLaunchKernelGGL(scan_block_kernel, dim3((unsigned)n_blocks), dim3(256), 0, stream, s.indeg, N, s.offset, s.block_sum);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(256), 0, stream, s.block_sum, n_blocks);
    hipLaunchKernelGGL(scan_add_kernel, dim3(blocks_for(N, 256)), dim3(256), 0, stream, s.offset, N, s.block_sum);
    hipLaunchKernelGGL(bucket_fill_kernel, dim3(blocks_for(n_edges, 256)), dim3(256), 0, stream, g, N, d, ld, s.offset, s.cursor, s.bucket);
    hipLaunchKernelGGL(reverse_select_kernel, dim3((unsigned)N), dim3(64), 0, stream, s.bucket, s.offset, s.indeg, N, d, rev, rev_len);
    return hipGetLastError();
}

hipError_t launch_optimize(const uint32_t *knn, const float *knn_dist, int64_t N, int d_init, int d, uint32_t *graph,
                           uint32_t *pruned, uint32_t *rev, uint32_t *rev_len,
                           const OptimizeScratch &s, hipStream_t stream)
{
    hipLaunchKernelGGL(prune_kernel, dim3((unsigned)N), dim3(256), 0, stream, knn, knn_dist, N, d_init, d, pruned);
    hipError_t e = launch_reverse(pruned, N, d, d, rev, rev_len, s, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(merge_kernel, dim3(blocks_for(N, 128)), dim3(128), 0, stream, pruned, rev, rev_len, N, d, graph);
    return hipGetLastError();
}

}  // namespace cagra
