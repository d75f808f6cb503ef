// Exhaustive k-nearest-neighbour search (Eq. 1) for gfx950: also the exact initial
// k-NN graph of Sec. III-B.1 (with the node itself left out).
//
// Two kernels per block of query rows and slice of dataset rows (at most kMaxCols of them, so
// that a block of thousands of query rows fits the scratch space also for very large N; the k
// best of a row are carried from slice to slice):
//   dist_tile_kernel   all distances of a block of rows to every dataset row of the slice,
//                      written to a row-major scratch block.  Each output is accumulated one
//                      dimension after the other with one fused multiply-add per
//                      dimension, so its bits do not depend on the tiling and equal
//                      those of a plain sequential loop.
//   row_select_kernel  per row, the k smallest (distance, id) keys in order: a
//                      streaming threshold filter into an LDS pool that is sorted
//                      (bitonic) whenever it fills.
#include "device_util.h"
#include "build_kernels.h"

namespace cagra {

constexpr int kTile = 128;     // output tile edge
constexpr int kKC = 16;        // dimensions staged per step
constexpr int kPad = 4;

__global__ void __launch_bounds__(256)
dist_tile_kernel(const float *__restrict__ A, int64_t rowsA, int64_t ldA, int64_t row0,
                 const float *__restrict__ X, int64_t N, int64_t ldX, int dim, int metric,
                 int exclude_self, int64_t self_offset, float *__restrict__ D, int64_t pitch,
                 const uint32_t *gate)
{
    if (gate != nullptr && *gate == 0u) return;   // a launch that is only needed when the flag is up
    __shared__ float As[kKC][kTile + kPad];
    __shared__ float Xs[kKC][kTile + kPad];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t tile_r = (int64_t)blockIdx.y * kTile;   // local row of the block
    const int64_t tile_c = (int64_t)blockIdx.x * kTile;

    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;

    // each thread stages 8 consecutive dimensions of one row of each operand
    const int lrow = tid >> 1, lk = (tid & 1) * 8;
    const int64_t arow = row0 + tile_r + lrow, xrow = tile_c + lrow;
    const bool a_ok = arow < rowsA, x_ok = xrow < N;
    const float *ap = A + (a_ok ? arow : 0) * ldA;
    const float *xp = X + (x_ok ? xrow : 0) * ldX;

    for (int k0 = 0; k0 < dim; k0 += kKC) {
        float4 a0 = make_float4(0, 0, 0, 0), a1 = a0, x0 = a0, x1 = a0;
        const int ka = k0 + lk;
        if (a_ok && ka < dim) a0 = *reinterpret_cast<const float4 *>(ap + ka);
        if (a_ok && ka + 4 < dim) a1 = *reinterpret_cast<const float4 *>(ap + ka + 4);
        if (x_ok && ka < dim) x0 = *reinterpret_cast<const float4 *>(xp + ka);
        if (x_ok && ka + 4 < dim) x1 = *reinterpret_cast<const float4 *>(xp + ka + 4);
        __syncthreads();
        As[lk + 0][lrow] = a0.x; As[lk + 1][lrow] = a0.y; As[lk + 2][lrow] = a0.z; As[lk + 3][lrow] = a0.w;
        As[lk + 4][lrow] = a1.x; As[lk + 5][lrow] = a1.y; As[lk + 6][lrow] = a1.z; As[lk + 7][lrow] = a1.w;
        Xs[lk + 0][lrow] = x0.x; Xs[lk + 1][lrow] = x0.y; Xs[lk + 2][lrow] = x0.z; Xs[lk + 3][lrow] = x0.w;
        Xs[lk + 4][lrow] = x1.x; Xs[lk + 5][lrow] = x1.y; Xs[lk + 6][lrow] = x1.z; Xs[lk + 7][lrow] = x1.w;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kKC; ++kk) {
            float a[8], x[8];
            const float4 av0 = *reinterpret_cast<const float4 *>(&As[kk][ty * 8]);
            const float4 av1 = *reinterpret_cast<const float4 *>(&As[kk][ty * 8 + 4]);
            const float4 xv0 = *reinterpret_cast<const float4 *>(&Xs[kk][tx * 8]);
            const float4 xv1 = *reinterpret_cast<const float4 *>(&Xs[kk][tx * 8 + 4]);
            a[0] = av0.x; a[1] = av0.y; a[2] = av0.z; a[3] = av0.w; a[4] = av1.x; a[5] = av1.y; a[6] = av1.z; a[7] = av1.w;
            x[0] = xv0.x; x[1] = xv0.y; x[2] = xv0.z; x[3] = xv0.w; x[4] = xv1.x; x[5] = xv1.y; x[6] = xv1.z; x[7] = xv1.w;
            if (metric == 0) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        float t = a[i] - x[j];
                        acc[i][j] = fmaf(t, t, acc[i][j]);
                    }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(a[i], x[j], acc[i][j]);
            }
        }
    }

    const float inf = __uint_as_float(0x7F800000u);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int64_t lr = tile_r + ty * 8 + i;          // row within the scratch block
        const int64_t grow = row0 + lr;
        if (grow >= rowsA) continue;
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t col = tile_c + tx * 8 + j;
            float d = metric == 0 ? acc[i][j] : 0.0f - acc[i][j];
            if (col >= N || (exclude_self && col == self_offset + grow)) d = inf;
            o[j] = d;
        }
        float *dst = D + lr * pitch + tile_c + tx * 8;
        *reinterpret_cast<float4 *>(dst) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(o[4], o[5], o[6], o[7]);
    }
}

// ---- k smallest keys of a stream, one workgroup of 256 threads per stream -----------------

constexpr int kPool = 2048;
constexpr uint64_t kKeyInf = ((uint64_t)0xFF800000u) << 32;   // ordered(+inf), id 0: nothing finite reaches it

// Ascending bitonic sort of pool[0..kPool) by 256 threads.
__device__ void pool_sort(uint64_t *pool, int tid)
{
    for (int k = 2; k <= kPool; k <<= 1)
        for (int j = k >> 1; j >= 1; j >>= 1) {
            __syncthreads();
            for (int i = tid; i < kPool / 2; i += 256) {
                int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                int hi = lo | j;
                uint64_t a = pool[lo], b = pool[hi];
                bool asc = (lo & k) == 0;
                if ((a > b) == asc) { pool[lo] = b; pool[hi] = a; }
            }
        }
    __syncthreads();
}

// D holds the distances to dataset rows col0 .. col0 + pitch (beyond the dataset: +inf).  With
// `carry` the k best found in earlier slices (ids_out, best_d) compete as well.  best_d[rows_total, k]
// receives the distances of the result; it is dists_out itself where the caller wants distances.
__global__ void __launch_bounds__(256)
row_select_kernel(const float *__restrict__ D, int64_t pitch, int64_t rows, int k,
                  uint32_t *__restrict__ ids_out, float *__restrict__ best_d, int64_t out_row0,
                  int64_t best_row0, int64_t col0, int carry, const uint32_t *gate)
{
    if (gate != nullptr && *gate == 0u) return;
    __shared__ uint64_t pool[kPool];
    __shared__ int count;
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    if (row >= rows) return;
    const float *src = D + row * pitch;
    uint32_t *ids_row = ids_out + (out_row0 + row) * k;
    float *d_row = best_d + (best_row0 + row) * k;
    uint64_t tau = kKeyInf;
    if (carry) {
        // the earlier result is sorted and its valid entries come first
        for (int i = tid; i < k; i += 256)
            pool[i] = ((uint64_t)f32_to_ordered(d_row[i]) << 32) | ids_row[i];
        __syncthreads();
        int n = 0;
        for (int i = 0; i < k; ++i) n += (uint32_t)pool[i] != kInvalidId;   // k <= 512, once per slice
        if (tid == 0) count = n;
        if (n >= k) tau = pool[k - 1];
    } else if (tid == 0) {
        count = 0;
    }
    __syncthreads();
    for (int64_t base = 0; base < pitch; base += 1024) {
        const int64_t c = base + tid * 4;
        if (c < pitch) {
            const float4 v = *reinterpret_cast<const float4 *>(src + c);
            const float vals[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                uint64_t key = ((uint64_t)f32_to_ordered(vals[u]) << 32) | (uint32_t)(col0 + c + u);
                if (key < tau) pool[atomicAdd(&count, 1)] = key;
            }
        }
        __syncthreads();
        const int n = count;
        __syncthreads();   // everyone has read the count before the next round appends to it
        if (n > kPool - 1024) {
            for (int i = n + tid; i < kPool; i += 256) pool[i] = ~0ull;
            pool_sort(pool, tid);
            if (tid == 0) count = n < k ? n : k;
            if (n >= k) tau = pool[k - 1];
            __syncthreads();
        }
    }
    const int n = count;
    for (int i = n + tid; i < kPool; i += 256) pool[i] = ~0ull;
    pool_sort(pool, tid);
    for (int i = tid; i < k; i += 256) {
        const bool ok = i < n;
        const uint64_t key = pool[i];
        ids_row[i] = ok ? (uint32_t)key : kInvalidId;
        d_row[i] = ok ? ordered_to_f32((uint32_t)(key >> 32)) : __uint_as_float(kFltMaxBits);
    }
}

constexpr int64_t kMaxCols = 1 << 20;   // dataset rows per slice (a multiple of kTile)

int64_t exact_search_pitch(int64_t N)
{
    const int64_t cols = N < kMaxCols ? N : kMaxCols;
    return (cols + kTile - 1) / kTile * kTile;
}

// The k smallest of every row of a dense block D[rows, pitch] (columns are the ids); no carry.
void launch_row_select(const float *D, int64_t pitch, int64_t rows, int k, uint32_t *ids_out, float *best_d,
                       hipStream_t stream)
{
    hipLaunchKernelGGL(row_select_kernel, dim3((unsigned)rows), dim3(256), 0, stream, D, pitch, rows, k, ids_out,
                       best_d, (int64_t)0, (int64_t)0, (int64_t)0, 0, (const uint32_t *)nullptr);
}

// scratch: block_rows x exact_search_pitch(N) floats, then block_rows x k floats (the running
// distances of a block when the caller does not ask for distances).  Query rows row_begin .. row_end;
// with a gate every kernel returns at once unless *gate != 0.
hipError_t launch_exact_search_gated(const float *X, int64_t N, int dim, int64_t ldX, int metric,
                                     const float *Q, int64_t row_end, int64_t ldQ, int64_t row_begin, int k,
                                     int exclude_self, int64_t self_offset, uint32_t *ids, float *dists,
                                     float *scratch, int64_t block_rows, const uint32_t *gate, hipStream_t stream)
{
    const int64_t pitch = exact_search_pitch(N);
    float *running = scratch + block_rows * pitch;
    for (int64_t r0 = row_begin; r0 < row_end; r0 += block_rows) {
        const int64_t rows = row_end - r0 < block_rows ? row_end - r0 : block_rows;
        for (int64_t c0 = 0; c0 < N; c0 += kMaxCols) {
            const int64_t cols = N - c0 < kMaxCols ? N - c0 : kMaxCols;
            dim3 grid((unsigned)(pitch / kTile), (unsigned)((rows + kTile - 1) / kTile));
            // rows of X from c0 on; the row to leave out is given relative to that slice
            hipLaunchKernelGGL(dist_tile_kernel, grid, dim3(256), 0, stream, Q, r0 + rows, ldQ, r0, X + c0 * ldX,
                               cols, ldX, dim, metric, exclude_self, self_offset - c0, scratch, pitch, gate);
            hipLaunchKernelGGL(row_select_kernel, dim3((unsigned)rows), dim3(256), 0, stream, scratch, pitch,
                               rows, k, ids, dists ? dists : running, r0, dists ? r0 : (int64_t)0, c0,
                               c0 > 0 ? 1 : 0, gate);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_exact_search(const float *X, int64_t N, int dim, int64_t ldX, int metric,
                               const float *Q, int64_t B, int64_t ldQ, int k, int exclude_self,
                               int64_t self_offset, uint32_t *ids, float *dists, float *scratch,
                               int64_t block_rows, hipStream_t stream)
{
    return launch_exact_search_gated(X, N, dim, ldX, metric, Q, B, ldQ, 0, k, exclude_self, self_offset, ids, dists,
                                     scratch, block_rows, nullptr, stream);
}

}  // namespace cagra
