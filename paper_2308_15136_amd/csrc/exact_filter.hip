// Exhaustive k-nearest-neighbour search (Eq. 1) with the bulk of the arithmetic on the matrix
// cores, and the result still that of the plain path bit for bit.
//
// The distance matrix of a block of query rows against the dataset is a dense contraction, the one
// place in this library where MFMA applies.  An fp16 product does not round like the sequential
// fp32 chain that defines the result, so it only *filters*:
//   1. the dataset (and the queries) are copied once as fp16, scaled by a power of two so that
//      the largest magnitude lies in [2^13, 2^14), together with their squared norms in fp32;
//   2. per block of query rows, approximate distances to every `stride`-th dataset row give a
//      per-row threshold tau (the t-th smallest of the sample, so that about t * stride dataset
//      rows lie below it);
//   3. the filter kernel forms approximate distances to all dataset rows tile by tile
//      (v_mfma_f32_32x32x16_f16) and appends the ids with  approx <= tau + eps  to the row's
//      candidate buffer, eps bounding |approx - exact| for the pair;
//   4. the re-rank kernel computes the exact distance (the same fused multiply-add chain as the
//      plain path) of every buffered candidate and sorts by (distance, id).  Every dataset row
//      whose exact distance is <= tau is in the buffer (by the choice of eps), so if the buffer
//      did not overflow and holds at least k entries with exact distance <= tau, its first k
//      are the global first k.  Otherwise the row raises its block's flag;
//   5. a block whose flag is up is done again by the plain kernels (they are always enqueued
//      and return at once when the flag is down), so the call stays asynchronous and exact
//      whatever the data: duplicates in their thousands or an unlucky sample only cost time.
//
// Bound used for eps (u = 2^-24; x~, q~ the fp16 copies; g = |x| |q|, S = |x|^2 + |q|^2):
//   fp16 rounding of both operands: |x~.q~ - x.q| <= (2^-10 + 2^-22) sum|x_i q_i| <= 2^-10 * 1.001 * g
//   (scaled values below the fp16 normal range add at most dim * 2^-38 * g);
//   fp32 accumulation inside the MFMA (rounded or truncated; the accumulators start at minus the right-hand
//   side of the test, see mfma_tile_kernel, so a partial sum can be as large as S resp. 2 g in scaled units),
//   of the norms, the start value, the final additions, and the rounding of the exact chain itself: together
//   <= (8.1 dim + 12) u S for squared L2, <= (5.1 dim + 6) u g for the inner product.
//   squared L2 (the product enters twice):  eps = 2 * 1.01 * 2^-10 * g + (12 dim + 48) u * S
//   inner product:                          eps = 2 * (1.01 * 2^-10 + (12 dim + 48) u) * g   (more than twice what is needed)
// g rather than S in the leading term keeps the filter sharp when queries and dataset rows differ
// much in norm.
#include <algorithm>
#include "device_util.h"
#include "build_kernels.h"

namespace cagra {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // 16 bytes in flight between global memory and LDS

constexpr int kFT = 128;          // output tile edge (4 wavefronts, 64 x 64 each)
constexpr int kFK = 64;           // dimensions staged per step (rows are padded to a multiple of 32)
constexpr int kFRow = kFK + 8;    // halfs per staged row in LDS (144 bytes: 16-byte aligned, banks spread)
constexpr int kStrip = 8;         // column tiles per workgroup
constexpr int kCap = kFilterCap;  // candidate buffer entries per query row

// ---- step 1: fp16 copy and norms ------------------------------------------------------------

// Largest |x| of a matrix as the bit pattern of a non-negative float (ordered like the value).
__global__ void __launch_bounds__(256)
maxabs_kernel(const float *__restrict__ X, int64_t rows, int dim, int64_t ld, uint32_t *out)
{
    uint32_t m = 0;
    const int64_t total = rows * dim;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / dim;
        const uint32_t b = __float_as_uint(X[r * ld + (i - r * dim)]) & 0x7FFFFFFFu;
        m = b > m ? b : m;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const uint32_t v = (uint32_t)__shfl_xor((int)m, o);
        m = v > m ? v : m;
    }
    if ((threadIdx.x & 63) == 0 && m != 0) atomicMax(out, m);
}

// Data whose largest magnitude lies below 2^kMinExponent is not scaled all the way up, and the error
// bound of the filter does not cover it: the re-rank kernel then certifies nothing.
constexpr int kMinExponent = -40;
__device__ __forceinline__ bool too_small(uint32_t maxbits)
{
    return maxbits != 0 && (int)(maxbits >> 23) - 127 < kMinExponent;
}

// Power of two that brings a largest magnitude with the given bits into [2^13, 2^14).
__device__ __forceinline__ float scale_of(uint32_t maxbits)
{
    if (maxbits == 0) return 1.0f;
    int e = (int)(maxbits >> 23) - 127;
    if (e < kMinExponent) e = kMinExponent;       // keeps the product of two scales finite; see too_small()
    return __uint_as_float((uint32_t)(127 + 13 - e) << 23);
}

// X16[r, 0..dimP) = fp16(X[r, :] * scale), zero beyond dim; norms[r] = sum of squares in fp32.
__global__ void __launch_bounds__(256)
to_half_kernel(const float *__restrict__ X, int64_t rows, int dim, int64_t ld, const uint32_t *maxbits,
               _Float16 *__restrict__ X16, int dimP, float *__restrict__ norms)
{
    const float scale = scale_of(*maxbits);
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // one wavefront per row
    if (r >= rows) return;
    float acc = 0.f;
    for (int c = lane; c < dimP; c += 64) {
        const float v = c < dim ? X[r * ld + c] : 0.f;
        acc = fmaf(v, v, acc);
        X16[r * dimP + c] = (_Float16)(v * scale);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) norms[r] = acc;
}

static __global__ void filter_fill_kernel(uint32_t *p, int64_t n, uint32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---- steps 2 and 3: approximate distances on the matrix cores -----------------------------------

struct FilterParams {
    const _Float16 *Q16;      // fp16 queries, rows dimP apart
    const _Float16 *X16;      // fp16 dataset, rows dimP apart
    const float *nq, *nx;     // squared norms (original scale)
    const uint32_t *q_maxbits, *x_maxbits;
    int64_t q_row0, q_rows;   // the block: query rows q_row0 .. ; rows >= q_rows do not exist
    int64_t n_cols;           // columns: dataset rows j * col_step for j < n_cols
    int64_t col_step;
    int dimP, metric;
    int row_tiles;            // tiles of 128 query rows in the block
    int64_t n_strips;         // strips of kStrip column tiles
    float c16, c32;           // eps = 2 c16 |q||x| + c32 (|q|^2 + |x|^2)  (L2),  2 (c16 + c32) |q||x|  (inner product)
    // dense output (the sample): out[local row, column], +inf beyond n_cols
    float *out;
    int64_t pitch;
    // filter output: ids with approx <= thr[local row * thr_stride] + eps appended to buf[local row, 0..cap)
    const float *thr;
    int64_t thr_stride;
    uint32_t *count, *buf;
    int exclude_self;
    int64_t self_offset;
};

// One workgroup: a tile of 128 query rows against a strip of kStrip tiles of 128 columns.  Four wavefronts,
// 64 x 64 outputs each (2 x 2 blocks of v_mfma_f32_32x32x16_f16).  The operands travel global -> registers -> LDS
// in steps of 64 dimensions; the loads of the next step are issued before the matrix instructions of the current
// one.  (Keeping the query rows in LDS for the whole strip and fetching the dataset rows two steps ahead was tried
// and is slower: 1.03 against 0.84 ms per block of 2,048 x 1M x 128.)
//
// Filter test without forming the distance: with inv = 1 / (scale_q scale_x) and acc the raw product,
//   squared L2:     |q|^2 + |x|^2 - 2 acc inv <= thr + 2 c16 |q||x| + c32 (|q|^2 + |x|^2)
//              <=>  acc >= Rr[row] + Cn[col] - Xr[row] |x|,   Rr = (|q|^2 (1 - c32) - thr) / (2 inv),
//                   Cn = |x|^2 (1 - c32) / (2 inv),  Xr = c16 |q| / inv
//   inner product:  -acc inv <= thr + 2 (c16 + c32) |q||x|
//              <=>  acc >= Rr[row] - Xr[row] |x|,   Rr = -thr / inv,  Xr = 2 (c16 + c32) |q| / inv
// (c32 leaves room for the few roundings of this rearrangement.)
// The filter instance does not even form the right-hand side at the end: the accumulators of a tile START at
// minus that value (one add and one fused multiply-add per output, which also spares clearing them), the matrix
// instructions add the product, and what is left to test is the sign: one compare per output whose lane mask
// lands in scalar registers, and a branch around everything else where no lane passed -- about one output in a
// thousand does.  A column that does not exist starts at minus infinity.
// The outputs that pass are not appended to their rows' candidate buffers one by one: an append is an atomic on device
// memory whose answer the wavefront would await (a few microseconds, longer than the matrix instructions of a whole
// tile, with its three companions waiting at the next barrier).  Each wavefront notes (row, id) in a list of its own in
// LDS -- positions from a count it keeps in a register, no atomics -- and empties the list into the buffers at the end
// of its strip of tiles, all lanes at once: one round trip for some thirty candidates.  A list that fills up is
// emptied early.
constexpr int kHitCap = 256;      // entries of a wavefront's list (about 33 are expected per strip)
constexpr size_t kFilterSmem = 1024 + (size_t)2 * kFT * kFRow * 2 + (size_t)4 * kHitCap * 8 + (size_t)kStrip * kFT * 4;

template <bool DENSE>
__global__ void __launch_bounds__(256, 2)     // at least two wavefronts per SIMD: two workgroups per CU
mfma_tile_kernel(const FilterParams P)
{
    extern __shared__ __align__(16) unsigned char f_smem[];
    float2 *s_row = reinterpret_cast<float2 *>(f_smem);     // [kFT]  filter: (Rr, Xr); dense: (|q|^2, unused)
    _Float16 *Xs = reinterpret_cast<_Float16 *>(f_smem + 1024);          // [kFT][kFRow]
    _Float16 *As = Xs + kFT * kFRow;                                       // [kFT][kFRow]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    uint2 *hit_list = reinterpret_cast<uint2 *>(As + kFT * kFRow) + wave * kHitCap;   // this wavefront's (row, id) notes
    // squared norms of the strip's columns, +inf for a column that does not exist: fetched once, so that no tile has to
    // wait for device memory (a wait for one load is a wait for every load issued before it, the staged pieces included)
    float *nx_s = reinterpret_cast<float *>(reinterpret_cast<uint2 *>(As + kFT * kFRow) + 4 * kHitCap);   // [kStrip * kFT]
    int n_listed = 0;                                                                    // the same in every lane
    // Workgroups are handed to the eight XCDs in turn, and each XCD has its own L2: the row tiles of
    // one column strip are numbered so that they all run on the same XCD, one after the other, and
    // the strip is fetched from memory once instead of once per row tile.
    const int64_t within = blockIdx.x % (8 * P.row_tiles);
    const int64_t strip = blockIdx.x / (8 * P.row_tiles) * 8 + within % 8;
    if (strip >= P.n_strips) return;
    const int64_t tile_r = within / 8 * kFT;                          // local row of the block
    const int64_t strip_c = strip * (kFT * kStrip);                   // first column of the strip
    const int m0 = (wave >> 1) * 64, n0 = (wave & 1) * 64;
    const float inv = 1.0f / (scale_of(*P.q_maxbits) * scale_of(*P.x_maxbits));   // powers of two: exact
    const float half_inv = 0.5f / inv;
    const float inf = __uint_as_float(0x7F800000u);

    if (tid < kFT) {
        const int64_t grow = P.q_row0 + tile_r + tid;
        const bool ok = grow < P.q_rows;
        const float nqv = ok ? P.nq[grow] : 0.f;
        if (DENSE) {
            s_row[tid] = make_float2(nqv, 0.f);
        } else {
            const float thr = ok ? P.thr[(tile_r + tid) * P.thr_stride] : 0.f;
            const float sq = sqrtf(nqv);
            s_row[tid] = P.metric == 0 ? make_float2((nqv * (1.0f - P.c32) - thr) * half_inv, P.c16 * sq / inv)
                                       : make_float2((0.0f - thr) / inv, 2.0f * (P.c16 + P.c32) * sq / inv);
        }
    }
    for (int i = tid; i < kStrip * kFT; i += 256) {
        const int64_t col = strip_c + i;
        nx_s[i] = col < P.n_cols ? P.nx[col * P.col_step] : inf;
    }
    __syncthreads();

    // staging: 1024 16-byte pieces per operand and step, four per thread
    const int n_chunks = (P.dimP + kFK - 1) / kFK;       // dimP is a multiple of 32: the last step may be half a step
    int64_t n_tiles = (P.n_cols - strip_c + kFT - 1) / kFT;
    if (DENSE) n_tiles = (P.pitch - strip_c) / kFT;                   // the padding columns are written too
    if (n_tiles > kStrip) n_tiles = kStrip;
    const int total = (int)n_tiles * n_chunks;
    int dst[4];
    const _Float16 *src_a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int p = tid + 256 * u;
        const int row = p >> 3, part = p & 7;
        const int64_t grow = P.q_row0 + tile_r + row;
        src_a[u] = P.Q16 + (grow < P.q_rows ? grow : P.q_rows - 1) * P.dimP;
        dst[u] = row * kFRow + part * 8;
    }
    // The 16-byte pieces this thread stages in one step: piece tid + 256 u of the 128 x 64 block of each operand.  The
    // loads carry no predicate: a row or column that does not exist reads the last one that does, a piece beyond the
    // row's dimensions reads the row's last piece, and none of that is ever used (the outputs of such rows and columns
    // are ignored, the matrix instructions stop at the row's dimensions).
    const int64_t last_col = P.n_cols - 1;
    const _Float16 *src_x[4];        // this thread's four dataset rows of the tile being fetched
    int src_tile = -1;
    auto fetch = [&](int f_step, u32x4_t (&xa)[4], u32x4_t (&xx)[4]) __attribute__((always_inline)) {
        const int f_tile = f_step / n_chunks, f_k0 = (f_step - f_tile * n_chunks) * kFK;
        if (f_tile != src_tile) {    // (uniform) the row addresses are formed once per tile, not once per step
            src_tile = f_tile;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int64_t f_col = strip_c + (int64_t)f_tile * kFT + ((tid + 256 * u) >> 3);
                f_col = f_col < last_col ? f_col : last_col;
                src_x[u] = P.X16 + f_col * P.col_step * P.dimP;
            }
        }
        int f_k = (tid & 7) * 8 + f_k0;          // (tid + 256 u) & 7 is the same for all four pieces
        f_k = f_k < P.dimP ? f_k : P.dimP - 8;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            xa[u] = *reinterpret_cast<const u32x4_t *>(src_a[u] + f_k);
            xx[u] = *reinterpret_cast<const u32x4_t *>(src_x[u] + f_k);
        }
    };
    floatx16_t acc[2][2];
    // Start values of a tile's accumulators: minus the right-hand side of the test (filter), zero (dense).
    auto start_tile = [&](int tile) __attribute__((always_inline)) {
        // (the 32 row constants of a lane are read anew for every tile: kept in registers they would cost 64 of them,
        // which is what the compiler does unless the address is opaque to it)
        int row_base = m0 + 4 * (lane >> 5);
        if (!DENSE) asm volatile("" : "+v"(row_base));
        float sx[2], cn[2];
        bool col_ok[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const float nxv = DENSE ? 0.f : nx_s[tile * kFT + n0 + nb * 32 + (lane & 31)];   // this lane's column of each 32-wide block
            // a column that does not exist: cn = +inf, so that its outputs start at minus infinity and stay there
            col_ok[nb] = nxv != inf;
            sx[nb] = sqrtf(col_ok[nb] ? nxv : 0.f);
            cn[nb] = !col_ok[nb] ? inf : P.metric == 0 ? nxv * (1.0f - P.c32) * half_inv : 0.f;
        }
#pragma unroll
        for (int ma = 0; ma < 2; ++ma)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (DENSE) {
                    acc[ma][0][r] = 0.f;
                    acc[ma][1][r] = 0.f;
                } else {
                    const float2 rc = s_row[row_base + ma * 32 + 8 * (r >> 2) + (r & 3)];
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        acc[ma][nb][r] = fmaf(rc.y, sx[nb], 0.0f - (rc.x + cn[nb]));
                }
            }
    };
    // operand layout of v_mfma_f32_32x32x16_f16: lane l holds row (l % 32), k = 8 * (l / 32) .. + 7
    const int fr = lane & 31, fk = (lane >> 5) * 8;

    // Empties this wavefront's list into the rows' candidate buffers.
    auto flush_hits = [&]() __attribute__((always_inline)) {
        wave_sync();                                     // the notes of all lanes are in LDS
        const int n = n_listed < kHitCap ? n_listed : kHitCap;
        for (int i = lane; i < n; i += 64) {
            const uint2 e = hit_list[i];
            const uint32_t at = atomicAdd(&P.count[e.x], 1u);
            if (at < (uint32_t)kCap) P.buf[(int64_t)e.x * kCap + at] = e.y;
        }
        wave_sync();                                     // read before the next notes overwrite them
        n_listed = 0;
    };

    // One step: the staged pieces go to LDS, the loads of a later step are issued into the registers they
    // leave, the matrix instructions of this step run, and a tile that is complete is tested (or written).
    auto do_step = [&](int step, u32x4_t (&xa)[4], u32x4_t (&xx)[4]) __attribute__((always_inline)) {
        __syncthreads();                       // the previous step's fragments have been read
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<u32x4_t *>(&As[dst[u]]) = xa[u];
            *reinterpret_cast<u32x4_t *>(&Xs[dst[u]]) = xx[u];
        }
        __syncthreads();
        // (a step without successor fetches itself once more rather than branch around the loads)
        fetch(step + 1 < total ? step + 1 : step, xa, xx);
        const int tile = step / n_chunks;
        const int chunk = step - tile * n_chunks;
        const int k0 = chunk * kFK;
#pragma unroll
        for (int ks = 0; ks < kFK / 16; ++ks) {
            if (k0 + ks * 16 >= P.dimP) break;          // the half step: its second half holds zeros
            half8_t a[2], b[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                a[h] = *reinterpret_cast<const half8_t *>(&As[(m0 + h * 32 + fr) * kFRow + ks * 16 + fk]);
                b[h] = *reinterpret_cast<const half8_t *>(&Xs[(n0 + h * 32 + fr) * kFRow + ks * 16 + fk]);
            }
#pragma unroll
            for (int ma = 0; ma < 2; ++ma)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    acc[ma][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ma], b[nb], acc[ma][nb], 0, 0, 0);
        }
        if (chunk != n_chunks - 1) return;

        // the tile is complete.  Result layout: register r of lane l is row 8 * (r / 4) + 4 * (l / 32) + r % 4,
        // column l % 32
        const int64_t tile_c = strip_c + (int64_t)tile * kFT;
        if (DENSE) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int64_t col = tile_c + n0 + nb * 32 + (lane & 31);
                const bool col_ok = col < P.n_cols;
                const float nxv = col_ok ? nx_s[tile * kFT + n0 + nb * 32 + (lane & 31)] : 0.f;
#pragma unroll
                for (int ma = 0; ma < 2; ++ma)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int lrow = m0 + ma * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                        const int64_t lr = tile_r + lrow;
                        if (P.q_row0 + lr < P.q_rows) {
                            const float dot = acc[ma][nb][r] * inv;
                            const float approx = P.metric == 0 ? (s_row[lrow].x + nxv) - 2.0f * dot : 0.0f - dot;
                            P.out[lr * P.pitch + col] = col_ok ? approx : inf;
                        }
                    }
            }
        } else {
            // The few that passed (about one in a thousand) are first only noted, bit nb * 32 + ma * 16 + r of `hits`,
            // where no lane of four registers passed behind one scalar branch; then all lanes append theirs together,
            // so that the wavefront waits for one atomic round trip per pass of that loop, not per register.
            uint32_t hits[2] = {0u, 0u};
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int ma = 0; ma < 2; ++ma)
#pragma unroll
                    for (int r0 = 0; r0 < 16; r0 += 4) {
                        uint64_t passed[4], any = 0ull;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            passed[r] = __ballot(acc[ma][nb][r0 + r] >= 0.f);
                            any |= passed[r];
                        }
                        if (any == 0ull) continue;
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (passed[r] != 0ull && acc[ma][nb][r0 + r] >= 0.f) hits[nb] |= 1u << (ma * 16 + r0 + r);
                    }
            uint64_t todo = ((uint64_t)hits[1] << 32) | hits[0];
            while (__ballot(todo != 0ull) != 0ull) {
                bool valid = false;
                uint32_t row = 0u, id32 = 0u;
                if (todo != 0ull) {
                    const int bit = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    const int nb = bit >> 5, ma = (bit >> 4) & 1, r = bit & 15;
                    const int lrow = m0 + ma * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const int64_t lr = tile_r + lrow, grow = P.q_row0 + lr;
                    const int64_t id = (tile_c + n0 + nb * 32 + (lane & 31)) * P.col_step;
                    valid = grow < P.q_rows && !(P.exclude_self && id == P.self_offset + grow);
                    row = (uint32_t)lr; id32 = (uint32_t)id;
                }
                const uint64_t mv = __ballot(valid);
                const int pos = n_listed + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mv >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mv, 0u));
                if (valid) {
                    if (pos < kHitCap) {
                        hit_list[pos] = make_uint2(row, id32);
                    } else {      // the list is full (a threshold that lets thousands pass): straight to the buffer
                        const uint32_t at = atomicAdd(&P.count[row], 1u);
                        if (at < (uint32_t)kCap) P.buf[(int64_t)row * kCap + at] = id32;
                    }
                }
                n_listed += __popcll(mv);
            }
            if (n_listed >= kHitCap / 2) flush_hits();
        }
        if (step + 1 < total) start_tile(tile + 1);
    };

    if (total <= 0) return;
    start_tile(0);
    u32x4_t va[4], vx[4];
    fetch(0, va, vx);
    for (int step = 0; step < total; ++step) do_step(step, va, vx);
    if (!DENSE) flush_hits();
}

// ---- step 4: exact distances of the candidates, order, certificate ----------------------------

__device__ void sort_keys(uint64_t *keys, int n_pow2, int tid)
{
    for (int k = 2; k <= n_pow2; k <<= 1)
        for (int j = k >> 1; j >= 1; j >>= 1) {
            __syncthreads();
            for (int i = tid; i < n_pow2 / 2; i += 256) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const uint64_t a = keys[lo], b = keys[hi];
                const bool asc = (lo & k) == 0;
                if ((a > b) == asc) { keys[lo] = b; keys[hi] = a; }
            }
        }
    __syncthreads();
}

__global__ void __launch_bounds__(256)
rerank_kernel(const float *__restrict__ X, int dim, int64_t ldX, int metric, const float *__restrict__ Q,
              int64_t ldQ, int64_t q_row0, const uint32_t *__restrict__ count, const uint32_t *__restrict__ buf,
              const float *__restrict__ thr, int64_t thr_stride, const uint32_t *q_maxbits,
              const uint32_t *x_maxbits, int k, uint32_t *__restrict__ ids_out, float *__restrict__ dists_out,
              uint32_t *flag)
{
    __shared__ uint64_t keys[kCap];
    extern __shared__ __align__(16) float qs[];
    const int tid = threadIdx.x;
    const int64_t lr = blockIdx.x, grow = q_row0 + lr;
    const uint32_t offered = count[lr];
    const int n = offered < (uint32_t)kCap ? (int)offered : kCap;
    for (int j = tid; j < dim; j += 256) qs[j] = Q[grow * ldQ + j];
    int n_pow2 = 256;
    while (n_pow2 < n) n_pow2 <<= 1;
    __syncthreads();
    for (int i = tid; i < n_pow2; i += 256) {
        uint64_t key = ~0ull;
        if (i < n) {
            const uint32_t id = buf[lr * kCap + i];
            const float *x = X + (int64_t)id * ldX;
            float acc = 0.f;
            // the plain path's chain: one fused multiply-add per dimension, in order
            if (metric == 0) {
                for (int j = 0; j < dim; j += 4) {
                    const float4 xv = *reinterpret_cast<const float4 *>(x + j);
                    float t = qs[j] - xv.x;     acc = fmaf(t, t, acc);
                    t = qs[j + 1] - xv.y;       acc = fmaf(t, t, acc);
                    t = qs[j + 2] - xv.z;       acc = fmaf(t, t, acc);
                    t = qs[j + 3] - xv.w;       acc = fmaf(t, t, acc);
                }
            } else {
                for (int j = 0; j < dim; j += 4) {
                    const float4 xv = *reinterpret_cast<const float4 *>(x + j);
                    acc = fmaf(qs[j], xv.x, acc);     acc = fmaf(qs[j + 1], xv.y, acc);
                    acc = fmaf(qs[j + 2], xv.z, acc); acc = fmaf(qs[j + 3], xv.w, acc);
                }
                acc = 0.0f - acc;
            }
            key = ((uint64_t)f32_to_ordered(acc) << 32) | id;
        }
        keys[i] = key;
    }
    sort_keys(keys, n_pow2, tid);
    // certificate: no overflow, and the k-th exact distance does not exceed the threshold
    const uint32_t tau = f32_to_ordered(thr[lr * thr_stride]);
    const bool certain = offered <= (uint32_t)kCap && n >= k && (uint32_t)(keys[k - 1] >> 32) <= tau &&
                         !too_small(*q_maxbits) && !too_small(*x_maxbits);
    if (tid == 0 && !certain) atomicOr(flag, 1u);
    for (int i = tid; i < k; i += 256) {
        const bool ok = i < n;
        const uint64_t key = keys[i < n_pow2 ? i : 0];
        ids_out[grow * k + i] = ok ? (uint32_t)key : kInvalidId;
        if (dists_out) dists_out[grow * k + i] = ok ? ordered_to_f32((uint32_t)(key >> 32)) : __uint_as_float(kFltMaxBits);
    }
}

// *out = number of flags that are up (one flag per block of query rows)
static __global__ void count_flags_kernel(const uint32_t *flags, int64_t n, uint32_t *out)
{
    uint32_t c = 0;
    for (int64_t i = threadIdx.x; i < n; i += 64) c += flags[i] != 0u;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) c += (uint32_t)__shfl_xor((int)c, o);
    if (threadIdx.x == 0) *out = c;
}

// ---- host side --------------------------------------------------------------------------------

void launch_fill_u32(uint32_t *p, int64_t n, uint32_t value, hipStream_t stream)
{
    hipLaunchKernelGGL(filter_fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n, value);
}

static size_t up256f(size_t v) { return (v + 255) & ~(size_t)255; }



FilterPlan plan_exact_filter(int64_t N, int dim, int64_t B, int k, bool share_queries)
{
    FilterPlan pl = {};
    pl.dimP = (dim + 31) / 32 * 32;
    pl.block_rows = std::min<int64_t>(2048, (B + kFT - 1) / kFT * kFT);
    pl.stride = std::max<int64_t>(32, (N + (1 << 20) - 1) >> 20);
    pl.n_sample = (N + pl.stride - 1) / pl.stride;
    const int64_t target = std::max<int64_t>(768, 3 * (int64_t)k);
    pl.t = (int)std::min<int64_t>(512, std::max<int64_t>(1, (target + pl.stride - 1) / pl.stride));
    pl.sample_pitch = (pl.n_sample + kFT - 1) / kFT * kFT;
    pl.n_blocks = (B + pl.block_rows - 1) / pl.block_rows;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += up256f(bytes); return at; };
    pl.off_x16 = take((size_t)N * pl.dimP * 2);
    pl.off_nx = take((size_t)N * 4);
    pl.off_q16 = share_queries ? pl.off_x16 : take((size_t)B * pl.dimP * 2);
    pl.off_nq = share_queries ? pl.off_nx : take((size_t)B * 4);
    pl.off_max = take(2 * 4);
    pl.off_thr_ids = take((size_t)pl.block_rows * pl.t * 4);
    pl.off_thr_d = take((size_t)pl.block_rows * pl.t * 4);
    pl.off_count = take((size_t)pl.block_rows * 4);
    pl.off_buf = take((size_t)pl.block_rows * kCap * 4);
    pl.off_flags = take((size_t)pl.n_blocks * 4);
    pl.bytes = off;
    return pl;
}

hipError_t launch_exact_filter(const float *X, int64_t N, int dim, int64_t ldX, int metric, const float *Q,
                               int64_t B, int64_t ldQ, int k, int exclude_self, int64_t self_offset, uint32_t *ids,
                               float *dists, float *plain_scratch, int64_t plain_block_rows, void *extra,
                               const FilterPlan &pl, bool share_queries, uint32_t *blocks_redone, hipStream_t stream)
{
    unsigned char *w = static_cast<unsigned char *>(extra);
    _Float16 *X16 = reinterpret_cast<_Float16 *>(w + pl.off_x16);
    _Float16 *Q16 = reinterpret_cast<_Float16 *>(w + pl.off_q16);
    float *nx = reinterpret_cast<float *>(w + pl.off_nx), *nq = reinterpret_cast<float *>(w + pl.off_nq);
    uint32_t *maxbits = reinterpret_cast<uint32_t *>(w + pl.off_max);
    uint32_t *thr_ids = reinterpret_cast<uint32_t *>(w + pl.off_thr_ids);
    float *thr_d = reinterpret_cast<float *>(w + pl.off_thr_d);
    uint32_t *count = reinterpret_cast<uint32_t *>(w + pl.off_count);
    uint32_t *buf = reinterpret_cast<uint32_t *>(w + pl.off_buf);
    uint32_t *flags = reinterpret_cast<uint32_t *>(w + pl.off_flags);

    // step 1
    hipLaunchKernelGGL(filter_fill_kernel, dim3(1), dim3(64), 0, stream, maxbits, (int64_t)2, 0u);
    hipLaunchKernelGGL(filter_fill_kernel, dim3((unsigned)((pl.n_blocks + 255) / 256)), dim3(256), 0, stream, flags,
                       pl.n_blocks, 0u);
    hipLaunchKernelGGL(maxabs_kernel, dim3(2048), dim3(256), 0, stream, X, N, dim, ldX, maxbits);
    hipLaunchKernelGGL(to_half_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, stream, X, N, dim, ldX, maxbits,
                       X16, pl.dimP, nx);
    if (!share_queries) {
        hipLaunchKernelGGL(maxabs_kernel, dim3(2048), dim3(256), 0, stream, Q, B, dim, ldQ, maxbits + 1);
        hipLaunchKernelGGL(to_half_kernel, dim3((unsigned)((B + 3) / 4)), dim3(256), 0, stream, Q, B, dim, ldQ,
                           maxbits + 1, Q16, pl.dimP, nq);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    FilterParams P = {};
    P.Q16 = Q16; P.X16 = X16; P.nq = nq; P.nx = nx;
    P.q_maxbits = share_queries ? maxbits : maxbits + 1; P.x_maxbits = maxbits;
    P.q_rows = B; P.dimP = pl.dimP; P.metric = metric;
    P.c16 = 1.01f / 1024.0f;
    P.c32 = (float)(12 * dim + 48) / 16777216.0f;
    P.thr = thr_d + (pl.t - 1); P.thr_stride = pl.t;
    P.count = count; P.buf = buf; P.exclude_self = exclude_self; P.self_offset = self_offset;

    for (int64_t b = 0; b < pl.n_blocks; ++b) {
        const int64_t r0 = b * pl.block_rows;
        const int64_t rows = std::min<int64_t>(pl.block_rows, B - r0);
        const unsigned row_tiles = (unsigned)((rows + kFT - 1) / kFT);
        P.q_row0 = r0;
        // step 2: the sample, dense, into the plain path's distance block; its t-th smallest per row
        FilterParams S = P;
        S.n_cols = pl.n_sample; S.col_step = pl.stride; S.out = plain_scratch; S.pitch = pl.sample_pitch;
        S.row_tiles = (int)row_tiles; S.n_strips = (pl.sample_pitch + kFT * kStrip - 1) / (kFT * kStrip);
        hipLaunchKernelGGL(mfma_tile_kernel<true>, dim3((unsigned)((S.n_strips + 7) / 8 * 8 * row_tiles)), dim3(256), kFilterSmem,
                           stream, S);
        launch_row_select(plain_scratch, pl.sample_pitch, rows, pl.t, thr_ids, thr_d, stream);
        // step 3
        hipLaunchKernelGGL(filter_fill_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, stream, count, rows, 0u);
        FilterParams F = P;
        F.n_cols = N; F.col_step = 1;
        F.row_tiles = (int)row_tiles; F.n_strips = (N + kFT * kStrip - 1) / (kFT * kStrip);
        hipLaunchKernelGGL(mfma_tile_kernel<false>, dim3((unsigned)((F.n_strips + 7) / 8 * 8 * row_tiles)), dim3(256), kFilterSmem,
                           stream, F);
        // step 4
        hipLaunchKernelGGL(rerank_kernel, dim3((unsigned)rows), dim3(256), (size_t)dim * 4, stream, X, dim, ldX, metric,
                           Q, ldQ, r0, count, buf, P.thr, P.thr_stride, P.q_maxbits, P.x_maxbits, k, ids, dists, flags + b);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        // step 5: the plain kernels over the same rows, gated by the block's flag
        e = launch_exact_search_gated(X, N, dim, ldX, metric, Q, r0 + rows, ldQ, r0, k, exclude_self, self_offset, ids,
                                      dists, plain_scratch, plain_block_rows, flags + b, stream);
        if (e != hipSuccess) return e;
    }
    if (blocks_redone != nullptr)
        hipLaunchKernelGGL(count_flags_kernel, dim3(1), dim3(64), 0, stream, flags, pl.n_blocks, blocks_redone);
    return hipGetLastError();
}

}  // namespace cagra
