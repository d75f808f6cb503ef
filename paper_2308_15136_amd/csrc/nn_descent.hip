// Initial k-NN graph by NN-descent (Sec. III-B.1 names NN-descent and gives no details) for
// gfx950, in synchronous rounds in which every node pulls its candidates, so that the result does
// not depend on the order in which nodes are processed:
//   round 0   L_0(x) = the k best of k pseudo-random nodes (slot j of node x comes from the
//             search's step-0 generator applied to (seed, x, j));
//   round t   F(x) = the s entries of L_{t-1}(x) from rank w_t on, where the window
//             w_t = min(((t - 1) mod ceil(k / s)) * s, k - s) moves through the list from round to
//             round; R(x) = up to s nodes y with x in F(y), ordered by (rank of x in F(y), y);
//             L_t(x) = the k best of L_{t-1}(x) and every entry of L_{t-1}(v), v in F(x) then
//             R(x), each node once, x itself left out.
// One wavefront per node runs what is a search pass with fixed parents: the node's list sits in
// registers as sorted 64-bit keys, the rows of its parents are its candidates, a visited table in
// LDS keeps nodes from being measured twice, teams of lanes compute the distances, the winners
// are merged into the list (same device functions as the search kernels).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "../../include/cagra_hip.h"
#include "build_kernels.h"
#include "device_util.h"
#include "search_device.h"
#include "team_distance.h"

namespace cagra {

constexpr int kNndTableWords = 3072;                 // visited table: 768 sets of four ids
constexpr int kNndRowsInFlight = 4;

struct NndParams {
    const float *X;
    int64_t N, ld;
    int32_t dim, metric, k, s, team_log2;
    int32_t window;            // first rank of the forward sample of this round
    uint64_t seed;
    const uint32_t *prev_id;   // [N, k] lists of the previous round, nullptr in round 0
    const float *prev_d;       // [N, k]
    const uint32_t *rev;       // [N, s] reverse sample of this round
    const uint32_t *rev_len;   // [N]
    uint32_t *out_id;          // [N, k]
    float *out_d;              // [N, k]
};

template <int MR>
__global__ void __launch_bounds__(kWave)
nnd_round_kernel(const NndParams P)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *table = reinterpret_cast<uint32_t *>(smem);
    uint32_t *cursor = table + kNndTableWords;
    constexpr uint32_t sets = kNndTableWords / 4;
    uint32_t *newid = cursor + sets / 4;
    float *newdist = reinterpret_cast<float *>(newid + kWave);
    float *qlds = newdist + kWave;
    const int lane = lane_id();
    const int k = P.k;

    for (int64_t x = blockIdx.x; x < P.N; x += gridDim.x) {
        // the node's own vector is the query
        const float *q = P.X + x * P.ld;
        for (int j = lane; j < P.dim; j += kWave) qlds[j] = q[j];
        for (int j = 4 * lane; j < kNndTableWords; j += 4 * kWave)
            *reinterpret_cast<uint4 *>(table + j) = make_uint4(kInvalidId, kInvalidId, kInvalidId, kInvalidId);
        for (int j = lane; j < (int)sets / 4; j += kWave) cursor[j] = 0u;

        // the list of the previous round (round 0: empty)
        uint32_t thi[MR], tlo[MR];
#pragma unroll
        for (int r = 0; r < MR; ++r) {
            const int e = r * kWave + lane;
            uint32_t id = kInvalidId;
            float d = 0.f;
            if (P.prev_id != nullptr && e < k) { id = P.prev_id[x * k + e]; d = P.prev_d[x * k + e]; }
            thi[r] = id != kInvalidId ? f32_to_ordered(d) : kDummyHi;
            tlo[r] = id != kInvalidId ? (id << 1) : kInvalidId;
        }
        // parents: the first s entries of that list, then the reverse sample
        uint32_t par_f = kInvalidId, par_r = kInvalidId;
        int n_rev = 0;
        if (P.prev_id != nullptr) {
            if (lane < P.s) par_f = P.prev_id[x * k + P.window + lane];
            n_rev = (int)P.rev_len[x];
            if (lane < n_rev) par_r = P.rev[x * P.s + lane];
        }
        __syncthreads();

        bool forgot = false;
        // the node itself and its list are "seen": register them in the visited table
        {
            uint32_t set;
            const uint32_t self = (uint32_t)x;
            bool fresh = sets_lookup(table, sets, self, lane == 0, set);
            if (fresh) (void)sets_insert(table, cursor, set, self, forgot);
            lds_order();
#pragma unroll
            for (int r = 0; r < MR; ++r) {
                const uint32_t id = tlo[r] >> 1;
                fresh = sets_lookup(table, sets, id, tlo[r] != kInvalidId, set);
                lds_order();
                if (fresh) (void)sets_insert(table, cursor, set, id, forgot);
                lds_order();
            }
        }

        // batches of up to 64 candidates: round 0 draws them, later rounds read the parents' rows
        const uint64_t xh = seed_query_hash(P.seed, (uint64_t)x);
        const int chunks = (k + kWave - 1) / kWave;
        const int n_parents = P.prev_id != nullptr ? P.s + n_rev : 1;
        for (int pi = 0; pi < n_parents; ++pi) {
            uint32_t v = kInvalidId;
            if (P.prev_id != nullptr) {
                v = pi < P.s ? __builtin_amdgcn_readlane(par_f, pi) : __builtin_amdgcn_readlane(par_r, pi - P.s);
                if (v == kInvalidId) continue;
            }
            for (int ch = 0; ch < chunks; ++ch) {
                const int e = ch * kWave + lane;
                uint32_t raw[1] = {kInvalidId};
                if (e < k)
                    raw[0] = P.prev_id != nullptr ? P.prev_id[(int64_t)v * k + e]
                                                  : seed_slot_id(xh, (uint64_t)e, (uint64_t)P.N);
                if (raw[0] == (uint32_t)x) raw[0] = kInvalidId;

                // first-time test (the table may forget; list entry below rejects repeats)
                bool lost = false;
                uint32_t set, count = 0;
                bool fresh = sets_lookup(table, sets, raw[0], raw[0] != kInvalidId, set);
                lds_order();
                if (fresh) count = sets_insert(table, cursor, set, raw[0], forgot);
                lds_order();
                fresh = fresh && sets_confirm(table, cursor, set, count, raw[0], forgot, lost);
                const uint64_t m = __ballot(fresh);
                const int n_new = __popcll(m);
                if (n_new == 0) continue;
                const int pos = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                if (fresh) newid[pos] = raw[0];
                __syncthreads();
                team_distances<0, kNndRowsInFlight>(P.X, P.ld, P.dim, P.metric, P.team_log2, newid, n_new, qlds, newdist);
                __syncthreads();
                uint32_t chi[1], clo[1];
                chi[0] = lane < n_new ? f32_to_ordered(newdist[lane]) : kDummyHi;
                clo[0] = lane < n_new ? (newid[lane] << 1) : kInvalidId;
                __syncthreads();   // the candidate arrays are scratch for the update below
                int unused = 0;
                update_topm<MR, 1, true>(thi, tlo, chi, clo, k, lost, forgot, newid, newdist, lane, unused);
            }
        }

        // the list is sorted: write it out
#pragma unroll
        for (int r = 0; r < MR; ++r) {
            const int e = r * kWave + lane;
            if (e < k) {
                const bool valid = tlo[r] != kInvalidId;
                P.out_id[x * k + e] = valid ? (tlo[r] >> 1) : kInvalidId;
                P.out_d[x * k + e] = valid ? ordered_to_f32(thi[r]) : __uint_as_float(kFltMaxBits);
            }
        }
        __syncthreads();
    }
}

static size_t nnd_smem_bytes(int dim)
{
    return (size_t)4 * kNndTableWords + kNndTableWords / 4 + (size_t)4 * kWave * 2 + (size_t)4 * ((dim + 3) & ~3);
}

static size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct NndCarve {
    uint32_t *tmp_id, *rev, *rev_len;
    float *tmp_d;
    OptimizeScratch s;
    size_t bytes;
};

static NndCarve carve_nnd(void *base, int64_t N, int k, int s)
{
    unsigned char *p = static_cast<unsigned char *>(base);
    size_t used = 0;
    auto take = [&](size_t bytes) {
        unsigned char *r = p ? p + used : nullptr;
        used += up256(bytes);
        return r;
    };
    NndCarve c;
    c.tmp_id = reinterpret_cast<uint32_t *>(take((size_t)N * k * 4));
    c.tmp_d = reinterpret_cast<float *>(take((size_t)N * k * 4));
    c.rev = reinterpret_cast<uint32_t *>(take((size_t)N * s * 4));
    c.rev_len = reinterpret_cast<uint32_t *>(take((size_t)N * 4));
    c.s.indeg = reinterpret_cast<uint32_t *>(take((size_t)N * 4));
    c.s.cursor = reinterpret_cast<uint32_t *>(take((size_t)N * 4));
    c.s.offset = reinterpret_cast<uint64_t *>(take((size_t)N * 8));
    c.s.block_sum = reinterpret_cast<uint64_t *>(take((size_t)((N + 1023) / 1024) * 8));
    c.s.bucket = reinterpret_cast<uint64_t *>(take((size_t)N * s * 8));
    c.bytes = used;
    return c;
}

size_t nn_descent_workspace_bytes(int64_t N, int k, int s) { return carve_nnd(nullptr, N, k, s).bytes; }

int nn_descent_auto_rounds(int64_t N)
{
    // candidates spread over the neighbour-of-neighbour graph exponentially; measured, the lists stop
    // improving after about log2(N) / 2 + 2 rounds (6 at 20,000 nodes), the rest is margin
    int lg = 0;
    while (((int64_t)1 << lg) < N) ++lg;
    return lg / 2 + 5;
}

hipError_t launch_nn_descent(const float *X, int64_t N, int dim, int64_t ld, int metric, int k, int rounds,
                             int s, uint64_t seed, uint32_t *ids_out, float *dists_out, void *workspace,
                             hipStream_t stream)
{
    NndCarve c = carve_nnd(workspace, N, k, s);
    NndParams P = {};
    P.X = X; P.N = N; P.ld = ld; P.dim = dim; P.metric = metric; P.k = k; P.s = s; P.seed = seed;
    const int pieces = dim / 4;
    int team = 4;
    while (team < 32 && (pieces + team - 1) / team > 4) team *= 2;
    P.team_log2 = team == 4 ? 2 : team == 8 ? 3 : team == 16 ? 4 : 5;
    P.rev = c.rev; P.rev_len = c.rev_len;
    const size_t smem = nnd_smem_bytes(dim);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    const unsigned grid = (unsigned)std::min<int64_t>(N, (int64_t)cus * 10);
    const int mr = k <= 64 ? 1 : k <= 128 ? 2 : k <= 256 ? 4 : 8;
    // the result of the last round (number `rounds`) has to land in the caller's arrays
    for (int t = 0; t <= rounds; ++t) {
        const bool to_out = ((rounds - t) & 1) == 0;
        P.out_id = to_out ? ids_out : c.tmp_id;
        P.out_d = to_out ? dists_out : c.tmp_d;
        P.prev_id = t == 0 ? nullptr : (to_out ? c.tmp_id : ids_out);
        P.prev_d = t == 0 ? nullptr : (to_out ? c.tmp_d : dists_out);
        if (t > 0) {
            // the sample moves through the list from round to round, so that every entry gets to
            // propose its own neighbours (measured on 1M x 128: the lists of a sample fixed at the
            // closest entries miss the few far entries that tie clusters together)
            const int nwin = (k + s - 1) / s;
            P.window = std::min(((t - 1) % nwin) * s, k - s);
            hipError_t e = launch_reverse(P.prev_id + P.window, N, s, k, c.rev, c.rev_len, c.s, stream);
            if (e != hipSuccess) return e;
        }
        switch (mr) {
            case 1: hipLaunchKernelGGL(nnd_round_kernel<1>, dim3(grid), dim3(kWave), smem, stream, P); break;
            case 2: hipLaunchKernelGGL(nnd_round_kernel<2>, dim3(grid), dim3(kWave), smem, stream, P); break;
            case 4: hipLaunchKernelGGL(nnd_round_kernel<4>, dim3(grid), dim3(kWave), smem, stream, P); break;
            default: hipLaunchKernelGGL(nnd_round_kernel<8>, dim3(grid), dim3(kWave), smem, stream, P); break;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace cagra

using namespace cagra;

extern "C" {

size_t cagra_nn_descent_workspace_bytes(int64_t N, int32_t k, int32_t sample)
{
    if (sample == 0) sample = std::min(32, k);
    if (N < 2 || k < 1 || sample < 1) return 256;
    return nn_descent_workspace_bytes(N, k, sample);
}

int cagra_nn_descent(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric, int32_t k,
                     int32_t rounds, int32_t sample, uint64_t seed, uint32_t *knn_out, float *dists_out,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!dataset || !knn_out || !dists_out) return CAGRA_ERR_NULL_POINTER;
    if (N < 2 || N > 0x7FFFFFFFll || dim < 1 || dim > 0x7FFFFFFF - 4 || ld < ((dim + 3) & ~3) || (ld & 3) || ((uintptr_t)dataset & 15))
        return CAGRA_ERR_BAD_SHAPE;
    dim = (dim + 3) & ~3;   // rows are read four floats at a time; the caller vouches for zeros beyond dim
    if (metric != CAGRA_L2 && metric != CAGRA_IP) return CAGRA_ERR_BAD_OPTION;
    if (k < 1 || k > 512 || k >= N) return CAGRA_ERR_BAD_DEGREE;
    if (rounds > 1000) return CAGRA_ERR_BAD_OPTION;
    if (sample == 0) sample = std::min(32, k);
    if (sample < 1 || sample > 64 || sample > k) return CAGRA_ERR_BAD_OPTION;
    if (rounds < 0) rounds = nn_descent_auto_rounds(N);
    if (nnd_smem_bytes(dim) > 64 * 1024) return CAGRA_ERR_BAD_SHAPE;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < nn_descent_workspace_bytes(N, k, sample))
        return CAGRA_ERR_WORKSPACE;
    hipError_t e = launch_nn_descent(dataset, N, dim, ld, (int)metric, k, rounds, sample, seed, knn_out, dists_out,
                                     workspace, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}

}  // extern "C"
