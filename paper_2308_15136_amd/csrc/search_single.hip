// Single-workgroup-per-query CAGRA search for gfx950 (Sec. IV-A, IV-B, IV-C.1).
//
// One wavefront (64 lanes) owns one query at a time and runs the whole loop of
// steps 0-3 inside one kernel; workgroups are persistent and pull query indices
// from a device counter.  Per wavefront:
//   - top-M list and candidate list live in registers, one 64-bit key per
//     element: high word = order-preserving image of the fp32 distance, low
//     word = (node id << 1) | parent flag.  One unsigned 64-bit compare is the
//     (distance, id) order; the flag bit sits below the id so it cannot change
//     that order (Sec. IV-B.4 keeps the flag in the index word as well).
//   - element e of a list is held by lane e % 64 in register e / 64.
//   - step 1 is a bitonic sort of the candidates followed by a bitonic merge
//     into the sorted top-M list (Sec. IV-B.2).
//   - the visited table is an open-addressing hash in LDS that is cleared every
//     `reset_interval` passes and re-filled with the current top-M ids
//     (forgettable management, Sec. IV-B.3).
//   - distances are computed by teams of 4/8/16/32 lanes, one dataset row per
//     team, 16-byte loads, butterfly reduction (Sec. IV-B.1).
#include "device_util.h"
#include "search_params.h"

namespace cagra {

// ---- 64-bit keys spread over two 32-bit registers ------------------------------------------

__device__ __forceinline__ bool key_less(uint32_t ahi, uint32_t alo, uint32_t bhi, uint32_t blo)
{
    return (((uint64_t)ahi << 32) | alo) < (((uint64_t)bhi << 32) | blo);
}

// Compare-exchange with the lane `j` apart; keep_min lanes keep the smaller key.
__device__ __forceinline__ void ce_lanes(uint32_t &hi, uint32_t &lo, int j, bool keep_min)
{
    uint32_t phi = shfl_xor_u32(hi, j), plo = shfl_xor_u32(lo, j);
    bool pless = key_less(phi, plo, hi, lo);
    bool take = keep_min ? pless : !pless;
    hi = take ? phi : hi;
    lo = take ? plo : lo;
}

// Compare-exchange between two registers of the same lane.
__device__ __forceinline__ void ce_regs(uint32_t &ahi, uint32_t &alo, uint32_t &bhi, uint32_t &blo, bool a_min)
{
    bool bless = key_less(bhi, blo, ahi, alo);
    bool swap = a_min ? bless : !bless;
    uint32_t th = ahi, tl = alo;
    ahi = swap ? bhi : ahi;
    alo = swap ? blo : alo;
    bhi = swap ? th : bhi;
    blo = swap ? tl : blo;
}

// Bitonic merge of a bitonic sequence of 64*R elements (register-major layout) into
// ascending (ASC) or descending order.
template <int R, bool ASC>
__device__ __forceinline__ void bitonic_merge(uint32_t (&hi)[R], uint32_t (&lo)[R], int lane)
{
#pragma unroll
    for (int jr = R / 2; jr >= 1; jr >>= 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
            if ((r & jr) == 0) ce_regs(hi[r], lo[r], hi[r | jr], lo[r | jr], ASC);
    }
#pragma unroll
    for (int j = 32; j >= 1; j >>= 1) {
        bool keep_min = ((lane & j) == 0) == ASC;
#pragma unroll
        for (int r = 0; r < R; ++r) ce_lanes(hi[r], lo[r], j, keep_min);
    }
}

// Full bitonic sort, ascending, of 64*R elements.
template <int R>
__device__ __forceinline__ void bitonic_sort(uint32_t (&hi)[R], uint32_t (&lo)[R], int lane)
{
#pragma unroll
    for (int k = 2; k <= 64 * R; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j >= 1; j >>= 1) {
            if (j >= 64) {
                const int jr = j / 64;
#pragma unroll
                for (int r = 0; r < R; ++r)
                    if ((r & jr) == 0) {
                        bool asc = ((r * 64) & k) == 0;
                        ce_regs(hi[r], lo[r], hi[r | jr], lo[r | jr], asc);
                    }
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    int e = r * 64 + lane;
                    bool keep_min = ((e & j) == 0) == ((e & k) == 0);
                    ce_lanes(hi[r], lo[r], j, keep_min);
                }
            }
        }
    }
}

// Step 1 (Sec. IV-A, IV-B.2): sorted candidates c (ascending) merged into the sorted top-M
// list t; t keeps the 64*MR smallest.  Only the min(CR, MR) lowest candidate registers can
// matter.  The largest 64*C elements of t are replaced by the 64*C smallest of (those, c);
// that block is sorted descending so that t as a whole is bitonic, then merged.
template <int MR, int CR>
__device__ __forceinline__ void merge_into_topm(uint32_t (&thi)[MR], uint32_t (&tlo)[MR],
                                                uint32_t (&chi)[CR], uint32_t (&clo)[CR], int lane)
{
    constexpr int C = CR < MR ? CR : MR;
    uint32_t bhi[C], blo[C];
#pragma unroll
    for (int i = 0; i < C; ++i) {
        uint32_t phi = shfl_u32(chi[C - 1 - i], 63 - lane);
        uint32_t plo = shfl_u32(clo[C - 1 - i], 63 - lane);
        bool pless = key_less(phi, plo, thi[MR - C + i], tlo[MR - C + i]);
        bhi[i] = pless ? phi : thi[MR - C + i];
        blo[i] = pless ? plo : tlo[MR - C + i];
    }
    if constexpr (C == MR) {
        bitonic_merge<C, true>(bhi, blo, lane);
#pragma unroll
        for (int i = 0; i < C; ++i) { thi[i] = bhi[i]; tlo[i] = blo[i]; }
    } else {
        bitonic_merge<C, false>(bhi, blo, lane);
#pragma unroll
        for (int i = 0; i < C; ++i) { thi[MR - C + i] = bhi[i]; tlo[MR - C + i] = blo[i]; }
        bitonic_merge<MR, true>(thi, tlo, lane);
    }
}

// ---- visited table (Sec. IV-B.3) -------------------------------------------------------------

__device__ __forceinline__ uint32_t hash_slot(uint32_t id, int bits)
{
    return (id * 2654435761u) >> (32 - bits);
}

// true if id was not in the table (and is now).  `overflow` is raised if no free slot exists.
__device__ __forceinline__ bool visited_insert(uint32_t *table, int bits, uint32_t id, bool &overflow)
{
    const uint32_t mask = (1u << bits) - 1u;
    uint32_t s = hash_slot(id, bits);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        uint32_t old = atomicCAS(&table[s], kInvalidId, id);
        if (old == kInvalidId) return true;
        if (old == id) return false;
        s = (s + 1) & mask;
    }
    overflow = true;
    return true;
}

// ---- the kernel --------------------------------------------------------------------------------

template <int MR, int CR>
__global__ void __launch_bounds__(kWave)
search_single_kernel(const SingleParams P)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *table = reinterpret_cast<uint32_t *>(smem);
    float *qlds = reinterpret_cast<float *>(smem + P.off_query);
    uint32_t *newid = reinterpret_cast<uint32_t *>(smem + P.off_newid);
    float *newdist = reinterpret_cast<float *>(smem + P.off_newdist);
    uint32_t *parents = reinterpret_cast<uint32_t *>(smem + P.off_parents);

    const int lane = lane_id();
    const int team_log2 = P.team_log2;
    const int team = 1 << team_log2;
    const int n_teams = kWave >> team_log2;
    const int g = lane >> team_log2;       // team of this lane
    const int t = lane & (team - 1);       // lane within the team
    const int n_cand = P.search_width * P.degree;
    const int nchunk = P.dim >> 2;         // 16-byte pieces per row
    const int table_words = 1 << P.hash_bits;

    // candidate slot c = r*64 + lane expands neighbour (c % degree) of parent (c / degree)
    int slot_parent[CR], slot_nbr[CR];
#pragma unroll
    for (int r = 0; r < CR; ++r) {
        int c = r * 64 + lane;
        slot_parent[r] = c / P.degree;
        slot_nbr[r] = c - slot_parent[r] * P.degree;
    }

    for (;;) {
        // ---- persistent scheduling: next query ---------------------------------------------
        uint32_t qi = 0;
        if (lane == 0) qi = atomicAdd(P.counter, 1u);
        qi = __builtin_amdgcn_readfirstlane(qi);
        if ((int64_t)qi >= P.B) break;

        const float *q = P.queries + (size_t)qi * P.ld_queries;
        for (int j = lane; j < P.dim; j += kWave) qlds[j] = q[j];
        for (int j = lane; j < table_words; j += kWave) table[j] = kInvalidId;

        uint32_t thi[MR], tlo[MR], chi[CR], clo[CR];
#pragma unroll
        for (int r = 0; r < MR; ++r) { thi[r] = kDummyHi; tlo[r] = kInvalidId; }

        // step 0: random sampling (Sec. IV-A)
        const uint64_t qh = seed_query_hash(P.seed, qi);
        uint32_t raw[CR];
#pragma unroll
        for (int r = 0; r < CR; ++r) {
            int c = r * 64 + lane;
            raw[r] = c < n_cand ? seed_slot_id(qh, (uint64_t)c, (uint64_t)P.N) : kInvalidId;
        }
        __syncthreads();

        uint32_t n_iter = 0, n_parent_total = 0, n_dist_total = 0, flags = 0;
        bool overflow = false;

        for (int it = 0;; ++it) {
            // ---- step 3: first-time test, compaction, team distances ---------------------
            int n_new = 0;
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                bool isnew = false;
                if (raw[r] != kInvalidId) isnew = visited_insert(table, P.hash_bits, raw[r], overflow);
                uint64_t m = __ballot(isnew);
                int pos = n_new + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                       __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                if (isnew) newid[pos] = raw[r];
                n_new += __popcll(m);
            }
            __syncthreads();
            n_dist_total += (uint32_t)n_new;

            for (int c0 = 0; c0 < n_new; c0 += 2 * n_teams) {
                // two dataset rows per team in flight
                const int ca = c0 + g, cb = c0 + n_teams + g;
                const bool va = ca < n_new, vb = cb < n_new;
                const float *rowa = P.dataset + (size_t)(va ? newid[ca] : 0u) * P.ld;
                const float *rowb = P.dataset + (size_t)(vb ? newid[cb] : 0u) * P.ld;
                float acca = 0.f, accb = 0.f;
                for (int base = 0; base < nchunk; base += 4 * team) {
                    float4 xa[4], xb[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        int ch = base + i * team + t;
                        bool in = ch < nchunk;
                        xa[i] = (va && in) ? *reinterpret_cast<const float4 *>(rowa + 4 * ch) : make_float4(0, 0, 0, 0);
                        xb[i] = (vb && in) ? *reinterpret_cast<const float4 *>(rowb + 4 * ch) : make_float4(0, 0, 0, 0);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        int ch = base + i * team + t;
                        if (ch < nchunk) {
                            float4 qv = *reinterpret_cast<const float4 *>(qlds + 4 * ch);
                            if (P.metric == 0) {
                                float d0 = xa[i].x - qv.x, d1 = xa[i].y - qv.y, d2 = xa[i].z - qv.z, d3 = xa[i].w - qv.w;
                                acca = fmaf(d0, d0, acca); acca = fmaf(d1, d1, acca);
                                acca = fmaf(d2, d2, acca); acca = fmaf(d3, d3, acca);
                                float e0 = xb[i].x - qv.x, e1 = xb[i].y - qv.y, e2 = xb[i].z - qv.z, e3 = xb[i].w - qv.w;
                                accb = fmaf(e0, e0, accb); accb = fmaf(e1, e1, accb);
                                accb = fmaf(e2, e2, accb); accb = fmaf(e3, e3, accb);
                            } else {
                                acca = fmaf(xa[i].x, qv.x, acca); acca = fmaf(xa[i].y, qv.y, acca);
                                acca = fmaf(xa[i].z, qv.z, acca); acca = fmaf(xa[i].w, qv.w, acca);
                                accb = fmaf(xb[i].x, qv.x, accb); accb = fmaf(xb[i].y, qv.y, accb);
                                accb = fmaf(xb[i].z, qv.z, accb); accb = fmaf(xb[i].w, qv.w, accb);
                            }
                        }
                    }
                }
                for (int s = 1; s < team; s <<= 1) {
                    acca += __shfl_xor(acca, s, kWave);
                    accb += __shfl_xor(accb, s, kWave);
                }
                if (P.metric != 0) { acca = 0.0f - acca; accb = 0.0f - accb; }
                if (t == 0) {
                    if (va) newdist[ca] = acca;
                    if (vb) newdist[cb] = accb;
                }
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                int c = r * 64 + lane;
                bool v = c < n_new;
                chi[r] = v ? f32_to_ordered(newdist[c]) : kDummyHi;
                clo[r] = v ? (newid[c] << 1) : kInvalidId;
            }

            // ---- step 1: top-M update (skipped when no candidate can enter) ---------------
            {
                const int last = P.itopk - 1;
                uint32_t whi = shfl_u32(thi[MR - 1], last & 63), wlo = shfl_u32(tlo[MR - 1], last & 63);
                bool any = false;
#pragma unroll
                for (int r = 0; r < CR; ++r) any |= key_less(chi[r], clo[r], whi, wlo);
                if (__ballot(any) != 0ull) {
                    bitonic_sort<CR>(chi, clo, lane);
                    merge_into_topm<MR, CR>(thi, tlo, chi, clo, lane);
                    // logical length is itopk: the padding of the last register stays dummy
                    if ((MR - 1) * 64 + lane >= P.itopk) { thi[MR - 1] = kDummyHi; tlo[MR - 1] = kInvalidId; }
                }
            }
            if (it == P.max_iterations) { flags |= 1u; break; }

            // ---- forgettable management: periodic reset (Sec. IV-B.3) ---------------------
            if (P.reset_interval > 0 && it > 0 && (it % P.reset_interval) == 0) {
                __syncthreads();
                for (int j = lane; j < table_words; j += kWave) table[j] = kInvalidId;
                __syncthreads();
#pragma unroll
                for (int r = 0; r < MR; ++r)
                    if (tlo[r] != kInvalidId) (void)visited_insert(table, P.hash_bits, tlo[r] >> 1, overflow);
            }

            // ---- step 2: parents = first search_width entries without the flag ------------
            int n_par = 0;
#pragma unroll
            for (int r = 0; r < MR; ++r) {
                uint64_t m = __ballot((tlo[r] & 1u) == 0u);
                while (m != 0ull && n_par < P.search_width) {
                    int l = __builtin_ctzll(m);
                    m &= m - 1;
                    uint32_t w = __builtin_amdgcn_readlane(tlo[r], l);
                    if (lane == l) tlo[r] |= 1u;
                    if (lane == 0) parents[n_par] = w >> 1;
                    ++n_par;
                }
            }
            if (n_par == 0) break;
            n_parent_total += (uint32_t)n_par;
            ++n_iter;
            __syncthreads();
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                bool v = slot_parent[r] < n_par;
                raw[r] = v ? P.graph[(size_t)parents[v ? slot_parent[r] : 0] * P.degree + slot_nbr[r]] : kInvalidId;
            }
        }

        // ---- output: first k of the top-M list (Sec. IV-A) --------------------------------
#pragma unroll
        for (int r = 0; r < MR; ++r) {
            int e = r * 64 + lane;
            if (e < P.k) {
                bool valid = tlo[r] != kInvalidId;
                P.ids_out[(size_t)qi * P.k + e] = valid ? (tlo[r] >> 1) : kInvalidId;
                P.dists_out[(size_t)qi * P.k + e] = valid ? ordered_to_f32(thi[r]) : __uint_as_float(kFltMaxBits);
            }
        }
        if (__ballot(overflow) != 0ull) flags |= 2u;
        if (P.stats != nullptr && lane == 0) {
            uint32_t *s = P.stats + (size_t)qi * 4;
            s[0] = n_iter; s[1] = n_parent_total; s[2] = n_dist_total; s[3] = flags;
        }
        __syncthreads();
    }
}

__global__ void zero_counter_kernel(uint32_t *counter) { *counter = 0u; }

template <int MR, int CR>
static hipError_t launch_one(const SingleParams &P, int grid, size_t smem, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, stream, P.counter);
    hipLaunchKernelGGL((search_single_kernel<MR, CR>), dim3(grid), dim3(kWave), smem, stream, P);
    return hipGetLastError();
}

template <int MR>
static hipError_t launch_cr(const SingleParams &P, int cr, int grid, size_t smem, hipStream_t stream)
{
    switch (cr) {
        case 1: return launch_one<MR, 1>(P, grid, smem, stream);
        case 2: return launch_one<MR, 2>(P, grid, smem, stream);
        case 4: return launch_one<MR, 4>(P, grid, smem, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_search_single(const SingleParams &P, int mr, int cr, int grid, size_t smem, hipStream_t stream)
{
    switch (mr) {
        case 1: return launch_cr<1>(P, cr, grid, smem, stream);
        case 2: return launch_cr<2>(P, cr, grid, smem, stream);
        case 4: return launch_cr<4>(P, cr, grid, smem, stream);
        case 8: return launch_cr<8>(P, cr, grid, smem, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace cagra
