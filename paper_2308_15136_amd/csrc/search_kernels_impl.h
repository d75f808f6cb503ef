// CAGRA search kernels for gfx950 (Sec. IV-A, IV-B, IV-C).
//
// One wavefront (64 lanes) runs the whole loop of steps 0-3 for one query (single mode)
// or for one worker of a query (multi mode):
//   - top-M list and candidate list live in registers, one 64-bit key per element: high
//     word = order-preserving image of the fp32 distance, low word = (node id << 1) |
//     parent flag.  One unsigned 64-bit compare is the (distance, id) order; the flag bit
//     sits below the id so it cannot change that order (Sec. IV-B.4 keeps the flag in the
//     index word as well).  Element e of a list is held by lane e % 64 in register e / 64.
//   - step 1 (update_topm): candidates that beat the last entry enter the sorted list, a few by
//     ordered insertion, many by a bitonic sort followed by a bitonic merge (Sec. IV-B.2).
//   - distances are computed by teams of 4/8/16/32 lanes, one dataset row per team,
//     16-byte loads, butterfly reduction (team_distances; Sec. IV-B.1).
// Single mode (Sec. IV-C.1): workgroups are persistent and pull query indices from a
// device counter; the visited table lives in LDS and forgets (Sec. IV-B.3), in one of two
// ways: kTableSets -- sets of four ids in which a new id replaces the oldest, with
// duplicates rejected where candidates enter the top-M list -- or kTableReset -- the
// paper's open-addressing table that is cleared every `reset_interval` passes and re-filled
// with the current top-M ids.  Both give the same results (a forgotten node that is measured
// again cannot enter the list a second time); they differ in how many distances are
// computed twice.
// Multi mode (Sec. IV-C.2): `workers` workgroups per query, each with one parent per pass,
// its own seeds and its own list, sharing one visited table in device memory; the last
// worker of a query to finish merges the lists and writes the result.
//
// This file is the implementation shared by the three storage types of the dataset; it is
// included by search_kernels_f32.hip, _f16.hip and _u8.hip, each of which sets CAGRA_ELEM
// (0 fp32, 1 fp16, 2 uint8).  Rows are always fetched as 16-byte pieces and widened to fp32
// in registers; distances are accumulated in fp32 (Sec. IV-C.1, last paragraph: lower
// precision storage relieves the memory-bandwidth limit).
#include "device_util.h"
#include "search_device.h"
#include "team_distance.h"
#include "search_params.h"

#ifndef CAGRA_ELEM
#error "include this file from search_kernels_<type>.hip"
#endif

namespace cagra {

constexpr int kElem = CAGRA_ELEM;

// Multi mode issues the first probe of every candidate before the dataset rows are fetched and
// looks at its answer afterwards (the row loads do not wait for the table).  `old` is what the
// first probe at the home slot returned; further probes only after a collision.
__device__ __forceinline__ bool visited_resolve_global(uint32_t *table, int bits, uint32_t id, uint32_t old, bool &overflow)
{
    if (old == kInvalidId) return true;
    if (old == id) return false;
    const uint32_t mask = (1u << bits) - 1u;
    uint32_t s = (hash_slot(id, bits) + 1) & mask;
    for (uint32_t probe = 1; probe <= mask; ++probe) {
        old = atomicCAS(&table[s], kInvalidId, id);
        if (old == kInvalidId) return true;
        if (old == id) return false;
        s = (s + 1) & mask;
    }
    overflow = true;
    return true;
}

// dataset rows each team keeps in flight (16 VGPRs apiece)
#ifndef CAGRA_ROWS_IN_FLIGHT
#define CAGRA_ROWS_IN_FLIGHT 4
#endif
constexpr int kRowsInFlight = CAGRA_ROWS_IN_FLIGHT;
constexpr int kRowsInFlightMulti = 8;   // multi mode: latency matters, registers do not
// Wide passes of fp32 rows: the kernel is bound to 8 wavefronts per CU by its LDS, which leaves each
// wavefront 256 VGPRs, enough for eight rows in flight (measured 1 to 2 % faster).  Not with lists
// beyond 128 entries or the narrow storage types, where eight rows would halve the wavefronts per CU
// (or, for fp16, gain nothing).
// The same for the narrow kernel with 129 to 256 candidates per pass, whose larger table and candidate
// buffers bind it to 8 wavefronts per CU as well.
// Byte rows: three in flight; two where the kernel is built for four wavefronts per SIMD (see min_waves).
#ifndef CAGRA_ROWS_IN_FLIGHT_U8
#define CAGRA_ROWS_IN_FLIGHT_U8 3
#endif
#ifndef CAGRA_ROWS_IN_FLIGHT_MAX
#define CAGRA_ROWS_IN_FLIGHT_MAX 8
#endif
// SHORT: variants for fp32 rows of at most 384 bytes with lists up to 128 entries, where one more wavefront per SIMD is
// worth more than rows in flight (measured on the 1M x 96 workload; rows of 512 and 800 bytes measured the other way
// round, and so did wide passes in chunks of 256).
//  - 129 to 256 candidates per pass: three wavefronts per SIMD, four rows in flight, which fits 168 registers
//    (256 candidates, list of 64: 1.24 -> 1.16 ms; list of 128: 1.69 -> 1.49 ms);
//  - up to 64 candidates per pass: four wavefronts per SIMD, three rows in flight, 128 registers
//    (64 candidates, list of 128: 1.49 -> 1.30 ms; 32 candidates: 2.33 -> 1.99 ms).
constexpr int short_rows_in_flight(int cr) { return cr == 1 ? 3 : 4; }
constexpr int short_waves(int cr) { return cr == 1 ? 4 : 3; }
#ifndef CAGRA_NARROW_4_MAX_MR
#define CAGRA_NARROW_4_MAX_MR 2
#endif
template <int ELEM, int MR, int CR>
constexpr bool narrow_small_pass() { return ELEM != 0 && CR == 1 && MR <= (ELEM == 1 ? 1 : CAGRA_NARROW_4_MAX_MR); }
template <int ELEM, int MR, int CR, bool SHORT = false>
constexpr int rows_in_flight_single()
{
    return SHORT ? short_rows_in_flight(CR) : (ELEM == 0 && MR <= 2 && CR == 4) ? CAGRA_ROWS_IN_FLIGHT_MAX
         : ELEM == 2 ? (narrow_small_pass<ELEM, MR, CR>() ? 2 : CAGRA_ROWS_IN_FLIGHT_U8) : kRowsInFlight;
}
#ifndef CAGRA_WIDE_LONG_ROWS_MAX_MR
#define CAGRA_WIDE_LONG_ROWS_MAX_MR 4
#endif
template <int ELEM, int MR>
constexpr int rows_in_flight_wide() { return (ELEM == 0 && MR <= CAGRA_WIDE_LONG_ROWS_MAX_MR) ? CAGRA_ROWS_IN_FLIGHT_MAX : ELEM == 2 ? CAGRA_ROWS_IN_FLIGHT_U8 : kRowsInFlight; }

// Optional phase timers (compile with -DCAGRA_PHASE_CLOCKS): shader-clock cycles that lane 0 of
// every wavefront spends in each part of the loop, summed over the launch into a device array
// that cagra_debug_phase_clocks_<type>() reads back.  Off by default; the timers cost a scalar
// memory-time read and a wait per phase.
#ifdef CAGRA_PHASE_CLOCKS
static __device__ unsigned long long g_phase_clocks[8];
static __device__ unsigned long long g_query_times[2 * 131072];   // start / end wall clock (100 MHz) of the first queries
#define CAGRA_PHASE_BEGIN() unsigned long long ph_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}; unsigned long long ph_t = __builtin_amdgcn_s_memtime();
#define CAGRA_PHASE(i) { const unsigned long long ph_n = __builtin_amdgcn_s_memtime(); ph_acc[i] += ph_n - ph_t; ph_t = ph_n; }
#define CAGRA_PHASE_END() if (lane == 0) { _Pragma("unroll") for (int ph_i = 0; ph_i < 8; ++ph_i) if (ph_acc[ph_i]) atomicAdd(&g_phase_clocks[ph_i], ph_acc[ph_i]); }
#else
#define CAGRA_PHASE_BEGIN()
#define CAGRA_PHASE(i)
#define CAGRA_PHASE_END()
#endif

// kinds of visited table
constexpr int kTableSets = 0;     // LDS, 4-way sets, replacement of the oldest
constexpr int kTableReset = 1;    // LDS, open addressing, periodic reset (Sec. IV-B.3)
constexpr int kTableGlobal = 2;   // device memory, open addressing, never forgets (multi mode)

struct QueryStats {
    uint32_t n_iter, n_parent, n_dist, flags;
};

// The search of one (query, worker): on return thi/tlo hold the sorted top-M list.
// `table` is the LDS table (single) or this query's device-memory table (multi).
template <int MR, int CR, int KIND, int RIF>
__device__ __forceinline__ void search_body(const SearchParams &P, uint32_t qi, int worker,
                                            uint32_t *table, float *qlds, uint32_t *newid,
                                            float *newdist, uint32_t *parents,
                                            const int (&slot_parent)[CR], const int (&slot_nbr)[CR],
                                            uint32_t (&thi)[MR], uint32_t (&tlo)[MR], QueryStats &qs)
{
    const int lane = lane_id();
    const int team_log2 = P.team_log2;
    const int n_cand = P.search_width * P.degree;
    constexpr bool MULTI = KIND == kTableGlobal;
    const int table_words = P.table_words;   // single mode: LDS table
    uint32_t *cursor = table + table_words;  // kTableSets: one byte per set behind the table
    const uint32_t sets = (uint32_t)table_words >> 2;

    CAGRA_PHASE_BEGIN()
    const float *q = P.queries + (size_t)qi * P.ld_queries;
    for (int j = lane; j < P.dim; j += kWave) qlds[j] = j < P.dim_query ? q[j] : 0.f;
    if (!MULTI) {
        for (int j = 4 * lane; j < table_words; j += 4 * kWave)
            *reinterpret_cast<uint4 *>(table + j) = make_uint4(kInvalidId, kInvalidId, kInvalidId, kInvalidId);
        if (KIND == kTableSets)
            for (int j = lane; j < (int)(sets + 3) / 4; j += kWave) cursor[j] = 0u;
    }

    uint32_t chi[CR], clo[CR];
#pragma unroll
    for (int r = 0; r < MR; ++r) { thi[r] = kDummyHi; tlo[r] = kInvalidId; }

    // step 0: random sampling (Sec. IV-A); worker w draws slots w * n_cand ...
    const uint64_t qh = seed_query_hash(P.seed, qi);
    uint32_t raw[CR];
#pragma unroll
    for (int r = 0; r < CR; ++r) {
        int c = r * 64 + lane;
        raw[r] = c < n_cand ? seed_slot_id(qh, (uint64_t)worker * n_cand + c, (uint64_t)P.N) : kInvalidId;
    }
    __syncthreads();

    uint32_t n_iter = 0, n_parent_total = 0, n_dist_total = 0, flags = 0;
    bool overflow = false;
    bool forgot = false;                 // kTableSets: the table has dropped an id it once held
    int lead = 0;                        // entries before this position are known to carry the parent flag
    uint32_t ahead[CR];                  // graph row read ahead for the likely next parent
    uint32_t ahead_id = kInvalidId;
#pragma unroll
    for (int r = 0; r < CR; ++r) ahead[r] = kInvalidId;

    CAGRA_PHASE(0)
    for (int it = 0;; ++it) {
        // ---- step 3: first-time test, compaction, team distances -------------------------
        int n_new = 0;
        bool lost = false;               // kTableSets: an id of this pass did not survive its own insertion
        bool fresh[CR];
        if constexpr (KIND == kTableSets) {
            uint32_t set[CR], way[CR];   // way: the set's insertion count before this lane's
#pragma unroll
            for (int r = 0; r < CR; ++r) fresh[r] = sets_lookup(table, sets, raw[r], raw[r] != kInvalidId, set[r]);
            lds_order();   // the 16-byte reads and the 4-byte writes below touch the same words
#pragma unroll
            for (int r = 0; r < CR; ++r) way[r] = fresh[r] ? sets_insert(table, cursor, set[r], raw[r], forgot) : 0u;
            lds_order();
#pragma unroll
            for (int r = 0; r < CR; ++r) fresh[r] = fresh[r] && sets_confirm(table, cursor, set[r], way[r], raw[r], forgot, lost);
        }
        uint32_t first_probe[CR];        // kTableGlobal: answer of the first probe, read after the distances
        if constexpr (KIND == kTableGlobal) {
            // Small batches are bound by latency, not by bandwidth: every candidate's row is fetched
            // while its table probe is still under way, and the distance of a node that turns out to
            // have been seen is thrown away.
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                first_probe[r] = kInvalidId;
                if (raw[r] != kInvalidId)
                    first_probe[r] = atomicCAS(&table[hash_slot(raw[r], P.hash_bits)], kInvalidId, raw[r]);
                newid[r * kWave + lane] = raw[r];
            }
            n_new = n_cand;
        } else {
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                bool isnew = false;
                if constexpr (KIND == kTableSets) isnew = fresh[r];
                else if (raw[r] != kInvalidId) isnew = visited_insert(table, (uint32_t)table_words, raw[r], overflow);
                const uint64_t m = __ballot(isnew);
                const int pos = n_new + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                             __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                if (isnew) newid[pos] = raw[r];
                n_new += __popcll(m);
            }
            n_dist_total += (uint32_t)n_new;
        }
        __syncthreads();
        CAGRA_PHASE(1)

        team_distances<kElem, RIF>(P.dataset, P.ld, P.dim, P.metric, team_log2, newid, n_new, qlds, newdist);
        __syncthreads();
        CAGRA_PHASE(2)
#pragma unroll
        for (int r = 0; r < CR; ++r) {
            int c = r * 64 + lane;
            bool v = c < n_new;
            if constexpr (KIND == kTableGlobal) {
                v = raw[r] != kInvalidId && visited_resolve_global(table, P.hash_bits, raw[r], first_probe[r], overflow);
                n_dist_total += (uint32_t)__popcll(__ballot(v));
            }
            chi[r] = v ? f32_to_ordered(newdist[c]) : kDummyHi;
            clo[r] = v ? (newid[c] << 1) : kInvalidId;
        }

        // ---- step 1: top-M update (skipped when no candidate can enter) -------------------
        update_topm<MR, CR, KIND == kTableSets>(thi, tlo, chi, clo, P.itopk, lost, forgot, newid, newdist, lane, lead);
        CAGRA_PHASE(3)
        if (it == P.max_iterations) { flags |= 1u; break; }

        // ---- forgettable management: periodic reset (Sec. IV-B.3), single mode only ------
        if (KIND == kTableReset && P.reset_interval > 0 && it > 0 && (it % P.reset_interval) == 0) {
            __syncthreads();
            for (int j = lane; j < table_words; j += kWave) table[j] = kInvalidId;
            __syncthreads();
#pragma unroll
            for (int r = 0; r < MR; ++r)
                if (tlo[r] != kInvalidId) (void)visited_insert(table, (uint32_t)table_words, tlo[r] >> 1, overflow);
        }

        CAGRA_PHASE(4)
        // ---- step 2: parents = first search_width entries without the flag ----------------
        int n_par = 0;
#pragma unroll
        for (int r = 0; r < MR; ++r) {
            if ((r + 1) * kWave <= lead || n_par == P.search_width) continue;   // nothing to find there
            uint64_t m = __ballot((tlo[r] & 1u) == 0u);
            while (m != 0ull && n_par < P.search_width) {
                int l = __builtin_ctzll(m);
                m &= m - 1;
                uint32_t w = __builtin_amdgcn_readlane(tlo[r], l);
                if (lane == l) tlo[r] |= 1u;
                if (lane == 0) parents[n_par] = w >> 1;
                ++n_par;
                lead = r * kWave + l + 1;    // everything up to the parent just taken has the flag
            }
        }
        if (n_par == 0) break;
        n_parent_total += (uint32_t)n_par;
        ++n_iter;
        __syncthreads();
        if (P.search_width == 1) {
            // One parent per pass: its graph row was usually fetched a pass ago (see below).
            const uint32_t par = parents[0];
            if (par == ahead_id) {
#pragma unroll
                for (int r = 0; r < CR; ++r) raw[r] = ahead[r];
            } else {
#pragma unroll
                for (int r = 0; r < CR; ++r)
                    raw[r] = slot_parent[r] == 0 ? P.graph[(size_t)par * P.degree + slot_nbr[r]] : kInvalidId;
            }
            // Read ahead: unless this pass finds something closer, the next parent is the first
            // entry still without the flag; its row travels while this pass computes distances.
            ahead_id = kInvalidId;
#pragma unroll
            for (int r = 0; r < MR; ++r) {
                if ((r + 1) * kWave <= lead || ahead_id != kInvalidId) continue;
                const uint64_t m = __ballot((tlo[r] & 1u) == 0u);
                if (m != 0ull) ahead_id = __builtin_amdgcn_readlane(tlo[r], __builtin_ctzll(m)) >> 1;
            }
            if (ahead_id != kInvalidId) {
#pragma unroll
                for (int r = 0; r < CR; ++r)
                    ahead[r] = slot_parent[r] == 0 ? P.graph[(size_t)ahead_id * P.degree + slot_nbr[r]] : kInvalidId;
            }
        } else {
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                bool v = slot_parent[r] < n_par;
                raw[r] = v ? P.graph[(size_t)parents[v ? slot_parent[r] : 0] * P.degree + slot_nbr[r]] : kInvalidId;
            }
        }
        CAGRA_PHASE(5)
    }
    CAGRA_PHASE_END()
    if (__ballot(overflow) != 0ull) flags |= 2u;
    qs.n_iter = n_iter; qs.n_parent = n_parent_total; qs.n_dist = n_dist_total; qs.flags = flags;
}

// One chunk of a wide pass: up to 64 * CRC candidates (raw[], kInvalidId where there is none) through the
// first-time test, the distance computation and the top-M update.
template <int MR, int CRC, int KIND, int RIF>
__device__ __forceinline__ void wide_chunk(const SearchParams &P, const uint32_t (&raw)[4], uint32_t *table,
                                           float *qlds, uint32_t *newid, float *newdist,
                                           uint32_t (&thi)[MR], uint32_t (&tlo)[MR], uint32_t &n_dist_total,
                                           bool &forgot, bool &overflow, int &lead, int lane)
{
    const int table_words = P.table_words;
    uint32_t *cursor = table + table_words;
    const uint32_t sets = (uint32_t)table_words >> 2;
    int n_new = 0;
    bool lost = false;
    bool fresh[CRC];
    if constexpr (KIND == kTableSets) {
        uint32_t set[CRC], way[CRC];
#pragma unroll
        for (int r = 0; r < CRC; ++r) fresh[r] = sets_lookup(table, sets, raw[r], raw[r] != kInvalidId, set[r]);
        lds_order();
#pragma unroll
        for (int r = 0; r < CRC; ++r) way[r] = fresh[r] ? sets_insert(table, cursor, set[r], raw[r], forgot) : 0u;
        lds_order();
#pragma unroll
        for (int r = 0; r < CRC; ++r) fresh[r] = fresh[r] && sets_confirm(table, cursor, set[r], way[r], raw[r], forgot, lost);
    }
#pragma unroll
    for (int r = 0; r < CRC; ++r) {
        bool isnew = false;
        if constexpr (KIND == kTableSets) isnew = fresh[r];
        else if (raw[r] != kInvalidId) isnew = visited_insert(table, (uint32_t)table_words, raw[r], overflow);
        const uint64_t m = __ballot(isnew);
        const int pos = n_new + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        if (isnew) newid[pos] = raw[r];
        n_new += __popcll(m);
    }
    n_dist_total += (uint32_t)n_new;
    __syncthreads();
    team_distances<kElem, RIF>(P.dataset, P.ld, P.dim, P.metric, P.team_log2, newid, n_new, qlds, newdist);
    __syncthreads();
    uint32_t chi[CRC], clo[CRC];
#pragma unroll
    for (int r = 0; r < CRC; ++r) {
        const int c = r * kWave + lane;
        const bool v = c < n_new;
        chi[r] = v ? f32_to_ordered(newdist[c]) : kDummyHi;
        clo[r] = v ? (newid[c] << 1) : kInvalidId;
    }
    update_topm<MR, CRC, KIND == kTableSets>(thi, tlo, chi, clo, P.itopk, lost, forgot, newid, newdist, lane, lead);
    __syncthreads();   // the update used newid / newdist as its staging space
}

// Candidate lists beyond 256 entries (search_width * degree up to 2048): the pass takes its
// candidates in chunks of 256 (four per lane), each through the same first-time test, distance
// computation and top-M update as a whole narrow pass.  The list after the last chunk holds the
// itopk best of (list + all candidates of the pass), whatever the chunking, because an entry the
// update drops is worse than itopk others and stays so.  Where the paper sorts such a candidate
// list with a radix sort (Sec. IV-B.2), the update here keeps only the candidates that beat the
// list's last entry (a threshold already at hand) and sorts those few.
template <int MR, int KIND, int RIF>
__device__ __forceinline__ void search_body_wide(const SearchParams &P, uint32_t qi,
                                                 uint32_t *table, float *qlds, uint32_t *newid,
                                                 float *newdist, uint32_t *parents,
                                                 uint32_t (&thi)[MR], uint32_t (&tlo)[MR], QueryStats &qs)
{
    constexpr int CR = 4;
    constexpr int kChunk = CR * kWave;
    static_assert(KIND == kTableSets || KIND == kTableReset, "single mode only");
    const int lane = lane_id();
    const int n_cand = P.search_width * P.degree;
    const int table_words = P.table_words;
    uint32_t *cursor = table + table_words;
    const uint32_t sets = (uint32_t)table_words >> 2;

    CAGRA_PHASE_BEGIN()
    const float *q = P.queries + (size_t)qi * P.ld_queries;
    for (int j = lane; j < P.dim; j += kWave) qlds[j] = j < P.dim_query ? q[j] : 0.f;
    for (int j = 4 * lane; j < table_words; j += 4 * kWave)
        *reinterpret_cast<uint4 *>(table + j) = make_uint4(kInvalidId, kInvalidId, kInvalidId, kInvalidId);
    if (KIND == kTableSets)
        for (int j = lane; j < (int)(sets + 3) / 4; j += kWave) cursor[j] = 0u;
#pragma unroll
    for (int r = 0; r < MR; ++r) { thi[r] = kDummyHi; tlo[r] = kInvalidId; }
    const uint64_t qh = seed_query_hash(P.seed, qi);
    __syncthreads();

    uint32_t n_iter = 0, n_parent_total = 0, n_dist_total = 0, flags = 0;
    bool overflow = false, forgot = false;
    int lead = 0, n_par = 0;
    // ceil(2^32 / degree); a wide pass has more than 256 candidates from at most 64 parents, so degree >= 5
    const uint32_t degree_magic = 0xFFFFFFFFu / (uint32_t)P.degree + 1u;

    CAGRA_PHASE(0)
    for (int it = 0;; ++it) {
        // sources of this pass: the random slots of step 0 (Sec. IV-A), later the parents' graph rows
        const int n_src = it == 0 ? n_cand : n_par * P.degree;
        auto fetch = [&](int base, uint32_t (&dst)[CR]) {
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                const int c = base + r * kWave + lane;
                if (it == 0) {
                    dst[r] = c < n_src ? seed_slot_id(qh, (uint64_t)c, (uint64_t)P.N) : kInvalidId;
                } else {
                    const int pi = (int)__umulhi((uint32_t)c, degree_magic);   // c / degree, exact for c < 2^16
                    const bool v = c < n_src;
                    dst[r] = v ? P.graph[(size_t)parents[v ? pi : 0] * P.degree + (c - pi * P.degree)] : kInvalidId;
                }
            }
        };
        uint32_t raw[CR], nxt[CR];
        fetch(0, raw);
        for (int base = 0; base < n_src; base += kChunk) {
            // the next chunk's graph entries travel while this chunk's distances are computed
            if (base + kChunk < n_src) fetch(base + kChunk, nxt);
            // a last chunk of at most 64 or 128 candidates takes the shorter code
            const int left = n_src - base;
            if (left <= kWave)
                wide_chunk<MR, 1, KIND, RIF>(P, raw, table, qlds, newid, newdist, thi, tlo, n_dist_total, forgot, overflow, lead, lane);
            else if (left <= 2 * kWave)
                wide_chunk<MR, 2, KIND, RIF>(P, raw, table, qlds, newid, newdist, thi, tlo, n_dist_total, forgot, overflow, lead, lane);
            else
                wide_chunk<MR, 4, KIND, RIF>(P, raw, table, qlds, newid, newdist, thi, tlo, n_dist_total, forgot, overflow, lead, lane);
#pragma unroll
            for (int r = 0; r < CR; ++r) raw[r] = nxt[r];
            CAGRA_PHASE(3)
        }
        if (it == P.max_iterations) { flags |= 1u; break; }

        if (KIND == kTableReset && P.reset_interval > 0 && it > 0 && (it % P.reset_interval) == 0) {
            for (int j = lane; j < table_words; j += kWave) table[j] = kInvalidId;
            __syncthreads();
#pragma unroll
            for (int r = 0; r < MR; ++r)
                if (tlo[r] != kInvalidId) (void)visited_insert(table, (uint32_t)table_words, tlo[r] >> 1, overflow);
        }

        // step 2: parents = first search_width entries without the flag
        n_par = 0;
#pragma unroll
        for (int r = 0; r < MR; ++r) {
            if ((r + 1) * kWave <= lead || n_par == P.search_width) continue;
            uint64_t m = __ballot((tlo[r] & 1u) == 0u);
            while (m != 0ull && n_par < P.search_width) {
                const int l = __builtin_ctzll(m);
                m &= m - 1;
                const uint32_t w = __builtin_amdgcn_readlane(tlo[r], l);
                if (lane == l) tlo[r] |= 1u;
                if (lane == 0) parents[n_par] = w >> 1;
                ++n_par;
                lead = r * kWave + l + 1;
            }
        }
        if (n_par == 0) break;
        n_parent_total += (uint32_t)n_par;
        ++n_iter;
        __syncthreads();
        CAGRA_PHASE(5)
    }
    CAGRA_PHASE_END()
    if (__ballot(overflow) != 0ull) flags |= 2u;
    qs.n_iter = n_iter; qs.n_parent = n_parent_total; qs.n_dist = n_dist_total; qs.flags = flags;
}

// ---- wave teams: several wavefronts of one workgroup on one query (Sec. IV-C.1 maps a query to a CTA
// of several warps) ------------------------------------------------------------------------------------
// Every wavefront of the team keeps its own copy of the top-M list in registers; the copies are identical
// at the start of every pass.  The candidates of a pass are split evenly among the wavefronts; each tests its
// share against the shared visited table, computes the distances of the first-time ones and updates its own
// copy.  It then publishes those of its candidates that are still in its copy (at most itopk), the team meets at
// a workgroup barrier, and every wavefront takes in what the others published.  Because the itopk best of a
// union are among the itopk best of each part, all copies are again the itopk best of (list + all candidates
// of the pass), which is the list of the one-wavefront search.  Parents are then selected by every wavefront
// for itself (same list, same choice; the number of parents that steers the loop is wavefront 0's), so no list is
// ever handed over.
// The shared table is used in three steps per round, separated by workgroup barriers: all wavefronts test their
// candidates, then all insert the missing ones, then all read their sets again.  One thing differs from one
// wavefront: the insertions of different wavefronts reach the table in any order, so an id written under an older
// count may land after, and replace, one written under a newer count of the same way.  sets_confirm<true>
// therefore also looks whether the lane's own id is still where it put it and reports `lost` if not.  With that,
// two lanes of one wavefront that both count their (same) node as new always come with a `lost` report in that
// wavefront, and the complete check runs; the same node counted as new by two wavefronts is caught where a
// published copy enters the other's list (always checked against the list first).  What the table forgets is
// caught where candidates enter a list copy, as in the one-wavefront search.

// sets_insert for a table shared by several wavefronts: `forgot` is a workgroup-wide word
__device__ __forceinline__ uint32_t sets_insert_shared(uint32_t *table, uint32_t *cursor, uint32_t set, uint32_t id,
                                                       uint32_t *forgot_word)
{
    const uint32_t sh = 8u * (set & 3u);
    const uint32_t count = (atomicAdd(&cursor[set >> 2], 1u << sh) >> sh) & 0xFFu;
    if (count >= 4u) *forgot_word = 1u;
    table[4 * set + (count & 3u)] = id;
    return count;
}

// This wavefront's share of a round: up to 64 * CRC candidates through the first-time test, the distance
// computation and the update of its list copy; then the survivors are published in (pub_hi, pub_lo, pub_count).
template <int MR, int CRC, int RIF>
__device__ __forceinline__ void team_chunk(const SearchParams &P, const uint32_t (&raw)[4], uint32_t *table,
                                           uint32_t *forgot_word, float *qlds, uint32_t *newid, float *newdist,
                                           uint32_t (&thi)[MR], uint32_t (&tlo)[MR], uint32_t &n_dist_total, int &lead, int lane,
                                           uint32_t *pub_hi, uint32_t *pub_lo, uint32_t *pub_count, int pub_cap)
{
    const int table_words = P.table_words;
    uint32_t *cursor = table + table_words;
    const uint32_t sets = (uint32_t)table_words >> 2;
    int n_new = 0;
    bool lost = false, forgot_lane = false;
    bool fresh[CRC];
    uint32_t set[CRC], way[CRC];
#pragma unroll
    for (int r = 0; r < CRC; ++r) fresh[r] = sets_lookup(table, sets, raw[r], raw[r] != kInvalidId, set[r]);
    __syncthreads();   // every wavefront of the team makes the same calls with the same CRC
#pragma unroll
    for (int r = 0; r < CRC; ++r) way[r] = fresh[r] ? sets_insert_shared(table, cursor, set[r], raw[r], forgot_word) : 0u;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < CRC; ++r) fresh[r] = fresh[r] && sets_confirm<true>(table, cursor, set[r], way[r], raw[r], forgot_lane, lost);
#pragma unroll
    for (int r = 0; r < CRC; ++r) {
        const uint64_t m = __ballot(fresh[r]);
        const int pos = n_new + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        if (fresh[r]) newid[pos] = raw[r];
        n_new += __popcll(m);
    }
    n_dist_total += (uint32_t)n_new;
    wave_sync();
    team_distances<kElem, RIF>(P.dataset, P.ld, P.dim, P.metric, P.team_log2, newid, n_new, qlds, newdist);
    wave_sync();
    uint32_t chi[CRC], clo[CRC];
#pragma unroll
    for (int r = 0; r < CRC; ++r) {
        const int c = r * kWave + lane;
        const bool v = c < n_new;
        chi[r] = v ? f32_to_ordered(newdist[c]) : kDummyHi;
        clo[r] = v ? (newid[c] << 1) : kInvalidId;
    }
    wave_sync();   // the update uses newid / newdist as its staging space
    const bool forgot = *forgot_word != 0u;
    update_topm<MR, CRC, true>(thi, tlo, chi, clo, P.itopk, lost, forgot, newid, newdist, lane, lead);
    // publish the candidates that are in the list now: those not beyond its last entry
    const int last = P.itopk - 1;
    uint32_t whi = kDummyHi, wlo = kInvalidId;
#pragma unroll
    for (int r = 0; r < MR; ++r)
        if (r == (last >> 6)) {
            whi = __builtin_amdgcn_readlane(thi[r], last & 63);
            wlo = __builtin_amdgcn_readlane(tlo[r], last & 63);
        }
    int n_pub = 0;
#pragma unroll
    for (int r = 0; r < CRC; ++r) {
        const bool in = clo[r] != kInvalidId && !key_less(whi, wlo | 1u, chi[r], clo[r]);
        const uint64_t m = __ballot(in);
        const int pos = n_pub + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        if (in && pos < pub_cap) { pub_hi[pos] = chi[r]; pub_lo[pos] = clo[r]; }
        n_pub += __popcll(m);
    }
    if (lane == 0) *pub_count = (uint32_t)(n_pub < pub_cap ? n_pub : pub_cap);
}

// What another wavefront published goes into this wavefront's copy of the list; every arrival is checked
// against the list first (update_topm with `forgot` set).
template <int MR, int CRX>
__device__ __forceinline__ void team_take(const SearchParams &P, const uint32_t *pub_hi, const uint32_t *pub_lo, int first, int count,
                                          uint32_t (&thi)[MR], uint32_t (&tlo)[MR], uint32_t *scratch_id, float *scratch_key,
                                          int lane, int &lead)
{
    uint32_t chi[CRX], clo[CRX];
#pragma unroll
    for (int r = 0; r < CRX; ++r) {
        const int c = first + r * kWave + lane;
        const bool v = c < count;
        chi[r] = v ? pub_hi[c] : kDummyHi;
        clo[r] = v ? pub_lo[c] : kInvalidId;
    }
    update_topm<MR, CRX, true>(thi, tlo, chi, clo, P.itopk, false, true, scratch_id, scratch_key, lane, lead);
}

#ifndef CAGRA_TEAM_ROWS_IN_FLIGHT
#define CAGRA_TEAM_ROWS_IN_FLIGHT 4
#endif

// The search of one query by a team of NW wavefronts (single mode, replacement table).  Called by all
// wavefronts of the workgroup; on return every one of them holds the sorted top-M list in thi / tlo.
template <int MR, int NW>
__device__ __forceinline__ void search_body_team(const SearchParams &P, uint32_t qi, int wave, uint32_t *table,
                                                 uint32_t *team_words, float *qlds, uint32_t *newid, float *newdist,
                                                 uint32_t *parents, uint32_t *pub_hi, uint32_t *pub_lo,
                                                 uint32_t (&thi)[MR], uint32_t (&tlo)[MR], QueryStats &qs)
{
    constexpr int CR = 4;
    constexpr int kChunk = CR * kWave;
    constexpr int RIF = CAGRA_TEAM_ROWS_IN_FLIGHT;
    const int lane = lane_id();
    const int tid = wave * kWave + lane;
    const int n_cand = P.search_width * P.degree;
    const int table_words = P.table_words;
    uint32_t *cursor = table + table_words;
    const uint32_t sets = (uint32_t)table_words >> 2;
    const int pub_cap = P.pub_cap;
    uint32_t *forgot_word = team_words;          // [0]
    uint32_t *pub_count = team_words + 4;        // [4 .. 4 + 2 * NW)

    const float *q = P.queries + (size_t)qi * P.ld_queries;
    for (int j = tid; j < P.dim; j += kWave * NW) qlds[j] = j < P.dim_query ? q[j] : 0.f;
    for (int j = 4 * tid; j < table_words; j += 4 * kWave * NW)
        *reinterpret_cast<uint4 *>(table + j) = make_uint4(kInvalidId, kInvalidId, kInvalidId, kInvalidId);
    for (int j = tid; j < (int)(sets + 3) / 4; j += kWave * NW) cursor[j] = 0u;
    if (tid == 0) *forgot_word = 0u;
#pragma unroll
    for (int r = 0; r < MR; ++r) { thi[r] = kDummyHi; tlo[r] = kInvalidId; }
    const uint64_t qh = seed_query_hash(P.seed, qi);
    __syncthreads();

    uint32_t n_iter = 0, n_parent_total = 0, n_dist_total = 0, flags = 0;
    int lead = 0, n_par = 0;
    uint32_t round = 0;
    const uint32_t degree_magic = 0xFFFFFFFFu / (uint32_t)P.degree + 1u;   // ceil(2^32 / degree), degree >= 2

    for (int it = 0;; ++it) {
        const int n_src = it == 0 ? n_cand : n_par * P.degree;
        for (int base = 0; base < n_src; base += NW * kChunk, ++round) {
            const int n_round = n_src - base < NW * kChunk ? n_src - base : NW * kChunk;
            const int share = (n_round + NW - 1) / NW;
            const int lo = base + wave * share;
            const int hi = lo + share < base + n_round ? lo + share : base + n_round;
            uint32_t raw[CR];
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                const int c = lo + r * kWave + lane;
                const bool v = c < hi;
                if (it == 0) {
                    raw[r] = v ? seed_slot_id(qh, (uint64_t)c, (uint64_t)P.N) : kInvalidId;
                } else {
                    const int pi = (int)__umulhi((uint32_t)c, degree_magic);   // c / degree, exact for c < 2^16
                    raw[r] = v ? P.graph[(size_t)parents[v ? pi : 0] * P.degree + (c - pi * P.degree)] : kInvalidId;
                }
            }
            const int buf = (int)(round & 1u);
            uint32_t *my_hi = pub_hi + (buf * NW + wave) * pub_cap;
            uint32_t *my_lo = pub_lo + (buf * NW + wave) * pub_cap;
            if (share <= kWave)
                team_chunk<MR, 1, RIF>(P, raw, table, forgot_word, qlds, newid, newdist, thi, tlo, n_dist_total, lead, lane,
                                       my_hi, my_lo, pub_count + buf * NW + wave, pub_cap);
            else if (share <= 2 * kWave)
                team_chunk<MR, 2, RIF>(P, raw, table, forgot_word, qlds, newid, newdist, thi, tlo, n_dist_total, lead, lane,
                                       my_hi, my_lo, pub_count + buf * NW + wave, pub_cap);
            else
                team_chunk<MR, 4, RIF>(P, raw, table, forgot_word, qlds, newid, newdist, thi, tlo, n_dist_total, lead, lane,
                                       my_hi, my_lo, pub_count + buf * NW + wave, pub_cap);
            __syncthreads();
            // Two publication buffers, used in turn: a wavefront writes a buffer again two rounds later, after the
            // barrier of the round in between, which every wavefront reaches only once it has read this one.
#pragma unroll
            for (int v = 0; v < NW; ++v) {
                if (v == wave) continue;
                const int cnt = (int)pub_count[buf * NW + v];
                const uint32_t *o_hi = pub_hi + (buf * NW + v) * pub_cap;
                const uint32_t *o_lo = pub_lo + (buf * NW + v) * pub_cap;
                if (cnt == 0) continue;
                if (cnt <= kWave) {
                    team_take<MR, 1>(P, o_hi, o_lo, 0, cnt, thi, tlo, newid, newdist, lane, lead);
                } else {
                    for (int first = 0; first < cnt; first += kChunk)
                        team_take<MR, 4>(P, o_hi, o_lo, first, cnt, thi, tlo, newid, newdist, lane, lead);
                }
                wave_sync();
            }
        }
        if (it == P.max_iterations) { flags |= 1u; break; }

        // step 2: parents = first search_width entries without the flag.  Every wavefront marks them in its own
        // copy; the ids the team expands and the decision to go on are wavefront 0's, handed over through LDS, so
        // that all wavefronts make the same number of rounds whatever their copies hold.
        int n_sel = 0;
#pragma unroll
        for (int r = 0; r < MR; ++r) {
            if ((r + 1) * kWave <= lead || n_sel == P.search_width) continue;
            uint64_t m = __ballot((tlo[r] & 1u) == 0u);
            while (m != 0ull && n_sel < P.search_width) {
                const int l = __builtin_ctzll(m);
                m &= m - 1;
                const uint32_t w = __builtin_amdgcn_readlane(tlo[r], l);
                if (lane == l) tlo[r] |= 1u;
                if (tid == 0) parents[n_sel] = w >> 1;
                ++n_sel;
                lead = r * kWave + l + 1;
            }
        }
        if (tid == 0) team_words[3] = (uint32_t)n_sel;
        __syncthreads();
        n_par = (int)team_words[3];
        if (n_par == 0) break;
        n_parent_total += (uint32_t)n_par;
        ++n_iter;
    }
    qs.n_iter = n_iter; qs.n_parent = n_parent_total; qs.n_dist = n_dist_total; qs.flags = flags;
}

// First k of the sorted list -> ids / dists (Sec. IV-A, last sentence).
template <int MR>
__device__ __forceinline__ void write_result(const SearchParams &P, uint32_t qi,
                                             const uint32_t (&thi)[MR], const uint32_t (&tlo)[MR])
{
    const int lane = lane_id();
#pragma unroll
    for (int r = 0; r < MR; ++r) {
        int e = r * 64 + lane;
        if (e < P.k) {
            bool valid = tlo[r] != kInvalidId;
            P.ids_out[(size_t)qi * P.k + e] = valid ? (tlo[r] >> 1) : kInvalidId;
            P.dists_out[(size_t)qi * P.k + e] = valid ? ordered_to_f32(thi[r]) : __uint_as_float(kFltMaxBits);
        }
    }
}

#define CAGRA_LDS_VIEWS                                                          \
    extern __shared__ __align__(16) unsigned char smem[];                       \
    float *qlds = reinterpret_cast<float *>(smem + P.off_query);               \
    uint32_t *newid = reinterpret_cast<uint32_t *>(smem + P.off_newid);        \
    float *newdist = reinterpret_cast<float *>(smem + P.off_newdist);          \
    uint32_t *parents = reinterpret_cast<uint32_t *>(smem + P.off_parents);    \
    const int lane = lane_id();                                                  \
    int slot_parent[CR], slot_nbr[CR];                                           \
    _Pragma("unroll") for (int r = 0; r < CR; ++r) {                             \
        int c = r * 64 + lane;                                                   \
        slot_parent[r] = c / P.degree;                                           \
        slot_nbr[r] = c - slot_parent[r] * P.degree;                             \
    }

// Wavefronts per SIMD the compiler has to leave room for.  Two everywhere (256 registers; a few kernels would
// otherwise take a handful more and drop to one).  Three (168 registers) for the narrow storage types with lists up
// to CAGRA_NARROW_3_MAX_MR * 64 entries: their rows are short, the memory system is not what limits them, and a
// third wavefront per SIMD is worth 12 to 15 % (measured on the 1M x 128 workload); three as well for the SHORT
// variant (see rows_in_flight_single).  Four (128 registers) for the narrow types with at most 64
// candidates per pass, where a pass is a short chain of dependent loads and little else (one parent per pass, itopk
// 128, 1M x 128: byte rows 2.42 -> 2.09 ms, fp16 rows at itopk 64 1.51 -> 1.39 ms); fp16 only up to 64 entries,
// beyond that its kernel would spill.
#ifndef CAGRA_NARROW_3_MAX_MR
#define CAGRA_NARROW_3_MAX_MR 2
#endif
template <int ELEM, int MR, int CR = 4, bool SHORT = false>
constexpr int min_waves()
{
    return narrow_small_pass<ELEM, MR, CR>() ? 4 : SHORT ? short_waves(CR) : (ELEM != 0 && MR <= CAGRA_NARROW_3_MAX_MR) ? 3 : 2;
}

template <int ELEM, int MR, int CR, int KIND, bool SHORT = false>
__global__ void __launch_bounds__(kWave, (min_waves<ELEM, MR, CR, SHORT>()))
search_single_kernel(const SearchParams P)
{
    CAGRA_LDS_VIEWS
    uint32_t *table = reinterpret_cast<uint32_t *>(smem);
    for (;;) {
        // persistent scheduling: next query
        uint32_t qi = 0;
        if (lane == 0) qi = atomicAdd(P.counter, 1u);
        qi = __builtin_amdgcn_readfirstlane(qi);
        if ((int64_t)qi >= P.B) break;
        uint32_t thi[MR], tlo[MR];
        QueryStats qs;
#ifdef CAGRA_PHASE_CLOCKS
        if (lane == 0 && qi < 131072u) g_query_times[2 * qi] = wall_clock64();
#endif
        search_body<MR, CR, KIND, rows_in_flight_single<ELEM, MR, CR, SHORT>()>(P, qi, 0, table, qlds, newid, newdist, parents, slot_parent, slot_nbr,
                                   thi, tlo, qs);
        write_result<MR>(P, qi, thi, tlo);
#ifdef CAGRA_PHASE_CLOCKS
        if (lane == 0 && qi < 131072u) g_query_times[2 * qi + 1] = wall_clock64();
#endif
        if (P.stats != nullptr && lane == 0) {
            uint32_t *s = P.stats + (size_t)qi * 4;
            s[0] = qs.n_iter; s[1] = qs.n_parent; s[2] = qs.n_dist; s[3] = qs.flags;
        }
        __syncthreads();
    }
}

// Single mode with more than 256 candidates per pass (search_body_wide).
template <int ELEM, int MR, int KIND>
__global__ void __launch_bounds__(kWave, (min_waves<ELEM, MR>()))
search_single_wide_kernel(const SearchParams P)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *qlds = reinterpret_cast<float *>(smem + P.off_query);
    uint32_t *newid = reinterpret_cast<uint32_t *>(smem + P.off_newid);
    float *newdist = reinterpret_cast<float *>(smem + P.off_newdist);
    uint32_t *parents = reinterpret_cast<uint32_t *>(smem + P.off_parents);
    uint32_t *table = reinterpret_cast<uint32_t *>(smem);
    const int lane = lane_id();
    for (;;) {
        uint32_t qi = 0;
        if (lane == 0) qi = atomicAdd(P.counter, 1u);
        qi = __builtin_amdgcn_readfirstlane(qi);
        if ((int64_t)qi >= P.B) break;
        uint32_t thi[MR], tlo[MR];
        QueryStats qs;
#ifdef CAGRA_PHASE_CLOCKS
        if (lane == 0 && qi < 131072u) g_query_times[2 * qi] = wall_clock64();
#endif
        search_body_wide<MR, KIND, rows_in_flight_wide<ELEM, MR>()>(P, qi, table, qlds, newid, newdist, parents, thi, tlo, qs);
        write_result<MR>(P, qi, thi, tlo);
#ifdef CAGRA_PHASE_CLOCKS
        if (lane == 0 && qi < 131072u) g_query_times[2 * qi + 1] = wall_clock64();
#endif
        if (P.stats != nullptr && lane == 0) {
            uint32_t *s = P.stats + (size_t)qi * 4;
            s[0] = qs.n_iter; s[1] = qs.n_parent; s[2] = qs.n_dist; s[3] = qs.flags;
        }
        __syncthreads();
    }
}

// Single mode with a team of NW wavefronts per query (search_body_team).  Workgroups are persistent and
// take queries from the device counter like the one-wavefront kernels.
template <int ELEM, int MR, int NW>
__global__ void __launch_bounds__(kWave * NW)
search_team_kernel(const SearchParams P)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    uint32_t *table = reinterpret_cast<uint32_t *>(smem);
    uint32_t *team_words = reinterpret_cast<uint32_t *>(smem + P.off_team);
    float *qlds = reinterpret_cast<float *>(smem + P.off_query);
    uint32_t *newid = reinterpret_cast<uint32_t *>(smem + P.off_newid) + wave * 256;
    float *newdist = reinterpret_cast<float *>(smem + P.off_newdist) + wave * 256;
    uint32_t *parents = reinterpret_cast<uint32_t *>(smem + P.off_parents);   // one copy, written by wavefront 0
    uint32_t *pub_hi = reinterpret_cast<uint32_t *>(smem + P.off_pub);
    uint32_t *pub_lo = pub_hi + 2 * NW * P.pub_cap;
    for (;;) {
        if (threadIdx.x == 0) team_words[1] = atomicAdd(P.counter, 1u);
        __syncthreads();
        const uint32_t qi = team_words[1];
        if ((int64_t)qi >= P.B) break;
        if (threadIdx.x == 0) team_words[2] = 0u;
        uint32_t thi[MR], tlo[MR];
        QueryStats qs;
#ifdef CAGRA_PHASE_CLOCKS
        if (threadIdx.x == 0 && qi < 131072u) g_query_times[2 * qi] = wall_clock64();
#endif
        search_body_team<MR, NW>(P, qi, wave, table, team_words, qlds, newid, newdist, parents, pub_hi, pub_lo, thi, tlo, qs);
#ifdef CAGRA_PHASE_CLOCKS
        if (threadIdx.x == 0 && qi < 131072u) g_query_times[2 * qi + 1] = wall_clock64();
#endif
        if (P.stats != nullptr && lane == 0) atomicAdd(team_words + 2, qs.n_dist);
        if (wave == 0) write_result<MR>(P, qi, thi, tlo);
        __syncthreads();
        if (P.stats != nullptr && threadIdx.x == 0) {
            uint32_t *s = P.stats + (size_t)qi * 4;
            s[0] = qs.n_iter; s[1] = qs.n_parent; s[2] = team_words[2]; s[3] = qs.flags;
        }
        __syncthreads();
    }
}

// Result of a multi-mode query from the heads of its workers' lists: the lists are sorted and disjoint, so
// the first k of their union are among the first k of each.  W * k keys (at most 64 * R) are read in
// one go, sorted and the first k written; `stride` is the distance between two lists in keys.
template <int R>
__device__ __forceinline__ void result_from_heads(const SearchParams &P, uint32_t qi, const uint64_t *lists, int stride)
{
    const int lane = lane_id();
    const int heads = P.workers * P.k;
    uint32_t hi[R], lo[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int idx = r * 64 + lane;
        const int w = idx / P.k;
        const bool valid = idx < heads;
        const uint64_t key = valid ? __builtin_nontemporal_load(lists + (size_t)w * stride + (idx - w * P.k)) : 0ull;
        hi[r] = valid ? (uint32_t)(key >> 32) : kDummyHi;
        lo[r] = valid ? (uint32_t)key : kInvalidId;
    }
    bitonic_sort<R>(hi, lo, lane);
    write_result<R>(P, qi, hi, lo);
}

// What a multi-mode worker leaves in the workspace besides its list: eight words (passes, parents, distances, flags,
// four unused), summed over the workers by the last one.
constexpr int kNoteWords = 8;

// Every query has two visited tables in the workspace and a word that says which one is in use.  The workers of a
// query use that one, and each of them, before it starts, empties its share of the other one -- the table the
// previous search on this workspace filled.  The last worker to finish switches the word over and resets the
// ticket.  So a workspace that came in clean (table in use empty, ticket zero) goes out clean, the emptying is
// spread over all workers and overlaps their first memory round trip, and nothing has to be zeroed by a launch
// of its own before a call.
template <int ELEM, int MR, int CR>
__global__ void __launch_bounds__(kWave)
search_multi_kernel(const SearchParams P)
{
    CAGRA_LDS_VIEWS
    const uint32_t qi = blockIdx.x / (uint32_t)P.workers;
    const int worker = (int)(blockIdx.x - qi * (uint32_t)P.workers);
    const uint32_t in_use = __builtin_amdgcn_readfirstlane(P.which[qi]) & 1u;
    uint32_t *table = P.tables + (((size_t)qi * 2 + in_use) << P.hash_bits);
    {
        uint32_t *other = P.tables + (((size_t)qi * 2 + (in_use ^ 1u)) << P.hash_bits);
        const uint32_t words = 1u << P.hash_bits;                                       // a multiple of 1024
        const uint32_t share = ((words / 4 + (uint32_t)P.workers - 1) / (uint32_t)P.workers) * 4;
        const uint32_t lo = (uint32_t)worker * share;
        const uint32_t hi = lo + share < words ? lo + share : words;
        for (uint32_t j = lo + 4 * (uint32_t)lane; j < hi; j += 4 * kWave)
            *reinterpret_cast<uint4 *>(other + j) = make_uint4(kInvalidId, kInvalidId, kInvalidId, kInvalidId);
    }
    uint32_t *my_note = P.notes + ((size_t)qi * P.workers + worker) * kNoteWords;
    uint32_t thi[MR], tlo[MR];
    QueryStats qs;
    search_body<MR, CR, kTableGlobal, kRowsInFlightMulti>(P, qi, worker, table, qlds, newid, newdist, parents, slot_parent, slot_nbr,
                              thi, tlo, qs);
    if (lane == 0) { my_note[0] = qs.n_iter; my_note[1] = qs.n_parent; my_note[2] = qs.n_dist; my_note[3] = qs.flags; }
    // publish this worker's list, then see whether every worker of the query has done so
    uint64_t *mine = P.lists + ((size_t)qi * P.workers + worker) * (64 * MR);
#pragma unroll
    for (int r = 0; r < MR; ++r) mine[r * 64 + lane] = ((uint64_t)thi[r] << 32) | tlo[r];
    __threadfence();
    uint32_t ticket = 0;
    if (lane == 0) ticket = atomicAdd(&P.done[qi], 1u);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket != (uint32_t)P.workers - 1u) return;
    __threadfence();
    // last worker: the other table is in use from now on, the ticket starts at zero again
    if (lane == 0) { P.which[qi] = in_use ^ 1u; P.done[qi] = 0u; }
    if (P.stats != nullptr) {
        uint32_t s_iter = 0, s_parent = 0, s_dist = 0, s_flags = 0;
        const uint32_t *notes = P.notes + (size_t)qi * P.workers * kNoteWords;
        for (int w = lane; w < P.workers; w += kWave) {
            const uint32_t *h = notes + (size_t)w * kNoteWords;
            s_iter = max(s_iter, __builtin_nontemporal_load(h));
            s_parent += __builtin_nontemporal_load(h + 1);
            s_dist += __builtin_nontemporal_load(h + 2);
            s_flags |= __builtin_nontemporal_load(h + 3);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            s_iter = max(s_iter, shfl_xor_u32(s_iter, off));
            s_parent += shfl_xor_u32(s_parent, off);
            s_dist += shfl_xor_u32(s_dist, off);
            s_flags |= shfl_xor_u32(s_flags, off);
        }
        if (lane == 0) {
            uint32_t *s = P.stats + (size_t)qi * 4;
            s[0] = s_iter; s[1] = s_parent; s[2] = s_dist; s[3] = s_flags;
        }
    }
    // Few enough heads (W * k <= 1024): one sort of the first k of every list
    const int heads = P.workers * P.k;
    if (heads <= 1024) {
        const uint64_t *first = P.lists + (size_t)qi * P.workers * (64 * MR);
        if (heads <= 64) result_from_heads<1>(P, qi, first, 64 * MR);
        else if (heads <= 128) result_from_heads<2>(P, qi, first, 64 * MR);
        else if (heads <= 256) result_from_heads<4>(P, qi, first, 64 * MR);
        else if (heads <= 512) result_from_heads<8>(P, qi, first, 64 * MR);
        else result_from_heads<16>(P, qi, first, 64 * MR);
        return;
    }
    // otherwise fold the other lists into its own, one bitonic merge each; the lists are read four at a
    // time so that their latencies overlap
    constexpr int kFold = 4;
    for (int w0 = 0; w0 < P.workers; w0 += kFold) {
        uint64_t key[kFold][MR];
#pragma unroll
        for (int u = 0; u < kFold; ++u) {
            const int w = w0 + u;
            const bool take = w < P.workers && w != worker;
            const uint64_t *other = P.lists + ((size_t)qi * P.workers + (take ? w : worker)) * (64 * MR);
#pragma unroll
            for (int r = 0; r < MR; ++r) key[u][r] = __builtin_nontemporal_load(other + r * 64 + lane);
        }
#pragma unroll
        for (int u = 0; u < kFold; ++u) {
            const int w = w0 + u;
            if (w >= P.workers || w == worker) continue;
            uint32_t ohi[MR], olo[MR];
#pragma unroll
            for (int r = 0; r < MR; ++r) { ohi[r] = (uint32_t)(key[u][r] >> 32); olo[r] = (uint32_t)key[u][r]; }
            merge_into_topm<MR, MR>(thi, tlo, ohi, olo, lane);
        }
    }
    write_result<MR>(P, qi, thi, tlo);
}

template <int MR, int CR>
static hipError_t launch_single_one(const SearchParams &P, int grid, size_t smem, hipStream_t stream)
{
    launch_zero_counter(P.counter, stream);
    if constexpr (kElem == 0 && MR <= 2 && CR != 2) {
        if (P.short_rows && P.reset_interval == 0) {
            hipLaunchKernelGGL((search_single_kernel<kElem, MR, CR, kTableSets, true>), dim3(grid), dim3(kWave), smem, stream, P);
            return hipGetLastError();
        }
    }
    if (P.reset_interval > 0)
        hipLaunchKernelGGL((search_single_kernel<kElem, MR, CR, kTableReset>), dim3(grid), dim3(kWave), smem, stream, P);
    else
        hipLaunchKernelGGL((search_single_kernel<kElem, MR, CR, kTableSets>), dim3(grid), dim3(kWave), smem, stream, P);
    return hipGetLastError();
}

template <int MR>
static hipError_t launch_wide_one(const SearchParams &P, int grid, size_t smem, hipStream_t stream)
{
    launch_zero_counter(P.counter, stream);
    if (P.reset_interval > 0)
        hipLaunchKernelGGL((search_single_wide_kernel<kElem, MR, kTableReset>), dim3(grid), dim3(kWave), smem, stream, P);
    else
        hipLaunchKernelGGL((search_single_wide_kernel<kElem, MR, kTableSets>), dim3(grid), dim3(kWave), smem, stream, P);
    return hipGetLastError();
}

template <int MR, int CR>
static hipError_t launch_multi_one(const SearchParams &P, size_t smem, hipStream_t stream)
{
    if (!P.workspace_clean) launch_multi_init(P, stream);
    hipLaunchKernelGGL((search_multi_kernel<kElem, MR, CR>), dim3((unsigned)(P.B * P.workers)), dim3(kWave), smem, stream, P);
    return hipGetLastError();
}

// `grid` comes in as (workgroups per CU the caller allows) x (compute units); it is cut down to what the kernel's
// registers and LDS let reside at once, so that every workgroup of the persistent grid starts at once.
template <int MR, int NW>
static hipError_t launch_team_one(const SearchParams &P, int grid, int cus, size_t smem, hipStream_t stream)
{
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, search_team_kernel<kElem, MR, NW>, kWave * NW, smem) == hipSuccess &&
        per_cu > 0 && (int64_t)per_cu * cus < grid)
        grid = per_cu * cus;
    launch_zero_counter(P.counter, stream);
    hipLaunchKernelGGL((search_team_kernel<kElem, MR, NW>), dim3(grid), dim3(kWave * NW), smem, stream, P);
    return hipGetLastError();
}

#define CAGRA_CAT_(a, b) a##b
#define CAGRA_CAT(a, b) CAGRA_CAT_(a, b)
#define CAGRA_DISPATCH(FN, ...)                                                          \
    switch (mr * 8 + cr) {                                                               \
        case 1 * 8 + 1: return FN<1, 1>(__VA_ARGS__);                                    \
        case 1 * 8 + 2: return FN<1, 2>(__VA_ARGS__);                                    \
        case 1 * 8 + 4: return FN<1, 4>(__VA_ARGS__);                                    \
        case 2 * 8 + 1: return FN<2, 1>(__VA_ARGS__);                                    \
        case 2 * 8 + 2: return FN<2, 2>(__VA_ARGS__);                                    \
        case 2 * 8 + 4: return FN<2, 4>(__VA_ARGS__);                                    \
        case 4 * 8 + 1: return FN<4, 1>(__VA_ARGS__);                                    \
        case 4 * 8 + 2: return FN<4, 2>(__VA_ARGS__);                                    \
        case 4 * 8 + 4: return FN<4, 4>(__VA_ARGS__);                                    \
        case 8 * 8 + 1: return FN<8, 1>(__VA_ARGS__);                                    \
        case 8 * 8 + 2: return FN<8, 2>(__VA_ARGS__);                                    \
        case 8 * 8 + 4: return FN<8, 4>(__VA_ARGS__);                                    \
    }                                                                                    \
    return hipErrorInvalidValue;

hipError_t CAGRA_CAT(launch_search_single_, CAGRA_ELEM_NAME)(const SearchParams &P, int mr, int cr, int grid, size_t smem, hipStream_t stream)
{
    CAGRA_DISPATCH(launch_single_one, P, grid, smem, stream)
}

hipError_t CAGRA_CAT(launch_search_multi_, CAGRA_ELEM_NAME)(const SearchParams &P, int mr, int cr, size_t smem, hipStream_t stream)
{
    CAGRA_DISPATCH(launch_multi_one, P, smem, stream)
}

hipError_t CAGRA_CAT(launch_search_wide_, CAGRA_ELEM_NAME)(const SearchParams &P, int mr, int grid, size_t smem, hipStream_t stream)
{
    switch (mr) {
        case 1: return launch_wide_one<1>(P, grid, smem, stream);
        case 2: return launch_wide_one<2>(P, grid, smem, stream);
        case 4: return launch_wide_one<4>(P, grid, smem, stream);
        case 8: return launch_wide_one<8>(P, grid, smem, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t CAGRA_CAT(launch_search_team_, CAGRA_ELEM_NAME)(const SearchParams &P, int mr, int waves, int grid, int cus, size_t smem, hipStream_t stream)
{
    switch (mr * 8 + waves) {
        case 1 * 8 + 2: return launch_team_one<1, 2>(P, grid, cus, smem, stream);
        case 2 * 8 + 2: return launch_team_one<2, 2>(P, grid, cus, smem, stream);
        case 4 * 8 + 2: return launch_team_one<4, 2>(P, grid, cus, smem, stream);
        case 8 * 8 + 2: return launch_team_one<8, 2>(P, grid, cus, smem, stream);
        case 1 * 8 + 4: return launch_team_one<1, 4>(P, grid, cus, smem, stream);
        case 2 * 8 + 4: return launch_team_one<2, 4>(P, grid, cus, smem, stream);
        case 4 * 8 + 4: return launch_team_one<4, 4>(P, grid, cus, smem, stream);
        case 8 * 8 + 4: return launch_team_one<8, 4>(P, grid, cus, smem, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace cagra

#ifdef CAGRA_PHASE_CLOCKS
// Start and end wall clock (100 MHz) of the first n queries of the last single-mode launch.
extern "C" int CAGRA_CAT(cagra_debug_query_times_, CAGRA_ELEM_NAME)(unsigned long long *out_host, int n)
{
    if (hipDeviceSynchronize() != hipSuccess || n < 0 || n > 131072) return -1;
    return hipMemcpyFromSymbol(out_host, HIP_SYMBOL(cagra::g_query_times), sizeof(unsigned long long) * 2 * n) == hipSuccess ? 0 : -1;
}

// Reads (and optionally clears) the phase timers of this storage type's kernels; synchronises the device.
extern "C" int CAGRA_CAT(cagra_debug_phase_clocks_, CAGRA_ELEM_NAME)(unsigned long long *out_host, int clear)
{
    if (hipDeviceSynchronize() != hipSuccess) return -1;
    if (out_host && hipMemcpyFromSymbol(out_host, HIP_SYMBOL(cagra::g_phase_clocks), sizeof(unsigned long long) * 8) != hipSuccess) return -1;
    if (clear) {
        unsigned long long z[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (hipMemcpyToSymbol(HIP_SYMBOL(cagra::g_phase_clocks), z, sizeof(z)) != hipSuccess) return -1;
    }
    return 0;
}
#endif
