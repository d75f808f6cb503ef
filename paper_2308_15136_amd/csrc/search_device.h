// Device code shared by the search kernels: 64-bit (distance, id) keys held in register
// pairs, wavefront-wide bitonic sort / merge (Sec. IV-B.2), the LDS visited table
// (Sec. IV-B.3).  Element e of a list lives in lane e % 64, register e / 64.
#pragma once
#include "device_util.h"

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

// Ordered insertion of one key (wavefront-uniform) into the sorted list t: entries from its
// position on move up by one element (one lane to the right, lane 63 into lane 0 of the next
// register), the last element of the list falls off.
// Returns the position the key went to.
template <int MR>
__device__ __forceinline__ int insert_into_topm(uint32_t (&thi)[MR], uint32_t (&tlo)[MR],
                                                uint32_t khi, uint32_t klo, int lane)
{
    int pos = 0;   // entries smaller than the key form a prefix of the sorted list
#pragma unroll
    for (int r = 0; r < MR; ++r) pos += __popcll(__ballot(key_less(thi[r], tlo[r], khi, klo)));
#pragma unroll
    for (int r = MR - 1; r >= 0; --r) {
        if ((r + 1) * kWave <= pos) continue;   // registers wholly below the position stay as they are
        // what arrives in lane 0: the last element of the register below (untouched so far)
        const uint32_t carry_hi = r > 0 ? __builtin_amdgcn_readlane(thi[r > 0 ? r - 1 : 0], 63) : 0u;
        const uint32_t carry_lo = r > 0 ? __builtin_amdgcn_readlane(tlo[r > 0 ? r - 1 : 0], 63) : 0u;
        // DPP wave_shr:1 -- lane i takes lane i-1, lane 0 keeps `old` (the carry)
        const uint32_t up_hi = (uint32_t)__builtin_amdgcn_update_dpp((int)carry_hi, (int)thi[r], 0x138, 0xF, 0xF, false);
        const uint32_t up_lo = (uint32_t)__builtin_amdgcn_update_dpp((int)carry_lo, (int)tlo[r], 0x138, 0xF, 0xF, false);
        const int e = r * 64 + lane;
        thi[r] = e > pos ? up_hi : (e == pos ? khi : thi[r]);
        tlo[r] = e > pos ? up_lo : (e == pos ? klo : tlo[r]);
    }
    return pos;
}

// Lane i takes the value of lane i - 1, lane 0 that of lane 63 (DPP wave_ror:1).
__device__ __forceinline__ uint32_t wave_rotate1(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x13C, 0xF, 0xF, false);
}

// Turns into dummies (a) every candidate whose node is already in the list t and (b) all but the
// first (lowest element index) of candidates that name the same node.  Every candidate travels
// once around the wavefront and is compared with what each lane holds.  The slow, complete
// check: used only in a pass in which the visited table lost an id it had just taken (see
// visited_insert_sets).
template <int MR, int CR>
__device__ __forceinline__ void drop_duplicates(const uint32_t (&tlo)[MR], uint32_t (&chi)[CR], uint32_t (&clo)[CR], int lane)
{
    uint32_t rid[CR];                 // travelling node ids (0x7FFFFFFF for a dummy: no node has it)
    uint32_t dup = 0;                 // bit r: the travelling candidate of register r is a duplicate
    uint32_t home = (uint32_t)lane;   // lane the travelling candidates belong to
#pragma unroll
    for (int r = 0; r < CR; ++r) rid[r] = clo[r] >> 1;
    for (int step = 0; step < kWave; ++step) {
#pragma unroll
        for (int r = 0; r < CR; ++r) {
            bool m = false;
#pragma unroll
            for (int t = 0; t < MR; ++t) m |= (tlo[t] >> 1) == rid[r];
#pragma unroll
            for (int r2 = 0; r2 < CR; ++r2)
                m |= ((clo[r2] >> 1) == rid[r]) & ((uint32_t)(r2 * kWave + lane) < (uint32_t)r * kWave + home);
            dup |= m ? (1u << r) : 0u;
        }
#pragma unroll
        for (int r = 0; r < CR; ++r) rid[r] = wave_rotate1(rid[r]);
        dup = wave_rotate1(dup);
        home = wave_rotate1(home);
    }
    // after 64 rotations every candidate is back in its own lane
#pragma unroll
    for (int r = 0; r < CR; ++r)
        if (dup & (1u << r)) { chi[r] = kDummyHi; clo[r] = kInvalidId; }
}

// at most this many winning candidates are inserted one by one; more go through sort + merge
#ifndef CAGRA_INSERT_LIMIT
#define CAGRA_INSERT_LIMIT 8
#endif
constexpr int kInsertLimit = CAGRA_INSERT_LIMIT;

// Step 1 (Sec. IV-A): the sorted list t of logical length `length` (its registers are padded to a
// power of two with dummies) takes in the candidates c.  Skipped when no candidate beats the last
// entry.  With DEDUP (a visited table that may forget) candidates that repeat a list member or each
// other are dropped first; `lost` / `forgot` are the table's flags (see sets_insert, sets_confirm).
// scratch_id / scratch_key: 64 * CR words of LDS each, free at this point.
// `lead` is the caller's count of leading entries known to carry the parent flag; it is lowered to
// the first position a candidate (which has no flag) went to.
template <int MR, int CR, bool DEDUP>
__device__ __forceinline__ void update_topm(uint32_t (&thi)[MR], uint32_t (&tlo)[MR], uint32_t (&chi)[CR],
                                            uint32_t (&clo)[CR], int length, bool lost, bool forgot,
                                            uint32_t *scratch_id, float *scratch_key, int lane, int &lead)
{
    const int last = length - 1;
    // key of the last logical entry
    uint32_t whi = kDummyHi, wlo = kInvalidId;
#pragma unroll
    for (int r = 0; r < MR; ++r)
        if (r == (last >> 6)) {
            whi = __builtin_amdgcn_readlane(thi[r], last & 63);
            wlo = __builtin_amdgcn_readlane(tlo[r], last & 63);
        }
    uint64_t better[CR];
    int n_better = 0;
#pragma unroll
    for (int r = 0; r < CR; ++r) {
        better[r] = __ballot(key_less(chi[r], clo[r], whi, wlo));
        n_better += __popcll(better[r]);
    }
    if constexpr (DEDUP) {
        // The table only filters: where it may have let a node through twice, winners are checked
        // before they enter the list (a node that is measured again has the same key, so only a
        // winner can be a copy of a list member).
        if (n_better != 0 && __ballot(lost) != 0ull) {
            drop_duplicates<MR, CR>(tlo, chi, clo, lane);
            n_better = 0;
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                better[r] = __ballot(key_less(chi[r], clo[r], whi, wlo));
                n_better += __popcll(better[r]);
            }
        } else if (n_better != 0 && __ballot(forgot) != 0ull) {
#pragma unroll
            for (int r = 0; r < CR; ++r) {
                uint64_t m = better[r];
                while (m != 0ull) {
                    const int l = __builtin_ctzll(m);
                    m &= m - 1;
                    const uint32_t id = __builtin_amdgcn_readlane(clo[r], l) >> 1;
                    bool same = false;
#pragma unroll
                    for (int t2 = 0; t2 < MR; ++t2) same |= (tlo[t2] >> 1) == id;
                    if (__ballot(same) != 0ull) {
                        if (lane == l) { chi[r] = kDummyHi; clo[r] = kInvalidId; }
                        better[r] &= ~(1ull << l);
                        --n_better;
                    }
                }
            }
        }
    }
    if (n_better == 0) return;
    if (n_better <= kInsertLimit) {
        // few winners (the usual case once the list has settled): one ordered insertion each
        // instead of the sorting network
#pragma unroll
        for (int r = 0; r < CR; ++r) {
            uint64_t m = better[r];
            while (m != 0ull) {
                const int l = __builtin_ctzll(m);
                m &= m - 1;
                const int pos = insert_into_topm<MR>(thi, tlo, __builtin_amdgcn_readlane(chi[r], l),
                                                     __builtin_amdgcn_readlane(clo[r], l), lane);
                lead = pos < lead ? pos : lead;
            }
        }
    } else if (CR > 1 && n_better <= kWave) {
        lead = 0;
        // the winners fit one register: gather them through LDS, sort 64 keys instead of 64 * CR
        int before = 0;
#pragma unroll
        for (int r = 0; r < CR; ++r) {
            const uint64_t m = better[r];
            const int pos = before + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                         __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            if ((m >> lane) & 1ull) { scratch_id[pos] = clo[r]; scratch_key[pos] = __uint_as_float(chi[r]); }
            before += __popcll(m);
        }
        wave_sync();
        uint32_t whi1[1], wlo1[1];
        whi1[0] = lane < n_better ? __float_as_uint(scratch_key[lane]) : kDummyHi;
        wlo1[0] = lane < n_better ? scratch_id[lane] : kInvalidId;
        wave_sync();
        bitonic_sort<1>(whi1, wlo1, lane);
        merge_into_topm<MR, 1>(thi, tlo, whi1, wlo1, lane);
    } else {
        lead = 0;
        bitonic_sort<CR>(chi, clo, lane);
        merge_into_topm<MR, CR>(thi, tlo, chi, clo, lane);
    }
    // logical length: whatever lies beyond it is padding and stays dummy
#pragma unroll
    for (int r = 0; r < MR; ++r)
        if (r * 64 + lane >= length) { thi[r] = kDummyHi; tlo[r] = kInvalidId; }
}

// ---- visited table (Sec. IV-B.3) -------------------------------------------------------------

__device__ __forceinline__ uint32_t hash_slot(uint32_t id, int bits)
{
    return (id * 2654435761u) >> (32 - bits);
}

// Slot of id in a table of `words` entries (any size): multiplicative hash scaled by multiply-shift.
__device__ __forceinline__ uint32_t hash_slot_words(uint32_t id, uint32_t words)
{
    return (uint32_t)(((uint64_t)(id * 2654435761u) * words) >> 32);
}

// LDS table of `words` ids, linear probing.  true if id was not in the table (and is now).
// `overflow` is raised if no free slot exists.
__device__ __forceinline__ bool visited_insert(uint32_t *table, uint32_t words, uint32_t id, bool &overflow)
{
    uint32_t s = hash_slot_words(id, words);
    for (uint32_t probe = 0; probe < words; ++probe) {
        uint32_t old = atomicCAS(&table[s], kInvalidId, id);
        if (old == kInvalidId) return true;
        if (old == id) return false;
        s = s + 1 == words ? 0u : s + 1;
    }
    overflow = true;
    return true;
}

// LDS table organised as sets of four ids (one 16-byte read tests a node) in which a new id
// replaces the oldest of its set: forgetting by replacement instead of the periodic reset of
// Sec. IV-B.3.  `cursor` holds one byte per set, four sets per word, counting the set's
// insertions; a byte that wraps carries into its neighbour, which only shifts that set's
// replacement order.  The table never reports an unseen node as seen.  It may forget a node,
// also one that is still in the top-M list; the two flags tell the caller when list entry has
// to look for duplicates:
//   forgot -- an id that the table held was overwritten (by this lane): from now on a candidate
//             may be a node that is already in the list;
//   lost   -- this lane's own id did not survive the insertions of the same pass (five or more
//             of them hit one set): candidates of this pass may repeat each other unnoticed.
// Keeps the compiler from moving or merging LDS accesses across this point (the hardware runs
// one wavefront's LDS instructions in order).
__device__ __forceinline__ void lds_order() { __asm__ volatile("" ::: "memory"); }

// A pass tests all its candidates first, then inserts the missing ones, then reads the sets
// again: lanes that inserted the same id all found it missing, and only the copy in the lowest
// way counts as new.  All lanes call these together; `valid` lanes take part.
__device__ __forceinline__ bool sets_lookup(const uint32_t *table, uint32_t sets, uint32_t id, bool valid, uint32_t &set)
{
    set = valid ? hash_slot_words(id, sets) : 0u;
    const uint4 e = *reinterpret_cast<const uint4 *>(table + 4 * set);
    return valid && !(e.x == id || e.y == id || e.z == id || e.w == id);   // true: not in the table
}

// returns the set's insertion count before this one; the id goes to way count & 3
__device__ __forceinline__ uint32_t sets_insert(uint32_t *table, uint32_t *cursor, uint32_t set, uint32_t id, bool &forgot)
{
    const uint32_t sh = 8u * (set & 3u);
    const uint32_t count = (atomicAdd(&cursor[set >> 2], 1u << sh) >> sh) & 0xFFu;
    forgot |= count >= 4u;
    table[4 * set + (count & 3u)] = id;
    return count;
}

// true if this lane's insertion makes its id a new node.  SHARED: the table is shared by several wavefronts,
// whose writes land in no particular order (an older count's id may replace a newer one's): the lane also checks
// that its own id is still in its way.
template <bool SHARED = false>
__device__ __forceinline__ bool sets_confirm(const uint32_t *table, const uint32_t *cursor, uint32_t set, uint32_t count,
                                             uint32_t id, bool &forgot, bool &lost)
{
    const uint4 f = *reinterpret_cast<const uint4 *>(table + 4 * set);
    const uint32_t now = (cursor[set >> 2] >> (8u * (set & 3u))) & 0xFFu;
    const uint32_t way = count & 3u;
    const uint32_t fw[4] = {f.x, f.y, f.z, f.w};
    bool gone = ((now - count) & 0xFFu) > 4u;   // four or more insertions into this set came after this lane's
    if constexpr (SHARED) {
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) gone |= (k == way) & (fw[k] != id);
    }
    if (gone) {
        // this lane's way was written again
        lost = true;
        forgot = true;
        return true;
    }
    bool lower = false;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) lower |= (k < way) & (fw[k] == id);
    return !lower;
}

}  // namespace cagra
