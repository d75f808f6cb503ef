// Step 3b of the search (Sec. IV-B.1): distances between the query in LDS and a list of dataset
// rows, one row per team of 4/8/16/32 lanes, 16-byte loads, DPP butterfly reduction.  Shared by
// the search kernels and the NN-descent rounds of the graph build.
#pragma once
#include "device_util.h"

namespace cagra {

// storage types of dataset rows: 0 fp32, 1 fp16, 2 uint8
template <int ELEM>
__host__ __device__ constexpr int elems_per_piece() { return ELEM == 0 ? 4 : ELEM == 1 ? 8 : 16; }

// The i-th group of four consecutive elements of a 16-byte piece, widened to fp32.
template <int ELEM>
__device__ __forceinline__ float4 widen4(const uint4 &p, int i)
{
    const uint32_t w[4] = {p.x, p.y, p.z, p.w};
    if constexpr (ELEM == 0) {
        return make_float4(__uint_as_float(w[0]), __uint_as_float(w[1]), __uint_as_float(w[2]), __uint_as_float(w[3]));
    } else if constexpr (ELEM == 1) {
        const uint32_t a = w[2 * i], b = w[2 * i + 1];
        return make_float4(__half2float(__ushort_as_half((unsigned short)(a & 0xFFFFu))),
                           __half2float(__ushort_as_half((unsigned short)(a >> 16))),
                           __half2float(__ushort_as_half((unsigned short)(b & 0xFFFFu))),
                           __half2float(__ushort_as_half((unsigned short)(b >> 16))));
    } else {
        const uint32_t a = w[i];
        return make_float4((float)(a & 0xFFu), (float)((a >> 8) & 0xFFu), (float)((a >> 16) & 0xFFu), (float)(a >> 24));
    }
}

// acc += sum of (x_j - q_j)^2 over the i-th group of four elements of a 16-byte piece, one subtraction and one fused
// multiply-add per element in fp32, in order.  fp16 rows: the subtraction is written as fma(x, one, -q) with `one` a
// register that holds 1.0 but is opaque to the compiler -- the same value with the same single rounding as
// float(x) - q, but a form the hardware evaluates straight from the fp16 half of a register (v_fma_mix_f32), which
// spares the conversion: two vector instructions per element instead of three.  (The inner product needs no such
// help: fma(float(x), q, acc) is that instruction already.)
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
template <int ELEM>
__device__ __forceinline__ void l2_accumulate4(const uint4 &p, int i, const float4 &qv, float one, float &acc)
{
    if constexpr (ELEM == 1) {
        const uint32_t w[4] = {p.x, p.y, p.z, p.w};
        const half2_t a = __builtin_bit_cast(half2_t, w[2 * i]), b = __builtin_bit_cast(half2_t, w[2 * i + 1]);
        const float d0 = fmaf((float)a[0], one, 0.0f - qv.x), d1 = fmaf((float)a[1], one, 0.0f - qv.y);
        const float d2 = fmaf((float)b[0], one, 0.0f - qv.z), d3 = fmaf((float)b[1], one, 0.0f - qv.w);
        acc = fmaf(d0, d0, acc); acc = fmaf(d1, d1, acc);
        acc = fmaf(d2, d2, acc); acc = fmaf(d3, d3, acc);
    } else {
        const float4 xv = widen4<ELEM>(p, i);
        const float d0 = xv.x - qv.x, d1 = xv.y - qv.y, d2 = xv.z - qv.z, d3 = xv.w - qv.w;
        acc = fmaf(d0, d0, acc); acc = fmaf(d1, d1, acc);
        acc = fmaf(d2, d2, acc); acc = fmaf(d3, d3, acc);
    }
}

// newdist[c] = distance(query, dataset row newid[c]) for c < n_new (entries equal to kInvalidId are
// skipped).  Called by all 64 lanes of a wavefront; qlds holds the query as fp32, `ld` is the row
// stride in elements, RIF the rows each team keeps in flight (all loads of a round are issued
// before any is used).  metric 0: squared L2, else 0 - <x, q>.
template <int ELEM, int RIF, int SLOTS>
__device__ __forceinline__ void team_distances_impl(const void *dataset, int64_t ld, int dim, int metric, int team_log2,
                                                    const uint32_t *newid, int n_new, const float *qlds, float *newdist)
{
    constexpr int kPiece = elems_per_piece<ELEM>();
    constexpr int kBytes = 16 / kPiece;
    const int lane = lane_id();
    const int team = 1 << team_log2;
    const int n_teams = kWave >> team_log2;
    const int g = lane >> team_log2;       // team of this lane
    const int t = lane & (team - 1);       // lane within the team
    const int nchunk = dim / kPiece;       // 16-byte pieces per row
    float one = 1.0f;                      // see l2_accumulate4
    if constexpr (ELEM == 1) asm volatile("" : "+v"(one));
    for (int c0 = 0; c0 < n_new; c0 += RIF * n_teams) {
        const unsigned char *row[RIF];
        bool ok[RIF];
        float acc[RIF];
#pragma unroll
        for (int u = 0; u < RIF; ++u) {
            const int c = c0 + u * n_teams + g;
            const uint32_t node = c < n_new ? newid[c] : kInvalidId;
            ok[u] = node != kInvalidId;
            row[u] = static_cast<const unsigned char *>(dataset) + (size_t)(ok[u] ? node : 0u) * ld * kBytes;
            acc[u] = 0.f;
        }
        for (int base = 0; base < nchunk; base += SLOTS * team) {
            // Loads carry no per-lane predicate: a lane whose piece lies beyond the row reads the row's last piece
            // instead (its neighbours read it anyway), a team without a row reads row 0, and what they fetched is
            // never used.  A load then costs one address addition instead of a predicate, a branch and four
            // register clears, which is what the instruction stream of this loop mostly consisted of.
            int ch[SLOTS];
            bool in_row[SLOTS];
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
                ch[i] = base + i * team + t;
                in_row[i] = ch[i] < nchunk;
            }
            uint4 x[RIF][SLOTS];
#pragma unroll
            for (int u = 0; u < RIF; ++u)
#pragma unroll
                for (int i = 0; i < SLOTS; ++i)
                    x[u][i] = *reinterpret_cast<const uint4 *>(row[u] + 16 * (in_row[i] ? ch[i] : nchunk - 1));
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
                if (in_row[i]) {
#pragma unroll
                    for (int h = 0; h < kPiece / 4; ++h) {
                        const float4 qv = *reinterpret_cast<const float4 *>(qlds + kPiece * ch[i] + 4 * h);
                        if (metric == 0) {
#pragma unroll
                            for (int u = 0; u < RIF; ++u) l2_accumulate4<ELEM>(x[u][i], h, qv, one, acc[u]);
                        } else {
#pragma unroll
                            for (int u = 0; u < RIF; ++u) {
                                const float4 xv = widen4<ELEM>(x[u][i], h);
                                acc[u] = fmaf(xv.x, qv.x, acc[u]); acc[u] = fmaf(xv.y, qv.y, acc[u]);
                                acc[u] = fmaf(xv.z, qv.z, acc[u]); acc[u] = fmaf(xv.w, qv.w, acc[u]);
                            }
                        }
                    }
                }
            }
        }
        // butterfly over the team's lanes; every lane ends with the same bits
#pragma unroll
        for (int u = 0; u < RIF; ++u) acc[u] = team_sum(acc[u], team_log2);
#pragma unroll
        for (int u = 0; u < RIF; ++u) {
            if (metric != 0) acc[u] = 0.0f - acc[u];
            if (t == 0 && ok[u]) newdist[c0 + u * n_teams + g] = acc[u];
        }
    }
}

// SLOTS = 16-byte loads per lane and row in one sweep of a team over a row.  Four in general.  Byte rows are
// often so short that a team's lanes have only two pieces each (128 bytes by a team of four): then two slots
// issue no load that nobody needs.
template <int ELEM, int RIF>
__device__ __forceinline__ void team_distances(const void *dataset, int64_t ld, int dim, int metric, int team_log2,
                                               const uint32_t *newid, int n_new, const float *qlds, float *newdist)
{
    if constexpr (ELEM == 2) {
        if (dim / elems_per_piece<ELEM>() <= (2 << team_log2)) {
            team_distances_impl<ELEM, RIF, 2>(dataset, ld, dim, metric, team_log2, newid, n_new, qlds, newdist);
            return;
        }
    }
    team_distances_impl<ELEM, RIF, 4>(dataset, ld, dim, metric, team_log2, newid, n_new, qlds, newdist);
}

}  // namespace cagra
