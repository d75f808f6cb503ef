// Device-side helpers shared by the gfx950 kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace cagra {

constexpr int kWave = 64;                      // CDNA wavefront width
constexpr uint32_t kInvalidId = 0xFFFFFFFFu;
constexpr uint32_t kFltMaxBits = 0x7F7FFFFFu;  // bit pattern of FLT_MAX

// fp32 -> unsigned integer with the same order (and back).  -0 is folded into
// +0 first so that equal distances always have equal keys.
__device__ __forceinline__ uint32_t f32_to_ordered(float f)
{
    uint32_t u = __float_as_uint(f + 0.0f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_f32(uint32_t u)
{
    return __uint_as_float(u ^ (((u >> 31) - 1u) | 0x80000000u));
}
constexpr uint32_t kDummyHi = kFltMaxBits ^ 0x80000000u;  // ordered(FLT_MAX)

// SplitMix64 output function; the step-0 seed of (query, slot) is two rounds of
// it, scaled to [0, N) by a multiply-shift (Sec. IV-A step 0 only asks for "a
// pseudo-random number generator").
__host__ __device__ __forceinline__ uint64_t splitmix_fin(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ uint64_t seed_query_hash(uint64_t seed, uint64_t query)
{
    return splitmix_fin(seed + 0x9E3779B97F4A7C15ull * (query + 1));
}
__host__ __device__ __forceinline__ uint32_t seed_slot_id(uint64_t qhash, uint64_t slot, uint64_t N)
{
    uint64_t h = splitmix_fin(qhash + 0x9E3779B97F4A7C15ull * (slot + 1));
    return (uint32_t)(((h >> 32) * N) >> 32);
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Orders the LDS accesses of ONE wavefront: what lanes wrote before this point, other lanes of the same
// wavefront read after it.  The hardware executes a wavefront's LDS instructions in order, so this only
// has to keep the compiler from moving accesses across it; no barrier instruction, and wavefronts of the
// same workgroup may pass it any number of times independently of each other.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint32_t shfl_xor_u32(uint32_t v, int mask)
{
    return (uint32_t)__shfl_xor((int)v, mask, kWave);
}
__device__ __forceinline__ uint32_t shfl_u32(uint32_t v, int src)
{
    return (uint32_t)__shfl((int)v, src, kWave);
}

// Value of `v` in another lane of the same 16-lane row, by a DPP move (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7 - i within each group of 8
constexpr int kDppMirror = 0x140;       // lane i <-> 15 - i within each row of 16

// Sum over the 2^team_log2 lanes of a team (teams are aligned groups of 4, 8, 16 or 32 lanes;
// Sec. IV-B.1).  Each step adds the partial sum of the other half; after the first two steps
// all lanes of a quad agree, so mirrored partners serve as well as xor partners.
__device__ __forceinline__ float team_sum(float v, int team_log2)
{
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    if (team_log2 >= 3) v += dpp_f32<kDppHalfMirror>(v);
    if (team_log2 >= 4) v += dpp_f32<kDppMirror>(v);
    if (team_log2 >= 5) v += __shfl_xor(v, 16, kWave);
    return v;
}

}  // namespace cagra
