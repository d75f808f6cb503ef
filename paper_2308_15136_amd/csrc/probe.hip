// Device-memory bandwidth references for the search (Sec. IV-C.1 and Sec. V name the memory
// bandwidth as the search's limiter): what this GPU delivers for (0) a plain streaming read of
// a matrix and (1) reading whole rows at random, the access pattern of the distance step of
// Sec. IV-B.1 with every dependency taken away (row ids come from a counter hash, teams of
// lanes fetch 16-byte pieces, many rows in flight per lane).  Measurement aids: they compute
// nothing of the method.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "../../include/cagra_hip.h"     // status codes
#include "../../include/cagra_probe.h"
#include "device_util.h"

namespace cagra {

__device__ __forceinline__ uint32_t fold(const uint4 &v) { return v.x ^ v.y ^ v.z ^ v.w; }

// streaming read of n16 16-byte pieces: every workgroup takes whole tiles of 32 KB (eight loads of 16 bytes
// per lane, all in flight at once), tiles handed out round-robin over the grid
__global__ void __launch_bounds__(256)
probe_stream_kernel(const uint4 *__restrict__ src, size_t n16, uint32_t *sink)
{
    constexpr size_t kTile = 256 * 8;   // pieces per tile
    const size_t n_tiles = n16 / kTile;
    uint32_t acc = 0;
    for (size_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint4 *p = src + tile * kTile + threadIdx.x;
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= fold(v[u]);
    }
    for (size_t i = n_tiles * kTile + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
        acc ^= fold(src[i]);
    if (acc == 0x9E3779B9u) *sink = acc;   // keeps the loads alive; practically never taken
}

// Random whole rows: team of 2^team_log2 lanes per row, each lane up to four 16-byte pieces of
// it, RIF rows per team in flight.  Row r of the sequence is a hash of (seed, r).
template <int RIF>
__global__ void __launch_bounds__(kWave)
probe_gather_kernel(const unsigned char *__restrict__ data, uint64_t rows, int pieces, size_t stride_bytes,
                    int team_log2, uint64_t n_read, uint64_t seed, uint32_t *sink)
{
    const int lane = lane_id();
    const int team = 1 << team_log2, n_teams = kWave >> team_log2;
    const int g = lane >> team_log2, t = lane & (team - 1);
    const uint64_t qh = seed_query_hash(seed, 0);
    const uint64_t per_round = (uint64_t)gridDim.x * n_teams * RIF;
    uint32_t acc = 0;
    for (uint64_t r0 = (uint64_t)blockIdx.x * n_teams * RIF; r0 < n_read; r0 += per_round) {
        const unsigned char *row[RIF];
        bool ok[RIF];
#pragma unroll
        for (int u = 0; u < RIF; ++u) {
            const uint64_t r = r0 + (uint64_t)u * n_teams + g;
            ok[u] = r < n_read;
            row[u] = data + (size_t)seed_slot_id(qh, r, rows) * stride_bytes;
        }
        for (int base = 0; base < pieces; base += 4 * team) {
            uint4 x[RIF][4];
#pragma unroll
            for (int u = 0; u < RIF; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int ch = base + i * team + t;
                    x[u][i] = (ok[u] && ch < pieces) ? *reinterpret_cast<const uint4 *>(row[u] + 16 * ch)
                                                     : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
            for (int u = 0; u < RIF; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc ^= fold(x[u][i]);
        }
    }
    if (acc == 0x9E3779B9u) *sink = acc;
}

}  // namespace cagra

using namespace cagra;

extern "C" int cagra_probe_bandwidth(const void *data, int64_t rows, int64_t row_bytes, int64_t stride_bytes,
                                     int32_t pattern, int64_t n_read, int32_t team_size, int32_t rows_in_flight,
                                     int32_t waves_per_cu, uint64_t seed, uint32_t *sink, void *hip_stream)
{
    if (!data || !sink) return CAGRA_ERR_NULL_POINTER;
    if (rows < 1 || rows > 0x7FFFFFFFll || row_bytes < 16 || (row_bytes & 15) || stride_bytes < row_bytes ||
        (stride_bytes & 15) || ((uintptr_t)data & 15) || n_read < 0)
        return CAGRA_ERR_BAD_SHAPE;
    if (waves_per_cu < 0 || waves_per_cu > 32) return CAGRA_ERR_BAD_OPTION;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    const int wpc = waves_per_cu == 0 ? 16 : waves_per_cu;
    if (pattern == 0) {
        if (stride_bytes != row_bytes) return CAGRA_ERR_BAD_SHAPE;   // the stream reads one dense block
        const size_t n16 = (size_t)rows * (size_t)row_bytes / 16;
        const int blocks = std::max(1, cus * wpc / 4);
        hipLaunchKernelGGL(probe_stream_kernel, dim3(blocks), dim3(256), 0, stream,
                           static_cast<const uint4 *>(data), n16, sink);
    } else if (pattern == 1) {
        if (n_read == 0) return CAGRA_OK;
        const int pieces = (int)std::min<int64_t>(row_bytes / 16, 1 << 20);
        int team = team_size;
        if (team == 0) {
            team = 4;
            while (team < 32 && (pieces + team - 1) / team > 4) team *= 2;
        }
        if (team != 4 && team != 8 && team != 16 && team != 32) return CAGRA_ERR_BAD_OPTION;
        const int team_log2 = team == 4 ? 2 : team == 8 ? 3 : team == 16 ? 4 : 5;
        const int grid = cus * wpc;
        const unsigned char *p = static_cast<const unsigned char *>(data);
        switch (rows_in_flight) {
            case 0:
            case 4:
                hipLaunchKernelGGL(probe_gather_kernel<4>, dim3(grid), dim3(kWave), 0, stream, p, (uint64_t)rows,
                                   pieces, (size_t)stride_bytes, team_log2, (uint64_t)n_read, seed, sink);
                break;
            case 2:
                hipLaunchKernelGGL(probe_gather_kernel<2>, dim3(grid), dim3(kWave), 0, stream, p, (uint64_t)rows,
                                   pieces, (size_t)stride_bytes, team_log2, (uint64_t)n_read, seed, sink);
                break;
            case 8:
                hipLaunchKernelGGL(probe_gather_kernel<8>, dim3(grid), dim3(kWave), 0, stream, p, (uint64_t)rows,
                                   pieces, (size_t)stride_bytes, team_log2, (uint64_t)n_read, seed, sink);
                break;
            default:
                return CAGRA_ERR_BAD_OPTION;
        }
    } else {
        return CAGRA_ERR_BAD_OPTION;
    }
    return hipGetLastError() == hipSuccess ? CAGRA_OK : CAGRA_ERR_LAUNCH;
}
