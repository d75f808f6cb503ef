// Small helper kernels of the search entry points, shared by all dataset storage types, and
// the conversion of an fp32 dataset to the narrower storage types.
#include "device_util.h"
#include "search_params.h"

namespace cagra {

__global__ void zero_counter_kernel(uint32_t *counter) { *counter = 0u; }

// multi mode: both visited tables of every query empty, ticket counters zero, table 0 in use (a clean workspace;
// every search leaves the table that is in use next empty and the tickets zero)
__global__ void multi_init_kernel(uint32_t *tables, size_t table_words_total, uint32_t *done, uint32_t *which, int64_t B)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < table_words_total) tables[i] = kInvalidId;
    if (i < (size_t)B) { done[i] = 0u; which[i] = 0u; }
}

void launch_zero_counter(uint32_t *counter, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, stream, counter);
}

void launch_multi_init(const SearchParams &P, hipStream_t stream)
{
    const size_t words = (size_t)2 * P.B << P.hash_bits;
    const size_t n = words > (size_t)P.B ? words : (size_t)P.B;
    hipLaunchKernelGGL(multi_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       P.tables, words, P.done, P.which, P.B);
}

// fp32 -> fp32 (another row stride), fp16 (round to nearest even) or uint8 (round to nearest even, clamped to 0..255).
// Every destination row is written in full: the elements from `dim` to the row stride are set to zero, which is what
// the search kernels ask of a row whose width is not a whole number of 16-byte pieces.
__global__ void convert_kernel(const float *__restrict__ src, int64_t rows, int dim, int64_t ld_src,
                               int elem, void *__restrict__ dst, int64_t ld_dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * ld_dst) return;
    const int64_t r = i / ld_dst;
    const int64_t c = i - r * ld_dst;
    const float v = c < dim ? src[r * ld_src + c] : 0.f;
    if (elem == 0) {
        static_cast<float *>(dst)[i] = v;
    } else if (elem == 1) {
        static_cast<__half *>(dst)[i] = __float2half_rn(v);
    } else {
        float t = rintf(v);
        t = t < 0.f ? 0.f : (t > 255.f ? 255.f : t);
        static_cast<unsigned char *>(dst)[i] = (unsigned char)t;
    }
}

hipError_t launch_convert(const float *src, int64_t rows, int dim, int64_t ld_src, int elem, void *dst,
                          int64_t ld_dst, hipStream_t stream)
{
    const int64_t n = rows * ld_dst;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(convert_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, src, rows, dim,
                       ld_src, elem, dst, ld_dst);
    return hipGetLastError();
}

}  // namespace cagra
