// Second pass of Split-K (Algorithm 1, Phase 3): C = sum_{i<S} C_i element by
// element in FP32, i ascending, then one round-to-nearest-even cast to FP16 (or
// to bfloat16, for bfloat16 activations).
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {


// One thread owns four consecutive columns of one row (N % 8 == 0 keeps the
// 16-byte loads aligned and inside the row).
template <typename Act>
__global__ __launch_bounds__(256) void reduce_kernel(const float *__restrict__ partials, int S, size_t MN,
                                                    uint16_t *__restrict__ Y)
{
    const size_t i4 = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i4 >= MN) return;
    float4_t acc = *reinterpret_cast<const float4_t *>(partials + i4);
    int s = 1;
    for (; s + 8 <= S; s += 8) {  // eight independent loads in flight, added in slice order
        float4_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = *reinterpret_cast<const float4_t *>(partials + (size_t)(s + e) * MN + i4);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += v[e];
    }
    for (; s < S; ++s) acc += *reinterpret_cast<const float4_t *>(partials + (size_t)s * MN + i4);
    *reinterpret_cast<uint2_t *>(Y + i4) = (uint2_t){Act::pack2(acc[0], acc[1]), Act::pack2(acc[2], acc[3])};
}

// Clears n words of a fixed-point accumulator (a fill kernel, so that a caller may capture it in a HIP graph).
__global__ __launch_bounds__(256) void clear_kernel(unsigned long long *p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

}  // namespace

hipError_t launch_accumulator_clear(unsigned long long *acc, size_t n, hipStream_t stream)
{
    hipLaunchKernelGGL(clear_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, acc, n);
    return hipGetLastError();
}

hipError_t launch_reduce(const float *partials, int S, int M, int N, uint16_t *Y, bool bf16, hipStream_t stream)
{
    const size_t MN = (size_t)M * N;
    const unsigned blocks = (unsigned)((MN / 4 + 255) / 256);
    if (bf16)
        hipLaunchKernelGGL(reduce_kernel<ActBF16>, dim3(blocks), dim3(256), 0, stream, partials, S, MN, Y);
    else
        hipLaunchKernelGGL(reduce_kernel<ActF16>, dim3(blocks), dim3(256), 0, stream, partials, S, MN, Y);
    return hipGetLastError();
}

}  // namespace w4a16
