// Phase 1 of Algorithm 1 alone: the INT4 weights dequantised to an FP16 matrix in
// global memory, W16[k, n] = fp16(s (q - z)) (Eq. 2).  The multiply kernels never
// materialise this matrix; it exists for the unfused variant of Section 4.2 (the
// FP16 weights take a round trip through memory before an FP16 GEMM reads them),
// which the benchmark times beside the fused path.
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));

// One thread owns one packed row (eight k) of four consecutive columns: a 16-byte
// load of codes, eight 8-byte stores.  A wave covers 256 columns, so every store
// instruction writes 512 contiguous bytes of one row of W16.
__global__ __launch_bounds__(256) void dequant_kernel(const uint32_t *__restrict__ Wp, const uint16_t *__restrict__ scales,
                                                     const uint32_t *__restrict__ Zp, int group, int N, int rows,
                                                     uint16_t *__restrict__ W16)
{
    const int quads = N >> 2;  // groups of four columns per row
    const long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (long long)rows * quads) return;
    const int r = (int)(id / quads), c4 = (int)(id % quads) * 4;
    const int g = (r * 8) / group;
    const uint4_t w = *reinterpret_cast<const uint4_t *>(Wp + (size_t)r * N + c4);
    const uint2_t sc = *reinterpret_cast<const uint2_t *>(scales + (size_t)g * N + c4);
    const uint32_t zw = (Zp ? Zp[(size_t)g * (N >> 3) + (c4 >> 3)] : 0x88888888u) >> ((c4 & 4) * 4);  // no tensor: symmetric, z = 8
    H2 s01, s23;
    s01.u = sc[0];
    s23.u = sc[1];
    const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
    int z[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) z[c] = (int)((zw >> (4 * c)) & 15u);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        half4_t h;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int q = (int)((w[c] >> (4 * i)) & 15u);
            h[c] = (_Float16)(s[c] * (float)(q - z[c]));  // the FP32 product is exact; one rounding, to nearest even
        }
        *reinterpret_cast<half4_t *>(W16 + (size_t)(r * 8 + i) * N + c4) = h;
    }
}

}  // namespace

hipError_t launch_dequant(const uint32_t *Wp, const uint16_t *scales, const uint32_t *Zp, int group, int N, int K,
                          uint16_t *W16, hipStream_t stream)
{
    const long long threads = (long long)(K / 8) * (N / 4);
    const long long blocks = (threads + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dequant_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, Wp, scales, Zp, group, N, K / 8, W16);
    return hipGetLastError();
}

}  // namespace w4a16
