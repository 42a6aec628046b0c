// Offline tool, not on the hot path: uniform affine quantization of FP16 weights to the
// INT4 codes, FP16 scales and INT4 zero points the multiply reads (Section 2.1, Eq. 1:
// x_q = round(x / s) + z).  The paper does not say how s and z are found; here, per
// quantisation group of one column, in FP32: lo = min(min w, 0), hi = max(max w, 0),
// s = fp16((hi - lo) / 15) (1 if that is 0), z = clamp(rint(-lo / s), 0, 15),
// q = clamp(rint(w / s) + z, 0, 15), round to nearest even.
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

// One thread owns one (group, column): consecutive lanes read consecutive columns of a row of W
// (128 contiguous bytes per wave and row), walk the group twice (range, then codes; the second
// walk hits the cache), and write one packed word per eight k.  Eight neighbouring lanes put
// their zero points together into one word.
__global__ __launch_bounds__(256) void quantize_kernel(const uint16_t *__restrict__ W16, int group, int N, long long cells,
                                                      uint32_t *__restrict__ Wp, uint16_t *__restrict__ scales,
                                                      uint32_t *__restrict__ Zp)
{
    const long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = id < cells;  // cells = groups x N, a multiple of 8: eight lanes of a zero-point word live or die together
    const long long g = live ? id / N : 0;
    const int n = live ? (int)(id - g * N) : 0;
    const _Float16 *w = reinterpret_cast<const _Float16 *>(W16) + (size_t)g * group * N + n;
    float lo = 0.f, hi = 0.f;
    for (int k = 0; k < group; ++k) {
        const float x = (float)w[(size_t)k * N];
        lo = fminf(lo, x);
        hi = fmaxf(hi, x);
    }
    _Float16 s16 = (_Float16)((hi - lo) / 15.0f);
    if (s16 == (_Float16)0.f) s16 = (_Float16)1.f;
    const float s = (float)s16;
    const float z = fminf(fmaxf(rintf(-lo / s), 0.f), 15.f);
    const int rows = group >> 3;
    for (int r = 0; r < rows; ++r) {
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float x = (float)w[(size_t)(r * 8 + i) * N];
            const float q = fminf(fmaxf(rintf(x / s) + z, 0.f), 15.f);
            word |= (uint32_t)q << (4 * i);
        }
        if (live) Wp[((size_t)g * rows + r) * N + n] = word;
    }
    uint32_t zw = (uint32_t)z << (4 * (n & 7));
    zw |= __shfl_xor(zw, 1, 64);
    zw |= __shfl_xor(zw, 2, 64);
    zw |= __shfl_xor(zw, 4, 64);
    if (live) {
        H2 b;
        b.h = (half2_t){s16, s16};
        scales[(size_t)g * N + n] = (uint16_t)(b.u & 0xFFFFu);
        if ((n & 7) == 0) Zp[(size_t)g * (N >> 3) + (n >> 3)] = zw;
    }
}

}  // namespace

hipError_t launch_quantize(const uint16_t *W16, int group, int N, int K, uint32_t *Wp, uint16_t *scales, uint32_t *Zp,
                           hipStream_t stream)
{
    const long long cells = (long long)(K / group) * N;
    const long long blocks = (cells + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, W16, group, N, cells, Wp, scales, Zp);
    return hipGetLastError();
}

}  // namespace w4a16
