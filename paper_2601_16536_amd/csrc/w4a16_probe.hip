// Measurement aid, not a step of the method: reads what one multiply reads (packed weights, scales, zero points) once,
// with the kernels' own 16-byte nontemporal buffer loads, and does nothing with it.  Its time is the practical
// ceiling that the benchmark prints beside a multiply's time (the roofline stays the published peak).
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

constexpr int kThreads = 512;
constexpr int kInFlight = 4;  // 16-byte loads per thread in flight

// One array of `pieces` 16-byte pieces, read in the order of the grid: consecutive lanes on consecutive pieces,
// consecutive workgroups on consecutive 8 KiB, the whole grid one stride further per round.
__device__ __forceinline__ uint4_t read_all(const void *p, unsigned long long bytes, uint4_t acc)
{
    const unsigned long long pieces = bytes >> 4;
    const unsigned long long stride = (unsigned long long)gridDim.x * kThreads;
    const uint4_t *src = static_cast<const uint4_t *>(p);
    for (unsigned long long i = (unsigned long long)blockIdx.x * kThreads + threadIdx.x; i < pieces; i += kInFlight * stride) {
        uint4_t v[kInFlight];
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) {
            const unsigned long long e = i + q * stride;
            v[q] = e < pieces ? __builtin_nontemporal_load(src + e) : (uint4_t){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) acc ^= v[q];
    }
    return acc;
}

__global__ __launch_bounds__(kThreads) void stream_probe_kernel(const void *a, unsigned long long na, const void *b, unsigned long long nb,
                                                               const void *c, unsigned long long nc, uint32_t *sink)
{
    uint4_t acc = {0u, 0u, 0u, 0u};
    if (a) acc = read_all(a, na, acc);
    if (b) acc = read_all(b, nb, acc);
    if (c) acc = read_all(c, nc, acc);
    // keeps the loads alive; a store happens only if every word read cancels to this one pattern
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u && (acc[0] & acc[1]) == 0x7F4A7C15u) sink[0] = acc[2];
}

}  // namespace

hipError_t launch_stream_probe(const void *a, size_t na, const void *b, size_t nb, const void *c, size_t nc, uint32_t *sink, int cus,
                               hipStream_t stream)
{
    hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)cus), dim3(kThreads), 0, stream, a, (unsigned long long)na, b,
                       (unsigned long long)nb, c, (unsigned long long)nc, sink);
    return hipGetLastError();
}

}  // namespace w4a16
