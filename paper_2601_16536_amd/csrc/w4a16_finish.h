// How a workgroup's waves, and then the K slices of different workgroups, meet
// (Algorithm 1, Phase 3: C = sum_i C_i, then the cast to FP16).  Shared by the
// STRIPE and TILE families.
#pragma once
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {

// Fixed-point form of a slice sum for the cross-workgroup accumulator: the value
// in units of 2^-24 (clamped far outside the FP16 range), biased to be positive,
// in bits 0-55; one arrival in bits 56-63.  Up to 255 slices cannot carry into
// the count.
constexpr float kFixScale = 16777216.0f;            // 2^24
constexpr float kFixClamp = 2097152.0f;             // 2^21
constexpr unsigned long long kFixBias = 1ull << 46;
constexpr unsigned long long kFixOne = 1ull << 56;

__device__ __forceinline__ unsigned long long to_fixed(float v)
{
    v = fminf(fmaxf(v, -kFixClamp), kFixClamp);
    const long long fx = (long long)__builtin_rintf(v * kFixScale);  // |v| <= 2^21: the product is exact, |fx| <= 2^45
    return (unsigned long long)(fx + (long long)kFixBias) + kFixOne;
}

__device__ __forceinline__ float from_fixed(unsigned long long total)
{
    const unsigned long long cnt = total >> 56;
    const long long fx = (long long)(total & (kFixOne - 1)) - (long long)(cnt * kFixBias);
    return (float)((double)fx * (1.0 / 16777216.0));
}

// Sum of the waves' result tiles (ROWS x COLS each) in wave order, `red_waves` waves per round through
// LDS (red[wave in round][row][column]; `write_mine` puts the calling wave's tile there as float4
// groups), then the workgroup's finish.  A thread owns groups of VW neighbouring columns of one row;
// the atomic finish wants VW = 1 (consecutive lanes on consecutive outputs, four cache lines per
// wave-wide atomic), the others VW = 4.  `sync` is the accumulator [M, N] (64-bit words, all zero
// before the launch and left zero by it).
template <int ROWS, int COLS, int VW, int MIN_WAVES, typename WriteMine>
__device__ __forceinline__ void reduce_and_finish(const GemmArgs &a, const int finish, unsigned long long *__restrict__ sync, unsigned char *smem,
                                                  const WriteMine &write_mine, int red_waves, int row0, int col0, int slice)
{
    typedef float vec_t __attribute__((ext_vector_type(VW)));
    constexpr int kGroups = ROWS * COLS / VW;
    constexpr int kOwn = (kGroups + 64 * MIN_WAVES - 1) / (64 * MIN_WAVES);  // groups per thread, at most
    const int tid = threadIdx.x, wave = tid >> 6, waves = blockDim.x >> 6;
    vec_t v[kOwn];
#pragma unroll
    for (int k = 0; k < kOwn; ++k) v[k] = vec_t(0.f);
    const vec_t *red = reinterpret_cast<const vec_t *>(smem);
    for (int w0 = 0; w0 < waves; w0 += red_waves) {
        __syncthreads();  // the staged X (first round) or the previous round's sums are no longer needed
        if (wave >= w0 && wave < w0 + red_waves)
            write_mine(reinterpret_cast<float4_t *>(smem) + (size_t)(wave - w0) * (ROWS * COLS / 4));
        __syncthreads();
        const int nw = waves - w0 < red_waves ? waves - w0 : red_waves;
#pragma unroll
        for (int k = 0; k < kOwn; ++k) {
            if (k * (int)blockDim.x >= kGroups) continue;  // uniform: no thread owns a k-th group
            const int o = tid + k * (int)blockDim.x;
            const int oc = o < kGroups ? o : 0;  // threads past the last group read group 0 and store nothing
            // four reads in flight at a time (past the last wave the last one is read again and not added)
            for (int w = 0; w < nw; w += 4) {
                vec_t t0 = red[(size_t)w * kGroups + oc];
                vec_t t1 = red[(size_t)(w + 1 < nw ? w + 1 : nw - 1) * kGroups + oc];
                vec_t t2 = red[(size_t)(w + 2 < nw ? w + 2 : nw - 1) * kGroups + oc];
                vec_t t3 = red[(size_t)(w + 3 < nw ? w + 3 : nw - 1) * kGroups + oc];
                v[k] += t0;
                if (w + 1 < nw) v[k] += t1;
                if (w + 2 < nw) v[k] += t2;
                if (w + 3 < nw) v[k] += t3;
            }
        }
    }
#pragma unroll
    for (int k = 0; k < kOwn; ++k) {
        const int o = tid + k * (int)blockDim.x;
        const int m = row0 + o / (COLS / VW), col = col0 + VW * (o % (COLS / VW));
        if (o >= kGroups || m >= a.M || col >= a.N) continue;
        const size_t out = (size_t)m * a.N + col;
        if constexpr (VW == 4) {
            if (finish == kFinishDirect)
                *reinterpret_cast<uint2_t *>(a.Y + out) = (uint2_t){pack_half2(v[k][0], v[k][1]), pack_half2(v[k][2], v[k][3])};
            else
                *reinterpret_cast<float4_t *>(a.partials + (size_t)slice * a.M * a.N + out) = v[k];
        } else {
            const unsigned long long add = to_fixed(v[k][0]);
            const unsigned long long total = __hip_atomic_fetch_add(sync + out, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
            if ((total >> 56) == (unsigned long long)a.split) {
                a.Y[out] = (uint16_t)(pack_half2(from_fixed(total), 0.f) & 0xFFFFu);
                __hip_atomic_store(sync + out, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

}  // namespace w4a16
