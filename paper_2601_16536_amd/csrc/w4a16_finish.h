// How a workgroup's waves, and then the K slices of different workgroups, meet
// (Algorithm 1, Phase 3: C = sum_i C_i, then the cast to the 16-bit output format).  Shared by the
// STRIPE and TILE families.
#pragma once
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {

// Fixed-point form of a slice sum for the cross-workgroup accumulator, one 64-bit word per output:
//   bits  0-56  the sum of the slices' values in units of 2^-24, each clamped to +-2^25 (far outside the FP16
//               range, so that slice sums of a few million that cancel each other still add up right) and
//               biased by 2^50 to be positive: 63 slices stay below 2^57;
//   bit   57    set (by an atomic OR that precedes its slice's add) when a slice sum is NaN: the result is NaN;
//   bits 58-63  arrivals: up to 63 slices.
constexpr float kFixScale = 16777216.0f;            // 2^24
constexpr float kFixClamp = 33554432.0f;            // 2^25
constexpr int kFixMaxSlices = 63;
constexpr unsigned long long kFixBias = 1ull << 50;
constexpr unsigned long long kFixPoison = 1ull << 57;
constexpr unsigned long long kFixOne = 1ull << 58;

// A slice sum that is not NaN.
__device__ __forceinline__ unsigned long long to_fixed(float v)
{
    v = fminf(fmaxf(v, -kFixClamp), kFixClamp);
    const long long fx = (long long)__builtin_rintf(v * kFixScale);  // |v| <= 2^25: the product is exact, |fx| <= 2^49
    return (unsigned long long)(fx + (long long)kFixBias) + kFixOne;
}

// The same from a sum already in units of 2^-24.
__device__ __forceinline__ unsigned long long to_fixed(long long fx)
{
    constexpr long long lim = 1ll << 49;
    fx = fx < -lim ? -lim : (fx > lim ? lim : fx);
    return (unsigned long long)(fx + (long long)kFixBias) + kFixOne;
}

__device__ __forceinline__ float from_fixed(unsigned long long total)
{
    const unsigned long long cnt = total >> 58;
    const long long fx = (long long)(total & (kFixPoison - 1)) - (long long)(cnt * kFixBias);
    return (float)((double)fx * (1.0 / 16777216.0));
}

// One slice's sum into the accumulator word of an output; the last of `split` arrivals casts, stores Y and
// clears the word.  `nan` says the slice sum is NaN (`add` then carries the value 0).  Act: the output's format.
template <typename Act>
__device__ __forceinline__ void add_slice(unsigned long long *word, unsigned long long add, bool nan, int split, uint16_t *y)
{
    if (nan) __hip_atomic_fetch_or(word, kFixPoison, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ahead of this slice's add: same thread, same address
    const unsigned long long total = __hip_atomic_fetch_add(word, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
    if ((total >> 58) == (unsigned long long)split) {
        *y = (total & kFixPoison) ? Act::kNaN : (uint16_t)(Act::pack2(from_fixed(total), 0.f) & 0xFFFFu);
        __hip_atomic_store(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Sum of the waves' result tiles (ROWS x COLS each) in wave order, `red_waves` waves per round through
// LDS (red[wave in round][row][column]; `write_mine` puts the calling wave's tile there as float4
// groups), then the workgroup's finish.  A thread owns groups of VW neighbouring columns of one row;
// the atomic finish wants VW = 1 (consecutive lanes on consecutive outputs, four cache lines per
// wave-wide atomic), the others VW = 4.  `sync` is the accumulator [M, N] (64-bit words, all zero
// before the launch and left zero by it).
template <typename Act, int ROWS, int COLS, int VW, int MIN_WAVES, typename WriteMine>
__device__ __forceinline__ void reduce_and_finish(const GemmArgs &a, const int finish, unsigned long long *__restrict__ sync, unsigned char *smem,
                                                  const WriteMine &write_mine, int red_waves, int row0, int col0, int slice)
{
    typedef float vec_t __attribute__((ext_vector_type(VW)));
    constexpr int kGroups = ROWS * COLS / VW;
    constexpr int kOwn = (kGroups + 64 * MIN_WAVES - 1) / (64 * MIN_WAVES);  // groups per thread, at most
    const int tid = threadIdx.x, wave = tid >> 6, waves = blockDim.x >> 6;
    const int nthreads = (int)blockDim.x;
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
            if (k * nthreads >= kGroups) continue;  // uniform: no thread owns a k-th group
            const int o = tid + k * nthreads;
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
        const int o = tid + k * nthreads;
        const int m = row0 + o / (COLS / VW), col = col0 + VW * (o % (COLS / VW));
        if (o >= kGroups || m >= a.M || col >= a.N) continue;
        const size_t out = (size_t)m * a.N + col;
        if constexpr (VW == 4) {
            if (finish == kFinishDirect)
                *reinterpret_cast<uint2_t *>(a.Y + out) = (uint2_t){Act::pack2(v[k][0], v[k][1]), Act::pack2(v[k][2], v[k][3])};
            else
                *reinterpret_cast<float4_t *>(a.partials + (size_t)slice * a.M * a.N + out) = v[k];
        } else {
            const float sum = v[k][0];
            const bool nan = sum != sum;
            add_slice<Act>(sync + out, to_fixed(nan ? 0.f : sum), nan, a.split, a.Y + out);
        }
    }
}

}  // namespace w4a16
