// Internal interface between the C-ABI layer (w4a16_api.hip) and the kernel
// launchers (w4a16_*.hip).  Not installed; callers use include/w4a16.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace w4a16 {

// Arguments every multiply kernel takes (Eq. 2 operands plus the Split-K
// partition of Algorithm 1, Phase 2).
struct GemmArgs {
    const uint16_t *X;        // fp16 [M,K]
    const uint32_t *Wp;       // [K/8,N]
    const uint16_t *scales;   // fp16 [K/group,N]
    const uint32_t *Zp;       // [K/group,N/8]
    uint16_t *Y;              // fp16 [M,N]
    float *partials;          // fp32 [S,M,N] (unused when split == 1)
    int group, M, N, K;
    int split;                // S
    int groups_per_split;
};

constexpr int kTileN = 256;         // columns per workgroup of the MFMA_REG family (4 waves x 64)
constexpr int kThreads = 256;
constexpr int kLdsBudget = 32768;   // bytes of LDS one workgroup stages X into

// Multiply launchers: enqueue on `stream`, return the launch status.
hipError_t launch_mfma_reg(const GemmArgs &a, hipStream_t stream);
hipError_t launch_wave_split(const GemmArgs &a, int tile_n, hipStream_t stream);
hipError_t launch_mfma_rows(const GemmArgs &a, int tile_m, hipStream_t stream);
// STRIPE family (M <= 16): `waves` waves per workgroup (stripe_min_waves .. stripe_max_waves).  With
// split > 1 the K slices of different workgroups meet either in `acc`, the fixed-point accumulator [M,N]
// of 64-bit words (all zero before and after every launch; split <= 255), or, when acc is null, in
// a.partials (FP32 [S,M,N]) for the second pass.
hipError_t launch_stripe(const GemmArgs &a, unsigned long long *acc, int waves, hipStream_t stream);
size_t stripe_lds_bytes(int M, int group, int groups_per_split, int waves);  // LDS one workgroup needs
int stripe_lds_limit();                                                       // most it may use
int stripe_min_waves(int M);
int stripe_max_waves(int M);
// TILE family (the scheduler takes it for M >= 5): 64-column tiles, `rows_x` (16, 32 or 64) rows of X per workgroup,
// `waves` (4..8) waves per workgroup that split the K slice; with split > 1 the slices meet in `acc`
// or, when acc is null, in a.partials, as in the STRIPE family.
hipError_t launch_tile(const GemmArgs &a, unsigned long long *acc, int rows_x, int waves, hipStream_t stream);
size_t tile_lds_bytes(int rows_x, int waves);
// Clears n words of a fixed-point accumulator.
hipError_t launch_accumulator_clear(unsigned long long *acc, size_t n, hipStream_t stream);
// Second pass (Algorithm 1, Phase 3).
hipError_t launch_reduce(const float *partials, int S, int M, int N, uint16_t *Y, hipStream_t stream);

}  // namespace w4a16
