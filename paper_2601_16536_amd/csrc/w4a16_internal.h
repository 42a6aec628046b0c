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
    const uint16_t *X;        // fp16 [M,K], or bfloat16 when bf16 is set
    const uint32_t *Wp;       // [K/8,N]
    const uint16_t *scales;   // fp16 [K/group,N]
    const uint32_t *Zp;       // [K/group,N/8], or null: symmetric quantisation, every zero point is 8
    uint16_t *Y;              // [M,N] in the format of X
    float *partials;          // fp32 [S,M,N] (unused when split == 1)
    int group, M, N, K;
    int split;                // S
    int groups_per_split;
    int groups;               // K / group (kept here so that no kernel divides for it)
    int bf16;                 // X and Y are bfloat16 (scales stay FP16: they belong to the weights)
};


// Multiply launchers: enqueue on `stream`, return the launch status.
hipError_t launch_wave_split(const GemmArgs &a, int tile_n, hipStream_t stream);
// Measurement aid: reads up to three arrays once, one workgroup per compute unit (w4a16_probe.hip).
hipError_t launch_stream_probe(const void *a, size_t na, const void *b, size_t nb, const void *c, size_t nc, uint32_t *sink, int cus,
                               hipStream_t stream);
// How the K slices of different workgroups meet (the scheduler's choice per shape).
enum Finish : int {
    kFinishDirect = 0,       // S = 1: the workgroup casts and stores Y
    kFinishAccumulator = 1,  // one atomic add per output and slice into the fixed-point accumulator; the last arriver casts
    kFinishSecondPass = 2    // FP32 partials [S, M, N], summed by the separate reduction kernel
};

// What a launch needs for its finish: S = 1 exactly when direct, the accumulator's count holds 63 slices.
inline bool finish_args_ok(const GemmArgs &a, int finish, const unsigned long long *sync)
{
    switch (finish) {
    case kFinishDirect: return a.split == 1;
    case kFinishAccumulator: return a.split > 1 && a.split <= 63 && sync;
    case kFinishSecondPass: return a.split > 1 && a.partials;
    default: return false;
    }
}

// STRIPE family (M <= 16): `waves` waves per workgroup (stripe_min_waves .. stripe_max_waves).  `finish`
// says how the K slices of different workgroups meet; `sync` is the fixed-point accumulator [M, N] that
// finish may need: 64-bit words, all zero before and after every launch.
hipError_t launch_stripe(const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream);
size_t stripe_lds_bytes(int M, int group, int groups_per_split, int waves);  // LDS one workgroup needs
int stripe_lds_limit();                                                       // most it may use
int stripe_min_waves(int M);
int stripe_max_waves(int M);
// STRIPE family for M <= 4: the slice is handed out to the waves in units of `unit_rows` packed rows (2 or 4) by an
// LDS ticket counter, `depth` units in flight per wave; X, scales and zero points of the slice are staged in LDS.
// `dot2`: the dot products on the vector ALU instead of the MFMA (measurement only).
hipError_t launch_stripe_dyn(const GemmArgs &a, int finish, unsigned long long *sync, int waves, int unit_rows, int depth, bool dot2, hipStream_t stream);
size_t stripe_dyn_lds_bytes(int M, int group, int groups_per_split);  // LDS one workgroup needs
int stripe_dyn_lds_limit();                                           // most it may use
// TILE family (the scheduler takes it for M >= 5): 64-column tiles, `rows_x` (16, 32 or 64) rows of X per
// workgroup, `waves` (4..8) waves per workgroup that split the K slice; `finish` and `sync` as in the STRIPE
// family.
hipError_t launch_tile(const GemmArgs &a, int finish, unsigned long long *sync, int rows_x, int waves, hipStream_t stream);
// TILE family at 64 or 32 rows of X per workgroup, FP16, group = 128: four waves per workgroup (w4a16_tile_wide.hip).
hipError_t launch_tile_wide(const GemmArgs &a, int finish, unsigned long long *sync, int rows_x, hipStream_t stream);
// TILE family, 16 rows of X per workgroup, the slice handed out to the waves by ticket (w4a16_tile_dyn.hip); `depth` (1, 2)
// units in flight per wave.
hipError_t launch_tile_dyn(const GemmArgs &a, int finish, unsigned long long *sync, int waves, int depth, int unit_blocks, hipStream_t stream);
// Clears n words of a fixed-point accumulator.
hipError_t launch_accumulator_clear(unsigned long long *acc, size_t n, hipStream_t stream);
// Phase 1 alone (Algorithm 1): W16[K, N] = fp16(s (q - z)) in global memory, for the unfused variant.
hipError_t launch_dequant(const uint32_t *Wp, const uint16_t *scales, const uint32_t *Zp, int group, int N, int K,
                          uint16_t *W16, hipStream_t stream);
// Offline quantizer (Eq. 1): FP16 weights [K, N] -> packed codes, FP16 scales, packed zero points.
hipError_t launch_quantize(const uint16_t *W16, int group, int N, int K, uint32_t *Wp, uint16_t *scales, uint32_t *Zp,
                           hipStream_t stream);
// Second pass (Algorithm 1, Phase 3).
hipError_t launch_reduce(const float *partials, int S, int M, int N, uint16_t *Y, bool bf16, hipStream_t stream);

}  // namespace w4a16
