// W4A16 multiply for few rows of X (the scheduler's choice for 2 <= M <= 16 where the stripe family does not
// pay): one workgroup per (64-column tile, K slice, block of 16 rows of X), the slice handed out to the
// workgroup's waves in units as they become free.
//
// Operands of the 16x16x32 MFMA in its plain form, as in the tile family (w4a16_tile.hip): a lane's 32-bit
// word (eight k of one column) is its B-operand slice, lane (g, j) holding packed row 4 b + g of block b
// (32 k) and columns 4 j .. 4 j + 3 of the tile (one 16-byte load: a wave-wide load reads 256 contiguous bytes
// of each of four packed rows); the A operand is row j of the workgroup's rows of X, k-group g, from LDS.
// sum_k x_k per row comes from one more MFMA per block, X against a constant operand of ones.
//
// How the slice is shared is the decode kernel's way (w4a16_stripe_dyn.hip): a unit is kUnitBlocks blocks of one
// quantisation group (the whole group for group = 128), a wave draws its next unit from an LDS ticket counter,
// every unit's contribution (Eq. 2, fp32) is rounded to a multiple of 2^-24, and from there on all sums are exact
// (integer-valued doubles per wave, 64-bit integers in LDS and across workgroups): Algorithm 1's Phase 3 with
// results that do not depend on which wave took which unit.  A wave stages the X of a unit itself, in its own
// LDS (no barrier in the loop).
#include "w4a16_device.h"
#include "w4a16_finish.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

constexpr int kTileCols = 64;
constexpr int kRowsX = 16;
constexpr int kBlockRows = 4;                    // packed rows per block: one MFMA step of 32 k
// LDS entries per packed row, padded: a 16-byte LDS write goes eight lanes at a time (two rows of X x four packed rows)
// over 32 banks; with 18 entries a packed row starts 8 banks after its predecessor and a row of X 4 banks after its own
// (measured: SQ_LDS_BANK_CONFLICT 2.4 times lower than with 17).
constexpr int kRowStride = kRowsX + 2;
constexpr double kSumMax = 562949953421312.0;    // 2^49 = 2^25 in units of 2^-24: the clamp of a wave's sum
constexpr long long kNaNMark = 1ll << 58;        // added to the LDS sum of an output by a wave whose sum is NaN

// LDS: ticket counter (16 B), the workgroup's sums [16][64] (64-bit), then per wave and ring place one unit of X.
constexpr uint32_t kLdsAcc = 16;
constexpr uint32_t kLdsX = kLdsAcc + kRowsX * kTileCols * 8;
template <int UB>
constexpr uint32_t unit_x_bytes() { return UB * kBlockRows * kRowStride * 16; }

// BOUND: the most threads of a workgroup (the registers a wave may use follow from it: 128 at 1024, 256 at 512).
template <typename Act, int UB, int D, int BOUND>
__global__ __launch_bounds__(BOUND) void tile_dyn_kernel(const GemmArgs a, const int finish, unsigned long long *__restrict__ sync)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = blockDim.x >> 6;
    const int nthreads = blockDim.x;
    const int g4 = lane >> 4, j = lane & 15;
    // grid: x = K slice (the slices of one tile are neighbours in the launch order, hence on different XCDs),
    // y = column tile, z = block of 16 rows of X
    const int slice = blockIdx.x, tile = blockIdx.y, m0 = blockIdx.z * kRowsX;
    const int col0 = tile * kTileCols + 4 * j;
    const bool ok = col0 < a.N;

    // the workgroup's K slice: groups, blocks, units
    const int gbeg = slice * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.groups) gend = a.groups;
    const int groups = gend - gbeg;
    const int bpg = a.group >> 5;                    // blocks per group
    const int upg = bpg / UB;                        // units per group
    const int units = groups * upg;
    const int row_base = gbeg * (a.group >> 3);      // first packed row of the slice

    const uint32_t row_w = (uint32_t)a.N * 4u, row_s = (uint32_t)a.N * 2u, row_z = (uint32_t)(a.N >> 3) * 4u;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Wp) + (size_t)row_base * a.N, 0, (uint32_t)groups * (uint32_t)(a.group >> 3) * row_w, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.scales) + (size_t)gbeg * a.N, 0, (uint32_t)groups * row_s, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Zp) + (size_t)gbeg * (a.N >> 3), 0, zero_point_bytes(a.Zp, (uint32_t)groups * row_z), kRawBuffer);
    const uint32_t zfill = symmetric_fill(a.Zp);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, (uint32_t)((size_t)a.M * a.K * 2), kRawBuffer);
    const uint32_t vw = ok ? (uint32_t)(g4 * a.N + col0) * 4u : kOutOfRange;
    const uint32_t vs = ok ? (uint32_t)col0 * 2u : kOutOfRange;
    const uint32_t vz = ok ? (uint32_t)(col0 >> 3) * 4u : kOutOfRange;
    // X: four neighbouring lanes fetch the 64 bytes one block takes of one row of X; load q of a lane is block q
    const uint32_t xm = (uint32_t)m0 + (uint32_t)(lane >> 2);
    const uint32_t vx = xm < (uint32_t)a.M ? (xm * (uint32_t)a.K + ((uint32_t)row_base + (uint32_t)(lane & 3)) * 8u) * 2u : kOutOfRange;
    const uint32_t xl = (uint32_t)(((lane & 3) * kRowStride + (lane >> 2)) * 16);  // where it goes in the unit's LDS

    struct Unit {
        uint4_t w[UB], x[UB];
        uint2_t sc;
        uint32_t zw;
    };
    Unit ring[D];
    int uidx[D];  // unit in ring place p, -1 = none
    auto load_unit = [&](Unit &r, int u) {
        const bool valid = u >= 0;
        const uint32_t uu = valid ? (uint32_t)u : 0u;
        const uint32_t g = uu / (uint32_t)upg, b0 = uu * UB;  // group and first block (of the slice)
#pragma unroll
        for (int q = 0; q < UB; ++q)  // X ahead of the weights: loads return in order, and these mostly come from cache
            r.x[q] = __builtin_amdgcn_raw_buffer_load_b128(rx, valid ? vx : kOutOfRange, (b0 + q) * (kBlockRows * 16u), 0);
        r.sc = __builtin_amdgcn_raw_buffer_load_b64(rs, valid ? vs : kOutOfRange, g * row_s, 0);
        r.zw = __builtin_amdgcn_raw_buffer_load_b32(rz, valid ? vz : kOutOfRange, g * row_z, 0) | zfill;
#pragma unroll
        for (int q = 0; q < UB; ++q)  // read once from DRAM: nontemporal
            r.w[q] = __builtin_amdgcn_raw_buffer_load_b128(rw, valid ? vw : kOutOfRange, (b0 + q) * (kBlockRows * row_w), 2);
    };
#pragma unroll
    for (int p = 0; p < D; ++p) {
        const int u = wave + p * waves;
        uidx[p] = u < units ? u : -1;
        load_unit(ring[p], uidx[p]);
    }

    uint32_t *const tickets = reinterpret_cast<uint32_t *>(smem);
    unsigned long long *const acc = reinterpret_cast<unsigned long long *>(smem + kLdsAcc);
    if (tid == 0) tickets[0] = (uint32_t)(waves * D);
    for (int e = tid; e < kRowsX * kTileCols; e += nthreads) acc[e] = 0ull;
    __syncthreads();

    unsigned char *const myx = smem + kLdsX + (uint32_t)wave * unit_x_bytes<UB>();  // one unit of X, this wave's own
    const uint32_t xa = (uint32_t)((g4 * kRowStride + j) * 16);                      // this lane's A entry of block 0
    const uint32_t zsh = (uint32_t)(col0 & 4) * 4u;                                   // this lane's four nibbles in its zero-point word

    double tot[4][4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i) tot[c][i] = 0.0;
    const Masks masks = make_masks();
    // sum_k x_k over a unit comes from the MFMA too: X against ones (FP16: 16 where the staged x was divided by 16)
    const typename Act::operand_t ones = Act::ones();
    const float4_t zero4 = {0.f, 0.f, 0.f, 0.f};

    auto draw = [&]() -> int {
        uint32_t t = 0;
        if (lane == 0) t = __hip_atomic_fetch_add(tickets, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return (int)__builtin_amdgcn_readfirstlane(t);
    };
    int next = draw();

    auto compute_unit = [&](Unit &r) {
        // only this wave touches its LDS and the LDS operations of one wave complete in order; the fences only
        // keep the compiler from moving them across the staging
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int q = 0; q < UB; ++q)
            *reinterpret_cast<uint4_t *>(myx + (uint32_t)q * (kBlockRows * kRowStride * 16) + xl) = Act::stage_x(r.x[q]);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        float4_t part[4], xsum;
#pragma unroll
        for (int q = 0; q < UB; ++q) {
            const typename Act::operand_t x = Act::x_operand(*reinterpret_cast<const uint4_t *>(myx + (uint32_t)q * (kBlockRows * kRowStride * 16) + xa));
#pragma unroll
            for (int c = 0; c < 4; ++c) part[c] = Act::mfma(x, Act::unpack(r.w[q][c], masks), q == 0 ? zero4 : part[c]);
            xsum = Act::mfma(x, ones, q == 0 ? zero4 : xsum);
        }
        // the unit is done: scale and zero point (Eq. 2), then the exact sums
        H2 s01, s23;
        s01.u = r.sc[0];
        s23.u = r.sc[1];
        const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
        const uint32_t zw = r.zw >> zsh;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float sp = s[c] * (Act::kCodeScale * kFixScale);  // FP16: 2^48 s (P carries 2^-24, the sums are in units of 2^-24)
            const float sz24 = -s[c] * ((float)((zw >> (4 * c)) & 15u) + Act::kCodeOffset) * kFixScale;  // -2^24 s z
#pragma unroll
            for (int i = 0; i < 4; ++i)  // exact from here on: integers, the sum below 2^53 (an infinity or a NaN stays one)
                tot[c][i] += (double)__builtin_rintf(__builtin_fmaf(sp, part[c][i], sz24 * xsum[i]));
        }
    };

    for (;;) {
        bool any = false;
#pragma unroll
        for (int p = 0; p < D; ++p) {
            if (uidx[p] >= 0) {
                any = true;
                compute_unit(ring[p]);
                uidx[p] = next < units ? next : -1;
                load_unit(ring[p], uidx[p]);
                if (next < units) next = draw();
            }
        }
        if (!any) break;
    }

    // ---- Phase 3 inside the workgroup: exact 64-bit sums in LDS (lane (g, j) holds rows 4 g + i, columns 4 j + c) ----
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            double t = tot[c][i];
            const bool nan = t != t;
            t = t > kSumMax ? kSumMax : (t < -kSumMax ? -kSumMax : t);
            const long long fx = nan ? kNaNMark : (long long)t;
            if (fx != 0) __hip_atomic_fetch_add(acc + (4 * g4 + i) * kTileCols + 4 * j + c, (unsigned long long)fx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    __syncthreads();
    // ---- and across workgroups ----
    for (int o = tid; o < kRowsX * kTileCols; o += nthreads) {
        const int m = m0 + o / kTileCols, col = tile * kTileCols + (o % kTileCols);
        if (m >= a.M || col >= a.N) continue;
        const long long fx = (long long)acc[o];
        const bool nan = fx >= (kNaNMark >> 1);  // sixteen waves' clamped sums stay below 2^53
        const size_t out = (size_t)m * a.N + col;
        if (finish == kFinishAccumulator) {
            add_slice<Act>(sync + out, to_fixed(nan ? 0ll : fx), nan, a.split, a.Y + out);
        } else {
            constexpr long long lim = 1ll << 49;
            const float v = nan ? __builtin_nanf("") : (float)((double)(fx < -lim ? -lim : (fx > lim ? lim : fx)) * (1.0 / 16777216.0));
            if (finish == kFinishDirect)
                a.Y[out] = nan ? Act::kNaN : (uint16_t)(Act::pack2(v, 0.f) & 0xFFFFu);
            else
                a.partials[(size_t)slice * a.M * a.N + out] = v;
        }
    }
}

template <typename Act, int UB, int D, int BOUND>
hipError_t launch_udb(const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream)
{
    const size_t lds = kLdsX + (size_t)waves * unit_x_bytes<UB>();
    const int ntiles = (a.N + kTileCols - 1) / kTileCols, row_blocks = (a.M + kRowsX - 1) / kRowsX;
    if (ntiles > 65535 || row_blocks > 65535) return hipErrorInvalidValue;
    if (lds > 48 * 1024) {  // beyond the default dynamic-LDS allowance
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tile_dyn_kernel<Act, UB, D, BOUND>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((tile_dyn_kernel<Act, UB, D, BOUND>), dim3(a.split, ntiles, row_blocks), dim3(waves * 64), lds, stream, a, finish, sync);
    return hipGetLastError();
}

template <typename Act, int UB, int D>
hipError_t launch_ud(const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream)
{
    // two units in flight need more than 128 registers: up to eight waves per workgroup only
    if constexpr (D == 2) {
        if (waves > 8) return hipErrorInvalidValue;
        return launch_udb<Act, UB, D, 512>(a, finish, sync, waves, stream);
    } else {
        return launch_udb<Act, UB, D, 1024>(a, finish, sync, waves, stream);
    }
}

}  // namespace

// `finish` says how the slices meet (w4a16_finish.h); `sync` is the accumulator it may need.  `depth`: units in
// flight per wave (1 or 2).
hipError_t launch_tile_dyn(const GemmArgs &a, int finish, unsigned long long *sync, int waves, int depth, int unit_blocks, hipStream_t stream)
{
    if (a.group % 32 != 0 || waves < 1 || waves > 16) return hipErrorInvalidValue;
    if (!finish_args_ok(a, finish, sync)) return hipErrorInvalidValue;
    const unsigned long long rows = (unsigned long long)a.groups_per_split * (a.group / 8);
    if (rows * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;  // slice-relative 32-bit buffer offsets
    if ((unsigned long long)a.M * a.K * 2ull >= 0x7F000000ull) return hipErrorInvalidValue;
    const int bpg = a.group / 32;
    int ub = bpg % 4 == 0 ? 4 : (bpg % 2 == 0 ? 2 : 1);  // blocks per unit: a unit never crosses a quantisation group
    if ((unit_blocks == 1 || unit_blocks == 2) && unit_blocks < ub) ub = unit_blocks;  // smaller on request (sweeps)
    if (a.bf16) {  // bfloat16 activations: the scheduler's depth only
        if (depth != 1) return hipErrorInvalidValue;
        if (ub == 4) return launch_ud<ActBF16, 4, 1>(a, finish, sync, waves, stream);
        if (ub == 2) return launch_ud<ActBF16, 2, 1>(a, finish, sync, waves, stream);
        return launch_ud<ActBF16, 1, 1>(a, finish, sync, waves, stream);
    }
    if (depth == 2) {
        if (ub == 4) return launch_ud<ActF16, 4, 2>(a, finish, sync, waves, stream);
        if (ub == 2) return launch_ud<ActF16, 2, 2>(a, finish, sync, waves, stream);
        return launch_ud<ActF16, 1, 2>(a, finish, sync, waves, stream);
    }
    if (ub == 4) return launch_ud<ActF16, 4, 1>(a, finish, sync, waves, stream);
    if (ub == 2) return launch_ud<ActF16, 2, 1>(a, finish, sync, waves, stream);
    return launch_ud<ActF16, 1, 1>(a, finish, sync, waves, stream);
}

}  // namespace w4a16
