// W4A16 multiply for the decode case (M <= 16): one workgroup per (256-column
// stripe, K slice).  Every wave-wide load reads one whole KiB of one packed row
// (64 lanes x 4 words); the waves of a workgroup own contiguous runs of the
// slice's packed rows.
//
// This is Algorithm 1's Split-K at two levels.  Inside a workgroup the waves'
// runs of K are Phase 2's slices (C_i = A * B_i) and their sums meet in LDS.
// Across workgroups (S > 1) the per-slice sums meet in a 64-bit fixed-point
// accumulator per output element (Phase 3: C = sum_i C_i, then the cast to
// FP16): one returning atomic add carries the value and an arrival count, the
// last arriver casts and stores Y and clears the accumulator.  Integer adds
// commute, so the result does not depend on the arrival order, and there is no
// second launch.
//
// Why stripes of 256 columns: with one 128-byte-wide column tile per workgroup
// the 128-byte lines of one class of address bits 7-9 are served ~13 % slower
// than the others on this GPU and the workgroups that own them set the kernel
// time.  A 1 KiB-wide stripe holds every class of line in equal parts.  Measured
// on K = 28672, N = 8192 and kept: contiguous runs of rows per wave (interleaving
// the waves' rows costs 10 %), two blocks of two rows in flight per wave (both
// deeper and shallower prefetch are slower), nontemporal weight loads (+5 %).
//
// MFMA operand trick for M <= 4: all 64 lanes hold words of the SAME packed row
// (eight k) but of different columns.  Lane group g (lanes 16g..16g+15) feeds its
// words as k-group g of the 16x16x32 MFMA's B operand; the A operand holds row r
// of X in MFMA row 4g+r for k-group g only and zeros elsewhere, so result row
// 4g+r, column j -- which is exactly what lane (g, j) holds as element r -- is
// the dot product of X row r with lane (g, j)'s own column.
//
// For 5 <= M <= 16 the same idea uses the 32x32x16 MFMA: lanes 0-31 feed k-group
// 0, lanes 32-63 k-group 1; a lane of group g owns result rows 8i + 4g + j
// (i, j < 4), so the A operand holds row m = 4i + j of X in MFMA row 8i + 4g + j
// for k-group g only, and the lane's sixteen result elements are the sixteen rows
// of X against its own column.  With many rows the sums of a slice are large next
// to the weights it read, so there the slices go to the FP32 workspace [S, M, N]
// and the second pass (Algorithm 1, Phase 3 as a launch of its own) instead of
// one atomic add per output and slice.
//
// The MFMA sums P = 2^-24 sum_k x_k q_k run over all of a wave's rows of one
// quantisation group before scale and zero point are applied (Eq. 2, in fp32).
// X reaches the MFMA through LDS, staged by each wave for its own run of rows in
// double-buffered chunks (no workgroup barrier before the final sum; staging the
// whole slice behind one barrier was measured 1 to 4 us slower, growing with M).
// Scales and zero points travel with the weight blocks (one 8-byte and one
// 4-byte load per block, mostly cache hits): staging them in LDS ahead of the
// loop instead was measured 1 us slower.
#include "w4a16_device.h"
#include "w4a16_finish.h"
#include "w4a16_internal.h"
#include <type_traits>

namespace w4a16 {
namespace {

constexpr int kStripe = 256;    // columns per workgroup: 64 lanes x 4 words
constexpr int kBlockRows = 2;   // packed rows per block (16 k)
constexpr int kRing = 2;        // blocks in flight per wave
constexpr int kLdsLimit = 144 * 1024;

// X reaches the MFMA through LDS in chunks that each wave stages for itself (a wave only needs the X of
// its own run of rows, so no workgroup barrier is involved): kChunkRows packed rows at a time, double
// buffered.  A chunk holds 64 (M <= 8) or 128 (M = 16) A-operand entries of 16 bytes and the fp32 sums
// of x per block and row of X; one more entry per wave is all zero.
template <int MROWS>
struct Chunk {
    static constexpr int kRows = MROWS >= 8 ? 8 : 64 / MROWS;        // packed rows per chunk
    static constexpr int kBlocks = kRows / kBlockRows;
    static constexpr int kEntries = kRows * MROWS;                    // 16-byte entries per chunk
    static constexpr int kPerLane = kEntries / 64;
    static constexpr int kBufBytes = kEntries * 16 + kBlocks * MROWS * 4;
    static constexpr int kWaveBytes = 2 * kBufBytes + 16;             // two buffers and the zero entry
};

typedef float float16_t __attribute__((ext_vector_type(16)));

template <int MROWS>
struct Mma {
    static constexpr bool wide = MROWS > 4;  // 32x32x16 (sixteen result rows per lane) instead of 16x16x32 (four)
    typedef typename std::conditional<wide, float16_t, float4_t>::type Acc;
    static constexpr int kMaxThreads = wide ? 512 : 1024;  // the wide form needs up to 256 registers per lane
    static constexpr int kMinWaves = wide ? 4 : 1;
    static constexpr int kRedWaves = wide ? 64 / MROWS : 16;         // waves per round of the final sum, at most
};

template <int MROWS>
__global__ __launch_bounds__(Mma<MROWS>::kMaxThreads) void stripe_kernel(const GemmArgs a, const int finish, unsigned long long *__restrict__ sync, const int red_waves)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = blockDim.x >> 6;
    // grid: x = stripe, y = K slice.  Integer divisions cost dozens of dependent scalar instructions each,
    // all of them ahead of the first load, so the index arithmetic below avoids them.
    const int stripe = blockIdx.x, slice = blockIdx.y;
    const int col0 = stripe * kStripe + 4 * lane;
    const bool ok = col0 < a.N;

    // the workgroup's K slice: groups, packed rows, blocks; this wave's run of blocks
    const int gbeg = slice * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.groups) gend = a.groups;
    const int groups = gend - gbeg;
    const int rows = groups * (a.group / 8);
    const int row_base = gbeg * (a.group / 8);
    const uint32_t nblocks = (uint32_t)rows / kBlockRows;
    const uint32_t bpg = (uint32_t)a.group / (8 * kBlockRows);  // blocks per group
    // runs of nblocks / waves blocks, the first nblocks % waves of them one block longer
    const uint32_t per = nblocks / (uint32_t)waves, extra = nblocks - per * (uint32_t)waves;
    const uint32_t wb0 = per * (uint32_t)wave + ((uint32_t)wave < extra ? (uint32_t)wave : extra);
    const uint32_t wb1 = wb0 + per + ((uint32_t)wave < extra ? 1u : 0u);

    const uint32_t row_w = (uint32_t)a.N * 4u, row_s = (uint32_t)a.N * 2u, row_z = (uint32_t)(a.N >> 3) * 4u;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Wp) + (size_t)row_base * a.N, 0, (uint32_t)rows * row_w, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.scales) + (size_t)gbeg * a.N, 0, (uint32_t)groups * row_s, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Zp) + (size_t)gbeg * (a.N >> 3), 0, zero_point_bytes(a.Zp, (uint32_t)groups * row_z), kRawBuffer);
    const uint32_t zfill = symmetric_fill(a.Zp);
    const uint32_t vw = ok ? (uint32_t)col0 * 4u : kOutOfRange;
    const uint32_t vs = ok ? (uint32_t)col0 * 2u : kOutOfRange;
    const uint32_t vz = ok ? (uint32_t)(col0 >> 3) * 4u : kOutOfRange;

    // Block b of the slice, with the scales and zero points of its group, if b < wb1, else nothing (the
    // per-lane offset, which the hardware range-checks against the slice size, is pushed out of range:
    // zeros, no traffic).  Weights are read once: nontemporal.
    struct Block {
        uint4_t w[kBlockRows];
        uint2_t sc;
        uint32_t zw;
    };
    Block buf[kRing];
    auto load_block = [&](Block &r, uint32_t b, uint32_t g) {
        const bool valid = b < wb1;
        const uint32_t base = valid ? b * kBlockRows * row_w : 0u;
        const uint32_t gu = __builtin_amdgcn_readfirstlane(valid ? g : 0u);  // wave-uniform: keeps the row offsets scalar
        r.sc = __builtin_amdgcn_raw_buffer_load_b64(rs, valid ? vs : kOutOfRange, gu * row_s, 0);
        r.zw = __builtin_amdgcn_raw_buffer_load_b32(rz, valid ? vz : kOutOfRange, gu * row_z, 0) | zfill;
#pragma unroll
        for (int t = 0; t < kBlockRows; ++t)
            r.w[t] = __builtin_amdgcn_raw_buffer_load_b128(rw, valid ? vw : kOutOfRange, base + (uint32_t)t * row_w, 2);
    };
    // ---- X: this wave's LDS, chunk loader and chunk writer ----
    typedef Chunk<MROWS> Ch;
    unsigned char *wl = smem + (size_t)wave * Ch::kWaveBytes;  // buffer 0, buffer 1, zero entry
    const uint32_t zero_off = (uint32_t)(wave * Ch::kWaveBytes + 2 * Ch::kBufBytes);
    // X as a buffer: rows past the wave's run (or past M) are read through an out-of-range offset, so that
    // every chunk issues the same number of loads (exact wait counts) and the missing entries are zero.
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, (uint32_t)((size_t)a.M * a.K * 2), kRawBuffer);
    const uint32_t row_end = (uint32_t)row_base + wb1 * kBlockRows;  // first packed row (of K) past the wave's run
    // entry e of a chunk = packed row e / MROWS of X row e % MROWS: consecutive lanes write consecutive LDS
    // entries (no bank conflicts) and read 64 / MROWS neighbouring rows' worth of each row of X
    auto x_load = [&](uint4_t(&d)[Ch::kPerLane], uint32_t first_block) {
#pragma unroll
        for (int q = 0; q < Ch::kPerLane; ++q) {
            const uint32_t e = (uint32_t)lane + 64u * q, m = e & (MROWS - 1), kr = (uint32_t)row_base + first_block * kBlockRows + e / MROWS;
            const bool valid = kr < row_end && m < (uint32_t)a.M;
            d[q] = __builtin_amdgcn_raw_buffer_load_b128(rx, valid ? (m * (uint32_t)a.K + kr * 8u) * 2u : kOutOfRange, 0, 0);
        }
    };
    auto x_store = [&](const uint4_t(&d)[Ch::kPerLane], int par) {
        uint4_t *xs = reinterpret_cast<uint4_t *>(wl + par * Ch::kBufBytes);
        float *bs = reinterpret_cast<float *>(wl + par * Ch::kBufBytes + Ch::kEntries * 16);
#pragma unroll
        for (int q = 0; q < Ch::kPerLane; ++q) {
            const int e = lane + 64 * q, m = e & (MROWS - 1), kl = e / MROWS;
            float sum = sum8(d[q]);
            sum += __shfl_xor(sum, MROWS, 64);  // the other packed row of the block, same row of X
            xs[e] = permute_x(d[q]);
            if ((kl & 1) == 0) bs[(kl >> 1) * MROWS + m] = sum;
        }
    };

    // X of the first chunk goes ahead of the weights: loads return in order, and X (mostly cache hits) must
    // not queue behind the first weight blocks, which come from DRAM.
    uint4_t xd[Ch::kPerLane];
    x_load(xd, wb0);
    // (lg, lnext): group of the next block to load and the first block of the group after it
    uint32_t lg = wb0 / bpg, lnext = (lg + 1) * bpg;
#pragma unroll
    for (int p = 0; p < kRing; ++p) {
        load_block(buf[p], wb0 + p, lg);
        if (wb0 + p + 1 == lnext) { ++lg; lnext += bpg; }
    }
    if (lane == 0) *reinterpret_cast<uint4_t *>(smem + zero_off) = (uint4_t){0u, 0u, 0u, 0u};
    x_store(xd, 0);

    // this lane's A-operand entry of packed row 0 of a chunk: a row of X, or the zero entry
    int r;
    bool has_row;
    if constexpr (Mma<MROWS>::wide) {
        const int g2 = lane >> 5, q = lane & 31;            // MFMA row q, k-group g2
        r = 4 * (q >> 3) + (q & 3);                         // row 8i + 4g + j holds X row 4i + j ...
        has_row = ((q >> 2) & 1) == g2 && r < MROWS;        // ... for k-group g only
    } else {
        const int g4 = lane >> 4, j = lane & 15;            // MFMA row j, k-group g4
        r = j - 4 * g4;                                     // row 4g + r holds X row r for k-group g only
        has_row = r >= 0 && r < MROWS;
    }
    const uint32_t xa0 = has_row ? (uint32_t)(wave * Ch::kWaveBytes + r * 16) : zero_off;  // in buffer 0
    const uint32_t xstep = has_row ? (uint32_t)(MROWS * 16) : 0u;                          // bytes per packed row
    const uint32_t xpar = has_row ? (uint32_t)Ch::kBufBytes : 0u;                          // buffer 1 - buffer 0
    const uint32_t zsh = (uint32_t)(col0 & 7) * 4u;  // this lane's four nibbles in its zero-point word

    float tot[4][MROWS];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < MROWS; ++i) tot[c][i] = 0.f;
    typedef typename Mma<MROWS>::Acc Acc;
    Acc part[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) part[c] = Acc(0.f);
    float xsum[MROWS];
#pragma unroll
    for (int i = 0; i < MROWS; ++i) xsum[i] = 0.f;
    const Masks masks = make_masks();

    uint32_t gnext = (wb0 / bpg + 1) * bpg;  // first block of the group after the current one

    // Only this wave touches its LDS and the LDS operations of one wave complete in order; the
    // fences only keep the compiler from moving them across the staging.
    int par = 0;
    for (uint32_t cb = wb0; cb < wb1; cb += Ch::kBlocks, par ^= 1) {
        x_load(xd, cb + Ch::kBlocks);  // the next chunk's X (nothing past the wave's run)
        const uint32_t xa = xa0 + (uint32_t)par * xpar;
        const float *bs = reinterpret_cast<const float *>(wl + par * Ch::kBufBytes + Ch::kEntries * 16);
        const uint32_t nb = wb1 - cb < (uint32_t)Ch::kBlocks ? wb1 - cb : (uint32_t)Ch::kBlocks;  // blocks of this chunk
        for (uint32_t bb = 0; bb < nb; bb += kRing) {
#pragma unroll
            for (int p = 0; p < kRing; ++p) {
                const uint32_t lb = bb + p, cur = cb + lb;  // block of the chunk, block of the slice
                if (cur < wb1) {
                    // Loads return in order and the block's scales and zero points were issued ahead of its
                    // weights.  Naming them here, used or not, tells the compiler that they have landed, so
                    // that reloading their registers below needs no wait on younger loads.
                    asm volatile("" ::"v"(buf[p].sc[0]), "v"(buf[p].sc[1]), "v"(buf[p].zw));
#pragma unroll
                    for (int t = 0; t < kBlockRows; ++t) {
                        H8 x;
                        x.u = *reinterpret_cast<const uint4_t *>(smem + xa + (lb * kBlockRows + t) * xstep);
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            if constexpr (Mma<MROWS>::wide)
                                part[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x.h, unpack8(buf[p].w[t][c], masks), part[c], 0, 0, 0);
                            else
                                part[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x.h, unpack8(buf[p].w[t][c], masks), part[c], 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < MROWS; ++i) xsum[i] += bs[lb * MROWS + i];
                    if (cur + 1 == gnext || cur + 1 == wb1) {
                        // the wave's rows of this group are done: scale and zero point (Eq. 2)
                        H2 s01, s23;
                        s01.u = buf[p].sc[0];
                        s23.u = buf[p].sc[1];
                        const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
                        const uint32_t zw = buf[p].zw >> zsh;
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const float z = (float)((zw >> (4 * c)) & 15u);
#pragma unroll
                            for (int i = 0; i < MROWS; ++i) tot[c][i] = apply_scale_zero(tot[c][i], s[c], z, part[c][i], xsum[i]);
                            part[c] = Acc(0.f);
                        }
#pragma unroll
                        for (int i = 0; i < MROWS; ++i) xsum[i] = 0.f;
                        gnext += bpg;
                    }
                }
                load_block(buf[p], cur + kRing, lg);
                if (cur + kRing + 1 == lnext) { ++lg; lnext += bpg; }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        x_store(xd, par ^ 1);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }

    // Phase 3 inside the workgroup, then across workgroups.  The atomic finish wants consecutive lanes on
    // consecutive outputs (one 8-byte atomic per lane: four cache lines per wave-wide instruction); the
    // other finishes move four neighbouring outputs per lane.
    const auto write_mine = [&](float4_t *mine) {  // [row][column / 4] of this wave's 256 columns
#pragma unroll
        for (int i = 0; i < MROWS; ++i) mine[i * 64 + lane] = (float4_t){tot[0][i], tot[1][i], tot[2][i], tot[3][i]};
    };
    if (finish == kFinishAccumulator)
        reduce_and_finish<ActF16, MROWS, kStripe, 1, Mma<MROWS>::kMinWaves>(a, finish, sync, smem, write_mine, red_waves, 0, stripe * kStripe, slice);
    else
        reduce_and_finish<ActF16, MROWS, kStripe, 4, Mma<MROWS>::kMinWaves>(a, finish, sync, smem, write_mine, red_waves, 0, stripe * kStripe, slice);
}

int mrows_of(int M) { return M == 1 ? 1 : (M == 2 ? 2 : (M <= 4 ? 4 : (M <= 8 ? 8 : 16))); }

template <int MROWS>
hipError_t launch_m(const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream)
{
    if (waves < Mma<MROWS>::kMinWaves || waves * 64 > Mma<MROWS>::kMaxThreads) return hipErrorInvalidValue;
    const size_t lds = stripe_lds_bytes(a.M, a.group, a.groups_per_split, waves);
    if (lds > (size_t)stripe_lds_limit()) return hipErrorInvalidValue;
    int red_waves = (int)(lds / ((size_t)MROWS * kStripe * 4));  // >= 1 by stripe_lds_bytes
    if (red_waves > waves) red_waves = waves;
    if (red_waves > Mma<MROWS>::kRedWaves) red_waves = Mma<MROWS>::kRedWaves;
    const unsigned long long rows = (unsigned long long)a.groups_per_split * (a.group / 8);
    if (rows * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;  // slice-relative 32-bit buffer offsets
    const int nstripes = (a.N + kStripe - 1) / kStripe;
    if (lds > 48 * 1024) {  // beyond the default dynamic-LDS allowance
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&stripe_kernel<MROWS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, stripe_lds_limit());
        if (e != hipSuccess) return e;
    }
    if (a.split > 65535) return hipErrorInvalidValue;  // slices are the grid's y
    hipLaunchKernelGGL((stripe_kernel<MROWS>), dim3(nstripes, a.split), dim3(waves * 64), lds, stream, a, finish, sync, red_waves);
    return hipGetLastError();
}

}  // namespace

int stripe_lds_limit() { return kLdsLimit; }
int stripe_min_waves(int M) { return M > 4 ? 4 : 1; }
int stripe_max_waves(int M) { return M > 4 ? 8 : 16; }

// The waves' chunk buffers; the final sums reuse the space, at least one wave's worth of them (more waves
// per round when there is room: fewer barriers).
size_t stripe_lds_bytes(int M, int group, int groups_per_split, int waves)
{
    (void)group;
    (void)groups_per_split;
    const int mrows = mrows_of(M);
    size_t stage = 0;
    switch (mrows) {
    case 1: stage = Chunk<1>::kWaveBytes; break;
    case 2: stage = Chunk<2>::kWaveBytes; break;
    case 4: stage = Chunk<4>::kWaveBytes; break;
    case 8: stage = Chunk<8>::kWaveBytes; break;
    default: stage = Chunk<16>::kWaveBytes; break;
    }
    stage *= waves;
    const size_t one = (size_t)mrows * kStripe * 4;
    size_t red = one * waves;
    if (red > 64 * 1024) red = 64 * 1024 < one ? one : 64 * 1024 / one * one;
    return stage > red ? stage : red;
}

// `finish` says how the slices meet (w4a16_finish.h); `sync` is the accumulator it may need.
hipError_t launch_stripe(const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream)
{
    if (a.M > 16 || a.group % (8 * kBlockRows) != 0) return hipErrorInvalidValue;
    if (a.bf16) return hipErrorInvalidValue;  // FP16 activations only (the scheduler never takes this form by itself)
    if (!finish_args_ok(a, finish, sync)) return hipErrorInvalidValue;
    switch (mrows_of(a.M)) {
    case 1: return launch_m<1>(a, finish, sync, waves, stream);
    case 2: return launch_m<2>(a, finish, sync, waves, stream);
    case 4: return launch_m<4>(a, finish, sync, waves, stream);
    case 8: return launch_m<8>(a, finish, sync, waves, stream);
    default: return launch_m<16>(a, finish, sync, waves, stream);
    }
}

}  // namespace w4a16
