// W4A16 multiply, any M (the scheduler's choice except for M <= 4 on large weight
// matrices): one workgroup per (64-column tile, block of 16 RT
// rows of X, K slice), RT = 1, 2 or 4.  The waves of a workgroup own contiguous
// runs of the slice's K (Algorithm 1, Phase 2 with the slices held by waves) and
// their results meet in LDS; with S = 1 the workgroup casts and stores Y itself,
// with S > 1 the slices meet in the fixed-point accumulator or go to the FP32
// workspace and the second pass (Phase 3), as in the STRIPE family.
//
// Operands of the 16x16x32 MFMA in its plain form: a lane's 32-bit word (eight k
// of one column) is its B-operand slice, lane (g, j) holding packed row 4 b + g
// of block b (32 k) and columns 4 j .. 4 j + 3 of the tile (one 16-byte load:
// a wave-wide load reads 256 contiguous bytes of each of four packed rows); the
// A operand is row 16 rt + j of the workgroup's rows of X, k-group g, from LDS.
// Every unpacked word feeds RT MFMAs.  As in the other families the MFMA sums
// P = 2^-24 sum_k x_k q_k run over a wave's rows of one quantisation group, then
// (2^24 s) P - (s z) sum_k x_k in fp32 (Eq. 2); sum_k x_k comes from one more
// MFMA per block and row tile, X against a constant operand of ones (cheaper here
// than summing on the vector ALU while staging, which every column tile repeats).
//
// X reaches LDS per wave: a wave needs only the X of its own run of K, stages it
// in double-buffered chunks of one, two or four blocks, and so never waits at a
// workgroup barrier before the final sum.  Neighbouring lanes fetch contiguous
// bytes of one row of X; the LDS rows are padded so that these writes, and the
// MFMA's reads, are free of bank conflicts.  Two kernels follow: a loop over
// single blocks for any group size, and one laid out around the group for
// group = 128.
//
// The row blocks of one column tile read the same weights.  Workgroups are
// numbered so that they sit on the same XCD (workgroup b runs on XCD b mod 8) and
// start together: the second reader finds the weights in that XCD's L2.
#include "w4a16_device.h"
#include "w4a16_finish.h"
#include "w4a16_internal.h"
#include <type_traits>

namespace w4a16 {
namespace {

constexpr int kTileCols = 64;
constexpr int kBlockRows = 4;   // packed rows per block: one MFMA step of 32 k
constexpr int kXcds = 8;

template <int RT>
struct Shape {
    static constexpr int kRowsX = 16 * RT;                       // rows of X per workgroup
    static constexpr int kChunkBlocks = RT == 4 ? 1 : 2;         // blocks per staged chunk of X
    static constexpr int kRing = 4;                              // blocks in flight per wave
    static constexpr int kRowStride = kRowsX + 4;                // LDS entries per packed row (padded)
    static constexpr int kEntries = kChunkBlocks * kBlockRows * kRowsX;  // entries a chunk really holds
    static constexpr int kPerLane = kEntries / 64;
    static constexpr int kBufBytes = kChunkBlocks * kBlockRows * kRowStride * 16;
    static constexpr int kWaveBytes = 2 * kBufBytes;
    static constexpr int kOutBytes = kRowsX * kTileCols * 4;     // a wave's result tile in fp32
};

template <typename Act, int RT>
__global__ __launch_bounds__(512) void tile_kernel(const GemmArgs a, const int finish, unsigned long long *__restrict__ sync, const int row_blocks, const int red_waves)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef Shape<RT> Sh;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = blockDim.x >> 6;
    const int g4 = lane >> 4, j = lane & 15;

    // workgroup -> (column tile, K slice, row block): the row blocks of one (tile, slice) are neighbours on one XCD
    const int ntiles = (a.N + kTileCols - 1) / kTileCols;
    const int units = ntiles * a.split;
    // (integer divisions cost dozens of dependent scalar instructions each, all ahead of the first load:
    // the common cases take none)
    int rb = 0, unit = (int)blockIdx.x;
    if (row_blocks > 1) {
        const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
        rb = local % row_blocks;
        unit = (local / row_blocks) * kXcds + xcd;
    }
    if (unit >= units) return;  // the grid is rounded up to whole XCD rounds
    int tile = unit, slice = 0;
    if (a.split > 1) {
        slice = unit / ntiles;
        tile = unit - slice * ntiles;
    }
    const int m0 = rb * Sh::kRowsX;
    const int col0 = tile * kTileCols + 4 * j;
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
    const uint32_t vw = ok ? (uint32_t)(g4 * a.N + col0) * 4u : kOutOfRange;
    const uint32_t vs = ok ? (uint32_t)col0 * 2u : kOutOfRange;
    const uint32_t vz = ok ? (uint32_t)(col0 >> 3) * 4u : kOutOfRange;

    // Block b of the slice, with the scales and zero points of its group, if b < wb1, else nothing (the
    // per-lane offset, which the hardware range-checks against the slice size, is pushed out of range:
    // zeros, no traffic).  Weights are read once from DRAM: nontemporal.
    struct Block {
        uint4_t w;
        uint2_t sc;
        uint32_t zw;
    };
    constexpr int kRing = Sh::kRing;
    Block buf[kRing];
    auto load_block = [&](Block &r, uint32_t b, uint32_t g) {
        const bool valid = b < wb1;
        const uint32_t gu = __builtin_amdgcn_readfirstlane(valid ? g : 0u);  // wave-uniform: keeps the row offsets scalar
        r.sc = __builtin_amdgcn_raw_buffer_load_b64(rs, vs, gu * row_s, 0);   // past the run: group 0 again, unused
        r.zw = __builtin_amdgcn_raw_buffer_load_b32(rz, vz, gu * row_z, 0) | zfill;
        r.w = __builtin_amdgcn_raw_buffer_load_b128(rw, valid ? vw : kOutOfRange, valid ? b * kBlockRows * row_w : 0u, 2);
    };

    // ---- X: this wave's LDS, chunk loader and chunk writer ----
    unsigned char *wl = smem + (size_t)wave * Sh::kWaveBytes;  // buffer 0, buffer 1
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, (uint32_t)((size_t)a.M * a.K * 2), kRawBuffer);
    // entry e of a chunk: four neighbouring lanes take the four packed rows of one block of one row of X.
    // Per lane and entry the global offset (at block 0 of the slice) and the LDS slot never change: a chunk's
    // loads differ only in a scalar offset.  Rows past M read through an out-of-range offset (zeros); blocks
    // past the wave's run are staged but never used.
    uint32_t xg[Sh::kPerLane], xl[Sh::kPerLane];
#pragma unroll
    for (int q = 0; q < Sh::kPerLane; ++q) {
        const uint32_t e = (uint32_t)lane + 64u * q;
        const uint32_t r = e & 3u, m = (e >> 2) % Sh::kRowsX, blk = (e >> 2) / Sh::kRowsX;
        xg[q] = (uint32_t)m0 + m < (uint32_t)a.M
                    ? (((uint32_t)m0 + m) * (uint32_t)a.K + ((uint32_t)row_base + blk * kBlockRows + r) * 8u) * 2u
                    : kOutOfRange;
        xl[q] = ((blk * kBlockRows + r) * Sh::kRowStride + m) * 16u;
    }
    auto x_load = [&](uint4_t(&d)[Sh::kPerLane], uint32_t first_block) {
#pragma unroll
        for (int q = 0; q < Sh::kPerLane; ++q)
            d[q] = __builtin_amdgcn_raw_buffer_load_b128(rx, xg[q], first_block * (kBlockRows * 16u), 0);
    };
    auto x_store = [&](const uint4_t(&d)[Sh::kPerLane], int par) {
#pragma unroll
        for (int q = 0; q < Sh::kPerLane; ++q)
            *reinterpret_cast<uint4_t *>(wl + par * Sh::kBufBytes + xl[q]) = Act::stage_x(d[q]);
    };

    // X of the first chunk goes ahead of the weights: loads return in order, and X (mostly cache hits) must
    // not queue behind the first weight blocks.
    uint4_t xd[Sh::kPerLane];
    x_load(xd, wb0);
    uint32_t lg = wb0 / bpg, lnext = (lg + 1) * bpg;  // group of the next block to load, first block of the group after it
#pragma unroll
    for (int p = 0; p < kRing; ++p) {
        load_block(buf[p], wb0 + p, lg);
        if (wb0 + p + 1 == lnext) { ++lg; lnext += bpg; }
    }
    x_store(xd, 0);

    const uint32_t xa0 = (uint32_t)(wave * Sh::kWaveBytes + (g4 * Sh::kRowStride + j) * 16);  // A entry of block 0, row tile 0
    const uint32_t zsh = (uint32_t)(col0 & 4) * 4u;  // this lane's four nibbles in its zero-point word

    float4_t tot[RT][4], part[RT][4], xsum[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            tot[rt][c] = (float4_t){0.f, 0.f, 0.f, 0.f};
            part[rt][c] = (float4_t){0.f, 0.f, 0.f, 0.f};
        }
        xsum[rt] = (float4_t){0.f, 0.f, 0.f, 0.f};
    }
    const Masks masks = make_masks();
    // sum_k x_k over a block comes from the MFMA too: X against ones (FP16: 16 where the staged x was divided by 16)
    const typename Act::operand_t ones = Act::ones();
    uint32_t gnext = (wb0 / bpg + 1) * bpg;  // first block of the group after the current one

    // Only this wave touches its LDS and the LDS operations of one wave complete in order; the
    // fences only keep the compiler from moving them across the staging.
    const int par = 0;  // a round holds an even number of chunks: chunk (p / kChunkBlocks) of a round uses buffer (p / kChunkBlocks) & 1
    for (uint32_t cb = wb0; cb < wb1; cb += kRing) {
#pragma unroll
        for (int p = 0; p < kRing; ++p) {
            const uint32_t cur = cb + p;
            const int lb = p % Sh::kChunkBlocks;                   // block of its chunk
            const int cpar = par ^ ((p / Sh::kChunkBlocks) & 1);   // buffer that holds its chunk
            if (lb == 0) x_load(xd, cur + Sh::kChunkBlocks);       // the next chunk's X
            if (cur < wb1) {
                // Loads return in order and the block's scales and zero points were issued ahead of its
                // weights.  Naming them here, used or not, tells the compiler that they have landed, so
                // that reloading their registers below needs no wait on younger loads.
                asm volatile("" ::"v"(buf[p].sc[0]), "v"(buf[p].sc[1]), "v"(buf[p].zw));
                const unsigned char *xb = smem + xa0 + cpar * Sh::kBufBytes + lb * (kBlockRows * Sh::kRowStride * 16);
                typename Act::operand_t bop[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) bop[c] = Act::unpack(buf[p].w[c], masks);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const typename Act::operand_t x = Act::x_operand(*reinterpret_cast<const uint4_t *>(xb + rt * 256));
#pragma unroll
                    for (int c = 0; c < 4; ++c) part[rt][c] = Act::mfma(x, bop[c], part[rt][c]);
                    xsum[rt] = Act::mfma(x, ones, xsum[rt]);
                }
                if (cur + 1 == gnext || cur + 1 == wb1) {
                    // the wave's rows of this group are done: scale and zero point (Eq. 2)
                    H2 s01, s23;
                    s01.u = buf[p].sc[0];
                    s23.u = buf[p].sc[1];
                    const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
                    const uint32_t zw = buf[p].zw >> zsh;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float sp = s[c] * Act::kCodeScale;                                          // FP16: 2^24 s
                        const float sz = -s[c] * ((float)((zw >> (4 * c)) & 15u) + Act::kCodeOffset);   // -s z
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                tot[rt][c][i] = __builtin_fmaf(sp, part[rt][c][i], __builtin_fmaf(sz, xsum[rt][i], tot[rt][c][i]));
                            part[rt][c] = (float4_t){0.f, 0.f, 0.f, 0.f};
                        }
                    }
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) xsum[rt] = (float4_t){0.f, 0.f, 0.f, 0.f};
                    gnext += bpg;
                }
            }
            load_block(buf[p], cur + kRing, lg);
            if (cur + kRing + 1 == lnext) { ++lg; lnext += bpg; }
            if (lb == Sh::kChunkBlocks - 1) {  // the chunk is done: its successor's X goes to the other buffer
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                x_store(xd, cpar ^ 1);
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            }
        }
    }

    // Phase 3 inside the workgroup, then across workgroups (see w4a16_finish.h).
    const auto write_mine = [&](float4_t *mine) {  // [row][column / 4] of the 64-column tile
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                mine[(16 * rt + 4 * g4 + i) * (kTileCols / 4) + j] = (float4_t){tot[rt][0][i], tot[rt][1][i], tot[rt][2][i], tot[rt][3][i]};
    };
    if (finish == kFinishAccumulator)
        reduce_and_finish<Act, Sh::kRowsX, kTileCols, 1, 4>(a, finish, sync, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
    else
        reduce_and_finish<Act, Sh::kRowsX, kTileCols, 4, 4>(a, finish, sync, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
}

// ---- group = 128: the waves' runs are whole quantisation groups ----
//
// With four blocks to the group a wave's loop can be laid out around the group: the scales and zero
// points are read once per group (not with every block), the step of Eq. 2 sits at a fixed place (no
// test per block), each group's MFMA sums start from a zero operand (no clearing), and the weights of
// two groups (eight blocks, 8 KB per wave) are in flight, which is what the memory latency of about
// 1.3 us asks for at eight waves per compute unit.  Every buffer descriptor ends where the wave's run
// ends, so loads past the run are cut off by the hardware's range check (zeros, no traffic) and need
// no test either.
template <int RT>
struct GroupShape {
    static constexpr int kRowsX = 16 * RT;
    static constexpr int kChunkBlocks = RT == 4 ? 1 : 4;         // blocks per staged chunk of X
    static constexpr int kChunks = 4 / kChunkBlocks;             // chunks per group
    static constexpr int kRingGroups = RT == 4 ? 1 : 2;          // groups of weights in flight per wave (registers)
    // LDS entries per packed row, padded (a 16-byte LDS write goes eight lanes at a time over 32 banks): odd where
    // neighbouring lanes write the packed rows of one row of X; rows + 2 where eight lanes are two rows of X x four packed
    // rows (measured at 64 rows: SQ_LDS_BANK_CONFLICT three times lower than with rows + 4)
    static constexpr int kRowStride = kChunkBlocks == 4 ? kRowsX + 1 : kRowsX + 2;
    static constexpr int kPerLane = kChunkBlocks * kBlockRows * kRowsX / 64;
    static constexpr int kBufBytes = kChunkBlocks * kBlockRows * kRowStride * 16;
    static constexpr int kWaveBytes = 2 * kBufBytes;
    static constexpr int kOutBytes = kRowsX * kTileCols * 4;
};

template <typename Act, int RT>
__global__ __launch_bounds__(512) void tile_group_kernel(const GemmArgs a, const int finish, unsigned long long *__restrict__ sync, const int row_blocks, const int red_waves)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef GroupShape<RT> Sh;
    constexpr int kBpg = 4;  // blocks per group

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = blockDim.x >> 6;
    const int g4 = lane >> 4, j = lane & 15;

    const int ntiles = (a.N + kTileCols - 1) / kTileCols;
    const int units = ntiles * a.split;
    // (integer divisions cost dozens of dependent scalar instructions each, all ahead of the first load:
    // the common cases take none)
    int rb = 0, unit = (int)blockIdx.x;
    if (row_blocks > 1) {
        const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
        rb = local % row_blocks;
        unit = (local / row_blocks) * kXcds + xcd;
    }
    if (unit >= units) return;  // the grid is rounded up to whole XCD rounds
    int tile = unit, slice = 0;
    if (a.split > 1) {
        slice = unit / ntiles;
        tile = unit - slice * ntiles;
    }
    const int m0 = rb * Sh::kRowsX;
    const int col0 = tile * kTileCols + 4 * j;
    const bool ok = col0 < a.N;

    // the slice's groups, and this wave's run of them
    const int gbeg = slice * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.groups) gend = a.groups;
    const int groups = gend - gbeg;
    // runs of groups / waves groups, the first groups % waves of them one group longer
    const int per = (int)((uint32_t)groups / (uint32_t)waves), extra = groups - per * waves;
    const int g0 = gbeg + per * wave + (wave < extra ? wave : extra);
    const int ng = per + (wave < extra ? 1 : 0);

    const uint32_t row_w = (uint32_t)a.N * 4u, row_s = (uint32_t)a.N * 2u, row_z = (uint32_t)(a.N >> 3) * 4u;
    const uint32_t step_w = kBlockRows * row_w;  // one block further
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Wp) + (size_t)g0 * 16 * a.N, 0, (uint32_t)ng * 16u * row_w, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.scales) + (size_t)g0 * a.N, 0, (uint32_t)ng * row_s, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Zp) + (size_t)g0 * (a.N >> 3), 0, zero_point_bytes(a.Zp, (uint32_t)ng * row_z), kRawBuffer);
    const uint32_t zfill = symmetric_fill(a.Zp);
    // running per-lane offsets of the next block / group to load; the range check is on these
    uint32_t vw = ok ? (uint32_t)(g4 * a.N + col0) * 4u : kOutOfRange;
    uint32_t vs = ok ? (uint32_t)col0 * 2u : kOutOfRange;
    uint32_t vz = ok ? (uint32_t)(col0 >> 3) * 4u : kOutOfRange;

    constexpr int kRG = Sh::kRingGroups;
    uint4_t wq[kRG * kBpg];  // the weights in flight
    auto load_w = [&](uint4_t &d) {
        d = __builtin_amdgcn_raw_buffer_load_b128(rw, vw, 0, 2);  // read once from DRAM: nontemporal
        vw += step_w;
    };

    // ---- X: this wave's LDS (two chunk buffers), chunk loader and chunk writer ----
    // Whole-group chunks (16 or 32 rows of X per workgroup): sixteen neighbouring lanes fetch the 256 contiguous
    // bytes the group takes of one row of X, so that every cache line is used up by the instruction that brings
    // it (64-byte pieces, one block per instruction, cost twice the L2 traffic: the other half of each line was
    // gone from the L1 by the time the next block asked for it).  Load q of a lane: row 4 q + lane / 16, packed
    // row lane % 16 of the group.  One-block chunks (64 rows): four neighbouring lanes fetch the 64 bytes of the
    // block, load q: row lane / 4 + 16 q.
    unsigned char *wl = smem + (size_t)wave * Sh::kWaveBytes;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, (uint32_t)((size_t)a.M * a.K * 2), kRawBuffer);
    constexpr bool kWholeGroup = Sh::kChunkBlocks == 4;
    uint32_t xg[Sh::kPerLane];
#pragma unroll
    for (int q = 0; q < Sh::kPerLane; ++q) {
        const uint32_t m = (uint32_t)m0 + (kWholeGroup ? 4u * q + (uint32_t)(lane >> 4) : 16u * q + (uint32_t)(lane >> 2));
        const uint32_t prow = (uint32_t)g0 * 16u + (uint32_t)(kWholeGroup ? lane & 15 : lane & 3);
        xg[q] = m < (uint32_t)a.M ? (m * (uint32_t)a.K + prow * 8u) * 2u : kOutOfRange;
    }
    const uint32_t xl0 = kWholeGroup ? (uint32_t)(((lane & 15) * Sh::kRowStride + (lane >> 4)) * 16)
                                     : (uint32_t)(((lane & 3) * Sh::kRowStride + (lane >> 2)) * 16);
    uint4_t xd[Sh::kPerLane];
    auto x_load = [&](uint32_t chunk) {  // chunk of the wave's run
        const uint32_t so = chunk * (Sh::kChunkBlocks * kBlockRows * 16u);
#pragma unroll
        for (int q = 0; q < Sh::kPerLane; ++q) xd[q] = __builtin_amdgcn_raw_buffer_load_b128(rx, xg[q], so, 0);
    };
    auto x_store = [&](int par) {
#pragma unroll
        for (int q = 0; q < Sh::kPerLane; ++q)
            *reinterpret_cast<uint4_t *>(wl + par * Sh::kBufBytes + xl0 + (kWholeGroup ? 4 * q : 16 * q) * 16) = Act::stage_x(xd[q]);
    };

    float4_t tot[RT][4];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int c = 0; c < 4; ++c) tot[rt][c] = (float4_t){0.f, 0.f, 0.f, 0.f};

    if (ng > 0) {
        const uint32_t zsh = (uint32_t)(col0 & 4) * 4u;  // this lane's four nibbles in its zero-point word
        // X of the first chunk goes ahead of the weights: loads return in order, and X (mostly cache hits)
        // must not queue behind the first weight blocks.
        const uint32_t nchunks = (uint32_t)ng * Sh::kChunks;
        x_load(0);
#pragma unroll
        for (int h = 0; h < kRG; ++h)
#pragma unroll
            for (int p = 0; p < kBpg; ++p) load_w(wq[h * kBpg + p]);
        x_store(0);
        if (nchunks > 1) x_load(1);

        const uint32_t xa0 = (uint32_t)(wave * Sh::kWaveBytes + (g4 * Sh::kRowStride + j) * 16);  // A entry of block 0, row tile 0
        const Masks masks = make_masks();
        // sum_k x_k over a group comes from the MFMA too: X against ones (FP16: 16 where the staged x was divided by 16)
        const typename Act::operand_t ones = Act::ones();
        const float4_t zero4 = {0.f, 0.f, 0.f, 0.f};

        // One group: its four blocks from ring place R, chunk buffers by parity of the chunk number.  Only this
        // wave touches its LDS and the LDS operations of one wave complete in order; the fences only keep the
        // compiler from moving them across the staging.
        auto do_group = [&](auto half, const uint32_t gi) {
            constexpr int H = decltype(half)::value;  // parity of the group in the run: its chunk buffers
            constexpr int R = H % kRG;                 // its place in the ring
            float4_t part[RT][4], xsum[RT];
            // The group's scales and zero points, wanted when its four blocks are done.  Loads return in order:
            // these come in behind the weights of the groups in flight, which are wanted earlier anyway.
            const uint2_t sc = __builtin_amdgcn_raw_buffer_load_b64(rs, vs, 0, 0);
            const uint32_t zw = __builtin_amdgcn_raw_buffer_load_b32(rz, vz, 0, 0) | zfill;
            vs += row_s;
            vz += row_z;
#pragma unroll
            for (int p = 0; p < kBpg; ++p) {
                constexpr int CB = Sh::kChunkBlocks;
                const int c = p / CB, lb = p % CB;
                const int par = (H * Sh::kChunks + c) & 1;
                const unsigned char *xb = smem + xa0 + par * Sh::kBufBytes + lb * (kBlockRows * Sh::kRowStride * 16);
                typename Act::operand_t bop[4];
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) bop[cc] = Act::unpack(wq[R * kBpg + p][cc], masks);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const typename Act::operand_t x = Act::x_operand(*reinterpret_cast<const uint4_t *>(xb + rt * 256));
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) part[rt][cc] = Act::mfma(x, bop[cc], p == 0 ? zero4 : part[rt][cc]);
                    xsum[rt] = Act::mfma(x, ones, p == 0 ? zero4 : xsum[rt]);
                }
                if (lb == CB - 1) {
                    // The chunk is done.  Its successor's X, asked for a chunk ago, goes to the other buffer, and
                    // the chunk after that is asked for: ahead of the weight load below, because loads return in
                    // order and waiting for X must not mean waiting for weights wanted much later.
                    const uint32_t n = gi * Sh::kChunks + c;  // this chunk of the run
                    if (n + 1 < nchunks) {
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                        x_store(par ^ 1);
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    }
                    if (n + 2 < nchunks) x_load(n + 2);
                }
                load_w(wq[R * kBpg + p]);  // the same block kRG groups on
            }
            // the group is done: scale and zero point (Eq. 2)
            H2 s01, s23;
            s01.u = sc[0];
            s23.u = sc[1];
            const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
            const uint32_t z = zw >> zsh;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const float sp = s[cc] * Act::kCodeScale;                                         // FP16: 2^24 s
                const float sz = -s[cc] * ((float)((z >> (4 * cc)) & 15u) + Act::kCodeOffset);  // -s z
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        tot[rt][cc][i] = __builtin_fmaf(sp, part[rt][cc][i], __builtin_fmaf(sz, xsum[rt][i], tot[rt][cc][i]));
            }
        };

        // Ring places and chunk buffers are fixed per copy of the group's code: two copies where consecutive
        // groups differ in either, one where they do not.
        if constexpr (kRG == 2 || Sh::kChunks % 2 == 1) {
            for (uint32_t gi = 0; gi < (uint32_t)ng; gi += 2) {
                do_group(std::integral_constant<int, 0>{}, gi);
                if (gi + 1 < (uint32_t)ng) do_group(std::integral_constant<int, 1>{}, gi + 1);
            }
        } else {
            for (uint32_t gi = 0; gi < (uint32_t)ng; ++gi) do_group(std::integral_constant<int, 0>{}, gi);
        }
    }

    // Phase 3 inside the workgroup, then across workgroups (see w4a16_finish.h).  The sums are regrouped
    // here, once, into the four neighbouring columns a lane hands over per row.
    float4_t mine4[RT][4];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int i = 0; i < 4; ++i) mine4[rt][i] = (float4_t){tot[rt][0][i], tot[rt][1][i], tot[rt][2][i], tot[rt][3][i]};
    const auto write_mine = [&](float4_t *mine) {  // [row][column / 4] of the 64-column tile
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int i = 0; i < 4; ++i) mine[(16 * rt + 4 * g4 + i) * (kTileCols / 4) + j] = mine4[rt][i];
    };
    if (finish == kFinishAccumulator)
        reduce_and_finish<Act, Sh::kRowsX, kTileCols, 1, 4>(a, finish, sync, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
    else
        reduce_and_finish<Act, Sh::kRowsX, kTileCols, 4, 4>(a, finish, sync, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
}

// The waves' chunk buffers; the final sums reuse the space, a whole number of waves' tiles per round.
enum Loop { kLoopBlocks = 0, kLoopGroups = 1 };  // which kernel: any group size; group = 128

size_t lds_bytes(int rows_x, int waves, int loop)
{
    const int rt = rows_x / 16;
    const size_t wave_bytes = loop == kLoopGroups ? (rt == 1 ? GroupShape<1>::kWaveBytes : rt == 2 ? GroupShape<2>::kWaveBytes : GroupShape<4>::kWaveBytes)
                                                  : (rt == 1 ? Shape<1>::kWaveBytes : rt == 2 ? Shape<2>::kWaveBytes : Shape<4>::kWaveBytes);
    const size_t stage = (size_t)waves * wave_bytes;
    const size_t one = (size_t)rows_x * kTileCols * 4;
    size_t red = one * waves;
    if (red > 64 * 1024) red = 64 * 1024 / one * one;
    return stage > red ? stage : red;
}

struct Launch {
    int grid, row_blocks, red_waves;
    size_t lds;
};

// Grid and LDS of a launch; false if the shape is beyond the kernels' 32-bit offsets.
bool prepare(const GemmArgs &a, int rows_x, int waves, int loop, Launch *l)
{
    l->lds = lds_bytes(rows_x, waves, loop);
    l->red_waves = (int)(l->lds / ((size_t)rows_x * kTileCols * 4));
    if (l->red_waves < 1) return false;
    if (l->red_waves > waves) l->red_waves = waves;
    const unsigned long long rows = (unsigned long long)a.groups_per_split * (a.group / 8);
    if (rows * a.N * 4ull >= 0x7F000000ull) return false;  // slice-relative 32-bit buffer offsets
    if ((unsigned long long)a.M * a.K * 2ull >= 0x7F000000ull) return false;
    const int ntiles = (a.N + kTileCols - 1) / kTileCols;
    l->row_blocks = (a.M + rows_x - 1) / rows_x;
    const long long units = (long long)ntiles * a.split;
    const long long grid = (units + kXcds - 1) / kXcds * kXcds * l->row_blocks;
    if (grid > 0x7FFFFFFF) return false;
    l->grid = (int)grid;
    return true;
}

template <typename Kernel>
hipError_t launch_kernel(Kernel kernel, const Launch &l, const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream)
{
    if (l.lds > 48 * 1024) {  // beyond the default dynamic-LDS allowance
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)l.lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)l.grid), dim3(waves * 64), l.lds, stream, a, finish, sync, l.row_blocks, l.red_waves);
    return hipGetLastError();
}

template <typename Act>
hipError_t launch_rows(const Launch &l, const GemmArgs &a, int finish, unsigned long long *sync, int rows_x, int waves, int loop, hipStream_t stream)
{
    if (loop == kLoopGroups) {
        if (rows_x == 16) return launch_kernel(&tile_group_kernel<Act, 1>, l, a, finish, sync, waves, stream);
        if (rows_x == 32) return launch_kernel(&tile_group_kernel<Act, 2>, l, a, finish, sync, waves, stream);
        return launch_kernel(&tile_group_kernel<Act, 4>, l, a, finish, sync, waves, stream);
    }
    if (rows_x == 16) return launch_kernel(&tile_kernel<Act, 1>, l, a, finish, sync, waves, stream);
    if (rows_x == 32) return launch_kernel(&tile_kernel<Act, 2>, l, a, finish, sync, waves, stream);
    return launch_kernel(&tile_kernel<Act, 4>, l, a, finish, sync, waves, stream);
}

}  // namespace

hipError_t launch_tile(const GemmArgs &a, int finish, unsigned long long *sync, int rows_x, int waves, hipStream_t stream)
{
    if (waves < 4 || waves > 8 || a.group % (8 * kBlockRows) != 0) return hipErrorInvalidValue;
    if (rows_x != 16 && rows_x != 32 && rows_x != 64) return hipErrorInvalidValue;
    if (!finish_args_ok(a, finish, sync)) return hipErrorInvalidValue;
    const int loop = a.group == 128 ? kLoopGroups : kLoopBlocks;  // the loop over single blocks: 0.5-0.7 us slower on small shapes, equal on large
    Launch l;
    if (!prepare(a, rows_x, waves, loop, &l)) return hipErrorInvalidValue;
    if (a.bf16) return launch_rows<ActBF16>(l, a, finish, sync, rows_x, waves, loop, stream);
    return launch_rows<ActF16>(l, a, finish, sync, rows_x, waves, loop, stream);
}

}  // namespace w4a16
