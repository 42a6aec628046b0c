// W4A16 multiply for M >= 5: one workgroup per (64-column tile, block of 16 RT
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
// in double-buffered chunks of one or two blocks, and so never waits at a
// workgroup barrier before the final sum.  Four lanes fetch the 64 contiguous
// bytes a block takes of one row of X; the LDS rows are padded by four entries so
// that these writes, and the MFMA's reads, are free of bank conflicts.
//
// The row blocks of one column tile read the same weights.  Workgroups are
// numbered so that they sit on the same XCD (workgroup b runs on XCD b mod 8) and
// start together: the second reader finds the weights in that XCD's L2.
#include "w4a16_device.h"
#include "w4a16_finish.h"
#include "w4a16_internal.h"

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

template <int RT>
__global__ __launch_bounds__(512) void tile_kernel(const GemmArgs a, unsigned long long *__restrict__ acc, const int row_blocks, const int red_waves)
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
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int rb = local % row_blocks, unit = (local / row_blocks) * kXcds + xcd;
    if (unit >= units) return;  // the grid is rounded up to whole XCD rounds
    const int tile = unit % ntiles, slice = unit / ntiles;
    const int m0 = rb * Sh::kRowsX;
    const int col0 = tile * kTileCols + 4 * j;
    const bool ok = col0 < a.N;

    // the workgroup's K slice: groups, packed rows, blocks; this wave's run of blocks
    const int gbeg = slice * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.K / a.group) gend = a.K / a.group;
    const int groups = gend - gbeg;
    const int rows = groups * (a.group / 8);
    const int row_base = gbeg * (a.group / 8);
    const uint32_t nblocks = (uint32_t)rows / kBlockRows;
    const uint32_t bpg = (uint32_t)a.group / (8 * kBlockRows);  // blocks per group
    const uint32_t wb0 = (uint32_t)((unsigned long long)nblocks * wave / waves);
    const uint32_t wb1 = (uint32_t)((unsigned long long)nblocks * (wave + 1) / waves);

    const uint32_t row_w = (uint32_t)a.N * 4u, row_s = (uint32_t)a.N * 2u, row_z = (uint32_t)(a.N >> 3) * 4u;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Wp) + (size_t)row_base * a.N, 0, (uint32_t)rows * row_w, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.scales) + (size_t)gbeg * a.N, 0, (uint32_t)groups * row_s, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Zp) + (size_t)gbeg * (a.N >> 3), 0, (uint32_t)groups * row_z, kRawBuffer);
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
        r.zw = __builtin_amdgcn_raw_buffer_load_b32(rz, vz, gu * row_z, 0);
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
            *reinterpret_cast<uint4_t *>(wl + par * Sh::kBufBytes + xl[q]) = permute_x(d[q]);
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
    // sum_k x_k over a block comes from the MFMA too: X against ones (16 where the staged x was divided by 16)
    const half8_t ones = {(_Float16)1.f, (_Float16)1.f, (_Float16)16.f, (_Float16)16.f, (_Float16)1.f, (_Float16)1.f, (_Float16)16.f, (_Float16)16.f};
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
                half8_t bop[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) bop[c] = unpack8(buf[p].w[c], masks);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    H8 x;
                    x.u = *reinterpret_cast<const uint4_t *>(xb + rt * 256);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        part[rt][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x.h, bop[c], part[rt][c], 0, 0, 0);
                    xsum[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x.h, ones, xsum[rt], 0, 0, 0);
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
                        const float sp = s[c] * 16777216.0f;                       // 2^24 s
                        const float sz = -s[c] * (float)((zw >> (4 * c)) & 15u);   // -s z
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
    if (a.split > 1 && !a.partials)
        reduce_and_finish<Sh::kRowsX, kTileCols, 1, 4>(a, acc, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
    else
        reduce_and_finish<Sh::kRowsX, kTileCols, 4, 4>(a, acc, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
}

template <int RT>
hipError_t launch_rt(const GemmArgs &a, unsigned long long *acc, int waves, hipStream_t stream)
{
    typedef Shape<RT> Sh;
    const size_t lds = tile_lds_bytes(Sh::kRowsX, waves);
    int red_waves = (int)(lds / Sh::kOutBytes);
    if (red_waves < 1) return hipErrorInvalidValue;
    if (red_waves > waves) red_waves = waves;
    const unsigned long long rows = (unsigned long long)a.groups_per_split * (a.group / 8);
    if (rows * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;  // slice-relative 32-bit buffer offsets
    if ((unsigned long long)a.M * a.K * 2ull >= 0x7F000000ull) return hipErrorInvalidValue;
    const int ntiles = (a.N + kTileCols - 1) / kTileCols;
    const int row_blocks = (a.M + Sh::kRowsX - 1) / Sh::kRowsX;
    const long long units = (long long)ntiles * a.split;
    const long long grid = (units + kXcds - 1) / kXcds * kXcds * row_blocks;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (lds > 48 * 1024) {  // beyond the default dynamic-LDS allowance
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tile_kernel<RT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((tile_kernel<RT>), dim3((unsigned)grid), dim3(waves * 64), lds, stream, a, acc, row_blocks, red_waves);
    return hipGetLastError();
}

}  // namespace

// The waves' chunk buffers; the final sums reuse the space, a whole number of waves' tiles per round.
size_t tile_lds_bytes(int rows_x, int waves)
{
    const size_t stage = (size_t)waves * (rows_x == 16 ? Shape<1>::kWaveBytes : rows_x == 32 ? Shape<2>::kWaveBytes : Shape<4>::kWaveBytes);
    const size_t one = (size_t)rows_x * kTileCols * 4;
    size_t red = one * waves;
    if (red > 64 * 1024) red = 64 * 1024 / one * one;
    return stage > red ? stage : red;
}

hipError_t launch_tile(const GemmArgs &a, unsigned long long *acc, int rows_x, int waves, hipStream_t stream)
{
    if (waves < 4 || waves > 8 || a.group % (8 * kBlockRows) != 0) return hipErrorInvalidValue;
    if (a.split > 1 && !acc && !a.partials) return hipErrorInvalidValue;
    if (a.split > 1 && acc && a.split > 255) return hipErrorInvalidValue;
    GemmArgs b = a;
    if (acc || a.split == 1) b.partials = nullptr;  // the kernel reads the finish mode off this pointer
    if (rows_x == 16) return launch_rt<1>(b, acc, waves, stream);
    if (rows_x == 32) return launch_rt<2>(b, acc, waves, stream);
    if (rows_x == 64) return launch_rt<4>(b, acc, waves, stream);
    return hipErrorInvalidValue;
}

}  // namespace w4a16
