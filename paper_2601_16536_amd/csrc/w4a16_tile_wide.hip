// W4A16 multiply, TILE family at 64 or 32 rows of X per workgroup (M > 16 on wide matrices), FP16, group = 128: one
// workgroup of FOUR waves per (64-column tile, 16 RT rows of X, K slice); at 64 rows each wave is alone on its SIMD
// with the whole register file.
//
// Why this form.  At 64 rows a wave issues 16 MFMAs 16x16x32 per block of 32 k, and what bounds the kernel is
// instruction issue (measured on M = 128, K = N = 8192): a vector instruction costs a wave 4 cycles, an MFMA 8 when
// vector instructions sit between it and the previous MFMA, 16 when it follows another MFMA.  The eight-wave form
// (w4a16_tile.hip) has 238 registers per wave: one group of weights in flight, X one block ahead, operands prepared
// just before their MFMAs, 95 vector instructions and 20 MFMAs per block, one kind after the other, and the waves
// wait a quarter of their time.  With four waves a wave has 512 registers, enough to
//   - keep the arithmetic exact and still drop the sum of x: the B operand is q - z as an exact FP16 integer
//     (twelve vector instructions per word instead of five, but no fifth MFMA per four, no 2^-4 scaling of X,
//     and Eq. 2's step is one FMA per output element and group, s (sum_k x_k (q_k - z)), instead of two);
//   - put the step of one group between the first MFMAs of the next (tile by tile: step, then the MFMA that restarts
//     the tile's sums);
//   - unpack the next block's operands and fetch its X operands from LDS between the MFMAs of the current block;
//   - keep two groups of weights in flight, and X three chunks ahead, loaded straight into LDS (loads return to a
//     wave in the order it asked, so X must be asked for as far ahead as the weights that were asked for just before).
// Arithmetic: products x (q - z) are exact in FP32, sums over a group in FP32 inside the MFMA, times s in FP32: the
// same values as the eight-wave form up to the order of the FP32 sums.
#include "w4a16_device.h"
#include "w4a16_finish.h"
#include "w4a16_internal.h"
#include <type_traits>

namespace w4a16 {
namespace {

constexpr int kTileCols = 64;
constexpr int kBlockRows = 4;   // packed rows per block: one MFMA step of 32 k
constexpr int kBpg = 4;         // blocks per group (group = 128)
constexpr int kXcds = 8;
constexpr int kWaves = 4;
constexpr int kRing = 2;        // groups of weights in flight per wave (registers): eight blocks, about 3 us, ahead
constexpr int kChunkBlocks = 2; // blocks per staged chunk of X: whole 128-byte lines of a row
constexpr int kBuffers = 4;     // chunks of X per wave in LDS: the one in use and three on their way

// Sizes that depend on the rows of X per workgroup, and the hand-written waits.  The compiler does not know that the
// loads into LDS must have landed before the LDS reads that use them: the waits are written by hand, as the number of
// vector-memory operations that may still be on their way (loads return to a wave in the order it asked); compiler
// fences around every fetch (x_fetch) keep the emitted order of the loads equal to the one counted here.  Per group
// a wave issues, in program order (see do_group), with X = kLoadsPerChunk:
//   block 0: W; block 1: W, X loads into LDS; block 2: W; block 3: scales, zero points, W, X loads into LDS.
template <int RT>
struct Wide {
    static constexpr int kRowsX = 16 * RT;
    static constexpr int kLoadsPerChunk = 2 * RT;              // wave-wide loads per chunk: eight rows of X each, 1 KiB
    static constexpr int kBufBytes = kLoadsPerChunk * 1024;    // a chunk in LDS: rows x 128 bytes, no padding
    static constexpr int kWaveBytes = kBuffers * kBufBytes;
    static constexpr int kPerGroup = 4 + 2 + 2 * kLoadsPerChunk;
    // at block 1, for the group's second chunk, asked for at block 3 two groups ago: one whole group + W + W since then
    static constexpr int kWaitChunk1 = kPerGroup + 2;
    // at block 3, for the next group's first chunk, asked for at block 1 of the group before: W, scales, zero points, W,
    // X loads; then W, W, X loads, W, scales, zero points, W
    static constexpr int kWaitChunk0 = (4 + kLoadsPerChunk) + (6 + kLoadsPerChunk);
    // at the start, for the first chunk: the first group's scales, zero points and weights (6), three chunks of X, the
    // second group's (6), and the first refill (3) were asked for after it
    static constexpr int kWaitFirst = 15 + 3 * kLoadsPerChunk;
    // vector instructions the schedule puts ahead of every MFMA: 48 per block for the next block's operands, and in a
    // group's first block 16 RT more for the step of the group before
    static constexpr int kValuFirst = RT == 4 ? 7 : 11, kValu = RT == 4 ? 3 : 6;
};

// The B operand q - z, exact in either 16-bit format, and what it takes per group: for the four columns of a lane the
// pair to subtract and the scale as a float.
struct GroupConst {
    uint32_t negz[4];
    float s[4];
};
__device__ __forceinline__ void group_scales(GroupConst &g, uint2_t sc)
{
    H2 s01, s23;
    s01.u = sc[0];
    s23.u = sc[1];
    g.s[0] = (float)s01.h[0];
    g.s[1] = (float)s01.h[1];
    g.s[2] = (float)s23.h[0];
    g.s[3] = (float)s23.h[1];
}

// FP16.  Byte e of a column's word holds the codes of k = 2e (bits 0-3) and 2e + 1 (bits 4-7); copied into both
// halves of a register and left where they are, under the exponent of 1024 (unit in the last place 1) and of 64 (unit
// 2^-4, i.e. bits 4-7 count ones), they read 1024 + q and 64 + q; minus 1024 + z and 64 + z.  k ascending.
struct CodesF16 {
    typedef ActF16 Act;
    static constexpr uint32_t kMask = 0x00F0000Fu, kMagic = 0x54006400u;
    static __device__ __forceinline__ GroupConst group_const(uint2_t sc, uint32_t z)
    {
        GroupConst g;
        group_scales(g, sc);
#pragma unroll
        for (int c = 0; c < 4; ++c) g.negz[c] = (((z >> (4 * c)) & 15u) * 0x00100001u) | 0xD400E400u;  // sign | 64 or 1024 | z in the bits that count ones
        return g;
    }
    static __device__ __forceinline__ ActF16::operand_t unpack(uint32_t w, uint32_t negz, uint32_t mask, uint32_t magic)
    {
        H2 zv;
        zv.u = negz;
        H8 r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // byte selectors of v_perm_b32: 0-3 pick from the second operand, 0x0c gives zero: byte e into both halves
            const uint32_t u = __builtin_amdgcn_perm(w, w, 0x0C000C00u + 0x00010001u * (uint32_t)e);
            H2 t;
            t.u = (u & mask) | magic;
            t.h = t.h + zv.h;
            r.u[e] = t.u;
        }
        return r.h;
    }
};

// (BF16 activations stay with the eight-wave form: gfx950 has no packed BF16 add, and q - z through FP32 costs more
// than that form's sum of x.)

// A chunk of X into LDS: each wave-wide load puts lane l's 16 bytes at (base + 16 l), 1 KiB per load.
template <int LOADS>
__device__ __forceinline__ void fetch_chunk(__amdgpu_buffer_rsrc_t rx, unsigned char *base, const uint32_t (&xg)[LOADS], uint32_t so)
{
    typedef __attribute__((address_space(3))) void *lds_ptr_t;
#pragma unroll
    for (int q = 0; q < LOADS; ++q) __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr_t)(base + q * 1024), 16, xg[q], so, 0, 0);
}

template <typename Codes, int RT>
__global__ __launch_bounds__(64 * kWaves) void tile_wide_kernel(const GemmArgs a, const int finish, unsigned long long *__restrict__ sync, const int row_blocks, const int red_waves)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef Wide<RT> Sh;
    constexpr int kRT = RT, kRowsX = Sh::kRowsX, kLoadsPerChunk = Sh::kLoadsPerChunk, kBufBytes = Sh::kBufBytes, kWaveBytes = Sh::kWaveBytes;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g4 = lane >> 4, j = lane & 15;

    // workgroup -> (column tile, K slice, row block): the row blocks of one (tile, slice) are neighbours on one XCD
    // (workgroup b runs on XCD b mod 8) and start together: the second reader finds the weights in that XCD's L2
    const int ntiles = (a.N + kTileCols - 1) / kTileCols;
    const int units = ntiles * a.split;
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
    const int m0 = rb * kRowsX;
    const int col0 = tile * kTileCols + 4 * j;
    const bool ok = col0 < a.N;

    // the slice's groups, and this wave's run of them: groups / waves each, the first groups % waves one more
    const int gbeg = slice * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.groups) gend = a.groups;
    const int groups = gend - gbeg;
    const int per = (int)((uint32_t)groups / (uint32_t)kWaves), extra = groups - per * kWaves;
    const int g0 = gbeg + per * wave + (wave < extra ? wave : extra);
    const int ng = per + (wave < extra ? 1 : 0);

    // every buffer descriptor ends where the wave's run ends: loads past the run are cut off by the hardware's
    // range check (zeros, no traffic)
    const uint32_t row_w = (uint32_t)a.N * 4u, row_s = (uint32_t)a.N * 2u, row_z = (uint32_t)(a.N >> 3) * 4u;
    const uint32_t step_w = kBlockRows * row_w;  // one block further
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Wp) + (size_t)g0 * 16 * a.N, 0, (uint32_t)ng * 16u * row_w, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.scales) + (size_t)g0 * a.N, 0, (uint32_t)ng * row_s, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Zp) + (size_t)g0 * (a.N >> 3), 0, zero_point_bytes(a.Zp, (uint32_t)ng * row_z), kRawBuffer);
    const uint32_t zfill = symmetric_fill(a.Zp);
    const uint32_t zsh = (uint32_t)(col0 & 4) * 4u;  // this lane's four nibbles in its zero-point word
    uint32_t vw = ok ? (uint32_t)(g4 * a.N + col0) * 4u : kOutOfRange;  // running offsets of the next block / group to load
    uint32_t vs = ok ? (uint32_t)col0 * 2u : kOutOfRange;
    uint32_t vz = ok ? (uint32_t)(col0 >> 3) * 4u : kOutOfRange;

    uint4_t wq[kRing * kBpg];  // the weights in flight
    auto load_w = [&](uint4_t &d) {
        d = __builtin_amdgcn_raw_buffer_load_b128(rw, vw, 0, 2);  // read once from DRAM: nontemporal
        vw += step_w;
    };
    // The scales and zero points of the groups in flight, asked for just ahead of their group's weights.
    uint2_t scq[kRing];
    uint32_t zwq[kRing];
    auto load_sz = [&](int place) {
        scq[place] = __builtin_amdgcn_raw_buffer_load_b64(rs, vs, 0, 0);
        zwq[place] = __builtin_amdgcn_raw_buffer_load_b32(rz, vz, 0, 0);
        vs += row_s;
        vz += row_z;
    };

    // ---- X: straight from global memory into this wave's LDS (four chunk buffers), no registers ----
    // A wave-wide load into LDS puts lane l's 16 bytes at (base + 16 l): eight lanes fetch the 128 contiguous bytes a
    // chunk takes of one row of X (eight packed rows), eight rows per load.  So that the MFMA's operand reads (sixteen
    // consecutive rows, one packed row) do not all fall into the same banks, lane (row r, place x) fetches packed row
    // x ^ r: within a row's 128 bytes the packed rows sit rotated by the row number.  X is staged as it is: the operand
    // order of the unpack (CodesF16) is the order of k.
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, (uint32_t)((size_t)a.M * a.K * 2), kRawBuffer);
    uint32_t xg[kLoadsPerChunk];
#pragma unroll
    for (int q = 0; q < kLoadsPerChunk; ++q) {
        const uint32_t rl = (uint32_t)lane >> 3, m = (uint32_t)m0 + (uint32_t)(8 * q) + rl;
        const uint32_t prow = (uint32_t)g0 * 16u + (((uint32_t)lane & 7u) ^ rl);
        xg[q] = m < (uint32_t)a.M ? (m * (uint32_t)a.K + prow * 8u) * 2u : kOutOfRange;
    }
    // The fences keep the compiler from moving other memory operations across the fetch: the hand-written waits
    // count the loads asked for after it, and the LDS reads of the buffer it refills must stay ahead of it.
    auto x_fetch = [&](int buffer, uint32_t chunk) {  // chunk of the wave's run into LDS buffer `buffer` (past the run: other k, unused)
        asm volatile("" ::: "memory");
        fetch_chunk<kLoadsPerChunk>(rx, smem + (size_t)wave * kWaveBytes + buffer * kBufBytes, xg, chunk * (kChunkBlocks * kBlockRows * 16u));
        asm volatile("" ::: "memory");
    };
    // this lane's A entry of block lb of a chunk, row tile 0: row j of the tile = load j / 8, row j % 8 of it; packed row 4 lb + g4
    uint32_t xa[kChunkBlocks];
#pragma unroll
    for (int lb = 0; lb < kChunkBlocks; ++lb)
        xa[lb] = (uint32_t)(wave * kWaveBytes + (j >> 3) * 1024 + (j & 7) * 128 + (((4 * lb + g4) ^ (j & 7)) * 16));

    float4_t tot[kRT][4];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
        for (int c = 0; c < 4; ++c) tot[rt][c] = (float4_t){0.f, 0.f, 0.f, 0.f};

    if (ng > 0) {
        // X of the first chunk and each group's scales go ahead of that group's weights: loads return in order
        x_fetch(0, 0);
#pragma unroll
        for (int h = 0; h < kRing; ++h) {
            load_sz(h);
#pragma unroll
            for (int p = 0; p < kBpg; ++p) load_w(wq[h * kBpg + p]);
            if (h == 0) {
                x_fetch(1, 1);
                x_fetch(2, 2);
                x_fetch(3, 3);
            }
        }
        uint32_t mask = Codes::kMask, magic = Codes::kMagic;
        asm volatile("" : "+v"(mask), "+v"(magic));  // kept in vector registers: v_and_or_b32 has no room for two constants
        const float4_t zero4 = {0.f, 0.f, 0.f, 0.f};

        // operands of the block in use and of the next one; the sums of the group in use
        typedef typename Codes::Act Act;
        typename Act::operand_t bop[2][4];
        uint4_t xop[2][kRT];
        float4_t part[kRT][4];
        GroupConst gc = Codes::group_const(scq[0], (zwq[0] | zfill) >> zsh);
        float s_prev[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) bop[0][c] = Codes::unpack(wq[0][c], gc.negz[c], mask, magic);
        load_sz(0);     // the same place, and its first block, kRing groups on (past the run: zeros, no traffic)
        load_w(wq[0]);
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
            for (int c = 0; c < 4; ++c) part[rt][c] = zero4;  // "the group before the first": nothing
        // chunk 0 has landed when at most the operations asked for after it are on their way
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(Sh::kWaitFirst) : "memory");
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) xop[0][rt] = *reinterpret_cast<const uint4_t *>(smem + xa[0] + rt * 2048);

        // One group from ring place R.  Entering, bop[0] and xop[0] hold its first block, gc its constants, s_prev and
        // part the previous group's scales and sums: Eq. 2's step for an output tile of the previous group,
        // tot += s part, sits just ahead of the MFMA that starts the tile's sums of this group.  Only this
        // wave touches its LDS and the LDS operations of one wave complete in order; the fences only keep the
        // compiler from moving them across the staging.
        auto do_group = [&](auto place, const uint32_t gi) {
            constexpr int R = decltype(place)::value;
            constexpr int RN = (R + 1) % kRing;
            constexpr int PC = R & 1, PP = PC ^ 1;  // parity of this group, of the next one: their chunks' LDS buffers
            float s_next[4];
#pragma unroll
            for (int p = 0; p < kBpg; ++p) {
                const int c = p / kChunkBlocks, lb = p % kChunkBlocks;
                // the next block's operands, independent of the MFMAs below
                if (p + 1 < kBpg) {
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) bop[(p + 1) & 1][cc] = Codes::unpack(wq[R * kBpg + p + 1][cc], gc.negz[cc], mask, magic);
                    load_w(wq[R * kBpg + p + 1]);  // the same block kRing groups on
                } else {
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) s_next[cc] = gc.s[cc];
                    gc = Codes::group_const(scq[RN], (zwq[RN] | zfill) >> zsh);  // the next group's first block
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) bop[0][cc] = Codes::unpack(wq[RN * kBpg][cc], gc.negz[cc], mask, magic);
                    load_sz(RN);
                    load_w(wq[RN * kBpg]);
                }
                // the next block's X operands: the other block of this chunk, or the first block of the next chunk, which
                // must have landed by now
                {
                    const int pn = (p + 1) % kBpg, lbn = pn % kChunkBlocks;
                    const int bn = p + 1 < kBpg ? 2 * PC + pn / kChunkBlocks : 2 * PP;  // its chunk's LDS buffer
                    if (lb == kChunkBlocks - 1) {
                        if (c == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(Sh::kWaitChunk1) : "memory");
                        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(Sh::kWaitChunk0) : "memory");
                    }
                    const unsigned char *xb = smem + xa[lbn] + bn * kBufBytes;
#pragma unroll
                    for (int rt = 0; rt < kRT; ++rt) xop[(p + 1) & 1][rt] = *reinterpret_cast<const uint4_t *>(xb + rt * 2048);
                }
                // this block's MFMAs; ahead of the group's first ones the previous group's step
#pragma unroll
                for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) {
                        if (p == 0) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) tot[rt][cc][i] = __builtin_fmaf(s_prev[cc], part[rt][cc][i], tot[rt][cc][i]);
                        }
                        part[rt][cc] = Act::mfma(Act::x_operand(xop[p & 1][rt]), bop[p & 1][cc], p == 0 ? zero4 : part[rt][cc]);
                    }
                // the schedule of the block: every MFMA with its share of the vector instructions around it
#pragma unroll
                for (int i = 0; i < 4 * kRT; ++i) {
                    if (p == 0) __builtin_amdgcn_sched_group_barrier(0x002, Sh::kValuFirst, 0);
                    else __builtin_amdgcn_sched_group_barrier(0x002, Sh::kValu, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                if (lb == kChunkBlocks - 1) {
                    // This chunk's last block is in registers (xop[p & 1]): its buffer takes the chunk four chunks on.
                    x_fetch(2 * PC + c, gi * 2 + c + 4);
                }
            }
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) s_prev[cc] = s_next[cc];
        };

        for (uint32_t gi = 0; gi < (uint32_t)ng; gi += kRing) {
            do_group(std::integral_constant<int, 0>{}, gi);
            if (gi + 1 < (uint32_t)ng) do_group(std::integral_constant<int, 1>{}, gi + 1);
        }
        // the fetches past the run's end write into this wave's LDS too: they must have landed before the final sums
        // reuse the space
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // the last group's step
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
            for (int cc = 0; cc < 4; ++cc)
#pragma unroll
                for (int i = 0; i < 4; ++i) tot[rt][cc][i] = __builtin_fmaf(s_prev[cc], part[rt][cc][i], tot[rt][cc][i]);
    }

    // Phase 3 inside the workgroup, then across workgroups (see w4a16_finish.h).  The sums are regrouped
    // here, once, into the four neighbouring columns a lane hands over per row.
    float4_t mine4[kRT][4];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
        for (int i = 0; i < 4; ++i) mine4[rt][i] = (float4_t){tot[rt][0][i], tot[rt][1][i], tot[rt][2][i], tot[rt][3][i]};
    const auto write_mine = [&](float4_t *mine) {  // [row][column / 4] of the 64-column tile
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
            for (int i = 0; i < 4; ++i) mine[(16 * rt + 4 * g4 + i) * (kTileCols / 4) + j] = mine4[rt][i];
    };
    if (finish == kFinishAccumulator) {
        // one atomic add per output: consecutive lanes on consecutive outputs (w4a16_finish.h)
        reduce_and_finish<typename Codes::Act, kRowsX, kTileCols, 1, 4>(a, finish, sync, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
        return;
    }
    // Y, or FP32 partials: the waves exchange their sums in the layout the registers have.  The 4 kRT (row tile, i)
    // pieces of a lane are dealt out to the four waves, kRT neighbouring ones each; a wave writes the pieces it does
    // not own into its own staging space (nobody else ever touched it, and its loads have landed: no barrier before),
    // and after one barrier adds up its pieces, in the order of the waves whoever the owner is, and stores them.
    float4_t *const own_space = reinterpret_cast<float4_t *>(smem + (size_t)wave * kWaveBytes);
#pragma unroll
    for (int u = 0; u < 4 * kRT; ++u)
        if (u / kRT != wave) own_space[u * 64 + lane] = mine4[u >> 2][u & 3];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 4 * kRT; ++u) {
        if (u / kRT != wave) continue;  // uniform
        float4_t v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (w == wave) v += mine4[u >> 2][u & 3];
            else v += reinterpret_cast<const float4_t *>(smem + (size_t)w * kWaveBytes)[u * 64 + lane];
        }
        const int m = m0 + 16 * (u >> 2) + 4 * g4 + (u & 3), col = tile * kTileCols + 4 * j;
        if (m >= a.M || col >= a.N) continue;  // N is a multiple of 8: the four columns are inside together
        const size_t out = (size_t)m * a.N + col;
        typedef typename Codes::Act Act;
        if (finish == kFinishDirect)
            *reinterpret_cast<uint2_t *>(a.Y + out) = (uint2_t){Act::pack2(v[0], v[1]), Act::pack2(v[2], v[3])};
        else
            *reinterpret_cast<float4_t *>(a.partials + (size_t)slice * a.M * a.N + out) = v;
    }
}

template <int RT>
hipError_t launch_rt(const GemmArgs &a, int finish, unsigned long long *sync, hipStream_t stream)
{
    typedef Wide<RT> Sh;
    const size_t stage = (size_t)kWaves * Sh::kWaveBytes;
    const size_t one = (size_t)Sh::kRowsX * kTileCols * 4;  // a wave's result tile in fp32: the final sums reuse the space
    const size_t red = one * kWaves;
    const size_t lds = stage > red ? stage : red;
    const int ntiles = (a.N + kTileCols - 1) / kTileCols;
    const int row_blocks = (a.M + Sh::kRowsX - 1) / Sh::kRowsX;
    const long long grid = ((long long)ntiles * a.split + kXcds - 1) / kXcds * kXcds * row_blocks;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tile_wide_kernel<CodesF16, RT>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);  // beyond the default dynamic-LDS allowance
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((tile_wide_kernel<CodesF16, RT>), dim3((unsigned)grid), dim3(64 * kWaves), lds, stream, a, finish, sync, row_blocks, kWaves);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_tile_wide(const GemmArgs &a, int finish, unsigned long long *sync, int rows_x, hipStream_t stream)
{
    if (a.group != 128 || a.bf16 || (rows_x != 32 && rows_x != 64)) return hipErrorInvalidValue;
    if (!finish_args_ok(a, finish, sync)) return hipErrorInvalidValue;
    const unsigned long long rows = (unsigned long long)a.groups_per_split * (a.group / 8);
    if (rows * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;  // slice-relative 32-bit buffer offsets
    if ((unsigned long long)a.M * a.K * 2ull >= 0x7F000000ull) return hipErrorInvalidValue;
    return rows_x == 64 ? launch_rt<4>(a, finish, sync, stream) : launch_rt<2>(a, finish, sync, stream);
}

}  // namespace w4a16
