// W4A16 multiply for many rows of X (M > 16), group = 128, FP16, an opt-in form (knob "tile_deq"): the TILE family's
// workgroup (one 64-column tile x 16 RT rows of X x one K slice, eight waves that own contiguous runs of the
// slice's groups and meet in LDS), with Algorithm 1's Phase 1 taken literally: a wave dequantizes its weights to
// FP16 in registers,
//     B = fp16(s (q - z))                                      (Eq. 2)
// and the FP16 MFMA (Phase 2) accumulates x B over the wave's whole run in FP32.
//
// Why it exists beside w4a16_tile.hip (codes as exact subnormal operands, scale and zero point applied per group
// in FP32): with 64 rows of X per workgroup that form is bound by instruction issue (measured on M = 128,
// K = N = 8192: 115 vector instructions and 20 MFMAs per block of 32 k and wave, mostly one kind after the other):
// 2 FMAs per output element and group for Eq. 2, a fifth MFMA per four for sum_k x_k, the 2^-4 scaling of every
// second x, and two accumulator sets (128 registers) that leave no room to prepare the next operands while the MFMAs
// of the current ones run.  Here the unpack costs more (16 instead of 5 instructions per eight weights) but nothing
// else is left: no step per group, no sum of x, X staged as it is, one accumulator set; the registers that frees
// hold the next block's operands, unpacked between the current block's MFMAs, and two groups of weights in flight:
// 65 vector instructions and 16 MFMAs per block, 28.7 us against 33.3 us on that shape.
//
// Why it is not the scheduler's choice: the price is one FP16 rounding per weight (relative 2^-11), the paper's own
// Phase 1.  Random in sign, it adds up to about sqrt(K) rms(x) rms(w) 2^-12.5: measured on that shape, every
// output, 0.55 of the tolerance 1e-2 (1 + |ref|) where the exact-code form spends 0.05, and it grows with sqrt(K)
// and with the magnitude of X (activations with outlier channels would exceed the tolerance).  At 32 and 16 rows
// of X per workgroup, where fewer MFMAs share an unpacked word, it is also 5 to 15 % slower than the exact form.
//
// Unpack, eight codes of consecutive k in one 32-bit word, operand k order 0,1 | 2,3 | 4,5 | 6,7 (X needs no
// reordering): see dequant8.
#include "w4a16_device.h"
#include "w4a16_finish.h"
#include "w4a16_internal.h"
#include <type_traits>

#ifdef W4A16_TIMELINE
// Profiling build only: per-wave time stamps (kernel entry, first chunk of X staged, loop end, exit; 100 MHz ticks),
// eight 64-bit words per wave, workgroup-major.  w4a16_timeline_buffer_tile sets where they go (NULL = nowhere).
__device__ unsigned long long *g_timeline_tile;
extern "C" int w4a16_timeline_buffer_tile(void *device_words)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_timeline_tile), &device_words, sizeof device_words);
}
#endif

namespace w4a16 {
namespace {

constexpr int kTileCols = 64;
constexpr int kBlockRows = 4;   // packed rows per block: one MFMA step of 32 k
constexpr int kBpg = 4;         // blocks per group (group = 128)
constexpr int kXcds = 8;

template <int RT>
struct DeqShape {
    static constexpr int kRowsX = 16 * RT;
    static constexpr int kChunkBlocks = RT == 4 ? 2 : 4;         // blocks per staged chunk of X: whole 128-byte lines of a row
    static constexpr int kChunks = kBpg / kChunkBlocks;          // chunks per group
    static constexpr int kRingGroups = 2;                        // groups of weights in flight per wave (registers)
    static constexpr int kLanesPerRow = 4 * kChunkBlocks;        // lanes that fetch one row's bytes of a chunk (16 bytes each)
    static constexpr int kRowsPerLoad = 64 / kLanesPerRow;       // rows of X one wave-wide load covers
    static constexpr int kRowStride = kRowsX + 1;                // LDS entries per packed row: odd, so that the eight lanes of a
                                                                 // write pass (one row, eight packed rows) hit different banks
    static constexpr int kPerLane = kChunkBlocks * kBlockRows * kRowsX / 64;
    static constexpr int kBufBytes = kChunkBlocks * kBlockRows * kRowStride * 16;
    static constexpr int kWaveBytes = 2 * kBufBytes;
};

// (s, s) and -(1024 + z), -(64 + z), for the four columns of a lane
struct GroupConst {
    uint32_t s2[4], negz[4];
};
__device__ __forceinline__ GroupConst group_const(uint2_t sc, uint32_t z)
{
    GroupConst g;
    g.s2[0] = __builtin_amdgcn_perm(sc[0], sc[0], 0x01000100u);
    g.s2[1] = __builtin_amdgcn_perm(sc[0], sc[0], 0x03020302u);
    g.s2[2] = __builtin_amdgcn_perm(sc[1], sc[1], 0x01000100u);
    g.s2[3] = __builtin_amdgcn_perm(sc[1], sc[1], 0x03020302u);
#pragma unroll
    for (int c = 0; c < 4; ++c) g.negz[c] = (((z >> (4 * c)) & 15u) * 0x00100001u) | 0xD400E400u;  // sign | 64 or 1024 | z in the bits that count ones
    return g;
}

// One column's word -> its eight FP16 weights, k ascending.  Byte e of the word holds the codes of k = 2e (bits 0-3)
// and 2e + 1 (bits 4-7); left where they are, under the exponent of 1024 (unit in the last place 1) and of 64 (unit
// 2^-4, i.e. bits 4-7 count ones), they read 1024 + q and 64 + q.  `mask` and `magic` come in vector registers so
// that the compiler can take v_and_or_b32 (which has no room for two constants).
__device__ __forceinline__ half8_t dequant8(uint32_t w, uint32_t s2, uint32_t negz, uint32_t mask, uint32_t magic)
{
    H2 sv, zv;
    sv.u = s2;
    zv.u = negz;
    H8 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        // byte selectors of v_perm_b32: 0-3 pick from the second operand, 0x0c gives zero: byte e into both halves
        const uint32_t u = __builtin_amdgcn_perm(w, w, 0x0C000C00u + 0x00010001u * (uint32_t)e);
        H2 t;
        t.u = (u & mask) | magic;
        t.h = (t.h + zv.h) * sv.h;
        r.u[e] = t.u;
    }
    return r.h;
}

template <int RT>
__global__ __launch_bounds__(512) void tile_deq_kernel(const GemmArgs a, const int finish, unsigned long long *__restrict__ sync, const int row_blocks, const int red_waves)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
#ifdef W4A16_TIMELINE
    const unsigned long long T0 = __builtin_amdgcn_s_memrealtime();
    unsigned long long T1 = T0;
#endif
    typedef DeqShape<RT> Sh;
    constexpr int kValuPerMfma = RT == 4 ? 5 : (RT == 2 ? 9 : 18);  // about 70 vector instructions per block of 4 RT MFMAs

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = blockDim.x >> 6;
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
    const int m0 = rb * Sh::kRowsX;
    const int col0 = tile * kTileCols + 4 * j;
    const bool ok = col0 < a.N;

    // the slice's groups, and this wave's run of them: groups / waves each, the first groups % waves one more
    const int gbeg = slice * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.groups) gend = a.groups;
    const int groups = gend - gbeg;
    const int per = (int)((uint32_t)groups / (uint32_t)waves), extra = groups - per * waves;
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

    constexpr int kRG = Sh::kRingGroups;
    uint4_t wq[kRG * kBpg];  // the weights in flight
    auto load_w = [&](uint4_t &d) {
        d = __builtin_amdgcn_raw_buffer_load_b128(rw, vw, 0, 2);  // read once from DRAM: nontemporal
        vw += step_w;
    };
    // The scales and zero points of the groups in flight, asked for just ahead of their group's weights: loads
    // return in order, so they are there when the group's first block is.
    uint2_t scq[kRG];
    uint32_t zwq[kRG];
    auto load_sz = [&](int place) {
        scq[place] = __builtin_amdgcn_raw_buffer_load_b64(rs, vs, 0, 0);
        zwq[place] = __builtin_amdgcn_raw_buffer_load_b32(rz, vz, 0, 0);
        vs += row_s;
        vz += row_z;
    };

    // ---- X: this wave's LDS (two chunk buffers), chunk loader and chunk writer ----
    // kLanesPerRow neighbouring lanes fetch the contiguous bytes a chunk takes of one row of X (whole 128-byte
    // lines, or two of them); load q of a lane: row q kRowsPerLoad + lane / kLanesPerRow, packed row lane % kLanesPerRow.
    // X is staged as it is: the operand order of dequant8 is the order of k.
    unsigned char *wl = smem + (size_t)wave * Sh::kWaveBytes;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, (uint32_t)((size_t)a.M * a.K * 2), kRawBuffer);
    uint32_t xg[Sh::kPerLane];
#pragma unroll
    for (int q = 0; q < Sh::kPerLane; ++q) {
        const uint32_t m = (uint32_t)m0 + (uint32_t)(q * Sh::kRowsPerLoad + lane / Sh::kLanesPerRow);
        const uint32_t prow = (uint32_t)g0 * 16u + (uint32_t)(lane % Sh::kLanesPerRow);
        xg[q] = m < (uint32_t)a.M ? (m * (uint32_t)a.K + prow * 8u) * 2u : kOutOfRange;
    }
    const uint32_t xl0 = (uint32_t)(((lane % Sh::kLanesPerRow) * Sh::kRowStride + lane / Sh::kLanesPerRow) * 16);
    uint4_t xd[Sh::kPerLane];
    auto x_load = [&](uint32_t chunk) {  // chunk of the wave's run
        const uint32_t so = chunk * (Sh::kChunkBlocks * kBlockRows * 16u);
#pragma unroll
        for (int q = 0; q < Sh::kPerLane; ++q) xd[q] = __builtin_amdgcn_raw_buffer_load_b128(rx, xg[q], so, 0);
    };
    auto x_store = [&](int par) {
#pragma unroll
        for (int q = 0; q < Sh::kPerLane; ++q)
            *reinterpret_cast<uint4_t *>(wl + par * Sh::kBufBytes + xl0 + q * Sh::kRowsPerLoad * 16) = xd[q];
    };

    float4_t tot[RT][4];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int c = 0; c < 4; ++c) tot[rt][c] = (float4_t){0.f, 0.f, 0.f, 0.f};

    if (ng > 0) {
        // X of the first chunk and the first group's scales go ahead of the weights: loads return in order
        const uint32_t nchunks = (uint32_t)ng * Sh::kChunks;
        x_load(0);
#pragma unroll
        for (int h = 0; h < kRG; ++h) {
            load_sz(h);
#pragma unroll
            for (int p = 0; p < kBpg; ++p) load_w(wq[h * kBpg + p]);
        }
        x_store(0);
#ifdef W4A16_TIMELINE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        T1 = __builtin_amdgcn_s_memrealtime();
#endif
        if (nchunks > 1) x_load(1);

        const uint32_t xa0 = (uint32_t)(wave * Sh::kWaveBytes + (g4 * Sh::kRowStride + j) * 16);  // A entry of block 0, row tile 0
        uint32_t mask = 0x00F0000Fu, magic = 0x54006400u;
        asm volatile("" : "+v"(mask), "+v"(magic));  // kept in vector registers

        // The operands of the block in use and of the next one: the next block is dequantized (vector ALU) between
        // the MFMAs of the current one.  Measured on this GPU: an MFMA that follows vector instructions costs the
        // wave 8 cycles of issue, one that follows another MFMA 16.
        half8_t bop[2][4];
        GroupConst gc = group_const(scq[0], (zwq[0] | zfill) >> zsh);
#pragma unroll
        for (int c = 0; c < 4; ++c) bop[0][c] = dequant8(wq[0][c], gc.s2[c], gc.negz[c], mask, magic);
        load_sz(0);     // the same group, and its first block, kRG groups on (past the run: zeros, no traffic)
        load_w(wq[0]);

        // One group: its four blocks from ring place R, chunk buffers by parity of the chunk number.  Entering, bop[0]
        // holds the group's first block.  Only this wave touches its LDS and the LDS operations of one wave complete
        // in order; the fences only keep the compiler from moving them across the staging.
        auto do_group = [&](auto half, const uint32_t gi) {
            constexpr int H = decltype(half)::value;  // parity of the group in the run: its chunk buffers
            constexpr int R = H % kRG;                 // its place in the ring
            constexpr int RN = (H + 1) % kRG;          // the next group's
#pragma unroll
            for (int p = 0; p < kBpg; ++p) {
                constexpr int CB = Sh::kChunkBlocks;
                const int c = p / CB, lb = p % CB;
                const int par = (H * Sh::kChunks + c) & 1;
                const unsigned char *xb = smem + xa0 + par * Sh::kBufBytes + lb * (kBlockRows * Sh::kRowStride * 16);
                H8 x[RT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) x[rt].u = *reinterpret_cast<const uint4_t *>(xb + rt * 256);
                // the next block's operands: independent of the MFMAs below, which run meanwhile
                if (p + 1 < kBpg) {
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) bop[(p + 1) & 1][cc] = dequant8(wq[R * kBpg + p + 1][cc], gc.s2[cc], gc.negz[cc], mask, magic);
                    load_w(wq[R * kBpg + p + 1]);
                } else {
                    gc = group_const(scq[RN], (zwq[RN] | zfill) >> zsh);  // the next group's first block
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) bop[0][cc] = dequant8(wq[RN * kBpg][cc], gc.s2[cc], gc.negz[cc], mask, magic);
                    load_sz(RN);
                    load_w(wq[RN * kBpg]);
                }
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc)
                        tot[rt][cc] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x[rt].h, bop[p & 1][cc], tot[rt][cc], 0, 0, 0);
                // the schedule of this step: the X operands, then every MFMA followed by its share of the vector
                // instructions that prepare the next block (left alone, the compiler puts those first)
                __builtin_amdgcn_sched_group_barrier(0x100, RT, 0);
#pragma unroll
                for (int i = 0; i < 4 * RT; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);
                }
                if (lb == CB - 1) {
                    // The chunk is done.  Its successor's X, asked for a chunk ago, goes to the other buffer, and the
                    // chunk after that is asked for.
                    const uint32_t n = gi * Sh::kChunks + c;  // this chunk of the run
                    if (n + 1 < nchunks) {
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                        x_store(par ^ 1);
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    }
                    if (n + 2 < nchunks) x_load(n + 2);
                }
            }
        };

        // Ring places and chunk buffers are fixed per copy of the group's code: two copies.
        for (uint32_t gi = 0; gi < (uint32_t)ng; gi += 2) {
            do_group(std::integral_constant<int, 0>{}, gi);
            if (gi + 1 < (uint32_t)ng) do_group(std::integral_constant<int, 1>{}, gi + 1);
        }
    }

#ifdef W4A16_TIMELINE
    asm volatile("" ::"v"(tot[0][0][0]));
    const unsigned long long T2 = __builtin_amdgcn_s_memrealtime();
#endif
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
        reduce_and_finish<ActF16, Sh::kRowsX, kTileCols, 1, 4>(a, finish, sync, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
    else
        reduce_and_finish<ActF16, Sh::kRowsX, kTileCols, 4, 4>(a, finish, sync, smem, write_mine, red_waves, m0, tile * kTileCols, slice);
#ifdef W4A16_TIMELINE
    if (g_timeline_tile && lane == 0) {
        unsigned long long *p = g_timeline_tile + ((size_t)blockIdx.x * 8 + wave) * 8;
        unsigned xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        p[0] = T0; p[1] = T1; p[2] = T2; p[3] = __builtin_amdgcn_s_memrealtime(); p[4] = xcc; p[5] = (unsigned long long)ng; p[6] = 0;
    }
#endif
}

template <int RT>
hipError_t launch_rt(const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream)
{
    typedef DeqShape<RT> Sh;
    const size_t stage = (size_t)waves * Sh::kWaveBytes;
    const size_t one = (size_t)Sh::kRowsX * kTileCols * 4;  // a wave's result tile in fp32: the final sums reuse the space
    size_t red = one * waves;
    if (red > 64 * 1024) red = 64 * 1024 / one * one;
    const size_t lds = stage > red ? stage : red;
    int red_waves = (int)(lds / one);
    if (red_waves > waves) red_waves = waves;
    const int ntiles = (a.N + kTileCols - 1) / kTileCols;
    const int row_blocks = (a.M + Sh::kRowsX - 1) / Sh::kRowsX;
    const long long grid = ((long long)ntiles * a.split + kXcds - 1) / kXcds * kXcds * row_blocks;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (lds > 48 * 1024) {  // beyond the default dynamic-LDS allowance
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tile_deq_kernel<RT>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(tile_deq_kernel<RT>, dim3((unsigned)grid), dim3(waves * 64), lds, stream, a, finish, sync, row_blocks, red_waves);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_tile_deq(const GemmArgs &a, int finish, unsigned long long *sync, int rows_x, int waves, hipStream_t stream)
{
    if (waves < 4 || waves > 8 || a.group != 128 || a.bf16) return hipErrorInvalidValue;
    if (rows_x != 16 && rows_x != 32 && rows_x != 64) return hipErrorInvalidValue;
    if (!finish_args_ok(a, finish, sync)) return hipErrorInvalidValue;
    const unsigned long long rows = (unsigned long long)a.groups_per_split * (a.group / 8);
    if (rows * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;  // slice-relative 32-bit buffer offsets
    if ((unsigned long long)a.M * a.K * 2ull >= 0x7F000000ull) return hipErrorInvalidValue;
    if (rows_x == 16) return launch_rt<1>(a, finish, sync, waves, stream);
    if (rows_x == 32) return launch_rt<2>(a, finish, sync, waves, stream);
    return launch_rt<4>(a, finish, sync, waves, stream);
}

}  // namespace w4a16
