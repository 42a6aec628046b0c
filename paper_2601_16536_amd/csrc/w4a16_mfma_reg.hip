// W4A16 multiply with the weights unpacked straight into MFMA operand registers.
//
// Computes the Split-K partial products C_i = A * B_i of Algorithm 1, Phase 2,
// where B_i = s (W - z) (Eq. 2) restricted to the i-th K slice -- but B_i never
// exists in memory (Algorithm 1, Phase 1 writes it to a workspace; that round
// trip is the bottleneck Section 4.2 diagnoses).  Each lane loads 16 bytes of
// packed codes (four columns x eight k) and feeds them to 16x16x32 fp16 MFMAs
// after five integer instructions per 32-bit word:
//
//   A nibble left in place in bits 0-3 of an fp16 whose other bits are zero IS
//   the subnormal fp16 number q * 2^-24; in bits 4-7 it is q * 2^-20.  The MFMA
//   takes subnormal inputs exactly, so masking a word with 0x000F000F and
//   0x00F000F0 (and the same after a shift by 8) yields the four operand
//   registers directly.  X is staged with the k positions that meet the
//   bits-4-7 nibbles divided by 16, so every product carries the same 2^-24.
//
// With P = 2^-24 sum_k x_k q_k (fp32, from the MFMA) over one unit of k inside a
// quantisation group, Eq. 2 gives
//
//   sum_k x_k s (q_k - z) = (2^24 s) P - (s z) sum_k x_k
//
// applied in fp32 once per (unit, column); the unit sums of X are computed when
// X is staged.  Nothing is rounded to fp16 before the final cast.
//
// Work split: a workgroup is four waves side by side along N (4 x 64 columns, so
// every packed row it touches is a contiguous 1 KiB), all walking the same K
// slice.  blockIdx.x is the slice (so the slices of one column tile land on
// different XCDs and each XCD's L2 sees only an eighth of X), blockIdx.y the
// column tile, blockIdx.z a tile of 16 rows of X.  With S > 1 the slice results
// go to the fp32 workspace and the second pass (Algorithm 1, Phase 3) adds them
// in slice order and casts to fp16; the kernel boundary is Algorithm 1's "wait
// for all cores".  (A last-arriver reduction inside this kernel was measured:
// the device-scope fence it needs on this multi-die GPU costs more than the
// second launch.)
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

// What a lane holds of one unit = STEPS x 32 consecutive k of its 4 columns.
template <int STEPS>
struct Unit {
    uint4_t w[STEPS];  // packed codes, row 4t + lane/16 of the unit, columns col0..col0+3
    uint2_t sc;        // four fp16 scales
    uint32_t zw;       // the zero-point word that holds the four columns
};

struct Streams {
    __amdgpu_buffer_rsrc_t w, s, z;  // slice-relative buffers: unit u of the slice starts at u * bytes_per_unit
    uint32_t vw, vs, vz;             // this lane's byte offsets inside a unit / scale row / zero row
    uint32_t unit_w, row_w;          // bytes per unit and per packed row of Wp
    uint32_t row_s, row_z;           // bytes per row of scales / zeros
};

// Loads unit `u` (slice-relative) if u < n, else nothing (registers become 0).
// Weights are read once: nontemporal, so they do not push X and the scales out of L2.
template <int STEPS>
__device__ __forceinline__ void load_unit(Unit<STEPS> &r, const Streams &st, int u, int n, int g_of_unit_num, int g_of_unit_den)
{
    // Past the end of the slice the lane offset (which the hardware range-checks
    // against the slice size) is pushed out of range and the scalar offset stays 0.
    const bool valid = u < n;
    const uint32_t base = valid ? (uint32_t)u * st.unit_w : 0u;
    const uint32_t vw = valid ? st.vw : kOutOfRange, vs = valid ? st.vs : kOutOfRange, vz = valid ? st.vz : kOutOfRange;
#pragma unroll
    for (int t = 0; t < STEPS; ++t)
        r.w[t] = __builtin_amdgcn_raw_buffer_load_b128(st.w, vw, valid ? base + (uint32_t)t * 4u * st.row_w : 0u, 2);
    const uint32_t g = valid ? (uint32_t)(u * g_of_unit_num) / (uint32_t)g_of_unit_den : 0u;  // group of the unit, slice-relative
    r.sc = __builtin_amdgcn_raw_buffer_load_b64(st.s, vs, g * st.row_s, 0);
    r.zw = __builtin_amdgcn_raw_buffer_load_b32(st.z, vz, g * st.row_z, 0);
}

// NI = rows of the 16-row tile a lane must keep: lane group g4 owns rows 4 g4 .. 4 g4 + 3.
template <int MROWS, int STEPS, int NI>
__device__ __forceinline__ void compute_unit(const Unit<STEPS> &u, const uint4_t *xs, const float *gs, int lrow0, int lunit,
                                             int mm, int g4, int gq, int zshift, const Masks &k, float (&tot)[4][NI])
{
    float4_t part[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) part[c] = (float4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        H8 x;
        x.u = xs[(lrow0 + 4 * t + g4) * MROWS + mm];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            part[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x.h, unpack8(u.w[t][c], k), part[c], 0, 0, 0);
    }
    float xsum[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) xsum[i] = gs[lunit * MROWS + gq * NI + i];
    H2 s01, s23;
    s01.u = u.sc[0];
    s23.u = u.sc[1];
    const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
    const uint32_t zs = u.zw >> zshift;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float z = (float)((zs >> (4 * c)) & 15u);
#pragma unroll
        for (int i = 0; i < NI; ++i) tot[c][i] = apply_scale_zero(tot[c][i], s[c], z, part[c][i], xsum[i]);
    }
}

// X rows m0 .. m0+MROWS-1, packed rows row0 .. row0+nrows-1 (nrows a multiple of
// RPU = rows per unit) into LDS: xs[row][m] = the eight halves of that row in
// unpack order, positions 1,5,3,7 divided by 16; gs[unit][m] = fp32 sum of the
// unit's x.  Consecutive threads take consecutive packed rows of one m, so RPU
// neighbouring lanes hold one unit and a butterfly adds them.  Eight loads per
// thread are in flight before the first is used.
constexpr int kStageBatch = 8;

template <int MROWS, int RPU>
__device__ __forceinline__ void stage_x(uint4_t *xs, float *gs, const GemmArgs &a, int m0, int row0, int nrows)
{
    const int total = nrows * MROWS;
    for (int base = 0; base < total; base += kThreads * kStageBatch) {
        uint4_t d[kStageBatch];
#pragma unroll
        for (int it = 0; it < kStageBatch; ++it) {
            const int idx = base + it * kThreads + threadIdx.x;
            const int m = idx / nrows, kb = idx - m * nrows;
            d[it] = (uint4_t){0u, 0u, 0u, 0u};
            if (idx < total && m0 + m < a.M)
                d[it] = *reinterpret_cast<const uint4_t *>(a.X + (size_t)(m0 + m) * a.K + (size_t)(row0 + kb) * 8);
        }
#pragma unroll
        for (int it = 0; it < kStageBatch; ++it) {
            const int idx = base + it * kThreads + threadIdx.x;
            const int m = idx / nrows, kb = idx - m * nrows;
            float sum = sum8(d[it]);
#pragma unroll
            for (int off = 1; off < RPU; off <<= 1) sum += __shfl_xor(sum, off, 64);
            if (idx < total) {
                xs[kb * MROWS + m] = permute_x(d[it]);
                if ((kb & (RPU - 1)) == 0) gs[(kb / RPU) * MROWS + m] = sum;
            }
        }
    }
}

template <int MROWS, int STEPS>
__global__ __launch_bounds__(kThreads) void mfma_reg_kernel(const GemmArgs a, const int chunk_units)
{
    constexpr int NI = MROWS < 4 ? MROWS : 4;
    constexpr int RPU = 4 * STEPS;  // packed rows per unit
    extern __shared__ uint4_t smem[];
    uint4_t *xs = smem;
    float *gs = reinterpret_cast<float *>(smem + (size_t)chunk_units * RPU * MROWS);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, g4 = lane >> 4;
    const int col0 = blockIdx.y * kTileN + wave * 64 + 4 * j;
    const bool ok = col0 < a.N;
    const int m0 = blockIdx.z * 16;
    const int mm = j < MROWS ? j : MROWS - 1;
    const int gq = g4 < MROWS / NI ? g4 : MROWS / NI - 1;  // lane groups past the last row read a valid (ignored) slot
    const int zshift = (col0 & 4) * 4;

    const int units_per_group = a.group / (32 * STEPS);
    const int gbeg = blockIdx.x * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.K / a.group) gend = a.K / a.group;
    const int nunits = (gend - gbeg) * units_per_group;  // units in this slice
    const int row_base = gbeg * (a.group / 8);           // first packed row of the slice

    Streams st;
    st.row_w = (uint32_t)a.N * 4u;
    st.unit_w = st.row_w * RPU;
    st.row_s = (uint32_t)a.N * 2u;
    st.row_z = (uint32_t)(a.N >> 3) * 4u;
    st.w = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.Wp) + (size_t)row_base * a.N, 0,
                                             (uint32_t)nunits * st.unit_w, kRawBuffer);
    st.s = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(a.scales) + (size_t)gbeg * a.N, 0,
                                             (uint32_t)(gend - gbeg) * st.row_s, kRawBuffer);
    st.z = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(a.Zp) + (size_t)gbeg * (a.N >> 3), 0,
                                             (uint32_t)(gend - gbeg) * st.row_z, kRawBuffer);
    st.vw = ok ? (uint32_t)(g4 * a.N + col0) * 4u : kOutOfRange;
    st.vs = ok ? (uint32_t)col0 * 2u : kOutOfRange;
    st.vz = ok ? (uint32_t)(col0 >> 3) * 4u : kOutOfRange;

    float tot[4][NI];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < NI; ++i) tot[c][i] = 0.f;

    const Masks masks = make_masks();
    Unit<STEPS> buf[kPrefetch + 1];
#pragma unroll
    for (int p = 0; p < kPrefetch; ++p) load_unit<STEPS>(buf[p], st, p, nunits, 1, units_per_group);

    for (int cbeg = 0; cbeg < nunits; cbeg += chunk_units) {
        const int cn = cbeg + chunk_units < nunits ? chunk_units : nunits - cbeg;
        if (cbeg) __syncthreads();  // everyone is done with the previous chunk of X
        stage_x<MROWS, RPU>(xs, gs, a, m0, row_base + cbeg * RPU, cn * RPU);
        __syncthreads();
        // chunk_units is a multiple of kPrefetch + 1 (or covers the slice), so buffer p always holds unit = p mod (kPrefetch + 1)
        for (int u = 0; u < cn; u += kPrefetch + 1) {
#pragma unroll
            for (int p = 0; p <= kPrefetch; ++p) {
                load_unit<STEPS>(buf[(p + kPrefetch) % (kPrefetch + 1)], st, cbeg + u + p + kPrefetch, nunits, 1, units_per_group);
                if (u + p < cn)
                    compute_unit<MROWS, STEPS, NI>(buf[p], xs, gs, (u + p) * RPU, u + p, mm, g4, gq, zshift, masks, tot);
            }
        }
    }

    // Lane group g4 holds rows m0 + 4 g4 + i (i < NI), columns col0 .. col0+3.
    const bool mine = ok && g4 < MROWS / NI;
    if (a.split == 1) {
        if (mine) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int m = m0 + 4 * g4 + i;
                if (m >= a.M) continue;
                *reinterpret_cast<uint2_t *>(a.Y + (size_t)m * a.N + col0) =
                    (uint2_t){pack_half2(tot[0][i], tot[1][i]), pack_half2(tot[2][i], tot[3][i])};
            }
        }
        return;
    }
    // Slice result to the fp32 workspace; the second pass adds the slices (Algorithm 1, Phase 3).
    if (mine) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int m = m0 + 4 * g4 + i;
            if (m >= a.M) continue;
            *reinterpret_cast<float4_t *>(a.partials + ((size_t)blockIdx.x * a.M + m) * a.N + col0) =
                (float4_t){tot[0][i], tot[1][i], tot[2][i], tot[3][i]};
        }
    }
}

template <int MROWS>
hipError_t launch_rows(const GemmArgs &a, hipStream_t stream, dim3 grid)
{
    const int steps = a.group % 128 == 0 ? 4 : (a.group % 64 == 0 ? 2 : 1);
    const int rpu = steps * 4;
    const int units_per_group = a.group / (32 * steps);
    const int slice_units = a.groups_per_split * units_per_group;
    // LDS per unit: rpu rows x MROWS x 16 bytes of X plus MROWS unit sums
    const int per_unit = rpu * MROWS * 16 + MROWS * 4;
    int chunk_units = kLdsBudget / per_unit;
    chunk_units -= chunk_units % (kPrefetch + 1);
    if (chunk_units < kPrefetch + 1) return hipErrorInvalidValue;
    if (chunk_units > slice_units) chunk_units = slice_units;
    const size_t lds = (size_t)chunk_units * per_unit;
    // slice-relative 32-bit buffer offsets must stay below the out-of-range marker
    if ((unsigned long long)slice_units * rpu * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;
    switch (steps) {
    case 4: hipLaunchKernelGGL((mfma_reg_kernel<MROWS, 4>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    case 2: hipLaunchKernelGGL((mfma_reg_kernel<MROWS, 2>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    default: hipLaunchKernelGGL((mfma_reg_kernel<MROWS, 1>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_mfma_reg(const GemmArgs &a, hipStream_t stream)
{
    dim3 grid(a.split, (a.N + kTileN - 1) / kTileN, (a.M + 15) / 16);
    if (a.M == 1) return launch_rows<1>(a, stream, grid);
    if (a.M == 2) return launch_rows<2>(a, stream, grid);
    if (a.M <= 4) return launch_rows<4>(a, stream, grid);
    if (a.M <= 8) return launch_rows<8>(a, stream, grid);
    return launch_rows<16>(a, stream, grid);
}

}  // namespace w4a16
