// W4A16 multiply for M >= 17: the MFMA_REG work split (four waves x 64 columns per
// workgroup, one K slice per workgroup, weights unpacked straight into MFMA operand
// registers) with RT row tiles of 16 rows of X per workgroup, so that every loaded
// and unpacked weight word feeds RT MFMAs instead of one and W is read from HBM
// once per 16 RT rows instead of once per 16.
//
// Same arithmetic as the other families (Eq. 2; Algorithm 1, Phase 2 per K slice):
// P = 2^-24 sum_k x_k q_k per unit of 128 k from the MFMA, then
// (2^24 s) P - (s z) sum_k x_k in fp32 per (unit, row, column).  X for the
// workgroup's rows and the current chunk of K is staged in LDS (permuted into the
// unpack's k order) and is the A operand of all four waves; the unpacked weights
// never leave registers.  Slices across workgroups go to the fp32 workspace and the
// second pass (Algorithm 1, Phase 3).
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

constexpr int kRowsLds = 57344;  // bytes of LDS for the staged chunk of X (two workgroups fit a compute unit)
constexpr int kStageBatch = 8;

template <int STEPS>
struct Unit {
    uint4_t w[STEPS];  // packed codes, row 4t + lane/16 of the unit, columns col0..col0+3
    uint2_t sc;        // four fp16 scales
    uint32_t zw;       // the zero-point word that holds the four columns
};

struct Streams {
    __amdgpu_buffer_rsrc_t w, s, z;
    uint32_t vw, vs, vz;
    uint32_t unit_w, row_w, row_s, row_z;
};

// Unit `u` of the slice if u < n, else nothing (the per-lane offset, which the
// hardware range-checks against the slice size, is pushed out of range).
template <int STEPS>
__device__ __forceinline__ void load_unit(Unit<STEPS> &r, const Streams &st, int u, int n, int group_of_u)
{
    const bool valid = u < n;
    const uint32_t base = valid ? (uint32_t)u * st.unit_w : 0u;
    const uint32_t vw = valid ? st.vw : kOutOfRange, vs = valid ? st.vs : kOutOfRange, vz = valid ? st.vz : kOutOfRange;
#pragma unroll
    for (int t = 0; t < STEPS; ++t)
        r.w[t] = __builtin_amdgcn_raw_buffer_load_b128(st.w, vw, base + (uint32_t)t * 4u * st.row_w, 2);
    const uint32_t g = valid ? (uint32_t)group_of_u : 0u;
    r.sc = __builtin_amdgcn_raw_buffer_load_b64(st.s, vs, g * st.row_s, 0);
    r.zw = __builtin_amdgcn_raw_buffer_load_b32(st.z, vz, g * st.row_z, 0);
}

// Lane (j = lane % 16, g4 = lane / 16) holds, per row tile rt and column c, the four
// result rows 16 rt + 4 g4 + i of column col0 + c.
template <int RT, int STEPS>
__device__ __forceinline__ void compute_unit(const Unit<STEPS> &u, const uint4_t *xs, const float *gs, int lrow0, int lunit,
                                             int j, int g4, int zshift, const Masks &k, float4_t (&tot)[RT][4])
{
    constexpr int MROWS = 16 * RT;
    float4_t part[RT][4];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) part[r][c] = (float4_t){0.f, 0.f, 0.f, 0.f};
    // A fragments for step t + 1 are read from LDS before the MFMAs of step t are issued,
    // so that a wave alone on its SIMD does not sit out the LDS latency sixteen times per unit.
    H8 x[2][RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) x[0][r].u = xs[(lrow0 + g4) * MROWS + 16 * r + j];
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        if (t + 1 < STEPS) {
#pragma unroll
            for (int r = 0; r < RT; ++r) x[(t + 1) & 1][r].u = xs[(lrow0 + 4 * (t + 1) + g4) * MROWS + 16 * r + j];
        }
        half8_t b[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) b[c] = unpack8(u.w[t][c], k);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < RT; ++r) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                part[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x[t & 1][r].h, b[c], part[r][c], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    H2 s01, s23;
    s01.u = u.sc[0];
    s23.u = u.sc[1];
    const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
    const uint32_t zs = u.zw >> zshift;
    float sp[4], sz[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        sp[c] = s[c] * 16777216.0f;                        // 2^24 s
        sz[c] = -s[c] * (float)((zs >> (4 * c)) & 15u);    // -s z
    }
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const float4_t xsum = *reinterpret_cast<const float4_t *>(gs + lunit * MROWS + 16 * r + 4 * g4);
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                tot[r][c][i] = __builtin_fmaf(sp[c], part[r][c][i], __builtin_fmaf(sz[c], xsum[i], tot[r][c][i]));
    }
}

// X rows m0 .. m0+MROWS-1, packed rows row0 .. row0+nrows-1 into LDS: xs[row][m] =
// that row's eight halves in unpack order, gs[unit][m] = fp32 sum of the unit's x.
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

template <int RT, int STEPS>
__global__ __launch_bounds__(kThreads) void mfma_rows_kernel(const GemmArgs a, const int chunk_units)
{
    constexpr int MROWS = 16 * RT;
    constexpr int RPU = 4 * STEPS;
    constexpr int PF = kPrefetch, RING = PF + 1;
    extern __shared__ uint4_t smem[];
    uint4_t *xs = smem;
    float *gs = reinterpret_cast<float *>(smem + (size_t)chunk_units * RPU * MROWS);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, g4 = lane >> 4;
    const int col0 = blockIdx.y * kTileN + wave * 64 + 4 * j;
    const bool ok = col0 < a.N;
    const int m0 = blockIdx.z * MROWS;
    const int zshift = (col0 & 4) * 4;

    const int units_per_group = a.group / (32 * STEPS);
    const int gbeg = blockIdx.x * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.K / a.group) gend = a.K / a.group;
    const int nunits = (gend - gbeg) * units_per_group;
    const int row_base = gbeg * (a.group / 8);

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

    float4_t tot[RT][4];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) tot[r][c] = (float4_t){0.f, 0.f, 0.f, 0.f};

    const Masks masks = make_masks();
    int lg = 0, lpos = 0;  // quantisation group (slice-relative) of the next unit to load, and its position in the group
    Unit<STEPS> buf[RING];
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        load_unit<STEPS>(buf[p], st, p, nunits, lg);
        if (++lpos == units_per_group) { lpos = 0; ++lg; }
    }

    // chunk_units is a multiple of RING (or covers the slice): buffer p always holds unit = p mod RING
    for (int cbeg = 0; cbeg < nunits; cbeg += chunk_units) {
        const int cn = cbeg + chunk_units < nunits ? chunk_units : nunits - cbeg;
        if (cbeg) __syncthreads();  // everyone is done with the previous chunk of X
        stage_x<MROWS, RPU>(xs, gs, a, m0, row_base + cbeg * RPU, cn * RPU);
        __syncthreads();
        for (int u = 0; u < cn; u += RING) {
#pragma unroll
            for (int p = 0; p < RING; ++p) {
                load_unit<STEPS>(buf[(p + PF) % RING], st, cbeg + u + p + PF, nunits, lg);
                if (++lpos == units_per_group) { lpos = 0; ++lg; }
                if (u + p < cn) compute_unit<RT, STEPS>(buf[p], xs, gs, (u + p) * RPU, u + p, j, g4, zshift, masks, tot);
            }
        }
    }

    if (!ok) return;
#pragma unroll
    for (int r = 0; r < RT; ++r) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + 16 * r + 4 * g4 + i;
            if (m >= a.M) continue;
            if (a.split == 1) {
                *reinterpret_cast<uint2_t *>(a.Y + (size_t)m * a.N + col0) =
                    (uint2_t){pack_half2(tot[r][0][i], tot[r][1][i]), pack_half2(tot[r][2][i], tot[r][3][i])};
            } else {
                *reinterpret_cast<float4_t *>(a.partials + ((size_t)blockIdx.x * a.M + m) * a.N + col0) =
                    (float4_t){tot[r][0][i], tot[r][1][i], tot[r][2][i], tot[r][3][i]};
            }
        }
    }
}

template <int RT>
hipError_t launch_rt(const GemmArgs &a, hipStream_t stream)
{
    constexpr int MROWS = 16 * RT;
    const int steps = a.group % 128 == 0 ? 4 : (a.group % 64 == 0 ? 2 : 1);
    const int rpu = steps * 4;
    const int units_per_group = a.group / (32 * steps);
    const int slice_units = a.groups_per_split * units_per_group;
    const int per_unit = rpu * MROWS * 16 + MROWS * 4;  // LDS bytes per unit: X rows plus the unit sums
    int chunk_units = kRowsLds / per_unit;
    chunk_units -= chunk_units % (kPrefetch + 1);
    if (chunk_units < kPrefetch + 1) return hipErrorInvalidValue;
    if (chunk_units > slice_units) chunk_units = slice_units;
    const size_t lds = (size_t)chunk_units * per_unit;
    if ((unsigned long long)slice_units * rpu * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;
    const dim3 grid(a.split, (a.N + kTileN - 1) / kTileN, (a.M + MROWS - 1) / MROWS);
    switch (steps) {
    case 4: hipLaunchKernelGGL((mfma_rows_kernel<RT, 4>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    case 2: hipLaunchKernelGGL((mfma_rows_kernel<RT, 2>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    default: hipLaunchKernelGGL((mfma_rows_kernel<RT, 1>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_mfma_rows(const GemmArgs &a, int tile_m, hipStream_t stream)
{
    if (tile_m == 32) return launch_rt<2>(a, stream);
    if (tile_m == 64) return launch_rt<4>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace w4a16
