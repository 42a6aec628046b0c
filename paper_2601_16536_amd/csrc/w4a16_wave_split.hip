// W4A16 multiply for the decode case (M <= 4): one workgroup per narrow column
// tile, its sixteen waves split K among themselves, and the sixteen partial
// results meet in LDS.
//
// This is Algorithm 1's Split-K (Phase 2: C_i = A * B_i per K slice; Phase 3:
// C = sum_i C_i, then the cast to FP16) with the slices held by the waves of one
// workgroup, so the partial results never leave the compute unit: the sum over
// slices is a fixed-order LDS reduction behind one barrier instead of a
// workspace in device memory, a device-wide wait and a second pass.  A further
// split across workgroups (blockIdx.x, partials to the workspace, second pass)
// stays available for shapes whose N gives too few column tiles.
//
// Each lane loads VEC consecutive 32-bit words of one packed row (VEC columns x
// eight k); a wave-wide load covers four packed rows x 16 VEC columns.  The
// unpack (five integer instructions per word, subnormal-fp16 MFMA operands) and
// the fp32 scale / zero-point step are those of w4a16_device.h.  Each wave
// stages the X values of its own K slice in a private 4 KiB of LDS, so the main
// loop has no workgroup barrier.
//
// Measured and dropped: handing the units of K to the waves through an LDS
// counter (the waves of a workgroup finish up to 2x apart, but the compute unit's
// memory throughput, not the slowest wave, sets the time: no gain); more than two
// units of prefetch per wave (slower: the compute unit's outstanding-miss
// capacity is already full at two); feeding the MFMA's X operand straight from
// global memory with the unit sums from an extra MFMA against an all-ones operand
// (no LDS staging, M up to 16: 20-25 % slower, the extra vector-memory
// instructions cost more than the staging they replace).
#include "w4a16_device.h"
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

constexpr int kWaves = 16;
constexpr int kWaveLds = 4096;  // bytes of LDS per wave for its X slice

template <int VEC>
struct WordVec;
template <>
struct WordVec<2> {
    typedef uint2_t type;
};
template <>
struct WordVec<4> {
    typedef uint4_t type;
};

// What a lane holds of one unit = STEPS x 32 consecutive k of its VEC columns.
template <int STEPS, int VEC>
struct Unit {
    typename WordVec<VEC>::type w[STEPS];
    uint32_t sc[VEC / 2];  // VEC fp16 scales
    uint32_t zw;           // the zero-point word that holds the VEC columns
};

struct Streams {
    __amdgpu_buffer_rsrc_t w, s, z;  // buffers that start at the workgroup's K slice
    uint32_t vw, vs, vz;             // this lane's byte offsets inside a unit / scale row / zero row
    uint32_t unit_w, row_w;          // bytes per unit and per packed row of Wp
    uint32_t row_s, row_z;           // bytes per row of scales / zeros
    uint32_t zfill;                  // ORed into every zero-point word: 0, or eight 8s without a zero-point tensor
};

// Loads unit `u` (relative to the workgroup's slice) if u < end, else nothing
// (registers become 0): past the end the per-lane offset, which the hardware
// range-checks against the slice size, is pushed out of range.  Weights are read
// once: nontemporal.
template <int STEPS, int VEC>
__device__ __forceinline__ void load_unit(Unit<STEPS, VEC> &r, const Streams &st, int u, int end, int group_of_u)
{
    const bool valid = u < end;
    const uint32_t base = valid ? (uint32_t)u * st.unit_w : 0u;
    const uint32_t vw = valid ? st.vw : kOutOfRange, vs = valid ? st.vs : kOutOfRange, vz = valid ? st.vz : kOutOfRange;
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        const uint32_t so = base + (uint32_t)t * 4u * st.row_w;
        if constexpr (VEC == 4) r.w[t] = __builtin_amdgcn_raw_buffer_load_b128(st.w, vw, so, 2);
        else r.w[t] = __builtin_amdgcn_raw_buffer_load_b64(st.w, vw, so, 2);
    }
    const uint32_t g = valid ? (uint32_t)group_of_u : 0u;
    if constexpr (VEC == 4) {
        const uint2_t s = __builtin_amdgcn_raw_buffer_load_b64(st.s, vs, g * st.row_s, 0);
        r.sc[0] = s[0];
        r.sc[1] = s[1];
    } else {
        r.sc[0] = __builtin_amdgcn_raw_buffer_load_b32(st.s, vs, g * st.row_s, 0);
    }
    r.zw = __builtin_amdgcn_raw_buffer_load_b32(st.z, vz, g * st.row_z, 0) | st.zfill;
}

template <int MROWS, int STEPS, int VEC>
__device__ __forceinline__ void compute_unit(const Unit<STEPS, VEC> &u, const uint4_t *xs, const float *gs, int lrow0,
                                             int lunit, int mm, int g4, int zshift, const Masks &k,
                                             float (&tot)[VEC][MROWS])
{
    float4_t part[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) part[c] = (float4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        H8 x;
        x.u = xs[(lrow0 + 4 * t + g4) * MROWS + mm];
#pragma unroll
        for (int c = 0; c < VEC; ++c)
            part[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x.h, unpack8(u.w[t][c], k), part[c], 0, 0, 0);
    }
    float xsum[MROWS];
#pragma unroll
    for (int i = 0; i < MROWS; ++i) xsum[i] = gs[lunit * MROWS + i];
    const uint32_t zs = u.zw >> zshift;
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        H2 sc;
        sc.u = u.sc[c / 2];
        const float s = (float)sc.h[c & 1];
        const float z = (float)((zs >> (4 * c)) & 15u);
#pragma unroll
        for (int i = 0; i < MROWS; ++i) tot[c][i] = apply_scale_zero(tot[c][i], s, z, part[c][i], xsum[i]);
    }
}

// One wave stages X rows 0..MROWS-1, packed rows row0 .. row0+nrows-1 (nrows a
// multiple of RPU = rows per unit, nrows * MROWS <= 256) into its own LDS:
// xs[row][m] = that row's eight halves in unpack order, gs[unit][m] = fp32 sum
// of the unit's x.  Split in two so that all loads are in flight together (and
// the first weight loads can be issued between the halves).
constexpr int kStageIters = kWaveLds / 16 / 64;  // 16-byte entries per lane

struct StagedX {
    uint4_t d[kStageIters];
};

template <int MROWS>
__device__ __forceinline__ void stage_x_load(StagedX &r, const GemmArgs &a, int lane, int row0, int nrows)
{
    const int total = nrows * MROWS;
    const int nr = nrows > 0 ? nrows : 1;  // a wave with no units stages nothing
#pragma unroll
    for (int it = 0; it < kStageIters; ++it) {
        const int idx = lane + 64 * it;
        const int m = idx / nr, kb = idx - m * nr;
        uint4_t d = {0u, 0u, 0u, 0u};
        if (idx < total && m < a.M) d = *reinterpret_cast<const uint4_t *>(a.X + (size_t)m * a.K + (size_t)(row0 + kb) * 8);
        r.d[it] = d;
    }
}

template <int MROWS, int RPU>
__device__ __forceinline__ void stage_x_store(const StagedX &r, uint4_t *xs, float *gs, int lane, int nrows)
{
    const int total = nrows * MROWS;
    const int nr = nrows > 0 ? nrows : 1;
#pragma unroll
    for (int it = 0; it < kStageIters; ++it) {
        const int idx = lane + 64 * it;
        const int m = idx / nr, kb = idx - m * nr;
        float sum = sum8(r.d[it]);
#pragma unroll
        for (int off = 1; off < RPU; off <<= 1) sum += __shfl_xor(sum, off, 64);
        if (idx < total) {
            xs[kb * MROWS + m] = permute_x(r.d[it]);
            if ((kb & (RPU - 1)) == 0) gs[(kb / RPU) * MROWS + m] = sum;
        }
    }
}

template <int MROWS, int STEPS, int VEC, int PF>
__global__ __launch_bounds__(kWaves * 64) void wave_split_kernel(const GemmArgs a, const int chunk_units)
{
    constexpr int RPU = 4 * STEPS;     // packed rows per unit
    constexpr int TILE = 16 * VEC;     // columns per workgroup
    constexpr int RING = PF + 1;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kWaves * kWaveLds];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15, g4 = lane >> 4;
    // Workgroups go round-robin over the 8 XCDs.  Without a split across workgroups,
    // hand each XCD a contiguous run of column tiles, so that the 128-byte lines of
    // scales and zero points that neighbouring tiles share are fetched by one L2 only.
    const int ntiles = gridDim.y;
    int tile = blockIdx.y;
    if (gridDim.x == 1 && (ntiles & 7) == 0) tile = (tile & 7) * (ntiles >> 3) + (tile >> 3);
    const int col0 = tile * TILE + VEC * j;
    const bool ok = col0 < a.N;
    const int mm = j < MROWS ? j : MROWS - 1;
    const int zshift = (col0 & 7) * 4;

    // the workgroup's K slice in groups, then in units, then this wave's share of the units
    const int units_per_group = a.group / (32 * STEPS);
    const int gbeg = blockIdx.x * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.K / a.group) gend = a.K / a.group;
    const int nunits = (gend - gbeg) * units_per_group;
    const int ubeg = (int)((long long)nunits * wave / kWaves);
    const int uend = (int)((long long)nunits * (wave + 1) / kWaves);
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
                                             zero_point_bytes(a.Zp, (uint32_t)(gend - gbeg) * st.row_z), kRawBuffer);
    st.zfill = symmetric_fill(a.Zp);
    st.vw = ok ? (uint32_t)(g4 * a.N + col0) * 4u : kOutOfRange;
    st.vs = ok ? (uint32_t)col0 * 2u : kOutOfRange;
    st.vz = ok ? (uint32_t)(col0 >> 3) * 4u : kOutOfRange;

    float tot[VEC][MROWS];
#pragma unroll
    for (int c = 0; c < VEC; ++c)
#pragma unroll
        for (int i = 0; i < MROWS; ++i) tot[c][i] = 0.f;

    const Masks masks = make_masks();
    uint4_t *xs = reinterpret_cast<uint4_t *>(smem + wave * kWaveLds);
    float *gs = reinterpret_cast<float *>(xs + (size_t)chunk_units * RPU * MROWS);

    // X of the first chunk first (mostly L2 hits), then the weight stream.
    StagedX sx;
    {
        const int cn = chunk_units < uend - ubeg ? chunk_units : uend - ubeg;
        stage_x_load<MROWS>(sx, a, lane, row_base + ubeg * RPU, cn * RPU);
    }
    // (lg, lpos): quantisation group of the next unit to load and its position inside the group
    int lg = ubeg / units_per_group, lpos = ubeg - lg * units_per_group;
    Unit<STEPS, VEC> buf[RING];
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        load_unit<STEPS, VEC>(buf[p], st, ubeg + p, uend, lg);
        if (++lpos == units_per_group) { lpos = 0; ++lg; }
    }

    // chunk_units is a multiple of RING, so buffer p always holds unit ubeg + (multiple of RING) + p.
    // Only this wave touches its LDS and the LDS operations of one wave complete in
    // order; the fences only keep the compiler from moving them across the staging.
    // The staging stays outside the unrolled ring so that the loads' wait counts
    // stay exact (a conditional load inside it makes every wait a full drain).
    for (int cbeg = ubeg; cbeg < uend; cbeg += chunk_units) {
        const int cn = cbeg + chunk_units < uend ? chunk_units : uend - cbeg;
        if (cbeg != ubeg) stage_x_load<MROWS>(sx, a, lane, row_base + cbeg * RPU, cn * RPU);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        stage_x_store<MROWS, RPU>(sx, xs, gs, lane, cn * RPU);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        for (int u = 0; u < cn; u += RING) {
#pragma unroll
            for (int p = 0; p < RING; ++p) {
                load_unit<STEPS, VEC>(buf[(p + PF) % RING], st, cbeg + u + p + PF, uend, lg);
                if (++lpos == units_per_group) { lpos = 0; ++lg; }
                if (u + p < cn)
                    compute_unit<MROWS, STEPS, VEC>(buf[p], xs, gs, (u + p) * RPU, u + p, mm, g4, zshift, masks, tot);
            }
        }
    }

    // Sum over the sixteen waves in wave order: red[wave][m][column of the tile].
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);
    if (g4 == 0) {  // lane group 0 holds rows 0..3 of the MFMA result, columns VEC j + c
#pragma unroll
        for (int c = 0; c < VEC; ++c)
#pragma unroll
            for (int i = 0; i < MROWS; ++i) red[(wave * MROWS + i) * TILE + VEC * j + c] = tot[c][i];
    }
    __syncthreads();
    const int t = threadIdx.x;
    if (t < MROWS * TILE) {
        const int m = t / TILE, c = t - m * TILE;
        const int col = tile * TILE + c;
        if (m < a.M && col < a.N) {
            float acc = red[m * TILE + c];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) acc += red[(w * MROWS + m) * TILE + c];
            if (a.split == 1) {
                H2 h;
                h.h = (half2_t){(_Float16)acc, (_Float16)0.f};
                a.Y[(size_t)m * a.N + col] = (uint16_t)(h.u & 0xFFFFu);
            } else {
                a.partials[((size_t)blockIdx.x * a.M + m) * a.N + col] = acc;
            }
        }
    }
}

template <int MROWS, int VEC>
hipError_t launch_rows(const GemmArgs &a, hipStream_t stream, dim3 grid)
{
    const int steps = a.group % 128 == 0 ? 4 : (a.group % 64 == 0 ? 2 : 1);
    const int rpu = steps * 4;
    const int units_per_group = a.group / (32 * steps);
    const int per_unit = rpu * MROWS * 16 + MROWS * 4;  // LDS bytes per unit: X rows plus the unit sums
    constexpr int PF = kPrefetch;
    constexpr int ring = PF + 1;
    int chunk_units = kWaveLds / per_unit;
    chunk_units -= chunk_units % ring;
    if (chunk_units < ring) return hipErrorInvalidValue;
    // slice-relative 32-bit buffer offsets must stay below the out-of-range marker
    if ((unsigned long long)a.groups_per_split * units_per_group * rpu * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;
    const dim3 block(kWaves * 64);
    switch (steps) {
    case 4: hipLaunchKernelGGL((wave_split_kernel<MROWS, 4, VEC, PF>), grid, block, 0, stream, a, chunk_units); break;
    case 2: hipLaunchKernelGGL((wave_split_kernel<MROWS, 2, VEC, PF>), grid, block, 0, stream, a, chunk_units); break;
    default: hipLaunchKernelGGL((wave_split_kernel<MROWS, 1, VEC, PF>), grid, block, 0, stream, a, chunk_units); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_wave_split(const GemmArgs &a, int tile_n, hipStream_t stream)
{
    if (a.M > 4 || (tile_n != 32 && tile_n != 64)) return hipErrorInvalidValue;
    if (a.bf16) return hipErrorInvalidValue;  // FP16 activations only (the scheduler never takes this family by itself)
    const dim3 grid(a.split, (a.N + tile_n - 1) / tile_n, 1);
    if (tile_n == 64) {
        if (a.M == 1) return launch_rows<1, 4>(a, stream, grid);
        if (a.M == 2) return launch_rows<2, 4>(a, stream, grid);
        return launch_rows<4, 4>(a, stream, grid);
    }
    if (a.M == 1) return launch_rows<1, 2>(a, stream, grid);
    if (a.M == 2) return launch_rows<2, 2>(a, stream, grid);
    return launch_rows<4, 2>(a, stream, grid);
}

}  // namespace w4a16
