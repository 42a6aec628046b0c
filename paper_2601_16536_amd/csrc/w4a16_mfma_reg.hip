// W4A16 multiply with the weights unpacked straight into MFMA operand registers.
//
// Computes the Split-K partial products C_i = A * B_i of Algorithm 1, Phase 2,
// where B_i = s (W - z) (Eq. 2) restricted to the i-th K slice -- but B_i never
// exists in memory (Algorithm 1, Phase 1 writes it to a workspace; that round
// trip is the bottleneck Section 4.2 diagnoses).  Each lane loads 16 bytes of
// packed codes (four columns x eight k), turns each 32-bit word into the eight
// exact fp16 integers (q - z) that form its slice of a 16x16x32 MFMA B operand,
// and the per-group fp32 result is multiplied by the fp32 scale once per
// (group, column): sum_k x_k s (q_k - z) = s * sum_k x_k (q_k - z).
//
// Work split: a workgroup is four waves side by side along N (4 x 64 columns,
// so every packed row it touches is a contiguous 1 KiB), all walking the same
// K slice; blockIdx.y is the slice, blockIdx.z a tile of 16 rows of X.
// X for the slice is staged once per chunk in LDS, already permuted into the
// k order the unpack produces, and serves all four waves.
#include "w4a16_internal.h"

namespace w4a16 {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

union H2 {
    uint32_t u;
    half2_t h;
};
union H8 {
    uint4_t u;
    half8_t h;
};

// One 32-bit word = codes of k = 8r .. 8r+7 of one column.  OR-ing a nibble
// into the mantissa of 1024.0 (bits 0-3) or of 64.0 (bits 4-7) gives the
// fp16 numbers 1024+q and 64+q exactly; adding -(1024+z) or -(64+z) leaves the
// exact integer q - z.  Result order along k: 0,4,1,5,2,6,3,7 (X is staged in
// the same order, a contraction does not care).
struct Magic {
    uint32_t lo, hi;      // nibble masks 0x000F000F, 0x00F000F0 (scalar registers)
    uint32_t b1024, b64;  // fp16 pairs 1024.0, 64.0 (vector registers)
};

// The four constants are made opaque to the optimiser so that each (w & mask) | bias
// stays one three-operand v_and_or_b32 (one scalar and two vector operands)
// instead of two instructions with a 32-bit literal each.
__device__ __forceinline__ Magic make_magic()
{
    Magic m;
    m.lo = 0x000F000Fu;
    m.hi = 0x00F000F0u;
    m.b1024 = 0x64006400u;
    m.b64 = 0x54005400u;
    asm volatile("" : "+s"(m.lo), "+s"(m.hi), "+v"(m.b1024), "+v"(m.b64));
    return m;
}

__device__ __forceinline__ half8_t unpack8(uint32_t w, half2_t zlo, half2_t zhi, const Magic &k)
{
    uint32_t w8 = w >> 8;
    H2 a0, a1, a2, a3;
    a0.u = (w & k.lo) | k.b1024;
    a1.u = (w & k.hi) | k.b64;
    a2.u = (w8 & k.lo) | k.b1024;
    a3.u = (w8 & k.hi) | k.b64;
    half2_t p0 = a0.h + zlo, p1 = a1.h + zhi, p2 = a2.h + zlo, p3 = a3.h + zhi;
    half8_t r;
    r[0] = p0[0]; r[1] = p0[1]; r[2] = p1[0]; r[3] = p1[1];
    r[4] = p2[0]; r[5] = p2[1]; r[6] = p3[0]; r[7] = p3[1];
    return r;
}

// What a lane holds of one unit = STEPS x 32 consecutive k of its 4 columns.
template <int STEPS>
struct Unit {
    uint4_t w[STEPS];  // packed codes, row 4t + lane/16 of the unit, columns col0..col0+3
    uint2_t sc;        // four fp16 scales
    uint32_t zw;       // the zero-point word that holds the four columns
};

template <int STEPS>
__device__ __forceinline__ void load_unit(Unit<STEPS> &u, const GemmArgs &a, int unit, int col0, int g4, bool ok)
{
    const int row0 = unit * (STEPS * 4);
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        uint4_t v = {0u, 0u, 0u, 0u};
        if (ok) v = *reinterpret_cast<const uint4_t *>(a.Wp + (size_t)(row0 + 4 * t + g4) * a.N + col0);
        u.w[t] = v;
    }
    const int g = (row0 * 8) / a.group;
    uint2_t sc = {0u, 0u};
    uint32_t zw = 0u;
    if (ok) {
        sc = *reinterpret_cast<const uint2_t *>(a.scales + (size_t)g * a.N + col0);
        zw = a.Zp[(size_t)g * (a.N >> 3) + (col0 >> 3)];
    }
    u.sc = sc;
    u.zw = zw;
}

template <int MROWS, int STEPS>
__device__ __forceinline__ void compute_unit(const Unit<STEPS> &u, const uint4_t *xs, int lrow0, int mm, int g4,
                                             int zshift, const Magic &k, float4_t (&tot)[4])
{
    half2_t zlo[4], zhi[4];
    const uint32_t zs = u.zw >> zshift;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        uint32_t z = (zs >> (4 * c)) & 15u;
        uint32_t zb = z | (z << 16);
        H2 lo, hi;
        lo.u = zb | 0xE400E400u;         // -(1024 + z)
        hi.u = (zb << 4) | 0xD400D400u;  // -(64 + z)
        zlo[c] = lo.h;
        zhi[c] = hi.h;
    }
    float4_t part[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) part[c] = (float4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        H8 x;
        x.u = xs[(lrow0 + 4 * t + g4) * MROWS + mm];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            part[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x.h, unpack8(u.w[t][c], zlo[c], zhi[c], k), part[c], 0, 0, 0);
    }
    H2 s01, s23;
    s01.u = u.sc[0];
    s23.u = u.sc[1];
    const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
#pragma unroll
    for (int c = 0; c < 4; ++c) tot[c] += s[c] * part[c];
}

// X rows m0 .. m0+MROWS-1, packed rows row0 .. row0+nrows-1, into LDS as
// xs[row][m] = the eight halves of that row's k in unpack order.
template <int MROWS>
__device__ __forceinline__ void stage_x(uint4_t *xs, const GemmArgs &a, int m0, int row0, int nrows)
{
    for (int idx = threadIdx.x; idx < nrows * MROWS; idx += kThreads) {
        const int kb = idx / MROWS, m = idx % MROWS;
        uint4_t d = {0u, 0u, 0u, 0u};
        if (m0 + m < a.M) d = *reinterpret_cast<const uint4_t *>(a.X + (size_t)(m0 + m) * a.K + (size_t)(row0 + kb) * 8);
        uint4_t o;
        o[0] = (d[0] & 0xFFFFu) | (d[2] << 16);          // x0, x4
        o[1] = (d[0] >> 16) | (d[2] & 0xFFFF0000u);      // x1, x5
        o[2] = (d[1] & 0xFFFFu) | (d[3] << 16);          // x2, x6
        o[3] = (d[1] >> 16) | (d[3] & 0xFFFF0000u);      // x3, x7
        xs[idx] = o;
    }
}

template <int MROWS, int STEPS>
__global__ __launch_bounds__(kThreads) void mfma_reg_kernel(const GemmArgs a, const int chunk_units)
{
    extern __shared__ uint4_t xs[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, g4 = lane >> 4;
    const int col0 = blockIdx.x * kTileN + wave * 64 + 4 * j;
    const bool ok = col0 < a.N;
    const int m0 = blockIdx.z * 16;
    const int mm = j < MROWS ? j : MROWS - 1;
    const int zshift = (col0 & 4) * 4;

    const int units_per_group = a.group / (32 * STEPS);
    const int total_units = a.K / (32 * STEPS);
    const int ubeg = blockIdx.y * a.groups_per_split * units_per_group;
    int uend = ubeg + a.groups_per_split * units_per_group;
    if (uend > total_units) uend = total_units;

    float4_t tot[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) tot[c] = (float4_t){0.f, 0.f, 0.f, 0.f};

    const Magic magic = make_magic();
    Unit<STEPS> cur, nxt;
    if (ubeg < uend) load_unit<STEPS>(cur, a, ubeg, col0, g4, ok);
    for (int cbeg = ubeg; cbeg < uend; cbeg += chunk_units) {
        const int cend = cbeg + chunk_units < uend ? cbeg + chunk_units : uend;
        __syncthreads();
        stage_x<MROWS>(xs, a, m0, cbeg * STEPS * 4, (cend - cbeg) * STEPS * 4);
        __syncthreads();
        for (int u = cbeg; u < cend; ++u) {
            if (u + 1 < uend) load_unit<STEPS>(nxt, a, u + 1, col0, g4, ok);
            compute_unit<MROWS, STEPS>(cur, xs, (u - cbeg) * STEPS * 4, mm, g4, zshift, magic, tot);
            cur = nxt;
        }
    }

    // Lane holds rows m0 + 4*g4 + i, columns col0 .. col0+3 (tot[c][i]).
    if (!ok) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + 4 * g4 + i;
        if (m >= a.M) continue;
        const float4_t v = {tot[0][i], tot[1][i], tot[2][i], tot[3][i]};
        if (a.split == 1) {
            half2_t h01 = {(_Float16)v[0], (_Float16)v[1]}, h23 = {(_Float16)v[2], (_Float16)v[3]};
            H2 p, q;
            p.h = h01;
            q.h = h23;
            *reinterpret_cast<uint2_t *>(a.Y + (size_t)m * a.N + col0) = (uint2_t){p.u, q.u};
        } else {
            *reinterpret_cast<float4_t *>(a.partials + ((size_t)blockIdx.y * a.M + m) * a.N + col0) = v;
        }
    }
}

template <int MROWS>
hipError_t launch_rows(const GemmArgs &a, hipStream_t stream, dim3 grid)
{
    const int steps = a.group % 128 == 0 ? 4 : (a.group % 64 == 0 ? 2 : 1);
    const int rows_per_unit = steps * 4;
    const int units_per_group = a.group / (32 * steps);
    // whole groups per LDS chunk, at least one
    int chunk_groups = kLdsBudget / (16 * MROWS * rows_per_unit * units_per_group);
    if (chunk_groups < 1) chunk_groups = 1;
    if (chunk_groups > a.groups_per_split) chunk_groups = a.groups_per_split;
    const int chunk_units = chunk_groups * units_per_group;
    const size_t lds = (size_t)chunk_units * rows_per_unit * MROWS * 16;
    if (lds > 65536) return hipErrorInvalidValue;
    switch (steps) {
    case 4: hipLaunchKernelGGL((mfma_reg_kernel<MROWS, 4>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    case 2: hipLaunchKernelGGL((mfma_reg_kernel<MROWS, 2>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    default: hipLaunchKernelGGL((mfma_reg_kernel<MROWS, 1>), grid, dim3(kThreads), lds, stream, a, chunk_units); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_mfma_reg(const GemmArgs &a, hipStream_t stream, int *workgroups)
{
    dim3 grid((a.N + kTileN - 1) / kTileN, a.split, (a.M + 15) / 16);
    if (workgroups) *workgroups = grid.x * grid.y * grid.z;
    if (a.M == 1) return launch_rows<1>(a, stream, grid);
    if (a.M == 2) return launch_rows<2>(a, stream, grid);
    if (a.M <= 4) return launch_rows<4>(a, stream, grid);
    if (a.M <= 8) return launch_rows<8>(a, stream, grid);
    return launch_rows<16>(a, stream, grid);
}

}  // namespace w4a16
