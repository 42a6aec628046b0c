// W4A16 multiply for the decode case, M <= 4: one workgroup per (256-column
// stripe, K slice), the slice handed out to the workgroup's waves in small units
// as they become free.
//
// Algorithm 1's Split-K at two levels, as in the many-row form of this family
// (w4a16_stripe.hip): inside a workgroup the waves share the slice (Phase 2,
// C_i = A * B_i) and their sums meet in LDS; across workgroups the per-slice
// sums meet in the 64-bit fixed-point accumulator, or go to the FP32 workspace
// and the second pass (Phase 3).
//
// What is different here is how a slice is shared.  Measured on K = 28672,
// N = 8192 with equal contiguous runs per wave: the waves of one workgroup end
// their runs up to 3.5 us apart (the memory system serves whoever asked first,
// and a head start is never given back), and the workgroup waits for its last
// wave.  So the slice is cut into units of kUnitRows packed rows (a fixed
// partition: a unit never crosses a quantisation group), and a wave draws its
// next unit from an LDS ticket counter when it has issued the loads of the
// previous one.  Which wave computes which unit now differs from run to run, so
// the sums must not depend on it: every unit's contribution
//     sum_k x_k s (q_k - z)  =  (2^24 s) P - (s z) sum_k x_k        (Eq. 2, fp32)
// is rounded to a multiple of 2^-24 (and clamped far outside the FP16 range),
// and from there on everything is added exactly: as integer-valued doubles per
// wave, as 64-bit integers in LDS and in the cross-workgroup accumulator.
// Integer adds commute, hence bitwise reproducible results whatever the
// schedule.
//
// X, the scales and the zero points of the whole slice are staged in LDS once,
// by all waves together, ahead of the first weight loads (loads return in
// order, and these mostly come from cache): the loop then issues nothing but
// the 1 KiB wave-wide loads of packed weights.
//
// MFMA operand trick (as in w4a16_stripe.hip): all 64 lanes hold words of the
// SAME packed row (eight k) but of different columns.  Lane group g (lanes
// 16g..16g+15) feeds its words as k-group g of the 16x16x32 MFMA's B operand;
// the A operand holds row r of X in MFMA row 4g+r for k-group g only and zeros
// elsewhere, so result row 4g+r, column j -- element r of lane (g, j) -- is the
// dot product of X row r with lane (g, j)'s own column.
#include "w4a16_device.h"
#include "w4a16_finish.h"
#include "w4a16_internal.h"

#ifdef W4A16_TIMELINE
// Profiling build only (python -m paper_2601_16536_amd.build --timeline): per-wave time stamps of the kernel's
// phases, eight 64-bit words per wave: kernel entry, first unit in use, loop end, workgroup's sums done, atomic
// add back, exit, XCD id; 100 MHz ticks.  w4a16_timeline_buffer sets where they go (NULL = nowhere).
__device__ unsigned long long *g_timeline;
extern "C" int w4a16_timeline_buffer(void *device_words)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &device_words, sizeof device_words);
}
#endif

namespace w4a16 {
namespace {

constexpr int kStripe = 256;            // columns per workgroup: 64 lanes x 4 words
constexpr int kLdsLimit = 144 * 1024;
constexpr double kSumMax = 562949953421312.0;   // 2^49 = 2^25 in units of 2^-24: the clamp of a wave's and a workgroup's sum
constexpr long long kNaNMark = 1ll << 58;       // added to the LDS sum of an output by a wave whose sum is NaN

// LDS of a workgroup, in this order (all 16-byte aligned):
//   zero entry            16 B
//   tickets               16 B   (one counter)
//   acc   [MROWS][256]    64-bit sums of the waves, in units of 2^-24
//   xs    [rows][MROWS]   A-operand entries: eight halves of one packed row of X in unpack order
//   xsum  [MROWS][rows]   fp32 sum of the eight x of each packed row
//   sc    [groups][256]   FP16 scales of the stripe
//   zp    [groups][32]    packed zero points of the stripe
struct Lds {
    uint32_t acc, xs, xsum, sc, zp, bytes;
};
__host__ __device__ inline Lds lds_layout(int mrows, int rows, int groups)
{
    Lds l;
    l.acc = 32;
    l.xs = l.acc + (uint32_t)mrows * kStripe * 8;
    l.xsum = l.xs + (uint32_t)rows * mrows * 16;
    l.sc = l.xsum + (((uint32_t)rows * mrows * 4 + 15) & ~15u);
    l.zp = l.sc + (uint32_t)groups * kStripe * 2;
    l.bytes = l.zp + (uint32_t)groups * 32 * 4;
    return l;
}

// D units in flight per wave, a unit's successor requested when the unit has been used; or, AHEAD (D = 2 buffers):
// one unit in flight, its successor requested just before the unit is used, so that a wave always has a request out.
// DOT2: the dot products on the vector ALU (v_dot2_f32_f16, two k per instruction and row of X) instead of the MFMA:
// the form a wavefront-level FMA design would take, kept for the measurement that decided against it.
template <typename Act, int MROWS, int U, int D, bool AHEAD, bool DOT2>
__global__ __launch_bounds__(1024) void stripe_dyn_kernel(const GemmArgs a, const int finish, unsigned long long *__restrict__ sync)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
#ifdef W4A16_TIMELINE
    const unsigned long long T0 = __builtin_amdgcn_s_memrealtime();
    unsigned long long TF = 0;
#endif
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = blockDim.x >> 6;
    // grid: x = K slice, y = stripe: the slices of one stripe are neighbours in the launch order, hence on
    // different XCDs (workgroup b runs on XCD b mod 8); measured, the XCDs do not all stream equally fast
    // and a stripe spread over all of them ends earlier than one that sits on a slow one.
    const int slice = blockIdx.x, stripe = blockIdx.y;
    const int col0 = stripe * kStripe + 4 * lane;
    const bool ok = col0 < a.N;

    // the workgroup's K slice: groups, packed rows, units
    const int gbeg = slice * a.groups_per_split;
    int gend = gbeg + a.groups_per_split;
    if (gend > a.groups) gend = a.groups;
    const int groups = gend - gbeg;
    const int rpg = a.group >> 3;                    // packed rows per group (a multiple of 4)
    const int rows = groups * rpg;
    const int row_base = gbeg * rpg;
    const int units = rows / U;

    const uint32_t row_w = (uint32_t)a.N * 4u;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Wp) + (size_t)row_base * a.N, 0, (uint32_t)rows * row_w, kRawBuffer);
    const uint32_t vw = ok ? (uint32_t)col0 * 4u : kOutOfRange;

    const Lds L = lds_layout(MROWS, rows, groups);
    uint32_t *const tickets = reinterpret_cast<uint32_t *>(smem + 16);

    // ---- staging loads first (X, scales, zero points of the slice), then the first weight units ----
    // Every thread takes entries tid, tid + threads, ...; the first kStage of them are in flight ahead of the
    // weights, the rest (long slices only) follow in a loop behind the barrier's first half.
    constexpr int kStage = 2;
    const int nthreads = blockDim.x;
    const int n_x = rows * MROWS;                    // A-operand entries: e = row * MROWS + m
    const int n_sc = groups * (kStripe / 8);         // 16-byte pieces of the scales: e = g * 32 + piece
    const int n_zp = groups * (kStripe / 32);        // 16-byte pieces of the zero points: e = g * 8 + piece
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.X), 0, (uint32_t)((size_t)a.M * a.K * 2), kRawBuffer);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.scales) + (size_t)gbeg * a.N, 0, (uint32_t)groups * (uint32_t)a.N * 2u, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.Zp) + (size_t)gbeg * (a.N >> 3), 0, zero_point_bytes(a.Zp, (uint32_t)groups * (uint32_t)(a.N >> 3) * 4u), kRawBuffer);
    const uint32_t zfill = symmetric_fill(a.Zp);
    auto x_offset = [&](int e) -> uint32_t {  // global byte offset of entry e of X, or out of range
        const uint32_t row = (uint32_t)e / MROWS, m = (uint32_t)e % MROWS;
        return (e < n_x && m < (uint32_t)a.M) ? (m * (uint32_t)a.K + ((uint32_t)row_base + row) * 8u) * 2u : kOutOfRange;
    };
    auto sc_offset = [&](int e) -> uint32_t {
        const uint32_t g = (uint32_t)e >> 5, c = (uint32_t)stripe * kStripe + ((uint32_t)e & 31u) * 8u;
        return (e < n_sc && c < (uint32_t)a.N) ? (g * (uint32_t)a.N + c) * 2u : kOutOfRange;
    };
    auto zp_offset = [&](int e) -> uint32_t {
        const uint32_t g = (uint32_t)e >> 3, c = (uint32_t)stripe * kStripe + ((uint32_t)e & 7u) * 32u;
        return (e < n_zp && c < (uint32_t)a.N) ? (g * (uint32_t)(a.N >> 3) + (c >> 3)) * 4u : kOutOfRange;
    };
    // zero points are read in 16-byte pieces; N % 32 != 0 leaves the last piece of a row partly beyond the row:
    // those words belong to the next group's row (or are out of the buffer: zeros) and are never used.
    auto x_put = [&](int e, uint4_t d) {
        if (e >= n_x) return;
        const int row = e / MROWS, m = e % MROWS;
        *reinterpret_cast<uint4_t *>(smem + L.xs + (uint32_t)e * 16u) = Act::stage_x(d);
        *reinterpret_cast<float *>(smem + L.xsum + ((uint32_t)m * rows + row) * 4u) = Act::sum_x(d);
    };
    auto sc_put = [&](int e, uint4_t d) { if (e < n_sc) *reinterpret_cast<uint4_t *>(smem + L.sc + (uint32_t)e * 16u) = d; };
    auto zp_put = [&](int e, uint4_t d) { if (e < n_zp) *reinterpret_cast<uint4_t *>(smem + L.zp + (uint32_t)e * 16u) = d | zfill; };

    uint4_t sx[kStage], ss[kStage], sz;
#pragma unroll
    for (int q = 0; q < kStage; ++q) sx[q] = __builtin_amdgcn_raw_buffer_load_b128(rx, x_offset(tid + q * nthreads), 0, 0);
#pragma unroll
    for (int q = 0; q < kStage; ++q) ss[q] = __builtin_amdgcn_raw_buffer_load_b128(rs, sc_offset(tid + q * nthreads), 0, 0);
    sz = __builtin_amdgcn_raw_buffer_load_b128(rz, zp_offset(tid), 0, 0);

    // ---- weights: D units in flight per wave; the first D per wave are handed out statically ----
    uint4_t buf[D][U];
    int urow[D];  // first packed row (of the slice) of the unit in ring place p, -1 = none
    auto load_unit = [&](uint4_t(&b)[U], int row) {
        const bool valid = row >= 0;
#pragma unroll
        for (int t = 0; t < U; ++t)
            b[t] = __builtin_amdgcn_raw_buffer_load_b128(rw, valid ? vw : kOutOfRange, valid ? (uint32_t)(row + t) * row_w : 0u, 2);  // read once: nontemporal
    };
    constexpr int kStatic = AHEAD ? 1 : D;  // units per wave handed out without a ticket
#pragma unroll
    for (int p = 0; p < kStatic; ++p) {
        const int u = wave + p * waves;
        urow[p] = u < units ? u * U : -1;
        load_unit(buf[p], urow[p]);
    }

    // ---- LDS set-up ----
    if (tid == 0) {
        *reinterpret_cast<uint4_t *>(smem) = (uint4_t){0u, 0u, 0u, 0u};
        tickets[0] = (uint32_t)(waves * kStatic);
    }
    for (int e = tid; e < MROWS * kStripe; e += nthreads) reinterpret_cast<unsigned long long *>(smem + L.acc)[e] = 0ull;
#pragma unroll
    for (int q = 0; q < kStage; ++q) x_put(tid + q * nthreads, sx[q]);
#pragma unroll
    for (int q = 0; q < kStage; ++q) sc_put(tid + q * nthreads, ss[q]);
    zp_put(tid, sz);
    // long slices: the rest of the staging
    for (int e = tid + kStage * nthreads; e < n_x; e += nthreads) x_put(e, __builtin_amdgcn_raw_buffer_load_b128(rx, x_offset(e), 0, 0));
    for (int e = tid + kStage * nthreads; e < n_sc; e += nthreads) sc_put(e, __builtin_amdgcn_raw_buffer_load_b128(rs, sc_offset(e), 0, 0));
    for (int e = tid + nthreads; e < n_zp; e += nthreads) zp_put(e, __builtin_amdgcn_raw_buffer_load_b128(rz, zp_offset(e), 0, 0));
    __syncthreads();

    // this lane's A-operand entry of a packed row: a row of X, or the zero entry
    const int g4 = lane >> 4, r = (lane & 15) - 4 * g4;  // MFMA row 4g + r holds X row r for k-group g only
    const bool has_row = r >= 0 && r < MROWS;
    const uint32_t xa0 = has_row ? L.xs + (uint32_t)r * 16u : 0u;
    const uint32_t xstep = has_row ? (uint32_t)(MROWS * 16) : 0u;  // bytes per packed row
    const uint32_t zsh = (uint32_t)(col0 & 7) * 4u;                 // this lane's four nibbles in its zero-point word
    const uint32_t sc_lane = L.sc + (uint32_t)lane * 8u, zp_lane = L.zp + (uint32_t)(lane >> 1) * 4u;

    double tot[4][MROWS];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < MROWS; ++i) tot[c][i] = 0.0;
    const Masks masks = make_masks();
    const float4_t zero4 = {0.f, 0.f, 0.f, 0.f};

    auto draw = [&]() -> int {  // the next unit of the slice, by ticket
        uint32_t t = 0;
        if (lane == 0) t = __hip_atomic_fetch_add(tickets, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return (int)__builtin_amdgcn_readfirstlane(t);
    };
    int next = draw();

    auto compute_unit = [&](uint4_t(&b)[U], int row) {
        float4_t part[4];
        if constexpr (DOT2) {
            static_assert(!DOT2 || !Act::kBF16, "the vector-ALU form exists for FP16 only");
#pragma unroll
            for (int c = 0; c < 4; ++c) part[c] = zero4;
#pragma unroll
            for (int t = 0; t < U; ++t) {
                H8 w[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) w[c].h = unpack8(b[t][c], masks);
#pragma unroll
                for (int i = 0; i < MROWS; ++i) {
                    H8 x;  // the same entry for every lane: an LDS broadcast
                    x.u = *reinterpret_cast<const uint4_t *>(smem + L.xs + (uint32_t)((row + t) * MROWS + i) * 16u);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            H2 xp, wp;
                            xp.u = x.u[h];
                            wp.u = w[c].u[h];
                            part[c][i] = __builtin_amdgcn_fdot2(xp.h, wp.h, part[c][i], false);
                        }
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const typename Act::operand_t x = Act::x_operand(*reinterpret_cast<const uint4_t *>(smem + xa0 + (uint32_t)(row + t) * xstep));
#pragma unroll
                for (int c = 0; c < 4; ++c) part[c] = Act::mfma(x, Act::unpack(b[t][c], masks), t == 0 ? zero4 : part[c]);
            }
        }
        // the unit is done: scale and zero point (Eq. 2), then the exact sums
        const int g = (int)((uint32_t)row / (uint32_t)rpg);
        const uint2_t sc = *reinterpret_cast<const uint2_t *>(smem + sc_lane + (uint32_t)g * (kStripe * 2));
        const uint32_t zw = *reinterpret_cast<const uint32_t *>(smem + zp_lane + (uint32_t)g * 128u) >> zsh;
        float xs[MROWS];
#pragma unroll
        for (int i = 0; i < MROWS; ++i) {
            const float *p = reinterpret_cast<const float *>(smem + L.xsum + ((uint32_t)i * rows + row) * 4u);
            float s = p[0];
#pragma unroll
            for (int t = 1; t < U; ++t) s += p[t];
            xs[i] = s;
        }
        H2 s01, s23;
        s01.u = sc[0];
        s23.u = sc[1];
        const float s[4] = {(float)s01.h[0], (float)s01.h[1], (float)s23.h[0], (float)s23.h[1]};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float sp = s[c] * (Act::kCodeScale * kFixScale);  // FP16: 2^48 s (P carries 2^-24, the sums are in units of 2^-24)
            const float sz24 = -s[c] * ((float)((zw >> (4 * c)) & 15u) + Act::kCodeOffset) * kFixScale;  // -2^24 s z
#pragma unroll
            for (int i = 0; i < MROWS; ++i) {
                float v = __builtin_fmaf(sp, part[c][i], sz24 * xs[i]);            // the unit's contribution, in units of 2^-24
                // exact from here on: integers, the sum below 2^53 unless the values are beyond 2^28, far outside
                // the range the final clamp keeps anyway (an infinity or a NaN stays one)
                tot[c][i] += (double)__builtin_rintf(v);
            }
        }
    };

    if constexpr (AHEAD) {
        static_assert(!AHEAD || D == 2, "two buffers");
        int row = urow[0];
        auto step = [&](uint4_t(&cur)[U], uint4_t(&nxt)[U]) -> bool {  // uses `cur`, requests its successor into `nxt` first
            if (row < 0) return false;
            const int rown = next < units ? next * U : -1;
            load_unit(nxt, rown);
            if (next < units) next = draw();
#ifdef W4A16_TIMELINE
            if (TF == 0) { asm volatile("" ::"v"(cur[0][0])); TF = __builtin_amdgcn_s_memrealtime(); }
#endif
            compute_unit(cur, row);
            row = rown;
            return true;
        };
        while (step(buf[0], buf[1]) && step(buf[1], buf[0])) {}
    } else {
        for (;;) {
            bool any = false;
#pragma unroll
            for (int p = 0; p < D; ++p) {
                const int row = urow[p];
                if (row >= 0) {
                    any = true;
#ifdef W4A16_TIMELINE
                    if (TF == 0) { asm volatile("" ::"v"(buf[p][0][0])); TF = __builtin_amdgcn_s_memrealtime(); }
#endif
                    compute_unit(buf[p], row);
                    urow[p] = next < units ? next * U : -1;
                    load_unit(buf[p], urow[p]);
                    if (next < units) next = draw();
                }
            }
            if (!any) break;
        }
    }
#ifdef W4A16_TIMELINE
    const unsigned long long T1 = __builtin_amdgcn_s_memrealtime();
#endif

    // ---- Phase 3 inside the workgroup: exact 64-bit sums in LDS ----
    unsigned long long *acc = reinterpret_cast<unsigned long long *>(smem + L.acc);
#pragma unroll
    for (int i = 0; i < MROWS; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            double t = tot[c][i];
            const bool nan = t != t;
            t = t > kSumMax ? kSumMax : (t < -kSumMax ? -kSumMax : t);
            const long long fx = nan ? kNaNMark : (long long)t;
            if (fx != 0) __hip_atomic_fetch_add(acc + i * kStripe + 4 * lane + c, (unsigned long long)fx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    __syncthreads();
#ifdef W4A16_TIMELINE
    const unsigned long long TA = __builtin_amdgcn_s_memrealtime();
    unsigned long long TB = TA;
#endif
    // ---- and across workgroups ----
    for (int o = tid; o < MROWS * kStripe; o += nthreads) {
        const int m = o / kStripe, col = stripe * kStripe + (o % kStripe);
        if (m >= a.M || col >= a.N) continue;
        const long long fx = (long long)acc[o];
        const bool nan = fx >= (kNaNMark >> 1);  // sixteen waves' clamped sums stay below 2^53
        const size_t out = (size_t)m * a.N + col;
        if (finish == kFinishAccumulator) {
            add_slice<Act>(sync + out, to_fixed(nan ? 0ll : fx), nan, a.split, a.Y + out);
#ifdef W4A16_TIMELINE
            TB = __builtin_amdgcn_s_memrealtime();
#endif
        } else {
            constexpr long long lim = 1ll << 49;
            const float v = nan ? __builtin_nanf("") : (float)((double)(fx < -lim ? -lim : (fx > lim ? lim : fx)) * (1.0 / 16777216.0));
            if (finish == kFinishDirect)
                a.Y[out] = nan ? Act::kNaN : (uint16_t)(Act::pack2(v, 0.f) & 0xFFFFu);
            else
                a.partials[(size_t)slice * a.M * a.N + out] = v;
        }
    }
#ifdef W4A16_TIMELINE
    if (g_timeline && lane == 0) {
        unsigned long long *p = g_timeline + ((size_t)(slice * gridDim.y + stripe) * 16 + wave) * 8;
        unsigned xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        p[0] = T0; p[1] = TF; p[2] = T1; p[3] = TA; p[4] = TB; p[5] = __builtin_amdgcn_s_memrealtime(); p[6] = xcc;
    }
#endif
}

int mrows_of(int M) { return M == 1 ? 1 : (M == 2 ? 2 : 4); }

template <typename Act, int MROWS, int U, int D, bool AHEAD, bool DOT2>
hipError_t launch_m(const GemmArgs &a, int finish, unsigned long long *sync, int waves, hipStream_t stream)
{
    const size_t lds = stripe_dyn_lds_bytes(a.M, a.group, a.groups_per_split);
    if (lds > (size_t)kLdsLimit) return hipErrorInvalidValue;
    const int nstripes = (a.N + kStripe - 1) / kStripe;
    if (lds > 48 * 1024) {  // beyond the default dynamic-LDS allowance
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&stripe_dyn_kernel<Act, MROWS, U, D, AHEAD, DOT2>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((stripe_dyn_kernel<Act, MROWS, U, D, AHEAD, DOT2>), dim3(a.split, nstripes), dim3(waves * 64), lds, stream, a, finish, sync);
    return hipGetLastError();
}

}  // namespace

// LDS of one workgroup for a slice of `groups_per_split` groups.
size_t stripe_dyn_lds_bytes(int M, int group, int groups_per_split)
{
    return lds_layout(mrows_of(M), groups_per_split * (group / 8), groups_per_split).bytes;
}
int stripe_dyn_lds_limit() { return kLdsLimit; }

// `finish` says how the slices meet (w4a16_finish.h); `sync` is the accumulator it may need.
hipError_t launch_stripe_dyn(const GemmArgs &a, int finish, unsigned long long *sync, int waves, int unit_rows, int depth, bool dot2, hipStream_t stream)
{
    if (a.M > 4 || a.group % 32 != 0 || waves < 1 || waves > 16) return hipErrorInvalidValue;
    if ((a.group / 8) % unit_rows != 0) return hipErrorInvalidValue;  // a unit never crosses a quantisation group
    if (!finish_args_ok(a, finish, sync)) return hipErrorInvalidValue;
    const unsigned long long rows = (unsigned long long)a.groups_per_split * (a.group / 8);
    if (rows * a.N * 4ull >= 0x7F000000ull) return hipErrorInvalidValue;        // slice-relative 32-bit buffer offsets
    if ((unsigned long long)a.M * a.K * 2ull >= 0x7F000000ull) return hipErrorInvalidValue;
    if ((a.N + kStripe - 1) / kStripe > 65535) return hipErrorInvalidValue;  // stripes are the grid's y
    // depth 0 = one unit in flight, its successor requested ahead of its use
#define W4A16_DYN_CASE(MR, UU, DD, DOT) \
    if (mrows_of(a.M) == MR && unit_rows == UU && depth == DD && dot2 == DOT && !a.bf16) \
        return launch_m<ActF16, MR, UU, (DD ? DD : 2), DD == 0, DOT>(a, finish, sync, waves, stream);
#define W4A16_DYN_M(UU, DD, DOT) W4A16_DYN_CASE(1, UU, DD, DOT) W4A16_DYN_CASE(2, UU, DD, DOT) W4A16_DYN_CASE(4, UU, DD, DOT)
    W4A16_DYN_M(4, 1, false)  // the scheduler's choice
    W4A16_DYN_M(2, 1, false)  // the rest: for sweeps
    W4A16_DYN_M(2, 2, false)
    W4A16_DYN_M(4, 2, false)
    W4A16_DYN_M(8, 1, false)
    W4A16_DYN_M(4, 0, false)
    W4A16_DYN_M(4, 1, true)
    if (a.bf16 && unit_rows == 4 && depth == 1 && !dot2) {  // bfloat16 activations: the scheduler's choice only
        if (mrows_of(a.M) == 1) return launch_m<ActBF16, 1, 4, 1, false, false>(a, finish, sync, waves, stream);
        if (mrows_of(a.M) == 2) return launch_m<ActBF16, 2, 4, 1, false, false>(a, finish, sync, waves, stream);
        return launch_m<ActBF16, 4, 4, 1, false, false>(a, finish, sync, waves, stream);
    }
#undef W4A16_DYN_M
#undef W4A16_DYN_CASE
    return hipErrorInvalidValue;
}

}  // namespace w4a16
