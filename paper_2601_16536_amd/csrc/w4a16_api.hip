// C-ABI layer of the W4A16 GEMM library: argument checks, the Split-K
// scheduler (Algorithm 1 takes the split factor S and the block sizes as
// inputs and gives no rule for them; the rule lives here), workspace
// management and dispatch to the kernel launchers.
#include "../../include/w4a16.h"
#include "w4a16_internal.h"

#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <string.h>
#include <vector>

namespace {

using namespace w4a16;

constexpr int kMaxDevices = 64;

// Split buffers for callers that cannot allocate (w4a16_gemm_noalloc): one array per GPU the library is loaded on,
// held until the process ends.  Host code never uses the array's name as an address: each device's copy is
// looked up once with hipGetSymbolAddress.
constexpr size_t kScratchBytes = W4A16_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

struct DeviceState {
    int cus = 0;             // compute units (0 = not read yet)
    void *ws = nullptr;      // library-owned workspace (fp32 partials of the two-pass plans)
    size_t ws_bytes = 0;
    void *acc = nullptr;     // library-owned fixed-point accumulator: all zero between calls
    size_t acc_bytes = 0;
    bool acc_dirty = false;  // a launch that used it failed: cleared again before the next use
    std::vector<void *> retired;  // outgrown buffers: work already enqueued (or captured in a graph) may still use them
    void *user_ws = nullptr;      // w4a16_set_workspace: the caller's split buffers for this device
    size_t user_ws_bytes = 0;
    void *scratch_ptr = nullptr;  // this device's copy of `scratch`
};

std::mutex g_mutex;
DeviceState g_dev[kMaxDevices];
thread_local char t_hip_error[256] = "";

void note_hip_error(hipError_t e)
{
    const char *s = hipGetErrorString(e);
    strncpy(t_hip_error, s ? s : "unknown HIP error", sizeof(t_hip_error) - 1);
    t_hip_error[sizeof(t_hip_error) - 1] = 0;
}

// ---- tuning knobs (for sweeps and tests only) ----------------------------------
//
// Process-wide; each starts from the environment variable of the same name in capitals with the prefix
// W4A16_ (read once, when the library first needs it) and can be changed with w4a16_tune.  0 = the
// scheduler's own choice.
struct Tuning {
    int stripe_finish = 0;  // 1: slices always meet in the accumulator, 2: always in the workspace + second pass
    int stripe_waves = 0;   // waves per STRIPE workgroup
    int stripe_dyn = 0;     // M <= 4: 0/1 = units handed out by ticket (the default), 2 = equal contiguous runs per wave
    int stripe_unit = 0;    // packed rows per unit of the ticket form (2 or 4)
    int stripe_depth = 0;   // units in flight per wave of the ticket form (1, 2; 9 = one, its successor requested ahead of use)
    int stripe_dot2 = 0;    // 1: v_dot2_f32_f16 on the vector ALU instead of the MFMA (measurement only)
    int tile_rows = 0;      // rows of X per TILE workgroup (16, 32, 64)
    int tile_dyn = 0;       // 16 rows of X per workgroup: 1 = units always handed out by ticket, 2 = never (equal runs per wave)
    int tile_depth = 0;     // units in flight per wave of the ticket form (1, 2)
    int tile_waves = 0;     // waves per TILE workgroup (4..8)
    int tile_unit = 0;      // 16 rows of X per workgroup, by ticket: blocks of 32 k per unit (1, 2; default: up to 4 within a group)
    int tile_wide = 0;      // TILE at 32 or 64 rows of X per workgroup, FP16, group 128: 2 = the eight-wave form instead of the four-wave one
    int log = 0;            // 1: every call prints its plan on stderr
};

struct Knob {
    const char *name;
    int Tuning::*field;
};
const Knob kKnobs[] = {
    {"stripe_finish", &Tuning::stripe_finish}, {"stripe_waves", &Tuning::stripe_waves}, {"stripe_dyn", &Tuning::stripe_dyn},
    {"stripe_unit", &Tuning::stripe_unit},     {"stripe_depth", &Tuning::stripe_depth}, {"stripe_dot2", &Tuning::stripe_dot2},
    {"tile_rows", &Tuning::tile_rows},         {"tile_dyn", &Tuning::tile_dyn},         {"tile_depth", &Tuning::tile_depth},
    {"tile_waves", &Tuning::tile_waves},       {"tile_wide", &Tuning::tile_wide},         {"tile_unit", &Tuning::tile_unit},
    {"log", &Tuning::log},
};

Tuning &tuning()
{
    static Tuning t = [] {
        Tuning v;
        for (const Knob &k : kKnobs) {
            char env[64] = "W4A16_";
            size_t n = strlen(env);
            for (const char *c = k.name; *c && n + 1 < sizeof env; ++c) env[n++] = (char)(*c >= 'a' && *c <= 'z' ? *c - 32 : *c);
            env[n] = 0;
            if (const char *e = getenv(env)) v.*(k.field) = atoi(e);
        }
        return v;
    }();
    return t;
}

// Current device index, or -1 when no GPU is usable (planning still works then,
// with the MI355X's 256 compute units assumed).
int current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return (dev >= 0 && dev < kMaxDevices) ? dev : -1;
}

int compute_units(int dev)
{
    if (dev < 0) return 256;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (g_dev[dev].cus == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
            (void)hipGetLastError();
            cus = 256;
        }
        g_dev[dev].cus = cus;
    }
    return g_dev[dev].cus;
}

int check_shape(int group, int M, int N, int K)
{
    if (M < 1 || N < 8 || K < 8) return W4A16_ERR_SHAPE;
    if (N % 8 != 0 || K % 8 != 0) return W4A16_ERR_SHAPE;
    if (M > 16 * 65535 || N > (1 << 22) || (long long)K > (1LL << 30)) return W4A16_ERR_SHAPE;
    if (group < 32 || group % 32 != 0 || K % group != 0) return W4A16_ERR_GROUP;
    return W4A16_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The kernels address X, and a K slice of the weights, with 32-bit byte offsets.
bool fits_32bit_offsets(int M, int N, int K, int group, int gps)
{
    return (unsigned long long)M * K * 2ull < 0x7F000000ull && (unsigned long long)gps * (group / 8) * N * 4ull < 0x7F000000ull;
}

// ---- the Split-K scheduler ---------------------------------------------------
//
// Algorithm 1 takes the split factor S and the block sizes as inputs.  Here the
// scheduler (kernel = AUTO, split = 0) chooses them from the shape alone:
//
// STRIPE (M = 1 from about 4 MB of packed weights on, M = 2 from about 20 MB, M <= 4 from about 32 MB): 256-column stripes
//   x S slices of K with S = compute units / stripes, rounded down: one workgroup per compute unit whose
//   waves share the slice.
// TILE (everything else): 64-column tiles x 16, 32 or 64 rows of X per workgroup (as many rows as still
//   leave a workgroup per compute unit at S = 1), eight waves own contiguous runs of the slice's K;
//   S = compute units / workgroups, rounded down (a workgroup too many would run as a second round).
//   Its time does not depend on M up to 16; STRIPE's grows with the S M N atomic adds of its finish.
//
// WAVE_SPLIT (M <= 4) is kept as a forced plan (w4a16_gemm_ex), the data-parallel form for comparisons:
//   one workgroup of sixteen waves per column tile of 32 or 64 columns; the sixteen waves are sixteen K
//   slices whose partial results meet in LDS.  A split across workgroups is added only when the column
//   tiles cover at most a quarter of the compute units and the slices stay long.
//
// How the K slices of different workgroups of a STRIPE or TILE plan meet: in the 64-bit fixed-point accumulator (one
// returning atomic add per output and slice; measured: the GPU retires about 150 of them per nanosecond)
// while that is cheaper than a second launch (about 3.3 us, measured), else in the FP32 workspace and the
// second pass.  Measured crossover: between 0.5 M and 1 M adds.  The other families always take the second pass.
bool slices_meet_in_accumulator(int M, int N, int S)
{
    if (S > 63) return false;  // the accumulator counts arrivals in six bits
    if (tuning().stripe_finish == 1) return true;
    if (tuning().stripe_finish == 2) return false;
    return (long long)S * M * N <= 640 * 1024;
}

int finish_of(int kernel, int M, int N, int S)
{
    if (S == 1) return kFinishDirect;
    if (kernel != W4A16_KERNEL_STRIPE && kernel != W4A16_KERNEL_TILE) return kFinishSecondPass;
    return slices_meet_in_accumulator(M, N, S) ? kFinishAccumulator : kFinishSecondPass;
}

// Workspace of a plan: nothing, the accumulator [M, N], or the FP32 partials [S, M, N].
size_t workspace_of(int kernel, int M, int N, int S)
{
    switch (finish_of(kernel, M, N, S)) {
    case kFinishDirect: return 0;
    case kFinishAccumulator: return (size_t)M * N * sizeof(unsigned long long);
    default: return (size_t)S * M * N * sizeof(float);
    }
}

bool stripe_by_ticket(int M) { return M <= 4 && tuning().stripe_dyn != 2; }
// TILE with one block of 16 rows of X: the ticket form (measured 1 to 6 % faster than equal runs per wave at M <= 16;
// with several row blocks, which re-read the weights from the L2, 3 % slower).
bool tile_by_ticket(int M, int rows_x) { return rows_x == 16 && (tuning().tile_dyn == 1 || (M <= 16 && tuning().tile_dyn != 2)); }

// TILE at 64 rows of X per workgroup and group = 128: four waves per workgroup, each alone on its SIMD
// (w4a16_tile_wide.hip; FP16 only: BF16 activations run such a plan with the eight-wave form).
bool tile_wide(int rows_x, int group) { return (rows_x == 64 || rows_x == 32) && group == 128 && tuning().tile_wide != 2; }

// LDS a STRIPE workgroup needs for a slice of gps groups, and the most it may use.
size_t stripe_lds(int M, int group, int gps, int waves)
{
    return stripe_by_ticket(M) ? stripe_dyn_lds_bytes(M, group, gps) : stripe_lds_bytes(M, group, gps, waves);
}
size_t stripe_lds_max(int M) { return (size_t)(stripe_by_ticket(M) ? stripe_dyn_lds_limit() : stripe_lds_limit()); }

// Estimated time (us) of a TILE plan for M > 16: `rows` of X per workgroup, K in S slices.  A model of three terms with
// constants measured on K = N = 8192 and on the paper's Fig. 2 shapes at M = 32 and 64 (it orders the 30 plans measured
// there as the clock does): a fixed 3 us; rounds of workgroups x blocks of 32 k per wave x the time of a block
// (four-wave form: 0.24 us at 32 rows, 0.37 at 64; eight-wave form: 0.37, 0.56, 0.94 at 16, 32, 64 rows); and how the
// slices meet (accumulator: 1 us, and beyond 200 K adds 1 us per 60 K; second pass: 3.3 us and the partials at 3 TB/s).
double tile_plan_cost(int M, int N, int K, int group, int rows, int S, int cus)
{
    const int G = K / group;
    const int gps = (G + S - 1) / S;
    S = (G + gps - 1) / gps;
    const bool four = tile_wide(rows, group);
    const int waves = four ? 4 : 8;
    const double per_block = four ? (rows == 64 ? 0.37 : 0.24) : (rows == 64 ? 0.94 : (rows == 32 ? 0.56 : 0.37));
    const long long tiles = (N + 63) / 64, wgs = tiles * ((M + rows - 1) / rows) * S;
    const long long rounds = (wgs + cus - 1) / cus;
    const long long blocks = ((long long)gps * (group / 32) + waves - 1) / waves;
    double finish = 0.0;
    if (S > 1) {
        const double adds = (double)S * M * N;
        finish = slices_meet_in_accumulator(M, N, S) ? 1.0 + (adds > 2e5 ? (adds - 2e5) / 6e4 : 0.0) : 3.3 + 2.0 * adds * 4.0 / 3e6;
    }
    return 3.0 + (double)rounds * (double)blocks * per_block + finish;
}

int make_plan(int M, int N, int K, int group, int kernel, int split, int cus, w4a16_plan *p)
{
    const int G = K / group;
    if (kernel == W4A16_KERNEL_AUTO) {
        // STRIPE streams large weight matrices faster than TILE, but its 256-column stripes need four
        // times the slices, hence four times the atomic adds (S M N), and its work per unit of K grows with M.
        // Measured on the five configurations, the six (N, K) pairs of the paper's Fig. 2 and three K << N shapes
        // (2 MB to 117 MB of packed weights): STRIPE wins at M = 1 from about 4 MB on, at M = 2 from about
        // 20 MB on, at M = 3, 4 from about 32 MB on; TILE everywhere else.
        const double packed = 0.5 * (double)K * (double)N;
        const bool stripe = (M == 1 && packed >= 4e6) || (M == 2 && packed >= 20e6) || (M <= 4 && packed >= 32e6);
        kernel = stripe ? W4A16_KERNEL_STRIPE : W4A16_KERNEL_TILE;
    }
    if (kernel != W4A16_KERNEL_WAVE_SPLIT && kernel != W4A16_KERNEL_STRIPE && kernel != W4A16_KERNEL_TILE)
        return W4A16_ERR_UNSUPPORTED;
    if (kernel == W4A16_KERNEL_WAVE_SPLIT && M > 4) return W4A16_ERR_UNSUPPORTED;
    if (kernel == W4A16_KERNEL_STRIPE && M > 16) return W4A16_ERR_UNSUPPORTED;
    if (split < 0 || split > G) return W4A16_ERR_UNSUPPORTED;
    p->kernel = kernel;
    long long tiles;
    int S = split;
    if (kernel == W4A16_KERNEL_STRIPE) {
        p->tile_n = 256;
        p->tile_m = M <= 4 ? 4 : 16;
        tiles = (N + 255) / 256;
        if (tiles > 65535) return W4A16_ERR_UNSUPPORTED;  // a grid dimension
        const int wmin = stripe_min_waves(M), wmax = stripe_max_waves(M);
        if (S == 0) S = (int)(cus / tiles);  // at most one workgroup per compute unit (measured, N = 14336: 280 workgroups 11.4 us, 224 8.9 us)
        if (S < 1) S = 1;
        if (S > G) S = G;
        int gps = (G + S - 1) / S;
        // the slice's X rows (and, handed out by ticket, its scales) must fit the workgroup's LDS and its weights a
        // 31-bit buffer: shorten the slice if not
        while (gps > 1 && (stripe_lds(M, group, gps, wmin) > stripe_lds_max(M) || !fits_32bit_offsets(1, N, 8, group, gps)))
            gps = (gps + 1) / 2;
        S = (G + gps - 1) / gps;
        if (stripe_lds(M, group, gps, wmin) > stripe_lds_max(M)) return W4A16_ERR_UNSUPPORTED;
        if (S > 65535) return W4A16_ERR_UNSUPPORTED;  // a grid dimension of the many-row form
        // waves: each should get at least four blocks of 16 k; eight measured best for the ticket form (M <= 4), which
        // is also the most the many-row form holds
        const long long nblocks = (long long)gps * (group / 16);
        int waves = (int)(nblocks / 4);
        const int wbest = stripe_by_ticket(M) ? 8 : (wmax > 12 ? 12 : wmax);
        waves = waves < wmin ? wmin : (waves > wbest ? wbest : waves);
        if (tuning().stripe_waves >= wmin && tuning().stripe_waves <= wmax) waves = tuning().stripe_waves;
        while (waves > wmin && stripe_lds(M, group, gps, waves) > stripe_lds_max(M)) --waves;
        p->waves_k = waves;
        p->threads = waves * 64;
        p->split = S;
        p->groups_per_split = gps;
        p->workgroups = (int)(tiles * S);
        p->workspace_bytes = workspace_of(kernel, M, N, S);
        return fits_32bit_offsets(M, N, K, group, gps) ? W4A16_OK : W4A16_ERR_UNSUPPORTED;
    }
    if (kernel == W4A16_KERNEL_TILE) {
        p->tile_n = 64;
        p->waves_k = 8;
        p->threads = 512;
        tiles = (N + 63) / 64;
        // Rows of X per workgroup: as many (16, 32 or 64: each loaded weight word feeds that many MFMA rows)
        // as still leave one workgroup per compute unit without splitting K across workgroups (a split costs
        // the FP32 partials and the second pass).
        int rows_x = 64;
        while (rows_x > 16 && (rows_x / 2 >= M || tiles * ((M + rows_x - 1) / rows_x) < cus)) rows_x /= 2;
        const int tr = tuning().tile_rows;
        if (tr == 16 || tr == 32 || tr == 64) {
            rows_x = tr;
        } else if (M > 16 && group % 32 == 0) {
            // M > 16, the scheduler's own S: the rule above is a poor one where it puts a few workgroups more than
            // compute units into a second round, or gives up large row blocks that a split of K would have filled
            // (measured, N = 7168, K = 18432, M = 64: 49.7 us at 16 rows against 33.0 at 64 rows, S = 2): the
            // cheapest of (rows, S) by the model, S up to one workgroup per compute unit (a forced S: the rows for it)
            double best = 1e30;
            for (int r = 16; r <= 64; r *= 2) {
                if (r > 16 && r / 2 >= M) break;  // more than half of the block's rows would be empty
                const long long w1 = tiles * ((M + r - 1) / r);
                const int smax = split ? split : ((int)(cus / w1) < 1 ? 1 : ((int)(cus / w1) > G ? G : (int)(cus / w1)));
                for (int s = split ? split : 1; s <= smax; ++s) {
                    const double c = tile_plan_cost(M, N, K, group, r, s, cus);
                    if (c < best) { best = c; rows_x = r; S = s; }
                }
            }
        }
        p->tile_m = rows_x;
        const int tw = tuning().tile_waves;
        if (tw >= 4 && tw <= (tile_by_ticket(M, rows_x) ? 16 : 8)) { p->waves_k = tw; p->threads = 64 * tw; }
        if (tile_wide(rows_x, group)) { p->waves_k = 4; p->threads = 256; }
        const long long wgs = tiles * ((M + rows_x - 1) / rows_x);
        if (S == 0) S = (int)(cus / wgs);  // never more workgroups than compute units: the extra ones would run as a second round
        if (S < 1) S = 1;
        if (S > G) S = G;
        int gps = (G + S - 1) / S;
        while (gps > 1 && !fits_32bit_offsets(1, N, 8, group, gps)) gps = (gps + 1) / 2;
        S = (G + gps - 1) / gps;
        p->split = S;
        p->groups_per_split = gps;
        p->workgroups = (int)(wgs * S);
        p->workspace_bytes = workspace_of(kernel, M, N, S);
        if (((long long)tiles * S + 7) / 8 * 8 * ((M + rows_x - 1) / rows_x) > 0x7FFFFFFFLL) return W4A16_ERR_UNSUPPORTED;
        return fits_32bit_offsets(M, N, K, group, gps) ? W4A16_OK : W4A16_ERR_UNSUPPORTED;
    }
    {  // WAVE_SPLIT
        p->tile_n = (N + 63) / 64 >= cus ? 64 : 32;
        p->tile_m = 4;
        p->waves_k = 16;
        p->threads = 1024;
        tiles = (N + p->tile_n - 1) / p->tile_n;
        if (tiles > 65535) return W4A16_ERR_UNSUPPORTED;  // a grid dimension
        if (S == 0) {
            // One launch unless the tiles cover at most a quarter of the compute units AND each
            // workgroup would still stream at least 128 KiB per slice (below that the second
            // pass costs more than the idle units).
            S = 1;
            const long long per_wg = (long long)K * p->tile_n / 2;
            if (4 * tiles <= cus) {
                S = (int)(cus / tiles);
                if (S > per_wg / (128 * 1024)) S = (int)(per_wg / (128 * 1024));
            }
        }
    }
    if (S < 1) S = 1;
    if (S > G) S = G;
    int gps = (G + S - 1) / S;
    // slices keep 32-bit buffer offsets: raise S until a slice is below ~2 GiB
    while (gps > 1 && !fits_32bit_offsets(1, N, 8, group, gps)) gps = (gps + 1) / 2;
    S = (G + gps - 1) / gps;  // no empty slice
    p->split = S;
    p->groups_per_split = gps;
    p->workgroups = (int)(tiles * S);
    p->workspace_bytes = workspace_of(kernel, M, N, S);
    return fits_32bit_offsets(M, N, K, group, gps) ? W4A16_OK : W4A16_ERR_UNSUPPORTED;
}

// ---- split buffers --------------------------------------------------------------

// True when `stream` is being captured into a graph: nothing may be allocated or synchronised then.
bool capturing(hipStream_t stream)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

// Grows one of the library-owned buffers.  The old buffer is not freed: work enqueued earlier, or recorded in a
// graph, may still use it; it goes to the retired list until w4a16_shutdown.  Never called during stream capture.
int grow(DeviceState &d, void **buf, size_t *have, size_t bytes, size_t floor_bytes, bool zeroed)
{
    size_t want = bytes + bytes / 4;
    if (want < floor_bytes) want = floor_bytes;
    void *ptr = nullptr;
    hipError_t e = hipMalloc(&ptr, want);
    if (e != hipSuccess) { note_hip_error(e); (void)hipGetLastError(); return W4A16_ERR_WORKSPACE; }
    if (zeroed) {
        // cleared before any stream can see it: the copy engine's memset, then a wait for the device
        e = hipMemset(ptr, 0, want);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) { note_hip_error(e); (void)hipFree(ptr); return W4A16_ERR_HIP; }
    }
    if (*buf) d.retired.push_back(*buf);
    *buf = ptr;
    *have = want;
    return W4A16_OK;
}

enum Source { kFromLibrary, kFromCall, kFromScratch };

struct Buffers {
    unsigned long long *sync = nullptr;  // the accumulator: zero before the launch, left zero by it
    float *partials = nullptr;
    bool library_acc = false;
};

int find_buffers(int dev, const w4a16_plan &plan, int finish, int M, int N, hipStream_t st, Source src, void *call_ws,
                 size_t call_ws_bytes, Buffers *out)
{
    if (finish == kFinishDirect) return W4A16_OK;
    void *given = nullptr;
    size_t given_bytes = 0;
    if (src == kFromCall) {
        given = call_ws;
        given_bytes = call_ws_bytes;
    } else if (src == kFromScratch) {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState &d = g_dev[dev];
        if (!d.scratch_ptr) {  // once per device, with that device current
            void *ptr = nullptr;
            hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) { note_hip_error(e); (void)hipGetLastError(); return W4A16_ERR_HIP; }
            d.scratch_ptr = ptr;
        }
        given = d.scratch_ptr;
        given_bytes = kScratchBytes;
    } else {
        std::lock_guard<std::mutex> lock(g_mutex);
        if (g_dev[dev].user_ws) {
            given = g_dev[dev].user_ws;
            given_bytes = g_dev[dev].user_ws_bytes;
        }
    }
    if (given) {
        if (given_bytes < plan.workspace_bytes) return W4A16_ERR_WORKSPACE;
        if (finish == kFinishAccumulator) {  // contents unknown: cleared by a small launch first
            out->sync = static_cast<unsigned long long *>(given);
            hipError_t e = launch_accumulator_clear(out->sync, (size_t)M * N, st);
            if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
        } else {
            out->partials = static_cast<float *>(given);
        }
        return W4A16_OK;
    }
    // library-owned, grown on demand
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState &d = g_dev[dev];
    if (finish == kFinishAccumulator) {
        if (d.acc_bytes < plan.workspace_bytes) {
            if (capturing(st)) return W4A16_ERR_WORKSPACE;
            int rc = grow(d, &d.acc, &d.acc_bytes, plan.workspace_bytes, 1u << 20, true);
            if (rc) return rc;
            d.acc_dirty = false;
        }
        out->sync = static_cast<unsigned long long *>(d.acc);
        out->library_acc = true;
        if (d.acc_dirty) {
            hipError_t e = launch_accumulator_clear(out->sync, d.acc_bytes / 8, st);
            if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
            d.acc_dirty = false;
        }
    } else {
        if (d.ws_bytes < plan.workspace_bytes) {
            if (capturing(st)) return W4A16_ERR_WORKSPACE;
            int rc = grow(d, &d.ws, &d.ws_bytes, plan.workspace_bytes, 0, false);
            if (rc) return rc;
        }
        out->partials = static_cast<float *>(d.ws);
    }
    return W4A16_OK;
}

void log_plan(const char *entry, int M, int N, int K, int group, const w4a16_plan &p, int finish)
{
    static const char *const kFinish[] = {"direct", "accumulator", "second pass"};
    fprintf(stderr, "w4a16: %s M=%d N=%d K=%d group=%d -> kernel=%d S=%d groups/slice=%d tile=%dx%d waves=%d workgroups=%d finish=%s workspace=%zu\n",
            entry, M, N, K, group, p.kernel, p.split, p.groups_per_split, p.tile_m, p.tile_n, p.waves_k, p.workgroups,
            kFinish[finish], p.workspace_bytes);
}

int run(const char *entry, const void *X, const uint32_t *Wp, const void *scales, const uint32_t *zeros, int group, int M, int N,
        int K, void *Y, void *stream, int kernel, int split, Source src, void *call_ws, size_t call_ws_bytes, bool bf16 = false)
{
    t_hip_error[0] = 0;
    if (!X || !Wp || !scales || !Y) return W4A16_ERR_NULL;  // zeros may be null: symmetric quantisation
    if (src == kFromCall && !call_ws) return W4A16_ERR_NULL;
    int rc = check_shape(group, M, N, K);
    if (rc) return rc;
    if (!aligned16(X) || !aligned16(Wp) || !aligned16(scales) || !aligned16(zeros) || !aligned16(Y)) return W4A16_ERR_ALIGN;
    if (src == kFromCall && (reinterpret_cast<uintptr_t>(call_ws) & 255u)) return W4A16_ERR_ALIGN;

    const int dev = current_device();
    if (dev < 0) { note_hip_error(hipErrorNoDevice); return W4A16_ERR_HIP; }
    w4a16_plan plan;
    rc = make_plan(M, N, K, group, kernel, split, compute_units(dev), &plan);
    if (rc) return rc;
    // bfloat16 activations: the forms the scheduler chooses from (STRIPE by ticket for M <= 4, TILE)
    if (bf16 && (plan.kernel == W4A16_KERNEL_WAVE_SPLIT || (plan.kernel == W4A16_KERNEL_STRIPE && !stripe_by_ticket(M))))
        return W4A16_ERR_UNSUPPORTED;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int finish = finish_of(plan.kernel, M, N, plan.split);
    if (tuning().log) log_plan(entry, M, N, K, group, plan, finish);
    Buffers b;
    rc = find_buffers(dev, plan, finish, M, N, st, src, call_ws, call_ws_bytes, &b);
    if (rc) return rc;

    GemmArgs a;
    a.X = static_cast<const uint16_t *>(X);
    a.Wp = Wp;
    a.scales = static_cast<const uint16_t *>(scales);
    a.Zp = zeros;
    a.Y = static_cast<uint16_t *>(Y);
    a.partials = b.partials;
    a.group = group; a.M = M; a.N = N; a.K = K;
    a.split = plan.split;
    a.groups_per_split = plan.groups_per_split;
    a.groups = K / group;
    a.bf16 = bf16 ? 1 : 0;

    hipError_t e;
    if (plan.kernel == W4A16_KERNEL_STRIPE && stripe_by_ticket(M)) {
        // measured on K = 4096 ... 28672 at M = 1, 2, 4: units of four packed rows, one in flight per wave, eight waves
        // (deeper rings, smaller or larger units, a successor requested ahead of use: all slower by 2 to 10 %)
        const int tu = tuning().stripe_unit, td = tuning().stripe_depth;
        const int unit = tu == 2 ? 2 : (tu == 8 && group % 64 == 0 ? 8 : 4), depth = td == 2 ? 2 : (td == 9 ? 0 : 1);
        if (bf16)
            e = launch_stripe_dyn(a, finish, b.sync, plan.waves_k, 4, 1, false, st);
        else
            e = launch_stripe_dyn(a, finish, b.sync, plan.waves_k, unit, depth, tuning().stripe_dot2 == 1, st);
    } else if (plan.kernel == W4A16_KERNEL_STRIPE) {
        e = launch_stripe(a, finish, b.sync, plan.waves_k, st);
    } else if (plan.kernel == W4A16_KERNEL_TILE && tile_by_ticket(M, plan.tile_m)) {
        e = launch_tile_dyn(a, finish, b.sync, plan.waves_k, tuning().tile_depth == 2 && !bf16 && plan.waves_k <= 8 ? 2 : 1, tuning().tile_unit, st);
    } else if (plan.kernel == W4A16_KERNEL_TILE && tile_wide(plan.tile_m, group) && !bf16) {
        // four waves with the whole register file each; measured on M = 128, K = N = 8192: 27.5 us against 33.1 us with eight
        e = launch_tile_wide(a, finish, b.sync, plan.tile_m, st);
    } else if (plan.kernel == W4A16_KERNEL_TILE) {
        e = launch_tile(a, finish, b.sync, plan.tile_m, tile_wide(plan.tile_m, group) ? 8 : plan.waves_k, st);
    } else {
        e = launch_wave_split(a, plan.tile_n, st);
    }
    if (e == hipSuccess && finish == kFinishSecondPass) e = launch_reduce(a.partials, plan.split, M, N, a.Y, bf16, st);
    if (e != hipSuccess) {
        note_hip_error(e);
        if (b.library_acc) {  // what the failed launch left in the accumulator is unknown
            std::lock_guard<std::mutex> lock(g_mutex);
            g_dev[dev].acc_dirty = true;
        }
        return W4A16_ERR_HIP;
    }
    return W4A16_OK;
}

}  // namespace

extern "C" {

int w4a16_gemm(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
               int N, int K, void *Y, void *stream)
{
    return run("gemm", X, Wpacked, scales, zeros, group, M, N, K, Y, stream, W4A16_KERNEL_AUTO, 0, kFromLibrary, nullptr, 0);
}

int w4a16_gemm_ex(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
                  int N, int K, void *Y, void *stream, int kernel, int split)
{
    return run("gemm_ex", X, Wpacked, scales, zeros, group, M, N, K, Y, stream, kernel, split, kFromLibrary, nullptr, 0);
}

int w4a16_gemm_ws(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
                  int N, int K, void *Y, void *stream, int kernel, int split, void *workspace, size_t workspace_bytes)
{
    return run("gemm_ws", X, Wpacked, scales, zeros, group, M, N, K, Y, stream, kernel, split, kFromCall, workspace, workspace_bytes);
}

int w4a16_gemm_noalloc(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
                       int N, int K, void *Y, void *stream, int kernel, int split)
{
    return run("gemm_noalloc", X, Wpacked, scales, zeros, group, M, N, K, Y, stream, kernel, split, kFromScratch, nullptr, 0);
}

int w4a16_gemm_bf16(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
                    int N, int K, void *Y, void *stream, int kernel, int split)
{
    return run("gemm_bf16", X, Wpacked, scales, zeros, group, M, N, K, Y, stream, kernel, split, kFromLibrary, nullptr, 0, true);
}

int w4a16_set_workspace(void *workspace, size_t workspace_bytes)
{
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return W4A16_ERR_ALIGN;
    if (workspace && workspace_bytes < 256) return W4A16_ERR_WORKSPACE;
    const int dev = current_device();
    if (dev < 0) { note_hip_error(hipErrorNoDevice); return W4A16_ERR_HIP; }
    std::lock_guard<std::mutex> lock(g_mutex);
    g_dev[dev].user_ws = workspace;
    g_dev[dev].user_ws_bytes = workspace ? workspace_bytes : 0;
    return W4A16_OK;
}

size_t w4a16_workspace_bytes(int M, int N, int K, int group)
{
    w4a16_plan p;
    if (check_shape(group, M, N, K)) return 0;
    if (make_plan(M, N, K, group, W4A16_KERNEL_AUTO, 0, compute_units(current_device()), &p)) return 0;
    return p.workspace_bytes ? p.workspace_bytes : 256;
}

int w4a16_query_plan(int M, int N, int K, int group, int kernel, int split, w4a16_plan *out)
{
    if (!out) return W4A16_ERR_NULL;
    int rc = check_shape(group, M, N, K);
    if (rc) return rc;
    return make_plan(M, N, K, group, kernel, split, compute_units(current_device()), out);
}

int w4a16_tune(const char *knob, int value)
{
    if (!knob) return W4A16_ERR_NULL;
    for (const Knob &k : kKnobs)
        if (strcmp(knob, k.name) == 0) {
            tuning().*(k.field) = value;
            return W4A16_OK;
        }
    return W4A16_ERR_UNSUPPORTED;
}

int w4a16_reduce(const float *partials, int S, int M, int N, void *Y, void *stream)
{
    t_hip_error[0] = 0;
    if (!partials || !Y) return W4A16_ERR_NULL;
    if (S < 1 || M < 1 || N < 8 || N % 8 != 0) return W4A16_ERR_SHAPE;
    if (!aligned16(partials) || !aligned16(Y)) return W4A16_ERR_ALIGN;
    hipError_t e = launch_reduce(partials, S, M, N, static_cast<uint16_t *>(Y), false, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
    return W4A16_OK;
}

int w4a16_dequant(const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int N, int K,
                  void *W16, void *stream)
{
    t_hip_error[0] = 0;
    if (!Wpacked || !scales || !W16) return W4A16_ERR_NULL;  // zeros may be null: symmetric quantisation
    int rc = check_shape(group, 1, N, K);
    if (rc) return rc;
    if (!aligned16(Wpacked) || !aligned16(scales) || !aligned16(zeros) || !aligned16(W16)) return W4A16_ERR_ALIGN;
    hipError_t e = launch_dequant(Wpacked, static_cast<const uint16_t *>(scales), zeros, group, N, K,
                                  static_cast<uint16_t *>(W16), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
    return W4A16_OK;
}

int w4a16_stream_probe(const void *a, size_t a_bytes, const void *b, size_t b_bytes, const void *c, size_t c_bytes, void *sink,
                       void *stream)
{
    t_hip_error[0] = 0;
    if (!sink || (!a && !b && !c)) return W4A16_ERR_NULL;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return W4A16_ERR_ALIGN;
    const int dev = current_device();
    if (dev < 0) { note_hip_error(hipErrorNoDevice); return W4A16_ERR_HIP; }
    hipError_t e = launch_stream_probe(a, a ? a_bytes : 0, b, b ? b_bytes : 0, c, c ? c_bytes : 0, static_cast<uint32_t *>(sink),
                                       compute_units(dev), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
    return W4A16_OK;
}

int w4a16_quantize(const void *W16, int group, int N, int K, uint32_t *Wpacked, void *scales, uint32_t *zeros,
                   void *stream)
{
    t_hip_error[0] = 0;
    if (!W16 || !Wpacked || !scales || !zeros) return W4A16_ERR_NULL;
    int rc = check_shape(group, 1, N, K);
    if (rc) return rc;
    if (!aligned16(W16) || !aligned16(Wpacked) || !aligned16(scales) || !aligned16(zeros)) return W4A16_ERR_ALIGN;
    hipError_t e = launch_quantize(static_cast<const uint16_t *>(W16), group, N, K, Wpacked, static_cast<uint16_t *>(scales),
                                   zeros, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
    return W4A16_OK;
}

const char *w4a16_status_string(int status)
{
    switch (status) {
    case W4A16_OK: return "ok";
    case W4A16_ERR_NULL: return "null pointer";
    case W4A16_ERR_SHAPE: return "bad shape (need M >= 1, N % 8 == 0, K % 8 == 0)";
    case W4A16_ERR_GROUP: return "bad group (need group % 32 == 0 and K % group == 0)";
    case W4A16_ERR_ALIGN: return "pointer not aligned (16 bytes for data, 256 for a workspace)";
    case W4A16_ERR_WORKSPACE: return "workspace too small, or it would have to be allocated while the stream is being captured, or allocation failed";
    case W4A16_ERR_HIP: return "HIP runtime error";
    case W4A16_ERR_UNSUPPORTED: return "forced kernel or split not valid for this shape, or the shape is beyond the kernels' 32-bit offsets";
    default: return "unknown status";
    }
}

const char *w4a16_last_hip_error(void) { return t_hip_error; }

void w4a16_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    for (int d = 0; d < kMaxDevices; ++d) {
        DeviceState &s = g_dev[d];
        if (!s.ws && !s.acc && s.retired.empty()) continue;
        int prev = -1;
        if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(d) == hipSuccess) {
            if (s.ws) (void)hipFree(s.ws);
            if (s.acc) (void)hipFree(s.acc);
            for (void *p : s.retired) (void)hipFree(p);
            (void)hipSetDevice(prev);
        }
        s.ws = nullptr;
        s.ws_bytes = 0;
        s.acc = nullptr;
        s.acc_bytes = 0;
        s.acc_dirty = false;
        s.retired.clear();
    }
}

}  // extern "C"
