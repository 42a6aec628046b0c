// C-ABI layer of the W4A16 GEMM library: argument checks, the Split-K
// scheduler (Algorithm 1 takes the split factor S and the block sizes as
// inputs and gives no rule for them; the rule lives here), workspace
// management and dispatch to the kernel launchers.
#include "../../include/w4a16.h"
#include "w4a16_internal.h"

#include <cstdlib>
#include <mutex>
#include <string.h>

namespace {

using namespace w4a16;

constexpr int kMaxDevices = 64;

struct DeviceState {
    int cus = 0;             // compute units (0 = not read yet)
    void *ws = nullptr;      // library-owned workspace (fp32 partials of the two-pass plans)
    size_t ws_bytes = 0;
    void *acc = nullptr;     // library-owned fixed-point accumulator of the STRIPE and TILE families: all zero between calls
    size_t acc_bytes = 0;
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

// ---- the Split-K scheduler ---------------------------------------------------
//
// Algorithm 1 takes the split factor S and the block sizes as inputs.  Here the
// scheduler (kernel = AUTO, split = 0) chooses them from the shape alone:
//
// STRIPE (M <= 2 from about 10 MB of packed weights on, M <= 4 from about 48 MB on): 256-column stripes
//   x S slices of K with S = compute units / stripes, rounded down: one workgroup per compute unit; ten
//   to sixteen waves of a workgroup own contiguous runs of the slice's rows.
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
    if (S > 255) return false;
    if (const char *e = getenv("W4A16_STRIPE_FINISH")) {  // tuning aid for sweeps, not part of the contract
        if (e[0] == 'a') return true;
        if (e[0] == 'w') return false;
    }
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

int make_plan(int M, int N, int K, int group, int kernel, int split, int cus, w4a16_plan *p)
{
    const int G = K / group;
    if (kernel == W4A16_KERNEL_AUTO) {
        // STRIPE streams large weight matrices about 8 % faster than TILE, but its 256-column stripes need four
        // times the slices, hence four times the atomic adds (S M N), and it carries more fixed cost.
        // Measured on sixteen shapes from 2 MB to 117 MB of packed weights: STRIPE wins for M <= 2 from about
        // 10 MB on, for M = 3, 4 only from about 48 MB on; TILE everywhere else.
        const double packed = 0.5 * (double)K * (double)N;
        const bool stripe = (M <= 2 && packed >= 10e6) || (M <= 4 && packed >= 48e6);
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
        const int wmin = stripe_min_waves(M), wmax = stripe_max_waves(M);
        if (S == 0) S = (int)(cus / tiles);  // at most one workgroup per compute unit (measured, N = 14336: 280 workgroups 11.4 us, 224 8.9 us)
        if (S < 1) S = 1;
        if (S > G) S = G;
        int gps = (G + S - 1) / S;
        // the slice's X rows must fit the workgroup's LDS and its weights a 31-bit buffer: shorten the slice if not
        while (gps > 1 && (stripe_lds_bytes(M, group, gps, wmin) > (size_t)stripe_lds_limit() ||
                           (unsigned long long)gps * (group / 8) * N * 4ull >= 0x7F000000ull))
            gps = (gps + 1) / 2;
        S = (G + gps - 1) / gps;
        if (stripe_lds_bytes(M, group, gps, wmin) > (size_t)stripe_lds_limit()) return W4A16_ERR_UNSUPPORTED;
        if (S > 65535) return W4A16_ERR_UNSUPPORTED;  // the slices are the grid's second dimension
        // waves: each should own at least four blocks of 16 k; twelve measured best on the large shapes for
        // M <= 4 (ten to sixteen are within 3 % of each other); the many-row form holds eight at most
        const long long nblocks = (long long)gps * (group / 16);
        int waves = (int)(nblocks / 4);
        const int wbest = wmax > 12 ? 12 : wmax;
        waves = waves < wmin ? wmin : (waves > wbest ? wbest : waves);
        if (const char *e = getenv("W4A16_STRIPE_WAVES")) {  // tuning aid for sweeps, not part of the contract
            const int w = atoi(e);
            if (w >= wmin && w <= wmax) waves = w;
        }
        while (waves > wmin && stripe_lds_bytes(M, group, gps, waves) > (size_t)stripe_lds_limit()) --waves;
        p->waves_k = waves;
        p->threads = waves * 64;
        p->split = S;
        p->groups_per_split = gps;
        p->workgroups = (int)(tiles * S);
        p->workspace_bytes = workspace_of(kernel, M, N, S);
        return W4A16_OK;
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
        if (const char *e = getenv("W4A16_TILE_ROWS")) {  // tuning aid for sweeps, not part of the contract
            const int r = atoi(e);
            if (r == 16 || r == 32 || r == 64) rows_x = r;
        }
        p->tile_m = rows_x;
        if (const char *e = getenv("W4A16_TILE_WAVES")) {  // tuning aid for sweeps, not part of the contract
            const int w = atoi(e);
            if (w >= 4 && w <= 8) { p->waves_k = w; p->threads = 64 * w; }
        }
        const long long wgs = tiles * ((M + rows_x - 1) / rows_x);
        if (S == 0) S = (int)(cus / wgs);  // never more workgroups than compute units: the extra ones would run as a second round
        if (S < 1) S = 1;
        if (S > G) S = G;
        int gps = (G + S - 1) / S;
        while (gps > 1 && (unsigned long long)gps * (group / 8) * N * 4ull >= 0x7F000000ull) gps = (gps + 1) / 2;
        S = (G + gps - 1) / gps;
        p->split = S;
        p->groups_per_split = gps;
        p->workgroups = (int)(wgs * S);
        p->workspace_bytes = workspace_of(kernel, M, N, S);
        return W4A16_OK;
    }
    {  // WAVE_SPLIT
        p->tile_n = (N + 63) / 64 >= cus ? 64 : 32;
        p->tile_m = 4;
        p->waves_k = 16;
        p->threads = 1024;
        tiles = (N + p->tile_n - 1) / p->tile_n;
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
    while ((unsigned long long)gps * (group / 8) * N * 4ull >= 0x7F000000ull && gps > 1) gps = (gps + 1) / 2;
    S = (G + gps - 1) / gps;  // no empty slice
    p->split = S;
    p->groups_per_split = gps;
    p->workgroups = (int)(tiles * S);
    p->workspace_bytes = workspace_of(kernel, M, N, S);
    return W4A16_OK;
}

int ensure_workspace(int dev, size_t bytes, void **out)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState &d = g_dev[dev];
    if (d.ws_bytes < bytes) {
        if (d.ws) {
            // hipFree waits for the device, so work still using the old buffer has drained
            hipError_t e = hipFree(d.ws);
            d.ws = nullptr;
            d.ws_bytes = 0;
            if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_WORKSPACE; }
        }
        size_t want = bytes + bytes / 4;
        void *ptr = nullptr;
        hipError_t e = hipMalloc(&ptr, want);
        if (e != hipSuccess) { note_hip_error(e); (void)hipGetLastError(); return W4A16_ERR_WORKSPACE; }
        d.ws = ptr;
        d.ws_bytes = want;
    }
    *out = d.ws;
    return W4A16_OK;
}

// The accumulator of the STRIPE and TILE families: grown on demand, cleared once when allocated (on `stream`,
// ahead of the launch that first uses it); every launch leaves it all zero again.
int ensure_accumulator(int dev, size_t bytes, hipStream_t stream, void **out)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState &d = g_dev[dev];
    if (d.acc_bytes < bytes) {
        if (d.acc) {
            hipError_t e = hipFree(d.acc);
            d.acc = nullptr;
            d.acc_bytes = 0;
            if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_WORKSPACE; }
        }
        size_t want = bytes < (1u << 20) ? (1u << 20) : bytes + bytes / 4;
        void *ptr = nullptr;
        hipError_t e = hipMalloc(&ptr, want);
        if (e != hipSuccess) { note_hip_error(e); (void)hipGetLastError(); return W4A16_ERR_WORKSPACE; }
        e = launch_accumulator_clear(static_cast<unsigned long long *>(ptr), want / 8, stream);
        if (e != hipSuccess) { note_hip_error(e); (void)hipFree(ptr); return W4A16_ERR_HIP; }
        d.acc = ptr;
        d.acc_bytes = want;
    }
    *out = d.acc;
    return W4A16_OK;
}

int run(const void *X, const uint32_t *Wp, const void *scales, const uint32_t *zeros, int group, int M, int N, int K,
        void *Y, void *stream, int kernel, int split, void *user_ws, size_t user_ws_bytes, bool user_ws_given)
{
    t_hip_error[0] = 0;
    if (!X || !Wp || !scales || !zeros || !Y) return W4A16_ERR_NULL;
    if (user_ws_given && !user_ws) return W4A16_ERR_NULL;
    int rc = check_shape(group, M, N, K);
    if (rc) return rc;
    if (!aligned16(X) || !aligned16(Wp) || !aligned16(scales) || !aligned16(zeros) || !aligned16(Y)) return W4A16_ERR_ALIGN;
    if (user_ws_given && (reinterpret_cast<uintptr_t>(user_ws) & 255u)) return W4A16_ERR_ALIGN;

    const int dev = current_device();
    if (dev < 0) { note_hip_error(hipErrorNoDevice); return W4A16_ERR_HIP; }
    w4a16_plan plan;
    rc = make_plan(M, N, K, group, kernel, split, compute_units(dev), &plan);
    if (rc) return rc;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int finish = finish_of(plan.kernel, M, N, plan.split);
    unsigned long long *sync = nullptr;  // the accumulator: zero before the launch, left zero by it
    float *partials = nullptr;
    if (user_ws_given && user_ws_bytes < plan.workspace_bytes) return W4A16_ERR_WORKSPACE;
    if (finish == kFinishAccumulator) {
        if (user_ws_given) {  // a caller's workspace comes uninitialised
            sync = static_cast<unsigned long long *>(user_ws);
            hipError_t e = launch_accumulator_clear(sync, (size_t)M * N, st);
            if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
        } else {
            void *ptr = nullptr;
            rc = ensure_accumulator(dev, plan.workspace_bytes, st, &ptr);
            if (rc) return rc;
            sync = static_cast<unsigned long long *>(ptr);
        }
    } else if (finish == kFinishSecondPass) {
        void *ptr = user_ws;
        if (!user_ws_given) {
            rc = ensure_workspace(dev, plan.workspace_bytes, &ptr);
            if (rc) return rc;
        }
        partials = static_cast<float *>(ptr);
    }

    GemmArgs a;
    a.X = static_cast<const uint16_t *>(X);
    a.Wp = Wp;
    a.scales = static_cast<const uint16_t *>(scales);
    a.Zp = zeros;
    a.Y = static_cast<uint16_t *>(Y);
    a.partials = partials;
    a.group = group; a.M = M; a.N = N; a.K = K;
    a.split = plan.split;
    a.groups_per_split = plan.groups_per_split;
    a.groups = K / group;

    hipError_t e = plan.kernel == W4A16_KERNEL_STRIPE       ? launch_stripe(a, finish, sync, plan.waves_k, st)
                   : plan.kernel == W4A16_KERNEL_TILE       ? launch_tile(a, finish, sync, plan.tile_m, plan.waves_k, st)
                                                            : launch_wave_split(a, plan.tile_n, st);
    if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
    if (finish == kFinishSecondPass) {
        e = launch_reduce(a.partials, plan.split, M, N, a.Y, st);
        if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
    }
    return W4A16_OK;
}

}  // namespace

extern "C" {

int w4a16_gemm(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
               int N, int K, void *Y, void *stream)
{
    return run(X, Wpacked, scales, zeros, group, M, N, K, Y, stream, W4A16_KERNEL_AUTO, 0, nullptr, 0, false);
}

int w4a16_gemm_ex(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
                  int N, int K, void *Y, void *stream, int kernel, int split)
{
    return run(X, Wpacked, scales, zeros, group, M, N, K, Y, stream, kernel, split, nullptr, 0, false);
}

int w4a16_gemm_ws(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int M,
                  int N, int K, void *Y, void *stream, int kernel, int split, void *workspace, size_t workspace_bytes)
{
    return run(X, Wpacked, scales, zeros, group, M, N, K, Y, stream, kernel, split, workspace, workspace_bytes, true);
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

int w4a16_reduce(const float *partials, int S, int M, int N, void *Y, void *stream)
{
    t_hip_error[0] = 0;
    if (!partials || !Y) return W4A16_ERR_NULL;
    if (S < 1 || M < 1 || N < 8 || N % 8 != 0) return W4A16_ERR_SHAPE;
    if (!aligned16(partials) || !aligned16(Y)) return W4A16_ERR_ALIGN;
    hipError_t e = launch_reduce(partials, S, M, N, static_cast<uint16_t *>(Y), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { note_hip_error(e); return W4A16_ERR_HIP; }
    return W4A16_OK;
}

int w4a16_dequant(const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int N, int K,
                  void *W16, void *stream)
{
    t_hip_error[0] = 0;
    if (!Wpacked || !scales || !zeros || !W16) return W4A16_ERR_NULL;
    int rc = check_shape(group, 1, N, K);
    if (rc) return rc;
    if (!aligned16(Wpacked) || !aligned16(scales) || !aligned16(zeros) || !aligned16(W16)) return W4A16_ERR_ALIGN;
    hipError_t e = launch_dequant(Wpacked, static_cast<const uint16_t *>(scales), zeros, group, N, K,
                                  static_cast<uint16_t *>(W16), static_cast<hipStream_t>(stream));
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
    case W4A16_ERR_WORKSPACE: return "workspace too small or allocation failed";
    case W4A16_ERR_HIP: return "HIP runtime error";
    case W4A16_ERR_UNSUPPORTED: return "forced kernel or split not valid for this shape";
    default: return "unknown status";
    }
}

const char *w4a16_last_hip_error(void) { return t_hip_error; }

void w4a16_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    for (int d = 0; d < kMaxDevices; ++d) {
        if (!g_dev[d].ws && !g_dev[d].acc) continue;
        int prev = -1;
        if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(d) == hipSuccess) {
            if (g_dev[d].ws) (void)hipFree(g_dev[d].ws);
            if (g_dev[d].acc) (void)hipFree(g_dev[d].acc);
            (void)hipSetDevice(prev);
        }
        g_dev[d].ws = nullptr;
        g_dev[d].ws_bytes = 0;
        g_dev[d].acc = nullptr;
        g_dev[d].acc_bytes = 0;
    }
}

}  // extern "C"
