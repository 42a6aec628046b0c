/*
 * w4a16.h -- C ABI of the MI355X (gfx950) W4A16 mixed-precision GEMM library.
 *
 * The operation (Section 3, Eq. 2 of the paper):
 *
 *     C = A * Dequant(W),     Dequant(W) = s (W - z)
 *
 * with A = X in FP16 [M,K], W in INT4 [K,N], partial sums in FP32 and one
 * final cast to FP16 (Section 3; Algorithm 1 lists the inputs X, W, s, z, the
 * split factor S and the FP16 output).  Split-K (Algorithm 1, Phases 2 and 3)
 * is how the library fills the GPU when N is small next to K: K is cut into S
 * slices on group boundaries; slices held by the waves of one workgroup meet in
 * LDS; slices held by different workgroups either add their sums into a 64-bit
 * fixed-point accumulator whose last arriver casts to FP16 (while the adds are few), or put FP32
 * partial results in a workspace that a second pass adds in a fixed order and
 * casts to FP16.
 * Unlike Algorithm 1 (Phase 1) the dequantized weights never travel through
 * device memory: they are unpacked in registers right after the load.
 *
 * Storage (Section 2.2 says only that 4-bit values are packed into wider
 * integers such as INT32; the layout below is this library's contract):
 *
 *   X       FP16   [M, K]        row-major.
 *   Wpacked uint32 [K/8, N]      row-major (n contiguous).  The unsigned code
 *                                 (0..15) of k = 8r+i is bits 4i..4i+3 of
 *                                 Wpacked[r, n].
 *   scales  FP16   [K/group, N]  row-major; s of (k, n) is scales[k/group, n].
 *   zeros   uint32 [K/group, N/8] row-major.  The unsigned zero point (0..15,
 *                                 stored as itself) of n = 8c+j is bits
 *                                 4j..4j+3 of zeros[g, c].
 *                                 `zeros` may be NULL: symmetric quantization
 *                                 (Section 2.1: z = 0 on signed codes), read as
 *                                 signed code = stored code - 8, i.e. every
 *                                 zero point is 8 and no tensor is read.
 *   Y       FP16   [M, N]        row-major, every element overwritten.
 *
 * All data pointers are DEVICE pointers owned by the caller, 16-byte aligned;
 * the library neither keeps nor frees them.  `stream` is a hipStream_t passed
 * as void* (NULL = the default stream).  Calls only enqueue work on `stream`;
 * the one exception is the call that makes the library allocate a split buffer
 * (see w4a16_gemm), which waits for the device once.
 *
 * Errors: every function returns a w4a16_status (0 = success).  On any error
 * nothing is launched and Y is untouched.  Nothing aborts, throws or prints.
 *
 * Shapes: M >= 1, N >= 8 with N % 8 == 0, K % group == 0, group a multiple of
 * 32 (the paper fixes no granularity for s and z; 128 is the tuned case).
 *
 * Threads and streams: the library-owned split buffers are one set per device,
 * used by every call on that device, so two calls that overlap in time on one
 * device (on different streams) race on them unless each passes its own
 * workspace through w4a16_gemm_ws.  Results are bitwise reproducible for a fixed
 * shape and plan.
 */
#ifndef W4A16_H
#define W4A16_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    W4A16_OK = 0,
    W4A16_ERR_NULL = 1,        /* a required pointer is NULL                          */
    W4A16_ERR_SHAPE = 2,       /* M, N or K out of range, or N % 8 / K % 8 != 0        */
    W4A16_ERR_GROUP = 3,       /* group not a multiple of 32, or K % group != 0        */
    W4A16_ERR_ALIGN = 4,       /* a data pointer is not 16-byte aligned                */
    W4A16_ERR_WORKSPACE = 5,   /* workspace too small, allocation failed, or allocation needed during stream capture */
    W4A16_ERR_HIP = 6,         /* the HIP runtime reported an error on launch          */
    W4A16_ERR_UNSUPPORTED = 7  /* forced kernel / split not valid for this shape, or M*K*2 >= 2^31 bytes (32-bit offsets) */
} w4a16_status;

/* Kernel families the scheduler chooses from (Algorithm 1, Phase 2 is the
 * one multiply phase of the paper; these are its gfx950 forms). */
typedef enum {
    W4A16_KERNEL_AUTO = -1,
    W4A16_KERNEL_WAVE_SPLIT = 0, /* M <= 4: narrow column tile per workgroup, its 16 waves split K, LDS reduction */
    /* 1 and 2 belonged to two earlier families, retired: W4A16_ERR_UNSUPPORTED */
    W4A16_KERNEL_STRIPE = 3,     /* M <= 16; the scheduler's choice for M = 1 (2; 3, 4) from about 4 MB (20 MB; 32 MB)
                                    of packed weights on: 256-column stripe x K slice per workgroup, its waves
                                    share the slice (exact sums in LDS); slices of different workgroups meet in a
                                    64-bit fixed-point accumulator by one atomic add each, no second launch        */
    W4A16_KERNEL_TILE = 4        /* any M, the scheduler's choice otherwise: 64-column tile x 16, 32 or 64 rows of X
                                    per workgroup, its waves (eight; four at 32 and 64 rows, group 128) own contiguous runs of K (LDS
                                    reduction), plain MFMA operand layout; slices of different workgroups meet as
                                    in STRIPE                                                                         */
} w4a16_kernel;

/* What the scheduler decided for a shape (Algorithm 1 takes S and the block
 * sizes as inputs without a rule; here the library derives them). */
typedef struct {
    int kernel;            /* a w4a16_kernel value                                            */
    int split;             /* S: K slices across workgroups (1 = no workspace, Y written directly) */
    int groups_per_split;  /* quantisation groups per slice (last slice may be shorter)       */
    int tile_n;            /* output columns per workgroup                                    */
    int tile_m;            /* output rows per workgroup                                       */
    int waves_k;           /* K slices inside a workgroup (waves whose results meet in LDS)   */
    int workgroups;        /* workgroups of the multiply launch                               */
    int threads;           /* threads per workgroup                                           */
    size_t workspace_bytes;/* 64-bit sums [M, N] or FP32 partials [S, M, N]; 0 when S == 1       */
} w4a16_plan;

/*
 * Y = X * s (W - z)   (Eq. 2), plan chosen by the library's Split-K scheduler.
 * The split buffers of Algorithm 1 (Phase 2 writes them, Phase 3 adds them)
 * are, in this order of preference: the workspace registered for the current
 * device with w4a16_set_workspace; else library-owned buffers of that device,
 * allocated with hipMalloc when a call first needs them (that call, and only
 * that one, waits for the device while it clears the new buffer), grown when a
 * later call needs more, kept until w4a16_shutdown and never freed before (work
 * already enqueued, or recorded in a HIP graph, keeps pointing at valid
 * memory).  While `stream` is being captured into a graph nothing can be
 * allocated: a call that would have to returns W4A16_ERR_WORKSPACE; run the
 * same shape once outside the capture first, or use w4a16_set_workspace,
 * w4a16_gemm_ws or w4a16_gemm_noalloc.  If a launch fails
 * (W4A16_ERR_HIP) the library clears its accumulator again before the next use.
 */
int w4a16_gemm(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros,
               int group, int M, int N, int K, void *Y, void *stream);

/*
 * The same with Algorithm 1's inputs chosen by the caller: `kernel` is a
 * w4a16_kernel (its block sizes; AUTO = choose), `split` the split factor S
 * (0 = choose; otherwise 1 <= S <= K/group; the library lowers it so that no
 * slice is empty, and raises it where a slice would not fit a workgroup's LDS
 * or a 31-bit buffer: w4a16_query_plan tells).  For sweeps and tests.
 */
int w4a16_gemm_ex(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros,
                  int group, int M, int N, int K, void *Y, void *stream, int kernel, int split);

/*
 * The same, with the split buffers of Algorithm 1 (Section 3: the per-slice
 * results C_i in global memory) brought by the caller for this one call:
 * `workspace` is device memory of at least the plan's workspace_bytes
 * (w4a16_query_plan; for the scheduler's own choice also
 * w4a16_workspace_bytes), 256-byte aligned.  Its contents need no
 * initialisation (a plan that uses it as accumulator clears it with one small
 * extra launch first).  Performs no allocation and keeps no state: calls with
 * different workspaces may overlap on one device.
 */
int w4a16_gemm_ws(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros,
                  int group, int M, int N, int K, void *Y, void *stream, int kernel, int split,
                  void *workspace, size_t workspace_bytes);

/*
 * The same operation with BF16 activations: X [M, K] and Y [M, N] are bfloat16 (the upper half of a binary32),
 * everything that belongs to the quantized weights is unchanged (packed codes, FP16 scales, packed zero points
 * or NULL).  Algorithm 1 lists A and C as 16-bit floating point; the paper's runs use FP16, this entry covers
 * the other 16-bit format (bf16 MFMA, FP32 sums, one round-to-nearest-even cast at the end).  Arguments, split
 * buffers, stream rules and errors as w4a16_gemm_ex; kernel = W4A16_KERNEL_AUTO and split = 0 give the
 * scheduler's plan (the same plan as for FP16).  Forced plans: W4A16_KERNEL_TILE for any M,
 * W4A16_KERNEL_STRIPE for M <= 4; the others return W4A16_ERR_UNSUPPORTED.  Results beyond +-2^25 saturate
 * there when K slices meet in the fixed-point accumulator or when the waves of a workgroup share a slice by
 * ticket (M <= 16), as for FP16, where that bound lies beyond the format's range.
 */
int w4a16_gemm_bf16(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros,
                    int group, int M, int N, int K, void *Y, void *stream, int kernel, int split);

/*
 * Registers caller-owned split buffers (Algorithm 1's C_i; Section 3) for the
 * current device: device memory, 256-byte aligned, at least 256 bytes, owned by
 * the caller and kept valid until it is replaced or removed (NULL removes it).
 * w4a16_gemm and w4a16_gemm_ex then use it instead of library-owned buffers and
 * never allocate; a plan that needs more than `workspace_bytes` returns
 * W4A16_ERR_WORKSPACE.  As with w4a16_gemm_ws the contents need no
 * initialisation.  Calls that overlap in time on one device share it and race.
 */
int w4a16_set_workspace(void *workspace, size_t workspace_bytes);

/*
 * w4a16_gemm_ex for callers that cannot allocate device memory or wait for the device: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as w4a16_gemm_ex
 * (kernel = W4A16_KERNEL_AUTO and split = 0 give w4a16_gemm's plan).  The split buffers are a fixed array of
 * W4A16_NOALLOC_SCRATCH_BYTES that the library's code object holds on every GPU it is loaded on until the
 * process ends; the call allocates nothing, frees nothing and waits for nothing.  A plan that needs more returns
 * W4A16_ERR_WORKSPACE and launches nothing (w4a16_query_plan tells what a plan needs; the scheduler's own plans
 * stay below 1.1 MiB on a GPU of 256 compute units).  A plan that uses the array as accumulator clears that part with one small extra launch first (a
 * kernel, so the call can be captured).  All such calls on one GPU share the one array: calls that overlap in
 * time on that GPU (different streams, or graphs replayed concurrently) race on it.
 */
#define W4A16_NOALLOC_SCRATCH_BYTES (4u << 20)
int w4a16_gemm_noalloc(const void *X, const uint32_t *Wpacked, const void *scales, const uint32_t *zeros,
                       int group, int M, int N, int K, void *Y, void *stream, int kernel, int split);

/* Bytes of split buffers (Section 3) that the plan the scheduler itself chooses for this shape needs (at least
 * 256); forced plans: w4a16_query_plan. */
size_t w4a16_workspace_bytes(int M, int N, int K, int group);

/* The plan w4a16_gemm_ex would run for these arguments (no launch, no GPU call
 * beyond reading the current device's properties once). */
int w4a16_query_plan(int M, int N, int K, int group, int kernel, int split, w4a16_plan *out);

/* Second pass alone (Algorithm 1, Phase 3): Y[m,n] = fp16(sum_{i<S} partials[i,m,n]),
 * i ascending, FP32 adds, round-to-nearest-even cast.  partials: FP32 [S, M, N]. */
int w4a16_reduce(const float *partials, int S, int M, int N, void *Y, void *stream);

/* Phase 1 alone (Algorithm 1; Eq. 2): W16[k,n] = fp16(scales[k/group, n] * (q[k,n] - z[k/group, n])), one
 * round-to-nearest-even cast of the exact FP32 product.  W16: device pointer, FP16 [K, N] row-major, 16-byte
 * aligned, owned by the caller, fully overwritten.  w4a16_gemm never materialises this matrix; the entry point
 * serves the unfused variant that Section 4.2 diagnoses (FP16 weights through global memory, then an FP16 GEMM),
 * which the benchmark times beside the fused path.  Same shape rules and error codes as w4a16_gemm. */
int w4a16_dequant(const uint32_t *Wpacked, const void *scales, const uint32_t *zeros, int group, int N, int K,
                  void *W16, void *stream);

/* Measurement aid, not a step of the method (for benchmarks that want the practical ceiling of the memory system
 * beside a multiply's time): reads up to three device arrays once (16-byte-aligned pointers; a null pointer skips
 * that array; trailing bytes beyond a multiple of 16 are not read), one workgroup per compute unit, and keeps
 * nothing.  `sink`: one 32-bit word of device memory that anchors the loads (written only in the practically
 * impossible case that everything read cancels to one bit pattern).  Enqueues one kernel on `stream`. */
int w4a16_stream_probe(const void *a, size_t a_bytes, const void *b, size_t b_bytes, const void *c, size_t c_bytes, void *sink,
                       void *stream);

/* Offline tool (Section 2.1, Eq. 1: x_q = round(x / s) + z): quantizes FP16 weights W16 [K, N] (row-major, device
 * pointer) into the three tensors w4a16_gemm reads, all owned by the caller and fully overwritten: Wpacked [K/8, N],
 * scales FP16 [K/group, N], zeros [K/group, N/8].  The paper leaves the choice of s and z open; per group of one
 * column, in FP32: lo = min(min w, 0), hi = max(max w, 0), s = fp16((hi - lo) / 15) (1 if that is 0),
 * z = clamp(rint(-lo / s), 0, 15), q = clamp(rint(w / s) + z, 0, 15), rounding to nearest even.  Inputs must be
 * finite.  Same shape rules and error codes as w4a16_gemm. */
int w4a16_quantize(const void *W16, int group, int N, int K, uint32_t *Wpacked, void *scales, uint32_t *zeros,
                   void *stream);

/*
 * Tuning knobs, for sweeps and tests only: process-wide state that changes the plans of every later call
 * (w4a16_query_plan reports them as changed).  Each knob starts from the environment variable W4A16_<KNOB IN
 * CAPITALS>, read once when the library first plans a call; 0 restores the scheduler's own choice.
 *   "stripe_finish"  1: K slices of different workgroups always meet in the accumulator, 2: always second pass
 *   "stripe_waves"   waves per STRIPE workgroup
 *   "stripe_dyn"     M <= 4: 2 = equal contiguous runs per wave instead of units handed out by ticket
 *   "stripe_unit"    packed rows per unit handed out (2, 4 or 8)
 *   "stripe_depth"   units in flight per wave (1, 2; 9 = one, its successor requested ahead of its use)
 *   "stripe_dot2"    1: dot products by v_dot2_f32_f16 on the vector ALU instead of the MFMA (measurement only)
 *   "tile_rows"      rows of X per TILE workgroup (16, 32, 64)
 *   "tile_dyn"       16 rows of X per workgroup: 1 = units of K always handed out by ticket, 2 = never
 *   "tile_depth"     units in flight per wave of that form (1, 2)
 *   "tile_unit"      blocks of 32 k per unit of that form (1, 2; default: a whole group, at most 4)
 *   "tile_waves"     waves per TILE workgroup (4..8)
 *   "tile_wide"      2: TILE at 32 or 64 rows of X per workgroup, FP16, group 128: the eight-wave form instead of
 *                    the four-wave one
 *   "log"            1: every w4a16_gemm* call prints its plan on stderr (the one case in which the library prints)
 * Returns W4A16_ERR_UNSUPPORTED for an unknown knob.
 */
int w4a16_tune(const char *knob, int value);

/* Text for a status code (static storage). */
const char *w4a16_status_string(int status);

/* Text of the last HIP error seen by this thread's failing call ("" if none). */
const char *w4a16_last_hip_error(void);

/* Frees the library-owned split buffers of all devices.  Call only when no
 * w4a16 work is in flight and no HIP graph that recorded w4a16 calls will be replayed. */
void w4a16_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* W4A16_H */
