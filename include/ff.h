/*
 * ff — fused linear + erf-GELU + LayerNorm for AMD MI355X (gfx950), C ABI.
 *
 *     Y = LayerNorm_N( GELU( X * W^T + b ) ) * gamma + beta
 *
 * The operation is the fused operator chain the paper's optimisation loop
 * targets: a GEMM whose epilogue (bias, activation, row statistic) stays in
 * registers instead of round-tripping through global memory (App. B.1, the
 * fused Linear -> row-mean -> GELU epilogue case; Sec. 4, shuffle-based row
 * reductions and removal of the second global read).  Its semantics are those
 * of the PyTorch reference operators the paper measures against (Sec. 2.1:
 * "functionally equivalent to its PyTorch reference"; Sec. 2.2, correctness
 * test on the same inputs within a small tolerance):
 *     z[m][n] = b[n] + sum_k X[m][k] * W[n][k]
 *     g       = 0.5 * z * (1 + erf(z / sqrt 2))
 *     y[m][n] = (g - mean_n g) / sqrt(var_n g + eps) * gamma[n] + beta[n]
 * with the biased variance (divide by N) and eps inside the square root.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, row-major,
 *     contiguous, 16-byte aligned.  X is [M,K], W is [N,K] (out-features by
 *     in-features), b / gamma / beta are [N], Y is [M,N].
 *   - All tensors share `dtype`: FF_F32 (fp32 in, fp32 accumulate, fp32 out) or
 *     FF_BF16 (bf16 in, fp32 accumulate and fp32 epilogue, bf16 out rounded to
 *     nearest even).  Nothing between the GEMM and the final store is rounded
 *     to bf16.
 *   - b, gamma, beta may each be NULL, meaning 0, 1, 0.
 *   - Shapes: M >= 1 arbitrary; bf16 needs K % 8 == 0 and N % 8 == 0, fp32 needs
 *     K % 4 == 0 and N % 4 == 0 (16-byte rows); anything else returns
 *     FF_ERR_UNSUPPORTED.  There is no fallback to any library GEMM or
 *     LayerNorm: the paper's audit of library fallbacks posing as custom
 *     kernels (Sec. 5, App. C) is the reason.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No host synchronisation is performed.  Y must not
 *     alias any input.  NaN / Inf propagate; nothing is checked on device.
 *   - Return value: FF_OK or an ff_status error code.  On error no kernel has
 *     been launched.
 *   - Scratch memory ("workspace") holds per-tile row statistics and arrival
 *     counters (and, for the two-pass variant only, an fp32 copy of G).  If no
 *     workspace is bound the library allocates one per device on first use and
 *     grows it when needed (growing synchronises the device).  Once a workspace
 *     that is large enough exists, a call allocates nothing, synchronises
 *     nothing and issues nothing but its kernels, so every call, the first
 *     included, can be recorded into a HIP graph; a call that would have to
 *     allocate or grow the library's own workspace while its stream is being
 *     captured returns FF_ERR_WORKSPACE instead (bind a workspace, or make one
 *     call of that shape, before capturing).  Calls that share a workspace must
 *     not overlap in time: use one stream, or bind distinct workspaces serially.
 */
#ifndef FF_H
#define FF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FF_F32 = 0, FF_BF16 = 1 } ff_dtype;

typedef enum {
    FF_OK = 0,
    FF_ERR_NULL = 1,        /* a required pointer is NULL */
    FF_ERR_SHAPE = 2,       /* M, K or N not positive, or M, N > 2^30, or K > 2^21 */
    FF_ERR_DTYPE = 3,       /* dtype is neither FF_F32 nor FF_BF16 */
    FF_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned */
    FF_ERR_UNSUPPORTED = 5, /* K or N not a multiple of the 16-byte vector; or a
                               forced variant cannot run this shape */
    FF_ERR_WORKSPACE = 6,   /* bound workspace too small / allocation failed */
    FF_ERR_LAUNCH = 7,      /* the HIP runtime refused the launch */
    FF_ERR_DEVICE = 8       /* a kernel reported a failed cross-tile wait */
} ff_status;

/* Kernel variants (for ff_debug_force_variant and ff_last_variant). */
typedef enum {
    FF_VARIANT_AUTO = 0,
    FF_VARIANT_TILED_FUSED = 1,   /* MFMA tiles; row statistics merged across
                                     tiles inside the launch, G stays in registers */
    FF_VARIANT_TILED_TWOPASS = 2, /* MFMA tiles write fp32 G + statistics; a second
                                     kernel normalises (used when a row spans more
                                     tiles than can be co-resident) */
    FF_VARIANT_SMALL_M = 3        /* M <= 32, bf16: streams W once at HBM rate */
} ff_variant;

/*
 * The fused operator.  Implements the chain above;
 * see the file header for argument meaning, layout, ownership and errors.
 *   X, W: required.  b, gamma, beta: optional (NULL).  Y: required, written.
 *   eps: added to the variance inside the square root.
 *   dtype: an ff_dtype.  stream: hipStream_t.
 */
int ff_fused_linear_gelu_ln(const void *X, const void *W, const void *b,
                            const void *gamma, const void *beta, float eps,
                            int64_t M, int64_t K, int64_t N, int dtype,
                            void *Y, void *stream);

/*
 * The same operator for callers that cannot allocate device memory: code under HIP graph capture
 * before any workspace exists, tight serving loops, harnesses that forbid hipMalloc.  Arguments,
 * layout, dtypes, errors and result (bit for bit) as ff_fused_linear_gelu_ln, but no workspace is
 * used, bound or allocated: the row statistics and arrival counters of the call live in a static
 * device array inside the library (ff_noalloc_max_bytes() bytes, 8 MiB, one copy on every device
 * that loads the library, held until the process ends).  The call makes no hipMalloc, hipFree,
 * memset or synchronising call; it launches one small kernel that clears the counters it is about
 * to use, then the operator's kernel, both on `stream`.  Shapes whose scratch need exceeds the array
 * return FF_ERR_WORKSPACE: that is every shape ff_workspace_bytes() reports above the limit, in
 * particular rows spanning more tiles than fit the device at once (the two-pass variant needs an fp32
 * copy of G).  All calls on one device share the one array: calls that overlap in time on a device
 * (two streams, two host threads) race on it and give wrong results; serialise them.
 * ff_check_device() covers these calls too.
 */
int ff_fused_linear_gelu_ln_noalloc(const void *X, const void *W, const void *b,
                                    const void *gamma, const void *beta, float eps,
                                    int64_t M, int64_t K, int64_t N, int dtype,
                                    void *Y, void *stream);

/* Size of the static scratch array behind ff_fused_linear_gelu_ln_noalloc, in bytes. */
size_t ff_noalloc_max_bytes(void);

/*
 * Row-wise cross-entropy with mean reduction, the row reduction of the paper's case
 * study (Sec. 4: row maximum, sum of exponentials, pick of the target's logit):
 *     loss[r] = log( sum_c exp(L[r][c]) ) - L[r][t[r]],   *mean_loss = (1/B) sum_r loss[r]
 *   logits   device, [B,C] row-major, dtype FF_F32 or FF_BF16, 16-byte aligned, read once.
 *            Any C >= 1 (rows whose byte length is a multiple of 16 use 16-byte loads).
 *   targets  device, [B] int64 class indices.  A target outside [0, C) makes that row's
 *            loss, and the mean, NaN; nothing is read out of bounds.
 *   row_loss device, [B] fp32, optional (NULL): the per-row losses.
 *   mean_loss device, one fp32, required.
 * Arithmetic is fp32 whatever the input dtype.  Asynchronous on `stream`; uses the
 * workspace (one number per workgroup and an arrival counter).  Results are bitwise
 * reproducible on a given device.  Returns an ff_status.
 */
int ff_cross_entropy_mean(const void *logits, const int64_t *targets, int64_t B, int64_t C,
                          int dtype, float *row_loss, float *mean_loss, void *stream);

/* Workspace bytes ff_cross_entropy_mean needs (0 for an invalid shape). */
size_t ff_cross_entropy_workspace_bytes(int64_t B, int64_t C, int dtype);

/*
 * Profiling-metric selection (the paper's Sec. 2.3, Steps 2 and 3; Alg. 2).
 *   values   device, double [n_tasks][n_kernels][n_metrics]: metric m of kernel v of task i.
 *   runtime  device, double [n_tasks][n_kernels].
 * Per task, r[i][m] = Pearson correlation over the task's kernels between metric m and the
 * runtime (NaN when undefined).  If 0 < collinear_tau <= 1, a metric whose |correlation| with an
 * earlier kept metric of the same task is >= collinear_tau is dropped for that task (needs
 * n_metrics <= 8192); any other value disables the filter.  Top-k per task by |r| (ties to the
 * lower index), candidates = union, score[m] = mean over all tasks of |r[i][m]| (NaN counts 0),
 * *threshold = the given percentile (0..100, linear interpolation) of the candidates' scores,
 * selected[m] = 1 for candidates in the Top-k of >= min_tasks tasks, with one sign of r over those
 * tasks and score > *threshold.  The paper uses top_k = 20, percentile = 75, min_tasks = 2.
 * Outputs are HOST pointers, each optional (NULL): r [n_tasks][n_metrics], score [n_metrics],
 * top int32 [n_tasks][top_k] (-1 padded), selected uint8 [n_metrics], threshold [1].
 * The correlations run on the device on `stream`; the call returns after the stream has been
 * synchronised and the host outputs are complete.  Uses the workspace.  Returns an ff_status.
 */
int ff_metric_selection(const double *values, const double *runtime, int64_t n_tasks,
                        int64_t n_kernels, int64_t n_metrics, int top_k, double percentile,
                        double collinear_tau, int min_tasks, double *r, double *score,
                        int32_t *top, uint8_t *selected, double *threshold, void *stream);

/*
 * The host part of the above on its own (no device is touched): r [n_tasks][n_metrics] and the
 * optional keep mask uint8 [n_tasks][n_metrics] (NULL = all kept) are host arrays; outputs as above.
 */
int ff_metric_select_host(const double *r, const uint8_t *keep, int64_t n_tasks, int64_t n_metrics,
                          int top_k, double percentile, int min_tasks, int32_t *top, double *score,
                          uint8_t *selected, double *threshold);

/*
 * Second fused chain, the paper's fused-epilogue case study (App. B.1: Linear ->
 * subtract -> row-mean -> GELU -> residual add):
 *     Out[m][k] = X[m][k] + GELU( mean_n( X[m] . W[n] + b[n] - s[n] ) )
 * X [M,K], W [N,K], b and s [N] (each may be NULL = 0), Out [M,K]; same dtype, layout,
 * alignment, stream and error conventions as above; additionally K <= 32768.  Out may
 * alias X (every row is read completely before it is written).  The row mean of a
 * linear layer is one dot product with the column means of W, so this entry point
 * reads W and X once and writes Out once; no GEMM is run.  Uses the workspace.
 */
int ff_fused_linear_sub_rowmean_gelu_residual(const void *X, const void *W, const void *b,
                                              const void *s, int64_t M, int64_t K, int64_t N,
                                              int dtype, void *Out, void *stream);

/* Bytes of workspace the second chain needs for this shape (0 on invalid arguments). */
size_t ff_rowmean_workspace_bytes(int64_t M, int64_t K, int64_t N, int dtype);

/*
 * Bytes of workspace a call with this shape needs under the current variant
 * selection (0 on invalid arguments).  Pure host arithmetic.
 */
size_t ff_workspace_bytes(int64_t M, int64_t K, int64_t N, int dtype);

/*
 * The launch plan a call with this shape would take under the current variant selection, without
 * launching anything: out[0] the ff_variant, out[1] rows and out[2] columns of the output tile a
 * workgroup owns (small-M: all M rows x one 32-column strip at a time), out[3] wavefronts per
 * workgroup, out[4] workgroups in the launch, out[5] tiles per workgroup (rounds), out[6] workgroups
 * per compute unit, out[7] 1 if the tile order is the XCD-aware one.  `out` is host memory of eight
 * ints.  Returns the status the call itself would return for a shape that cannot run.  With no GPU
 * visible it plans for 256 compute units.
 */
int ff_plan_query(int64_t M, int64_t K, int64_t N, int dtype, int out[8]);

/*
 * Bind caller-owned device memory (256-byte aligned) as the workspace of the
 * current device, or unbind with (NULL, 0), after which the library allocates
 * its own again.  The call clears the control region (the first MiB) of the
 * memory itself, synchronously, and synchronises the device; it must not be
 * made while a stream is being captured, and no work that uses the previous
 * workspace may be in flight.  The memory must stay valid until unbound and all
 * work using it has completed.
 */
int ff_set_workspace(void *dev_ptr, size_t bytes);

/*
 * Synchronise `stream`, then report whether any kernel since the last check
 * gave up waiting for the other tiles of its rows (FF_ERR_DEVICE) — which can
 * only happen if the launch's workgroups were not co-resident — and clear that
 * state.  FF_OK otherwise.
 */
int ff_check_device(void *stream);

/* Human-readable name of an ff_status value (static storage). */
const char *ff_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int ff_version(void);

/* The variant the most recent successful ff_fused_linear_gelu_ln call on this
 * host thread's device used (an ff_variant), or 0 if none yet. */
int ff_last_variant(void);

/* ---- test hooks: exported for the parity tests, not part of the product API ---- */

/*
 * Linear stage only (GEMM + bias) through the tiled MFMA core, fp32 result:
 * Z_f32[m][n] = b[n] + sum_k X[m][k] W[n][k].  Z_f32 is a device pointer to
 * M*N floats.  With integer-valued inputs of small magnitude the result is
 * exact, which pins the GEMM core independently of any tolerance.
 */
int ff_debug_linear(const void *X, const void *W, const void *b,
                    int64_t M, int64_t K, int64_t N, int dtype,
                    float *Z_f32, void *stream);

/* Force a variant for later calls (FF_VARIANT_AUTO restores selection by shape).
 * A forced variant that cannot run a shape makes the call return
 * FF_ERR_UNSUPPORTED; it never silently runs something else. */
int ff_debug_force_variant(int variant);

/* Plain device-to-device copy of `bytes` (a multiple of 16; both pointers 16-byte aligned, device,
 * not overlapping) on `stream`.  A kernel of exactly known HBM traffic, used to scale hardware byte
 * counters when the traffic of the other kernels is measured. */
int ff_debug_copy(const void *src, void *dst, size_t bytes, void *stream);

/* Measured ceilings, on the default (null) stream: a register-resident loop of independent bf16
 * 32x32x16 MFMAs, `iters` rounds of 8 per wavefront, four wavefronts per compute unit, with no memory
 * traffic (*flops, a host pointer, receives the flops the launch performs); and a streaming read of
 * `bytes` (a multiple of 16) from `src` (device, 16-byte aligned) with 16-byte loads, eight in flight
 * per thread.  Timed by the caller, they give what the chip sustains next to the published peaks. */
int ff_debug_mfma_loop(int64_t iters, double *flops);
int ff_debug_stream_read(const void *src, size_t bytes);

/* Tile shape of the tiled variants for later calls: tile = 0 (automatic), 64, 128 or 256 (columns);
 * wg_per_cu = 0 (automatic), 1 (a persistent grid of one workgroup per compute unit) or 2 (two).
 * (256, 0 or 1) is the 256 x 256 tile, one workgroup per compute unit; (256, 2) the 256-column x
 * 128-row tile, up to two per compute unit (the automatic plan takes it only where there are no more
 * such tiles than units).  The combinations the automatic plan does not pick exist as distinct
 * kernels of the same operator for the profiling-metric study and for tests.  FF_ERR_UNSUPPORTED
 * for any other combination. */
int ff_debug_force_tile(int tile, int wg_per_cu);

/* Wavefronts per workgroup of the 256 x 256 tile for later calls: 0 (automatic), 4 (2 x 2
 * wavefronts of 4 x 4 MFMA blocks) or 8 (2 x 4 wavefronts of 4 x 2 blocks).  While 4 or 8 is forced,
 * a call whose plan uses 256-column tiles runs the 256 x 256 tile with that many wavefronts, and a
 * call whose plan uses a narrower tile returns FF_ERR_UNSUPPORTED. */
int ff_debug_force_waves(int waves);

/* Start delay, in microseconds (0..1000, default 12), of the second workgroup of every compute unit
 * in launches of the 256-column x 128-row tile over a full grid: with it, the epilogue of one
 * workgroup falls into the K loop of the other from the first tile on. */
int ff_debug_set_stagger_us(int microseconds);

/* Phase timestamps of the tiled kernels.  Binds `bytes` of device memory (8-byte aligned; NULL
 * unbinds) for the current device.  While bound, thread 0 of every workgroup of a tiled launch
 * writes, for each of its tiles that fits, 16 uint64 words at
 * [(round * grid + workgroup) * 16]: words 0..6 the 100 MHz wall clock at tile start, first K slab
 * in LDS, end of the K loop, row statistics published, other tiles of the rows arrived, statistics
 * merged, stores issued; words 8, 9 the shader clock at the start and end of the K loop.  The
 * timings a launch reports this way differ from an untimed launch by the stores themselves. */
int ff_debug_set_timeline(void *dev_ptr, size_t bytes);

/* Upper bound, in microseconds, a workgroup waits for the other tiles of its
 * rows before it gives up and flags FF_ERR_DEVICE (default 2,000,000). */
int ff_debug_set_wait_limit_us(int64_t microseconds);

/* Make later launches wait for `count` arrivals more than will ever come (0 restores
 * normal operation).  With a short wait limit this forces every cross-tile wait to
 * expire: the kernels still run to completion, flag FF_ERR_DEVICE, and write
 * unspecified output.  Exists so that the failure path can be tested from the host. */
int ff_debug_expect_extra_arrivals(int count);

#ifdef __cplusplus
}
#endif
#endif /* FF_H */
