/*
 * fastsinkhorn.h -- C ABI of the MI355X (gfx950) log-domain Sinkhorn library.
 *
 * The library solves the entropic optimal-transport problem of the paper's
 * Eq. 3 by the log-domain Sinkhorn iteration (Eqs. 9-10, Alg. 1):
 *
 *     f_i <- -eps * LSE_j( (g_j - C_ij)/eps + log b_j )          (Eq. 9)
 *     g_j <- -eps * LSE_i( (f_i - C_ij)/eps + log a_i )          (Eq. 10, uses the new f)
 *
 * starting from f = g = 0 (Eqs. 6-7), with the row-marginal error
 * err = sum_i |r_i - a_i| (Alg. 1, Sec. 4.5) as the stopping test.
 * Notation: the paper's alpha, beta, mu, nu, pi are f, g, a, b, P here.
 *
 * Conventions shared by every entry point
 *   - Every array pointer is a DEVICE pointer (HBM of the current HIP device),
 *     owned by the caller.  The library neither frees nor keeps them after the
 *     work it enqueued on `stream` has run.  Outputs must not alias inputs.
 *   - C is row-major n x m, C[i*m + j], fp32 (Sec. 4.4; the solvers with options also
 *     take fp16 / bfloat16 storage, fs_options.cost_dtype).  X is n x d and Y is
 *     m x d, row-major fp32; the cost is then the squared Euclidean distance
 *     ||x_i - y_j||^2 and is recomputed on the fly, never written to memory.
 *   - a[n], b[m] are fp32 weights (non-negative; a zero weight carries no mass).
 *     They are meant to sum to 1 each: the marginal error is accumulated in fixed
 *     point and reported as NaN once it reaches 16.
 *     f[n], g[m] are fp32 potentials.  eps is the regularisation (> 0).
 *   - tol <= 0 means: run exactly max_iter iterations.  tol > 0 means: stop at
 *     the first iteration k with k mod check_every == 0 and err_k < tol, or at
 *     max_iter (Alg. 1).  The returned potentials are those after exactly
 *     `iters` iterations.
 *   - Scalars are validated on the host before anything is enqueued
 *     (1 <= n, m <= FS_MAX_POINTS; eps > 0 and finite; max_iter >= 0;
 *     1 <= d <= FS_MAX_DIM; non-null pointers); a violation returns FS_ERR_INVALID_ARG.  Array
 *     contents are the caller's responsibility; non-finite potentials are
 *     reported through fs_result.nonfinite, never by aborting.
 *   - No exception crosses this boundary.  fs_last_error() returns a
 *     thread-local description of the last failure.
 *   - Concurrency: every entry point that says it uses the library-owned workspace shares ONE
 *     cached workspace (and one pinned host block) per device; such calls on one device must not
 *     overlap, neither from two host threads nor by asynchronous work of two of them still running
 *     on different streams.  The *_ex entry points with a caller workspace and
 *     fs_sinkhorn_dense_batched have no such shared state and may overlap freely.
 *   - Internally the potentials are carried in fp64 (scaled by log2(e)/eps) and
 *     the exponent arguments are formed in fp64; exp2/log2 and the sums are fp32.
 */
#ifndef FASTSINKHORN_H
#define FASTSINKHORN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Opaque stream handle: a hipStream_t passed as void* (NULL = the default stream). */
typedef void *fs_stream;

#define FS_MAX_DIM 64
#define FS_MAX_POINTS 1048512   /* 16383 * 64 */
#define FS_COST_F32 0
#define FS_COST_F16 1
#define FS_COST_BF16 2
#define FS_SMALL_MAX 256        /* largest n, m of the single-workgroup / batched kernel */
#define FS_COOP_MAX 1024        /* largest n, m of the one-launch multi-workgroup kernel */

typedef enum {
    FS_OK = 0,
    FS_ERR_INVALID_ARG = -1,
    FS_ERR_WORKSPACE = -2,     /* caller workspace missing, misaligned or too small */
    FS_ERR_HIP = -3,           /* a HIP runtime call failed; see fs_last_error()     */
    FS_ERR_UNSUPPORTED = -4
} fs_status;

/* Written by the device at the end of a solve (also mirrored to the host by the
 * blocking entry points). */
typedef struct {
    int32_t iters;         /* iterations performed (f- and g-update pairs)               */
    int32_t converged;     /* 1 iff the tolerance test of Alg. 1 fired                   */
    int32_t nonfinite;     /* 1 iff some returned potential is NaN or +-inf; 2: a solver whose
                              workgroups wait for one another (kernel_mode 4, 5, 6, or the
                              asynchronous entry points' own choice of 4 for small problems)
                              gave up waiting, see kernel_mode: the potentials are not valid */
    float   marginal_err;  /* err after `iters` iterations; NaN if it was not evaluated  */
} fs_result;

/* Options of the _ex entry points.  Zero-initialise for the defaults. */
typedef struct {
    int32_t check_every;     /* c of Alg. 1; 0 -> 10 (Sec. 4.5)                                     */
    int32_t warm_start;      /* 0: start from f = g = 0 (Eqs. 6-7); 1: start from the f, g passed in */
    int32_t kernel_mode;     /* 0: automatic; 1: streaming row / column kernels; 2: fused row-panel
                                kernel (dense, m <= 16384, and m % 4 == 0 when m <= 1024; else
                                FS_ERR_UNSUPPORTED);
                                3: the whole solve in one single-workgroup kernel (dense, n, m <=
                                FS_SMALL_MAX, else FS_ERR_UNSUPPORTED; what 0 picks up to about 128 x 128);
                                4: the whole solve in one launch over up to 32 workgroups that hold C in
                                registers and exchange column partials once per iteration (n, m <= FS_COOP_MAX
                                and a dense fp32 cost, or point clouds up to about n * m = 2^19 - exactly:
                                roundup(n / 128, power of 2) * roundup(m / 256, power of 2) <= 16 - whose squared
                                distances are then formed once in fp64; else FS_ERR_UNSUPPORTED; what 0 picks
                                from there up to 2^18 entries or pairs - in the blocking dense solves only up
                                to 512 x 512, see 5);
                                5: the whole solve in one launch over up to one workgroup per compute unit,
                                two grid-wide exchanges per iteration (n <= 4096, m <= 2048; dense fp32 with at
                                most 16 entries of C per lane, or point clouds with at most 8 pairs per lane;
                                else FS_ERR_UNSUPPORTED; what 0 picks in the blocking solves for every such
                                problem with n or m above 512);
                                6: blocks of iterations in launches of the persistent form of the fused
                                row-panel kernel, one resident workgroup per compute unit, two grid-wide waits
                                per iteration (dense fp32, 128 < m <= 16384 and at least m / 64 row panels and
                                compute units, up to 1024 columns also at most 512 rows per compute unit; else
                                FS_ERR_UNSUPPORTED; what 0 picks in the blocking solves up to
                                8192 columns; the asynchronous solves take it on request only, because it
                                needs every compute unit of the device at the same moment).
                                The workgroups of 4, 5 and 6 wait for one another with a bounded number of
                                polls: should the device keep some of them from running for seconds (other
                                work on its compute units), the solve gives up and reports nonfinite = 2, never
                                a silent wrong result.  When the kernel was the library's own choice (0) a
                                blocking solve then simply runs the multi-kernel driver instead; an
                                asynchronous solve (which picks 4 by itself up to 2^18 entries) has nobody to
                                do that: its caller checks fs_result.nonfinite and, on 2, solves again with
                                kernel_mode = 1                                                             */
    int32_t use_graph;       /* 0: automatic; 1: plain stream launches; 2: hipGraph iteration blocks  */
    int32_t skip_final_err;  /* 1: do not spend the one trailing pass that evaluates err after the
                                last iteration when no stop fired (marginal_err is then NaN)          */
    int32_t fused_variant;   /* tuning knob: 0 default; 1..5 alternative tilings of the dense fused kernel
                                (kernel_mode 4: 1..3 = at most 16, 8, 4 workgroups);
                                +100: take the optimistic (fp32-sum) kernels from the first iteration on,
                                whatever the pace of the potentials (exercises the exact repair paths) */
    double *f64_out;         /* optional device [n]: f in double precision (NULL: not wanted)         */
    double *g64_out;         /* optional device [m]: g in double precision                            */
    const double *f64_in;    /* optional device [n], [m]: warm start in double precision; when both  */
    const double *g64_in;    /*   are given (and warm_start = 1) they take the place of f, g          */
    float  *err_history;     /* optional device [err_history_len]: err_k stored at index k-1          */
    int32_t err_history_len;
    int32_t cost_dtype;      /* storage of the dense cost matrix behind the `const float *C` argument:
                                FS_COST_F32 (0, default), FS_COST_F16 (IEEE half precision) or FS_COST_BF16,
                                n x m row-major entries of 2 bytes; the iteration then moves half the bytes.
                                Every entry is widened exactly to fp32 and the arithmetic is unchanged, so the
                                result is that of the solve on the rounded matrix.  Needs m % 8 == 0 and a
                                16-byte aligned C (else FS_ERR_UNSUPPORTED); honoured by every solver that
                                takes options (for fs_sinkhorn_dense_batched: every problem's C); kernel_mode 2
                                then needs 2048 < m <= 16384.  The after-the-loop entry points take fp32 only */
    int32_t wait_limit;      /* kernel_mode 4, 5 and 6: polls after which a workgroup stops waiting for the others
                                (0: default, about two million = seconds).  A tiny value makes the solve give
                                up early and report nonfinite = 2, which is how the bounded wait is tested   */
    int32_t time_kernel_every; /* blocking solves only: > 0 times the dominant kernel (row pass, fused pass
                                  or point-cloud LSE pass of the f-update) of every N-th iteration with a pair
                                  of HIP events that the runtime stamps with the start and the stop of that
                                  dispatch on `stream` (hipExtLaunchKernel); read back with
                                  fs_last_kernel_timing().  The persistent fused pass (kernel_mode 6) is one
                                  launch per block of iterations: every launch of a solve of up to 12
                                  blocks is timed, else about a dozen spread evenly over the solve         */
} fs_options;

/* ---- Blocking solves (Alg. 1).  Return the number of iterations performed (>= 0) or a
 * negative fs_status.  They use a library-owned, per-device cached workspace, enqueue the
 * iterations on `stream` in blocks without waiting for them, watch a host-visible stop flag,
 * and synchronise with the stream once, at the end.  check_every = 10. ---- */

/* Dense cost (Alg. 1 REQUIRE: C, mu, nu, eps, tau, K).  Writes f[n], g[m]. */
int fs_sinkhorn_dense(const float *C, const float *a, const float *b, int n, int m,
                      float eps, int max_iter, float tol, float *f, float *g, fs_stream stream);

/* Point clouds, squared-Euclidean cost recomputed on the fly (Sec. 1.1: "Euclidean point
 * cloud inputs").  Writes f[n], g[m]. */
int fs_sinkhorn_points(const float *X, const float *Y, int d, const float *a, const float *b,
                       int n, int m, float eps, int max_iter, float tol, float *f, float *g,
                       fs_stream stream);

/* ---- Asynchronous solves: caller workspace, device-side result, no host synchronisation.
 * All max_iter iterations (plus one trailing error pass) are enqueued; after the device-side
 * stop flag is set the remaining kernels return immediately.  `workspace` is device memory of at
 * least fs_workspace_bytes(n, m, d) bytes, 256-byte aligned, exclusively this call's until its
 * stream work has finished.  `opts` may be NULL.  `result_dev` (device, may be NULL) receives
 * the fs_result. ---- */
size_t fs_workspace_bytes(int n, int m, int d /* 0 = dense */);

fs_status fs_sinkhorn_dense_ex(const float *C, const float *a, const float *b, int n, int m,
                               float eps, int max_iter, float tol, float *f, float *g,
                               fs_stream stream, const fs_options *opts,
                               void *workspace, size_t workspace_bytes, fs_result *result_dev);

fs_status fs_sinkhorn_points_ex(const float *X, const float *Y, int d, const float *a, const float *b,
                                int n, int m, float eps, int max_iter, float tol, float *f, float *g,
                                fs_stream stream, const fs_options *opts,
                                void *workspace, size_t workspace_bytes, fs_result *result_dev);

/* ---- For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): fs_sinkhorn_dense_ex with a scratch buffer built into the library in place
 * of the caller's workspace.  The buffer is a static device array of FS_STATIC_SCRATCH_BYTES (each GPU the
 * library runs on holds its own copy until the process ends); its device address is looked up on the first
 * call on a device.  This entry point calls no hipMalloc, hipFree or other allocating routine, ever.
 * Takes every problem with fs_workspace_bytes(n, m, 0) <= FS_STATIC_SCRATCH_BYTES (n = m = 8192 fits; so do
 * 16384 x 4096 and 256 x 65536) and returns FS_ERR_WORKSPACE, having enqueued nothing, for a larger one.
 * Results are those of fs_sinkhorn_dense_ex bit for bit (same kernels).  All calls on one GPU share the one
 * buffer, which keeps the last call's contents (every solve initialises what it reads): calls that overlap on
 * one GPU -- two streams, or two host threads -- race; order them on one stream or with events. ---- */
#define FS_STATIC_SCRATCH_BYTES (20u << 20)
fs_status fs_sinkhorn_dense_static(const float *C, const float *a, const float *b, int n, int m,
                                   float eps, int max_iter, float tol, float *f, float *g,
                                   fs_stream stream, const fs_options *opts, fs_result *result_dev);

/* Blocking solve with options and a host-side result: like fs_sinkhorn_dense / _points
 * (library workspace, early stop watched from the host, one synchronisation at the end) but
 * honouring `opts` and filling *result_host (ordinary host memory, may be NULL).  Exactly one of
 * C or (X, Y, d > 0) is non-NULL.  Returns iterations performed or a negative fs_status. */
int fs_sinkhorn_solve(const float *C, const float *X, const float *Y, int d,
                      const float *a, const float *b, int n, int m,
                      float eps, int max_iter, float tol, float *f, float *g,
                      fs_stream stream, const fs_options *opts, fs_result *result_host);

/* ---- Plan and cost from potentials (Eq. 5 and the last step of Alg. 1).
 * Exactly one of C or (X, Y, d > 0) is non-NULL.  f64 / g64 (device, optional) give the
 * potentials in double precision and then take the place of f / g.  Asynchronous on `stream`. ---- */

/* P[i*m + j] = a_i b_j exp((f_i + g_j - C_ij)/eps), fp32, n x m row-major. */
fs_status fs_plan(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                  int n, int m, float eps, const float *f, const float *g, float *P, fs_stream stream);

/* cost_dev[0] = sum_ij C_ij P_ij (double, device). */
fs_status fs_cost(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                  int n, int m, float eps, const float *f, const float *g, double *cost_dev,
                  fs_stream stream);

/* Same as fs_plan / fs_cost with the potentials given in double precision. */
fs_status fs_plan_f64(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *f64, const double *g64, float *P,
                      fs_stream stream);
fs_status fs_cost_f64(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *f64, const double *g64, double *cost_dev,
                      fs_stream stream);

/* ---- Annealed regularisation (eps-scaling; named as future work in the paper's conclusion): stages at
 * eps_k = eps_start * decay^k while eps_k > eps, `stage_iters` iterations each, every stage started
 * from the potentials of the one before (handed on in f, g), then the final stage at `eps` with
 * max_iter / tol exactly as fs_sinkhorn_solve.  Blocking.  Returns the iterations of the final stage
 * (>= 0) or an fs_status error; *total_iters (optional, host) counts all stages; *result_host
 * describes the final stage.  eps_start >= eps, 0 < decay < 1, stage_iters >= 1. ---- */
int fs_sinkhorn_annealed(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                         int n, int m, float eps, float eps_start, float decay, int stage_iters, int max_iter,
                         float tol, float *f, float *g, fs_stream stream, const fs_options *opts,
                         fs_result *result_host, int32_t *total_iters);

/* ---- Many small dense problems of one shape in ONE launch (Alg. 1 entirely on the device, one
 * workgroup per problem, C held in registers; the paper's latency-sensitive regime, n >= 64 in its
 * Table 3).  n, m <= FS_SMALL_MAX.  Problem p reads C + p*n*m, a + p*n, b + p*m and writes f + p*n,
 * g + p*m and result_dev[p] (optional, device).  Options used: check_every, warm_start (f, g or f64_in,
 * g64_in hold `batch` starting points), skip_final_err, f64_out / g64_out ([batch][n], [batch][m]),
 * err_history ([batch][err_history_len]).  Asynchronous on `stream`; needs no workspace. ---- */
fs_status fs_sinkhorn_dense_batched(const float *C, const float *a, const float *b, int batch, int n, int m,
                                    float eps, int max_iter, float tol, float *f, float *g, fs_stream stream,
                                    const fs_options *opts, fs_result *result_dev);

/* ---- Diagnostics of a pair of potentials in ONE pass over C (or, for point clouds, one pass over all
 * pairs per side): everything Alg. 1 reports after the loop and everything Secs. 3 and 4.5 define on
 * the plan P of Eq. 5.  Potentials: either f, g (fp32) or f64, g64 (fp64), the other pair NULL.
 * out_dev: device, FS_DIAG_LEN doubles:
 *   [FS_DIAG_COST]    <C, P>                                   (last step of Alg. 1)
 *   [FS_DIAG_MASS]    sum_ij P_ij
 *   [FS_DIAG_KL]      KL(P | a x b) = sum P log(P/(a b)) - sum P + 1              (Eq. 4)
 *   [FS_DIAG_PRIMAL]  <C, P> + eps KL(P | a x b)                                  (Eq. 3)
 *   [FS_DIAG_DUAL]    <a, f> + <b, g> - eps sum P + eps                           (App. A.1)
 *   [FS_DIAG_ROW_ERR] sum_i |sum_j P_ij - a_i|                                    (Sec. 4.5)
 *   [FS_DIAG_COL_ERR] sum_j |sum_i P_ij - b_j|
 * row_marginal_dev[n], col_marginal_dev[m]: optional device outputs (double), NULL = not wanted.
 * Asynchronous on `stream`; uses the library-owned workspace; results are independent of timing. ---- */
#define FS_DIAG_COST 0
#define FS_DIAG_MASS 1
#define FS_DIAG_KL 2
#define FS_DIAG_PRIMAL 3
#define FS_DIAG_DUAL 4
#define FS_DIAG_ROW_ERR 5
#define FS_DIAG_COL_ERR 6
#define FS_DIAG_LEN 8
fs_status fs_diagnostics(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                         int n, int m, float eps, const float *f, const float *g, const double *f64,
                         const double *g64, double *out_dev, double *row_marginal_dev,
                         double *col_marginal_dev, fs_stream stream);

/* ---- Barycentric mapping of the plan (Sec. 5.6: colour transfer, point-cloud correspondences), in one
 * pass and without storing the plan:  T[i][t] = sum_j P_ij Z[j][t] / sum_j P_ij,  t < dz.
 * Z: device [m][dz] fp32 row-major (e.g. the target points themselves); T: device [n][dz] fp32;
 * 1 <= dz <= FS_MAX_BARY_DIM (wider Z: one call per group of columns).  Rows without mass give 0.
 * Potentials: either f, g (fp32) or f64, g64 (fp64), the other pair NULL.  Asynchronous on `stream`;
 * uses the library-owned workspace. ---- */
#define FS_MAX_BARY_DIM 4
fs_status fs_barycentric(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                         int n, int m, float eps, const float *f, const float *g, const double *f64,
                         const double *g64, const float *Z, int dz, float *T, fs_stream stream);

/* ---- One half-step on its own (Eq. 9 / Eq. 10), for kernel-level checks and for callers
 * that drive the loop themselves.  Potentials in double precision, device pointers;
 * asynchronous on `stream`; uses the library-owned workspace. ---- */
fs_status fs_update_f(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *g64, double *f64_out, fs_stream stream);
fs_status fs_update_g(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *f64, double *g64_out, fs_stream stream);

/* ---- Housekeeping ---- */
const char *fs_last_error(void);     /* thread-local, static storage, never NULL        */
void        fs_clear_cache(void);    /* frees cached workspaces and hipGraph executables */
const char *fs_version(void);

/* Which kernel a solve of this shape would run (host logic only, nothing is enqueued; d = 0: dense cost
 * matrix, assumed suitably aligned; blocking != 0: the blocking solves, else the asynchronous ones;
 * compute_units: of the device, 0 = ask the current device).  Returns FS_KERNEL_* or the negative fs_status
 * the solve itself would return for this shape and these options. */
#define FS_KERNEL_STREAM 1   /* dense, streaming row / column kernels, 2 passes over C per iteration */
#define FS_KERNEL_FUSED  2   /* dense, fused row-panel kernel, 1 pass over C per iteration           */
#define FS_KERNEL_SMALL  3   /* whole solve in one workgroup                                          */
#define FS_KERNEL_COOP   4   /* whole solve in one launch, up to 32 workgroups                        */
#define FS_KERNEL_GRID   5   /* whole solve in one launch, one workgroup per compute unit             */
#define FS_KERNEL_POINTS 6   /* point clouds, cost recomputed per pair in every pass                  */
#define FS_KERNEL_PERSIST 7  /* dense, persistent fused row-panel kernel, a block of iterations per launch */
int fs_kernel_choice(int n, int m, int d, const fs_options *opts, int blocking, int compute_units);

/* Average duration (ms) of the dominant kernel over the launches sampled by the most recent
 * blocking solve on this thread that had time_kernel_every > 0, the number of sampled launches, the
 * kernel's name (static storage) and the number of iterations the sampled launches performed in all
 * (= samples, except for the persistent fused pass, whose launches run a block of iterations each).
 * Any output pointer may be NULL.  FS_ERR_INVALID_ARG when there is no such solve.  The durations are read
 * from the events by this call, not by the solve: call it before the next timed solve on the device and before
 * fs_clear_cache().  For benchmarks; no effect on results. */
fs_status fs_last_kernel_timing(float *avg_ms, int32_t *samples, const char **kernel_name,
                                int32_t *iters_sampled);

/* Measurement aid, not part of the method: reads the `bytes` bytes of the device buffer `buf` (16-byte aligned)
 * `reps` times (after two untimed passes) with a plain streaming kernel -- one workgroup of 1024 lanes per
 * compute unit, 16-byte loads -- on `stream`, waits for it, and returns the average duration of a pass in
 * microseconds (HIP events around the `reps` launches) in *us_per_pass (host).  bytes / us_per_pass is the
 * practical read ceiling of the device for a buffer of that size, to be put beside the published HBM peak.
 * FS_ERR_INVALID_ARG for a null or misaligned buffer, bytes < 16 or reps < 1.  For benchmarks. */
fs_status fs_read_rate(const void *buf, size_t bytes, int reps, float *us_per_pass, fs_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTSINKHORN_H */
