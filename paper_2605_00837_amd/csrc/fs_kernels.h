// Host-visible declarations of the kernel launchers (one translation unit per
// kernel family; the C ABI in fs_api.hip drives them).
#pragma once
#include <hip/hip_ext.h>

#include "fs_device.h"

namespace fs {

// Arrays of one solve.  F, U, G, V are double-buffered by iteration parity:
// buffer (k & 1) holds the potentials after k iterations.
struct Pots {
    double *F, *U;        // [2][n_ld]   F_i = -s f_i,  U_i = log2 a_i - F_i
    double *G, *V;        // [2][m_ld]   G_j = -s g_j,  V_j = log2 b_j - G_j
    const double *la2;    // [n] log2 a_i
    const double *lb2;    // [m] log2 b_j
    const float *a;       // [n] weights (for the error terms)
    const float *b;       // [m]
    int32_t n, m, n_ld, m_ld;
    double s;             // log2(e) / eps
};

struct DenseArgs {
    const float *C;       // n x m row-major; fp32, or (c_dtype 1, 2) entries of 2 bytes: fp16, bfloat16
    int32_t c_dtype;
    Pots p;
    double *colpart;      // [P][m_ld] per-panel partial column LSE values
    int32_t P;            // number of row panels of the column pass
    int32_t rows_per_panel;
    // short and wide matrices: the row pass runs over row_splits column ranges of row_cps columns and writes
    // rowpart[split][n_ld] partial LSE values for the combine kernel (row_splits <= 1: it writes F and U itself)
    double *rowpart;
    int32_t row_splits, row_cps;
};

// The LDS-prefetch fused pass sums plan entries in fp32 (its column phase): a column whose total mass
// T_j is below kColMassFloor (or not a number) may have lost terms to fp32 underflow and is recomputed
// exactly by the combine kernel (see the kernel's header for the bound).  After every iteration the device
// publishes a hint (bit 1 of State::flags): FAST if at most 128 columns moved by more than kFastBelow (base-2
// units), ROBUST otherwise; the driver runs the exact streaming kernels while the hint says ROBUST.
constexpr double kFastBelow = 40.0;
constexpr double kColRepairBelow = 60.0;  // optimistic point-cloud pass: a value this far below the old one is recomputed
constexpr double kColMassFloor = 1.3552527156068805e-20;   // 2^-66
constexpr double kPadF = 1e300;           // F of the rows in the padding behind the n rows (see k_init)
constexpr double kRepairAbove = 100.0;    // optimistic point-cloud pass: fp32 sums stay finite up to 2^127

// Where the row-marginal error comes from.  r_i = a_i 2^(Fnew_i - Fold_i) is the row marginal of
// the iterate a launch started from (the new f-update computes exactly the LSE of Sec. 4.5), so
// err = sum_i a_i |2^(Fnew_i - Fold_i) - 1| needs only the two F buffers.
struct ErrSrc {
    const double *F;          // [2][n_ld]
    const float *a;           // [n]
    int32_t n, n_ld;
};

// One combine launch: out[j] = LSE2 over p < P of part[p][j] (+ rowconst[j]),
// then pot = out, shift = lw2 - out, optionally the error terms against the old
// potential, optionally the once-per-iteration state advance.
struct CombineArgs {
    const double *part;       // [P][ld]
    int32_t P, ld, len;
    const double *rowconst;   // [len] or null
    const double *lw2;        // [len] log2 weights of this side
    const float *w;           // [len] weights of this side (error terms)
    double *pot;              // [2][ld]
    double *shift;            // [2][ld]
    int32_t do_advance;       // 1: this is the g-update: also evaluate the error terms of Sec. 4.5 from
                              //    the old and new F, and let the last workgroup advance the state
    ErrSrc es;
    // Repair of columns whose partials come from the LDS-prefetch fused pass: when repair_C is
    // non-null, a column whose total is below kColMassFloor (or NaN) is recomputed exactly from
    // column j of C and the new U.
    const float *repair_C;    // n x len row-major, or null
    const double *repair_U;   // [2][repair_ld]
    int32_t repair_n, repair_ld, repair_dtype;   // repair_dtype: storage of repair_C as in DenseArgs::c_dtype
    double repair_s;
    // Repair of entries whose partials come from the optimistic point-cloud pass (only looked at while
    // the pace hint says FAST): when pr_rows is non-null, a combined value outside
    // [old - kColRepairBelow, old + kRepairAbove] (or NaN) is recomputed exactly over all columns.
    const double *pr_rows;      // [len][d] coordinates of this side
    const double *pr_cols2s;    // [pr_nc][d] other side, times 2s
    const double *pr_colconst;  // [pr_nc]
    const double *pr_colshift;  // [pr_nc] V or U the pass ran with (buffer already selected)
    int32_t pr_nc, pr_d;
    int32_t pr_shift_next;      // 1: pr_colshift is [2][pr_ld] and the pass used the NEXT buffer
    int32_t pr_ld;
};

// warm: bit 0 = start f from f_in / f64_in, bit 1 = start g from g_in / g64_in (else zero)
hipError_t launch_init(hipStream_t st, const Pots &p, State *state, const float *f_in, const float *g_in,
                       const double *f64_in, const double *g64_in, int warm, void *persist_sync = nullptr);
// out[t] = -pot[t] / s (potential in natural units, double precision)
hipError_t launch_export(hipStream_t st, const double *pot, int len, double s, double *out);
hipError_t launch_finalize(hipStream_t st, const Pots &p, State *state, float *f, float *g,
                           double *f64_out, double *g64_out, void *result_dev, void *result_host);
hipError_t launch_combine(hipStream_t st, const CombineArgs &a, const Ctl &c);
hipError_t launch_advance(hipStream_t st, const ErrSrc &es, const Ctl &c);

// Dense streaming kernels (any n, m).
void dense_stream_plan(int n, int m, int *P, int *rows_per_panel);
// A pair of events that the runtime stamps with the start and the stop of ONE dispatch (both null: an
// ordinary launch).  This is how the library times its dominant kernel: begin to end on the device, as a
// kernel trace does, without the dispatch gap that events recorded around a launch include.
struct Stamp {
    hipEvent_t t0 = nullptr, t1 = nullptr;
};
template <class... P, class... A>
inline void launch_stamped(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t st, const Stamp &tm, const A &...args) {
    if (tm.t0 && tm.t1) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, tm.t0, tm.t1, 0, static_cast<P>(args)...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, st, static_cast<P>(args)...);
}
hipError_t launch_dense_row(hipStream_t st, const DenseArgs &a, const Ctl &c, const Stamp &tm = Stamp());
// column ranges of the row pass (1: none): only for few rows and very many columns
void dense_row_split_plan(int n, int m, int *splits, int *cols_per_split);
hipError_t launch_dense_col(hipStream_t st, const DenseArgs &a, const Ctl &c);

// Dense fused row-panel kernel (m limited by what a workgroup holds in registers).
bool dense_fused_supported(int n, int m, const void *C, int c_dtype);
void dense_fused_plan(int n, int m, int *P);
hipError_t launch_dense_fused(hipStream_t st, const DenseArgs &a, const Ctl &c, int variant, const Stamp &tm = Stamp());
int dense_fused_grid(int n, int m, int variant, int c_dtype);
bool dense_fused_predicts(int m, int variant, int c_dtype);   // this shape / variant uses predicted column references

// Point-cloud kernels.
struct PointsArgs {
    // rows side (plain coordinates, fp64) and columns side (coordinates pre-multiplied by 2s)
    const double *rows;       // [nr][d]
    const double *cols2s;     // [nc][d]
    const double *colconst;   // [nc]  -s |col|^2
    const double *colshift;   // [nc]  V (or U) of the current iterate
    int32_t nr, nc, d;
    double *part;             // [JS][ld] partial LSE values per row
    int32_t JS, ld, cols_per_split;
    // reference for the optimistic pass: the rows' own potential ([2][ld], buffer of the current
    // iterate) and the row constant -s |row|^2 that the combine kernel adds to the LSE
    const double *rowpot;
    const double *rowconst;
};
void points_plan(int nr, int nc, int d, int *JS, int *cols_per_split);
void points_plan_tiles(int nr, int nc, int d, int *JS, int *cols_per_split);   // after-the-loop kernels, d > 4
// After-the-loop vector kernels (d <= 4, 256 rows x ib per workgroup): rows per lane and column slices of
// whole 64-column groups, about `wgs` workgroups and at most `max_slices` slices.
void points_plan_after(int nr, int nc, int wgs, int max_slices, int *JS, int *cols_per_split, int *ib);
bool points_optimistic(int d);      // does the LSE pass for this dimension have the optimistic (FAST) variant?
hipError_t launch_points_lse(hipStream_t st, const PointsArgs &a, const Ctl &c, int use_next_shift, int ld_shift,
                             const Stamp &tm = Stamp());
hipError_t launch_points_prep(hipStream_t st, const float *X, int n, int d, double s, double *plain,
                              double *scaled, double *negsq);

// Plan and cost.
struct PlanArgs {
    const float *C, *X, *Y;
    const float *a, *b;
    const float *f, *g;          // fp32 potentials, or
    const double *f64, *g64;     // fp64 potentials (take precedence when non-null)
    int32_t n, m, d;
    double s;
};
hipError_t launch_plan(hipStream_t st, const PlanArgs &a, float *P, double *scratch, int nscratch);
hipError_t launch_cost(hipStream_t st, const PlanArgs &a, double *cost_dev, double *scratch, int nscratch);
int cost_scratch_len(int n, int m);
int plan_scratch_len(int n, int m, int d);

// Diagnostics in one pass (cost, mass, KL, primal, dual, marginal errors; optional marginals).
size_t diag_scratch_bytes(int n, int m, int d);
hipError_t launch_diag(hipStream_t st, const PlanArgs &a, double *out8, double *row_marg, double *col_marg,
                       void *scratch, size_t scratch_bytes, unsigned int *tickets, double *cost_only_out = nullptr);

// ri = s f + log2 a, cj = s g + log2 b; for point clouds also the repacked clouds (plain, times 2s, s|.|^2).
hipError_t launch_plan_prep_all(hipStream_t st, const PlanArgs &a, double *ri, double *cj, double *xp, double *xs,
                                double *xq, double *yp, double *ys, double *yq);

// Barycentric mapping of the plan: T[i][t] = sum_j P_ij Z[j][t] / sum_j P_ij, t < dz <= kBaryMaxDim.
constexpr int kBaryMaxDim = 4;
size_t bary_scratch_bytes(int n, int m, int d);
hipError_t launch_bary(hipStream_t st, const PlanArgs &a, const float *Z, int dz, float *T, void *scratch,
                       size_t scratch_bytes);

// Whole solve of small dense problems in one launch (one workgroup per problem).
constexpr int kSmallMax = 256;
struct ResultRecord { int32_t iters, converged, nonfinite; float marginal_err; };    // = fs_result
constexpr int32_t kGaveUp = 2;                   // ResultRecord::nonfinite of a one-launch solve that abandoned a wait
struct SmallArgs {
    const float *C, *a, *b;          // [batch][n][m], [batch][n], [batch][m]
    int32_t c_dtype;                 // storage of C: 0 fp32, 1 fp16, 2 bfloat16 (entries of 2 bytes)
    int32_t n, m, batch;
    double s;
    int32_t max_iter, check_every;
    double tol;                      // <= 0: fixed iteration count
    int32_t warm;                    // 1: start from f_in, g_in (or f64_in, g64_in when non-null)
    const float *f_in, *g_in;
    const double *f64_in, *g64_in;
    float *f, *g;                    // [batch][n], [batch][m]
    double *f64_out, *g64_out;       // optional
    float *err_history;              // optional [batch][err_history_len]
    int32_t err_history_len;
    int32_t want_final_err;          // evaluate err of the last iterate when no stop fired
    ResultRecord *result;            // optional [batch], device or pinned host memory
};
hipError_t launch_small(hipStream_t st, const SmallArgs &a);

// ---- the grid-wide wait of the kernels whose workgroups stay resident on every compute unit (fs_persist.hip,
//      fs_resident.hip, fs_grid.hip; the code is in fs_persist_sync.h)
struct GridLine { unsigned long long v; unsigned long long pad[31]; };      // 256 bytes
// Counters of the persistent pass (all monotone over a solve).  A workgroup counts itself into one of 8 group
// counters; the last of a group writes the generation into the group's word of the `done` line -- of every copy of
// it: a polled line sees 8 plain stores per wait, no read-modify-write, and the polls of only a few workgroups
// (polled by all 256, a line takes hundreds of requests per microsecond and the store everybody waits for queues
// behind them).
constexpr int kSyncGroups = 8;                   // arrival counters (a workgroup counts itself into number workgroup mod kSyncGroups)
struct PersistSync {
    GridLine grp[kSyncGroups];
    unsigned long long done[kSyncGroups];        // generation each group has completed
    unsigned long long abort_flag;
    unsigned long long pad[31 - kSyncGroups];
    // kSyncCopies copies of that line (words 0 .. kSyncGroups-1: done, then the abort flag), 256 bytes apart: a workgroup polls
    // copy workgroup mod kSyncCopies, so that a line is watched by a few workgroups, not by all of them
    unsigned long long copy[64][32];
};
constexpr int kSyncCopies = 64;

// ---- mid-size dense problems: the whole solve in one launch over up to 32 workgroups (fs_coop.hip)
constexpr int kCoopMax = 1024;                   // largest n, m
// (up to 32 workgroups: one counter that everybody adds to and polls is the faster wait there, 5.66 against 5.81 us
// per iteration at 256 x 256)
struct CoopSync {                                // two 256-byte lines
    unsigned long long arrivals;                 // workgroups that have reached a grid-wide wait, ever
    unsigned long long pad0[31];
    unsigned int abort_flag, bad;                // a wait was abandoned; some returned potential is not finite
    unsigned int pad1[62];
};
struct CoopArgs : SmallArgs {                    // batch is ignored (one problem)
    const float *X, *Y;                          // point clouds [n][d], [m][d] (then C is null), or null
    int32_t d;
    double *xchg;                                // [2][W][ldx]: published partials by parity of the round
    CoopSync *sync;
    int32_t ldx;                                 // slots per workgroup: columns, the last one the error partial
    int32_t spin_limit;                          // polls before a grid-wide wait is abandoned (<= 0: default)
};
bool coop_supported(int n, int m);
bool coop_points_supported(int n, int m);
size_t coop_scratch_bytes();                     // device scratch (256-byte aligned) one solve needs
// variant 0: up to 32 workgroups; 1, 2, 3: at most 16, 8, 4 (more rows per lane)
hipError_t launch_coop(hipStream_t st, const CoopArgs &a, void *scratch, int variant);

// ---- dense problems up to 4096 x 2048: the whole solve in one launch over up to 256 workgroups, two
//      grid-wide waits per iteration (fs_grid.hip)
constexpr int kGridMaxN = 4096, kGridMaxM = 2048;
constexpr int kGridWMax = 256;                   // most workgroups (each needs a compute unit of its own)
// the one-launch kernel of fs_grid.hip waits the same way; `bad`: some workgroup met a non-finite value
struct GridSync { PersistSync ps; GridLine bad; };
struct GridArgs : SmallArgs {                    // batch is ignored (one problem)
    const float *X, *Y;                          // point clouds [n][d], [m][d] (then C is null), or null
    int32_t d;
    double *xchg1;                               // [W][ldx]: column partials of every workgroup; last slot: error partial
    double *xchg2;                               // [ldx]: the new V, written strip by strip
    GridSync *sync;
    int32_t ldx, spin_limit;
};
// ---- dense fp32 problems with 128 < m <= 16384: a block of iterations of the fused row-panel pass in one
//      launch, one resident workgroup per compute unit, two grid-wide waits per iteration (fs_persist.hip; up to
//      1024 columns only its resident form, fs_resident.hip)
struct PersistArgs {
    PersistSync *sync;
    double *wgpart;                              // [workgroups]: error terms of each workgroup's rows
    int32_t nb;                                  // iterations this launch runs at most
    int32_t spin_limit;                          // polls before a grid-wide wait is abandoned
    int32_t final_err;                           // 1: a launch that reaches max_iter without a stop goes on to evaluate
                                                 //    err of the last iterate (one more row phase over C) and closes the solve
#ifdef FS_PERSIST_TRACE
    long long *trace;                            // debug builds: [workgroups][8] time stamps of one iteration
#endif
};
// fs_calib.hip: a plain streaming read of `bytes` bytes (measurement aid; `sink` is never written)
hipError_t launch_read_stream(hipStream_t st, const void *buf, size_t bytes, int cus, float *sink);
bool dense_persist_supported(int n, int m, const void *C, int c_dtype);
int dense_persist_grid(int n, int m, int cus);   // workgroups of the launch on a device with `cus` compute units
size_t persist_scratch_bytes();
// variant 0: the 512-lane kernel of fs_resident.hip where the workgroups can hold their share of C, or most of the
// panels they stream are few (up to 32 panels per workgroup; 20 between 6145 and 8191 columns), else the 1024-lane streaming kernel; 1: always the
// 1024-lane streaming kernel; 2: the 512-lane kernel up to 32 panels per workgroup.  Up to 1024 columns there is only
// the 512-lane kernel, whatever the variant.
hipError_t launch_persist(hipStream_t st, const DenseArgs &a, const Ctl &c, void *scratch, int cus, int nb,
                          int spin_limit, int final_err, int variant, const Stamp &tm = Stamp());
bool dense_persist_resident(int n, int m, int cus, int variant);   // which of the two forms launch_persist takes
// fs_resident.hip: the same iteration with the workgroup's share of C held in LDS and registers for the whole launch
int dense_resident_grid(int n, int m, int cus, bool all);   // workgroups of its launch; 0: shape not taken
hipError_t launch_resident(hipStream_t st, const DenseArgs &a, const PersistArgs &x, const Ctl &c, int grid,
                           const Stamp &tm);

bool grid_supported(int n, int m, int wmax, bool points);   // wmax: workgroups that can be resident at once (compute units)
size_t grid_scratch_bytes();
hipError_t launch_grid(hipStream_t st, const GridArgs &a, void *scratch, int wmax);

}  // namespace fs
