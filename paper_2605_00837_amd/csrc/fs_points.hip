// Point-cloud kernels: the cost C_ij = |x_i - y_j|^2 is recomputed on the fly
// inside the LogSumExp of Eq. 9 / Eq. 10 and never stored.
//
// With s = log2(e)/eps the exponent of the f-update is
//     V_j - s|x_i - y_j|^2 = (-s|x_i|^2) + [ (V_j - s|y_j|^2) + x_i . (2 s y_j) ]
// so per pair only the bracket is evaluated: d fused multiply-adds in fp64
// (products of fp32 coordinates are exact in fp64, so the expanded form loses
// nothing), the row constant is added once after the LSE.  The g-update is the
// same kernel with the roles of the two clouds exchanged.
//
// Work split: a workgroup of 256 lanes owns 256*IB rows (IB per lane, kept in
// registers) and one slice of the columns; column tiles are staged in LDS and
// read back as wave-wide broadcasts.  Per-slice partial LSE values are merged
// by k_combine.  More than 4 coordinates: the matrix-core kernel further down.
#include "fs_kernels.h"

namespace fs {

constexpr int kPT = 256;       // threads per workgroup
constexpr int kTile = 256;     // columns staged per tile
constexpr int kIB = 4;         // rows per lane
constexpr int kChunk = 8;      // pairs folded per rescale

__global__ __launch_bounds__(256) void k_points_prep(const float *X, int n, int d, double s, double *plain,
                                                     double *scaled, double *negsq) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    double sq = 0.0;
    for (int t = 0; t < d; ++t) {
        const double x = (double)X[(size_t)i * d + t];
        plain[(size_t)i * d + t] = x;
        scaled[(size_t)i * d + t] = 2.0 * s * x;
        sq = fma(x, x, sq);
    }
    negsq[i] = -s * sq;
}

hipError_t launch_points_prep(hipStream_t st, const float *X, int n, int d, double s, double *plain,
                              double *scaled, double *negsq) {
    hipLaunchKernelGGL(k_points_prep, dim3((n + 255) / 256), dim3(256), 0, st, X, n, d, s, plain, scaled, negsq);
    return hipGetLastError();
}

// Two ways through the column slice, chosen by the pace hint the device keeps next to the
// iteration counter (the same for every workgroup of a launch, and for the combine kernel that
// follows):
//   ROBUST  exact online LogSumExp, one fp64 running maximum per row and chunk of kChunk pairs;
//   FAST    optimistic: the previous value of the row's own LSE is the reference, every pair costs
//           d fp64 FMAs, one fp64 subtraction, one conversion, v_exp_f32 and one fp32 addition.
//           Nothing is checked here: the combine kernel compares the merged result with the
//           reference and recomputes exactly whatever moved too far for the fp32 sums to be trusted.
template <int D, int IB>
__global__ __launch_bounds__(kPT) void k_points_lse(PointsArgs A, Ctl c, int use_next, int ld_shift) {
    __shared__ __align__(16) double tile[kTile][D + 1];
    const unsigned long long kd = load_counter(c);
    const int tid = threadIdx.x;

    double x[IB][D];
    double rconst[IB];
    int row[IB];
#pragma unroll
    for (int b = 0; b < IB; ++b) {
        row[b] = (blockIdx.x * IB + b) * kPT + tid;
        const bool ok = row[b] < A.nr;
#pragma unroll
        for (int t = 0; t < D; ++t) x[b][t] = ok ? A.rows[(size_t)row[b] * D + t] : 0.0;
        rconst[b] = ok ? A.rowconst[row[b]] : 0.0;
    }
    int k;
    bool fast;
    if (!counter_active(c, kd, k, &fast)) return;
    const int cur = k & 1;
    const int buf = use_next ? (cur ^ 1) : cur;
    const double *shift = A.colshift + (size_t)buf * ld_shift;
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);

    auto stage = [&](int jt) {
        __syncthreads();                                   // previous tile fully consumed
        const int j = jt + tid;
        if (j < j1) {
            tile[tid][0] = shift[j] + A.colconst[j];
#pragma unroll
            for (int t = 0; t < D; ++t) tile[tid][1 + t] = A.cols2s[(size_t)j * D + t];
        } else {
            tile[tid][0] = -__builtin_huge_val();          // contributes 2^-inf = 0
#pragma unroll
            for (int t = 0; t < D; ++t) tile[tid][1 + t] = 0.0;
        }
        __syncthreads();
    };

    if (fast) {
        double ref[IB];
        float sum[IB];
#pragma unroll
        for (int b = 0; b < IB; ++b) {
            // LSE of the bracket = potential - row constant
            ref[b] = row[b] < A.nr ? A.rowpot[(size_t)cur * A.ld + row[b]] - rconst[b] : 0.0;
            sum[b] = 0.0f;
        }
        for (int jt = j0; jt < j1; jt += kTile) {
            stage(jt);
            const int cnt = min(kTile, (j1 - jt + 3) & ~3);      // staged columns (the tile is padded with -inf)
#pragma unroll 4
            for (int jj = 0; jj < cnt; ++jj) {
                double w[D + 1];
#pragma unroll
                for (int t = 0; t <= D; ++t) w[t] = tile[jj][t];
#pragma unroll
                for (int b = 0; b < IB; ++b) {
                    double acc2 = w[0];
#pragma unroll
                    for (int t = 0; t < D; ++t) acc2 = fma(x[b][t], w[1 + t], acc2);
                    sum[b] += fast_exp2((float)(acc2 - ref[b]));
                }
            }
        }
#pragma unroll
        for (int b = 0; b < IB; ++b)
            if (row[b] < A.nr) A.part[(size_t)blockIdx.y * A.ld + row[b]] = ref[b] + log2_sum(sum[b]);
        return;
    }

    Lse acc[IB];
#pragma unroll
    for (int b = 0; b < IB; ++b) acc[b].init();
    constexpr int CH = IB <= 2 ? kChunk : 4;               // pairs folded per rescale
    for (int jt = j0; jt < j1; jt += kTile) {
        stage(jt);
        const int cnt = min(kTile, (j1 - jt + CH - 1) / CH * CH);
        for (int jj = 0; jj < cnt; jj += CH) {
            double val[IB][CH];
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                double w[D + 1];
#pragma unroll
                for (int t = 0; t <= D; ++t) w[t] = tile[jj + q][t];
#pragma unroll
                for (int b = 0; b < IB; ++b) {
                    double acc2 = w[0];
#pragma unroll
                    for (int t = 0; t < D; ++t) acc2 = fma(x[b][t], w[1 + t], acc2);
                    val[b][q] = acc2;
                }
            }
#pragma unroll
            for (int b = 0; b < IB; ++b) acc[b].template add<CH>(val[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < IB; ++b)
        if (row[b] < A.nr) A.part[(size_t)blockIdx.y * A.ld + row[b]] = acc[b].value();
}

// ---------------------------------------------------------------- d > 4: the dot products are a contraction
// For more than a handful of coordinates the bracket's x_i . (2 s y_j) is a dense n x m x d contraction,
// and it runs on the fp64 matrix cores: v_mfma_f64_16x16x4f64 computes a 16 x 16 tile of dot products
// over 4 coordinates per instruction (A: lane l holds x[row l % 16][k = l / 16]; B: lane l holds
// y'[col l % 16][k = l / 16]; D register r of lane l is entry (row l / 16 + 4 r, col l % 16)).  Products
// of fp32 coordinates are exact in fp64 and the accumulation is fp64, so nothing is lost against the
// d <= 4 kernels.  A wave keeps a few row tiles (16 rows each) of x in registers for the whole launch
// and streams column tiles of y' from LDS; the accumulator starts at the column constant
// (V_j - s|y_j|^2, minus the row's reference in the optimistic variant), so what comes out of the
// matrix core is the exponent itself.  (kRT = 4 row tiles up to d = 16, 2 beyond.)  Row sums live in the 16 lanes that share a row quad and meet by
// DPP at the end.  Both variants of the pass (see above k_points_lse) are here: FAST adds 2^(arg - ref);
// ROBUST is the exact online LSE with one running maximum per row, updated per tile of 16 columns.
constexpr int kMfmaTJ = 64;          // columns staged per LDS tile
// row tiles per wave: more of them reuse every B operand more often, as long as the A operands fit
constexpr int mfma_rt(int d4) { return d4 <= 4 ? 4 : 2; }
constexpr int mfma_rows(int d4) { return 4 * mfma_rt(d4) * 16; }      // rows per workgroup of 4 waves

typedef double double4_v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double row16_max_f64(double v) {      // all-reduce over a DPP row of 16 lanes
    v = dmax(v, dpp_f64<0x128>(v));
    v = dmax(v, dpp_f64<0x124>(v));
    v = dmax(v, dpp_f64<0x122>(v));
    v = dmax(v, dpp_f64<0x121>(v));
    return v;
}
__device__ __forceinline__ float row16_sum_f32(float v) {
    v += dpp_f32<0x128>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x122>(v);
    v += dpp_f32<0x121>(v);
    return v;
}

template <int D4>
__global__ __launch_bounds__(256) void k_points_mfma(PointsArgs A, Ctl c, int use_next, int ld_shift) {
    constexpr int kRT = mfma_rt(D4), kMfmaRows = mfma_rows(D4);
    constexpr int LDT = 4 * D4 + 1;                       // padded row of the LDS tile (doubles)
    __shared__ double tile[kMfmaTJ][LDT];
    __shared__ double tilew[kMfmaTJ];
#if defined(__HIP_DEVICE_COMPILE__)
    const unsigned long long kd = load_counter(c);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 15, lk = lane >> 4;
    const int d = A.d;
    const int row0 = blockIdx.x * kMfmaRows + wave * (kRT * 16);

    // A operands: x[row0 + rt*16 + lj][4 ks + lk], zero beyond nr and beyond d
    double a[kRT][D4];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) {
        const int row = row0 + rt * 16 + lj;
#pragma unroll
        for (int ks = 0; ks < D4; ++ks) {
            const int t = 4 * ks + lk;
            a[rt][ks] = (row < A.nr && t < d) ? A.rows[(size_t)row * d + t] : 0.0;
        }
    }
    // the rows this lane sees in the results: row0 + rt*16 + lk + 4 r
    double rconst[kRT][4];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + rt * 16 + lk + 4 * r;
            rconst[rt][r] = row < A.nr ? A.rowconst[row] : 0.0;
        }
    int k;
    bool fast;
    if (!counter_active(c, kd, k, &fast)) return;
    const int cur = k & 1;
    const int buf = use_next ? (cur ^ 1) : cur;
    const double *shift = A.colshift + (size_t)buf * ld_shift;
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);

    // FAST: ref = previous LSE of the bracket; ROBUST: M = running maximum
    double ref[kRT][4];
    float sum[kRT][4];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + rt * 16 + lk + 4 * r;
            ref[rt][r] = fast ? (row < A.nr ? A.rowpot[(size_t)cur * A.ld + row] - rconst[rt][r] : 0.0) : kNegHuge;
            sum[rt][r] = 0.0f;
        }

    for (int jt = j0; jt < j1; jt += kMfmaTJ) {
        __syncthreads();                                   // previous tile fully consumed
        for (int e = tid; e < kMfmaTJ * 4 * D4; e += 256) {
            const int jj = e / (4 * D4), t = e % (4 * D4);
            const int j = jt + jj;
            tile[jj][t] = (j < j1 && t < d) ? A.cols2s[(size_t)j * d + t] : 0.0;
        }
        if (tid < kMfmaTJ) {
            const int j = jt + tid;
            tilew[tid] = j < j1 ? shift[j] + A.colconst[j] : -__builtin_huge_val();
        }
        __syncthreads();
#pragma unroll
        for (int ct = 0; ct < kMfmaTJ / 16; ++ct) {
            double b[D4];
#pragma unroll
            for (int ks = 0; ks < D4; ++ks) b[ks] = tile[ct * 16 + lj][4 * ks + lk];
            const double w = tilew[ct * 16 + lj];
            // kRT independent accumulator chains, interleaved, so that a wave always has a matrix
            // instruction to issue while the previous ones are still in the pipeline
            double4_v acc[kRT];
#pragma unroll
            for (int rt = 0; rt < kRT; ++rt) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[rt][r] = fast ? w - ref[rt][r] : w;
            }
#pragma unroll
            for (int ks = 0; ks < D4; ++ks)
#pragma unroll
                for (int rt = 0; rt < kRT; ++rt)
                    acc[rt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[rt][ks], b[ks], acc[rt], 0, 0, 0);
#pragma unroll
            for (int rt = 0; rt < kRT; ++rt) {
                if (fast) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) sum[rt][r] += fast_exp2((float)acc[rt][r]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const double Mn = dmax(ref[rt][r], row16_max_f64(acc[rt][r]));    // the same in all 16 lanes of the row
                        sum[rt][r] = sum[rt][r] * fast_exp2((float)(ref[rt][r] - Mn)) + fast_exp2((float)(acc[rt][r] - Mn));
                        ref[rt][r] = Mn;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float S = row16_sum_f32(sum[rt][r]);
            const int row = row0 + rt * 16 + lk + 4 * r;
            if (lj == 0 && row < A.nr) A.part[(size_t)blockIdx.y * A.ld + row] = ref[rt][r] + log2_sum(S);
        }
#endif
}

bool points_optimistic(int d) { (void)d; return true; }

// Rows per lane of the vector kernels: 4 (every staged column is reused four times) once there are enough
// rows to fill the chip that way, 1 below (4096 x 4096: 27 against 29 us per iteration).
static int points_ib(int nr) { return nr < 8192 ? 1 : kIB; }

void points_plan(int nr, int nc, int d, int *JS, int *cols_per_split) {
    // About 2048 workgroups per launch: row blocks x column slices, a slice being a whole number of
    // 64-column groups (the matrix-core kernel's tile; the vector kernels stage up to kTile at a time).
    const int rows_per_wg = (d <= 4) ? kPT * points_ib(nr) : mfma_rows(d <= 8 ? 2 : d <= 16 ? 4 : d <= 32 ? 8 : 16);
    const int rowblocks = (nr + rows_per_wg - 1) / rows_per_wg;
    int want = (2048 + rowblocks - 1) / rowblocks;
    if (want > 256) want = 256;
    int cps = (nc + want - 1) / want;
    cps = ((cps + kMfmaTJ - 1) / kMfmaTJ) * kMfmaTJ;
    // whole tiles of kTile columns as soon as that still gives every compute unit two workgroups: fewer
    // partials for the combine kernel, fewer stage-and-wait rounds per column
    if (cps < kTile && (long long)rowblocks * ((nc + kTile - 1) / kTile) >= 512) cps = kTile;
    *JS = (nc + cps - 1) / cps;
    *cols_per_split = cps;
}

// The after-the-loop matrix-core kernels (diagnostics, barycentric mapping; one pass each): slices of whole
// tiles of kTile columns.
void points_plan_tiles(int nr, int nc, int d, int *JS, int *cols_per_split) {
    const int rows_per_wg = (d <= 4) ? kPT * kIB : kPT;
    const int rowblocks = (nr + rows_per_wg - 1) / rows_per_wg;
    int js = (2048 + rowblocks - 1) / rowblocks;
    const int maxjs = (nc + kTile - 1) / kTile;
    if (js > maxjs) js = maxjs;
    if (js > 256) js = 256;
    if (js < 1) js = 1;
    int cps = (nc + js - 1) / js;
    cps = ((cps + kTile - 1) / kTile) * kTile;
    *JS = (nc + cps - 1) / cps;
    *cols_per_split = cps;
}

void points_plan_after(int nr, int nc, int wgs, int max_slices, int *JS, int *cols_per_split, int *ib) {
    *ib = points_ib(nr);
    const int rows_per_wg = kPT * *ib;
    const int rowblocks = (nr + rows_per_wg - 1) / rows_per_wg;
    int want = (wgs + rowblocks - 1) / rowblocks;
    if (want > max_slices) want = max_slices;
    int cps = (nc + want - 1) / want;
    cps = ((cps + 63) / 64) * 64;
    *JS = (nc + cps - 1) / cps;
    *cols_per_split = cps;
}

hipError_t launch_points_lse(hipStream_t st, const PointsArgs &a, const Ctl &c, int use_next_shift, int ld_shift,
                             const Stamp &tm) {
    if (a.d <= 4 && points_ib(a.nr) == 1) {
        const dim3 grid((a.nr + kPT - 1) / kPT, a.JS);
        switch (a.d) {
            case 1: launch_stamped((k_points_lse<1, 1>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
            case 2: launch_stamped((k_points_lse<2, 1>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
            case 3: launch_stamped((k_points_lse<3, 1>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
            default: launch_stamped((k_points_lse<4, 1>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
        }
    } else if (a.d <= 4) {
        const dim3 grid((a.nr + kPT * kIB - 1) / (kPT * kIB), a.JS);
        switch (a.d) {
            case 1: launch_stamped((k_points_lse<1, kIB>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
            case 2: launch_stamped((k_points_lse<2, kIB>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
            case 3: launch_stamped((k_points_lse<3, kIB>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
            default: launch_stamped((k_points_lse<4, kIB>), grid, dim3(kPT), st, tm, a, c, use_next_shift, ld_shift); break;
        }
    } else {
        const int d4 = a.d <= 8 ? 2 : a.d <= 16 ? 4 : a.d <= 32 ? 8 : 16;
        const dim3 grid((a.nr + mfma_rows(d4) - 1) / mfma_rows(d4), a.JS);
        if (a.d <= 8) launch_stamped(k_points_mfma<2>, grid, dim3(256), st, tm, a, c, use_next_shift, ld_shift);
        else if (a.d <= 16) launch_stamped(k_points_mfma<4>, grid, dim3(256), st, tm, a, c, use_next_shift, ld_shift);
        else if (a.d <= 32) launch_stamped(k_points_mfma<8>, grid, dim3(256), st, tm, a, c, use_next_shift, ld_shift);
        else launch_stamped(k_points_mfma<16>, grid, dim3(256), st, tm, a, c, use_next_shift, ld_shift);
    }
    return hipGetLastError();
}

}  // namespace fs
