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
// by k_combine.
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
#pragma unroll 4
            for (int jj = 0; jj < kTile; ++jj) {
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
        for (int jj = 0; jj < kTile; jj += CH) {
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

// Any dimension: one row per lane, coordinates re-read through the cache.
__global__ __launch_bounds__(kPT) void k_points_lse_anyd(PointsArgs A, Ctl c, int use_next, int ld_shift) {
    extern __shared__ double dyn[];                        // [64][d + 1]
    constexpr int TJ = 64;
    int k;
    if (!launch_active(c, k)) return;
    const int buf = use_next ? ((k & 1) ^ 1) : (k & 1);
    const double *shift = A.colshift + (size_t)buf * ld_shift;
    const int tid = threadIdx.x, d = A.d, ldt = d + 1;
    const int row = blockIdx.x * kPT + tid;
    const bool rok = row < A.nr;
    const double *xr = A.rows + (size_t)(rok ? row : 0) * d;
    Lse acc; acc.init();
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);
    for (int jt = j0; jt < j1; jt += TJ) {
        __syncthreads();
        for (int e = tid; e < TJ * ldt; e += kPT) {
            const int jj = e / ldt, t = e % ldt;
            const int j = jt + jj;
            double v;
            if (j < j1) v = (t == 0) ? shift[j] + A.colconst[j] : A.cols2s[(size_t)j * d + (t - 1)];
            else v = (t == 0) ? -__builtin_huge_val() : 0.0;
            dyn[e] = v;
        }
        __syncthreads();
        for (int jj = 0; jj < TJ; jj += 4) {
            double val[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) val[q] = dyn[(jj + q) * ldt];
            for (int t = 0; t < d; ++t) {
                const double xv = xr[t];
#pragma unroll
                for (int q = 0; q < 4; ++q) val[q] = fma(xv, dyn[(jj + q) * ldt + 1 + t], val[q]);
            }
            acc.add<4>(val);
        }
    }
    if (rok) A.part[(size_t)blockIdx.y * A.ld + row] = acc.value();
}

bool points_optimistic(int d) { return d <= 4; }

void points_plan(int nr, int nc, int d, int *JS, int *cols_per_split) {
    const int rows_per_wg = (d <= 4) ? kPT * kIB : kPT;
    const int rowblocks = (nr + rows_per_wg - 1) / rows_per_wg;
    int js = (2048 + rowblocks - 1) / rowblocks;
    const int maxjs = (nc + kTile - 1) / kTile;
    if (js > maxjs) js = maxjs;
    if (js > 256) js = 256;
    if (js < 1) js = 1;
    int cps = (nc + js - 1) / js;
    cps = ((cps + kTile - 1) / kTile) * kTile;             // whole tiles per slice
    js = (nc + cps - 1) / cps;
    *JS = js;
    *cols_per_split = cps;
}

hipError_t launch_points_lse(hipStream_t st, const PointsArgs &a, const Ctl &c, int use_next_shift, int ld_shift) {
    if (a.d <= 4) {
        const dim3 grid((a.nr + kPT * kIB - 1) / (kPT * kIB), a.JS);
        switch (a.d) {
            case 1: hipLaunchKernelGGL((k_points_lse<1, kIB>), grid, dim3(kPT), 0, st, a, c, use_next_shift, ld_shift); break;
            case 2: hipLaunchKernelGGL((k_points_lse<2, kIB>), grid, dim3(kPT), 0, st, a, c, use_next_shift, ld_shift); break;
            case 3: hipLaunchKernelGGL((k_points_lse<3, kIB>), grid, dim3(kPT), 0, st, a, c, use_next_shift, ld_shift); break;
            default: hipLaunchKernelGGL((k_points_lse<4, kIB>), grid, dim3(kPT), 0, st, a, c, use_next_shift, ld_shift); break;
        }
    } else {
        const dim3 grid((a.nr + kPT - 1) / kPT, a.JS);
        const size_t lds = (size_t)64 * (a.d + 1) * sizeof(double);
        hipLaunchKernelGGL(k_points_lse_anyd, grid, dim3(kPT), lds, st, a, c, use_next_shift, ld_shift);
    }
    return hipGetLastError();
}

}  // namespace fs
