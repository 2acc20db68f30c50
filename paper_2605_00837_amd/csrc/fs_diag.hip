// Diagnostics of a pair of potentials in one pass over C (dense) or over all point pairs:
// transport cost (last step of Alg. 1), total mass, KL term and primal objective (Eq. 3), dual
// objective (Eq. 4 and App. A.1), both marginals of the plan of Eq. 5 and their L1 errors (Sec. 4.5).
//
//   P_ij = 2^(e_ij),  e_ij = ri_i + cj_j - s C_ij,  ri_i = s f_i + log2 a_i,  cj_j = s g_j + log2 b_j.
//
// The exponent is formed in fp64 and rounded to fp32 for v_exp_f32; sums over at most a few dozen
// entries are kept in fp32, everything longer in fp64.  The entropy term needs no sum over the entries:
// log(P_ij/(a_i b_j)) = (f_i + g_j - C_ij)/eps by Eq. 5, so  sum P log(P/(a b)) = (<r, f> + <c, g> - <C, P>)/eps
// with the marginals r, c of P, whatever f and g are.
//
// Dense: a workgroup of 1024 lanes owns a strip of 1024*VEC columns and a panel of rows; lanes keep
// their column sums, row sums go wave -> LDS -> one value per (strip, row).  Points: the layout of
// the LSE pass (rows in registers, column tiles in LDS), run once per side so that every marginal
// is a lane-local sum; the cost uses s C_ij = s|x_i|^2 + s|y_j|^2 - x_i . (2 s y_j).
// All partial results are combined in fixed order: the outputs do not depend on timing.
#include "fs_kernels.h"
#include "fs_mfma.h"

namespace fs {

namespace {

constexpr int kDT = 1024;           // threads of the dense kernel
constexpr int kDRows = 16;          // rows per LDS exchange
constexpr int kPT2 = 256;           // threads of the point-cloud kernel
constexpr int kTile2 = 256;
constexpr int kIB2 = 4;
constexpr double kLn2d = 0.6931471805599453094;

struct DiagLayout {
    // dense
    int vec, strip_cols, nstrips, P, rpp;
    // points
    int JSx, cpsx, JSy, cpsy, ibx, iby;
    // scratch offsets (bytes)
    size_t o_ri, o_cj, o_rowpart, o_colpart, o_scal, o_red, o_out, total;
    // points extras
    size_t o_xp, o_xs, o_xq, o_yp, o_ys, o_yq;
    int nred, nscal;
};

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

DiagLayout diag_layout(int n, int m, int d) {
    DiagLayout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
    L.o_ri = take(sizeof(double) * n);
    L.o_cj = take(sizeof(double) * m);
    const int len = n > m ? n : m;
    L.nred = (len + 63) / 64;
    L.o_red = take(sizeof(double) * 8 * L.nred);
    L.o_out = take(sizeof(double) * 8);
    if (d == 0) {
        L.vec = m >= 4 ? 4 : 1;
        L.strip_cols = kDT * L.vec;
        L.nstrips = (m + L.strip_cols - 1) / L.strip_cols;
        int P = (512 + L.nstrips - 1) / L.nstrips;
        const int maxP = (n + kDRows - 1) / kDRows;
        if (P > maxP) P = maxP;
        if (P < 1) P = 1;
        int rpp = (n + P - 1) / P;
        rpp = ((rpp + kDRows - 1) / kDRows) * kDRows;
        L.rpp = rpp;
        L.P = (n + rpp - 1) / rpp;
        L.o_rowpart = take(sizeof(double) * (size_t)L.nstrips * n);
        L.o_colpart = take(sizeof(float) * (size_t)L.P * m);
        L.nscal = L.nstrips * L.P;
        L.o_scal = take(sizeof(double) * 2 * L.nscal);
    } else {
        if (d <= 4) {
            points_plan_after(n, m, 2048, 128, &L.JSx, &L.cpsx, &L.ibx);
            points_plan_after(m, n, 2048, 128, &L.JSy, &L.cpsy, &L.iby);
        } else {
            points_plan_tiles(n, m, d, &L.JSx, &L.cpsx);
            points_plan_tiles(m, n, d, &L.JSy, &L.cpsy);
        }
        L.o_rowpart = take(sizeof(double) * (size_t)L.JSx * n);      // row sums per column slice
        const int rows_per_wg = d <= 4 ? kPT2 * L.ibx : kTileRows;
        const int gx = (n + rows_per_wg - 1) / rows_per_wg;
        // column sums: per block of rows (fp32, d <= 4: one pass does both sides) or per row slice of the second pass
        L.o_colpart = take(d <= 4 ? sizeof(float) * (size_t)gx * m : sizeof(double) * (size_t)L.JSy * m);
        L.nscal = gx * L.JSx;
        L.o_scal = take(sizeof(double) * 2 * L.nscal);
        L.o_xp = take(sizeof(double) * (size_t)n * d);
        L.o_xs = take(sizeof(double) * (size_t)n * d);
        L.o_xq = take(sizeof(double) * n);
        L.o_yp = take(sizeof(double) * (size_t)m * d);
        L.o_ys = take(sizeof(double) * (size_t)m * d);
        L.o_yq = take(sizeof(double) * m);
    }
    L.total = o;
    return L;
}

// ri, cj; for points also the repacked clouds: plain, times 2s, and s|.|^2.
__global__ __launch_bounds__(256) void k_diag_prep(PlanArgs A, double *ri, double *cj, double *xp, double *xs,
                                                   double *xq, double *yp, double *ys, double *yq) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < A.n) {
        const double f = A.f64 ? A.f64[t] : (double)A.f[t];
        ri[t] = fma(A.s, f, log2_weight(A.a[t]));
        if (A.d > 0) {
            double sq = 0.0;
            for (int q = 0; q < A.d; ++q) {
                const double x = (double)A.X[(size_t)t * A.d + q];
                xp[(size_t)t * A.d + q] = x;
                xs[(size_t)t * A.d + q] = 2.0 * A.s * x;
                sq = fma(x, x, sq);
            }
            xq[t] = A.s * sq;
        }
    }
    if (t < A.m) {
        const double g = A.g64 ? A.g64[t] : (double)A.g[t];
        cj[t] = fma(A.s, g, log2_weight(A.b[t]));
        if (A.d > 0) {
            double sq = 0.0;
            for (int q = 0; q < A.d; ++q) {
                const double y = (double)A.Y[(size_t)t * A.d + q];
                yp[(size_t)t * A.d + q] = y;
                ys[(size_t)t * A.d + q] = 2.0 * A.s * y;
                sq = fma(y, y, sq);
            }
            yq[t] = A.s * sq;
        }
    }
}

// Sum of v over the workgroup in a fixed order (tree in LDS); result in thread 0.
template <int T>
__device__ __forceinline__ double block_sum(double v, double *lds) {
    const int t = threadIdx.x;
    __syncthreads();
    lds[t] = v;
    __syncthreads();
#pragma unroll
    for (int w = T / 2; w >= 1; w >>= 1) {
        if (t < w) lds[t] += lds[t + w];
        __syncthreads();
    }
    return lds[0];
}

// ---------------------------------------------------------------- dense
struct DenseDiag {
    const float *C;
    const double *ri, *cj;
    int32_t n, m;
    double s;
    double *rowpart;     // [nstrips][n]
    float *colpart;      // [P][m]
    double *scal;        // [nstrips * P][2]: sum P (s C), sum P e
    int32_t rpp;
    unsigned int *ticket;   // cost only: arrival counter (0 before and after the launch)
    double *cost_out;       // cost only: <C, P>, written by the workgroup that arrives last
};

// COST_ONLY: only sum P C is wanted (fs_cost): no marginals, so no row reductions and no exchange in the loop,
// and the workgroup that arrives last adds the per-workgroup sums in index order and writes the cost: the whole
// call is this one launch after the preparation.
template <int VEC, bool COST_ONLY>
__global__ __launch_bounds__(kDT) void k_diag_dense(DenseDiag A) {
    __shared__ float sRow[COST_ONLY ? 1 : kDRows][kDT / 64];
    __shared__ double lds[kDT];
    __shared__ int sLast;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int strip = blockIdx.x, panel = blockIdx.y;
    const int j0 = (strip * kDT + tid) * VEC;
    double cjv[VEC];
    bool jok[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        jok[e] = j0 + e < A.m;
        cjv[e] = jok[e] ? A.cj[j0 + e] : -__builtin_huge_val();
    }
    float cs[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) cs[e] = 0.0f;
    double cost_acc = 0.0;
    const int i0 = panel * A.rpp;
    const int i1 = min(A.n, i0 + A.rpp);
    for (int ib = i0; ib < i1; ib += kDRows) {
        float cf = 0.0f;                       // this chunk's share of sum P C
#pragma unroll 4
        for (int r = 0; r < kDRows; ++r) {
            const int i = ib + r;
            float rs = 0.0f;
            if (i < i1) {
                float cv[VEC];
                if constexpr (VEC == 4) {
                    if (jok[3]) {
                        const float4_a4 c4 = *reinterpret_cast<const float4_a4 *>(A.C + (size_t)i * A.m + j0);
                        cv[0] = c4.x; cv[1] = c4.y; cv[2] = c4.z; cv[3] = c4.w;
                    } else {                                        // past m, or the last columns of an odd width
#pragma unroll
                        for (int e = 0; e < 4; ++e) cv[e] = jok[e] ? A.C[(size_t)i * A.m + j0 + e] : 0.0f;
                    }
                } else {
                    cv[0] = jok[0] ? A.C[(size_t)i * A.m + j0] : 0.0f;
                }
                const double rv = A.ri[i];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    // log2 of the plan entry; -inf (a zero weight) or NaN becomes -200, whose power of two is 0 in
                    // fp32, so such an entry adds nothing anywhere
                    const float argf = fmaxf((float)fma(-A.s, (double)cv[e], rv + cjv[e]), -200.0f);
                    const float p = fast_exp2(argf);
                    cf = fmaf(p, cv[e], cf);
                    if constexpr (!COST_ONLY) {
                        rs += p;
                        cs[e] += p;
                    }
                }
            }
            if constexpr (!COST_ONLY) {
                rs = wave_sum_f32(rs);
                if (lane == 0) sRow[r][wave] = rs;
            }
        }
        cost_acc += (double)cf;
        if constexpr (!COST_ONLY) {
            __syncthreads();
            if (tid < kDRows && ib + tid < i1) {
                double tot = 0.0;
#pragma unroll
                for (int w = 0; w < kDT / 64; ++w) tot += (double)sRow[tid][w];
                A.rowpart[(size_t)strip * A.n + ib + tid] = tot;
            }
            __syncthreads();
        }
    }
    const size_t w = (size_t)panel * gridDim.x + strip;
    const double c_tot = A.s * block_sum<kDT>(cost_acc, lds);        // sum P (s C), the unit the tail works in
    if constexpr (COST_ONLY) {
        const unsigned int total = gridDim.x * gridDim.y;
        if (tid == 0) agent_store_f64(&A.scal[2 * w], c_tot);
        if (!last_to_arrive(A.ticket, total, &sLast)) return;
        double acc = 0.0;
        for (unsigned int q = tid; q < total; q += kDT) acc += agent_load_f64(&A.scal[2 * (size_t)q]);
        const double tot = block_sum<kDT>(acc, lds);
        if (tid == 0) A.cost_out[0] = tot / A.s;
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            if (jok[e]) A.colpart[(size_t)panel * A.m + j0 + e] = cs[e];
        if (tid == 0) {
            A.scal[2 * w] = c_tot;
            A.scal[2 * w + 1] = 0.0;
        }
    }
}

// ---------------------------------------------------------------- points
struct PointsDiag {
    const double *rows;      // [nr][d] plain coordinates of the row side
    const double *rowq;      // [nr] s |row|^2
    const double *rowlog;    // [nr] ri (or cj): s pot + log2 weight
    const double *cols2s;    // [nc][d] other side times 2s
    const double *colq;      // [nc] s |col|^2
    const double *collog;    // [nc]
    int32_t nr, nc;
    double *part;            // [JS][nr] row sums of this column slice
    double *scal;            // [gridDim.x * JS][2] or null: sum P (s C), (unused)
    int32_t cols_per_split;
    float *colpart;          // d <= 4, everything in one pass: [gridDim.x][nc] column sums of each block of rows
    unsigned int *ticket;    // d <= 4, cost only: arrival counter, and where the last workgroup writes <C, P>
    double *cost_out;
    double s;
};

// d <= 4, on the vector ALUs.  MODE 0: the cost alone (fs_cost).  MODE 1: everything in ONE pass over the
// pairs: row sums are lane-local; the sum of a column over the rows of the workgroup takes 4 DPP additions
// inside each 16-lane row per column and one LDS word per row of lanes, and the 16 words of a column are added
// in a fixed order when the tile is done.  The entropy term needs no sum of its own (see the reduction below).
// A zero weight enters the tile as -1e300 instead of -inf: the exponent still rounds to -inf in fp32 (the plan
// entry is 0) while s C_ij = (s|x|^2 + cl_j) - (cl_j - s|y|^2 + 2 s x.y) stays finite, so no product 0 * inf can
// arise and the loop needs no guards.
template <int D, int MODE, int IB>
__global__ __launch_bounds__(kPT2) void k_diag_points(PointsDiag A) {
    __shared__ __align__(16) double tile[kTile2][D + 2];     // [0] collog - colq, [1..D] 2s y, [D+1] collog
    __shared__ double lds[kPT2];
    __shared__ float sCol[MODE == 1 ? 16 : 1][kTile2];
    __shared__ int sLast;
    const int tid = threadIdx.x;
    double x[IB][D], rc[IB], rq[IB];
    int row[IB];
    double rs[IB];
#pragma unroll
    for (int b = 0; b < IB; ++b) {
        row[b] = (blockIdx.x * IB + b) * kPT2 + tid;
        const bool ok = row[b] < A.nr;
#pragma unroll
        for (int t = 0; t < D; ++t) x[b][t] = ok ? A.rows[(size_t)row[b] * D + t] : 0.0;
        rq[b] = ok ? A.rowq[row[b]] : 0.0;
        rc[b] = ok ? A.rowlog[row[b]] - rq[b] : -__builtin_huge_val();
        rs[b] = 0.0;
    }
    double cost_acc = 0.0;
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);
    for (int jt = j0; jt < j1; jt += kTile2) {
        __syncthreads();
        {
            const int j = jt + tid;
            if (j < j1) {
                const double lg = fmax(A.collog[j], -1.0e300);
                tile[tid][0] = lg - A.colq[j];
#pragma unroll
                for (int t = 0; t < D; ++t) tile[tid][1 + t] = A.cols2s[(size_t)j * D + t];
                tile[tid][D + 1] = lg;
            } else {
                tile[tid][0] = -1.0e300;
#pragma unroll
                for (int t = 0; t < D; ++t) tile[tid][1 + t] = 0.0;
                tile[tid][D + 1] = -1.0e300;
            }
        }
        __syncthreads();
        float rf[IB], cf = 0.0f;
#pragma unroll
        for (int b = 0; b < IB; ++b) rf[b] = 0.0f;
        const int cnt = min(kTile2, (j1 - jt + 1) & ~1);       // staged columns (the tile is padded)
#pragma unroll 2
        for (int jj = 0; jj < cnt; ++jj) {
            double w[D + 2];
#pragma unroll
            for (int t = 0; t < D + 2; ++t) w[t] = tile[jj][t];
            float colsum = 0.0f;
#pragma unroll
            for (int b = 0; b < IB; ++b) {
                double tq = w[0];                                                  // collog - colq + 2 s x.y
#pragma unroll
                for (int t = 0; t < D; ++t) tq = fma(x[b][t], w[1 + t], tq);
                const float argf = fmaxf((float)(tq + rc[b]), -200.0f);            // -inf, NaN: the entry is 0
                const float p = fast_exp2(argf);
                const double sc = (rq[b] + w[D + 1]) - tq;                         // s |x - y|^2, w[D+1] = collog
                cf = fmaf(p, (float)sc, cf);
                if (MODE == 1) {
                    rf[b] += p;
                    colsum += p;
                }
            }
            if (MODE == 1) {
                colsum += dpp_f32<0x128>(colsum);
                colsum += dpp_f32<0x124>(colsum);
                colsum += dpp_f32<0x122>(colsum);
                colsum += dpp_f32<0x121>(colsum);
                if ((tid & 15) == 0) sCol[tid >> 4][jj] = colsum;
            }
        }
#pragma unroll
        for (int b = 0; b < IB; ++b) rs[b] += (double)rf[b];
        cost_acc += (double)cf;
        if (MODE == 1) {
            __syncthreads();
            if (tid < cnt && jt + tid < j1) {
                double tot = 0.0;
#pragma unroll
                for (int q = 0; q < 16; ++q) tot += (double)sCol[q][tid];
                A.colpart[(size_t)blockIdx.x * A.nc + jt + tid] = (float)tot;
            }
        }
    }
    if (MODE == 1) {
#pragma unroll
        for (int b = 0; b < IB; ++b)
            if (row[b] < A.nr) A.part[(size_t)blockIdx.y * A.nr + row[b]] = rs[b];
    }
    const double c_tot = block_sum<kPT2>(cost_acc, lds);
    const size_t w = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
    if (MODE == 1) {
        if (tid == 0) {
            A.scal[2 * w] = c_tot;
            A.scal[2 * w + 1] = 0.0;
        }
    } else {                                   // the workgroup that arrives last finishes the call
        const unsigned int total = gridDim.x * gridDim.y;
        if (tid == 0) agent_store_f64(&A.scal[2 * w], c_tot);
        if (!last_to_arrive(A.ticket, total, &sLast)) return;
        double acc = 0.0;
        for (unsigned int q = tid; q < total; q += kPT2) acc += agent_load_f64(&A.scal[2 * (size_t)q]);
        const double tot = block_sum<kPT2>(acc, lds);
        if (tid == 0) A.cost_out[0] = tot / A.s;
    }
}

// More than 4 coordinates: the dot products run on the fp64 matrix cores (fs_mfma.h).  The accumulator
// starts at (cj_j - s|y_j|^2) + (ri_i - s|x_i|^2), so the matrix core delivers log2 P_ij itself.
template <int D4, bool WITH_COST>
__global__ __launch_bounds__(256) void k_diag_points_mfma(PointsDiag A, int d) {
    __shared__ double tile[kTileJ][4 * D4 + 1];
    __shared__ double tw[kTileJ], tcl[kTileJ];
    __shared__ double lds[256];
    const int tid = threadIdx.x, lj = tid & 15;
    RowTiles<D4> R;
    R.load(A.rows, A.nr, d);
    double rc[kTileRT][4], rlog[kTileRT][4], rs[kTileRT][4];
    float rf[kTileRT][4];
#pragma unroll
    for (int rt = 0; rt < kTileRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = R.result_row(rt, r);
            const bool ok = row < A.nr;
            rlog[rt][r] = ok ? A.rowlog[row] : -__builtin_huge_val();
            rc[rt][r] = ok ? rlog[rt][r] - A.rowq[row] : -__builtin_huge_val();
            rs[rt][r] = 0.0;
            rf[rt][r] = 0.0f;
        }
    double cost_acc = 0.0, ent_acc = 0.0;
    float cf = 0.0f, ef = 0.0f;
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);
    mfma_walk<D4>(
        R, tile, A.cols2s, d, j0, j1,
        [&](int jt) {
            if (tid < kTileJ) {
                const int j = jt + tid;
                const double lg = j < j1 ? A.collog[j] : -__builtin_huge_val();
                tw[tid] = j < j1 ? lg - A.colq[j] : -__builtin_huge_val();
                tcl[tid] = lg;
            }
        },
        [&](int ct, int rt, int r) { return tw[ct * 16 + lj] + rc[rt][r]; },
        [&](int, int ct, int rt, const double4_m &acc) {
            const double cl = tcl[ct * 16 + lj];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const double arg = acc[r];
                const float argf = (float)arg;
                float p = fast_exp2(argf);
                p = p > 0.0f ? p : 0.0f;                                   // drops NaN
                rf[rt][r] += p;
                if (WITH_COST) {
                    const double sc = (rlog[rt][r] + cl) - arg;              // s |x - y|^2
                    cf = fmaf(p, fminf((float)sc, 1.0e30f), cf);             // 0 * inf (or NaN) must stay 0
                    ef = fmaf(p, fmaxf(argf, -1.0e30f), ef);
                }
            }
            if (ct == kTileJ / 16 - 1) {                                    // fp32 sums span one LDS tile
#pragma unroll
                for (int r = 0; r < 4; ++r) { rs[rt][r] += (double)rf[rt][r]; rf[rt][r] = 0.0f; }
                if (rt == kTileRT - 1) { cost_acc += (double)cf; ent_acc += (double)ef; cf = 0.0f; ef = 0.0f; }
            }
        });
#pragma unroll
    for (int rt = 0; rt < kTileRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const double tot = row16_sum(rs[rt][r]);
            const int row = R.result_row(rt, r);
            if (lj == 0 && row < A.nr) A.part[(size_t)blockIdx.y * A.nr + row] = tot;
        }
    if (WITH_COST) {
        const double c_tot = block_sum<256>(cost_acc, lds);
        const double e_tot = block_sum<256>(ent_acc, lds);
        if (tid == 0) {
            const size_t w = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
            A.scal[2 * w] = c_tot;
            A.scal[2 * w + 1] = e_tot;
        }
    }
}

// out[0] cost, [1] mass, [2] KL(P | a x b), [3] primal, [4] dual, [5] row-marginal L1 error,
// [6] column-marginal L1 error, [7] 0.  Called by all T threads of one workgroup: per-thread shares in index
// order, wave sums by DPP, then the waves one after the other, so the order of the additions is fixed.
template <int T>
__device__ __forceinline__ void diag_totals(const double *red, int nred, const double *scal, int nscal, double s,
                                            double *out, double *cost_out, double *lds, bool agent_loads) {
    double w9[9];
    for (int q = 0; q < 7; ++q) {
        double acc = 0.0;
        for (int w = threadIdx.x; w < nred; w += T)
            acc += agent_loads ? agent_load_f64(&red[(size_t)w * 8 + q]) : red[(size_t)w * 8 + q];
        w9[q] = acc;
    }
    for (int q = 0; q < 2; ++q) {
        double acc = 0.0;
        for (int w = threadIdx.x; w < nscal; w += T) acc += scal[(size_t)w * 2 + q];   // written by an earlier launch
        w9[7 + q] = acc;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < 9; ++q) {
        const double t = wave_sum_f64(w9[q]);
        if (lane == 0) lds[wave * 9 + q] = t;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double v[7], sc[2];
#pragma unroll
        for (int q = 0; q < 9; ++q) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < T / 64; ++w) t += lds[w * 9 + q];
            if (q < 7) v[q] = t;
            else sc[q - 7] = t;
        }
        const double eps = 1.4426950408889634074 / s;
        const double mass = v[0];
        const double cost = sc[0] / s;
        const double plogp = (v[5] + v[6] - cost) / eps;         // sum P log(P/(a b)) = (<r,f> + <c,g> - <C,P>)/eps
        const double kl = plogp - mass + 1.0;
        if (out) {
            out[0] = cost;
            out[1] = mass;
            out[2] = kl;
            out[3] = cost + eps * kl;
            out[4] = v[3] + v[4] - eps * mass + eps;
            out[5] = v[1];
            out[6] = v[2];
            out[7] = 0.0;
        }
        if (cost_out) cost_out[0] = cost;
    }
}

// ---------------------------------------------------------------- reduction of the partials
// Entry t = row t and column t: marginals, their L1 errors, <a,f>, <b,g>, and the sums
// r_i log2 a_i, c_j log2 b_j.  One record of 8 doubles per workgroup.
struct ReduceArgs {
    PlanArgs P;
    const double *rowpart; int32_t nrowpart;      // [nrowpart][n]
    const void *colpart; int32_t ncolpart;        // [ncolpart][m], float (dense) or double (points)
    int32_t colpart_is_float;
    double *row_marg, *col_marg;                  // optional outputs
    double *red;                                  // [gridDim.x][8]
    // the tail: the workgroup that arrives last adds the records of all workgroups and the per-workgroup sums of
    // the pass (scal) in index order and writes the results
    const double *scal; int32_t nscal;
    unsigned int *ticket;
    double *out8, *cost_out;
};

// A workgroup of 1024 threads finishes 64 rows and 64 columns: lane = entry, the 16 waves split the
// partial sets (8 loads in flight each) and meet in LDS.
constexpr int kRW = 16;             // waves of the reduction kernel
__global__ __launch_bounds__(kRW * 64) void k_diag_reduce(ReduceArgs A) {
    __shared__ double sR[kRW][64], sC[kRW][64];
    __shared__ double lds9[kRW * 9];
    __shared__ int sLast;
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int t = blockIdx.x * 64 + lane;
    double r = 0.0, c = 0.0;
    // partial sets grp, grp + 16, ...: eight loads in flight, added in index order
    auto gather = [&](auto ptr, int nsets, int ld) -> double {
        double acc = 0.0;
        int q = grp;
        for (; q + 7 * kRW < nsets; q += 8 * kRW) {
            double x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = (double)ptr[(size_t)(q + kRW * u) * ld + t];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += x[u];
        }
        for (; q < nsets; q += kRW) acc += (double)ptr[(size_t)q * ld + t];
        return acc;
    };
    if (t < A.P.n) r = gather(A.rowpart, A.nrowpart, A.P.n);
    if (t < A.P.m) {
        if (A.colpart_is_float) c = gather((const float *)A.colpart, A.ncolpart, A.P.m);
        else c = gather((const double *)A.colpart, A.ncolpart, A.P.m);
    }
    sR[grp][lane] = r;
    sC[grp][lane] = c;
    __syncthreads();
    double v[7] = {0, 0, 0, 0, 0, 0, 0};          // mass, row err, col err, <a,f>, <b,g>, <r,f>, <c,g>
    if (grp == 0) {
        r = 0.0;
        c = 0.0;
#pragma unroll
        for (int w = 0; w < kRW; ++w) { r += sR[w][lane]; c += sC[w][lane]; }
        if (t < A.P.n) {
            const float a = A.P.a[t];
            if (A.row_marg) A.row_marg[t] = r;
            v[0] = r;
            v[1] = fabs(r - (double)a);
            const double f = A.P.f64 ? A.P.f64[t] : (double)A.P.f[t];
            if (a > 0.0f) v[3] = (double)a * f;
            if (r > 0.0) v[5] = r * f;
        }
        if (t < A.P.m) {
            const float b = A.P.b[t];
            if (A.col_marg) A.col_marg[t] = c;
            v[2] = fabs(c - (double)b);
            const double g = A.P.g64 ? A.P.g64[t] : (double)A.P.g[t];
            if (b > 0.0f) v[4] = (double)b * g;
            if (c > 0.0) v[6] = c * g;
        }
#pragma unroll
        for (int q = 0; q < 7; ++q) {
            const double tot = wave_sum_f64(v[q]);
            if (lane == 0) agent_store_f64(&A.red[(size_t)blockIdx.x * 8 + q], tot);
        }
    }
    __syncthreads();                                  // (thread 0 is lane 0 of the wave that stored the record)
    if (!last_to_arrive(A.ticket, gridDim.x, &sLast)) return;
    diag_totals<kRW * 64>(A.red, (int)gridDim.x, A.scal, A.nscal, A.P.s, A.out8, A.cost_out, lds9, /*agent_loads=*/true);
}

// ---------------------------------------------------------------- small problems: everything in one workgroup
// n, m <= 1024 and at most 2^14 entries (point clouds, d <= 4: 2^16 pairs): one launch instead of four or
// five.  One compute unit evaluates about 1.4 entries per ns on these two sweeps, so beyond those sizes the
// multi-kernel path (26 us dense, 47 - 80 us point clouds, whatever the size) is as fast or faster.  1024 lanes
// as a 32 x 32 grid.  First sweep: lane (tr, tc) walks the entries (tr + 32 a, tc + 32 b); what belongs to a row
// meets in the 32 lanes of a half-wave (DPP + one swizzle).  Second sweep: the same with the roles of rows
// and columns exchanged, for the column marginals.  All sums in a fixed order.
constexpr int kOneMax = 1024;
constexpr int kOneEntries = 1 << 14, kOnePairs = 1 << 16;

__device__ __forceinline__ double half_sum(double v) {          // all-reduce over a half-wave (32 lanes)
    v += dpp_f64<0x128>(v);
    v += dpp_f64<0x124>(v);
    v += dpp_f64<0x122>(v);
    v += dpp_f64<0x121>(v);
    v += swz16_f64(v);
    return v;
}

struct OneArgs {
    PlanArgs P;
    double *row_marg, *col_marg;                  // optional outputs
    double *out8, *cost_out;                      // either may be null
};

template <bool PTS>
__global__ __launch_bounds__(1024) void k_diag_one(OneArgs A) {
    __shared__ double sRi[kOneMax], sCj[kOneMax], sLa[kOneMax], sLb[kOneMax];
    __shared__ double sXq[PTS ? kOneMax : 1], sYq[PTS ? kOneMax : 1];
    __shared__ double sX[PTS ? kOneMax * 4 : 1], sY[PTS ? kOneMax * 4 : 1];      // plain x; 2 s y
    __shared__ double lds[1024];
    const PlanArgs &P = A.P;
    const int n = P.n, m = P.m, d = P.d;
    const int tid = threadIdx.x, tc = tid & 31, tr = tid >> 5;
    const double s = P.s;
    const double ninf = -__builtin_huge_val();
    // ---- per-row and per-column constants
    {
        const int t = tid;
        double la = ninf, lb = ninf;
        if (t < n) {
            la = log2_weight(P.a[t]);
            sRi[t] = fma(s, P.f64 ? P.f64[t] : (double)P.f[t], la);
            if constexpr (PTS) {
                double sq = 0.0;
                for (int q = 0; q < 4; ++q) {
                    const double x = q < d ? (double)P.X[(size_t)t * d + q] : 0.0;
                    sX[t * 4 + q] = x;
                    sq = fma(x, x, sq);
                }
                sXq[t] = s * sq;
            }
        }
        if (t < m) {
            lb = log2_weight(P.b[t]);
            sCj[t] = fma(s, P.g64 ? P.g64[t] : (double)P.g[t], lb);
            if constexpr (PTS) {
                double sq = 0.0;
                for (int q = 0; q < 4; ++q) {
                    const double y = q < d ? (double)P.Y[(size_t)t * d + q] : 0.0;
                    sY[t * 4 + q] = 2.0 * s * y;
                    sq = fma(y, y, sq);
                }
                sYq[t] = s * sq;
            }
        }
        sLa[t] = la;
        sLb[t] = lb;
    }
    __syncthreads();
    // s C_ij of entry (i, j)
    auto scaled_cost = [&](int i, int j) -> double {
        if constexpr (PTS) {
            double dot = 0.0;
#pragma unroll
            for (int q = 0; q < 4; ++q) dot = fma(sX[i * 4 + q], sY[j * 4 + q], dot);
            return sXq[i] + sYq[j] - dot;
        } else {
            return s * (double)P.C[(size_t)i * m + j];
        }
    };
    // ---- first sweep: rows.  v[0] mass, [1] row error, [3] <a, f>, [5] r . log2 a; cost and sum P e
    double v[7] = {0, 0, 0, 0, 0, 0, 0};
    double cost_acc = 0.0, ent_acc = 0.0;
    for (int i = tr; i < n; i += 32) {
        const double ri = sRi[i];
        float rf = 0.0f, cf = 0.0f, ef = 0.0f;
#pragma unroll 8
        for (int j = tc; j < m; j += 32) {
            const double sc = scaled_cost(i, j);
            const float e = (float)(ri + sCj[j] - sc);
            float p = fast_exp2(e);
            p = p > 0.0f ? p : 0.0f;                               // drops NaN
            rf += p;
            cf = fmaf(p, (float)sc, cf);
            ef += p > 0.0f ? p * e : 0.0f;
        }
        const double r = half_sum((double)rf);
        cost_acc += (double)cf;
        ent_acc += (double)ef;
        if (tc == 0) {
            const float a = P.a[i];
            if (A.row_marg) A.row_marg[i] = r;
            v[0] += r;
            v[1] += fabs(r - (double)a);
            if (a > 0.0f) {
                v[3] += (double)a * (P.f64 ? P.f64[i] : (double)P.f[i]);
                v[5] += r * sLa[i];
            }
        }
    }
    // ---- second sweep: columns (lane (tr, tc) walks the entries (tc + 32 a, tr + 32 b))
    for (int j = tr; j < m; j += 32) {
        const double cj = sCj[j];
        float cs = 0.0f;
#pragma unroll 8
        for (int i = tc; i < n; i += 32) {
            float p = fast_exp2((float)(sRi[i] + cj - scaled_cost(i, j)));
            cs += p > 0.0f ? p : 0.0f;
        }
        const double c = half_sum((double)cs);
        if (tc == 0) {
            const float b = P.b[j];
            if (A.col_marg) A.col_marg[j] = c;
            v[2] += fabs(c - (double)b);
            if (b > 0.0f) {
                v[4] += (double)b * (P.g64 ? P.g64[j] : (double)P.g[j]);
                v[6] += c * sLb[j];
            }
        }
    }
    // ---- totals in a fixed order (wave sums by DPP, then the 16 waves one after the other) and the outputs
    {
        const int lane = tid & 63, wave = tid >> 6;
        double w9[9] = {v[0], v[1], v[2], v[3], v[4], v[5], v[6], cost_acc, ent_acc};
#pragma unroll
        for (int q = 0; q < 9; ++q) {
            const double t = wave_sum_f64(w9[q]);
            if (lane == 0) lds[wave * 9 + q] = t;
        }
    }
    __syncthreads();
    double tot[9];
    if (tid == 0) {
#pragma unroll
        for (int q = 0; q < 9; ++q) {
            double t = 0.0;
            for (int w = 0; w < 16; ++w) t += lds[w * 9 + q];
            tot[q] = t;
        }
    }
    if (tid == 0) {
        const double eps = 1.4426950408889634074 / s;
        const double mass = tot[0];
        const double cost = tot[7] / s;
        const double plogp = kLn2d * (tot[8] - tot[5] - tot[6]);     // sum P log(P/(a b))
        const double kl = plogp - mass + 1.0;
        if (A.out8) {
            A.out8[0] = cost;
            A.out8[1] = mass;
            A.out8[2] = kl;
            A.out8[3] = cost + eps * kl;
            A.out8[4] = tot[3] + tot[4] - eps * mass + eps;
            A.out8[5] = tot[1];
            A.out8[6] = tot[2];
            A.out8[7] = 0.0;
        }
        if (A.cost_out) A.cost_out[0] = cost;
    }
}

}  // namespace

size_t diag_scratch_bytes(int n, int m, int d) { return diag_layout(n, m, d).total; }

// cost_only_out non-null: only the cost is wanted (out8 may be null; the pass that exists only for the
// column marginals of a point-cloud problem is skipped).
hipError_t launch_plan_prep_all(hipStream_t st, const PlanArgs &a, double *ri, double *cj, double *xp, double *xs,
                                double *xq, double *yp, double *ys, double *yq) {
    const int len = a.n > a.m ? a.n : a.m;
    hipLaunchKernelGGL(k_diag_prep, dim3((len + 255) / 256), dim3(256), 0, st, a, ri, cj, xp, xs, xq, yp, ys, yq);
    return hipGetLastError();
}

hipError_t launch_diag(hipStream_t st, const PlanArgs &a, double *out8, double *row_marg, double *col_marg,
                       void *scratch, size_t scratch_bytes, unsigned int *tickets, double *cost_only_out) {
    if (!tickets) return hipErrorInvalidValue;
    if (a.n <= kOneMax && a.m <= kOneMax && a.d <= 4 &&
        (size_t)a.n * (size_t)a.m <= (size_t)(a.d > 0 ? kOnePairs : kOneEntries)) {
        OneArgs O{};
        O.P = a; O.row_marg = row_marg; O.col_marg = col_marg; O.out8 = out8; O.cost_out = cost_only_out;
        if (a.d > 0) hipLaunchKernelGGL(k_diag_one<true>, dim3(1), dim3(1024), 0, st, O);
        else hipLaunchKernelGGL(k_diag_one<false>, dim3(1), dim3(1024), 0, st, O);
        return hipGetLastError();
    }
    const DiagLayout L = diag_layout(a.n, a.m, a.d);
    if (scratch_bytes < L.total) return hipErrorInvalidValue;
    unsigned char *ws = (unsigned char *)scratch;
    const bool cost_only = cost_only_out != nullptr;
    double *ri = (double *)(ws + L.o_ri), *cj = (double *)(ws + L.o_cj);
    const int len = a.n > a.m ? a.n : a.m;
    double *xp = nullptr, *xs = nullptr, *xq = nullptr, *yp = nullptr, *ys = nullptr, *yq = nullptr;
    if (a.d > 0) {
        xp = (double *)(ws + L.o_xp); xs = (double *)(ws + L.o_xs); xq = (double *)(ws + L.o_xq);
        yp = (double *)(ws + L.o_yp); ys = (double *)(ws + L.o_ys); yq = (double *)(ws + L.o_yq);
    }
    hipLaunchKernelGGL(k_diag_prep, dim3((len + 255) / 256), dim3(256), 0, st, a, ri, cj, xp, xs, xq, yp, ys, yq);
    ReduceArgs R{};
    R.P = a;
    R.row_marg = row_marg; R.col_marg = col_marg;
    R.red = (double *)(ws + L.o_red);
    double *scal = (double *)(ws + L.o_scal);
    if (a.d == 0) {
        DenseDiag D{};
        D.C = a.C; D.ri = ri; D.cj = cj; D.n = a.n; D.m = a.m; D.s = a.s;
        D.rowpart = (double *)(ws + L.o_rowpart);
        D.colpart = (float *)(ws + L.o_colpart);
        D.scal = scal; D.rpp = L.rpp;
        D.ticket = tickets; D.cost_out = cost_only_out;
        const dim3 grid(L.nstrips, L.P);
        if (cost_only) {                        // the pass finishes the call itself
            if (L.vec == 4) hipLaunchKernelGGL((k_diag_dense<4, true>), grid, dim3(kDT), 0, st, D);
            else hipLaunchKernelGGL((k_diag_dense<1, true>), grid, dim3(kDT), 0, st, D);
            return hipGetLastError();
        }
        if (L.vec == 4) hipLaunchKernelGGL((k_diag_dense<4, false>), grid, dim3(kDT), 0, st, D);
        else hipLaunchKernelGGL((k_diag_dense<1, false>), grid, dim3(kDT), 0, st, D);
        R.rowpart = D.rowpart; R.nrowpart = L.nstrips;
        R.colpart = D.colpart; R.ncolpart = L.P; R.colpart_is_float = 1;
    } else {
        PointsDiag X{};                         // rows = x side: row marginals, cost, entropy
        X.rows = xp; X.rowq = xq; X.rowlog = ri; X.cols2s = ys; X.colq = yq; X.collog = cj;
        X.nr = a.n; X.nc = a.m; X.part = (double *)(ws + L.o_rowpart); X.scal = scal; X.cols_per_split = L.cpsx;
        PointsDiag Y{};                         // rows = y side: column marginals only
        Y.rows = yp; Y.rowq = yq; Y.rowlog = cj; Y.cols2s = xs; Y.colq = xq; Y.collog = ri;
        Y.nr = a.m; Y.nc = a.n; Y.part = (double *)(ws + L.o_colpart); Y.scal = nullptr; Y.cols_per_split = L.cpsy;
        if (a.d <= 4) {
            if (L.ibx != 1 && L.ibx != kIB2) return hipErrorInvalidValue;
            const dim3 gx((a.n + kPT2 * L.ibx - 1) / (kPT2 * L.ibx), L.JSx);
            X.colpart = (float *)(ws + L.o_colpart);
            X.ticket = tickets; X.cost_out = cost_only_out; X.s = a.s;
#define FS_DIAG_PTS(D)                                                                                       \
    do {                                                                                                     \
        if (cost_only) {                                                                                     \
            if (L.ibx == 1) hipLaunchKernelGGL((k_diag_points<D, 0, 1>), gx, dim3(kPT2), 0, st, X);          \
            else hipLaunchKernelGGL((k_diag_points<D, 0, kIB2>), gx, dim3(kPT2), 0, st, X);                  \
        } else {                                                                                             \
            if (L.ibx == 1) hipLaunchKernelGGL((k_diag_points<D, 1, 1>), gx, dim3(kPT2), 0, st, X);          \
            else hipLaunchKernelGGL((k_diag_points<D, 1, kIB2>), gx, dim3(kPT2), 0, st, X);                  \
        }                                                                                                    \
    } while (0)
            switch (a.d) {
                case 1: FS_DIAG_PTS(1); break;
                case 2: FS_DIAG_PTS(2); break;
                case 3: FS_DIAG_PTS(3); break;
                default: FS_DIAG_PTS(4); break;
            }
#undef FS_DIAG_PTS
            if (cost_only) return hipGetLastError();      // the pass has written the cost itself
            R.rowpart = X.part; R.nrowpart = L.JSx;
            R.colpart = X.colpart; R.ncolpart = (int)gx.x; R.colpart_is_float = 1;
        } else {
            const dim3 gx((a.n + kTileRows - 1) / kTileRows, L.JSx), gy((a.m + kTileRows - 1) / kTileRows, L.JSy);
#define FS_DIAG_MFMA(D4)                                                                                   \
    do {                                                                                                    \
        hipLaunchKernelGGL((k_diag_points_mfma<D4, true>), gx, dim3(256), 0, st, X, a.d);                  \
        if (!cost_only) hipLaunchKernelGGL((k_diag_points_mfma<D4, false>), gy, dim3(256), 0, st, Y, a.d); \
    } while (0)
            switch (mfma_d4(a.d)) {
                case 2: FS_DIAG_MFMA(2); break;
                case 4: FS_DIAG_MFMA(4); break;
                case 8: FS_DIAG_MFMA(8); break;
                default: FS_DIAG_MFMA(16); break;
            }
#undef FS_DIAG_MFMA
            R.rowpart = X.part; R.nrowpart = L.JSx;
            R.colpart = Y.part; R.ncolpart = cost_only ? 0 : L.JSy; R.colpart_is_float = 0;
        }
    }
    R.scal = scal; R.nscal = L.nscal;
    R.ticket = tickets + 1;
    R.out8 = out8; R.cost_out = cost_only_out;
    hipLaunchKernelGGL(k_diag_reduce, dim3(L.nred), dim3(kRW * 64), 0, st, R);
    return hipGetLastError();
}

}  // namespace fs
