// Plan (Eq. 5) and transport cost (last step of Alg. 1) from given potentials.
//
//   P_ij = a_i b_j exp((f_i + g_j - C_ij)/eps) = 2^( ri_i + cj_j - s C_ij ),
//   ri_i = s f_i + log2 a_i,  cj_j = s g_j + log2 b_j,  s = log2(e)/eps.
//
// ri, cj are prepared once in fp64; the exponent is formed in fp64 and rounded
// to fp32 only for v_exp_f32.  The cost is accumulated in fp64 per workgroup
// and the per-workgroup partials are summed in index order by one workgroup.
#include "fs_kernels.h"
#include "fs_mfma.h"

namespace fs {

__global__ __launch_bounds__(256) void k_plan_prep(PlanArgs A, double *ri, double *cj) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < A.n) {
        const double f = A.f64 ? A.f64[t] : (double)A.f[t];
        ri[t] = fma(A.s, f, log2_weight(A.a[t]));
    }
    if (t < A.m) {
        const double g = A.g64 ? A.g64[t] : (double)A.g[t];
        cj[t] = fma(A.s, g, log2_weight(A.b[t]));
    }
}

__device__ __forceinline__ double cost_entry(const PlanArgs &A, int i, int j) {
    if (A.C) return (double)A.C[(size_t)i * A.m + j];
    double sq = 0.0;
    for (int t = 0; t < A.d; ++t) {
        const double df = (double)A.X[(size_t)i * A.d + t] - (double)A.Y[(size_t)j * A.d + t];
        sq = fma(df, df, sq);
    }
    return sq;
}

// grid.x covers columns (256 per workgroup), grid.y strides over rows.
template <bool WRITE_PLAN>
__global__ __launch_bounds__(256) void k_plan_cost(PlanArgs A, const double *ri, const double *cj, float *P,
                                                   double *partial) {
    __shared__ double lds[256];
    const int j = blockIdx.x * 256 + threadIdx.x;
    const bool jok = j < A.m;
    const double cjv = jok ? cj[j] : 0.0;
    double acc = 0.0;
    for (int i = blockIdx.y; i < A.n; i += gridDim.y) {
        if (jok) {
            const double cst = cost_entry(A, i, j);
            const double e = ri[i] + cjv - A.s * cst;
            const float pij = fast_exp2((float)e);
            if (WRITE_PLAN) P[(size_t)i * A.m + j] = pij;
            else if (pij > 0.0f) acc = fma(cst, (double)pij, acc);
        }
    }
    if (!WRITE_PLAN) {
        lds[threadIdx.x] = acc;
        __syncthreads();
        for (int w = 128; w >= 1; w >>= 1) {
            if ((int)threadIdx.x < w) lds[threadIdx.x] += lds[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) partial[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = lds[0];
    }
}

// Dense plan: every lane owns 4 adjacent columns (16-byte loads of C, 16-byte streaming stores of P, at
// whatever 4-byte boundary the row starts), four rows in flight; the lane that owns the last columns
// of a width that is not a multiple of 4 works element by element.
__global__ __launch_bounds__(256) void k_plan_dense4(PlanArgs A, const double *ri, const double *cj, float *P) {
    const int j = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (j >= A.m) return;
    const int valid = A.m - j < 4 ? A.m - j : 4;
    double cjv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) cjv[e] = e < valid ? cj[j + e] : 0.0;
    const double ns = -A.s;
    for (int i0 = blockIdx.y * 4; i0 < A.n; i0 += gridDim.y * 4) {
        float c[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (i0 + r < A.n) {
                const float *src = A.C + (size_t)(i0 + r) * A.m + j;
                if (valid == 4) {
                    const float4_a4 v = *reinterpret_cast<const float4_a4 *>(src);
                    c[r][0] = v.x; c[r][1] = v.y; c[r][2] = v.z; c[r][3] = v.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) c[r][e] = e < valid ? src[e] : 0.0f;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (i0 + r < A.n) {
                const double rv = ri[i0 + r];
                float p[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) p[e] = fast_exp2((float)(fma(ns, (double)c[r][e], rv + cjv[e])));
                float *dst = P + (size_t)(i0 + r) * A.m + j;
                if (valid == 4) {
                    float4_a4 v;
                    v.x = p[0]; v.y = p[1]; v.z = p[2]; v.w = p[3];
                    __builtin_nontemporal_store(v, reinterpret_cast<float4_a4 *>(dst));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (e < valid) dst[e] = p[e];
                }
            }
        }
    }
}

// Plan of a point-cloud problem: 16 x 16 tiles of exponents from the fp64 matrix cores (fs_mfma.h; d <= 4
// is padded to one instruction), written as they come: result register r of lane l is entry
// (row l / 16 + 4 r, col l % 16), so every store instruction writes four 64-byte row segments.
struct PlanPoints {
    const double *rows, *rowq, *rowlog;     // x side: plain coordinates, s|x|^2, ri
    const double *cols2s, *colq, *collog;   // y side: 2 s y, s|y|^2, cj
    int32_t nr, nc;
    float *P;
    int32_t cols_per_split;
};

template <int D4>
__global__ __launch_bounds__(256) void k_plan_points_mfma(PlanPoints A, int d) {
    __shared__ double tile[kTileJ][4 * D4 + 1];
    __shared__ double tw[kTileJ];
    const int tid = threadIdx.x, lj = tid & 15;
    RowTiles<D4> R;
    R.load(A.rows, A.nr, d);
    double rc[kTileRT][4];
#pragma unroll
    for (int rt = 0; rt < kTileRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = R.result_row(rt, r);
            rc[rt][r] = row < A.nr ? A.rowlog[row] - A.rowq[row] : -__builtin_huge_val();
        }
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);
    mfma_walk<D4>(
        R, tile, A.cols2s, d, j0, j1,
        [&](int jt) {
            if (tid < kTileJ) {
                const int j = jt + tid;
                tw[tid] = j < j1 ? A.collog[j] - A.colq[j] : -__builtin_huge_val();
            }
        },
        [&](int ct, int rt, int r) { return tw[ct * 16 + lj] + rc[rt][r]; },
        [&](int jt, int ct, int rt, const double4_m &acc) {
            const int j = jt + ct * 16 + lj;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = R.result_row(rt, r);
                if (row < A.nr && j < j1) A.P[(size_t)row * A.nc + j] = fast_exp2((float)acc[r]);
            }
        });
}

__global__ __launch_bounds__(256) void k_sum_partials(const double *partial, int count, double *out) {
    __shared__ double lds[256];
    double acc = 0.0;
    for (int q = threadIdx.x; q < count; q += 256) acc += partial[q];
    lds[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) lds[threadIdx.x] += lds[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = lds[0];
}

static void plan_grid(int n, int m, dim3 *grid) {
    const int gx = (m + 255) / 256;
    int gy = (4096 + gx - 1) / gx;
    if (gy > n) gy = n;
    if (gy < 1) gy = 1;
    if (gy > 65535) gy = 65535;
    *grid = dim3(gx, gy);
}

int cost_scratch_len(int n, int m) {
    dim3 g;
    plan_grid(n, m, &g);
    return n + m + (int)(g.x * g.y);          // ri, cj, partials
}

hipError_t launch_cost(hipStream_t st, const PlanArgs &a, double *cost_dev, double *scratch, int nscratch) {
    dim3 grid;
    plan_grid(a.n, a.m, &grid);
    if (nscratch < a.n + a.m + (int)(grid.x * grid.y)) return hipErrorInvalidValue;
    double *ri = scratch, *cj = scratch + a.n, *partial = scratch + a.n + a.m;
    const int len = a.n > a.m ? a.n : a.m;
    hipLaunchKernelGGL(k_plan_prep, dim3((len + 255) / 256), dim3(256), 0, st, a, ri, cj);
    if (cost_dev) {
        hipLaunchKernelGGL(k_plan_cost<false>, grid, dim3(256), 0, st, a, ri, cj, (float *)nullptr, partial);
        hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(256), 0, st, partial, (int)(grid.x * grid.y), cost_dev);
    }
    return hipGetLastError();
}

int plan_scratch_len(int n, int m, int d) {
    return d > 0 ? n + m + (n + m) * (2 * d + 1) : cost_scratch_len(n, m);
}

hipError_t launch_plan(hipStream_t st, const PlanArgs &a, float *P, double *scratch, int nscratch) {
    dim3 grid;
    plan_grid(a.n, a.m, &grid);
    if (nscratch < plan_scratch_len(a.n, a.m, a.d)) return hipErrorInvalidValue;
    double *ri = scratch, *cj = scratch + a.n;
    const int len = a.n > a.m ? a.n : a.m;
    if (a.d > 0) {
        // point clouds: repacked clouds after ri, cj; tiles of the plan from the matrix cores
        double *xp = cj + a.m, *xs = xp + (size_t)a.n * a.d, *xq = xs + (size_t)a.n * a.d;
        double *yp = xq + a.n, *ys = yp + (size_t)a.m * a.d, *yq = ys + (size_t)a.m * a.d;
        hipError_t e = launch_plan_prep_all(st, a, ri, cj, xp, xs, xq, yp, ys, yq);
        if (e != hipSuccess) return e;
        PlanPoints pp{};
        pp.rows = xp; pp.rowq = xq; pp.rowlog = ri; pp.cols2s = ys; pp.colq = yq; pp.collog = cj;
        pp.nr = a.n; pp.nc = a.m; pp.P = P; pp.cols_per_split = 2048;
        const dim3 g2((a.n + kTileRows - 1) / kTileRows, (a.m + 2047) / 2048);
        switch (mfma_d4(a.d)) {
            case 1: hipLaunchKernelGGL(k_plan_points_mfma<1>, g2, dim3(256), 0, st, pp, a.d); break;
            case 2: hipLaunchKernelGGL(k_plan_points_mfma<2>, g2, dim3(256), 0, st, pp, a.d); break;
            case 4: hipLaunchKernelGGL(k_plan_points_mfma<4>, g2, dim3(256), 0, st, pp, a.d); break;
            case 8: hipLaunchKernelGGL(k_plan_points_mfma<8>, g2, dim3(256), 0, st, pp, a.d); break;
            default: hipLaunchKernelGGL(k_plan_points_mfma<16>, g2, dim3(256), 0, st, pp, a.d); break;
        }
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_plan_prep, dim3((len + 255) / 256), dim3(256), 0, st, a, ri, cj);
    if (a.C && a.m >= 4) {
        const int gx = ((a.m + 3) / 4 + 255) / 256;
        int gy = (2048 + gx - 1) / gx;
        if (gy > (a.n + 3) / 4) gy = (a.n + 3) / 4;
        hipLaunchKernelGGL(k_plan_dense4, dim3(gx, gy), dim3(256), 0, st, a, ri, cj, P);
    } else {
        hipLaunchKernelGGL(k_plan_cost<true>, grid, dim3(256), 0, st, a, ri, cj, P, (double *)nullptr);
    }
    return hipGetLastError();
}

}  // namespace fs
