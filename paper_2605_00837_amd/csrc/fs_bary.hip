// Barycentric mapping of the plan of Eq. 5 (the "barycentric mapping" of Sec. 5.6):
//   T[i][t] = sum_j P_ij Z[j][t] / sum_j P_ij,   t < dz <= 4,
// computed in one pass over C (or over all point pairs) without ever storing P.  Rows without mass
// give 0.  Layouts as in the diagnostics pass: dense = 1024 lanes own a strip of columns and walk
// down a panel of rows (row sums wave -> LDS); points = rows in registers, column tiles in LDS, every
// sum lane-local.  Partial numerators / denominators per (strip or slice, row) are added in fixed
// order by a finishing kernel.
#include "fs_kernels.h"
#include "fs_mfma.h"

namespace fs {

namespace {

constexpr int kBT = 1024;           // threads of the dense kernel
constexpr int kBRows = 16;          // rows per LDS exchange
constexpr int kBP = 256;            // threads of the point-cloud kernel
constexpr int kBTile = 256;
constexpr int kBIB = 4;
constexpr int kZ = kBaryMaxDim;

struct BaryLayout {
    int vec, nstrips, P, rpp;       // dense
    int JS, cps, ib;                // points
    int nparts;                     // partial sets per row (nstrips or JS)
    size_t o_ri, o_cj, o_part, o_xp, o_xs, o_xq, o_yp, o_ys, o_yq, total;
};

size_t up256b(size_t x) { return (x + 255) & ~(size_t)255; }

BaryLayout bary_layout(int n, int m, int d) {
    BaryLayout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += up256b(bytes); return at; };
    L.o_ri = take(sizeof(double) * n);
    L.o_cj = take(sizeof(double) * m);
    if (d == 0) {
        L.vec = m >= 4 ? 4 : 1;
        const int strip_cols = kBT * L.vec;
        L.nstrips = (m + strip_cols - 1) / strip_cols;
        int P = (512 + L.nstrips - 1) / L.nstrips;
        const int maxP = (n + kBRows - 1) / kBRows;
        if (P > maxP) P = maxP;
        if (P < 1) P = 1;
        int rpp = (n + P - 1) / P;
        rpp = ((rpp + kBRows - 1) / kBRows) * kBRows;
        L.rpp = rpp;
        L.P = (n + rpp - 1) / rpp;
        L.nparts = L.nstrips;
        if (m % 4 == 0) {                    // the matrix-core kernel (it also needs C 16-byte aligned): slices of 1024 columns
            const int slices = (m + 1023) / 1024;
            if (slices > L.nparts) L.nparts = slices;
        }
    } else {
        if (d <= 4) points_plan_after(n, m, 2048, 64, &L.JS, &L.cps, &L.ib);
        else points_plan_tiles(n, m, d, &L.JS, &L.cps);
        L.nparts = L.JS;
        L.o_xp = take(sizeof(double) * (size_t)n * d);
        L.o_xs = take(sizeof(double) * (size_t)n * d);
        L.o_xq = take(sizeof(double) * n);
        L.o_yp = take(sizeof(double) * (size_t)m * d);
        L.o_ys = take(sizeof(double) * (size_t)m * d);
        L.o_yq = take(sizeof(double) * m);
    }
    L.o_part = take(sizeof(float) * (size_t)L.nparts * n * (kZ + 1));     // [part][row][num0..3, den]
    L.total = o;
    return L;
}

struct BaryDense {
    const float *C;
    const double *ri, *cj;
    const float *Z;
    int32_t n, m, dz;
    double s;
    float *part;         // [nstrips][n][kZ + 1]
    int32_t rpp;
};

template <int VEC>
__global__ __launch_bounds__(kBT) void k_bary_dense(BaryDense A) {
    __shared__ float sRow[kBRows][kBT / 64][kZ + 1];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int strip = blockIdx.x, panel = blockIdx.y;
    const int j0 = (strip * kBT + tid) * VEC;
    double cjv[VEC];
    float zv[VEC][kZ];
    bool jok[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        jok[e] = j0 + e < A.m;
        cjv[e] = jok[e] ? A.cj[j0 + e] : -__builtin_huge_val();
#pragma unroll
        for (int t = 0; t < kZ; ++t) zv[e][t] = (jok[e] && t < A.dz) ? A.Z[(size_t)(j0 + e) * A.dz + t] : 0.0f;
    }
    const int i0 = panel * A.rpp;
    const int i1 = min(A.n, i0 + A.rpp);
    for (int ib = i0; ib < i1; ib += kBRows) {
#pragma unroll 4
        for (int r = 0; r < kBRows; ++r) {
            const int i = ib + r;
            float acc[kZ + 1];
#pragma unroll
            for (int t = 0; t <= kZ; ++t) acc[t] = 0.0f;
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
                    float p = fast_exp2((float)((rv + cjv[e]) - A.s * (double)cv[e]));
                    p = p > 0.0f ? p : 0.0f;                      // drops NaN
#pragma unroll
                    for (int t = 0; t < kZ; ++t) acc[t] = fmaf(p, zv[e][t], acc[t]);
                    acc[kZ] += p;
                }
            }
#pragma unroll
            for (int t = 0; t <= kZ; ++t) {
                const float w = wave_sum_f32(acc[t]);
                if (lane == 0) sRow[r][wave][t] = w;
            }
        }
        __syncthreads();
        if (tid < kBRows * (kZ + 1)) {
            const int r = tid / (kZ + 1), t = tid % (kZ + 1);
            if (ib + r < i1) {
                float tot = 0.0f;
#pragma unroll
                for (int w = 0; w < kBT / 64; ++w) tot += sRow[r][w][t];
                A.part[((size_t)strip * A.n + ib + r) * (kZ + 1) + t] = tot;
            }
        }
        __syncthreads();
    }
}

// Dense, m a multiple of 4 and C 16-byte aligned: the sums over j run on the matrix cores.  The five sums of a row
// (four numerators and the denominator) are the row of the product P Z' with Z' = [Z, 1]: a wave forms a 16 x 16
// patch of plan entries at a time, lane l holding row l mod 16 and the 4 columns of group l / 16 (one 16-byte load),
// and four v_mfma_f32_16x16x4_f32 add the patch's contribution to a 16 x 16 accumulator whose columns 0..4 are used:
// for element e of the load, operand A is P[row l mod 16][column 4 (l / 16) + e] and operand B is
// Z'[column 4 (l / 16) + e][l mod 16].  There is no cross-lane reduction and no barrier in the loop (the per-row
// wave reductions of the kernel above cost more than its arithmetic).  A workgroup of 8 waves owns a slice of
// 1024 columns, whose c_j and Z' it stages in LDS once, and 128 rows (16 per wave); partial sums per
// (slice, row) go to the finishing kernel as before.
constexpr int kMMSlice = 1024;          // columns per workgroup
constexpr int kMMWaves = 8;             // waves per workgroup, 16 rows each per round
constexpr int kMMRounds = 1;            // rounds per workgroup

typedef float float4_v __attribute__((ext_vector_type(4)));
typedef double double2_a __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(kMMWaves * 64) void k_bary_dense_mm(BaryDense A) {
    __shared__ __align__(16) double sCj[kMMSlice];
    __shared__ __align__(16) float sZ[kZ + 2][kMMSlice];      // rows 0..3: Z (0 beyond dz), 4: ones, 5: zeros
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int li = lane & 15, lk = lane >> 4;
    const int col0 = blockIdx.x * kMMSlice;
    for (int c = tid; c < kMMSlice; c += kMMWaves * 64) {
        const int j = col0 + c;
        const bool ok = j < A.m;
        sCj[c] = ok ? A.cj[j] : -__builtin_huge_val();
#pragma unroll
        for (int t = 0; t < kZ; ++t) sZ[t][c] = (ok && t < A.dz) ? A.Z[(size_t)j * A.dz + t] : 0.0f;
        sZ[kZ][c] = ok ? 1.0f : 0.0f;
        sZ[kZ + 1][c] = 0.0f;
    }
    __syncthreads();
    const float *zrow = sZ[li < kZ + 1 ? li : kZ + 1];
    const int nstep = (min(kMMSlice, A.m - col0) + 63) / 64;      // steps of 64 columns
    for (int rd = 0; rd < kMMRounds; ++rd) {
        const int r0 = ((blockIdx.y * kMMRounds + rd) * kMMWaves + wave) * 16;
        if (r0 >= A.n) break;                                  // uniform over the wave
        const int my_row = r0 + li;
        const bool rok = my_row < A.n;
        const double rv = rok ? A.ri[my_row] : -__builtin_huge_val();
        const float *crow = A.C + (size_t)(rok ? my_row : A.n - 1) * A.m;
        float4_v acc = {0.0f, 0.0f, 0.0f, 0.0f};
        // Four column groups (64 columns) per step; the loads of the next step are in flight while this one is
        // worked on.  Groups past the slice's last column read column 0 instead: their c_j is -inf in LDS.
        auto load4 = [&](float4_v (&c4)[4], int st) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int col = col0 + (st * 4 + u) * 16 + 4 * lk;
                if (col >= A.m) col = 0;
                c4[u] = *reinterpret_cast<const float4_v *>(crow + col);
            }
        };
        auto work4 = [&](const float4_v (&c4)[4], int st, double rv) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = (st * 4 + u) * 16 + 4 * lk;
                const double2_a cja = *reinterpret_cast<const double2_a *>(&sCj[c]);
                const double2_a cjb = *reinterpret_cast<const double2_a *>(&sCj[c + 2]);
                const float4_v zb = *reinterpret_cast<const float4_v *>(&zrow[c]);
                const double cj[4] = {cja.x, cja.y, cjb.x, cjb.y};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // an exponent of -inf or NaN (zero weights, potentials that are not finite) gives a plan entry of 0
                    const float arg = fmaxf((float)fma(-A.s, (double)c4[u][e], rv + cj[e]), -200.0f);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(fast_exp2(arg), zb[e], acc, 0, 0, 0);
                }
            }
        };
        // (Straight-line code: a step past the end loads the last step again and works on it with a row term of
        // -inf, which adds nothing; so the number of loads in flight at every wait is known at compile time.)
        // Every wave starts its sweep at a different step (and wraps round): waves that run side by side then read
        // different 256-byte blocks of their rows, which all lie a multiple of the row pitch apart.
        const int rot = (wave * 2 + blockIdx.y * 5 + blockIdx.x * 3) % nstep;
        auto at = [&](int st) { const int q = st + rot; return q >= nstep ? q - nstep : q; };
        float4_v ca[4], cb[4];
        load4(ca, at(0));
        for (int st = 0; st < nstep; st += 2) {
            const bool second = st + 1 < nstep;
            load4(cb, at(second ? st + 1 : st));
            work4(ca, at(st), rv);
            load4(ca, at(min(st + 2, nstep - 1)));
            work4(cb, at(second ? st + 1 : st), second ? rv : -__builtin_huge_val());
        }
        // accumulator register q of lane l: row 4 (l / 16) + q, column l mod 16
        if (li <= kZ) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = r0 + 4 * lk + q;
                if (row < A.n) A.part[((size_t)blockIdx.x * A.n + row) * (kZ + 1) + li] = acc[q];
            }
        }
    }
}

struct BaryPoints {
    const double *rows, *rowq, *rowlog;     // x side: plain coordinates, s|x|^2, ri
    const double *cols2s, *colq, *collog;   // y side: 2 s y, s|y|^2, cj
    const float *Z;
    int32_t nr, nc, dz;
    float *part;                            // [JS][nr][kZ + 1]
    int32_t cols_per_split;
};

template <int D, int IB>
__global__ __launch_bounds__(kBP) void k_bary_points(BaryPoints A) {
    __shared__ __align__(16) double tile[kBTile][D + 1];      // [0] collog - colq, [1..D] 2 s y
    __shared__ float tileZ[kBTile][kZ];
    const int tid = threadIdx.x;
    double x[IB][D], rc[IB];
    int row[IB];
    float acc[IB][kZ + 1];
#pragma unroll
    for (int b = 0; b < IB; ++b) {
        row[b] = (blockIdx.x * IB + b) * kBP + tid;
        const bool ok = row[b] < A.nr;
#pragma unroll
        for (int t = 0; t < D; ++t) x[b][t] = ok ? A.rows[(size_t)row[b] * D + t] : 0.0;
        rc[b] = ok ? A.rowlog[row[b]] - A.rowq[row[b]] : -__builtin_huge_val();
#pragma unroll
        for (int t = 0; t <= kZ; ++t) acc[b][t] = 0.0f;
    }
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);
    for (int jt = j0; jt < j1; jt += kBTile) {
        __syncthreads();
        {
            const int j = jt + tid;
            if (j < j1) {
                tile[tid][0] = A.collog[j] - A.colq[j];
#pragma unroll
                for (int t = 0; t < D; ++t) tile[tid][1 + t] = A.cols2s[(size_t)j * D + t];
#pragma unroll
                for (int t = 0; t < kZ; ++t) tileZ[tid][t] = t < A.dz ? A.Z[(size_t)j * A.dz + t] : 0.0f;
            } else {
                tile[tid][0] = -__builtin_huge_val();
#pragma unroll
                for (int t = 0; t < D; ++t) tile[tid][1 + t] = 0.0;
#pragma unroll
                for (int t = 0; t < kZ; ++t) tileZ[tid][t] = 0.0f;
            }
        }
        __syncthreads();
        const int cnt = min(kBTile, (j1 - jt + 1) & ~1);       // staged columns (the tile is padded with -inf)
#pragma unroll 2
        for (int jj = 0; jj < cnt; ++jj) {
            double w[D + 1];
#pragma unroll
            for (int t = 0; t <= D; ++t) w[t] = tile[jj][t];
            float z[kZ];
#pragma unroll
            for (int t = 0; t < kZ; ++t) z[t] = tileZ[jj][t];
#pragma unroll
            for (int b = 0; b < IB; ++b) {
                double tq = w[0];
#pragma unroll
                for (int t = 0; t < D; ++t) tq = fma(x[b][t], w[1 + t], tq);
                float p = fast_exp2((float)(tq + rc[b]));
                p = p > 0.0f ? p : 0.0f;
#pragma unroll
                for (int t = 0; t < kZ; ++t) acc[b][t] = fmaf(p, z[t], acc[b][t]);
                acc[b][kZ] += p;
            }
        }
    }
#pragma unroll
    for (int b = 0; b < IB; ++b)
        if (row[b] < A.nr) {
#pragma unroll
            for (int t = 0; t <= kZ; ++t) A.part[((size_t)blockIdx.y * A.nr + row[b]) * (kZ + 1) + t] = acc[b][t];
        }
}

// More than 4 coordinates: the dot products run on the fp64 matrix cores (fs_mfma.h); the accumulator
// starts at (cj_j - s|y_j|^2) + (ri_i - s|x_i|^2), so the matrix core delivers log2 P_ij itself.
template <int D4>
__global__ __launch_bounds__(256) void k_bary_points_mfma(BaryPoints A, int d) {
    __shared__ double tile[kTileJ][4 * D4 + 1];
    __shared__ double tw[kTileJ];
    __shared__ float tz[kTileJ][kZ];
    const int tid = threadIdx.x, lj = tid & 15;
    RowTiles<D4> R;
    R.load(A.rows, A.nr, d);
    double rc[kTileRT][4];
    float acc5[kTileRT][4][kZ + 1];
#pragma unroll
    for (int rt = 0; rt < kTileRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = R.result_row(rt, r);
            rc[rt][r] = row < A.nr ? A.rowlog[row] - A.rowq[row] : -__builtin_huge_val();
#pragma unroll
            for (int t = 0; t <= kZ; ++t) acc5[rt][r][t] = 0.0f;
        }
    const int j0 = blockIdx.y * A.cols_per_split;
    const int j1 = min(A.nc, j0 + A.cols_per_split);
    mfma_walk<D4>(
        R, tile, A.cols2s, d, j0, j1,
        [&](int jt) {
            if (tid < kTileJ) {
                const int j = jt + tid;
                tw[tid] = j < j1 ? A.collog[j] - A.colq[j] : -__builtin_huge_val();
#pragma unroll
                for (int t = 0; t < kZ; ++t) tz[tid][t] = (j < j1 && t < A.dz) ? A.Z[(size_t)j * A.dz + t] : 0.0f;
            }
        },
        [&](int ct, int rt, int r) { return tw[ct * 16 + lj] + rc[rt][r]; },
        [&](int, int ct, int rt, const double4_m &acc) {
            float z[kZ];
#pragma unroll
            for (int t = 0; t < kZ; ++t) z[t] = tz[ct * 16 + lj][t];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float p = fast_exp2((float)acc[r]);
                p = p > 0.0f ? p : 0.0f;
#pragma unroll
                for (int t = 0; t < kZ; ++t) acc5[rt][r][t] = fmaf(p, z[t], acc5[rt][r][t]);
                acc5[rt][r][kZ] += p;
            }
        });
#pragma unroll
    for (int rt = 0; rt < kTileRT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = R.result_row(rt, r);
#pragma unroll
            for (int t = 0; t <= kZ; ++t) {
                const float tot = row16_sum(acc5[rt][r][t]);
                if (lj == 0 && row < A.nr) A.part[((size_t)blockIdx.y * A.nr + row) * (kZ + 1) + t] = tot;
            }
        }
}

// T[i][t] = (sum over partial sets of the numerators) / (sum of the denominators), in double.
__global__ __launch_bounds__(256) void k_bary_finish(const float *part, int nparts, int n, int dz, float *T) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    double num[kZ] = {0, 0, 0, 0}, den = 0.0;
    for (int q = 0; q < nparts; ++q) {
        const float *src = part + ((size_t)q * n + i) * (kZ + 1);
#pragma unroll
        for (int t = 0; t < kZ; ++t) num[t] += (double)src[t];
        den += (double)src[kZ];
    }
    for (int t = 0; t < dz; ++t) T[(size_t)i * dz + t] = den > 0.0 ? (float)(num[t] / den) : 0.0f;
}

}  // namespace

size_t bary_scratch_bytes(int n, int m, int d) { return bary_layout(n, m, d).total; }

hipError_t launch_bary(hipStream_t st, const PlanArgs &a, const float *Z, int dz, float *T, void *scratch,
                       size_t scratch_bytes) {
    if (dz < 1 || dz > kZ) return hipErrorInvalidValue;
    const BaryLayout L = bary_layout(a.n, a.m, a.d);
    if (scratch_bytes < L.total) return hipErrorInvalidValue;
    unsigned char *ws = (unsigned char *)scratch;
    double *ri = (double *)(ws + L.o_ri), *cj = (double *)(ws + L.o_cj);
    double *xp = nullptr, *xs = nullptr, *xq = nullptr, *yp = nullptr, *ys = nullptr, *yq = nullptr;
    if (a.d > 0) {
        xp = (double *)(ws + L.o_xp); xs = (double *)(ws + L.o_xs); xq = (double *)(ws + L.o_xq);
        yp = (double *)(ws + L.o_yp); ys = (double *)(ws + L.o_ys); yq = (double *)(ws + L.o_yq);
    }
    hipError_t e = launch_plan_prep_all(st, a, ri, cj, xp, xs, xq, yp, ys, yq);
    if (e != hipSuccess) return e;
    float *part = (float *)(ws + L.o_part);
    int nparts = L.nparts;
    if (a.d == 0) nparts = L.nstrips;
    if (a.d == 0) {
        BaryDense D{};
        D.C = a.C; D.ri = ri; D.cj = cj; D.Z = Z; D.n = a.n; D.m = a.m; D.dz = dz; D.s = a.s;
        D.part = part; D.rpp = L.rpp;
        const dim3 grid(L.nstrips, L.P);
        if (a.m % 4 == 0 && (reinterpret_cast<uintptr_t>(a.C) & 15) == 0) {
            nparts = (a.m + kMMSlice - 1) / kMMSlice;
            const int rows_per_wg = kMMRounds * kMMWaves * 16;
            const dim3 gmm(nparts, (a.n + rows_per_wg - 1) / rows_per_wg);
            hipLaunchKernelGGL(k_bary_dense_mm, gmm, dim3(kMMWaves * 64), 0, st, D);
        }
        else if (L.vec == 4) hipLaunchKernelGGL(k_bary_dense<4>, grid, dim3(kBT), 0, st, D);
        else hipLaunchKernelGGL(k_bary_dense<1>, grid, dim3(kBT), 0, st, D);
    } else {
        BaryPoints X{};
        X.rows = xp; X.rowq = xq; X.rowlog = ri; X.cols2s = ys; X.colq = yq; X.collog = cj;
        X.Z = Z; X.nr = a.n; X.nc = a.m; X.dz = dz; X.part = part; X.cols_per_split = L.cps;
        if (a.d <= 4) {
            if (L.ib != 1 && L.ib != kBIB) return hipErrorInvalidValue;
            const dim3 grid((a.n + kBP * L.ib - 1) / (kBP * L.ib), L.JS);
#define FS_BARY_PTS(D)                                                                          \
    do {                                                                                        \
        if (L.ib == 1) hipLaunchKernelGGL((k_bary_points<D, 1>), grid, dim3(kBP), 0, st, X);    \
        else hipLaunchKernelGGL((k_bary_points<D, kBIB>), grid, dim3(kBP), 0, st, X);           \
    } while (0)
            switch (a.d) {
                case 1: FS_BARY_PTS(1); break;
                case 2: FS_BARY_PTS(2); break;
                case 3: FS_BARY_PTS(3); break;
                default: FS_BARY_PTS(4); break;
            }
#undef FS_BARY_PTS
        } else {
            const dim3 grid((a.n + kTileRows - 1) / kTileRows, L.JS);
            switch (mfma_d4(a.d)) {
                case 2: hipLaunchKernelGGL(k_bary_points_mfma<2>, grid, dim3(256), 0, st, X, a.d); break;
                case 4: hipLaunchKernelGGL(k_bary_points_mfma<4>, grid, dim3(256), 0, st, X, a.d); break;
                case 8: hipLaunchKernelGGL(k_bary_points_mfma<8>, grid, dim3(256), 0, st, X, a.d); break;
                default: hipLaunchKernelGGL(k_bary_points_mfma<16>, grid, dim3(256), 0, st, X, a.d); break;
            }
        }
    }
    hipLaunchKernelGGL(k_bary_finish, dim3((a.n + 255) / 256), dim3(256), 0, st, part, nparts, a.n, dz, T);
    return hipGetLastError();
}

}  // namespace fs
