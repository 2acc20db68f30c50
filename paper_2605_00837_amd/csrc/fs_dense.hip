// Dense-cost kernels for gfx950.
//
//   k_row_stream   f-update (Eq. 9): one workgroup owns 4 rows and streams them
//                  once with coalesced 16-byte loads, online (max, sum) LSE per
//                  lane, wave64 DPP reduction, LDS combine of the 4 waves.
//   k_col_stream   g-update (Eq. 10) without strided reads: a workgroup owns a
//                  strip of adjacent columns (4 per lane) and walks down a panel
//                  of rows; every load is a coalesced row segment and the
//                  reduction over rows is lane-local.  Per-panel partial LSE
//                  values are merged by k_combine.
//   k_fused        both half-steps in ONE pass over C: a workgroup holds a
//                  panel of R full rows in registers, finishes their row LSE
//                  (new f_i), and immediately folds the same registers into the
//                  running column LSE with the new f_i.  HBM sees C once per
//                  iteration instead of twice.
#include "fs_kernels.h"

namespace fs {

constexpr int kRowsPerWG = 4;      // k_row_stream
constexpr int kFewRows = 2048;     // below: k_row_stream_few, one row per workgroup
constexpr int kStreamT = 256;

template <int VEC>
struct VecLoad;
// Four adjacent costs with one 16-byte load.  Rows of C start at multiples of m floats, i.e. at any
// 4-byte boundary (float4_a4).  `valid` < 4 (the last columns of a row whose length is not a multiple
// of 4) falls back to single loads.
template <>
struct VecLoad<4> {
    static __device__ __forceinline__ void ld(const float *p, float (&o)[4], int valid) {
        if (valid >= 4) {
            const float4_a4 v = *reinterpret_cast<const float4_a4 *>(p);
            o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = e < valid ? p[e] : 0.0f;
        }
    }
};
template <>
struct VecLoad<1> {
    static __device__ __forceinline__ void ld(const float *p, float (&o)[1], int) { o[0] = *p; }
};

// VEC adjacent costs starting at entry `idx` of C, as fp32: 4 fp32 entries, or 8 entries stored in
// 2 bytes each (16-byte aligned: such matrices have m % 8 == 0).
template <int VEC, int DT>
__device__ __forceinline__ void load_costs(const float *C, size_t idx, float (&o)[VEC], int valid) {
    if constexpr (DT == 0) {
        VecLoad<VEC>::ld(C + idx, o, valid);
    } else {
        static_assert(VEC == 8, "2-byte costs are read 8 at a time");
        const uint4 raw = *reinterpret_cast<const uint4 *>(reinterpret_cast<const unsigned short *>(C) + idx);
        const unsigned w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            o[2 * h] = cost_from_bits<DT>(w4[h] & 0xffffu);
            o[2 * h + 1] = cost_from_bits<DT>(w4[h] >> 16);
        }
    }
}

// ---------------------------------------------------------------- row pass (streaming)
template <int VEC, int DT = 0>
__global__ __launch_bounds__(kStreamT) void k_row_stream(DenseArgs A, Ctl c) {
    __shared__ double sM[kRowsPerWG][kStreamT / 64];
    __shared__ float sS[kRowsPerWG][kStreamT / 64];
    int k;
    if (!launch_active(c, k)) return;
    const int cur = k & 1, nxt = cur ^ 1;
    const Pots &p = A.p;
    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * kRowsPerWG;
    const double *V = p.V + (size_t)cur * p.m_ld;
    const double ns = -p.s;

    Lse acc[kRowsPerWG];
#pragma unroll
    for (int r = 0; r < kRowsPerWG; ++r) acc[r].init();

    for (int col = tid * VEC; col < p.m; col += kStreamT * VEC) {
        const int valid = p.m - col;                   // >= VEC except in the last columns of the row
        double v[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = e < valid ? V[col + e] : -__builtin_huge_val();
#pragma unroll
        for (int r = 0; r < kRowsPerWG; ++r) {
            const int i = i0 + r;
            if (i < p.n) {
                float cv[VEC];
                load_costs<VEC, DT>(A.C, (size_t)i * p.m + col, cv, valid);
                double x[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e] = fma(ns, (double)cv[e], v[e]);
                acc[r].template add<VEC>(x);
            }
        }
    }
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int r = 0; r < kRowsPerWG; ++r) {
        acc[r].wave_reduce();
        if (lane == 0) { sM[r][wave] = acc[r].M; sS[r][wave] = acc[r].s; }
    }
    __syncthreads();
    if (tid < kRowsPerWG) {
        const int i = i0 + tid;
        if (i < p.n) {
            Lse t; t.init();
#pragma unroll
            for (int w = 0; w < kStreamT / 64; ++w) t.merge(sM[tid][w], sS[tid][w]);
            const double Fn = t.value();
            p.F[(size_t)nxt * p.n_ld + i] = Fn;
            p.U[(size_t)nxt * p.n_ld + i] = p.la2[i] - Fn;
        }
    }
}

// ---------------------------------------------------------------- row pass, few rows
// Short and wide matrices (fewer than kFewRows rows): with 4 rows per workgroup a 512 x 100000 problem is 128
// workgroups with one 16-byte load per row in flight per lane (1.3 TB/s).  Here a workgroup owns ONE row and every
// lane keeps UN column chunks of it in flight.
template <int VEC, int DT = 0>
__global__ __launch_bounds__(kStreamT) void k_row_stream_few(DenseArgs A, Ctl c) {
    constexpr int UN = 4;
    __shared__ double sM[kStreamT / 64];
    __shared__ float sS[kStreamT / 64];
    int k;
    if (!launch_active(c, k)) return;
    const int cur = k & 1, nxt = cur ^ 1;
    const Pots &p = A.p;
    const int tid = threadIdx.x;
    const int i = blockIdx.x;                          // the grid has exactly n workgroups
    const double *V = p.V + (size_t)cur * p.m_ld;
    const double ns = -p.s;
    Lse acc;
    acc.init();
    for (int col0 = tid * VEC; col0 < p.m; col0 += kStreamT * VEC * UN) {
        float cv[UN][VEC];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int col = col0 + u * kStreamT * VEC;
            if (col < p.m) {
                load_costs<VEC, DT>(A.C, (size_t)i * p.m + col, cv[u], p.m - col);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) cv[u][e] = 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int col = col0 + u * kStreamT * VEC;
            const int valid = p.m - col;               // <= 0 for a chunk past the end: every term is -inf
            double x[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[e] = e < valid ? fma(ns, (double)cv[u][e], V[col + e]) : -__builtin_huge_val();
            acc.template add<VEC>(x);
        }
    }
    const int wave = tid >> 6, lane = tid & 63;
    acc.wave_reduce();
    if (lane == 0) { sM[wave] = acc.M; sS[wave] = acc.s; }
    __syncthreads();
    if (tid == 0) {
        Lse t; t.init();
#pragma unroll
        for (int w = 0; w < kStreamT / 64; ++w) t.merge(sM[w], sS[w]);
        const double Fn = t.value();
        p.F[(size_t)nxt * p.n_ld + i] = Fn;
        p.U[(size_t)nxt * p.n_ld + i] = p.la2[i] - Fn;
    }
}

// Few rows and very many columns: one row and one column range per workgroup; the partial LSE values go to the
// combine kernel (512 x 100000: 4 ranges, 2048 workgroups instead of 512).
template <int VEC, int DT = 0>
__global__ __launch_bounds__(kStreamT) void k_row_split(DenseArgs A, Ctl c) {
    constexpr int UN = 4;
    __shared__ double sM[kStreamT / 64];
    __shared__ float sS[kStreamT / 64];
    int k;
    if (!launch_active(c, k)) return;
    const int cur = k & 1;
    const Pots &p = A.p;
    const int tid = threadIdx.x;
    const int i = blockIdx.x;                          // the grid has exactly n x row_splits workgroups
    const int j0 = blockIdx.y * A.row_cps;
    const int j1 = min(p.m, j0 + A.row_cps);
    const double *V = p.V + (size_t)cur * p.m_ld;
    const double ns = -p.s;
    Lse acc;
    acc.init();
    for (int col0 = j0 + tid * VEC; col0 < j1; col0 += kStreamT * VEC * UN) {
        float cv[UN][VEC];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int col = col0 + u * kStreamT * VEC;
            if (col < j1) {
                load_costs<VEC, DT>(A.C, (size_t)i * p.m + col, cv[u], j1 - col);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) cv[u][e] = 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int col = col0 + u * kStreamT * VEC;
            const int valid = j1 - col;                // <= 0 for a chunk past the end: every term is -inf
            double x[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[e] = e < valid ? fma(ns, (double)cv[u][e], V[col + e]) : -__builtin_huge_val();
            acc.template add<VEC>(x);
        }
    }
    const int wave = tid >> 6, lane = tid & 63;
    acc.wave_reduce();
    if (lane == 0) { sM[wave] = acc.M; sS[wave] = acc.s; }
    __syncthreads();
    if (tid == 0) {
        Lse t; t.init();
#pragma unroll
        for (int w = 0; w < kStreamT / 64; ++w) t.merge(sM[w], sS[w]);
        A.rowpart[(size_t)blockIdx.y * p.n_ld + i] = t.value();
    }
}

void dense_row_split_plan(int n, int m, int *splits, int *cols_per_split) {
    // about 2048 workgroups, ranges of whole 2048-column groups (every range starts 16-byte aligned for both
    // entry sizes) and of at least 4096 columns
    int S = 1, cps = m;
    if (n < 1024 && m >= 8192) {                        // from 1024 rows on the extra combine launch costs more than it saves
        S = (2048 + n - 1) / n;
        if (S > 64) S = 64;
        if (S > m / 4096) S = m / 4096;
        if (S > 1) {
            cps = (m + S - 1) / S;
            cps = ((cps + 2047) / 2048) * 2048;
            S = (m + cps - 1) / cps;
        }
        if (S <= 1) { S = 1; cps = m; }
    }
    *splits = S;
    *cols_per_split = cps;
}

// ---------------------------------------------------------------- column pass (streaming)
template <int VEC, int DT = 0>
__global__ __launch_bounds__(kStreamT) void k_col_stream(DenseArgs A, Ctl c) {
    int k;
    if (!launch_active(c, k)) return;
    const int nxt = (k & 1) ^ 1;
    const Pots &p = A.p;
    const int j0 = (blockIdx.x * kStreamT + threadIdx.x) * VEC;
    if (j0 >= p.m) return;                       // no cross-lane work below
    const int valid = p.m - j0;                  // >= VEC except for the lane that owns the last columns
    // panels are walked from the bottom of C upwards: the row pass that ran just before streamed C
    // top to bottom, so the rows still resident in the last-level cache are visited first
    const int panel = (int)gridDim.y - 1 - (int)blockIdx.y;
    const int r0 = panel * A.rows_per_panel;
    const int r1 = min(p.n, r0 + A.rows_per_panel);
    const double *U = p.U + (size_t)nxt * p.n_ld;     // the new f of this iteration (Gauss-Seidel order)
    const double ns = -p.s;

    Lse acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e].init();

    constexpr int RC = VEC == 8 ? 2 : 4;          // rows folded per rescale
    for (int i = r0; i < r1; i += RC) {
        double x[VEC][RC];
#pragma unroll
        for (int q = 0; q < RC; ++q) {
            const int ii = i + q;
            if (ii < r1) {
                float cv[VEC];
                load_costs<VEC, DT>(A.C, (size_t)ii * p.m + j0, cv, valid);
                const double u = U[ii];
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e][q] = fma(ns, (double)cv[e], u);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e][q] = kNegHuge;
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e].template add<RC>(x[e]);
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        if (e < valid) A.colpart[(size_t)panel * p.m_ld + j0 + e] = acc[e].value();
}

static bool vec4_ok(const DenseArgs &a) {
    return a.p.m >= 4 && ((reinterpret_cast<uintptr_t>(a.C) & 3u) == 0);
}

void dense_stream_plan(int n, int m, int *P, int *rows_per_panel) {
    const int strips = (m + kStreamT * 4 - 1) / (kStreamT * 4);   // conservative: vector path
    int want = (1024 + strips - 1) / strips;                      // about 1024 workgroups in total
    int maxP = (n + 15) / 16;                                     // at least 16 rows per panel
    int p = want < maxP ? want : maxP;
    if (p < 1) p = 1;
    if (p > 512) p = 512;
    int rpp = (n + p - 1) / p;
    p = (n + rpp - 1) / rpp;
    *P = p;
    *rows_per_panel = rpp;
}

hipError_t launch_dense_row(hipStream_t st, const DenseArgs &a, const Ctl &c, const Stamp &tm) {
    if (a.row_splits > 1) {
        if (!a.rowpart || a.row_cps % 2048 != 0) return hipErrorInvalidValue;
        const dim3 grid(a.p.n, a.row_splits);
        if (a.c_dtype == 1) launch_stamped((k_row_split<8, 1>), grid, dim3(kStreamT), st, tm, a, c);
        else if (a.c_dtype == 2) launch_stamped((k_row_split<8, 2>), grid, dim3(kStreamT), st, tm, a, c);
        else if (vec4_ok(a)) launch_stamped(k_row_split<4>, grid, dim3(kStreamT), st, tm, a, c);
        else launch_stamped(k_row_split<1>, grid, dim3(kStreamT), st, tm, a, c);
        return hipGetLastError();
    }
    if (a.p.n < kFewRows) {
        const dim3 grid(a.p.n);
        if (a.c_dtype == 1) launch_stamped((k_row_stream_few<8, 1>), grid, dim3(kStreamT), st, tm, a, c);
        else if (a.c_dtype == 2) launch_stamped((k_row_stream_few<8, 2>), grid, dim3(kStreamT), st, tm, a, c);
        else if (vec4_ok(a)) launch_stamped(k_row_stream_few<4>, grid, dim3(kStreamT), st, tm, a, c);
        else launch_stamped(k_row_stream_few<1>, grid, dim3(kStreamT), st, tm, a, c);
        return hipGetLastError();
    }
    const dim3 grid((a.p.n + kRowsPerWG - 1) / kRowsPerWG);
    if (a.c_dtype == 1) launch_stamped((k_row_stream<8, 1>), grid, dim3(kStreamT), st, tm, a, c);
    else if (a.c_dtype == 2) launch_stamped((k_row_stream<8, 2>), grid, dim3(kStreamT), st, tm, a, c);
    else if (vec4_ok(a)) launch_stamped(k_row_stream<4>, grid, dim3(kStreamT), st, tm, a, c);
    else launch_stamped(k_row_stream<1>, grid, dim3(kStreamT), st, tm, a, c);
    return hipGetLastError();
}

hipError_t launch_dense_col(hipStream_t st, const DenseArgs &a, const Ctl &c) {
    if (a.c_dtype != 0) {
        const dim3 grid((a.p.m + kStreamT * 8 - 1) / (kStreamT * 8), a.P);
        if (a.c_dtype == 1) hipLaunchKernelGGL((k_col_stream<8, 1>), grid, dim3(kStreamT), 0, st, a, c);
        else hipLaunchKernelGGL((k_col_stream<8, 2>), grid, dim3(kStreamT), 0, st, a, c);
    } else if (vec4_ok(a)) {
        const dim3 grid((a.p.m + kStreamT * 4 - 1) / (kStreamT * 4), a.P);
        hipLaunchKernelGGL(k_col_stream<4>, grid, dim3(kStreamT), 0, st, a, c);
    } else {
        const dim3 grid((a.p.m + kStreamT - 1) / kStreamT, a.P);
        hipLaunchKernelGGL(k_col_stream<1>, grid, dim3(kStreamT), 0, st, a, c);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- fused row-panel pass
// T threads, each owning Q groups of 4 adjacent columns: column(q, e) =
// (q*T + tid)*4 + e, so a panel row is read as Q fully coalesced 16-byte loads
// per lane and m <= 4*Q*T.  R rows are held at once.
template <int T, int Q, int R>
__global__ __launch_bounds__(T) void k_fused(DenseArgs A, Ctl c) {
    constexpr int NW = T / 64;
    static_assert(R * NW <= 64, "one wave merges all (row, wave) partials in one shot");
    __shared__ double sM[2][R][NW];
    __shared__ float sS[2][R][NW];
    int k;
    if (!launch_active(c, k)) return;
    const int cur = k & 1, nxt = cur ^ 1;
    const Pots &p = A.p;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const double ns = -p.s;
    const bool col_phase = (c.phase == 0);        // the trailing error pass needs the row LSE only
    const int m = p.m;                            // m % 4 == 0 on this path

    double v[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int col = (q * T + tid) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            v[q][e] = col < m ? p.V[(size_t)cur * p.m_ld + col + e] : -__builtin_huge_val();
    }
    Lse cs[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[q][e].init();

    const int npanels = (p.n + R - 1) / R;
    int par = 0;
    // odd iterations walk the panels from the bottom up: what the previous iteration read last is
    // still in the last-level cache and is read first
    const bool rev = (k & 1) != 0;
    // Small panels (16 registers) are loaded one panel ahead, so that a workgroup with many panels (a tall
    // matrix) does not wait out a full memory round trip per panel.
    constexpr bool kAhead = T == 256 && R * Q * 4 <= 16;
    auto load_panel = [&](int pq, float (&dst)[R][Q][4]) {
        const int i0 = (rev ? npanels - 1 - pq : pq) * R;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool rok = pq < npanels && (i0 + r) < p.n;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int col = (q * T + tid) * 4;
                if (rok && col < m) {
                    VecLoad<4>::ld(A.C + (size_t)(i0 + r) * m + col, dst[r][q], 4);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) dst[r][q][e] = 0.0f;
                }
            }
        }
    };
    float cv[R][Q][4], ahead[kAhead ? R : 1][kAhead ? Q : 1][4];
    if (kAhead) load_panel(blockIdx.x, cv);
    for (int pq = blockIdx.x; pq < npanels; pq += gridDim.x, par ^= 1) {
        const int pn = rev ? npanels - 1 - pq : pq;
        const int i0 = pn * R;
        if constexpr (kAhead) load_panel(pq + gridDim.x, ahead);
        else load_panel(pq, cv);
        // ---- row phase: lane-local LSE over the lane's 4Q columns (one row at a time, so that
        //      only one row's fp64 arguments are live), then the wave reductions of all R rows
        Lse rs[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            double x[Q * 4];
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) x[q * 4 + e] = fma(ns, (double)cv[r][q][e], v[q][e]);
            rs[r].init();
            rs[r].template add<Q * 4>(x);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            rs[r].wave_reduce();
            if (lane == 0) { sM[par][r][wave] = rs[r].M; sS[par][r][wave] = rs[r].s; }
        }
        __syncthreads();
        // ---- every wave merges the NW wave partials of all R rows: lane r*NW + w holds (row r, wave w)
        double Fn_lane;
        {
            const int rr = lane / NW, ww = lane % NW;
            Lse t; t.init();
            if (rr < R) { t.M = sM[par][rr][ww]; t.s = sS[par][rr][ww]; }
            double Mg = t.M;
#pragma unroll
            for (int off = NW / 2; off >= 1; off >>= 1) Mg = dmax(Mg, __shfl_xor(Mg, off));
            float sg = t.s * fast_exp2((float)(t.M - Mg));
#pragma unroll
            for (int off = NW / 2; off >= 1; off >>= 1) sg += __shfl_xor(sg, off);
            Fn_lane = Mg + log2_sum(sg);
        }
        // ---- new potentials: lane r*NW of wave 0 owns row r
        if (wave == 0 && (lane % NW) == 0 && (lane / NW) < R) {
            const int i = i0 + lane / NW;
            if (i < p.n) {
                p.F[(size_t)nxt * p.n_ld + i] = Fn_lane;
                p.U[(size_t)nxt * p.n_ld + i] = p.la2[i] - Fn_lane;
            }
        }
        // ---- column phase with the new f: lane-local over the R rows, one column at a time
        if (col_phase) {
            double u[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const double Fn = __shfl(Fn_lane, r * NW);
                u[r] = (i0 + r) < p.n ? p.la2[i0 + r] - Fn : -__builtin_huge_val();
            }
#pragma unroll
            for (int q = 0; q < Q; ++q) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    double y[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) y[r] = fma(ns, (double)cv[r][q][e], u[r]);
                    cs[q][e].template add<R>(y);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (kAhead) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) cv[r][q][e] = ahead[r][q][e];
        }
    }
    if (col_phase) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int col = (q * T + tid) * 4;
            if (col < m) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    A.colpart[(size_t)blockIdx.x * p.m_ld + col + e] = cs[q][e].value();
            }
        }
    }
}

// ---------------------------------------------------------------- fused pass, one wave per row
// Narrow matrices (m <= 256 Q): a row fits the 64 lanes of ONE wave (Q groups of 4 adjacent columns per lane),
// so the 4 waves of a workgroup walk different panels of R rows and never meet inside the loop: the row LSE is a
// wave reduction, no LDS, no barrier.  Their column LSE pairs meet once, at the end, in LDS, and the workgroup
// writes one set of column partials.  Same exact running-maximum arithmetic as k_fused; with all 256 lanes of
// k_fused<256, 1, 4> mapped to columns, three waves in four idled at m = 256 (65536 x 256: 86 us per pass).
template <int Q, int R>
__global__ __launch_bounds__(256) void k_fused_rows(DenseArgs A, Ctl c) {
    constexpr int NW = 4;
    __shared__ double sM[NW][Q * 256];
    __shared__ float sS[NW][Q * 256];
    int k;
    if (!launch_active(c, k)) return;
    const int cur = k & 1, nxt = cur ^ 1;
    const Pots &p = A.p;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const double ns = -p.s;
    const bool col_phase = (c.phase == 0);        // the trailing error pass needs the row LSE only
    const int m = p.m;                            // m % 4 == 0 on this path

    double v[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int col = (q * 64 + lane) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            v[q][e] = col < m ? p.V[(size_t)cur * p.m_ld + col + e] : -__builtin_huge_val();
    }
    Lse cs[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[q][e].init();

    const int npanels = (p.n + R - 1) / R;
    const int first = blockIdx.x * NW + wave, stride = gridDim.x * NW;
    auto load_panel = [&](int pq, float (&dst)[R][Q][4]) {
        const int i0 = pq * R;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool rok = pq < npanels && (i0 + r) < p.n;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int col = (q * 64 + lane) * 4;
                if (rok && col < m) {
                    VecLoad<4>::ld(A.C + (size_t)(i0 + r) * m + col, dst[r][q], 4);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) dst[r][q][e] = 0.0f;
                }
            }
        }
    };
    float cv[R][Q][4], ahead[R][Q][4];
    load_panel(first, cv);
    for (int pq = first; pq < npanels; pq += stride) {
        const int i0 = pq * R;
        load_panel(pq + stride, ahead);           // one panel ahead: the round trip runs under this panel's arithmetic
        double Fn[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            double x[Q * 4];
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) x[q * 4 + e] = fma(ns, (double)cv[r][q][e], v[q][e]);
            Lse rs;
            rs.init();
            rs.template add<Q * 4>(x);
            rs.wave_reduce();
            Fn[r] = rs.value();
            __builtin_amdgcn_sched_barrier(0);
        }
        double u[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool rok = (i0 + r) < p.n;
            const double la = rok ? p.la2[i0 + r] : 0.0;
            u[r] = rok ? la - Fn[r] : -__builtin_huge_val();
            if (lane == r && rok) {               // lane r writes row r
                p.F[(size_t)nxt * p.n_ld + i0 + r] = Fn[r];
                p.U[(size_t)nxt * p.n_ld + i0 + r] = u[r];
            }
        }
        if (col_phase) {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    double y[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) y[r] = fma(ns, (double)cv[r][q][e], u[r]);
                    cs[q][e].template add<R>(y);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) cv[r][q][e] = ahead[r][q][e];
    }
    if (col_phase) {                              // uniform over the workgroup: every wave arrives here
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sM[wave][(q * 64 + lane) * 4 + e] = cs[q][e].M;
                sS[wave][(q * 64 + lane) * 4 + e] = cs[q][e].s;
            }
        __syncthreads();
        for (int col = tid; col < m; col += 256) {
            Lse t;
            t.M = sM[0][col]; t.s = sS[0][col];
#pragma unroll
            for (int w = 1; w < NW; ++w) t.merge(sM[w][col], sS[w][col]);
            A.colpart[(size_t)blockIdx.x * p.m_ld + col] = t.value();
        }
    }
}

// ---------------------------------------------------------------- fused pass, asynchronous LDS prefetch
// The production form of the fused pass for m in (4096, 8192].
//
// Data movement
//   * every wave owns two private LDS staging buffers of R*Q KiB.  Panel p+1 is fetched into one of
//     them with buffer_load_dwordx4 ... lds (HBM -> LDS, no registers, no wait) while panel p is
//     consumed from the other with ds_read_b128, so the HBM stream runs under all of the arithmetic;
//   * the only barrier per panel is the one that exchanges the R*16 wave sums.  It is a bare
//     s_barrier after lgkmcnt(0): a fence would also wait for the prefetch in flight;
//   * the per-row scalars of the next panel (old F, log2 a, a) are loaded one panel ahead, before
//     the prefetch is issued, because vmcnt retires in order.
//
// Arithmetic
//   row phase    The reference of row i is its previous LSE value rho_i = F_old_i.  Every lane forms
//                e_ij = 2^(x_ij - rho_i) and sums it; if the workgroup-wide sum S_i lands in
//                [2^-20, 2^60] (always, once the potentials move by less than ~20 base-2 units per
//                iteration) then F_new_i = rho_i + log2 S_i with no max pass at all.  Otherwise
//                the panel is redone with the exact running-max form of Eq. 8.
//   column phase With the new f the plan entry is pi_ij = e_ij * a_i / S_i, all of
//                them in [0, 1].  The column pass is therefore one fused multiply-add per entry:
//                T_j += e_ij * alpha_i, alpha_i = a_i / S_i, and the partial column LSE is
//                log2 T_j - V_j.  This is the classical scaling form of Sinkhorn, usable here
//                because e_ij is already stabilised by the row reference.  It cannot overflow.  What
//                it can lose is what fp32 flushes: a factor e_ij or a product pi_ij below 2^-126.
//                With alpha_i <= 2^20 (the lower limit on S_i) every entry of at least 2^-40 of a
//                column total T_j >= 2^-66 survives both, so the combine kernel recomputes exactly,
//                from C, every column whose total is below 2^-66 or not a number (a column whose
//                weight b_j is that small, or zero, always is) and trusts the others.
//   While the potentials still move fast (early iterations) the driver runs the exact streaming
//   row and column kernels instead of this one; the device reports after every iteration whether
//   at most 128 columns moved by more than 40 (base 2), and the driver follows that hint.  The hint
//   only steers performance: this kernel plus the repair is correct in either regime.
// FULLW: m == 4*Q*T, every lane owns valid columns.  Then every wave issues exactly R*Q + 5
// prefetch loads per panel, which lets the kernel keep TWO panels in flight and wait with an
// exact vmcnt (vmcnt retires in order: "at most R*Q + 5 outstanding" means "everything but the
// youngest panel has landed").  Otherwise one panel is in flight and the wait is vmcnt(0).
//
// The per-row scalars of a panel (old F, log2 a, a) travel the same way as the panel itself:
// lanes 0..R-1 of every wave fetch them with dword-sized HBM -> LDS loads next to the panel's
// loads, so nothing that is prefetched occupies a register while it is in flight.
template <int Q, int R, bool FULLW, int DT = 0>
__global__ __launch_bounds__(1024) void k_fused_pf(DenseArgs A, Ctl c) {
    constexpr int T = 1024, NW = 16;
    constexpr int EPL = DT == 0 ? 4 : 8;       // cost entries per 16-byte chunk: fp32, or fp16 / bf16 storage
    constexpr int ES = 16 / EPL;               // bytes per stored cost entry
    static_assert(R * NW <= 64, "one wave merges all (row, wave) partials in one shot");
    static_assert(5 * R <= 16, "scalar staging holds 16 dwords per wave");
    constexpr int NDMA = R * Q + 5;            // loads per panel and wave (FULLW)
    constexpr float kRowHi = 1.1529215e18f;   // 2^60
    constexpr float kRowLo = 9.5367432e-07f;  // 2^-20
    __shared__ float4 stage[2][NW][R][Q][64];
    __shared__ int scal[2][NW][16];            // [0,R) F lo  [R,2R) F hi  [2R,3R) la2 lo  [3R,4R) la2 hi  [4R,5R) a
    __shared__ float sSum[2][R][NW];
    __shared__ double sM[2][R][NW];
    __shared__ float sS[2][R][NW];
    __shared__ int scalF0[NW][4];              // old F of the first panel, for either parity of the counter
#if defined(__HIP_DEVICE_COMPILE__)
    // Everything whose address does not depend on the iteration counter is requested before the
    // counter itself has arrived: the first panel of this workgroup (always the same one), its row
    // scalars (old F from both buffers) and both copies of V.
    const unsigned long long kd = load_counter(c);
    const Pots &p = A.p;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform, and the compiler knows it
    const double ns = -p.s;
    const bool col_phase = (c.phase == 0);
    const int m = p.m, n = p.n;
    const int rr = lane / NW;                  // the panel row this lane serves in the merge
    const int rc = rr < R ? rr : R - 1;
    auto colok = [&](int q) { return FULLW || ((q * T + tid) * EPL) < m; };
    // Staged costs of group q: the 16 bytes of a lane that owns the last columns of a row run on into the
    // next row (or past the panel, where the load returns 0); those entries are zeroed here and removed
    // by V = -inf, so that nothing foreign (a NaN of the next row, say) enters this row's sum.
    auto unpack = [&](const float4 &c4, int q, float (&o)[EPL]) {
        if constexpr (DT == 0) {
            o[0] = c4.x; o[1] = c4.y; o[2] = c4.z; o[3] = c4.w;
        } else {
            const unsigned w4[4] = {__float_as_uint(c4.x), __float_as_uint(c4.y), __float_as_uint(c4.z), __float_as_uint(c4.w)};
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                o[2 * h] = cost_from_bits<DT>(w4[h] & 0xffffu);
                o[2 * h + 1] = cost_from_bits<DT>(w4[h] >> 16);
            }
        }
        if (!FULLW) {
            const int col = (q * T + tid) * EPL;
#pragma unroll
            for (int e = 1; e < EPL; ++e)
                if (col + e >= m) o[e] = 0.0f;
        }
    };

    // Lanes whose columns lie past m never receive data (their loads are masked off); their staging
    // slots are cleared once so that they read as a finite cost and V = -inf removes them.
    if (!FULLW) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int q = 0; q < Q; ++q) stage[b][wave][r][q][lane] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    // This workgroup owns the panels b, b + G, b + 2G, ... (G workgroups).  It always starts with the
    // first of them and then walks the others upwards on even iterations and downwards on odd ones, so
    // that what the last-level cache still holds from the previous pass is read first.
    const int npanels = (n + R - 1) / R;
    const int G = gridDim.x;
    const int mine = ((int)blockIdx.x < npanels) ? (npanels - 1 - (int)blockIdx.x) / G + 1 : 0;
    const __amdgpu_buffer_rsrc_t rsF0 = __builtin_amdgcn_make_buffer_rsrc((void *)p.F, 0, p.n_ld * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsF1 =
        __builtin_amdgcn_make_buffer_rsrc((void *)(p.F + p.n_ld), 0, p.n_ld * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsL = __builtin_amdgcn_make_buffer_rsrc((void *)p.la2, 0, n * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc((void *)p.a, 0, n * 4, 0x00020000);
    // HBM -> LDS prefetch of one panel (rows i0, i0 + 1, ...) and of its weights into staging buffer
    // `buf`.  The descriptors of C and of the weights cover exactly the valid rows, so rows past n read as zero;
    // their old F comes from the padding of F, which holds kPadF: every term of such a row is exactly 0.
    // Per-lane offsets stay loop-invariant (lane * 8, tid * 16); everything that changes from load to
    // load goes through the scalar offset operand.  (The instruction's immediate offset is not used:
    // it would shift the LDS destination as well as the memory address.)
    auto issue_data = [&](int i0, int buf) {
        const int rows = (n - i0) < R ? (n - i0) : R;
        if (lane < R) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsL, &scal[buf][wave][2 * R], 4, lane * 8, i0 * 8, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsL, &scal[buf][wave][3 * R], 4, lane * 8, i0 * 8 + 4, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, &scal[buf][wave][4 * R], 4, lane * 4, i0 * 4, 0, 0);
        }
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((const char *)A.C + (size_t)i0 * m * ES), 0, rows * m * ES, 0x00020000);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int q = 0; q < Q; ++q)
                if (colok(q))
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, &stage[buf][wave][r][q][0], 16,
                                                             tid * 16, (r * m + q * T * EPL) * ES, 0, 0);
    };
    // old F of the rows of a panel, from the buffer the counter names
    auto issue_F = [&](const __amdgpu_buffer_rsrc_t &rsF, int i0, int *dst) {
        if (lane < R) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsF, dst, 4, lane * 8, i0 * 8, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsF, dst + R, 4, lane * 8, i0 * 8 + 4, 0, 0);
        }
    };
    static_assert(2 * R <= 4, "scalF0 holds two dwords per row and parity");

    // both copies of V while the counter is on its way (narrow shapes only: 16 Q registers each)
    constexpr bool kBothV = Q * EPL <= 8;
    constexpr int QV = kBothV ? Q : 1;
    double v0[QV][EPL], v1[QV][EPL];
    if constexpr (kBothV) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int col = (q * T + tid) * EPL;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const bool ok = FULLW || col + e < m;          // m need not be a multiple of 4
                v0[q][e] = ok ? p.V[col + e] : -__builtin_huge_val();
                v1[q][e] = ok ? p.V[(size_t)p.m_ld + col + e] : -__builtin_huge_val();
            }
        }
    }
    if (mine > 0) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);        // the clearing stores above are done
        issue_data((int)blockIdx.x * R, 0);
        // both candidates for the old F of the first panel: parity 0 -> scalF0[wave][0..2R), parity 1 -> scal[0]
        issue_F(rsF0, (int)blockIdx.x * R, &scalF0[wave][0]);
        issue_F(rsF1, (int)blockIdx.x * R, &scal[0][wave][0]);
        asm volatile("" ::: "memory");
    }

    int k;
    if (!counter_active(c, kd, k)) {
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0)); // no prefetch may land after the workgroup has given up its LDS
        return;
    }
    const int cur = k & 1, nxt = cur ^ 1;
    const bool rev = cur != 0;
    const __amdgpu_buffer_rsrc_t rsF = cur ? rsF1 : rsF0;
    // row index of the t-th panel this workgroup processes
    auto panel_row = [&](int t) { return ((int)blockIdx.x + (t == 0 ? 0 : (rev ? mine - t : t)) * G) * R; };
    auto issue = [&](int t, int buf) {
        const int i0 = panel_row(t);
        issue_F(rsF, i0, &scal[buf][wave][0]);
        issue_data(i0, buf);
    };
    double v[Q][EPL];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int col = (q * T + tid) * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            if constexpr (kBothV) v[q][e] = cur ? v1[q][e] : v0[q][e];
            else v[q][e] = (FULLW || col + e < m) ? p.V[(size_t)cur * p.m_ld + col + e] : -__builtin_huge_val();
        }
    }
    float cS[Q][EPL];                            // column sums of the plan entries
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int e = 0; e < EPL; ++e) cS[q][e] = 0.0f;

    if (FULLW && mine > 1) {
        asm volatile("" ::: "memory");
        issue(1, 1);
        asm volatile("" ::: "memory");
    }
    int buf = 0;
    for (int t = 0; t < mine; ++t, buf ^= 1) {
        const int i0 = panel_row(t);
        // Panel t and its row scalars must have landed.  FULLW: the only younger VMEM operations are
        // the NDMA prefetch loads of the next panel (if there is one), which may stay in flight.
        if (FULLW && t + 1 < mine) __builtin_amdgcn_s_waitcnt(waitcnt_vm(NDMA));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        asm volatile("" ::: "memory");             // no LDS read of the staging buffers may move above the wait
        const int *sc = scal[buf][wave];
        const int *scF = (t == 0 && cur == 0) ? scalF0[wave] : sc;
        const bool rowok = rr < R && (i0 + rr) < n;
        const double rho_lane = __hiloint2double(scF[R + rc], scF[rc]);
        const double la2_lane = rowok ? __hiloint2double(sc[3 * R + rc], sc[2 * R + rc]) : -__builtin_huge_val();
        const float a_lane = rowok ? __int_as_float(sc[4 * R + rc]) : 0.0f;
        double rho[R];
#pragma unroll
        for (int r = 0; r < R; ++r) rho[r] = __hiloint2double(scF[R + r], scF[r]);
        if (!FULLW && t + 1 < mine) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(0xc07f);    // every earlier read of the other staging buffer has returned
            issue(t + 1, buf ^ 1);
            asm volatile("" ::: "memory");
        }
        // FULLW: prefetch of the panel after next into the buffer this panel occupies, as soon as the
        // last read of that buffer has returned
        auto issue_ahead = [&]() {
            if (FULLW && t + 2 < mine) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xc07f);
                issue(t + 2, buf);
                asm volatile("" ::: "memory");
            }
        };
        // ---- row phase, optimistic: e = 2^(x - rho_r), summed
        float ev[R][Q][EPL];
        float racc[R];                     // (Q == 1 only)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float acc = 0.0f;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const float4 c4 = stage[buf][wave][r][q][lane];
                float cvv[EPL];
                unpack(c4, q, cvv);
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    ev[r][q][e] = fast_exp2((float)(fma(ns, (double)cvv[e], v[q][e]) - rho[r]));
                    acc += ev[r][q][e];
                }
            }
            if constexpr (Q == 1) {
                racc[r] = acc;       // two rows per lane exchange, below
            } else {
                // (with more columns per lane the kernel is at its register limit and the two-row form spills)
                acc = wave_sum_f32(acc);
                if (lane == 0) sSum[buf][r][wave] = acc;
            }
        }
        if constexpr (Q == 1) rows_sum_store<R>(racc, &sSum[buf][0][wave], NW, lane);
        lds_only_barrier();
        float S = rr < R ? sSum[buf][rc][lane % NW] : 1.0f;
        S += dpp_f32<0x128>(S);
        S += dpp_f32<0x124>(S);
        S += dpp_f32<0x122>(S);
        S += dpp_f32<0x121>(S);
        const bool fine = (S >= kRowLo) && (S <= kRowHi);    // false for NaN / inf / 0
        double Fn_lane = rho_lane + log2_sum(S);
        float alpha_lane = a_lane / S;                        // pi_ij = e_ij * a_i / S_i
        if (__builtin_expect(!__all(fine || !rowok), 0)) {
            // ---- exact redo of the row phase of this panel (uniform over the workgroup: every wave
            //      sees the same sums)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                Lse rs; rs.init();
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const float4 c4 = stage[buf][wave][r][q][lane];
                    float cvv[EPL];
                unpack(c4, q, cvv);
                    double x[EPL];
#pragma unroll
                    for (int e = 0; e < EPL; ++e) x[e] = fma(ns, (double)cvv[e], v[q][e]);
                    rs.template add<EPL>(x);
                }
                rs.wave_reduce();
                if (lane == 0) { sM[buf][r][wave] = rs.M; sS[buf][r][wave] = rs.s; }
            }
            lds_only_barrier();
            Lse t; t.init();
            if (rr < R) { t.M = sM[buf][rc][lane % NW]; t.s = sS[buf][rc][lane % NW]; }
            double Mg = t.M;
            Mg = dmax(Mg, dpp_f64<0x128>(Mg));
            Mg = dmax(Mg, dpp_f64<0x124>(Mg));
            Mg = dmax(Mg, dpp_f64<0x122>(Mg));
            Mg = dmax(Mg, dpp_f64<0x121>(Mg));
            float sg = t.s * fast_exp2((float)(t.M - Mg));
            sg += dpp_f32<0x128>(sg);
            sg += dpp_f32<0x124>(sg);
            sg += dpp_f32<0x122>(sg);
            sg += dpp_f32<0x121>(sg);
            Fn_lane = Mg + log2_sum(sg);
            alpha_lane = a_lane;                               // e is re-based on the new F below
            if (col_phase) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const double Fn = bcast_f64(Fn_lane, r * NW);
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        const float4 c4 = stage[buf][wave][r][q][lane];
                        float cvv[EPL];
                unpack(c4, q, cvv);
#pragma unroll
                        for (int e = 0; e < EPL; ++e)
                            ev[r][q][e] = fast_exp2((float)(fma(ns, (double)cvv[e], v[q][e]) - Fn));
                    }
                }
            }
        }
        if (wave == 0 && (lane % NW) == 0 && rowok) {
            p.F[(size_t)nxt * p.n_ld + i0 + rr] = Fn_lane;
            p.U[(size_t)nxt * p.n_ld + i0 + rr] = la2_lane - Fn_lane;
        }
        // ---- column phase with the new f: nothing below reads the stage any more
        issue_ahead();
        if (col_phase) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float alpha = bcast_f32(alpha_lane, r * NW);
                if (!(alpha == alpha) || (i0 + r) >= n) alpha = 0.0f;   // rows past n, or a row whose F is not finite
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) cS[q][e] = fmaf(ev[r][q][e], alpha, cS[q][e]);
            }
        }
    }
    if (col_phase) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int col = (q * T + tid) * EPL;
            if (colok(q)) {
                // The partial of this workgroup is the plain fp32 sum T_j of its plan entries: all
                // workgroups share the reference V_j, so the combine kernel only has to add them up
                // (G_j = log2 sum_p T_j - V_j).
                float *row = reinterpret_cast<float *>(A.colpart) + (size_t)blockIdx.x * p.m_ld + col;
#pragma unroll
                for (int h = 0; h < EPL / 4; ++h)
                    reinterpret_cast<float4 *>(row)[h] =
                        make_float4(cS[q][4 * h], cS[q][4 * h + 1], cS[q][4 * h + 2], cS[q][4 * h + 3]);
            }
        }
    }
#endif
}

// Which fused kernel a width gets.  T = 256, 512, 1024: k_fused<T, Q, R> (T lanes on columns, Q groups of 4 columns
// per lane, R rows per panel).  R = 301 / 302: k_fused_pf<Q, R - 300> (LDS prefetch, 1024 lanes).  T = 64:
// k_fused_rows<Q, R> (one wave per row, 4 waves per workgroup).  R % 100 is the number of rows per panel throughout.
struct FusedShape { int T, Q, R; };

// Workgroups the 256 compute units hold at once.
// k_fused_pf<1, 2, true> (m = 4096, fp32: 55 registers, 67 KiB of LDS) fits twice; with at least 16 panels per
// workgroup that is worth it (16384 x 4096: 60.7 -> 52.7 us per iteration), below and for the masked widths it is not.
static int fused_resident(const FusedShape &s, int c_dtype, int n, int m) {
    // one wave per row: 1024 workgroups once every wave still gets 4 panels, else 512 (half the column partials
    // for k_combine; 8192 x 512: 16.7 against 21.1 us per iteration, 100000 x 512: 86.5 against 73.8)
    if (s.T == 64) return (n + s.R - 1) / s.R >= 16384 ? 1024 : 512;
    if (s.T == 256) return 1024;
    if (s.R == 302 && s.Q == 1 && c_dtype == 0 && m == 4096 && n >= 8192) return 512;
    return 256;
}

// Shapes held in registers without spilling: 4*Q*T columns, R rows per panel.
static bool fused_shape(int m, int variant, int c_dtype, FusedShape *fsh) {
    if (variant >= 100) variant -= 100;
    if (c_dtype != 0) {
        // 2-byte costs: LDS-prefetch kernels only, 8 columns per lane and group, rows of whole 16-byte chunks
        if (m % 8 != 0 || m <= 2048 || m > 16384) return false;
        *fsh = {1024, m <= 8192 ? 1 : 2, m <= 8192 ? 302 : 301};
        return true;
    }
    // The LDS-prefetch kernels take any m (a row may start at any 4-byte boundary; columns past m are
    // masked by V = -inf); the register-panel kernels need whole groups of 4 columns.
    if (m % 4 != 0) {
        if (m <= 1024) return false;
        if (m <= 8192) variant = 0;
    }
    if (m <= 512 && variant != 1) { *fsh = {64, m <= 256 ? 1 : 2, m <= 256 ? 4 : 2}; return true; }    // one wave per row
    if (m <= 1024) { *fsh = {256, 1, 4}; return true; }
    if (m <= 4096) {
        if (variant == 1) *fsh = {1024, 1, 4};               // register panel, exact running-max arithmetic
        else *fsh = {1024, 1, 302};                          // asynchronous LDS prefetch, one 16-byte load per lane and row
        return true;
    }
    if (m > 8192 && m <= 16384) {
        *fsh = {1024, m <= 12288 ? 3 : 4, 301};              // asynchronous LDS prefetch, one row per panel
        return true;
    }
    if (m <= 8192) {
        if (variant == 1) *fsh = {512, 4, 4};
        else if (variant == 2) *fsh = {1024, 2, 4};
        else if (variant == 3) *fsh = {512, 4, 2};
        else if (variant == 4) *fsh = {1024, 2, 2};
        else if (variant == 5) *fsh = {1024, 2, 302};        // LDS prefetch, one panel in flight even at full width
        else *fsh = {1024, 2, 302};                          // asynchronous LDS prefetch, R = 2
        return true;
    }
    return false;
}

bool dense_fused_supported(int n, int m, const void *C, int c_dtype) {
    FusedShape s;
    (void)n;
    const uintptr_t mask = c_dtype != 0 ? 15u : 3u;
    return fused_shape(m, 0, c_dtype, &s) && ((reinterpret_cast<uintptr_t>(C) & mask) == 0);
}

void dense_fused_plan(int n, int m, int *P) {
    // the largest grid any variant uses: one panel set per resident workgroup
    FusedShape s{256, 1, 4};
    int best = 1;
    for (int variant = 0; variant < 8; ++variant) {        // 6, 7: the shapes for 2-byte costs
        if (!fused_shape(m, variant < 6 ? variant : 0, variant < 6 ? 0 : variant - 5, &s)) continue;
        int npanels = (n + (s.R % 100) - 1) / (s.R % 100);
        if (s.T == 64) npanels = (npanels + 3) / 4;        // four waves, a panel each
        const int resident = fused_resident(s, variant < 6 ? 0 : variant - 5, n, m);
        const int p = npanels < resident ? npanels : resident;
        if (p > best) best = p;
    }
    *P = best;
}

hipError_t launch_dense_fused(hipStream_t st, const DenseArgs &a, const Ctl &c, int variant, const Stamp &tm) {
    FusedShape s;
    if (!fused_shape(a.p.m, variant, a.c_dtype, &s)) return hipErrorInvalidValue;
    int npanels = (a.p.n + (s.R % 100) - 1) / (s.R % 100);
    if (s.T == 64) npanels = (npanels + 3) / 4;
    const int resident = fused_resident(s, a.c_dtype, a.p.n, a.p.m);
    int g = npanels < resident ? npanels : resident;
    if (g > a.P) g = a.P;
    DenseArgs b = a;
    b.P = g;
    const dim3 grid(g);
    if (a.c_dtype != 0) {
        const bool full = a.p.m == s.Q * 8192;
        const int key = (a.c_dtype == 1 ? 0 : 4) + (s.Q == 1 ? 0 : 2) + (full ? 0 : 1);
        switch (key) {
        case 0: launch_stamped((k_fused_pf<1, 2, true, 1>), grid, dim3(1024), st, tm, b, c); break;
        case 1: launch_stamped((k_fused_pf<1, 2, false, 1>), grid, dim3(1024), st, tm, b, c); break;
        case 2: launch_stamped((k_fused_pf<2, 1, true, 1>), grid, dim3(1024), st, tm, b, c); break;
        case 3: launch_stamped((k_fused_pf<2, 1, false, 1>), grid, dim3(1024), st, tm, b, c); break;
        case 4: launch_stamped((k_fused_pf<1, 2, true, 2>), grid, dim3(1024), st, tm, b, c); break;
        case 5: launch_stamped((k_fused_pf<1, 2, false, 2>), grid, dim3(1024), st, tm, b, c); break;
        case 6: launch_stamped((k_fused_pf<2, 1, true, 2>), grid, dim3(1024), st, tm, b, c); break;
        default: launch_stamped((k_fused_pf<2, 1, false, 2>), grid, dim3(1024), st, tm, b, c); break;
        }
        return hipGetLastError();
    }
    if (s.R == 301 && s.Q == 3 && a.p.m == 12288) launch_stamped((k_fused_pf<3, 1, true>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 301 && s.Q == 3) launch_stamped((k_fused_pf<3, 1, false>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 301 && a.p.m == 16384) launch_stamped((k_fused_pf<4, 1, true>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 301) launch_stamped((k_fused_pf<4, 1, false>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 302 && s.Q == 1 && a.p.m == 4096) launch_stamped((k_fused_pf<1, 2, true>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 302 && s.Q == 1) launch_stamped((k_fused_pf<1, 2, false>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 302 && a.p.m == 8192 && variant % 100 != 5) launch_stamped((k_fused_pf<2, 2, true>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 302) launch_stamped((k_fused_pf<2, 2, false>), grid, dim3(1024), st, tm, b, c);
    else if (s.T == 64 && s.Q == 1) launch_stamped((k_fused_rows<1, 4>), grid, dim3(256), st, tm, b, c);
    else if (s.T == 64) launch_stamped((k_fused_rows<2, 2>), grid, dim3(256), st, tm, b, c);
    else if (s.T == 256) launch_stamped((k_fused<256, 1, 4>), grid, dim3(256), st, tm, b, c);
    else if (s.T == 1024 && s.Q == 1) launch_stamped((k_fused<1024, 1, 4>), grid, dim3(1024), st, tm, b, c);
    else if (s.T == 1024 && s.R == 2) launch_stamped((k_fused<1024, 2, 2>), grid, dim3(1024), st, tm, b, c);
    else if (s.T == 1024) launch_stamped((k_fused<1024, 2, 4>), grid, dim3(1024), st, tm, b, c);
    else if (s.R == 2) launch_stamped((k_fused<512, 4, 2>), grid, dim3(512), st, tm, b, c);
    else launch_stamped((k_fused<512, 4, 4>), grid, dim3(512), st, tm, b, c);
    return hipGetLastError();
}

bool dense_fused_predicts(int m, int variant, int c_dtype) {
    FusedShape s;
    return fused_shape(m, variant, c_dtype, &s) && s.R > 300;
}

// number of column-partial sets the fused launch of this shape writes
int dense_fused_grid(int n, int m, int variant, int c_dtype) {
    FusedShape s;
    if (!fused_shape(m, variant, c_dtype, &s)) return 0;
    int npanels = (n + (s.R % 100) - 1) / (s.R % 100);
    if (s.T == 64) npanels = (npanels + 3) / 4;
    const int resident = fused_resident(s, c_dtype, n, m);
    return npanels < resident ? npanels : resident;
}

}  // namespace fs
