// Mid-size problems (n, m <= 1024; dense cost or point clouds): the whole of Alg. 1 inside ONE kernel launch spread
// over up to 32 workgroups, the cost matrix (or the table of squared distances) held in registers for the entire solve, ONE grid-wide exchange per
// iteration.  The multi-kernel driver spends 11 - 13 us per iteration at these sizes on its chain of
// dependent launches; here an iteration costs the arithmetic of a few registers per lane plus one
// round of "publish partials, wait for everyone, read everyone's partials".
//
// Decomposition.  Workgroup w owns 4 RA consecutive rows and ALL columns, so the f-update (Eq. 9) is
// local.  The g-update (Eq. 10) needs every row: each workgroup reduces its rows to one partial
// base-2 LSE value per column, publishes the m values, and after the grid-wide wait every workgroup
// merges all W partials per column itself (W m doubles, a few KiB) - every workgroup ends up with the
// same g, bit for bit, and nothing else has to be communicated.  The error terms of Sec. 4.5 travel
// with the partials, so every workgroup also takes the same stop decision without a second exchange.
//
// Layout inside a workgroup: 1024 lanes = 256 column lanes x 4 row groups; lane (tc, tr) keeps the
// entries (row0 + tr RA + a, tc + 256 b), a < RA, b < CB, in registers.  Row LSE: wave all-reduce
// (DPP), then the 4 waves of a row group meet in LDS.  Column LSE: lane-local over RA rows, the 4 row
// groups meet in LDS.  Arithmetic as everywhere else: exponent arguments in fp64 (base 2), v_exp_f32
// and the sums in fp32.
//
// Exchange without cache maintenance: partials are written with agent-scope relaxed atomic stores
// (write-through to the level all compute dies share) and read back with agent-scope relaxed atomic
// loads; every thread waits for its own stores (vmcnt 0) before the workgroup's arrival is counted.
// The arrival counter only grows (generation g is complete at W g arrivals), the exchange buffers
// alternate by the parity of the generation, and every wait is bounded: a workgroup that gives up
// raises a flag that makes all others give up too, the solve then reports that it gave up
// (nonfinite = 2, NaN potentials where a workgroup had stopped) instead of hanging.
#include <type_traits>

#include "fs_kernels.h"

namespace fs {

namespace {

constexpr int kCT = 1024;              // threads per workgroup
constexpr int kTC = 256;               // column lanes
constexpr int kTR = kCT / kTC;         // row groups
constexpr int kNWR = kTC / 64;         // waves per row group
constexpr int kRowsMax = kTR * 8;      // rows per workgroup at RA = 8

__device__ __forceinline__ void publish(double *p, double v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double fetch(const double *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Grid-wide wait number `gen` (1, 2, ...).  Every thread of the workgroup calls it after its last
// store of the round.  Returns false when the wait was abandoned (by this workgroup or by another).
__device__ __forceinline__ bool grid_wait(CoopSync *sy, unsigned long long gen, int W, int spin_limit, int *s_ok) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0);                       // this thread's published values have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        int good = 1;
        __hip_atomic_fetch_add(&sy->arrivals, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long target = gen * (unsigned long long)W;
        int spins = 0;
        while (__hip_atomic_load(&sy->arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++spins > spin_limit || __hip_atomic_load(&sy->abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                good = 0;
                __hip_atomic_store(&sy->abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        *s_ok = good;
    }
    __syncthreads();
    return *s_ok != 0;
#else
    return false;
#endif
}

__global__ void k_coop_reset(CoopSync *sy) {
    if (threadIdx.x == 0) {
        sy->arrivals = 0ull;
        sy->abort_flag = 0u;
        sy->bad = 0u;
    }
}

// PTS: point clouds - the tile holds |x_i - y_j|^2 in fp64, formed once from the fp32 coordinates in the
// difference form (nothing of the cost is rounded to fp32 on this path either).
template <int RA, int CB, bool PTS>
__global__ __launch_bounds__(kCT) void k_coop(CoopArgs A) {
    __shared__ double sF[2][kRowsMax];             // F = -s f of the workgroup's rows, by parity of k
    __shared__ double sLa[kRowsMax];               // log2 a
    __shared__ float sAw[kRowsMax];                // a
    __shared__ double sRM[kTR][RA][kNWR];          // row LSE: per-wave maxima and sums
    __shared__ float sRS[kTR][RA][kNWR];
    __shared__ double sCM[kTR][kTC * CB];          // column LSE: per-row-group maxima and sums
    __shared__ float sCS[kTR][kTC * CB];
    __shared__ double sV[kTC * CB];
    __shared__ double sErrG[kTR];
    __shared__ double sErrTot;
    __shared__ int sOk, sBad;

#if defined(__HIP_DEVICE_COMPILE__)
    const int n = A.n, m = A.m;
    const int W = gridDim.x, w = blockIdx.x;
    const int tid = threadIdx.x, tc = tid % kTC, tr = tid / kTC, lane = tid & 63, wave = tid >> 6;
    const int wr = wave % kNWR;
    constexpr int RWG = kTR * RA;                  // rows per workgroup
    const int row0 = w * RWG;
    const double s = A.s, ns = -A.s;
    const double ninf = -__builtin_huge_val();
    double *xchg = A.xchg;
    const size_t xstride = (size_t)W * A.ldx;      // one parity of the exchange buffer

    // ---- start: weights, initial potentials (zero, Eqs. 6-7, or the caller's), the cost tile
    if (tid < RWG) {
        const int i = row0 + tid;
        const float wgt = i < n ? A.a[i] : 0.0f;
        sAw[tid] = wgt;
        sLa[tid] = i < n ? log2_weight(wgt) : ninf;
        double F0 = 0.0;
        if (A.warm && i < n) F0 = ns * (A.f64_in ? A.f64_in[i] : (double)A.f_in[i]);
        sF[0][tid] = F0;
        sF[1][tid] = F0;
    }
    if (tid == 0) sBad = 0;
    // column t of the problem is looked after by thread t (all workgroups hold the same values)
    const bool colthread = tid < kTC * CB;
    double lb2 = ninf, Gt = 0.0;
    if (colthread && tid < m) {
        lb2 = log2_weight(A.b[tid]);
        if (A.warm) Gt = ns * (A.g64_in ? A.g64_in[tid] : (double)A.g_in[tid]);
    }
    if (colthread) sV[tid] = tid < m ? lb2 - Gt : ninf;
    typename std::conditional<PTS, double, float>::type c[RA][CB];
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            const int i = row0 + tr * RA + a, j = tc + kTC * b;
            if constexpr (PTS) {
                double sq = 0.0;
                if (i < n && j < m)
                    for (int t = 0; t < A.d; ++t) {
                        const double df = (double)A.X[(size_t)i * A.d + t] - (double)A.Y[(size_t)j * A.d + t];
                        sq = fma(df, df, sq);
                    }
                c[a][b] = sq;
            } else {
                c[a][b] = (i < n && j < m) ? cost_entry(A.C, A.c_dtype, (size_t)i * m + j) : 0.0f;
            }
        }
    __syncthreads();
    double V[CB];
#pragma unroll
    for (int b = 0; b < CB; ++b) V[b] = sV[tc + kTC * b];

    int iters = A.max_iter, converged = 0;
    double err_out = __builtin_nan("");
    unsigned long long gen = 0;
    bool alive = true;
    int k = 0;
    for (;; ++k) {
        const bool trailing = (k == A.max_iter);
        const bool checked = A.tol > 0.0 && k >= 1 && (k % A.check_every == 0);
        const bool hist = A.err_history && k >= 1 && (k - 1) < A.err_history_len;
        const bool need_err = k >= 1 && (checked || hist || (trailing && A.want_final_err));
        if (trailing && !need_err) break;
        const int cur = k & 1, nxt = cur ^ 1;
        const int par = (int)(gen & 1ull);
        double *xw = xchg + (size_t)par * xstride + (size_t)w * A.ldx;      // this workgroup's slots of this round

        // ---- f-update (Eq. 9): F_i = LSE2_j(V_j - s C_ij) over the whole row
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            double mx = kNegHuge;
#pragma unroll
            for (int b = 0; b < CB; ++b) mx = dmax(mx, fma(ns, cost_f64(c[a][b]), V[b]));
            mx = wave_max_f64(mx);
            float sm = 0.0f;
#pragma unroll
            for (int b = 0; b < CB; ++b) sm += fast_exp2((float)(fma(ns, cost_f64(c[a][b]), V[b]) - mx));
            sm = wave_sum_f32(sm);
            if (lane == 0) { sRM[tr][a][wr] = mx; sRS[tr][a][wr] = sm; }
        }
        __syncthreads();
        double Fnew[RA];
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            double mx = sRM[tr][a][0];
#pragma unroll
            for (int q = 1; q < kNWR; ++q) mx = dmax(mx, sRM[tr][a][q]);
            float sm = 0.0f;
#pragma unroll
            for (int q = 0; q < kNWR; ++q) sm += sRS[tr][a][q] * fast_exp2((float)(sRM[tr][a][q] - mx));
            Fnew[a] = mx + log2_sum(sm);
        }
        // the new F goes to the other buffer: should this round turn out to be the one that stops, the
        // iterate to return (old F, current G) is still there
        {
            // lane tc < RA of a row group looks after row tc of the group: it stores the new F and evaluates
            // the error term of Sec. 4.5 for that row, a_i |2^(Fnew_i - Fold_i) - 1|
            double fn = Fnew[0];
#pragma unroll
            for (int a = 1; a < RA; ++a) fn = (tc == a) ? Fnew[a] : fn;
            double e = 0.0;
            if (tc < RA) {
                const int li = tr * RA + tc;
                sF[nxt][li] = fn;
                if (need_err) {
                    const float wgt = sAw[li];
                    if (wgt > 0.0f) e = (double)wgt * fabs(exp2m1(fn - sF[cur][li]));
                }
            }
            if (wr == 0) {                     // lanes 0 .. RA-1 of the first wave of the row group hold the terms
                double tot = 0.0;
#pragma unroll
                for (int a = 0; a < RA; ++a) tot += bcast_f64(e, a);      // fixed order
                if (lane == 0) sErrG[tr] = tot;
            }
        }

        // ---- g-update (Eq. 10) with the new f, this workgroup's rows only: one partial LSE per column
        if (!trailing) {
            double U[RA];
#pragma unroll
            for (int a = 0; a < RA; ++a) U[a] = sLa[tr * RA + a] - Fnew[a];       // -inf for rows past n
#pragma unroll
            for (int b = 0; b < CB; ++b) {
                double mx = kNegHuge;
#pragma unroll
                for (int a = 0; a < RA; ++a) mx = dmax(mx, fma(ns, cost_f64(c[a][b]), U[a]));
                float sm = 0.0f;
#pragma unroll
                for (int a = 0; a < RA; ++a) sm += fast_exp2((float)(fma(ns, cost_f64(c[a][b]), U[a]) - mx));
                sCM[tr][tc + kTC * b] = mx;
                sCS[tr][tc + kTC * b] = sm;
            }
        }
        __syncthreads();
        if (!trailing && colthread && tid < m) {
            double mx = sCM[0][tid];
#pragma unroll
            for (int q = 1; q < kTR; ++q) mx = dmax(mx, sCM[q][tid]);
            float sm = 0.0f;
#pragma unroll
            for (int q = 0; q < kTR; ++q) sm += sCS[q][tid] * fast_exp2((float)(sCM[q][tid] - mx));
            publish(xw + tid, mx + log2_sum(sm));
        }
        if (tid == 0) publish(xw + A.ldx - 1, (sErrG[0] + sErrG[1]) + (sErrG[2] + sErrG[3]));

        // ---- everyone's partials
        if (!grid_wait(A.sync, ++gen, W, A.spin_limit, &sOk)) { alive = false; break; }
        const double *xr = xchg + (size_t)par * xstride;
        double Gnew = Gt;
        if (!trailing && colthread && tid < m) {
            double pv[32];
#pragma unroll
            for (int q = 0; q < 32; ++q) pv[q] = q < W ? fetch(xr + (size_t)q * A.ldx + tid) : kNegHuge;
            double mx = pv[0];
#pragma unroll
            for (int q = 1; q < 32; ++q) mx = dmax(mx, pv[q]);
            float sm = 0.0f;
#pragma unroll
            for (int q = 0; q < 32; ++q) sm += fast_exp2((float)(pv[q] - mx));
            Gnew = mx + log2_sum(sm);
            sV[tid] = lb2 - Gnew;
        }
        if (wave == kCT / 64 - 1) {
            // the error of the iterate this round started from: the same W terms in the same order everywhere
            double e = (need_err && lane < W) ? fetch(xr + (size_t)lane * A.ldx + A.ldx - 1) : 0.0;
            e = wave_sum_f64(e);
            if (lane == 0) sErrTot = e;
        }
        __syncthreads();
        if (need_err) {
            const double err = sErrTot;
            if (hist && w == 0 && tid == 0) A.err_history[k - 1] = (float)err;
            if (trailing) {
                iters = k;
                converged = (checked && err < A.tol) ? 1 : 0;
                err_out = err;
                break;
            }
            if (checked && err < A.tol) {          // stop at k: sF[cur] and Gt still hold iterate k
                iters = k;
                converged = 1;
                err_out = err;
                break;
            }
        }
        Gt = Gnew;
#pragma unroll
        for (int b = 0; b < CB; ++b) V[b] = sV[tc + kTC * b];
    }

    // ---- results: f = -F/s, g = -G/s of the returned iterate (k = iters at every regular exit of the loop)
    __syncthreads();
    const double inv = -1.0 / s;
    const double nan = __builtin_nan("");
    bool bad = false;
    if (tid < RWG && row0 + tid < n) {
        const double v = alive ? sF[iters & 1][tid] * inv : nan;
        A.f[row0 + tid] = (float)v;
        if (A.f64_out) A.f64_out[row0 + tid] = v;
        bad |= !(fabs(v) <= 1.7e308);
    }
    if (w == 0 && colthread && tid < m) {
        const double v = alive ? Gt * inv : nan;
        A.g[tid] = (float)v;
        if (A.g64_out) A.g64_out[tid] = v;
        bad |= !(fabs(v) <= 1.7e308);
    }
    if (bad) atomicOr(&sBad, 1);
    __syncthreads();
    if (tid == 0 && sBad) __hip_atomic_fetch_or(&A.sync->bad, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // one more round so that workgroup 0 sees every workgroup's flag (skipped once a wait has been abandoned)
    if (alive) alive = grid_wait(A.sync, ++gen, W, A.spin_limit, &sOk);
    if (w == 0 && tid == 0 && A.result) {
        ResultRecord r;
        r.iters = alive ? iters : k;
        r.converged = alive ? converged : 0;
        r.nonfinite = alive ? (int)__hip_atomic_load(&A.sync->bad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : kGaveUp;
        r.marginal_err = alive ? (float)err_out : __builtin_nanf("");
        A.result[0] = r;
        __threadfence_system();
    }
#endif
}

template <int RA, bool PTS>
hipError_t launch_cb(hipStream_t st, const CoopArgs &a, int W, int cb) {
    const dim3 grid(W), block(kCT);
    if (cb <= 1) hipLaunchKernelGGL((k_coop<RA, 1, PTS>), grid, block, 0, st, a);
    else if (cb <= 2) hipLaunchKernelGGL((k_coop<RA, 2, PTS>), grid, block, 0, st, a);
    else if constexpr (PTS && RA == 8) return hipErrorInvalidValue;       // 32 fp64 entries per lane: not built
    else hipLaunchKernelGGL((k_coop<RA, 4, PTS>), grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace

bool coop_supported(int n, int m) { return n >= 1 && m >= 1 && m <= kCoopMax && n <= kCoopMax; }

// Tile per lane: RA rows (the smallest of 1, 2, 4, 8 that keeps the grid within wmax workgroups) x CB columns.
static void coop_tile(int n, int m, int wmax, int *RA, int *CB) {
    int ra = 8;
    for (int r = 1; r <= 8; r *= 2)
        if ((n + kTR * r - 1) / (kTR * r) <= wmax) { ra = r; break; }
    const int cb = (m + kTC - 1) / kTC;
    *RA = ra;
    *CB = cb <= 1 ? 1 : cb <= 2 ? 2 : 4;
}

// point clouds: the tile is fp64, so half as many entries per lane (at most 16, with the largest grid)
bool coop_points_supported(int n, int m) {
    if (!coop_supported(n, m)) return false;
    int RA, CB;
    coop_tile(n, m, 32, &RA, &CB);
    return RA * CB <= 16;
}

constexpr int kCoopWMax = 32;                    // workgroups at most: each reads every other's partials
constexpr int kCoopLdx = kCoopMax + 32;

size_t coop_scratch_bytes() {
    return sizeof(double) * 2 * kCoopWMax * (size_t)kCoopLdx + sizeof(CoopSync);
}

hipError_t launch_coop(hipStream_t st, const CoopArgs &a0, void *scratch, int variant) {
    if (!coop_supported(a0.n, a0.m) || !scratch) return hipErrorInvalidValue;
    if (a0.X && (!a0.Y || a0.d < 1 || !coop_points_supported(a0.n, a0.m))) return hipErrorInvalidValue;
    // fewer workgroups on request (more rows per lane); point clouds always take the largest grid
    const int wmax = a0.X ? kCoopWMax : variant == 1 ? 16 : variant == 2 ? 8 : variant == 3 ? 4 : kCoopWMax;
    int RA, CB;
    coop_tile(a0.n, a0.m, wmax, &RA, &CB);
    const int W = (a0.n + kTR * RA - 1) / (kTR * RA);
    if (W < 1 || W > kCoopWMax) return hipErrorInvalidValue;      // cannot happen for n <= kCoopMax
    CoopArgs a = a0;
    a.ldx = kCoopLdx;
    a.xchg = reinterpret_cast<double *>(scratch);
    a.sync = reinterpret_cast<CoopSync *>(reinterpret_cast<char *>(scratch) + sizeof(double) * 2 * kCoopWMax * (size_t)kCoopLdx);
    if (a.spin_limit <= 0) a.spin_limit = 1 << 21;
    hipLaunchKernelGGL(k_coop_reset, dim3(1), dim3(64), 0, st, a.sync);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int cb = CB;
    if (a.X) {
        if (RA == 1) return launch_cb<1, true>(st, a, W, cb);
        if (RA == 2) return launch_cb<2, true>(st, a, W, cb);
        if (RA == 4) return launch_cb<4, true>(st, a, W, cb);
        return launch_cb<8, true>(st, a, W, cb);
    }
    if (RA == 1) return launch_cb<1, false>(st, a, W, cb);
    if (RA == 2) return launch_cb<2, false>(st, a, W, cb);
    if (RA == 4) return launch_cb<4, false>(st, a, W, cb);
    return launch_cb<8, false>(st, a, W, cb);
}

}  // namespace fs
