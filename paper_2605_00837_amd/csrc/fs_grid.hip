// Problems up to 4096 x 2048 whose cost matrix (or table of squared distances) fits the register files of the chip: the whole of
// Alg. 1 inside ONE kernel launch over up to 256 workgroups (one per compute unit), C read from memory
// once per SOLVE.  The multi-kernel driver pays two launches per iteration, each with a few us of
// fixed begin-to-end cost on top of its pass over C; here an iteration is register arithmetic plus two
// grid-wide waits.
//
// Decomposition.  Workgroup w owns RA consecutive rows and all columns: 1024 lanes, lane t keeps the
// entries (row0 + a, t + 1024 b), a < RA, b < CB, in registers (at most 16).  The f-update (Eq. 9) is
// local: wave all-reduce (DPP) per row, the 16 waves of a row meet in LDS.  For the g-update (Eq. 10)
// every workgroup reduces its rows to one partial base-2 LSE per column (lane-local) and publishes the
// m values; after the first grid-wide wait workgroup w merges the W partials of ITS strip of columns
// (one wave per column: 4 loads per lane, wave all-reduce) and publishes the new V_j = log2 b_j - G_j of
// the strip; after the second wait every lane reads the V of its own columns.  The error terms of
// Sec. 4.5 travel with the partials and every workgroup adds the same W terms in the same order, so
// the stop decision is taken identically everywhere.  Arithmetic as everywhere else: exponent
// arguments in fp64 (base 2), v_exp_f32 and the sums in fp32; both LSEs are exact (maximum first).
//
// Grid-wide waits: arrivals are counted in 8 group counters; the workgroup that completes a group says so in
// the `done` line, kept in 64 copies of which every workgroup polls one (as in the persistent pass,
// fs_persist_sync.h; all monotone, never reset during a solve), published values are
// written and read with agent-scope relaxed atomics and every thread waits for its own stores before
// its workgroup arrives.  Two waits per round make single exchange buffers safe: partials of round
// r + 1 are written after the second wait of round r, which every workgroup reaches only after it has
// read the partials of round r; the V strip of round r + 1 is written after the first wait of round
// r + 1, which every workgroup reaches only after it has read (and used) the V of round r.  Every wait
// is bounded: a workgroup that gives up raises a flag that makes all others give up too, and the solve
// then reports that it gave up (nonfinite = 2) instead of hanging.
#include <type_traits>

#include "fs_kernels.h"
#include "fs_persist_sync.h"

namespace fs {

namespace {

constexpr int kGT = 1024;                  // threads per workgroup = column lanes
constexpr int kGW = kGT / 64;              // waves
constexpr int kGRows = 16;                 // most rows per workgroup
constexpr int kGStripRounds = 1;           // columns of the strip that a wave merges per round

__device__ __forceinline__ void publish(double *p, double v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double fetch(const double *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long bump(unsigned long long *p) {
    return __hip_atomic_fetch_add(p, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double row16_max(double v) {            // all-reduce over a DPP row of 16 lanes
    v = dmax(v, dpp_f64<0x128>(v));
    v = dmax(v, dpp_f64<0x124>(v));
    v = dmax(v, dpp_f64<0x122>(v));
    v = dmax(v, dpp_f64<0x121>(v));
    return v;
}
__device__ __forceinline__ float row16_add(float v) {
    v += dpp_f32<0x128>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x122>(v);
    v += dpp_f32<0x121>(v);
    return v;
}

// Grid-wide wait number `gen` (1, 2, ...).  Every thread of the workgroup calls it after its last store
// of the phase; wave 0 counts the workgroup in and watches its copy of the `done` line (fs_persist_sync.h).
// Returns false when the wait was abandoned (by this workgroup or by another).
__device__ __forceinline__ bool grid_wait(GridSync *sy, unsigned long long gen, int W, int spin_limit, int *s_ok) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0);                       // this thread's published values have been acknowledged
    __syncthreads();
    if (threadIdx.x < 64) {
        const unsigned long long old = grid_arrive(&sy->ps);
        const int good = fs::grid_wait(&sy->ps, old, gen, W, spin_limit);
        if (threadIdx.x == 0) *s_ok = good;
    }
    __syncthreads();
    return *s_ok != 0;
#else
    return false;
#endif
}

__global__ void k_grid_reset(GridSync *sy) {
    const int t = threadIdx.x;
    if (t < kSyncGroups) { sy->ps.grp[t].v = 0ull; sy->ps.done[t] = 0ull; }
    if (t == kSyncGroups) sy->ps.abort_flag = 0ull;
    if (t == kSyncGroups + 1) sy->bad.v = 0ull;
    for (int q = t; q < kSyncCopies * (kSyncGroups + 1); q += blockDim.x)
        sy->ps.copy[q / (kSyncGroups + 1)][q % (kSyncGroups + 1)] = 0ull;
}

// PTS: point clouds - the tile holds |x_i - y_j|^2 in fp64, formed once from the fp32 coordinates in the
// difference form.
template <int RA, int CB, bool PTS>
__global__ __launch_bounds__(kGT) void k_grid(GridArgs A) {
    __shared__ double sF[2][kGRows];               // F = -s f of the workgroup's rows, by parity of k
    __shared__ double sLa[kGRows], sU[kGRows], sE[kGRows];
    __shared__ float sAw[kGRows];
    __shared__ double sRM[RA][kGW];                // row LSE: per-wave maxima and sums
    __shared__ float sRS[RA][kGW];
    __shared__ double sErrTot;
    __shared__ int sOk, sBad;

#if defined(__HIP_DEVICE_COMPILE__)
    const int n = A.n, m = A.m;
    const int W = gridDim.x, w = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row0 = w * RA;
    const double s = A.s, ns = -A.s;
    const double ninf = -__builtin_huge_val();
    // this workgroup's strip of columns for the second level: [strip0, strip1), one wave per column and round
    const int S = (m + W - 1) / W;
    const int strip0 = min(m, w * S), strip1 = min(m, strip0 + S);

    // ---- start: weights, initial potentials (zero, Eqs. 6-7, or the caller's), the cost tile
    if (tid < kGRows) {
        const int i = row0 + tid;
        const bool ok = tid < RA && i < n;
        const float wgt = ok ? A.a[i] : 0.0f;
        sAw[tid] = wgt;
        sLa[tid] = ok ? log2_weight(wgt) : ninf;
        double F0 = 0.0;
        if (A.warm && ok) F0 = ns * (A.f64_in ? A.f64_in[i] : (double)A.f_in[i]);
        sF[0][tid] = F0;
        sF[1][tid] = F0;
        sE[tid] = 0.0;
    }
    if (tid == 0) sBad = 0;
    auto start_G = [&](int col) -> double {
        if (!A.warm || col >= m) return 0.0;
        return ns * (A.g64_in ? A.g64_in[col] : (double)A.g_in[col]);
    };
    double V[CB];
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        const int j = tid + kGT * b;
        V[b] = j < m ? log2_weight(A.b[j]) - start_G(j) : ninf;
    }
    // strip columns of this wave: log2 b and the current G (uniform over the wave)
    double lb2c[kGStripRounds], Gc[kGStripRounds];
#pragma unroll
    for (int r = 0; r < kGStripRounds; ++r) {
        const int col = strip0 + kGW * r + wave;
        const bool ok = col < strip1;
        lb2c[r] = ok ? log2_weight(A.b[col]) : ninf;
        Gc[r] = ok ? start_G(col) : 0.0;
    }
    __builtin_amdgcn_sched_barrier(0);             // the logarithms above are done before the tile takes its registers
    typename std::conditional<PTS, double, float>::type c[RA][CB];
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        const int j = tid + kGT * b;
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            const int i = row0 + a;
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
    }
    __syncthreads();

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
            if (lane == 0) { sRM[a][wave] = mx; sRS[a][wave] = sm; }
            __builtin_amdgcn_sched_barrier(0);       // one row at a time: interleaving them costs registers
        }
        __syncthreads();
        if (tid < RA * kGW) {
            // 16 lanes (one DPP row) per matrix row merge the 16 wave partials; the new F goes to the other
            // buffer: should this round turn out to be the one that stops, the iterate to return (old F,
            // current G) is still there
            const int a = tid / kGW, q = tid % kGW;
            const double M = sRM[a][q];
            const double mx = row16_max(M);
            const float sm = row16_add(sRS[a][q] * fast_exp2((float)(M - mx)));
            if (q == 0) {
                const double fn = mx + log2_sum(sm);
                sF[nxt][a] = fn;
                sU[a] = sLa[a] - fn;                              // -inf for rows past n
                double e = 0.0;
                if (need_err) {
                    // error term of Sec. 4.5 for this row: a_i |2^(Fnew_i - Fold_i) - 1|
                    const float wgt = sAw[a];
                    if (wgt > 0.0f) e = (double)wgt * fabs(exp2m1(fn - sF[cur][a]));
                }
                sE[a] = e;
            }
        }
        __syncthreads();

        // ---- g-update (Eq. 10) with the new f, this workgroup's rows only: one partial LSE per column
        double *x1 = A.xchg1 + (size_t)w * A.ldx;
        if (!trailing) {
            // rows outermost: one U_i in a register at a time
            double mx[CB];
            float sm[CB];
#pragma unroll
            for (int b = 0; b < CB; ++b) { mx[b] = kNegHuge; sm[b] = 0.0f; }
#pragma unroll
            for (int a = 0; a < RA; ++a) {
                const double u = sU[a];
#pragma unroll
                for (int b = 0; b < CB; ++b) mx[b] = dmax(mx[b], fma(ns, cost_f64(c[a][b]), u));
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int a = 0; a < RA; ++a) {
                const double u = sU[a];
#pragma unroll
                for (int b = 0; b < CB; ++b) sm[b] += fast_exp2((float)(fma(ns, cost_f64(c[a][b]), u) - mx[b]));
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int b = 0; b < CB; ++b) {
                const int j = tid + kGT * b;
                if (j < m) publish(x1 + j, mx[b] + log2_sum(sm[b]));
            }
        }
        if (tid == 0) {
            double e = 0.0;
#pragma unroll
            for (int a = 0; a < RA; ++a) e += sE[a];             // fixed order
            publish(x1 + A.ldx - 1, e);
        }

        // ---- first wait, then the strip of this workgroup: merge everyone's partials, publish the new V
        if (!grid_wait(A.sync, ++gen, W, A.spin_limit, &sOk)) { alive = false; break; }
        double Gnew[kGStripRounds];
#pragma unroll
        for (int r = 0; r < kGStripRounds; ++r) {
            Gnew[r] = Gc[r];
            const int col = strip0 + kGW * r + wave;               // uniform over the wave
            if (!trailing && col < strip1) {
                double pv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int src = lane + 64 * q;
                    pv[q] = src < W ? fetch(A.xchg1 + (size_t)src * A.ldx + col) : kNegHuge;
                }
                double mx = dmax(dmax(pv[0], pv[1]), dmax(pv[2], pv[3]));
                mx = wave_max_f64(mx);
                float sm = 0.0f;
#pragma unroll
                for (int q = 0; q < 4; ++q) sm += fast_exp2((float)(pv[q] - mx));
                sm = wave_sum_f32(sm);
                Gnew[r] = mx + log2_sum(sm);
                if (lane == 0) publish(A.xchg2 + col, lb2c[r] - Gnew[r]);
            }
        }
        if (wave == kGW - 1 && need_err) {
            // the error of the iterate this round started from: the same W terms in the same order everywhere
            double e = 0.0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int src = lane + 64 * q;
                if (src < W) e += fetch(A.xchg1 + (size_t)src * A.ldx + A.ldx - 1);
            }
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
            if (checked && err < A.tol) {          // stop at k: sF[cur] and Gc still hold iterate k
                iters = k;
                converged = 1;
                err_out = err;
                break;
            }
        }

        // ---- second wait, then every lane takes the V of its own columns
        if (!grid_wait(A.sync, ++gen, W, A.spin_limit, &sOk)) { alive = false; break; }
#pragma unroll
        for (int r = 0; r < kGStripRounds; ++r) Gc[r] = Gnew[r];
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            const int j = tid + kGT * b;
            V[b] = j < m ? fetch(A.xchg2 + j) : ninf;
        }
    }

    // ---- results: f = -F/s, g = -G/s of the returned iterate (k = iters at every regular exit of the loop)
    __syncthreads();
    const double inv = -1.0 / s;
    const double nan = __builtin_nan("");
    bool bad = false;
    if (tid < RA && row0 + tid < n) {
        const double v = alive ? sF[iters & 1][tid] * inv : nan;
        A.f[row0 + tid] = (float)v;
        if (A.f64_out) A.f64_out[row0 + tid] = v;
        bad |= !(fabs(v) <= 1.7e308);
    }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < kGStripRounds; ++r) {
            const int col = strip0 + kGW * r + wave;
            if (col < strip1) {
                const double v = alive ? Gc[r] * inv : nan;
                A.g[col] = (float)v;
                if (A.g64_out) A.g64_out[col] = v;
                bad |= !(fabs(v) <= 1.7e308);
            }
        }
    }
    if (bad) atomicOr(&sBad, 1);
    __syncthreads();
    if (tid == 0 && sBad) __hip_atomic_fetch_or(&A.sync->bad.v, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // one more wait so that workgroup 0 sees every workgroup's flag (skipped once a wait has been abandoned)
    if (alive) alive = grid_wait(A.sync, ++gen, W, A.spin_limit, &sOk);
    if (w == 0 && tid == 0 && A.result) {
        ResultRecord r;
        r.iters = alive ? iters : k;
        r.converged = alive ? converged : 0;
        r.nonfinite = alive ? (int)(__hip_atomic_load(&A.sync->bad.v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull) : kGaveUp;
        r.marginal_err = alive ? (float)err_out : __builtin_nanf("");
        A.result[0] = r;
        __threadfence_system();
    }
#endif
}

template <int RA, bool PTS>
hipError_t launch_cb(hipStream_t st, const GridArgs &a, int W, int cb) {
    const dim3 grid(W), block(kGT);
    constexpr int kMost = PTS ? 8 : 16;             // entries per lane that were built (fp64 entries count double)
    if (cb <= 1) hipLaunchKernelGGL((k_grid<RA, 1, PTS>), grid, block, 0, st, a);
    else if constexpr (RA * 2 <= kMost) hipLaunchKernelGGL((k_grid<RA, 2, PTS>), grid, block, 0, st, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// Rows per workgroup: the smallest of 1, 2, 4, 8, 16 that keeps the grid within wmax workgroups.
int grid_rows(int n, int wmax) {
    for (int ra = 1; ra <= kGRows; ra *= 2)
        if ((n + ra - 1) / ra <= wmax) return ra;
    return 0;
}

constexpr int kGridLdx = kGridMaxM + 32;

}  // namespace

// Shapes taken: at most 16 entries per lane (beyond that the multi-kernel driver is as fast or faster: the tile
// and the working set no longer fit the 128 registers of a 1024-lane workgroup), and a strip of at most 16
// columns per workgroup in the second level (one wave per column).
bool grid_supported(int n, int m, int wmax, bool points) {
    if (n < 1 || m < 1 || n > kGridMaxN || m > kGridMaxM || wmax < 1) return false;
    if (wmax > kGridWMax) wmax = kGridWMax;
    const int ra = grid_rows(n, wmax);
    if (ra == 0) return false;
    const int cb = (m + kGT - 1) / kGT;
    if (ra * cb > (points ? 8 : 16)) return false;  // point clouds: the tile is fp64
    const int W = (n + ra - 1) / ra;
    return (m + W - 1) / W <= kGW * kGStripRounds;
}

size_t grid_scratch_bytes() {
    return sizeof(double) * ((size_t)kGridWMax * kGridLdx + kGridLdx) + sizeof(GridSync);
}

hipError_t launch_grid(hipStream_t st, const GridArgs &a0, void *scratch, int wmax) {
    if (wmax > kGridWMax) wmax = kGridWMax;
    if (!scratch || !grid_supported(a0.n, a0.m, wmax, a0.X != nullptr)) return hipErrorInvalidValue;
    if (a0.X && (!a0.Y || a0.d < 1)) return hipErrorInvalidValue;
    const int RA = grid_rows(a0.n, wmax);
    const int W = (a0.n + RA - 1) / RA;
    GridArgs a = a0;
    a.ldx = kGridLdx;
    a.xchg1 = reinterpret_cast<double *>(scratch);
    a.xchg2 = a.xchg1 + (size_t)kGridWMax * kGridLdx;
    a.sync = reinterpret_cast<GridSync *>(a.xchg2 + kGridLdx);
    if (a.spin_limit <= 0) a.spin_limit = 1 << 21;
    hipLaunchKernelGGL(k_grid_reset, dim3(1), dim3(256), 0, st, a.sync);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int cb = (a.m + kGT - 1) / kGT;
    if (a.X) {
        switch (RA) {
            case 1: return launch_cb<1, true>(st, a, W, cb);
            case 2: return launch_cb<2, true>(st, a, W, cb);
            case 4: return launch_cb<4, true>(st, a, W, cb);
            default: return launch_cb<8, true>(st, a, W, cb);
        }
    }
    switch (RA) {
        case 1: return launch_cb<1, false>(st, a, W, cb);
        case 2: return launch_cb<2, false>(st, a, W, cb);
        case 4: return launch_cb<4, false>(st, a, W, cb);
        case 8: return launch_cb<8, false>(st, a, W, cb);
        default: return launch_cb<16, false>(st, a, W, cb);
    }
}

}  // namespace fs
