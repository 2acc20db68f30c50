// Kernels every solve uses, whatever the cost representation: initialisation of
// the log-weights and potentials (Alg. 1, first two steps), the combine of
// partial LogSumExp values, the once-per-iteration state advance with the
// stopping test (Alg. 1, check every c iterations) and the final conversion of
// the scaled fp64 potentials to the caller's fp32 f, g.
#include "fs_kernels.h"

namespace fs {

// ---------------------------------------------------------------- init
// la2 = log2 a, lb2 = log2 b (Alg. 1 "precompute"); F = G = 0 (Eqs. 6-7) or the
// caller's warm start; U = la2 - F, V = lb2 - G; state cleared, and with it the arrival counters of the
// persistent pass when the solve uses it (psync, else null).
__global__ __launch_bounds__(256) void k_init(Pots p, State *state, const float *f_in,
                                              const float *g_in, const double *f64_in, const double *g64_in,
                                              int warm, PersistSync *psync) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t == 0) {
        state->k = 0; state->flags = 0; state->iters = 0; state->converged = 0; state->nonfinite = 0;
        state->err_valid = 0;
        state->err_acc = 0;
        state->big_acc[0] = 0; state->big_acc[1] = 0x7fffffffu;   // no count yet: the first hint says ROBUST
        state->fin_ticket = 0;
        state->err = __builtin_nan("");
    }
    if (psync && t >= 64 && t <= 64 + kSyncGroups) {
        if (t < 64 + kSyncGroups) { psync->grp[t - 64].v = 0ull; psync->done[t - 64] = 0ull; }
        else psync->abort_flag = 0ull;
    }
    if (psync)
        for (int q = t; q < kSyncCopies * (kSyncGroups + 1); q += gridDim.x * 256)
            psync->copy[q / (kSyncGroups + 1)][q % (kSyncGroups + 1)] = 0ull;
    double *la2 = const_cast<double *>(p.la2);
    double *lb2 = const_cast<double *>(p.lb2);
    if (t < p.n) {
        const double la = log2_weight(p.a[t]);
        double F = 0.0;
        if (warm & 1) F = -p.s * (f64_in ? f64_in[t] : (double)f_in[t]);
        la2[t] = la;
        p.F[t] = F;
        p.U[t] = la - F;
        p.F[p.n_ld + t] = F;
        p.U[p.n_ld + t] = la - F;
    }
    // The padding behind the n rows of F holds a reference no exponent reaches: a fused pass whose last panel
    // is ragged reads it as the old F of the rows past n, and every term of such a row becomes exactly 0
    // (with F = 0 there, 2^V_j overflows for large V_j and the column sums turn NaN: correct after the exact
    // repair of every column, but many times slower).
    if (t >= p.n && t < p.n_ld) {
        p.F[t] = kPadF;
        p.F[p.n_ld + t] = kPadF;
    }
    if (t < p.m) {
        const double lb = log2_weight(p.b[t]);
        double G = 0.0;
        if (warm & 2) G = -p.s * (g64_in ? g64_in[t] : (double)g_in[t]);
        lb2[t] = lb;
        p.G[t] = G;
        p.V[t] = lb - G;
        p.G[p.m_ld + t] = G;
        p.V[p.m_ld + t] = lb - G;
    }
}

hipError_t launch_init(hipStream_t st, const Pots &p, State *state, const float *f_in, const float *g_in,
                       const double *f64_in, const double *g64_in, int warm, void *persist_sync) {
    const int len = p.n > p.m ? p.n : p.m;
    hipLaunchKernelGGL(k_init, dim3((len + 255) / 256), dim3(256), 0, st, p, state, f_in, g_in, f64_in,
                       g64_in, warm, reinterpret_cast<PersistSync *>(persist_sync));
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_export(const double *pot, int len, double s, double *out) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < len) out[t] = -pot[t] / s;
}

hipError_t launch_export(hipStream_t st, const double *pot, int len, double s, double *out) {
    hipLaunchKernelGGL(k_export, dim3((len + 255) / 256), dim3(256), 0, st, pot, len, s, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------- finalize
// f = -F/s, g = -G/s from the buffer of the returned iterate; flags non-finite values.  The workgroup that
// finishes last writes the result record (to device memory, or to pinned host memory for the blocking solves)
// and closes the state, so a solve ends with this one launch.
__global__ __launch_bounds__(256) void k_finalize(Pots p, State *state, float *f, float *g, double *f64_out,
                                                  double *g64_out, ResultRecord *dev, ResultRecord *host) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int it = (state->flags & kFlagDone) ? state->iters : state->k;
    const int buf = it & 1;
    const double inv = -1.0 / p.s;
    bool bad = false;
    if (t < p.n) {
        const double v = p.F[buf * p.n_ld + t] * inv;
        f[t] = (float)v;
        if (f64_out) f64_out[t] = v;
        bad |= !(fabs(v) <= 1.7e308);
    }
    if (t < p.m) {
        const double v = p.G[buf * p.m_ld + t] * inv;
        g[t] = (float)v;
        if (g64_out) g64_out[t] = v;
        bad |= !(fabs(v) <= 1.7e308);
    }
    if (bad) __hip_atomic_fetch_or(&state->nonfinite, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // every thread's flag is out before its workgroup takes a ticket (the barrier orders the workgroup's atomics
    // before thread 0's, all on the same agent-scope path)
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x != 0) return;
    const unsigned ticket = __hip_atomic_fetch_add(&state->fin_ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (ticket != gridDim.x - 1) return;
    const int nonfinite = __hip_atomic_load(&state->nonfinite, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ResultRecord r;
    const bool done = (state->flags & kFlagDone) != 0;
    r.iters = done ? state->iters : state->k;
    r.converged = done ? state->converged : 0;
    r.nonfinite = (nonfinite & kGaveUp) ? kGaveUp : nonfinite;
    r.marginal_err = (done && state->err_valid) ? (float)state->err : __builtin_nanf("");
    if (!done) { state->iters = r.iters; state->flags |= kFlagDone; }
    state->fin_ticket = 0;
    if (dev) *dev = r;
    if (host) {
        *host = r;
        __threadfence_system();
    }
}

hipError_t launch_finalize(hipStream_t st, const Pots &p, State *state, float *f, float *g, double *f64_out,
                           double *g64_out, void *result_dev, void *result_host) {
    const int len = p.n > p.m ? p.n : p.m;
    hipLaunchKernelGGL(k_finalize, dim3((len + 255) / 256), dim3(256), 0, st, p, state, f, g, f64_out, g64_out,
                       (ResultRecord *)result_dev, (ResultRecord *)result_host);
    return hipGetLastError();
}

// ---------------------------------------------------------------- error terms + advance
// Sum over the 1024 threads of a workgroup in a fixed order (wave sums by DPP, 16 wave sums in LDS).
__device__ __forceinline__ double block_sum_1024(double v, double *lds16) {
    const double w = wave_sum_f64(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds16[threadIdx.x >> 6] = w;
    __syncthreads();
    double tot = 0.0;
#pragma unroll
    for (int q = 0; q < 16; ++q) tot += lds16[q];
    return tot;
}

// 1 if a potential moved by more than kFastBelow (or by a non-finite amount), else 0
__device__ __forceinline__ double big_move(double diff) { return (fabs(diff) <= kFastBelow) ? 0.0 : 1.0; }
// Error terms a_i |2^(Fnew_i - Fold_i) - 1| of the rows first, first+stride, ... (fp64, a series for
// the small differences near convergence).
__device__ __forceinline__ double err_terms(const ErrSrc &es, int cur, int first, int stride) {
    const double *Fo = es.F + (size_t)cur * es.n_ld;
    const double *Fn = es.F + (size_t)(cur ^ 1) * es.n_ld;
    double acc = 0.0;
    for (int i = first; i < es.n; i += stride) {
        const float a = es.a[i];
        const double diff = Fn[i] - Fo[i];
        if (a > 0.0f) acc += (double)a * fabs(exp2m1(diff));
    }
    return acc;
}

// Trailing pass: one workgroup evaluates err of the last iterate and closes the solve.
__global__ __launch_bounds__(1024) void k_advance(ErrSrc es, Ctl c) {
    __shared__ double lds[16];
    int k;
    if (!launch_active(c, k)) return;
    const double err = block_sum_1024(err_terms(es, k & 1, threadIdx.x, 1024), lds);
    if (threadIdx.x == 0) advance_state(c, k, err, 1.0e300);
}

hipError_t launch_advance(hipStream_t st, const ErrSrc &es, const Ctl &c) {
    hipLaunchKernelGGL(k_advance, dim3(1), dim3(1024), 0, st, es, c);
    return hipGetLastError();
}

// ---------------------------------------------------------------- combine
// out_j = LSE2_p part[p][j] (+ rowconst_j).  A workgroup of kCombW waves owns 64 adjacent entries;
// wave w folds the partial sets p = w, w + kCombW, ... (each read is one coalesced row segment, 16
// independent loads in flight per lane), the wave results meet in LDS and wave 0 finishes the columns.
// Partials of the LDS-prefetch fused pass are plain fp32 sums against a common reference and are
// simply added up.
//
// The g-update's combine also closes the iteration, on a second track that runs beside the column
// work: wave 1 of every workgroup evaluates the error terms of Sec. 4.5 for 64 rows and reports their
// sum with one atomic addition to the closing word of the solver state, which carries a fixed-point
// sum (integer addition: the total does not depend on the order of arrival) above a count of the
// workgroups that have reported.  The workgroup whose addition completes the count holds the total
// in the value the atomic returned; it applies the stopping rule of Alg. 1 and resets the word.  The count of fast-moving
// columns that steers the driver's choice of kernels is collected per parity of the iteration and
// read one iteration late, so that it never waits for the column work either.
//
// The kernel is a chain of memory latencies, so every load whose address does not depend on the
// iteration counter is issued before the counter itself has arrived.
constexpr int kErrWave = 1;
constexpr int kTicketBits = 14;                        // up to 16383 workgroups
constexpr double kErrScale = 35184372088832.0;         // 2^45: sums below 16 fit in bits 14..62, resolution 2.8e-14
constexpr unsigned long long kErrBad = 1ull << 63;

template <int kCombW>
__global__ __launch_bounds__(kCombW * 64) void k_combine(CombineArgs A, Ctl c) {
    constexpr int kCombT = kCombW * 64;
    static_assert(kCombW > kErrWave, "the error terms have a wave of their own");
    __shared__ double sM[kCombW][64];
    __shared__ float sS[kCombW][64];
    __shared__ unsigned long long s_mask;
    const unsigned long long kd = load_counter(c);
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int j = blockIdx.x * 64 + lane;
    const bool jok = j < A.len;
    const bool fast_mode = A.repair_C != nullptr;      // the partials come from the fp32 plan-unit column phase
    const bool err_wave = A.do_advance && wave == kErrWave;
    const float *pf = reinterpret_cast<const float *>(A.part);
    // first batch of partial sets p = wave, wave + kCombW, ...
    const bool batch = jok && (wave + 15 * kCombW < A.P);
    float xf[16];
    double xd[16];
    if (batch) {
        if (fast_mode) {
#pragma unroll
            for (int q = 0; q < 16; ++q) xf[q] = pf[(size_t)(wave + kCombW * q) * A.ld + j];
        } else {
#pragma unroll
            for (int q = 0; q < 16; ++q) xd[q] = A.part[(size_t)(wave + kCombW * q) * A.ld + j];
        }
    }
    // rows of the error sum: 64 per workgroup and round (both copies of F; the counter says which is new)
    const int estride = gridDim.x * 64;
    const int ei0 = blockIdx.x * 64 + lane;
    double F0[2] = {0.0, 0.0}, F1[2] = {0.0, 0.0};
    float aw[2] = {0.0f, 0.0f};
    if (err_wave) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int i = ei0 + q * estride;
            if (i < A.es.n) { F0[q] = A.es.F[i]; F1[q] = A.es.F[(size_t)A.es.n_ld + i]; aw[q] = A.es.a[i]; }
        }
    }
    unsigned big_ld[2] = {0u, 0u};
    if (err_wave && lane == 0) {
        big_ld[0] = __hip_atomic_load(&c.st->big_acc[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        big_ld[1] = __hip_atomic_load(&c.st->big_acc[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    double lw2_j = 0.0, rowconst_j = 0.0, pot_j[2] = {0.0, 0.0}, shift_b[2] = {0.0, 0.0};
    if (wave == 0 && jok) {
        lw2_j = A.lw2[j];
        if (A.rowconst) rowconst_j = A.rowconst[j];
        pot_j[0] = A.pot[j];
        pot_j[1] = A.pot[(size_t)A.ld + j];
        if (fast_mode) { shift_b[0] = A.shift[j]; shift_b[1] = A.shift[(size_t)A.ld + j]; }
    }

    // ---- everything that needs no counter
    Lse acc; acc.init();
    double tsum = 0.0;                             // fp32-sum partials: plain total (in double)
    if (jok) {
        int p = wave;
        if (fast_mode) {
            if (batch) {
#pragma unroll
                for (int q = 0; q < 16; ++q) tsum += (double)xf[q];
                p += 16 * kCombW;
            }
            for (; p + 15 * kCombW < A.P; p += 16 * kCombW) {
#pragma unroll
                for (int q = 0; q < 16; ++q) xf[q] = pf[(size_t)(p + kCombW * q) * A.ld + j];
#pragma unroll
                for (int q = 0; q < 16; ++q) tsum += (double)xf[q];
            }
            for (; p < A.P; p += kCombW) tsum += (double)pf[(size_t)p * A.ld + j];
        } else {
            if (batch) {
                acc.add<16>(xd);
                p += 16 * kCombW;
            }
            for (; p + 15 * kCombW < A.P; p += 16 * kCombW) {
#pragma unroll
                for (int q = 0; q < 16; ++q) xd[q] = A.part[(size_t)(p + kCombW * q) * A.ld + j];
                acc.add<16>(xd);
            }
            for (; p < A.P; p += kCombW) {
                double x[1] = {A.part[(size_t)p * A.ld + j]};
                acc.add<1>(x);
            }
        }
    }
    // error terms a_i |2^(Fnew_i - Fold_i) - 1| in fp64 (a series for the small differences near
    // convergence), for either role of the two copies of F
    double term_if[2] = {0.0, 0.0};                // [0]: copy 1 is the new one, [1]: copy 0 is
    if (err_wave) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (aw[q] > 0.0f) {
                const double x = F1[q] - F0[q];
                term_if[0] += (double)aw[q] * fabs(exp2m1(x));
                term_if[1] += (double)aw[q] * fabs(exp2m1(-x));
            }
        }
    }

    int k;
    bool fast_hint;
    if (!counter_active(c, kd, k, &fast_hint)) return;
    const int cur = k & 1, nxt = cur ^ 1;
    State *st = c.st;
    // the partials come from the optimistic point-cloud pass (it ran because of the same hint)
    const bool pts_check = A.pr_rows != nullptr && fast_hint;

    double err_part = 0.0;
    if (err_wave) {
        double term = term_if[cur];
        const double *Fo = A.es.F + (size_t)cur * A.es.n_ld;
        const double *Fn = A.es.F + (size_t)nxt * A.es.n_ld;
        for (int i = ei0 + 2 * estride; i < A.es.n; i += estride) {   // only when n > 128 * (workgroups of the grid)
            const float a = A.es.a[i];
            if (a > 0.0f) term += (double)a * fabs(exp2m1(Fn[i] - Fo[i]));
        }
        err_part = wave_sum_f64(term);
    }
    sM[wave][lane] = fast_mode ? tsum : acc.M;
    sS[wave][lane] = acc.s;
    __syncthreads();                                   // also: every wave of the workgroup has read the counter

    if (err_wave && lane == 0) {
        // close the iteration.  A share that is not a number (or absurd) sets the flag bit first; the two
        // atomics go to the same address, so they are performed in this order.
        unsigned long long add = 1;
        if (err_part >= 0.0 && err_part <= 4.0) add += (unsigned long long)(err_part * kErrScale) << kTicketBits;
        else atomicOr(&st->err_acc, kErrBad);
        const unsigned long long word = atomicAdd(&st->err_acc, add) + add;
        if ((word & ((1ull << kTicketBits) - 1)) == gridDim.x) {
            // fast-moving columns of the previous iteration (complete since the previous launch, read above)
            const unsigned bigc = cur ? big_ld[0] : big_ld[1];
            st->err_acc = 0; st->big_acc[nxt] = 0;
            const double err = (word & kErrBad) ? __builtin_nan("")
                                                : (double)((word & ~kErrBad) >> kTicketBits) / kErrScale;
            advance_state(c, k, err, (double)bigc);
        }
    }
    if (wave == 0) {
        bool suspect = false;
        double nbig = 0.0;                             // 1 if this column moved by more than kFastBelow
        if (jok) {
            const double old_j = cur ? pot_j[1] : pot_j[0];
            double out;
            if (fast_mode) {
#pragma unroll
                for (int w = 1; w < kCombW; ++w) tsum += sM[w][lane];
                out = log2_sum(tsum) - (cur ? shift_b[1] : shift_b[0]);      // log2 T_j - V_j (NaN if V_j = -inf)
            } else {
#pragma unroll
                for (int w = 1; w < kCombW; ++w) acc.merge(sM[w][lane], sS[w][lane]);
                out = acc.value();                     // -inf when every term was -inf
            }
            out += rowconst_j;
            // FAST column mode sums plan entries in fp32: a column whose total mass is below 2^-66
            // (or not a number) may have lost terms to underflow; tiny and zero weights always land here
            if (fast_mode) suspect = !(tsum >= kColMassFloor);
            else if (pts_check) suspect = !(out >= old_j - kColRepairBelow && out <= old_j + kRepairAbove);
            nbig = suspect ? 1.0 : big_move(out - old_j);
            A.pot[(size_t)nxt * A.ld + j] = out;
            A.shift[(size_t)nxt * A.ld + j] = lw2_j - out;
        }
        const unsigned long long mask = __ballot(suspect);
        if (lane == 0) s_mask = mask;
        if (A.do_advance) {
            const double wbig = wave_sum_f64(nbig);
            if (lane == 0 && wbig > 0.0) atomicAdd(&st->big_acc[cur], (unsigned)wbig);
        }
    }
    if (fast_mode || pts_check) {
        // ---- exact recomputation of the suspect entries of this workgroup (rare): all threads walk
        //      over the other side (down column j of C with the new U, or over all points of the other
        //      cloud), online LSE per thread, then wave + LDS merge
        __syncthreads();                               // s_mask is visible
        unsigned long long todo = s_mask;
        const double *U = fast_mode ? A.repair_U + (size_t)nxt * A.repair_ld : nullptr;
        const double *cshift = pts_check ? A.pr_colshift + (size_t)(A.pr_shift_next ? nxt : cur) * A.pr_ld : nullptr;
        while (todo) {
            const int bit = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            const int jj = blockIdx.x * 64 + bit;
            Lse ex; ex.init();
            if (fast_mode) {
                for (int i = t; i < A.repair_n; i += kCombT) {
                    double y[1] = {fma(-A.repair_s, (double)cost_entry(A.repair_C, A.repair_dtype, (size_t)i * A.len + jj), U[i])};
                    ex.add<1>(y);
                }
            } else {
                const double *xr = A.pr_rows + (size_t)jj * A.pr_d;
                for (int i = t; i < A.pr_nc; i += kCombT) {
                    double y[1] = {cshift[i] + A.pr_colconst[i]};
                    for (int q = 0; q < A.pr_d; ++q) y[0] = fma(xr[q], A.pr_cols2s[(size_t)i * A.pr_d + q], y[0]);
                    ex.add<1>(y);
                }
            }
            ex.wave_reduce();
            __syncthreads();                           // previous round's LDS reads are done
            if (lane == 0) { sM[wave][0] = ex.M; sS[wave][0] = ex.s; }
            __syncthreads();
            if (t == 0) {
                Lse tot; tot.init();
#pragma unroll
                for (int w = 0; w < kCombW; ++w) tot.merge(sM[w][0], sS[w][0]);
                const double out = tot.value() + (A.rowconst ? A.rowconst[jj] : 0.0);
                A.pot[(size_t)nxt * A.ld + jj] = out;
                A.shift[(size_t)nxt * A.ld + jj] = A.lw2[jj] - out;
            }
        }
    }
}

hipError_t launch_combine(hipStream_t st, const CombineArgs &a, const Ctl &c) {
    if ((a.len + 63) / 64 >= (1 << kTicketBits)) return hipErrorInvalidValue;     // the ticket field would overflow
    int grid = (a.len + 63) / 64;
    if (a.do_advance) {
        // the error sum runs over the OTHER side's es.n rows, 128 per workgroup without a loop: a tall problem
        // (65536 x 256: 4 workgroups by len) gets workgroups that own no entry and only carry error terms
        int want = (a.es.n + 127) / 128;
        if (want > 2048) want = 2048;
        if (want > grid) grid = want;
    }
    // 16 waves per 64 entries split up to hundreds of partial sets; with 16 sets or fewer (a tall point cloud:
    // 65536 rows against 256 columns leave 4 column slices) 4 waves do, and four times as many workgroups fit
    if (a.P <= 16) hipLaunchKernelGGL(k_combine<4>, dim3(grid), dim3(4 * 64), 0, st, a, c);
    else hipLaunchKernelGGL(k_combine<16>, dim3(grid), dim3(16 * 64), 0, st, a, c);
    return hipGetLastError();
}

}  // namespace fs
