// Small dense problems (n, m <= 256): the whole of Alg. 1 inside ONE kernel launch, one workgroup
// per problem, the cost matrix held in registers for the entire solve.  Many problems of one shape
// run side by side (one workgroup each), which is how the chip is filled at these sizes; a single
// problem pays one launch instead of two or three per iteration.
//
// Layout: 1024 lanes = 32 x 32; lane (tr, tc) = (tid / 32, tid % 32) owns the entries
// (tr + 32 a, tc + 32 b), a < RA, b < CB.  Row LSE (Eq. 9): the 32 lanes of a row group sit in one
// half-wave, so the maximum and the sum are all-reduced with DPP and one lane swap, no LDS.  Column
// LSE (Eq. 10): the two half-waves of a wave meet through a lane swap, the 16 waves through LDS.
// Both are the two-pass LogSumExp of Eq. 8 over registers: exact maximum first, then the sum.
// Arithmetic as everywhere else: potentials and exponent arguments in fp64 (scaled to base 2),
// v_exp_f32 and the sums in fp32.
//
// Stop rule as in the multi-kernel driver: err_k (Sec. 4.5) is the row-marginal error of the iterate
// after k iterations and falls out of the f-update of iteration k + 1; on a stop at k the potentials
// of iterate k are returned (they are still in LDS at that moment).
#include "fs_kernels.h"

namespace fs {

namespace {

constexpr int kST = 1024;

__device__ __forceinline__ double half_max_f64(double v) {      // all-reduce over a half-wave (32 lanes)
    v = dmax(v, dpp_f64<0x128>(v));
    v = dmax(v, dpp_f64<0x124>(v));
    v = dmax(v, dpp_f64<0x122>(v));
    v = dmax(v, dpp_f64<0x121>(v));
    v = dmax(v, swz16_f64(v));
    return v;
}
__device__ __forceinline__ float half_sum_f32(float v) {
    v += dpp_f32<0x128>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x122>(v);
    v += dpp_f32<0x121>(v);
    v += swz16_f32(v);
    return v;
}

template <int RA, int CB>
__global__ __launch_bounds__(kST) void k_small(SmallArgs A) {
    __shared__ double sLa[kSmallMax], sLb[kSmallMax];      // log2 weights
    __shared__ double sF[2][kSmallMax], sG[kSmallMax];     // potentials (scaled: F = -s f); F by parity of k
    __shared__ double sM[kST / 64][kSmallMax];
    __shared__ float sS[kST / 64][kSmallMax];
    __shared__ double sColM[kSmallMax], sV[kSmallMax];
    __shared__ double sErr[kST / 64];
    __shared__ double sErrTot;
    __shared__ int sBad;

    const int p = blockIdx.x;
    const int n = A.n, m = A.m;
    const size_t c0 = (size_t)p * n * m;              // first entry of this problem's cost matrix
    const float *aw = A.a + (size_t)p * n;
    const float *bw = A.b + (size_t)p * m;
    const int tid = threadIdx.x, tc = tid & 31, tr = tid >> 5, lane = tid & 63, wave = tid >> 6;
    const double s = A.s, ns = -A.s;
    const double ninf = -__builtin_huge_val();

    // ---- start: log2 weights and the initial potentials (zero, Eqs. 6-7, or the caller's)
    if (tid < kSmallMax) {
        const int t = tid;
        sLa[t] = t < n ? log2_weight(aw[t]) : ninf;
        sLb[t] = t < m ? log2_weight(bw[t]) : ninf;
        double F0 = 0.0, G0 = 0.0;
        if (A.warm) {
            if (t < n) F0 = ns * (A.f64_in ? A.f64_in[(size_t)p * n + t] : (double)A.f_in[(size_t)p * n + t]);
            if (t < m) G0 = ns * (A.g64_in ? A.g64_in[(size_t)p * m + t] : (double)A.g_in[(size_t)p * m + t]);
        }
        sF[0][t] = F0;
        sG[t] = G0;
        if (t == 0) sBad = 0;
    }
    __syncthreads();
    double U[RA], V[CB];
    float c[RA][CB];
#pragma unroll
    for (int a = 0; a < RA; ++a) {
        const int i = tr + 32 * a;
        U[a] = i < n ? sLa[i] - sF[0][i] : ninf;
    }
#pragma unroll
    for (int b = 0; b < CB; ++b) {
        const int j = tc + 32 * b;
        V[b] = j < m ? sLb[j] - sG[j] : ninf;
    }
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            const int i = tr + 32 * a, j = tc + 32 * b;
            c[a][b] = (i < n && j < m) ? cost_entry(A.C, A.c_dtype, c0 + (size_t)i * m + j) : 0.0f;
        }

    int iters = A.max_iter, converged = 0;
    double err_out = __builtin_nan("");
    int k = 0;
    for (;; ++k) {
        const bool trailing = (k == A.max_iter);
        const bool checked = A.tol > 0.0 && k >= 1 && (k % A.check_every == 0);
        const bool hist = A.err_history && k >= 1 && (k - 1) < A.err_history_len;
        const bool need_err = k >= 1 && (checked || hist || (trailing && A.want_final_err));
        if (trailing && !need_err) break;

        // ---- f-update (Eq. 9): F_i = LSE2_j(V_j - s C_ij), exact two-pass over registers.  The new F goes
        //      to the other LDS buffer: should this iteration turn out to be the one that stops, the
        //      iterate to return (old F, current G) is still there.
        const int cur = k & 1, nxt = cur ^ 1;
        double errloc = 0.0;
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            double mx = kNegHuge;
#pragma unroll
            for (int b = 0; b < CB; ++b) mx = dmax(mx, fma(ns, cost_f64(c[a][b]), V[b]));
            mx = half_max_f64(mx);
            float sm = 0.0f;
#pragma unroll
            for (int b = 0; b < CB; ++b) sm += fast_exp2((float)(fma(ns, cost_f64(c[a][b]), V[b]) - mx));
            sm = half_sum_f32(sm);
            const double Fnew = mx + log2_sum(sm);
            const int i = tr + 32 * a;
            if (tc == 0 && i < n) sF[nxt][i] = Fnew;
            U[a] = i < n ? sLa[i] - Fnew : ninf;
        }
        if (need_err) {
            // error terms of Sec. 4.5, a_i |2^(Fnew_i - Fold_i) - 1|: one row per thread of the first 4 waves
            __syncthreads();
            if (tid < kSmallMax) {
                if (tid < n) {
                    const float w = aw[tid];
                    if (w > 0.0f) errloc = (double)w * fabs(exp2m1(sF[nxt][tid] - sF[cur][tid]));
                }
                errloc = wave_sum_f64(errloc);
                if (lane == 0) sErr[wave] = errloc;
            }
            __syncthreads();
            if (tid == 0) {
                const double e = (sErr[0] + sErr[1]) + (sErr[2] + sErr[3]);
                sErrTot = e;
                if (hist) A.err_history[(size_t)p * A.err_history_len + (k - 1)] = (float)e;
            }
            __syncthreads();
            const double err = sErrTot;
            if (trailing) {
                iters = k;
                converged = (checked && err < A.tol) ? 1 : 0;
                err_out = err;
                break;
            }
            if (checked && err < A.tol) {           // stop at k: sF[cur], sG still hold iterate k
                iters = k;
                converged = 1;
                err_out = err;
                break;
            }
        }

        // ---- g-update (Eq. 10) with the new f: G_j = LSE2_i(U_i - s C_ij)
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            double mx = kNegHuge;
#pragma unroll
            for (int a = 0; a < RA; ++a) mx = dmax(mx, fma(ns, cost_f64(c[a][b]), U[a]));
            mx = dmax(mx, xor32_f64(mx));
            if (lane < 32) sM[wave][tc + 32 * b] = mx;
        }
        __syncthreads();
        if (tid < kSmallMax) {
            double mx = sM[0][tid];
#pragma unroll 4
            for (int w = 1; w < kST / 64; ++w) mx = dmax(mx, sM[w][tid]);
            sColM[tid] = mx;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            const double mx = sColM[tc + 32 * b];
            float sm = 0.0f;
#pragma unroll
            for (int a = 0; a < RA; ++a) sm += fast_exp2((float)(fma(ns, cost_f64(c[a][b]), U[a]) - mx));
            sm += xor32_f32(sm);
            if (lane < 32) sS[wave][tc + 32 * b] = sm;
        }
        __syncthreads();
        if (tid < kSmallMax) {
            float sm = 0.0f;
#pragma unroll 4
            for (int w = 0; w < kST / 64; ++w) sm += sS[w][tid];
            const double G = sColM[tid] + log2_sum(sm);
            sG[tid] = G;
            sV[tid] = tid < m ? sLb[tid] - G : ninf;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < CB; ++b) V[b] = sV[tc + 32 * b];
    }

    // ---- results: f = -F/s, g = -G/s of the returned iterate (k = iters at every exit of the loop)
    __syncthreads();
    if (tid < kSmallMax) {
        const double inv = -1.0 / s;
        bool bad = false;
        if (tid < n) {
            const double v = sF[iters & 1][tid] * inv;
            A.f[(size_t)p * n + tid] = (float)v;
            if (A.f64_out) A.f64_out[(size_t)p * n + tid] = v;
            bad |= !(fabs(v) <= 1.7e308);
        }
        if (tid < m) {
            const double v = sG[tid] * inv;
            A.g[(size_t)p * m + tid] = (float)v;
            if (A.g64_out) A.g64_out[(size_t)p * m + tid] = v;
            bad |= !(fabs(v) <= 1.7e308);
        }
        if (bad) atomicOr(&sBad, 1);
    }
    __syncthreads();
    if (tid == 0 && A.result) {
        ResultRecord r;
        r.iters = iters;
        r.converged = converged;
        r.nonfinite = sBad;
        r.marginal_err = (float)err_out;
        A.result[p] = r;
        __threadfence_system();
    }
}

template <int RA>
hipError_t launch_cb(hipStream_t st, const SmallArgs &a, int cb) {
    const dim3 grid(a.batch), block(kST);
    if (cb <= 2) hipLaunchKernelGGL((k_small<RA, 2>), grid, block, 0, st, a);
    else if (cb <= 4) hipLaunchKernelGGL((k_small<RA, 4>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((k_small<RA, 8>), grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_small(hipStream_t st, const SmallArgs &a) {
    if (a.n < 1 || a.m < 1 || a.n > kSmallMax || a.m > kSmallMax || a.batch < 1) return hipErrorInvalidValue;
    const int ra = (a.n + 31) / 32, cb = (a.m + 31) / 32;
    if (ra <= 2) return launch_cb<2>(st, a, cb);
    if (ra <= 4) return launch_cb<4>(st, a, cb);
    return launch_cb<8>(st, a, cb);
}

}  // namespace fs
