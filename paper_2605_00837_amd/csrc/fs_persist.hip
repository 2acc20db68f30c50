// Persistent form of the fused dense pass: a block of Sinkhorn iterations (Alg. 1, Eqs. 9-10) in ONE launch.
//
// The multi-kernel driver runs two kernels per iteration -- the fused row-panel pass over C and the combine
// of its per-workgroup column sums -- and pays, per iteration, the combine (7 us at n = m = 8192) plus the
// fixed begin-to-end cost of two full-width launches (dispatch, first memory round trip, tail, cache
// write-back).  Here one workgroup per compute unit stays resident for the whole block, streams ITS row
// panels of C once per iteration exactly as the fused pass does (HBM -> LDS prefetch two panels ahead,
// optimistic row phase with the exact redo, plan-unit column phase in fp32), and the workgroups exchange
// what the g-update needs through memory, between two grid-wide waits:
//
//   pass      every workgroup: its panels; new F, U of its rows; fp32 column sums T_j of its rows
//   publish   the m column sums and the error terms of its rows (Sec. 4.5)
//   wait 1
//   merge     workgroup w adds the W partial sums of ITS strip of columns in a fixed order,
//             G_j = log2 T_j - V_j, recomputes exactly (from C and the new U) every column whose total is
//             below 2^-66, and publishes the strip of the new G and V; every workgroup adds the same W
//             error terms in the same order and so takes the same stop decision (Alg. 1)
//   wait 2    --- the first panel of the NEXT iteration goes on its way into LDS as soon as the workgroup has
//             arrived, the second right after the read (C never changes)
//   read      every lane takes the new V of its own columns; workgroup 0 advances the solver state
//
// Everything exchanged is written with agent-scope stores and read with agent-scope loads (relaxed atomics,
// or 16-byte buffer accesses with the same cache policy; no cache maintenance); every wave waits for its own
// stores before the workgroup arrives.  Arrivals are counted in 8 group counters (monotone over a solve,
// reset by the init kernel); the workgroup that completes a group says so in a line (kept in 64 copies, each
// watched by 4 workgroups) that one wave per workgroup watches with one load per poll.  Every wait is bounded: a workgroup that gives up raises a flag that
// makes all others give up, the solve is marked as abandoned (nonfinite = 2) and the host runs the
// multi-kernel driver instead.  The results do not depend on timing: panel ownership is static and every
// sum has a fixed order.
#include <cstdlib>

#include "fs_kernels.h"
#include "fs_persist_sync.h"

namespace fs {

namespace {

// Q groups of 4 adjacent columns per lane (column(q, e) = (q 1024 + tid) 4 + e), R rows per panel.
// FULLW: m == 4096 Q, every lane owns valid columns; then two panels are in flight and the waits on the
// prefetch are exact (see k_fused_pf, whose pass this is).
template <int Q, int R, bool FULLW>
__global__ __launch_bounds__(1024) void k_persist(DenseArgs A, PersistArgs X, Ctl c) {
    constexpr int T = 1024, NW = 16;
    static_assert(R * NW <= 64, "one wave merges all (row, wave) partials in one shot");
    static_assert(5 * R <= 32, "scalar staging holds 16 or 32 dwords per wave");
    constexpr int NDMA = R * Q + 5;            // prefetch loads per panel and wave (FULLW)
    constexpr float kRowHi = 1.1529215e18f;    // 2^60
    constexpr float kRowLo = 9.5367432e-07f;   // 2^-20
    __shared__ float4 stage[2][NW][R][Q][64];
    __shared__ int scal[2][NW][5 * R > 16 ? 32 : 16];            // [0,R) F lo  [R,2R) F hi  [2R,3R) la2 lo  [3R,4R) la2 hi  [4R,5R) a
    __shared__ float sSum[2][R][NW];
    __shared__ double sM[2][R][NW];
    __shared__ float sS[2][R][NW];
    __shared__ double sPart[T];                // merge: partial totals by (set group, column)
    __shared__ int sSus[T];                    // merge: columns of this round to recompute exactly
    __shared__ int sNsus, sOk;
    __shared__ unsigned long long sGen;
    __shared__ double sErrTot;
#if defined(__HIP_DEVICE_COMPILE__)
    const Pots &p = A.p;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const double ns = -p.s;
    const int m = p.m, n = p.n;
    const int W = gridDim.x, w = blockIdx.x;
    const int rr = lane / NW;                  // the panel row this lane serves in the merge of the wave sums
    const int rc = rr < R ? rr : R - 1;
    auto colok = [&](int q) { return FULLW || ((q * T + tid) * 4) < m; };
    auto unpack = [&](const float4 &c4, int q, float (&o)[4]) {
        o[0] = c4.x; o[1] = c4.y; o[2] = c4.z; o[3] = c4.w;
        if (!FULLW) {
            const int col = (q * T + tid) * 4;
#pragma unroll
            for (int e = 1; e < 4; ++e)
                if (col + e >= m) o[e] = 0.0f;
        }
    };

    int k;
    if (!launch_active(c, k)) return;          // nothing is in flight yet
    const int k_end = min(k + X.nb, c.max_iter);
    // the launch that reaches max_iter goes on with one more row phase: it yields err of the last iterate
    const bool with_trailing = X.final_err != 0 && k_end == c.max_iter;

    if (!FULLW) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int q = 0; q < Q; ++q) stage[b][wave][r][q][lane] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (tid == 0) {
        // waits completed so far in this solve (every workgroup of the launches before this one has counted
        // itself in for each of them): the generation numbers of this launch go on from there
        sGen = __hip_atomic_load(&X.sync->done[w % kSyncGroups], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sNsus = 0;
    }
    __syncthreads();
    unsigned long long gen = sGen;

    // This workgroup owns the panels w, w + W, w + 2W, ... in every iteration: it starts with the first of them
    // and walks the others upwards on even iterations and downwards on odd ones (what the last-level cache
    // still holds from the previous pass is read first).
    const int npanels = (n + R - 1) / R;
    const int mine = (npanels - 1 - w) / W + 1;        // >= 1: the grid never has more workgroups than panels
    const __amdgpu_buffer_rsrc_t rsF0 = __builtin_amdgcn_make_buffer_rsrc((void *)p.F, 0, p.n_ld * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsF1 =
        __builtin_amdgcn_make_buffer_rsrc((void *)(p.F + p.n_ld), 0, p.n_ld * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsL = __builtin_amdgcn_make_buffer_rsrc((void *)p.la2, 0, n * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc((void *)p.a, 0, n * 4, 0x00020000);
    auto panel_row = [&](int t, bool rev) { return (w + (t == 0 ? 0 : (rev ? mine - t : t)) * W) * R; };
    // HBM -> LDS prefetch of one panel, of its weights and of the old F of its rows (from the buffer `par`),
    // into the staging slice of wave `tw` (a wave's own, except between iterations, see prefetch_first)
    auto issue = [&](int i0, int buf, int par, int tw) {
        const int rows = (n - i0) < R ? (n - i0) : R;
        const int ttid = tw * 64 + lane;           // the thread whose columns these are
        if (lane < R) {
            const __amdgpu_buffer_rsrc_t rsF = par ? rsF1 : rsF0;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsF, &scal[buf][tw][0], 4, lane * 8, i0 * 8, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsF, &scal[buf][tw][R], 4, lane * 8, i0 * 8 + 4, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsL, &scal[buf][tw][2 * R], 4, lane * 8, i0 * 8, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsL, &scal[buf][tw][3 * R], 4, lane * 8, i0 * 8 + 4, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, &scal[buf][tw][4 * R], 4, lane * 4, i0 * 4, 0, 0);
        }
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((const char *)A.C + (size_t)i0 * m * 4), 0, rows * m * 4, 0x00020000);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int q = 0; q < Q; ++q)
                if (FULLW || ((q * T + ttid) * 4) < m)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, &stage[buf][tw][r][q][0], 16,
                                                             ttid * 16, (r * m + q * T * 4) * 4, 0, 0);
    };
    // The first panels of iteration kk (C never changes, so they can be fetched while the exchange of the
    // iteration before is still going on): panel 0 into staging buffer 0 and, at full width, panel 1 into
    // buffer 1.  Panel 0 goes on its way as soon as the merge has its data.  Wave 0 does the waiting of the
    // exchange, with polls and store acknowledgements that would queue behind a prefetch of its own, so wave 1
    // fetches wave 0's slice of panel 0 as well as its own.  Panel 1 follows once every wave has its new V and
    // panel 0 (latency-critical loads of one wave would otherwise queue behind the bulk requests of another in
    // the compute unit's memory pipeline), every wave its own slice.
    auto prefetch_p0 = [&](int kk) {
        const int par = kk & 1;
        if (wave == 0) return;
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);            // this wave's reads of (and stores to) the staging buffers are done
        issue(panel_row(0, par != 0), 0, par, wave);
        if (wave == 1) issue(panel_row(0, par != 0), 0, par, 0);
        asm volatile("" ::: "memory");
    };
    auto prefetch_p1 = [&](int kk) {
        const int par = kk & 1;
        if (!(FULLW && mine > 1)) return;
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);
        issue(panel_row(1, par != 0), 1, par, wave);
        asm volatile("" ::: "memory");
    };
    // V of this lane's columns (written before this launch)
    double v[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int col = (q * T + tid) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            v[q][e] = (FULLW || col + e < m) ? p.V[(size_t)(k & 1) * p.m_ld + col + e] : -__builtin_huge_val();
    }
    // The strip of columns this workgroup merges: Sw columns (a multiple of 4, at most 64: the launcher sees to
    // it).  The exchange buffer is laid out by destination: [strip][source workgroup][Swp floats], Swp = Sw
    // rounded up to a power of two, so that a workgroup reads all it has to merge as ONE contiguous block.
    const int Sw = (((m + W - 1) / W) + 3) & ~3;
    const int strip0 = min(m, w * Sw), strip1 = min(m, strip0 + Sw);
    int lgSwp = 2;
    while ((1 << lgSwp) < Sw) ++lgSwp;
    const int Swp = 1 << lgSwp, lgQN = lgSwp - 2, QN = 1 << lgQN;    // QN 16-byte chunks per source set
    float *xchg = reinterpret_cast<float *>(A.colpart);
    // the column whose total this thread finishes in the merge
    const int own_col = strip0 + tid;
    const bool own_ok = tid < Sw && own_col < strip1;

    prefetch_p0(k);
    prefetch_p1(k);
    if (FULLW && mine > 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm(NDMA));
    else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    lds_only_barrier();

    bool alive = true;
    for (;;) {
        const int cur = k & 1, nxt = cur ^ 1;
        const bool rev = cur != 0;
        const bool trailing = k == c.max_iter;       // row phase only: the error of the last iterate
        float cS[Q][4];                              // column sums of the plan entries of this workgroup's rows
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) cS[q][e] = 0.0f;
        double err_acc = 0.0;                        // error terms of this workgroup's rows (lanes that own a row)

        FS_TRACE(0);
        int buf = 0;
        for (int t = 0; t < mine; ++t, buf ^= 1) {
            const int i0 = panel_row(t, rev);
            // Panel t and its row scalars must have landed.  FULLW: the only younger vector-memory operations
            // are the NDMA prefetch loads of the next panel (if there is one), which may stay in flight.
            if (FULLW && t + 1 < mine) __builtin_amdgcn_s_waitcnt(waitcnt_vm(NDMA));
            else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
            asm volatile("" ::: "memory");
            const int *sc = scal[buf][wave];
            const bool rowok = rr < R && (i0 + rr) < n;
            const double rho_lane = __hiloint2double(sc[R + rc], sc[rc]);
            const double la2_lane = rowok ? __hiloint2double(sc[3 * R + rc], sc[2 * R + rc]) : -__builtin_huge_val();
            const float a_lane = rowok ? __int_as_float(sc[4 * R + rc]) : 0.0f;
            double rho[R];
#pragma unroll
            for (int r = 0; r < R; ++r) rho[r] = __hiloint2double(sc[R + r], sc[r]);
            if (!FULLW && t + 1 < mine) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xc07f);  // every earlier read of the other staging buffer has returned
                issue(panel_row(t + 1, rev), buf ^ 1, cur, wave);
                asm volatile("" ::: "memory");
            }
            // ---- row phase, optimistic: e = 2^(x - rho_r), summed
            float ev[R][Q][4];
            float racc[R];                     // (Q == 1 only)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float acc = 0.0f;
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const float4 c4 = stage[buf][wave][r][q][lane];
                    float cvv[4];
                    unpack(c4, q, cvv);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
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
            // pi_ij = e_ij * a_i / S_i.  Every wave needs a_i / S_i (reciprocal, one Newton step, product: within 1.5
            // ulp); the new F = reference + log2 S is formed by the one wave that stores it, further down.
            double Fbase = rho_lane;
            float Ssum = S;
            float alpha_lane;
            {
                float rcp = __builtin_amdgcn_rcpf(S);
                rcp = fmaf(fmaf(-S, rcp, 1.0f), rcp, rcp);
                alpha_lane = a_lane * rcp;
            }
            if (__builtin_expect(!__all(fine || !rowok), 0)) {
                // ---- exact redo of the row phase of this panel (uniform over the workgroup): Eq. 8 as written,
                //      the maximum of the row first (no exponentials), then the sum relative to it
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    double mx = kNegHuge;
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        const float4 c4 = stage[buf][wave][r][q][lane];
                        float cvv[4];
                        unpack(c4, q, cvv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) mx = dmax(mx, fma(ns, (double)cvv[e], v[q][e]));
                    }
                    mx = wave_max_f64(mx);
                    if (lane == 0) sM[buf][r][wave] = mx;
                }
                lds_only_barrier();                              // (every wave has read sSum by now)
                double Mg = rr < R ? sM[buf][rc][lane % NW] : kNegHuge;
                Mg = dmax(Mg, dpp_f64<0x128>(Mg));
                Mg = dmax(Mg, dpp_f64<0x124>(Mg));
                Mg = dmax(Mg, dpp_f64<0x122>(Mg));
                Mg = dmax(Mg, dpp_f64<0x121>(Mg));
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const double Mr = bcast_f64(Mg, r * NW);
                    float acc = 0.0f;
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        const float4 c4 = stage[buf][wave][r][q][lane];
                        float cvv[4];
                        unpack(c4, q, cvv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            ev[r][q][e] = fast_exp2((float)(fma(ns, (double)cvv[e], v[q][e]) - Mr));
                            acc += ev[r][q][e];
                        }
                    }
                    acc = wave_sum_f32(acc);
                    if (lane == 0) sSum[buf][r][wave] = acc;
                }
                lds_only_barrier();
                float sg = rr < R ? sSum[buf][rc][lane % NW] : 1.0f;
                sg += dpp_f32<0x128>(sg);
                sg += dpp_f32<0x124>(sg);
                sg += dpp_f32<0x122>(sg);
                sg += dpp_f32<0x121>(sg);
                Fbase = Mg;
                Ssum = sg;
                alpha_lane = a_lane / sg;                          // e is relative to the row maximum: pi = e a / sum
            }
            if (wave == 0 && (lane % NW) == 0 && rowok) {
                // F stays with this workgroup (it is the old F of the same rows in the next iteration); U is
                // what a repair in another workgroup reads
                const double Fn_lane = Fbase + log2_sum(Ssum);
                p.F[(size_t)nxt * p.n_ld + i0 + rr] = Fn_lane;
                pub_f64(p.U + (size_t)nxt * p.n_ld + i0 + rr, la2_lane - Fn_lane);
                // error term of Sec. 4.5 for the iterate this iteration started from: a_i |2^(Fnew - Fold) - 1|
                if (a_lane > 0.0f) err_acc += (double)a_lane * fabs(exp2m1(Fn_lane - rho_lane));
            }
            // ---- prefetch of the panel after next into the buffer this panel occupied: nothing below reads it
            if (FULLW && t + 2 < mine) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xc07f);
                issue(panel_row(t + 2, rev), buf, cur, wave);
                asm volatile("" ::: "memory");
            }
            // ---- column phase with the new f (the trailing round does it too: its sums are simply not published)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float alpha = bcast_f32(alpha_lane, r * NW);
                if (!(alpha == alpha) || (i0 + r) >= n) alpha = 0.0f;   // rows past n, or a row whose F is not finite
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) cS[q][e] = fmaf(ev[r][q][e], alpha, cS[q][e]);
            }
        }

        FS_TRACE(1);
        // ---- publish: column sums of this workgroup's rows (16-byte stores), and the error terms of its rows
        {
            // where a group of 4 column sums goes: strip col / Sw, this workgroup's set, column col mod Sw
            const __amdgpu_buffer_rsrc_t rsX =
                __builtin_amdgcn_make_buffer_rsrc((void *)xchg, 0, ((W * W) << lgSwp) * 4, 0x00020000);
            if (!trailing)
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (colok(q)) {
                    const int col = (q * T + tid) * 4;
                    const int dest = col / Sw;
                    const v4u pk = {__float_as_uint(cS[q][0]), __float_as_uint(cS[q][1]), __float_as_uint(cS[q][2]),
                                    __float_as_uint(cS[q][3])};
                    __builtin_amdgcn_raw_buffer_store_b128(pk, rsX, ((((dest * W + w) << lgSwp) + (col - dest * Sw))) * 4, 0,
                                                           kAgent);
                }
            }
            if (wave == 0) {
                const double e = wave_sum_f64(err_acc);
                if (lane == 0) pub_f64(X.wgpart + w, e);
            }
        }
        // the old V of the column this thread will finish in the merge
        double myV = 0.0, myLb = 0.0;
        if (own_ok) {
            myV = get_f64(p.V + (size_t)cur * p.m_ld + own_col);
            myLb = p.lb2[own_col];
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));     // this wave's stores have been acknowledged
        lds_only_barrier();                            // ... and so have every wave's (the new F of this workgroup's rows too)
        FS_TRACE(2);
        const bool more = k + 1 < k_end || (k + 1 == k_end && with_trailing);
        ++gen;
        if (wave == 0) {
            const unsigned long long old = grid_arrive(X.sync);
            const int ok = grid_wait(X.sync, old, gen, W, X.spin_limit);
            if (lane == 0) sOk = ok;
        }
        lds_only_barrier();
        if (!sOk) { alive = false; break; }
        FS_TRACE(3);

        // ---- merge of this workgroup's strip; beside it, the error of the iterate this iteration started from
        //      (the same W terms in the same order in every workgroup, so that all take the same decision)
        {
            double *Vn = p.V + (size_t)nxt * p.m_ld, *Gn = p.G + (size_t)nxt * p.m_ld;
            const double *Un = p.U + (size_t)nxt * p.n_ld;
            // error terms of all workgroups: lane l of the last wave takes the terms 4 l .. 4 l + 3 (two 16-byte loads;
            // slots past the grid read as zero)
            v4u ep0 = {0u, 0u, 0u, 0u}, ep1 = {0u, 0u, 0u, 0u};
            if (wave == NW - 1) {
                const __amdgpu_buffer_rsrc_t rsE = __builtin_amdgcn_make_buffer_rsrc((void *)X.wgpart, 0, W * 8, 0x00020000);
                ep0 = __builtin_amdgcn_raw_buffer_load_b128(rsE, lane * 32, 0, kAgent);
                ep1 = __builtin_amdgcn_raw_buffer_load_b128(rsE, lane * 32 + 16, 0, kAgent);
            }
            // Chunk c of the block (16 bytes: 4 adjacent columns of one source set) belongs to set c / QN and
            // column group c % QN; thread t takes the chunks t, t + 1024, ..., i.e. always the same column group.
            // Four loads are in flight at a time; chunks past the end of the block read as zero.
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            const int nchunks = trailing ? 0 : W << lgQN;
            const __amdgpu_buffer_rsrc_t rsMine = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(xchg + ((size_t)(w * W) << lgSwp)), 0, (W << lgSwp) * 4, 0x00020000);
            for (int ch = tid; ch < nchunks; ch += 4 * T) {
                v4u x[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) x[u] = __builtin_amdgcn_raw_buffer_load_b128(rsMine, (ch + u * T) * 16, 0, kAgent);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    acc[0] += (double)__uint_as_float(x[u].x); acc[1] += (double)__uint_as_float(x[u].y);
                    acc[2] += (double)__uint_as_float(x[u].z); acc[3] += (double)__uint_as_float(x[u].w);
                }
            }
            double epart = (__hiloint2double((int)ep0.y, (int)ep0.x) + __hiloint2double((int)ep0.w, (int)ep0.z)) +
                           (__hiloint2double((int)ep1.y, (int)ep1.x) + __hiloint2double((int)ep1.w, (int)ep1.z));
#ifdef FS_PERSIST_TRACE
            asm volatile("" :: "v"(acc[0]), "v"(acc[1]), "v"(acc[2]), "v"(acc[3]));
            FS_TRACE(4);
#endif
            // lanes with the same column group (lane mod QN) meet inside the wave, in a fixed order
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double t4 = acc[e];
                if (lgQN <= 0) t4 += dpp_f64<0x121>(t4);
                if (lgQN <= 1) t4 += dpp_f64<0x122>(t4);
                if (lgQN <= 2) t4 += dpp_f64<0x124>(t4);
                if (lgQN <= 3) t4 += dpp_f64<0x128>(t4);
                if (lgQN <= 4) t4 += swz16_f64(t4);
                t4 += xor32_f64(t4);
                acc[e] = t4;
            }
            if (lane < QN) {
#pragma unroll
                for (int e = 0; e < 4; ++e) sPart[(wave << lgSwp) + lane * 4 + e] = acc[e];
            }
            if (wave == NW - 1) {
                epart = wave_sum_f64(epart);
                if (lane == 0) sErrTot = epart;
            }
            lds_only_barrier();
            FS_TRACE(5);
            if (own_ok && !trailing) {
                double tot = 0.0;
#pragma unroll
                for (int w2 = 0; w2 < NW; ++w2) tot += sPart[(w2 << lgSwp) + tid];
                // a column whose total mass is below 2^-66 (or not a number) may have lost terms to fp32
                // underflow: it is recomputed exactly below
                if (!(tot >= kColMassFloor)) {
                    sSus[atomicAdd(&sNsus, 1)] = own_col;
                } else {
                    const double out = log2_sum(tot) - myV;
                    pub_f64(Gn + own_col, out);
                    pub_f64(Vn + own_col, myLb - out);
                }
            }
            lds_only_barrier();
            const int nsus = sNsus;
            for (int q = 0; q < nsus; ++q) {
                const int jj = sSus[q];
                Lse ex; ex.init();
                for (int i = tid; i < n; i += T) {
                    double y[1] = {fma(ns, (double)A.C[(size_t)i * m + jj], get_f64(Un + i))};
                    ex.add<1>(y);
                }
                ex.wave_reduce();
                if (lane == 0) { sM[0][0][wave] = ex.M; sS[0][0][wave] = ex.s; }
                lds_only_barrier();
                if (tid == 0) {
                    Lse tl; tl.init();
#pragma unroll
                    for (int w2 = 0; w2 < NW; ++w2) tl.merge(sM[0][0][w2], sS[0][0][w2]);
                    const double out = tl.value();
                    pub_f64(Gn + jj, out);
                    pub_f64(Vn + jj, p.lb2[jj] - out);
                }
                lds_only_barrier();                    // sM is free again
            }
            if (tid == 0) sNsus = 0;                   // everyone has read it (a barrier lies behind every read)
        }
        const double err = sErrTot;
        if (trailing) {
            // nothing left to run: err of the last iterate closes the solve (potentials: F[cur], G[cur])
            if (w == 0 && tid == 0) {
                Ctl ct = c;
                ct.phase = 1;
                advance_state(ct, k, err, 0.0);
            }
            break;
        }
        if (c.tol > 0.0 && k >= 1 && (k % c.check_every == 0) && err < c.tol) {
            // stop at k (Alg. 1): F[cur], G[cur] still hold iterate k; what the merge wrote is the other buffer
            if (w == 0 && tid == 0) advance_state(c, k, err, 0.0);
            break;
        }
        ++gen;
        unsigned long long old2 = 0ull;
        if (wave == 0) {
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(0)); // the strip's new G and V (all published by this wave) are acknowledged
            old2 = grid_arrive(X.sync);
        }
        lds_only_barrier();
        // The first panel of the next iteration goes on its way now: the arrival is out, and by the time a poll
        // can see the last workgroup arrive, the memory pipeline of this compute unit has drained these requests.
        if (more) prefetch_p0(k + 1);
        if (wave == 0) {
            const int ok = grid_wait(X.sync, old2, gen, W, X.spin_limit);
            if (lane == 0) {
                sOk = ok;
                if (ok && w == 0) advance_state(c, k, err, 0.0);      // k + 1 iterations are complete
            }
        }
        lds_only_barrier();
        if (!sOk) { alive = false; break; }
        FS_TRACE(6);
        // ---- the new V of this lane's columns (16-byte loads, two values each)
        {
            const __amdgpu_buffer_rsrc_t rsV = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(p.V + (size_t)nxt * p.m_ld), 0, p.m_ld * 8, 0x00020000);
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int col = (q * T + tid) * 4;
                if (colok(q)) {
                    const v4u lo = __builtin_amdgcn_raw_buffer_load_b128(rsV, col * 8, 0, kAgent);
                    const v4u hi = __builtin_amdgcn_raw_buffer_load_b128(rsV, col * 8 + 16, 0, kAgent);
                    v[q][0] = __hiloint2double((int)lo.y, (int)lo.x);
                    v[q][1] = __hiloint2double((int)lo.w, (int)lo.z);
                    v[q][2] = __hiloint2double((int)hi.y, (int)hi.x);
                    v[q][3] = __hiloint2double((int)hi.w, (int)hi.z);
                    if (!FULLW) {
#pragma unroll
                        for (int e = 1; e < 4; ++e)
                            if (col + e >= m) v[q][e] = -__builtin_huge_val();
                    }
                }
            }
        }
        if (more) {
            // panel 1 behind the loads of V: "all but the youngest NDMA loads have landed" then means that V and
            // panel 0 are here (wave 0's panel 0 came through wave 1, hence the barrier)
            prefetch_p1(k + 1);
            if (FULLW && mine > 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm(NDMA));
            else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
            lds_only_barrier();
        }
        FS_TRACE(7);
        ++k;
        if (k >= k_end && !(k == k_end && with_trailing)) break;
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));         // no prefetch may land after the workgroup has given up its LDS
    if (!alive && tid == 0) {
        // abandoned: mark the solve as such and stop everything that was enqueued behind this launch
        atomicOr(&c.st->nonfinite, kGaveUp);
        atomicOr(&c.st->flags, kFlagDone);
        if (c.host_flag) {
            *c.host_flag = 1;
            __threadfence_system();
        }
    }
#endif
}

struct PShape { int Q, R; };

// the widths of the LDS-prefetch fused pass, fp32 costs: R = 2 rows per panel up to 8192 columns, else 1
bool persist_shape(int n, int m, PShape *s) {
    if (m <= 1024 || m > 16384) return false;
    // 4096 columns exactly (every lane owns valid columns) and enough rows: panels of 4 rows, 64 KiB like those of
    // 8192 columns (c3: 21.1 -> 20.3 us per iteration against panels of 2 rows, side by side)
    if (m == 4096 && n >= 2048) *s = {1, 4};
    else if (m <= 4096) *s = {1, 2};
    else if (m <= 8192) *s = {2, 2};
    else if (m <= 12288) *s = {3, 1};
    else *s = {4, 1};
    return true;
}

// widths that only the resident form takes (two, four or eight row groups per workgroup): the streaming form has no shape for them
bool narrow_shape(int m) { return m > 128 && m <= 1024; }

}  // namespace

bool dense_persist_supported(int n, int m, const void *C, int c_dtype) {
    PShape s;
    return c_dtype == 0 && (persist_shape(n, m, &s) || narrow_shape(m)) && ((reinterpret_cast<uintptr_t>(C) & 3u) == 0);
}

// Workgroups of the persistent launch: one per compute unit, never more than there are panels.  0 when the
// shape is not taken: every workgroup merges a strip of m / workgroups columns and the kernel holds 64 of
// them, so a short matrix (few panels) or a small device leaves too few workgroups for a wide one.
int dense_persist_grid(int n, int m, int cus) {
    PShape s;
    if (narrow_shape(m)) return dense_resident_grid(n, m, cus > 256 ? 256 : cus, true);
    if (!persist_shape(n, m, &s) || cus < 1) return 0;
    const int npanels = (n + s.R - 1) / s.R;
    int g = npanels < cus ? npanels : cus;
    if (g > kWgPartLd) g = kWgPartLd;
    if (g > 256) g = 256;                                  // the exchange buffer holds 256 sets of column sums
    const int strip = (((m + g - 1) / g) + 3) & ~3;
    return strip <= 64 ? g : 0;
}

size_t persist_scratch_bytes() { return sizeof(PersistSync) + sizeof(double) * kWgPartLd; }

bool dense_persist_resident(int n, int m, int cus, int variant) {
    if (narrow_shape(m)) return dense_resident_grid(n, m, cus > 256 ? 256 : cus, true) > 0;
    return variant != 1 && dense_resident_grid(n, m, cus > 256 ? 256 : cus, variant == 2) > 0;
}


hipError_t launch_persist(hipStream_t st, const DenseArgs &a, const Ctl &c, void *scratch, int cus, int nb,
                          int spin_limit, int final_err, int variant, const Stamp &tm) {
    PShape s{0, 0};
    const bool narrow = narrow_shape(a.p.m);
    if (!scratch || a.c_dtype != 0 || !(narrow || persist_shape(a.p.n, a.p.m, &s)) || nb < 1) return hipErrorInvalidValue;
    const int g = dense_persist_grid(a.p.n, a.p.m, cus);
    // the exchange buffer holds a.P sets of column sums, and [strip][source][strip width rounded up to a power of
    // two] floats must fit what a.P sets of doubles take
    auto exchange_fits = [&](int grid) {
        if (grid < 1 || grid > a.P) return false;
        const int strip = (((a.p.m + grid - 1) / grid) + 3) & ~3;
        int swp = 4;
        while (swp < strip) swp <<= 1;
        return (size_t)grid * grid * swp * sizeof(float) <= (size_t)a.P * a.p.m_ld * sizeof(double);
    };
    if (!exchange_fits(g)) return hipErrorInvalidValue;
    PersistArgs x;
    x.sync = reinterpret_cast<PersistSync *>(scratch);
    x.wgpart = reinterpret_cast<double *>(x.sync + 1);
    x.nb = nb;
    x.spin_limit = spin_limit > 0 ? spin_limit : (1 << 21);
    x.final_err = final_err;
#ifdef FS_PERSIST_TRACE
    x.trace = nullptr;
    if (const char *tp = getenv("FS_TRACE_PTR")) x.trace = reinterpret_cast<long long *>(strtoull(tp, nullptr, 0));
#endif
    if (narrow) return launch_resident(st, a, x, c, g, tm);      // (g is the resident grid, and it fits)
    if (variant != 1) {
        // (cus is at most a.P here: the exchange buffer holds a set of column sums per workgroup of either form)
        const int gr = dense_resident_grid(a.p.n, a.p.m, cus > 256 ? 256 : cus, variant == 2);
        if (gr > 0 && exchange_fits(gr)) return launch_resident(st, a, x, c, gr, tm);
    }
    const dim3 grid(g), block(1024);
    const int m = a.p.m;
    if (s.Q == 1 && s.R == 4) launch_stamped((k_persist<1, 4, true>), grid, block, st, tm, a, x, c);
    else if (s.Q == 1 && m == 4096) launch_stamped((k_persist<1, 2, true>), grid, block, st, tm, a, x, c);
    else if (s.Q == 1) launch_stamped((k_persist<1, 2, false>), grid, block, st, tm, a, x, c);
    else if (s.Q == 2 && m == 8192) launch_stamped((k_persist<2, 2, true>), grid, block, st, tm, a, x, c);
    else if (s.Q == 2) launch_stamped((k_persist<2, 2, false>), grid, block, st, tm, a, x, c);
    else if (s.Q == 3 && m == 12288) launch_stamped((k_persist<3, 1, true>), grid, block, st, tm, a, x, c);
    else if (s.Q == 3) launch_stamped((k_persist<3, 1, false>), grid, block, st, tm, a, x, c);
    else if (m == 16384) launch_stamped((k_persist<4, 1, true>), grid, block, st, tm, a, x, c);
    else launch_stamped((k_persist<4, 1, false>), grid, block, st, tm, a, x, c);
    return hipGetLastError();
}

}  // namespace fs
