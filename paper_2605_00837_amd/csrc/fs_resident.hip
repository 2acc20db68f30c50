// Resident form of the persistent fused pass (Alg. 1, Eqs. 9-10): a block of Sinkhorn iterations in ONE launch
// during which the cost matrix never leaves the chip.
//
// A compute unit of this device has 160 KiB of LDS and 512 KiB of vector registers.  With one workgroup of 512
// lanes per compute unit (two waves per SIMD, 256 registers per lane), a share of up to 4 panels of 64 KiB
// (256 KiB: a 64 MiB matrix on 256 compute units, e.g. 8192 x 2048, 4096 x 4096 or 2048 x 8192) is read from
// memory ONCE per launch -- panels 0 and 1 into 64 registers per lane, panels 2 and 3 into LDS -- and every
// iteration of the block runs its row and column phase from there.  The iteration is then bound by the vector
// ALUs (about 11 instructions per entry) and by the exchange, not by the memory system; the persistent pass
// that streams C (fs_persist.hip) reads it from the last-level cache every iteration.  (1024 lanes with 128
// registers each hold the same bytes, but 32 of 128 registers for the panels leave the hot loop short of
// registers and it runs 8 % slower.)
//
// Widths from 129 to 8192 columns are taken: a panel is 8 rows up to 2048 columns, 4 up to 4096, 2 beyond, and
// the lanes whose columns lie past m are masked.  Up to 1024 columns a row does not need 512 lanes: the workgroup
// splits into 2 (513 .. 1024 columns, panels of 16 rows), 4 (257 .. 512, 32 rows) or 8 (129 .. 256, 64 rows: a wave per
// row) row groups.  The grid is one workgroup per compute unit, fewer for a short
// matrix.  A share of more than 4 panels is streamed: the two register panels
// stay, the others go through the two LDS buffers two panels ahead, upwards in one iteration and downwards in
// the next, so that the two panels a pass ends with are already there for the next one.
//
// Everything else is the persistent pass: the same optimistic row phase with its exact redo, the same fp32
// column sums, the same exchange between two bounded grid-wide waits (publish, merge of the own strip with the
// exact repair of columns below 2^-66, new G and V, read), the same stop rule (Alg. 1), the same trailing row
// phase for the error of the last iterate (Sec. 4.5), a fixed order of every sum (results do not depend on timing).  The old F of the
// workgroup's rows stays in LDS as well (two parities); F and U still go to memory every iteration, for the
// repairs in other workgroups and for whatever runs after this launch.
#include <type_traits>

#include "fs_kernels.h"
#include "fs_persist_sync.h"

namespace fs {

namespace {

constexpr int kResRegs = 2;             // panels a workgroup keeps in registers (64 registers per lane)
constexpr int kResLds = 2;              // panels the LDS holds: the other resident ones, or the two staging buffers
constexpr int kResPanels = kResRegs + kResLds;   // up to here the whole share stays on the chip
constexpr int kResMaxPanels = 32;       // panels per workgroup at most (row scalars in LDS)
constexpr int kResAutoPanels = kResMaxPanels;   // this kernel is the faster one as far as it goes (measured, 8192 columns:
                                        // 31.7 against 36.3 us per iteration at 6144 rows, 40.5 / 46.0 at 8192, 53.0 / 57.6
                                        // at 10240, 66.7 / 69.6 at 12288, 78.1 / 80.2 at 14336, 87.0 / 90.8 at 16384; 4096
                                        // columns: 39.7 / 45.4 at 16384 rows, 51.9 / 56.7 at 20480, 66.3 / 68.6 at 24576,
                                        // 79.1 / 80.6 at 28672; 2048 columns, where the 1024-lane kernel has idle lanes:
                                        // 40.4 / 86.3 at 32768 rows) ...
constexpr int kResAutoPanelsWide = 20;  // ... except between 6145 and 8191 columns (8000 x 8000: 42.8 against 46.2,
                                        // 9000 x 8100: 49.6 / 52.9, 10000 x 7000: 50.0 / 51.9, 10000 x 8000: 55.4 / 57.4, but
                                        // 12000 x 8000: 69.5 / 68.1, 14000 x 7000: 78.0 / 71.1)

// All-reduce over aligned groups of LW lanes (16: a DPP row, rotated; 1: nothing to do; 2: lane ^ 1; 4: then lane ^ 2; 8: then the half row mirrored).
template <int LW>
__device__ __forceinline__ float group_sum_f32(float x) {
    if (LW == 16) {
        x += dpp_f32<0x128>(x);
        x += dpp_f32<0x124>(x);
        x += dpp_f32<0x122>(x);
        x += dpp_f32<0x121>(x);
    } else {
        if (LW >= 2) x += dpp_f32<0xB1>(x);     // quad_perm [1, 0, 3, 2]
        if (LW >= 4) x += dpp_f32<0x4E>(x);     // quad_perm [2, 3, 0, 1]
        if (LW == 8) x += dpp_f32<0x141>(x);    // row_half_mirror
    }
    return x;
}
template <int LW>
__device__ __forceinline__ double group_max_f64(double x) {
    if (LW == 16) {
        x = dmax(x, dpp_f64<0x128>(x));
        x = dmax(x, dpp_f64<0x124>(x));
        x = dmax(x, dpp_f64<0x122>(x));
        x = dmax(x, dpp_f64<0x121>(x));
    } else {
        if (LW >= 2) x = dmax(x, dpp_f64<0xB1>(x));
        if (LW >= 4) x = dmax(x, dpp_f64<0x4E>(x));
        if (LW == 8) x = dmax(x, dpp_f64<0x141>(x));
    }
    return x;
}

// Q groups of 4 adjacent columns per lane (column(q, e) = (q 512 + tid) 4 + e), R rows per panel, R Q <= 8 H (a panel
// is at most 64 KiB: 32 entries per lane; 48 KiB for the widths up to 6144 columns).  FULLW: m = 2048 Q / H, every
// lane owns valid columns; else m is less than that and the columns past m are masked (V = -inf, C = 0, nothing
// published).
// H > 1 (narrow matrices): the workgroup is H row groups of T / H lanes; a row is spread over the NW / H waves of
// its group only (column(q, e) = (q T / H + tid mod (T / H)) 4 + e) and group h works on the rows h R / H ...
// of every panel; the groups add their column sums in LDS before the workgroup publishes them.  The row scalars
// of kResMaxPanels panels of 16 rows fit the LDS; taller panels (H > 2) come with proportionally fewer of them.
template <int Q, int R, int NW, bool STREAM, bool FULLW, int H = 1>
__global__ __launch_bounds__(64 * NW) void k_resident(DenseArgs A, PersistArgs X, Ctl c) {
    constexpr int T = 64 * NW, NP = H > 2 ? 2 * kResMaxPanels / H : kResMaxPanels, NR = kResRegs, NL = kResLds;
    constexpr int TC = T / H, RH = R / H, NWH = NW / H;      // lanes per row, rows per group and panel, waves per row
    constexpr int NDMA = RH * Q;               // prefetch loads per panel and wave
    constexpr int LW = R <= 4 ? 16 : 64 / R;   // lanes per row in the merge of the wave sums: NWH partials (then zeros)
    static_assert(T % H == 0 && R % H == 0 && NW % H == 0 && TC % 64 == 0, "whole waves per row group");
    static_assert(RH * Q * NW <= 64, "a panel is at most 64 KiB");
    static_assert(R * LW <= 64 && NWH <= LW, "one wave merges all (row, wave) partials in one shot");
    constexpr float kRowHi = 1.1529215e18f;    // 2^60
    constexpr float kRowLo = 9.5367432e-07f;   // 2^-20
    __shared__ float4 stage[NL][NW][RH][Q][64]; // the panels behind the register panels (two: resident; more: staged), every wave its own slice
    __shared__ double sF[2][NP][R];            // F of this workgroup's rows by parity of the iteration; kPadF past n
    __shared__ double sLa2[NP][R];
    __shared__ float sA[NP][R];
    __shared__ float sSum[NR + NL][R][NWH];    // by register panel, then by staging buffer
    __shared__ double sM[R][NWH];              // exact redo: row maxima by wave
    __shared__ double sMr[NW];                 // exact repair of a column: running pairs by wave
    __shared__ float sSr[NW];
    constexpr int NPART = (H - 1) * TC * Q * 2 > T ? (H - 1) * TC * Q * 2 : T;
    __shared__ double sPart[NPART];            // merge: partial totals by (set group, column); the row groups' column sums
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
    const int rr = lane / LW, ww = lane % LW;  // the panel row and the wave whose partial this lane takes in the merge
    const int rc = rr < R ? rr : R - 1;
    const int wc = ww < NWH ? ww : NWH - 1;
    // (one row group: plain constants, so that nothing of this is left in the code)
    const int tc = H == 1 ? tid : tid % TC;    // the lane's place in its row group: it owns the columns (q TC + tc) 4 ...
    const int hh = H == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid / TC);       // row group
    const int wq = H == 1 ? wave : wave % NWH;                                 // the wave's place in it
    static_assert(sizeof(sPart) >= (size_t)(H - 1) * TC * Q * 16, "the row groups meet in sPart");

    int k;
    if (!launch_active(c, k)) return;
    const int k_end = min(k + X.nb, c.max_iter);
    // the launch that reaches max_iter goes on with one more row phase: it yields err of the last iterate
    const bool with_trailing = X.final_err != 0 && k_end == c.max_iter;

    // This workgroup owns the panels w, w + W, ... (3 .. NP of them, or at most NR + NL: the launcher sees to it), in
    // every iteration.  Panels 0 .. NR-1 live in registers.  The others live in LDS when there are at most NL of
    // them (loaded once); else they are streamed through the NL staging buffers every iteration, two panels
    // ahead, upwards on even and downwards on odd iterations: the two panels a pass ends with are the two the next
    // pass begins with, they stay in the staging buffers and are not fetched again (and what the last-level cache
    // still holds from the pass before is read first).
    const int npanels = (n + R - 1) / R;
    const int mine = (npanels - 1 - w) / W + 1;
    const int ms = mine > NR ? mine - NR : 0;          // panels behind the register panels
    const bool streaming = STREAM && ms > NL;      // (STREAM = false: the launcher has seen that no workgroup has more)
    if (tid == 0) {
        // waits completed so far in this solve: the generation numbers of this launch go on from there
        sGen = __hip_atomic_load(&X.sync->done[w % kSyncGroups], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sNsus = 0;
    }
    for (int x = tid; x < NP * R; x += T) {
        const int t = x / R, r = x % R;
        const int row = (w + t * W) * R + r;
        const bool ok = t < mine && row < n;
        sF[k & 1][t][r] = ok ? p.F[(size_t)(k & 1) * p.n_ld + row] : kPadF;
        sF[(k & 1) ^ 1][t][r] = kPadF;         // (rows of this workgroup: written before it is read)
        sLa2[t][r] = ok ? p.la2[row] : -__builtin_huge_val();
        sA[t][r] = ok ? p.a[row] : 0.0f;
    }
    // panel j of this workgroup: rows (w + j W) R ...; its descriptor covers exactly the valid rows (rows past n read as 0)
    auto panel_rsrc = [&](int j) {
        const int i0 = (w + j * W) * R;
        const int rows = j < mine ? ((n - i0) < R ? (n - i0) : R) : 0;
        return __builtin_amdgcn_make_buffer_rsrc((void *)((const char *)A.C + (size_t)(j < mine ? i0 : 0) * m * 4), 0,
                                                 rows * m * 4, 0x00020000);
    };
    // memory -> LDS without passing through registers: panel j into staging buffer buf, every wave its own slice
    // (slice tw: the wave's own, except between iterations, see below)
    auto issue = [&](int j, int buf, int tw) {
        const __amdgpu_buffer_rsrc_t rsrc = panel_rsrc(j);
        const int tslot = H == 1 ? tw * 64 + lane : (tw * 64 + lane) % TC;     // place in the row group
        const int tg = H == 1 ? 0 : (tw * 64) / TC;                             // row group of slice tw
#pragma unroll
        for (int r = 0; r < RH; ++r)
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                // a lane whose columns lie past m asks for an address outside the descriptor: nothing is read from
                // memory for it, zeros land in LDS, and every wave still issues the same number of loads
                const int voff = (FULLW || (q * TC + tslot) * 4 < m) ? tslot * 16 : 0x40000000;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, &stage[buf][tw][r][q][0], 16, voff,
                                                         ((tg * RH + r) * m + q * TC * 4) * 4, 0, 0);
            }
    };
    // the panel behind the register panels that a pass visits in position t
    auto lds_panel = [&](int t, bool rev) { return NR + (rev ? ms - 1 - t : t); };
    // ---- the register panels, once per launch
    float creg[NR][RH][Q][4];
#pragma unroll
    for (int t = 0; t < NR; ++t) {
        const __amdgpu_buffer_rsrc_t rsrc = panel_rsrc(t);
#pragma unroll
        for (int r = 0; r < RH; ++r)
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const v4u x = __builtin_amdgcn_raw_buffer_load_b128(rsrc, tc * 16, ((hh * RH + r) * m + q * TC * 4) * 4, 0);
                float (&cr)[4] = creg[t][r][q];
                cr[0] = __uint_as_float(x.x); cr[1] = __uint_as_float(x.y);
                cr[2] = __uint_as_float(x.z); cr[3] = __uint_as_float(x.w);
                if (!FULLW) {
                    // columns past m: what was read there belongs to the next row (or to nobody); the entry counts
                    // for nothing (V = -inf there) and is set to 0 so that it cannot turn -inf into NaN either
                    const int col = (q * TC + tc) * 4;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e >= m) cr[e] = 0.0f;
                }
            }
    }
    // ---- the LDS panels: the resident ones once per launch; a streaming workgroup the first two of its first pass
    //      (every later pass finds its first two where the pass before it left them)
    const bool rev0 = STREAM && (k & 1) != 0;
    if (ms > 0) issue(lds_panel(0, rev0), 0, wave);
    if (ms > 1) issue(lds_panel(1, rev0), 1, wave);
    // V of this lane's columns (written before this launch)
    double v[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int col = (q * TC + tc) * 4;
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
    const int lgQN = lgSwp - 2, QN = 1 << lgQN;        // QN 16-byte chunks per source set
    float *xchg = reinterpret_cast<float *>(A.colpart);
    // the column whose total this thread finishes in the merge
    const int own_col = strip0 + tid;
    const bool own_ok = tid < Sw && own_col < strip1;

    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));         // the LDS panels have landed
    if (!FULLW && !STREAM) {
        // the same for the LDS panels (every lane its own entries; once per launch: they are resident)
#pragma unroll
        for (int b = 0; b < NL; ++b)
#pragma unroll
            for (int r = 0; r < RH; ++r)
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const int col = (q * TC + tc) * 4;
                    if (col + 4 > m) {
                        float4 c4 = stage[b][wave][r][q][lane];
                        if (col >= m) c4.x = 0.0f;
                        if (col + 1 >= m) c4.y = 0.0f;
                        if (col + 2 >= m) c4.z = 0.0f;
                        if (col + 3 >= m) c4.w = 0.0f;
                        stage[b][wave][r][q][lane] = c4;
                    }
                }
    }
    __syncthreads();
    unsigned long long gen = sGen;

    bool alive = true;
    int flip = 0;                                // the staging buffer of the pass's first staged panel
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
        // One panel: REG >= 0: register panel REG (= panel REG of this workgroup); REG < 0: the panel j in staging
        // buffer slot - NR.  `slot` also names the row-sum staging this panel uses.
        auto do_panel = [&](auto reg_tag, int slot, int j, int jnext = -1) {
            constexpr int REG = decltype(reg_tag)::value;
            const int i0 = (w + j * W) * R;
            const bool rowok = rr < R && (i0 + rr) < n;
            const double rho_lane = sF[cur][j][rc];
            const double la2_lane = rowok ? sLa2[j][rc] : -__builtin_huge_val();
            const float a_lane = rowok ? sA[j][rc] : 0.0f;
            double rho[RH];                    // (r below: a row of this lane's group, row hh RH + r of the panel)
#pragma unroll
            for (int r = 0; r < RH; ++r) rho[r] = sF[cur][j][hh * RH + r];
            // the 4 entries (r, q, .) of this panel as fp64 values: from the lane's registers (through a compiler
            // barrier: every use converts the 4-byte register afresh; without it the converted values of all
            // register panels are kept over the iteration loop, in twice the registers), or from LDS
            auto cost4 = [&](int r, int q, double (&o)[4]) {
                if constexpr (REG >= 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = cost_f64(creg[REG][r][q][e]);
                } else {
                    const float4 c4 = stage[slot - NR][wave][r][q][lane];
                    o[0] = (double)c4.x; o[1] = (double)c4.y; o[2] = (double)c4.z; o[3] = (double)c4.w;
                }
            };
            if constexpr (REG < 0 && !FULLW && STREAM) {
                // a staged panel has just landed: the one lane per row that owns the last valid column clears what it
                // read past it (entries of the next row: they count for nothing, V = -inf there, and must not be NaN)
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const int col = (q * TC + tc) * 4;
                    if (col < m && col + 4 > m) {
#pragma unroll
                        for (int r = 0; r < RH; ++r) {
                            float4 c4 = stage[slot - NR][wave][r][q][lane];
                            if (col + 1 >= m) c4.y = 0.0f;
                            if (col + 2 >= m) c4.z = 0.0f;
                            if (col + 3 >= m) c4.w = 0.0f;
                            stage[slot - NR][wave][r][q][lane] = c4;
                        }
                    }
                }
            }
            // ---- row phase, optimistic: e = 2^(x - rho_r), summed
            float ev[RH][Q][4];
            float racc[RH];
#pragma unroll
            for (int r = 0; r < RH; ++r) {
                float acc = 0.0f;
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    double cvv[4];
                    cost4(r, q, cvv);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        ev[r][q][e] = fast_exp2((float)(fma(ns, cvv[e], v[q][e]) - rho[r]));
                        acc += ev[r][q][e];
                    }
                }
                racc[r] = acc;
            }
            rows_sum_store<RH>(racc, &sSum[slot][hh * RH][wq], NWH, lane);
            lds_only_barrier();
            float S = rr < R ? (ww < NWH ? sSum[slot][rc][wc] : 0.0f) : 1.0f;
            S = group_sum_f32<LW>(S);
            const bool fine = (S >= kRowLo) && (S <= kRowHi);    // false for NaN / inf / 0
            // pi_ij = e_ij * a_i / S_i.  Every wave needs a_i / S_i (reciprocal, one Newton step, product: within
            // 1.5 ulp); the new F = reference + log2 S is formed by the one wave that stores it, further down.
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
                for (int r = 0; r < RH; ++r) {
                    double mx = kNegHuge;
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        double cvv[4];
                        cost4(r, q, cvv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) mx = dmax(mx, fma(ns, cvv[e], v[q][e]));
                    }
                    mx = wave_max_f64(mx);
                    if (lane == 0) sM[hh * RH + r][wq] = mx;
                }
                lds_only_barrier();                              // (every wave has read sSum by now)
                double Mg = rr < R && ww < NWH ? sM[rc][wc] : kNegHuge;
                Mg = group_max_f64<LW>(Mg);
#pragma unroll
                for (int r = 0; r < RH; ++r) {
                    const double Mr = bcast_f64(Mg, (hh * RH + r) * LW);
                    float acc = 0.0f;
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        double cvv[4];
                        cost4(r, q, cvv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            ev[r][q][e] = fast_exp2((float)(fma(ns, cvv[e], v[q][e]) - Mr));
                            acc += ev[r][q][e];
                        }
                    }
                    acc = wave_sum_f32(acc);
                    if (lane == 0) sSum[slot][hh * RH + r][wq] = acc;
                }
                lds_only_barrier();                              // (and every wave has read sM)
                float sg = rr < R ? (ww < NWH ? sSum[slot][rc][wc] : 0.0f) : 1.0f;
                sg = group_sum_f32<LW>(sg);
                Fbase = Mg;
                Ssum = sg;
                alpha_lane = a_lane / sg;                          // e is relative to the row maximum: pi = e a / sum
            }
            if (wave == 0 && ww == 0 && rowok) {
                // the new F stays in LDS (the old F of the same rows in the next iteration) and goes to memory for
                // whatever runs after this launch; U is what a repair in another workgroup reads
                const double Fn_lane = Fbase + log2_sum(Ssum);
                int row = i0 + rr;
                asm volatile("" : "+v"(row));          // (addresses formed here, not kept in registers over the loop)
                sF[nxt][j][rr] = Fn_lane;
                p.F[(size_t)nxt * p.n_ld + row] = Fn_lane;
                pub_f64(p.U + (size_t)nxt * p.n_ld + row, la2_lane - Fn_lane);
                // error term of Sec. 4.5 for the iterate this iteration started from: a_i |2^(Fnew - Fold) - 1|
                if (a_lane > 0.0f) err_acc += (double)a_lane * fabs(exp2m1(Fn_lane - rho_lane));
            }
            if constexpr (REG < 0 && STREAM) {
                // nothing below reads the staging buffer: the panel after next goes into it now (this wave's own
                // slice, its reads are done)
                if (jnext >= 0) {
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_s_waitcnt(0xc07f);
                    issue(jnext, slot - NR, wave);
                    asm volatile("" ::: "memory");
                }
            }
            // ---- column phase with the new f (the trailing round does it too: its sums are simply not published)
#pragma unroll
            for (int r = 0; r < RH; ++r) {
                float alpha = bcast_f32(alpha_lane, (hh * RH + r) * LW);
                if (!(alpha == alpha) || (i0 + hh * RH + r) >= n) alpha = 0.0f;   // rows past n, or a row whose F is not finite
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) cS[q][e] = fmaf(ev[r][q][e], alpha, cS[q][e]);
            }
        };
        // A streaming workgroup is bound by the memory system (a panel arrives in 2.3 us and takes 1.7 us of
        // arithmetic): its register panels go early in the pass, one behind each of the first two staged panels (which
        // are already here when the pass begins), so that the first requests of the pass have a lead over the
        // arithmetic that absorbs the spread of the fetch times.  (With masked lanes: behind the second and the
        // third.  Measured; later in the pass, or both in one place, is 1 - 3 us per iteration slower at 8192 x 8192.)
        if constexpr (!STREAM) {
            // everything is on the chip: the panels in program order, every index a constant
            if (ms > 0) do_panel(std::integral_constant<int, -1>(), NR, NR);
            if (ms > 1) do_panel(std::integral_constant<int, -1>(), NR + 1, NR + 1);
            if (mine > 0) do_panel(std::integral_constant<int, 0>(), 0, 0);
            if (mine > 1) do_panel(std::integral_constant<int, 1>(), 1, 1);
        } else {
        int regs_done = 0;
        auto reg_panel = [&]() {
            if (regs_done == 0 && mine > 0) do_panel(std::integral_constant<int, 0>(), 0, 0);
            if (regs_done == 1 && mine > 1) do_panel(std::integral_constant<int, 1>(), 1, 1);
            ++regs_done;
        };
        for (int t = 0; t < ms; ++t) {
            const int buf = (t + flip) & 1;
            if (streaming && t >= (FULLW ? 1 : 2) && regs_done < NR) reg_panel();
            if (streaming) {
                // Panel t must have landed: the only younger vector-memory operations are the NDMA loads of panel
                // t + 1 (if there is one), which may stay in flight (loads return in order; what wave 0 stored
                // after them only makes its wait stricter).
                if (t + 1 < ms) __builtin_amdgcn_s_waitcnt(waitcnt_vm(NDMA));
                else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
                asm volatile("" ::: "memory");
            }
            do_panel(std::integral_constant<int, -1>(), NR + buf, lds_panel(t, rev),
                     streaming && t + 2 < ms ? lds_panel(t + 2, rev) : -1);
        }
        // The sweep turns round: the last two staged panels of this pass are the first two of the next one, they stay
        // where they are (no load of the exchange ever queues behind a prefetch), and the buffers swap roles when
        // the last panel sits in the buffer that the first one started in.
        if (ms > 0) flip ^= (ms - 1) & 1;
        while (regs_done < NR) reg_panel();
        }

        FS_TRACE(1);
        if constexpr (H > 1) {
            // the row groups add their column sums: groups 1 .. H-1 hand theirs over in LDS (sPart is free until the merge)
            float *sCS = reinterpret_cast<float *>(sPart);
            if (hh > 0) {
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) sCS[(((hh - 1) * Q + q) * 4 + e) * TC + tc] = cS[q][e];
            }
            lds_only_barrier();
            if (hh == 0) {
#pragma unroll
                for (int g2 = 1; g2 < H; ++g2)
#pragma unroll
                    for (int q = 0; q < Q; ++q)
#pragma unroll
                        for (int e = 0; e < 4; ++e) cS[q][e] += sCS[(((g2 - 1) * Q + q) * 4 + e) * TC + tc];
            }
        }                                              // (barriers lie between these reads and the merge's use of sPart)
        // ---- publish: column sums of this workgroup's rows (16-byte stores), and the error terms of its rows
        {
            // where a group of 4 column sums goes: strip col / Sw, this workgroup's set, column col mod Sw
            const __amdgpu_buffer_rsrc_t rsX =
                __builtin_amdgcn_make_buffer_rsrc((void *)xchg, 0, ((W * W) << lgSwp) * 4, 0x00020000);
            if (!trailing)
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int col = (q * TC + tc) * 4;
                if (hh == 0 && (FULLW || col < m)) {
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
        lds_only_barrier();                            // ... and so have every wave's
        FS_TRACE(2);
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
            // column group c % QN; thread t takes the chunks t, t + T, ..., i.e. always the same column group.
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
                if (lane == 0) { sMr[wave] = ex.M; sSr[wave] = ex.s; }
                lds_only_barrier();
                if (tid == 0) {
                    Lse tl; tl.init();
#pragma unroll
                    for (int w2 = 0; w2 < NW; ++w2) tl.merge(sMr[w2], sSr[w2]);
                    const double out = tl.value();
                    pub_f64(Gn + jj, out);
                    pub_f64(Vn + jj, p.lb2[jj] - out);
                }
                lds_only_barrier();                    // sMr is free again
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
                const int col = (q * TC + tc) * 4;
                if (FULLW || col < m) {
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
#ifdef FS_PERSIST_TRACE
        asm volatile("" :: "v"(v[0][0]), "v"(v[Q - 1][3]));
#endif
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

}  // namespace

// The shapes this kernel takes: fp32 costs, 128 < m <= 8192 (panels of 64 rows up to 256 columns, of 32 up to 512, of 16 up to 1024, of 8 up to 2048, of 4 up to 4096,
// of 2 beyond; 2048, 4096, 6144 or 8192 column slots), on a grid of one workgroup per compute unit, never more than there are panels and never so few
// that a workgroup would merge a strip of more than 64 columns.  Up to kResPanels panels per workgroup the whole
// share stays on the chip; beyond, the panels behind the register panels are streamed: up to kResAutoPanels as the
// library's own choice (between 6145 and 8191 columns: kResAutoPanelsWide), up to kResMaxPanels on request (`all`).  Up to 1024 columns: always up to kResMaxPanels (half of that up to 512
// columns, a quarter up to 256: the row scalars of a taller panel take more LDS), i.e. 512 rows per workgroup.
// Returns the workgroups of the launch, 0 when the shape is not taken.
int dense_resident_grid(int n, int m, int cus, bool all) {
    if (cus < 1 || n < 1 || m <= 128 || m > 8192) return 0;
    const int R = m <= 256 ? 64 : m <= 512 ? 32 : m <= 1024 ? 16 : m <= 2048 ? 8 : m <= 4096 ? 4 : 2;
    const long long npanels = ((long long)n + R - 1) / R;
    long long g = npanels < cus ? npanels : cus;
    if (g > 256) g = 256;                                  // the exchange buffer holds 256 sets of column sums
    const int strip = (int)(((m + g - 1) / g + 3) & ~3ll);
    if (strip > 64) return 0;
    // (widths with idle lanes: 6000 x 6000 30.7 against 34.0 us per iteration, 8000 x 5000 38.0 / 40.6,
    // 16384 x 3000 43.1 / 53.2, 12000 x 1500 22.5 / 40.5)
    const long long most = m <= 256 ? kResMaxPanels / 4 : m <= 512 ? kResMaxPanels / 2 : all ? kResMaxPanels : (m > 6144 && m < 8192) ? kResAutoPanelsWide : kResAutoPanels;
    return npanels <= most * g ? (int)g : 0;
}

hipError_t launch_resident(hipStream_t st, const DenseArgs &a, const PersistArgs &x, const Ctl &c, int grid,
                           const Stamp &tm) {
    if (a.c_dtype != 0 || grid < 1 || dense_resident_grid(a.p.n, a.p.m, grid, true) != grid) return hipErrorInvalidValue;
    const dim3 g(grid), block(512);
    const int m = a.p.m;
    const int R = m <= 256 ? 64 : m <= 512 ? 32 : m <= 1024 ? 16 : m <= 2048 ? 8 : m <= 4096 ? 4 : 2;
    const bool stream = ((long long)a.p.n + R - 1) / R > (long long)kResPanels * grid;
    if (m == 256) {
        if (stream) launch_stamped((k_resident<1, 64, 8, true, true, 8>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 64, 8, false, true, 8>), g, block, st, tm, a, x, c);
    } else if (m < 256) {
        if (stream) launch_stamped((k_resident<1, 64, 8, true, false, 8>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 64, 8, false, false, 8>), g, block, st, tm, a, x, c);
    } else if (m == 512) {
        if (stream) launch_stamped((k_resident<1, 32, 8, true, true, 4>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 32, 8, false, true, 4>), g, block, st, tm, a, x, c);
    } else if (m < 512) {
        if (stream) launch_stamped((k_resident<1, 32, 8, true, false, 4>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 32, 8, false, false, 4>), g, block, st, tm, a, x, c);
    } else if (m == 1024) {
        if (stream) launch_stamped((k_resident<1, 16, 8, true, true, 2>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 16, 8, false, true, 2>), g, block, st, tm, a, x, c);
    } else if (m < 1024) {
        if (stream) launch_stamped((k_resident<1, 16, 8, true, false, 2>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 16, 8, false, false, 2>), g, block, st, tm, a, x, c);
    } else if (m == 2048) {
        if (stream) launch_stamped((k_resident<1, 8, 8, true, true>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 8, 8, false, true>), g, block, st, tm, a, x, c);
    } else if (m == 4096) {
        if (stream) launch_stamped((k_resident<2, 4, 8, true, true>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<2, 4, 8, false, true>), g, block, st, tm, a, x, c);
    } else if (m == 6144) {
        if (stream) launch_stamped((k_resident<3, 2, 8, true, true>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<3, 2, 8, false, true>), g, block, st, tm, a, x, c);
    } else if (m == 8192) {
        if (stream) launch_stamped((k_resident<4, 2, 8, true, true>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<4, 2, 8, false, true>), g, block, st, tm, a, x, c);
    } else if (m < 2048) {
        if (stream) launch_stamped((k_resident<1, 8, 8, true, false>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<1, 8, 8, false, false>), g, block, st, tm, a, x, c);
    } else if (m < 4096) {
        if (stream) launch_stamped((k_resident<2, 4, 8, true, false>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<2, 4, 8, false, false>), g, block, st, tm, a, x, c);
    } else if (m < 6144) {
        if (stream) launch_stamped((k_resident<3, 2, 8, true, false>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<3, 2, 8, false, false>), g, block, st, tm, a, x, c);
    } else {
        if (stream) launch_stamped((k_resident<4, 2, 8, true, false>), g, block, st, tm, a, x, c);
        else launch_stamped((k_resident<4, 2, 8, false, false>), g, block, st, tm, a, x, c);
    }
    return hipGetLastError();
}

}  // namespace fs
