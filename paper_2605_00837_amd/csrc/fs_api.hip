// C ABI of the library (declared in include/fastsinkhorn.h) and the host-side
// driver of Alg. 1: validation, workspace layout, the iteration loop enqueued
// either as plain stream launches or as replayed hipGraph blocks, and the
// host-visible stop flag that lets the blocking entry points stop enqueuing
// without ever waiting on the device inside the loop.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <utility>
#include <vector>

#include "../../include/fastsinkhorn.h"
#include "fs_kernels.h"

namespace {

using namespace fs;

static_assert(kSmallMax == FS_SMALL_MAX && kCoopMax == FS_COOP_MAX, "the header states the kernels' limits");

thread_local char g_err[512] = "";

void set_err(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

#define FS_HIP(call)                                                                     \
    do {                                                                                 \
        hipError_t e__ = (call);                                                         \
        if (e__ != hipSuccess) {                                                         \
            set_err("%s failed: %s (%s:%d)", #call, hipGetErrorString(e__), __FILE__, __LINE__); \
            return FS_ERR_HIP;                                                           \
        }                                                                                \
    } while (0)

constexpr double kLog2e = 1.4426950408889634074;

inline size_t up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- workspace layout
struct Layout {
    int n, m, d, n_ld, m_ld;
    // dense
    int P_stream, rpp_stream, P_fused;
    int P_part;            // sets of m_ld doubles that o_part holds
    int row_splits, row_cps;     // column ranges of the streaming row pass (1: none)
    // points
    int JSf, cpsf, JSg, cpsg;
    size_t o_state, o_F, o_U, o_G, o_V, o_la2, o_lb2, o_part, o_part2;
    size_t o_rowpart;      // [row_splits][n_ld] partial row LSE values (dense, row_splits > 1)
    size_t o_Xp, o_Xs, o_cx, o_Yp, o_Ys, o_cy;
    size_t o_coop;         // scratch of the one-launch solver for mid-size dense problems (0: none)
    size_t o_grid;         // scratch of the one-launch solver over the whole chip (0: none)
    size_t o_persist;      // counters and error terms of the persistent fused pass (0: none)
    size_t o_start;        // [2][n_ld | m_ld] floats: starting potentials of an in-place warm start, kept for a second attempt
    size_t total;
};

Layout make_layout(int n, int m, int d) {
    Layout L{};
    L.n = n; L.m = m; L.d = d;
    L.n_ld = (int)up((size_t)n, 32);
    L.m_ld = (int)up((size_t)m, 32);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += up(bytes, 256); return o; };
    L.o_state = take(sizeof(State));
    L.o_F = take(sizeof(double) * 2 * L.n_ld);
    L.o_U = take(sizeof(double) * 2 * L.n_ld);
    L.o_G = take(sizeof(double) * 2 * L.m_ld);
    L.o_V = take(sizeof(double) * 2 * L.m_ld);
    L.o_la2 = take(sizeof(double) * L.n_ld);
    L.o_lb2 = take(sizeof(double) * L.m_ld);
    if (d == 0) {
        dense_stream_plan(n, m, &L.P_stream, &L.rpp_stream);
        dense_fused_plan(n, m, &L.P_fused);
        int Pmax = L.P_stream > L.P_fused ? L.P_stream : L.P_fused;
        // a width that only the resident form of the persistent pass takes: its exchange buffer holds 256 sets, and
        // 256 x 256 strips of 4 floats (it is laid out by strip, not by column: below 512 columns that is the larger)
        if (m <= 1024 && dense_persist_supported(n, m, nullptr, 0)) {
            const int sets = (int)std::max<size_t>(256, (size_t(256) * 256 * 16 + size_t(L.m_ld) * 8 - 1) / (size_t(L.m_ld) * 8));
            if (Pmax < sets) Pmax = sets;
        }
        L.P_part = Pmax;
        L.o_part = take(sizeof(double) * (size_t)Pmax * L.m_ld);
        L.o_part2 = L.o_part;
        dense_row_split_plan(n, m, &L.row_splits, &L.row_cps);
        if (L.row_splits > 1) L.o_rowpart = take(sizeof(double) * (size_t)L.row_splits * L.n_ld);
        if (coop_supported(n, m)) L.o_coop = take(coop_scratch_bytes());
        if (grid_supported(n, m, kGridWMax, false)) L.o_grid = take(grid_scratch_bytes());
        if (dense_persist_supported(n, m, nullptr, 0)) L.o_persist = take(persist_scratch_bytes());
    } else {
        points_plan(n, m, d, &L.JSf, &L.cpsf);
        points_plan(m, n, d, &L.JSg, &L.cpsg);
        L.o_part = take(sizeof(double) * (size_t)L.JSf * L.n_ld);
        L.o_part2 = take(sizeof(double) * (size_t)L.JSg * L.m_ld);
        L.o_Xp = take(sizeof(double) * (size_t)n * d);
        L.o_Xs = take(sizeof(double) * (size_t)n * d);
        L.o_cx = take(sizeof(double) * L.n_ld);
        L.o_Yp = take(sizeof(double) * (size_t)m * d);
        L.o_Ys = take(sizeof(double) * (size_t)m * d);
        if (coop_points_supported(n, m)) L.o_coop = take(coop_scratch_bytes());
        if (grid_supported(n, m, kGridWMax, true)) L.o_grid = take(grid_scratch_bytes());
        L.o_cy = take(sizeof(double) * L.m_ld);
    }
    L.o_start = take(sizeof(float) * ((size_t)L.n_ld + L.m_ld));
    L.total = off;
    return L;
}

// ---------------------------------------------------------------- per-device cache
// The host reads the hint of a block up to 3 blocks behind what it has enqueued; with blocks of at most
// kMaxBlock iterations the slot it reads has not been reused yet (3 * 64 < 256).
constexpr int kMaxBlock = 64;
static_assert(3 * kMaxBlock < kHintRing, "a hint must outlive the run-ahead of the host");

struct HostBlock {            // pinned, device-visible
    volatile int32_t flag;    // done
    volatile int32_t hint;    // latest pace hint (1 = potentials move slowly)
    volatile int32_t hints[kHintRing];   // pace hint after iteration k, at index k % kHintRing
    int32_t pad[2];
    fs_result res;
};

struct DeviceCache {
    void *ws = nullptr;
    size_t ws_bytes = 0;
    HostBlock *host = nullptr;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    std::vector<hipEvent_t> timing;     // start/stop pairs for sampled kernel timing
    hipStream_t cap_stream = nullptr;   // library-owned stream on which iteration blocks are captured
    unsigned int *tickets = nullptr;    // 64 arrival counters of the after-the-loop kernels; each returns to 0 after use
};

// Result of the sampled kernel timing of the last timed solve on this thread.  The solve only notes which event
// pairs count; the durations are read from the events when fs_last_kernel_timing() asks for them, so that this
// bookkeeping is not part of the solve's own run time.
struct KernelTiming {
    float avg_ms = 0.0f;
    int samples = 0;
    const char *name = "";
    int iters_sampled = 0;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pending;   // not yet read; the events live in the device cache
};
thread_local KernelTiming g_timing;

std::mutex g_mu;
std::map<int, DeviceCache> g_cache;

fs_status get_cache(size_t need_bytes, DeviceCache **out) {
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceCache &c = g_cache[dev];
    if (!c.host) {
        FS_HIP(hipHostMalloc((void **)&c.host, sizeof(HostBlock), hipHostMallocDefault));
        memset((void *)c.host, 0, sizeof(HostBlock));
        for (auto &e : c.ev) FS_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        FS_HIP(hipStreamCreateWithFlags(&c.cap_stream, hipStreamNonBlocking));
        FS_HIP(hipMalloc((void **)&c.tickets, 64 * sizeof(unsigned int)));
        FS_HIP(hipMemset(c.tickets, 0, 64 * sizeof(unsigned int)));
    }
    if (c.ws_bytes < need_bytes) {
        if (c.ws) {
            FS_HIP(hipDeviceSynchronize());
            FS_HIP(hipFree(c.ws));
            c.ws = nullptr;
            c.ws_bytes = 0;
        }
        const size_t want = up(need_bytes, (size_t)1 << 20);
        FS_HIP(hipMalloc(&c.ws, want));
        c.ws_bytes = want;
    }
    *out = &c;
    return FS_OK;
}

// ---------------------------------------------------------------- static scratch
// Workspace of the entry point that allocates nothing.  In host code the array's name is only a handle for
// hipGetSymbolAddress: every device holds its own copy at its own address, looked up once per device (with
// that device current) and used through the pointer from then on.
static __device__ __align__(256) unsigned char scratch[FS_STATIC_SCRATCH_BYTES];

std::map<int, void *> g_scratch_ptr;        // by device, guarded by g_mu

fs_status static_scratch(void **out) {
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_scratch_ptr.find(dev);
    if (it == g_scratch_ptr.end()) {
        void *ptr = nullptr;
        FS_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) { set_err("static scratch has no usable device address"); return FS_ERR_HIP; }
        it = g_scratch_ptr.emplace(dev, ptr).first;
    }
    *out = it->second;
    return FS_OK;
}

// ---------------------------------------------------------------- one solve, described
struct Problem {
    const float *C, *X, *Y, *a, *b;
    int d, n, m;
    float eps;
    int max_iter;
    float tol;
};

struct Solve {
    Problem pr;
    fs_options opt;
    Layout L;
    char *ws;
    hipStream_t st;
    Pots pots;
    State *state;
    int mode;              // 1 streaming, 2 fused (dense); 3 points
    bool persist = false;  // dense, mode 2: blocks of iterations run as launches of the persistent fused pass
    int cus = 0;           // compute units of the device (persistent pass: one workgroup each)
    volatile int32_t *host_flag;   // device-visible address of the pinned flag, or null

    Ctl ctl(int phase) const {
        Ctl c;
        c.st = state;
        c.max_iter = pr.max_iter;
        c.check_every = opt.check_every;
        c.tol = pr.tol > 0.0f ? (double)pr.tol : 0.0;
        c.err_history = opt.err_history;
        c.err_history_len = opt.err_history ? opt.err_history_len : 0;
        c.phase = phase;
        c.host_flag = host_flag;
        c.force_fast = opt.fused_variant >= 100 ? 1 : 0;
        return c;
    }
    // kind of an iteration of the dense solver: the exact streaming kernels, or a fused kernel
    enum Kind { STREAM = 1, FUSED = 2 };
    bool fused_is_fp32_cols() const { return mode == 2 && dense_fused_predicts(pr.m, opt.fused_variant, opt.cost_dtype); }
    DenseArgs dense(Kind kind) const {
        DenseArgs a;
        a.C = pr.C;
        a.c_dtype = opt.cost_dtype;
        a.p = pots;
        a.colpart = (double *)(ws + L.o_part);
        if (kind == FUSED) { a.P = dense_fused_grid(pr.n, pr.m, opt.fused_variant, opt.cost_dtype); a.rows_per_panel = 0; }
        else { a.P = L.P_stream; a.rows_per_panel = L.rpp_stream; }
        a.rowpart = nullptr; a.row_splits = 1; a.row_cps = pr.m;
        if (kind == STREAM && L.row_splits > 1) {
            a.rowpart = (double *)(ws + L.o_rowpart); a.row_splits = L.row_splits; a.row_cps = L.row_cps;
        }
        return a;
    }
    ErrSrc err_src() const {
        ErrSrc e;
        e.F = pots.F; e.a = pots.a; e.n = pr.n; e.n_ld = L.n_ld;
        return e;
    }
    CombineArgs combine_g(int P, const double *part, const double *rowconst) const {
        CombineArgs a{};
        a.part = part; a.P = P; a.ld = L.m_ld; a.len = pr.m;
        a.rowconst = rowconst; a.lw2 = pots.lb2; a.w = pots.b;
        a.pot = pots.G; a.shift = pots.V;
        a.do_advance = 1;
        a.es = err_src();
        return a;
    }
    CombineArgs combine_f(int P, const double *part, const double *rowconst) const {
        CombineArgs a{};
        a.part = part; a.P = P; a.ld = L.n_ld; a.len = pr.n;
        a.rowconst = rowconst; a.lw2 = pots.la2; a.w = pots.a;
        a.pot = pots.F; a.shift = pots.U;
        a.do_advance = 0;
        a.es = err_src();
        return a;
    }
    PointsArgs points_f() const {
        PointsArgs a{};
        a.rows = (const double *)(ws + L.o_Xp);
        a.cols2s = (const double *)(ws + L.o_Ys);
        a.colconst = (const double *)(ws + L.o_cy);
        a.colshift = pots.V;
        a.nr = pr.n; a.nc = pr.m; a.d = pr.d;
        a.part = (double *)(ws + L.o_part);
        a.JS = L.JSf; a.ld = L.n_ld; a.cols_per_split = L.cpsf;
        a.rowpot = pots.F; a.rowconst = (const double *)(ws + L.o_cx);
        return a;
    }
    PointsArgs points_g() const {
        PointsArgs a{};
        a.rows = (const double *)(ws + L.o_Yp);
        a.cols2s = (const double *)(ws + L.o_Xs);
        a.colconst = (const double *)(ws + L.o_cx);
        a.colshift = pots.U;
        a.nr = pr.m; a.nc = pr.n; a.d = pr.d;
        a.part = (double *)(ws + L.o_part2);
        a.JS = L.JSg; a.ld = L.m_ld; a.cols_per_split = L.cpsg;
        a.rowpot = pots.G; a.rowconst = (const double *)(ws + L.o_cy);
        return a;
    }

    // sets of column sums the exchange buffer of the persistent pass holds (up to 1024 columns the pass has its own count)
    int persist_sets() const { return pr.m <= 1024 ? L.P_part : L.P_fused; }
    const char *dominant_kernel() const {
        if (persist) return dense_persist_resident(pr.n, pr.m, cus < persist_sets() ? cus : persist_sets(), opt.fused_variant % 100) ? "k_resident" : "k_persist";
        return mode == 1 ? "k_row_stream" : mode == 2 ? (fused_is_fp32_cols() ? "k_fused_pf" : "k_fused") : "k_points_lse";
    }
    // a block of up to nb iterations in one launch of the persistent fused pass
    hipError_t enqueue_persist_block(int nb, hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr) const {
        Stamp tm;
        tm.t0 = t0;
        tm.t1 = t1;
        DenseArgs a = dense(FUSED);
        a.P = persist_sets();
        const int cu = cus < a.P ? cus : a.P;
        return launch_persist(st, a, ctl(0), ws + L.o_persist, cu, nb, opt.wait_limit, opt.skip_final_err ? 0 : 1,
                              opt.fused_variant % 100, tm);
    }
    // Eq. 9.  t0/t1 (optional) are stamped by the runtime with the start and stop of the dominant kernel
    // of the iteration: the row pass, the fused pass, or the point-cloud LSE pass of the f-update.
    hipError_t enqueue_f_update(int phase, Kind kind, hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr) const {
        const Ctl c = ctl(phase);
        hipError_t e = hipSuccess;
        Stamp tm;
        tm.t0 = t0;
        tm.t1 = t1;
        if (mode == 3) e = launch_points_lse(st, points_f(), c, 0, L.m_ld, tm);
        else if (kind == STREAM) {
            e = launch_dense_row(st, dense(STREAM), c, tm);
            if (e == hipSuccess && L.row_splits > 1)       // the row pass left partial values per column range
                e = launch_combine(st, combine_f(L.row_splits, (const double *)(ws + L.o_rowpart), nullptr), c);
        }
        else e = launch_dense_fused(st, dense(FUSED), c, opt.fused_variant, tm);     // both half-steps
        if (mode == 3 && e == hipSuccess) {
            CombineArgs ca = combine_f(L.JSf, (const double *)(ws + L.o_part), (const double *)(ws + L.o_cx));
            if (points_optimistic(pr.d)) {      // the pass may have run optimistically: let the combine check it
                const PointsArgs pa = points_f();
                ca.pr_rows = pa.rows; ca.pr_cols2s = pa.cols2s; ca.pr_colconst = pa.colconst;
                ca.pr_colshift = pa.colshift; ca.pr_nc = pa.nc; ca.pr_d = pa.d; ca.pr_shift_next = 0; ca.pr_ld = L.m_ld;
            }
            e = launch_combine(st, ca, c);
        }
        return e;
    }
    hipError_t enqueue_g_update(Kind kind) const {       // Eq. 10 + state advance
        const Ctl c = ctl(0);
        hipError_t e = hipSuccess;
        if (mode != 3 && kind == STREAM) {
            e = launch_dense_col(st, dense(STREAM), c);
            if (e == hipSuccess) e = launch_combine(st, combine_g(L.P_stream, (const double *)(ws + L.o_part), nullptr), c);
        } else if (mode == 2) {
            {
            const int g = dense_fused_grid(pr.n, pr.m, opt.fused_variant, opt.cost_dtype);
            CombineArgs ca = combine_g(g, (const double *)(ws + L.o_part), nullptr);
            if (dense_fused_predicts(pr.m, opt.fused_variant, opt.cost_dtype)) {
                ca.repair_C = pr.C; ca.repair_U = pots.U; ca.repair_n = pr.n; ca.repair_ld = L.n_ld;
                ca.repair_dtype = opt.cost_dtype;
                ca.repair_s = pots.s;
            }
            e = launch_combine(st, ca, c);
        }
        } else {
            e = launch_points_lse(st, points_g(), c, 1, L.n_ld);
            if (e == hipSuccess) {
                CombineArgs ca = combine_g(L.JSg, (const double *)(ws + L.o_part2), (const double *)(ws + L.o_cy));
                if (points_optimistic(pr.d)) {
                    const PointsArgs pa = points_g();
                    ca.pr_rows = pa.rows; ca.pr_cols2s = pa.cols2s; ca.pr_colconst = pa.colconst;
                    ca.pr_colshift = pa.colshift; ca.pr_nc = pa.nc; ca.pr_d = pa.d; ca.pr_shift_next = 1; ca.pr_ld = L.n_ld;
                }
                e = launch_combine(st, ca, c);
            }
        }
        return e;
    }
    Kind default_kind() const { return mode == 2 ? FUSED : STREAM; }
    hipError_t enqueue_iteration(Kind kind, hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr) const {
        hipError_t e = enqueue_f_update(0, kind, t0, t1);
        if (e == hipSuccess) e = enqueue_g_update(kind);
        return e;
    }
    hipError_t enqueue_trailing() const {                // err after the last iteration
        hipError_t e = enqueue_f_update(1, default_kind());
        if (e == hipSuccess) e = launch_advance(st, err_src(), ctl(1));
        return e;
    }
    hipError_t enqueue_init() const {
        int warm = 0;
        if (opt.warm_start) warm = 3;
        hipError_t e = launch_init(st, pots, state, /*f_in*/ warm_f, warm_g, opt.f64_in && opt.g64_in ? opt.f64_in : nullptr,
                                   opt.f64_in && opt.g64_in ? opt.g64_in : nullptr, warm,
                                   persist ? ws + L.o_persist : nullptr);     // the pass's arrival counters start at 0
        if (e == hipSuccess && mode == 3) {
            e = launch_points_prep(st, pr.X, pr.n, pr.d, pots.s, (double *)(ws + L.o_Xp), (double *)(ws + L.o_Xs),
                                   (double *)(ws + L.o_cx));
            if (e == hipSuccess)
                e = launch_points_prep(st, pr.Y, pr.m, pr.d, pots.s, (double *)(ws + L.o_Yp), (double *)(ws + L.o_Ys),
                                       (double *)(ws + L.o_cy));
        }
        return e;
    }
    const float *warm_f = nullptr, *warm_g = nullptr;
};

fs_status validate(const Problem &p, const float *f, const float *g) {
    if (p.n < 1 || p.m < 1) { set_err("n and m must be >= 1 (got %d, %d)", p.n, p.m); return FS_ERR_INVALID_ARG; }
    if (!(p.eps > 0.0f) || !std::isfinite(p.eps)) { set_err("eps must be positive and finite"); return FS_ERR_INVALID_ARG; }
    if (p.max_iter < 0) { set_err("max_iter must be >= 0"); return FS_ERR_INVALID_ARG; }
    if (std::isnan(p.tol)) { set_err("tol must not be NaN"); return FS_ERR_INVALID_ARG; }
    if (!p.a || !p.b) { set_err("a and b must be non-null"); return FS_ERR_INVALID_ARG; }
    if (!f || !g) { set_err("f and g must be non-null"); return FS_ERR_INVALID_ARG; }
    const bool dense = p.C != nullptr;
    const bool points = p.X != nullptr || p.Y != nullptr;
    if (dense == points) { set_err("exactly one of C or (X, Y) must be given"); return FS_ERR_INVALID_ARG; }
    if (points) {
        if (!p.X || !p.Y) { set_err("X and Y must both be non-null"); return FS_ERR_INVALID_ARG; }
        if (p.d < 1 || p.d > FS_MAX_DIM) { set_err("d must be in [1, %d] (got %d)", FS_MAX_DIM, p.d); return FS_ERR_INVALID_ARG; }
    }
    if (p.n > FS_MAX_POINTS || p.m > FS_MAX_POINTS) {
        set_err("n and m are limited to %d", FS_MAX_POINTS); return FS_ERR_INVALID_ARG;
    }
    return FS_OK;
}

fs_status setup(Solve &S, const Problem &pr, const fs_options *opts, float *f, float *g, hipStream_t st,
                void *ws, size_t ws_bytes) {
    S.pr = pr;
    S.opt = fs_options{};
    if (opts) S.opt = *opts;
    if (S.opt.check_every <= 0) S.opt.check_every = 10;
    if (S.opt.err_history && S.opt.err_history_len < 0) { set_err("err_history_len < 0"); return FS_ERR_INVALID_ARG; }
    S.L = make_layout(pr.n, pr.m, pr.C ? 0 : pr.d);
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) { set_err("workspace must be non-null and 256-byte aligned"); return FS_ERR_WORKSPACE; }
    if (ws_bytes < S.L.total) { set_err("workspace too small: %zu < %zu bytes", ws_bytes, S.L.total); return FS_ERR_WORKSPACE; }
    S.ws = (char *)ws;
    S.st = st;
    S.state = (State *)(S.ws + S.L.o_state);
    Pots &p = S.pots;
    p.F = (double *)(S.ws + S.L.o_F); p.U = (double *)(S.ws + S.L.o_U);
    p.G = (double *)(S.ws + S.L.o_G); p.V = (double *)(S.ws + S.L.o_V);
    p.la2 = (const double *)(S.ws + S.L.o_la2); p.lb2 = (const double *)(S.ws + S.L.o_lb2);
    p.a = pr.a; p.b = pr.b;
    p.n = pr.n; p.m = pr.m; p.n_ld = S.L.n_ld; p.m_ld = S.L.m_ld;
    p.s = kLog2e / (double)pr.eps;
    S.host_flag = nullptr;
    S.warm_f = f; S.warm_g = g;
    if (S.opt.cost_dtype < 0 || S.opt.cost_dtype > 2) { set_err("cost_dtype must be FS_COST_F32, FS_COST_F16 or FS_COST_BF16"); return FS_ERR_INVALID_ARG; }
    if (S.opt.cost_dtype != 0) {
        if (!pr.C) { set_err("cost_dtype applies to a dense cost matrix only"); return FS_ERR_INVALID_ARG; }
        if (pr.m % 8 != 0 || (reinterpret_cast<uintptr_t>(pr.C) & 15u)) {
            set_err("2-byte costs need m %% 8 == 0 (got %d) and a 16-byte aligned C", pr.m);
            return FS_ERR_UNSUPPORTED;
        }
    }
    if (pr.C) {
        const bool fused_ok = dense_fused_supported(pr.n, pr.m, pr.C, S.opt.cost_dtype);
        if (S.opt.kernel_mode == 2 && !fused_ok) {
            if (S.opt.cost_dtype != 0) set_err("fused kernel for 2-byte costs does not support m = %d (needs 2048 < m <= 16384)", pr.m);
            else set_err("fused kernel does not support m = %d (needs m <= 16384, and m %% 4 == 0 when m <= 1024)", pr.m);
            return FS_ERR_UNSUPPORTED;
        }
        const int km = S.opt.kernel_mode;
        if (km == 6) {
            if (!dense_persist_supported(pr.n, pr.m, pr.C, S.opt.cost_dtype)) {
                set_err("kernel_mode 6 needs a dense fp32 cost matrix with 128 < m <= 16384 (got m = %d)", pr.m);
                return FS_ERR_UNSUPPORTED;
            }
        } else if (km < 0 || km > 2) { set_err("kernel_mode %d does not take this problem", km); return FS_ERR_UNSUPPORTED; }
        // (6: the kernels around the persistent pass -- err of a solve of 0 iterations, the second attempt after a wait
        // that was abandoned -- are those of the automatic choice)
        S.mode = km == 0 || km == 6 ? (fused_ok ? 2 : 1) : km;
        if (S.mode == 2 && dense_fused_grid(pr.n, pr.m, S.opt.fused_variant, S.opt.cost_dtype) == 0) S.opt.fused_variant = 0;
    } else {
        S.mode = 3;
    }
    return FS_OK;
}

// Blocks of iterations replayed as one hipGraph.  The kernels read the iteration
// index from device memory, so one captured block serves every replay; a replay
// that overshoots max_iter, or that runs after the stop flag is set, is a no-op.
struct GraphKey {
    const void *ws, *C, *X, *a, *f;
    int n, m, d, mode, block, max_iter, check_every;
    float eps, tol;
    bool operator<(const GraphKey &o) const {
        return std::tie(ws, C, X, a, f, n, m, d, mode, block, max_iter, check_every, eps, tol) <
               std::tie(o.ws, o.C, o.X, o.a, o.f, o.n, o.m, o.d, o.mode, o.block, o.max_iter, o.check_every, o.eps, o.tol);
    }
};

// A block of `nb` iterations captured once as a hipGraph and replayed.  The kernels take the
// iteration index from device memory, so the same executable graph serves every block of the solve;
// a replay that overshoots max_iter, or that runs after the stop flag is set, does nothing.  The block
// is captured on a library-owned stream (the caller's may be the legacy default stream, which cannot
// be captured) and launched on the caller's stream.  No memset node is ever recorded.
struct BlockGraph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    ~BlockGraph() {
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
    }
};

fs_status build_block_graph(const Solve &S, hipStream_t cap, Solve::Kind kind, int nb, BlockGraph *out) {
    Solve T = S;
    T.st = cap;
    FS_HIP(hipStreamBeginCapture(cap, hipStreamCaptureModeThreadLocal));
    hipError_t e = hipSuccess;
    for (int q = 0; q < nb && e == hipSuccess; ++q) e = T.enqueue_iteration(kind);
    hipGraph_t g = nullptr;
    const hipError_t e2 = hipStreamEndCapture(cap, &g);
    out->graph = g;
    if (e != hipSuccess) { set_err("kernel launch failed during graph capture: %s", hipGetErrorString(e)); return FS_ERR_HIP; }
    FS_HIP(e2);
    FS_HIP(hipGraphInstantiate(&out->exec, out->graph, nullptr, nullptr, 0));
    return FS_OK;
}

constexpr int kPersistBlock = 50;       // iterations per launch of the persistent fused pass
constexpr int kAsyncExactFirst = 4;     // asynchronous solves: exact streaming iterations before the fused kernel
constexpr int kFirstBlock = 2;          // blocking solves: iterations before the first look at the pace hint

fs_status run_solve_async(Solve &S, float *f, float *g, fs_result *result_dev) {
    FS_HIP(S.enqueue_init());
    if (S.persist) {
        // the persistent pass, a block of iterations per launch; the launch that reaches max_iter evaluates the
        // error of the last iterate itself.  A launch whose wait is abandoned marks the solve (nonfinite = 2) and
        // everything enqueued behind it returns at once.
        for (int it = 0; it < S.pr.max_iter; it += kPersistBlock)
            FS_HIP(S.enqueue_persist_block(S.pr.max_iter - it < kPersistBlock ? S.pr.max_iter - it : kPersistBlock));
        if (S.pr.max_iter == 0 && !S.opt.skip_final_err) FS_HIP(S.enqueue_trailing());
        FS_HIP(launch_finalize(S.st, S.pots, S.state, f, g, S.opt.f64_out, S.opt.g64_out, result_dev, nullptr));
        return FS_OK;
    }
    // Without a host in the loop the pace hint cannot be followed: the fp32-column fused kernel takes
    // over after a fixed number of exact streaming iterations (its repair keeps it correct anyway).
    const bool two_kinds = S.fused_is_fp32_cols();
    const int exact_first = S.opt.fused_variant >= 100 ? 0 : kAsyncExactFirst;
    for (int it = 0; it < S.pr.max_iter; ++it)
        FS_HIP(S.enqueue_iteration(two_kinds && it < exact_first ? Solve::STREAM : S.default_kind()));
    if (!S.opt.skip_final_err) FS_HIP(S.enqueue_trailing());
    FS_HIP(launch_finalize(S.st, S.pots, S.state, f, g, S.opt.f64_out, S.opt.g64_out, result_dev, nullptr));
    return FS_OK;
}

int run_solve_blocking(Solve &S, DeviceCache *dc, float *f, float *g, fs_result *result_host) {
    HostBlock *hb = dc->host;
    hb->flag = 0;
    hb->hint = 0;
    for (auto &h : hb->hints) h = 0;
    memset((void *)&hb->res, 0, sizeof(hb->res));
    std::vector<int> sample_iter, sample_len;      // last iteration and number of iterations of a timed launch
    void *hb_dev = nullptr;
    FS_HIP(hipHostGetDevicePointer(&hb_dev, (void *)hb, 0));
    S.host_flag = (volatile int32_t *)hb_dev;
    // The persistent pass waits for all of its workgroups; should it give up (the device kept some of them from
    // running) the solve is run again by the multi-kernel driver, from the same start: an in-place warm start is
    // kept aside for that.
    const bool own_persist = S.persist && S.opt.kernel_mode == 0;
    const bool in_place = S.opt.warm_start && !(S.opt.f64_in && S.opt.g64_in);
    float *keep = (float *)(S.ws + S.L.o_start);
    if (own_persist && in_place) {
        FS_HIP(hipMemcpyAsync(keep, f, sizeof(float) * S.pr.n, hipMemcpyDeviceToDevice, S.st));
        FS_HIP(hipMemcpyAsync(keep + S.L.n_ld, g, sizeof(float) * S.pr.m, hipMemcpyDeviceToDevice, S.st));
    }
    FS_HIP(S.enqueue_init());
    // Iterations are enqueued in blocks; the stop rule itself runs on the device every check_every iterations,
    // a block is only how often the host looks at the stop flag (what it enqueued beyond a stop returns at
    // once), so small check intervals do not shrink it.
    int block = S.opt.check_every > 10 ? S.opt.check_every : 10;
    if (block > kMaxBlock) block = kMaxBlock;
    if (S.persist) block = kPersistBlock;
    const int tevery = S.opt.time_kernel_every > 0 ? S.opt.time_kernel_every : 0;
    int nsamples = 0;
    g_timing = KernelTiming{};
    // Dense solves whose fused kernel sums its column phase in fp32 run the exact streaming kernels
    // while the device reports fast-moving potentials.  The hint used for block b is the one the
    // device published at the end of the block whose completion the host has just waited for, so the
    // sequence of kernels, and with it every bit of the result, does not depend on host timing.
    // (The persistent pass takes every iteration itself: its repairs make it exact at any pace.)
    const bool two_kinds = S.fused_is_fp32_cols() && !S.persist;
    const bool force_fused = S.opt.fused_variant >= 100;
    // Launch-bound sizes replay each block as one hipGraph (never while kernels are being timed).
    const size_t cells = (size_t)S.pr.n * (size_t)S.pr.m;
    const bool small = S.mode == 3 ? cells <= ((size_t)1 << 24) : cells <= ((size_t)1 << 22);
    const bool use_graph = !tevery && !S.persist && S.pr.max_iter >= block &&
                           (S.opt.use_graph == 2 || (S.opt.use_graph == 0 && small));
    BlockGraph graphs[3];                              // indexed by kind
    int block_end[4] = {0, 0, 0, 0};
    int it = 0, blk = 0;
    auto timing_pair = [&](int q) -> fs_status {
        while ((int)dc->timing.size() < 2 * (q + 1)) {
            hipEvent_t e;
            FS_HIP(hipEventCreate(&e));
            dc->timing.push_back(e);
        }
        return FS_OK;
    };
    while (it < S.pr.max_iter) {
        if (hb->flag) break;                           // the device has stopped: enqueue nothing more
        Solve::Kind kind = S.default_kind();
        int hint_block = -1;
        if (blk >= 3) hint_block = blk - 3;            // bound the run-ahead to 3 blocks
        else if (blk >= 1 && two_kinds && !force_fused) hint_block = 0;
        if (hint_block >= 0) FS_HIP(hipEventSynchronize(dc->ev[hint_block & 3]));
        if (hb->flag) break;
        if (two_kinds && !force_fused) {
            if (blk == 0) kind = Solve::STREAM;
            else kind = hb->hints[block_end[hint_block & 3] & (kHintRing - 1)] ? Solve::FUSED : Solve::STREAM;
        }
        int nb = (blk == 0 && two_kinds && !force_fused) ? kFirstBlock : block;
        if (nb > S.pr.max_iter - it) nb = S.pr.max_iter - it;
        if (S.persist) {
            // one launch per block; when timing is asked for, about a dozen launches spread over the solve are
            // stamped with their begin and end (a stamped dispatch costs about 10 us of queue time)
            const int nblocks = (S.pr.max_iter + block - 1) / block;
            const int stride = nblocks > 12 ? nblocks / 12 : 1;
            const bool sample = tevery && (blk % stride) == 0 && nsamples < 4096;
            if (sample) {
                const fs_status ts = timing_pair(nsamples);
                if (ts != FS_OK) return ts;
                FS_HIP(S.enqueue_persist_block(nb, dc->timing[2 * nsamples], dc->timing[2 * nsamples + 1]));
                sample_iter.push_back(it + nb - 1);
                sample_len.push_back(nb);
                ++nsamples;
            } else {
                FS_HIP(S.enqueue_persist_block(nb));
            }
        } else if (use_graph && nb == block) {
            BlockGraph &bg = graphs[(int)kind];
            if (!bg.exec) {
                const fs_status gs = build_block_graph(S, dc->cap_stream, kind, block, &bg);
                if (gs != FS_OK) return gs;
            }
            FS_HIP(hipGraphLaunch(bg.exec, S.st));
        } else
        for (int q = 0; q < nb; ++q) {
            const bool sample = tevery && ((it + q) % tevery == 0) && nsamples < 4096 &&
                                kind == S.default_kind();       // only the dominant kernel is timed
            if (sample) {
                const fs_status ts = timing_pair(nsamples);
                if (ts != FS_OK) return ts;
                FS_HIP(S.enqueue_iteration(kind, dc->timing[2 * nsamples], dc->timing[2 * nsamples + 1]));
                sample_iter.push_back(it + q);
                ++nsamples;
            } else {
                FS_HIP(S.enqueue_iteration(kind));
            }
        }
        FS_HIP(hipEventRecord(dc->ev[blk & 3], S.st));
        it += nb;
        block_end[blk & 3] = it;
        ++blk;
    }
    // (the persistent pass evaluates err of the last iterate itself, in the launch that reaches max_iter)
    if (!S.opt.skip_final_err && !hb->flag && !(S.persist && S.pr.max_iter > 0)) FS_HIP(S.enqueue_trailing());
    FS_HIP(launch_finalize(S.st, S.pots, S.state, f, g, S.opt.f64_out, S.opt.g64_out, nullptr,
                           (char *)hb_dev + offsetof(HostBlock, res)));
    FS_HIP(hipStreamSynchronize(S.st));
    if (S.persist && hb->res.nonfinite == kGaveUp) {
        if (!own_persist) {                            // asked for by the caller: report it
            if (result_host) *result_host = hb->res;
            return hb->res.iters;
        }
        if (in_place) {
            FS_HIP(hipMemcpyAsync(f, keep, sizeof(float) * S.pr.n, hipMemcpyDeviceToDevice, S.st));
            FS_HIP(hipMemcpyAsync(g, keep + S.L.n_ld, sizeof(float) * S.pr.m, hipMemcpyDeviceToDevice, S.st));
        }
        S.persist = false;
        return run_solve_blocking(S, dc, f, g, result_host);
    }
    if (nsamples > 0) {
        // only launches that did work count: those of iterations the solve actually performed
        int used = 0, covered = 0;
        for (int q = 0; q < nsamples; ++q) {
            if (sample_iter[q] >= hb->res.iters) break;
            g_timing.pending.emplace_back(dc->timing[2 * q], dc->timing[2 * q + 1]);
            ++used;
            covered += S.persist ? sample_len[q] : 1;
        }
        g_timing.samples = used;
        g_timing.name = S.dominant_kernel();
        g_timing.iters_sampled = covered;
    }
    if (result_host) *result_host = hb->res;
    return hb->res.iters;
}

// Option values that make no sense for the problem at hand, whichever kernel would run it.
fs_status check_options(const Problem &pr, const fs_options *opts) {
    if (!opts) return FS_OK;
    if (opts->cost_dtype < 0 || opts->cost_dtype > 2) { set_err("cost_dtype must be FS_COST_F32, FS_COST_F16 or FS_COST_BF16"); return FS_ERR_INVALID_ARG; }
    if (opts->cost_dtype != 0 && !pr.C) { set_err("cost_dtype applies to a dense cost matrix only"); return FS_ERR_INVALID_ARG; }
    if (opts->cost_dtype != 0 && (pr.m % 8 != 0 || (reinterpret_cast<uintptr_t>(pr.C) & 15u))) {
        set_err("2-byte costs need m %% 8 == 0 (got %d) and a 16-byte aligned C", pr.m);
        return FS_ERR_UNSUPPORTED;
    }
    if (opts->kernel_mode < 0 || opts->kernel_mode > 6) { set_err("kernel_mode must be 0 ... 6"); return FS_ERR_INVALID_ARG; }
    return FS_OK;
}

// Small dense problems run whole inside one single-workgroup kernel (fs_small.hip).
bool small_path(const Problem &pr, const fs_options *opts, fs_status *err) {
    const int km = opts ? opts->kernel_mode : 0;
    const bool fits = pr.C && pr.n <= kSmallMax && pr.m <= kSmallMax;
    if (km == 3 && !fits) {
        set_err("kernel_mode 3 needs a dense problem with n, m <= %d", kSmallMax);
        *err = FS_ERR_UNSUPPORTED;
        return false;
    }
    if (!fits || (opts && opts->time_kernel_every > 0)) return false;
    if (km == 3) return true;
    // automatic: up to 16 entries per lane (e.g. 128 x 128, 256 x 64) one workgroup beats the multi-kernel
    // path (2.5 - 5 us against 10 us per iteration); beyond that a single compute unit is the limit
    auto slots = [](int x) { const int q = (x + 31) / 32; return q <= 2 ? 2 : q <= 4 ? 4 : 8; };
    return km == 0 && slots(pr.n) * slots(pr.m) <= 16;
}

// Mid-size problems can run whole inside one multi-workgroup kernel (fs_coop.hip): dense fp32 cost, or point
// clouds (the squared distances are then formed once, in fp64, and kept in registers like a cost matrix).
bool coop_path(const Problem &pr, const fs_options *opts, fs_status *err) {
    const int km = opts ? opts->kernel_mode : 0;
    const bool fits = pr.C ? coop_supported(pr.n, pr.m) : coop_points_supported(pr.n, pr.m);
    if (km == 4 && !fits) {
        set_err("kernel_mode 4 needs n, m <= %d and a dense cost matrix, or point clouds of at most 16 pairs per lane (n * m <= 2^19, less for ragged shapes)", kCoopMax);
        *err = FS_ERR_UNSUPPORTED;
        return false;
    }
    if (!fits || (opts && opts->time_kernel_every > 0)) return false;
    if (km == 4) return true;
    // automatic: up to 2^18 entries (512 x 512, 1024 x 256) one launch beats the chain of dependent launches of
    // the multi-kernel driver (5.6 against 11.3 us per iteration at 256 x 256, 8.4 against 12.7 at 512 x 512);
    // beyond that too few compute units are at work
    return km == 0 && (size_t)pr.n * (size_t)pr.m <= ((size_t)1 << 18);
}

// Compute units of the current device: the whole-chip one-launch solver needs one per workgroup.
thread_local int g_cus_override = 0;       // fs_kernel_choice: answer for a device with this many compute units

int device_cus() {
    if (g_cus_override > 0) return g_cus_override;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return cus;
}

// Dense problems up to 4096 x 4096 can run whole inside one kernel spread over the chip (fs_grid.hip).
bool grid_path(const Problem &pr, const fs_options *opts, bool blocking, fs_status *err, int *wmax) {
    const int km = opts ? opts->kernel_mode : 0;
    if (km != 5 && km != 0) return false;
    if (pr.n > kGridMaxN || pr.m > kGridMaxM) {
        if (km == 0) return false;
        set_err("kernel_mode 5 needs n <= %d, m <= %d", kGridMaxN, kGridMaxM);
        *err = FS_ERR_UNSUPPORTED;
        return false;
    }
    *wmax = device_cus();
    if (!grid_supported(pr.n, pr.m, *wmax, pr.C == nullptr)) {
        if (km == 0) return false;
        set_err("kernel_mode 5 takes at most 16 entries per lane (8 for point clouds: n / compute units, rounded up to a power of 2, times m / 1024) and at most 16 columns per workgroup");
        *err = FS_ERR_UNSUPPORTED;
        return false;
    }
    if (opts && opts->time_kernel_every > 0) return false;
    if (km == 5) return true;
    // automatic: it needs every compute unit of the chip at the same moment, so the library only picks it where
    // it can fall back (blocking solves); up to 512 x 512 the 32-workgroup kernel is as fast or faster
    // (256 x 256: 5.7 against 7.3 us per iteration), beyond that this one is (1024 x 256: 8.3 against 10.2) --
    // except where the persistent pass can keep its share of C on the chip (more than 128 columns) and the problem
    // is not small: that one runs an iteration in 9.4 us plus 1.5 us per 16 MiB of C (2048 x 2048: 10.5 against
    // 14.0 us per iteration, 1024 x 2048: 9.6 / 12.0, 256 x 2048: 9.4 / 10.9, 800 x 1200: 9.6 / 10.4; but 640 x 1280:
    // 9.7 / 9.3, 300 x 1100: 9.6 / 8.1; with the wait as it is now 1024 x 1024: 8.9 / 9.4, 2048 x 512: 8.7 / 9.9, but
    // 320 x 1024: 8.7 / 7.6, 700 x 520: 8.9 / 7.7)
    if (blocking && pr.C && (!opts || (opts->fused_variant == 0 && opts->cost_dtype == 0)) &&
        (pr.m >= 2048 || (size_t)pr.n * (size_t)pr.m >= 900000) &&
        dense_persist_supported(pr.n, pr.m, pr.C, 0) && dense_persist_grid(pr.n, pr.m, *wmax) >= 1 &&
        dense_persist_resident(pr.n, pr.m, *wmax, 0))
        return false;
    return blocking && (pr.n > 512 || pr.m > 512);
}

// Dense fp32 problems of the widths of the LDS-prefetch fused pass run their iterations in launches of the
// persistent form of that pass (fs_persist.hip): one workgroup per compute unit stays resident for a block of
// iterations.  The library's own choice in the blocking solves only (a solve that gives up is run again by the
// multi-kernel driver); the asynchronous entry points take it on request (kernel_mode 6) and report a wait that
// was abandoned as nonfinite = 2.
bool persist_path(const Problem &pr, const fs_options *opts, bool blocking, int *cus) {
    const int km = opts ? opts->kernel_mode : 0;
    if (!pr.C || (km != 0 && km != 6) || (!blocking && km != 6)) return false;
    if (!dense_persist_supported(pr.n, pr.m, pr.C, opts ? opts->cost_dtype : 0)) return false;
    *cus = device_cus();
    if (*cus < 1) return false;
    if (dense_persist_grid(pr.n, pr.m, *cus) < 1) return false;      // too few workgroups for this width
    if (km == 6) return true;
    if (opts && opts->fused_variant != 0) return false;      // a tuning / test knob of the multi-kernel path
    // automatic: where it is faster than the multi-kernel driver (5 - 19 % per iteration from 300 x 3000 to
    // 16384 x 8192, 65536 x 2048; 7 - 12 % at 4096 columns from 2048 to 16384 rows, with panels of 4 rows).
    // Beyond 8192 columns the two are level (one row per panel, the pass is long against the exchange).
    if (pr.m > 8192) return false;
    return true;
}

fs_status small_args(const Problem &pr, int batch, const fs_options *opts, float *f, float *g, SmallArgs *out) {
    fs_options o{};
    if (opts) o = *opts;
    if (o.check_every <= 0) o.check_every = 10;
    if (o.err_history && o.err_history_len < 0) { set_err("err_history_len < 0"); return FS_ERR_INVALID_ARG; }
    SmallArgs A{};
    A.C = pr.C; A.a = pr.a; A.b = pr.b;
    A.c_dtype = o.cost_dtype;
    A.n = pr.n; A.m = pr.m; A.batch = batch;
    A.s = kLog2e / (double)pr.eps;
    A.max_iter = pr.max_iter; A.check_every = o.check_every;
    A.tol = pr.tol > 0.0f ? (double)pr.tol : 0.0;
    A.warm = o.warm_start ? 1 : 0;
    A.f_in = f; A.g_in = g;
    A.f64_in = (o.f64_in && o.g64_in) ? o.f64_in : nullptr;
    A.g64_in = (o.f64_in && o.g64_in) ? o.g64_in : nullptr;
    A.f = f; A.g = g;
    A.f64_out = o.f64_out; A.g64_out = o.g64_out;
    A.err_history = o.err_history; A.err_history_len = o.err_history ? o.err_history_len : 0;
    A.want_final_err = o.skip_final_err ? 0 : 1;
    *out = A;
    return FS_OK;
}

int solve_blocking(const Problem &pr, float *f, float *g, hipStream_t st, const fs_options *opts,
                   fs_result *result_host) {
    fs_status v = validate(pr, f, g);
    if (v == FS_OK) v = check_options(pr, opts);
    if (v != FS_OK) return v;
    fs_status serr = FS_OK;
    if (small_path(pr, opts, &serr)) {
        DeviceCache *dc = nullptr;
        v = get_cache(256, &dc);
        if (v != FS_OK) return v;
        HostBlock *hb = dc->host;
        memset((void *)&hb->res, 0, sizeof(hb->res));
        void *hb_dev = nullptr;
        FS_HIP(hipHostGetDevicePointer(&hb_dev, (void *)hb, 0));
        SmallArgs A;
        v = small_args(pr, 1, opts, f, g, &A);
        if (v != FS_OK) return v;
        A.result = (ResultRecord *)((char *)hb_dev + offsetof(HostBlock, res));
        FS_HIP(launch_small(st, A));
        FS_HIP(hipStreamSynchronize(st));
        if (result_host) *result_host = hb->res;
        return hb->res.iters;
    }
    if (serr != FS_OK) return serr;
    Layout L = make_layout(pr.n, pr.m, pr.C ? 0 : pr.d);
    DeviceCache *dc = nullptr;
    v = get_cache(L.total, &dc);
    if (v != FS_OK) return v;
    // The one-launch solvers for mid-size problems.  Their workgroups wait for one another; should the device
    // keep part of a grid from running for seconds (other work holding its compute units) the solve gives up
    // and says so.  When the kernel was the library's own choice the problem is then simply solved again by
    // the multi-kernel driver; the starting potentials of an in-place warm start are kept for that.
    int wmax = 0;
    const bool grid = grid_path(pr, opts, /*blocking=*/true, &serr, &wmax);
    if (serr != FS_OK) return serr;
    const bool coop = !grid && coop_path(pr, opts, &serr);
    if (serr != FS_OK) return serr;
    if (coop || grid) {
        const bool own_choice = !opts || opts->kernel_mode == 0;
        const bool in_place = opts && opts->warm_start && !(opts->f64_in && opts->g64_in);
        float *keep = (float *)((char *)dc->ws + L.o_start);
        if (own_choice && in_place) {
            FS_HIP(hipMemcpyAsync(keep, f, sizeof(float) * pr.n, hipMemcpyDeviceToDevice, st));
            FS_HIP(hipMemcpyAsync(keep + L.n_ld, g, sizeof(float) * pr.m, hipMemcpyDeviceToDevice, st));
        }
        HostBlock *hb = dc->host;
        memset((void *)&hb->res, 0, sizeof(hb->res));
        void *hb_dev = nullptr;
        FS_HIP(hipHostGetDevicePointer(&hb_dev, (void *)hb, 0));
        ResultRecord *res_dev = (ResultRecord *)((char *)hb_dev + offsetof(HostBlock, res));
        if (coop) {
            CoopArgs A{};
            v = small_args(pr, 1, opts, f, g, &A);
            if (v != FS_OK) return v;
            A.result = res_dev;
            A.spin_limit = opts ? opts->wait_limit : 0;
            A.X = pr.X; A.Y = pr.Y; A.d = pr.C ? 0 : pr.d;
            FS_HIP(launch_coop(st, A, (char *)dc->ws + L.o_coop, opts ? opts->fused_variant : 0));
        } else {
            GridArgs A{};
            v = small_args(pr, 1, opts, f, g, &A);
            if (v != FS_OK) return v;
            A.result = res_dev;
            A.spin_limit = opts ? opts->wait_limit : 0;
            A.X = pr.X; A.Y = pr.Y; A.d = pr.C ? 0 : pr.d;
            FS_HIP(launch_grid(st, A, (char *)dc->ws + L.o_grid, wmax));
        }
        FS_HIP(hipStreamSynchronize(st));
        if (!(own_choice && hb->res.nonfinite == kGaveUp)) {
            if (result_host) *result_host = hb->res;
            return hb->res.iters;
        }
        if (in_place) {
            FS_HIP(hipMemcpyAsync(f, keep, sizeof(float) * pr.n, hipMemcpyDeviceToDevice, st));
            FS_HIP(hipMemcpyAsync(g, keep + L.n_ld, sizeof(float) * pr.m, hipMemcpyDeviceToDevice, st));
        }
    }
    if (serr != FS_OK) return serr;
    Solve S;
    v = setup(S, pr, opts, f, g, st, dc->ws, dc->ws_bytes);
    if (v != FS_OK) return v;
    S.persist = persist_path(pr, opts, /*blocking=*/true, &S.cus);
    if (!S.persist && opts && opts->kernel_mode == 6) {
        set_err("kernel_mode 6 needs at least m / 64 row panels and compute units (and up to 1024 columns at most 512 rows per compute unit) (n = %d, m = %d, %d compute units)", pr.n, pr.m, S.cus);
        return FS_ERR_UNSUPPORTED;
    }
    return run_solve_blocking(S, dc, f, g, result_host);
}

fs_status solve_async(const Problem &pr, float *f, float *g, hipStream_t st, const fs_options *opts,
                      void *ws, size_t ws_bytes, fs_result *result_dev) {
    fs_status v = validate(pr, f, g);
    if (v == FS_OK) v = check_options(pr, opts);
    if (v != FS_OK) return v;
    fs_status serr = FS_OK;
    if (small_path(pr, opts, &serr)) {
        // the workspace contract is the same whichever kernel ends up running
        if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) { set_err("workspace must be non-null and 256-byte aligned"); return FS_ERR_WORKSPACE; }
        const size_t need = make_layout(pr.n, pr.m, 0).total;
        if (ws_bytes < need) { set_err("workspace too small: %zu < %zu bytes", ws_bytes, need); return FS_ERR_WORKSPACE; }
        SmallArgs A;
        v = small_args(pr, 1, opts, f, g, &A);
        if (v != FS_OK) return v;
        A.result = (ResultRecord *)result_dev;
        FS_HIP(launch_small(st, A));
        return FS_OK;
    }
    if (serr != FS_OK) return serr;
    if (coop_path(pr, opts, &serr)) {
        const Layout L = make_layout(pr.n, pr.m, pr.C ? 0 : pr.d);
        if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) { set_err("workspace must be non-null and 256-byte aligned"); return FS_ERR_WORKSPACE; }
        if (ws_bytes < L.total) { set_err("workspace too small: %zu < %zu bytes", ws_bytes, L.total); return FS_ERR_WORKSPACE; }
        CoopArgs A{};
        v = small_args(pr, 1, opts, f, g, &A);
        if (v != FS_OK) return v;
        A.result = (ResultRecord *)result_dev;
        A.spin_limit = opts ? opts->wait_limit : 0;
        A.X = pr.X; A.Y = pr.Y; A.d = pr.C ? 0 : pr.d;
        FS_HIP(launch_coop(st, A, (char *)ws + L.o_coop, opts ? opts->fused_variant : 0));
        return FS_OK;
    }
    if (serr != FS_OK) return serr;
    int wmax = 0;
    if (grid_path(pr, opts, /*blocking=*/false, &serr, &wmax)) {
        const Layout L = make_layout(pr.n, pr.m, pr.C ? 0 : pr.d);
        if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) { set_err("workspace must be non-null and 256-byte aligned"); return FS_ERR_WORKSPACE; }
        if (ws_bytes < L.total) { set_err("workspace too small: %zu < %zu bytes", ws_bytes, L.total); return FS_ERR_WORKSPACE; }
        GridArgs A{};
        v = small_args(pr, 1, opts, f, g, &A);
        if (v != FS_OK) return v;
        A.result = (ResultRecord *)result_dev;
        A.spin_limit = opts ? opts->wait_limit : 0;
        A.X = pr.X; A.Y = pr.Y; A.d = pr.C ? 0 : pr.d;
        FS_HIP(launch_grid(st, A, (char *)ws + L.o_grid, wmax));
        return FS_OK;
    }
    if (serr != FS_OK) return serr;
    Solve S;
    v = setup(S, pr, opts, f, g, st, ws, ws_bytes);
    if (v != FS_OK) return v;
    S.persist = persist_path(pr, opts, /*blocking=*/false, &S.cus);      // on request only
    if (!S.persist && opts && opts->kernel_mode == 6) {
        set_err("kernel_mode 6 needs at least m / 64 row panels and compute units (and up to 1024 columns at most 512 rows per compute unit) (n = %d, m = %d, %d compute units)", pr.n, pr.m, S.cus);
        return FS_ERR_UNSUPPORTED;
    }
    return run_solve_async(S, f, g, result_dev);
}

fs_status plan_or_cost(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                       int n, int m, float eps, const float *f, const float *g, const double *f64,
                       const double *g64, float *P, double *cost_dev, hipStream_t st) {
    Problem pr{C, X, Y, a, b, d, n, m, eps, 0, 0.0f};
    const float *fchk = f ? f : (const float *)f64, *gchk = g ? g : (const float *)g64;
    fs_status v = validate(pr, (float *)fchk, (float *)gchk);
    if (v != FS_OK) return v;
    if (!P && !cost_dev) { set_err("output pointer is null"); return FS_ERR_INVALID_ARG; }
    const int dd = C ? 0 : d;
    const int need = plan_scratch_len(n, m, dd);
    const size_t bytes = P ? sizeof(double) * (size_t)need : diag_scratch_bytes(n, m, dd);
    DeviceCache *dc = nullptr;
    v = get_cache(bytes, &dc);
    if (v != FS_OK) return v;
    PlanArgs A{};
    A.C = C; A.X = X; A.Y = Y; A.a = a; A.b = b; A.f = f; A.g = g; A.f64 = f64; A.g64 = g64;
    A.n = n; A.m = m; A.d = dd;
    A.s = kLog2e / (double)eps;
    if (P) FS_HIP(launch_plan(st, A, P, (double *)dc->ws, need));
    else FS_HIP(launch_diag(st, A, nullptr, nullptr, nullptr, dc->ws, dc->ws_bytes, dc->tickets, cost_dev));   // one pass
    return FS_OK;
}

fs_status diagnostics(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const float *f, const float *g, const double *f64,
                      const double *g64, double *out8, double *row_marg, double *col_marg, hipStream_t st) {
    Problem pr{C, X, Y, a, b, d, n, m, eps, 0, 0.0f};
    if ((f == nullptr) != (g == nullptr) || (f64 == nullptr) != (g64 == nullptr) || (!f && !f64)) {
        set_err("potentials: give f and g, or f64 and g64"); return FS_ERR_INVALID_ARG;
    }
    const float *fchk = f ? f : (const float *)f64, *gchk = g ? g : (const float *)g64;
    fs_status v = validate(pr, (float *)fchk, (float *)gchk);
    if (v != FS_OK) return v;
    if (!out8) { set_err("out must be non-null"); return FS_ERR_INVALID_ARG; }
    const int dd = C ? 0 : d;
    DeviceCache *dc = nullptr;
    v = get_cache(diag_scratch_bytes(n, m, dd), &dc);
    if (v != FS_OK) return v;
    PlanArgs A{};
    A.C = C; A.X = X; A.Y = Y; A.a = a; A.b = b; A.f = f64 ? nullptr : f; A.g = g64 ? nullptr : g; A.f64 = f64; A.g64 = g64;
    A.n = n; A.m = m; A.d = dd;
    A.s = kLog2e / (double)eps;
    FS_HIP(launch_diag(st, A, out8, row_marg, col_marg, dc->ws, dc->ws_bytes, dc->tickets));
    return FS_OK;
}

fs_status barycentric(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const float *f, const float *g, const double *f64,
                      const double *g64, const float *Z, int dz, float *T, hipStream_t st) {
    Problem pr{C, X, Y, a, b, d, n, m, eps, 0, 0.0f};
    if ((f == nullptr) != (g == nullptr) || (f64 == nullptr) != (g64 == nullptr) || (!f && !f64)) {
        set_err("potentials: give f and g, or f64 and g64"); return FS_ERR_INVALID_ARG;
    }
    const float *fchk = f ? f : (const float *)f64, *gchk = g ? g : (const float *)g64;
    fs_status v = validate(pr, (float *)fchk, (float *)gchk);
    if (v != FS_OK) return v;
    if (!Z || !T) { set_err("Z and T must be non-null"); return FS_ERR_INVALID_ARG; }
    if (dz < 1 || dz > FS_MAX_BARY_DIM) { set_err("dz must be in [1, %d] (got %d)", FS_MAX_BARY_DIM, dz); return FS_ERR_INVALID_ARG; }
    const int dd = C ? 0 : d;
    DeviceCache *dc = nullptr;
    v = get_cache(bary_scratch_bytes(n, m, dd), &dc);
    if (v != FS_OK) return v;
    PlanArgs A{};
    A.C = C; A.X = X; A.Y = Y; A.a = a; A.b = b; A.f = f64 ? nullptr : f; A.g = g64 ? nullptr : g; A.f64 = f64; A.g64 = g64;
    A.n = n; A.m = m; A.d = dd;
    A.s = kLog2e / (double)eps;
    FS_HIP(launch_bary(st, A, Z, dz, T, dc->ws, dc->ws_bytes));
    return FS_OK;
}

fs_status half_step(bool update_f, const float *C, const float *X, const float *Y, int d, const float *a,
                    const float *b, int n, int m, float eps, const double *in64, double *out64, hipStream_t st) {
    Problem pr{C, X, Y, a, b, d, n, m, eps, 1, 0.0f};
    fs_status v = validate(pr, (float *)in64, (float *)out64);
    if (v != FS_OK) return v;
    Layout L = make_layout(n, m, C ? 0 : d);
    DeviceCache *dc = nullptr;
    v = get_cache(L.total, &dc);
    if (v != FS_OK) return v;
    Solve S;
    fs_options o{};
    o.kernel_mode = C ? 1 : 0;
    v = setup(S, pr, &o, nullptr, nullptr, st, dc->ws, dc->ws_bytes);
    if (v != FS_OK) return v;
    // start state: the given side from in64, the other side zero; iteration counter 0
    FS_HIP(launch_init(st, S.pots, S.state, nullptr, nullptr, update_f ? nullptr : in64, update_f ? in64 : nullptr,
                       update_f ? 2 : 1));
    if (S.mode == 3) {
        FS_HIP(launch_points_prep(st, X, n, d, S.pots.s, (double *)(S.ws + L.o_Xp), (double *)(S.ws + L.o_Xs), (double *)(S.ws + L.o_cx)));
        FS_HIP(launch_points_prep(st, Y, m, d, S.pots.s, (double *)(S.ws + L.o_Yp), (double *)(S.ws + L.o_Ys), (double *)(S.ws + L.o_cy)));
    }
    if (update_f) {
        FS_HIP(S.enqueue_f_update(0, Solve::STREAM));  // writes F into buffer 1
        FS_HIP(launch_export(st, S.pots.F + L.n_ld, n, S.pots.s, out64));
    } else {
        FS_HIP(S.enqueue_g_update(Solve::STREAM));     // reads U of buffer 1 (= the given f), writes G into buffer 1
        FS_HIP(launch_export(st, S.pots.G + L.m_ld, m, S.pots.s, out64));
    }
    return FS_OK;
}

}  // namespace

// ================================================================ C ABI
extern "C" {

const char *fs_last_error(void) { return g_err; }
const char *fs_version(void) { return "fastsinkhorn-gfx950 0.1"; }

void fs_clear_cache(void) {
    g_timing = KernelTiming{};              // its events are about to go
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto &kv : g_cache) {
        DeviceCache &c = kv.second;
        int cur = 0;
        if (hipGetDevice(&cur) != hipSuccess) continue;
        (void)hipSetDevice(kv.first);
        (void)hipDeviceSynchronize();
        if (c.ws) (void)hipFree(c.ws);
        if (c.host) (void)hipHostFree((void *)c.host);
        for (auto &e : c.ev) if (e) (void)hipEventDestroy(e);
        for (auto &e : c.timing) (void)hipEventDestroy(e);
        if (c.cap_stream) (void)hipStreamDestroy(c.cap_stream);
        if (c.tickets) (void)hipFree(c.tickets);
        (void)hipSetDevice(cur);
    }
    g_cache.clear();
}

int fs_kernel_choice(int n, int m, int d, const fs_options *opts, int blocking, int compute_units) {
    // the decisions of solve_blocking / solve_async in their order, on a problem that only has a shape
    const float *dummy = reinterpret_cast<const float *>(uintptr_t(4096));
    Problem pr{d == 0 ? dummy : nullptr, d == 0 ? nullptr : dummy, d == 0 ? nullptr : dummy, dummy, dummy, d, n, m, 1.0f, 1, 0.0f};
    fs_status v = validate(pr, const_cast<float *>(dummy), const_cast<float *>(dummy));
    if (v == FS_OK) v = check_options(pr, opts);
    if (v != FS_OK) return v;
    fs_status serr = FS_OK;
    if (small_path(pr, opts, &serr)) return FS_KERNEL_SMALL;
    if (serr != FS_OK) return serr;
    g_cus_override = compute_units;
    int wmax = 0;
    const bool grid = grid_path(pr, opts, blocking != 0, &serr, &wmax);
    g_cus_override = 0;
    if (serr != FS_OK) return serr;
    if (grid) return FS_KERNEL_GRID;
    if (coop_path(pr, opts, &serr)) return FS_KERNEL_COOP;
    if (serr != FS_OK) return serr;
    if (d != 0) return FS_KERNEL_POINTS;
    const int cd = opts ? opts->cost_dtype : 0, km = opts ? opts->kernel_mode : 0;
    const bool fused_ok = dense_fused_supported(n, m, dummy, cd);
    if (km == 6 && !blocking) { set_err("kernel_mode 6 is for the blocking solves"); return FS_ERR_UNSUPPORTED; }
    if (km == 6 && !dense_persist_supported(n, m, dummy, cd)) { set_err("kernel_mode 6 does not support m = %d", m); return FS_ERR_UNSUPPORTED; }
    g_cus_override = compute_units;
    int pcus = 0;
    const bool persist = persist_path(pr, opts, blocking != 0, &pcus);
    g_cus_override = 0;
    if (persist) return FS_KERNEL_PERSIST;
    if (km == 6) { set_err("kernel_mode 6 needs at least m / 64 row panels and compute units (and up to 1024 columns at most 512 rows per compute unit)"); return FS_ERR_UNSUPPORTED; }
    if (km == 2 && !fused_ok) { set_err("fused kernel does not support m = %d", m); return FS_ERR_UNSUPPORTED; }
    if (km > 2) { set_err("kernel_mode %d does not take this problem", km); return FS_ERR_UNSUPPORTED; }
    return (km == 2 || (km == 0 && fused_ok)) ? FS_KERNEL_FUSED : FS_KERNEL_STREAM;
}

fs_status fs_last_kernel_timing(float *avg_ms, int32_t *samples, const char **kernel_name, int32_t *iters_sampled) {
    if (g_timing.samples <= 0) { set_err("no timed solve has run on this thread"); return FS_ERR_INVALID_ARG; }
    if (!g_timing.pending.empty()) {
        double tot = 0.0;
        for (const auto &ev : g_timing.pending) {
            float ms = 0.0f;
            FS_HIP(hipEventElapsedTime(&ms, ev.first, ev.second));
            tot += ms;
        }
        g_timing.avg_ms = (float)(tot / (double)g_timing.pending.size());
        g_timing.pending.clear();
    }
    if (avg_ms) *avg_ms = g_timing.avg_ms;
    if (samples) *samples = g_timing.samples;
    if (kernel_name) *kernel_name = g_timing.name;
    if (iters_sampled) *iters_sampled = g_timing.iters_sampled;
    return FS_OK;
}

fs_status fs_read_rate(const void *buf, size_t bytes, int reps, float *us_per_pass, fs_stream stream) {
    if (!buf || !us_per_pass || bytes < 16 || reps < 1 || (reinterpret_cast<uintptr_t>(buf) & 15u) != 0) {
        set_err("fs_read_rate: buf (16-byte aligned) and us_per_pass must be non-null, bytes >= 16, reps >= 1");
        return FS_ERR_INVALID_ARG;
    }
    DeviceCache *dc = nullptr;
    const fs_status v = get_cache(256, &dc);
    if (v != FS_OK) return v;
    const int cus = device_cus();
    if (cus < 1) { set_err("fs_read_rate: no compute units reported"); return FS_ERR_HIP; }
    hipStream_t st = (hipStream_t)stream;
    float *sink = reinterpret_cast<float *>(dc->tickets) + 63;      // never written (see the kernel)
    hipEvent_t e0, e1;
    FS_HIP(hipEventCreate(&e0));
    FS_HIP(hipEventCreate(&e1));
    for (int r = 0; r < 2; ++r) FS_HIP(launch_read_stream(st, buf, bytes, cus, sink));
    FS_HIP(hipEventRecord(e0, st));
    for (int r = 0; r < reps; ++r) FS_HIP(launch_read_stream(st, buf, bytes, cus, sink));
    FS_HIP(hipEventRecord(e1, st));
    FS_HIP(hipEventSynchronize(e1));
    float ms = 0.0f;
    FS_HIP(hipEventElapsedTime(&ms, e0, e1));
    FS_HIP(hipEventDestroy(e0));
    FS_HIP(hipEventDestroy(e1));
    *us_per_pass = ms * 1e3f / (float)reps;
    return FS_OK;
}

size_t fs_workspace_bytes(int n, int m, int d) {
    if (n < 1 || m < 1 || d < 0 || d > FS_MAX_DIM) return 0;
    return make_layout(n, m, d).total;
}

int fs_sinkhorn_dense(const float *C, const float *a, const float *b, int n, int m, float eps, int max_iter,
                      float tol, float *f, float *g, fs_stream stream) {
    if (!C) { set_err("C must be non-null"); return FS_ERR_INVALID_ARG; }
    Problem pr{C, nullptr, nullptr, a, b, 0, n, m, eps, max_iter, tol};
    return solve_blocking(pr, f, g, (hipStream_t)stream, nullptr, nullptr);
}

int fs_sinkhorn_points(const float *X, const float *Y, int d, const float *a, const float *b, int n, int m,
                       float eps, int max_iter, float tol, float *f, float *g, fs_stream stream) {
    if (!X || !Y) { set_err("X and Y must be non-null"); return FS_ERR_INVALID_ARG; }
    Problem pr{nullptr, X, Y, a, b, d, n, m, eps, max_iter, tol};
    return solve_blocking(pr, f, g, (hipStream_t)stream, nullptr, nullptr);
}

int fs_sinkhorn_solve(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, int max_iter, float tol, float *f, float *g, fs_stream stream,
                      const fs_options *opts, fs_result *result_host) {
    Problem pr{C, X, Y, a, b, d, n, m, eps, max_iter, tol};
    return solve_blocking(pr, f, g, (hipStream_t)stream, opts, result_host);
}

int fs_sinkhorn_annealed(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                         int n, int m, float eps, float eps_start, float decay, int stage_iters, int max_iter,
                         float tol, float *f, float *g, fs_stream stream, const fs_options *opts,
                         fs_result *result_host, int32_t *total_iters) {
    if (!(eps_start >= eps) || !std::isfinite(eps_start)) { set_err("eps_start must be finite and >= eps"); return FS_ERR_INVALID_ARG; }
    if (!(decay > 0.0f && decay < 1.0f)) { set_err("decay must be in (0, 1)"); return FS_ERR_INVALID_ARG; }
    if (stage_iters < 1) { set_err("stage_iters must be >= 1"); return FS_ERR_INVALID_ARG; }
    fs_options o{};
    if (opts) o = *opts;
    const int user_warm = o.warm_start;
    int total = 0, stage = 0;
    // intermediate stages: fixed iteration count, no trailing error pass, potentials handed on in f, g
    for (float e = eps_start; e > eps; e *= decay, ++stage) {
        fs_options so = o;
        so.warm_start = (stage > 0) ? 1 : user_warm;
        so.skip_final_err = 1;
        so.err_history = nullptr; so.err_history_len = 0;
        so.f64_out = nullptr; so.g64_out = nullptr;
        if (stage > 0) { so.f64_in = nullptr; so.g64_in = nullptr; }
        so.time_kernel_every = 0;
        Problem pr{C, X, Y, a, b, d, n, m, e, stage_iters, 0.0f};
        const int it = solve_blocking(pr, f, g, (hipStream_t)stream, &so, nullptr);
        if (it < 0) return it;
        total += it;
    }
    fs_options fo = o;
    if (stage > 0) { fo.warm_start = 1; fo.f64_in = nullptr; fo.g64_in = nullptr; }
    Problem pr{C, X, Y, a, b, d, n, m, eps, max_iter, tol};
    const int it = solve_blocking(pr, f, g, (hipStream_t)stream, &fo, result_host);
    if (it < 0) return it;
    if (total_iters) *total_iters = total + it;
    return it;
}

fs_status fs_sinkhorn_dense_ex(const float *C, const float *a, const float *b, int n, int m, float eps,
                               int max_iter, float tol, float *f, float *g, fs_stream stream,
                               const fs_options *opts, void *workspace, size_t workspace_bytes,
                               fs_result *result_dev) {
    if (!C) { set_err("C must be non-null"); return FS_ERR_INVALID_ARG; }
    Problem pr{C, nullptr, nullptr, a, b, 0, n, m, eps, max_iter, tol};
    return solve_async(pr, f, g, (hipStream_t)stream, opts, workspace, workspace_bytes, result_dev);
}

fs_status fs_sinkhorn_dense_static(const float *C, const float *a, const float *b, int n, int m, float eps,
                                   int max_iter, float tol, float *f, float *g, fs_stream stream,
                                   const fs_options *opts, fs_result *result_dev) {
    if (!C) { set_err("C must be non-null"); return FS_ERR_INVALID_ARG; }
    Problem pr{C, nullptr, nullptr, a, b, 0, n, m, eps, max_iter, tol};
    fs_status v = validate(pr, f, g);
    if (v != FS_OK) return v;
    const size_t need = make_layout(n, m, 0).total;
    if (need > (size_t)FS_STATIC_SCRATCH_BYTES) {
        set_err("a %d x %d problem needs %zu bytes of scratch, the static buffer holds %zu: use fs_sinkhorn_dense_ex "
                "with a workspace of the caller's", n, m, need, (size_t)FS_STATIC_SCRATCH_BYTES);
        return FS_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    v = static_scratch(&ws);
    if (v != FS_OK) return v;
    return solve_async(pr, f, g, (hipStream_t)stream, opts, ws, (size_t)FS_STATIC_SCRATCH_BYTES, result_dev);
}

fs_status fs_sinkhorn_points_ex(const float *X, const float *Y, int d, const float *a, const float *b, int n,
                                int m, float eps, int max_iter, float tol, float *f, float *g, fs_stream stream,
                                const fs_options *opts, void *workspace, size_t workspace_bytes,
                                fs_result *result_dev) {
    if (!X || !Y) { set_err("X and Y must be non-null"); return FS_ERR_INVALID_ARG; }
    Problem pr{nullptr, X, Y, a, b, d, n, m, eps, max_iter, tol};
    return solve_async(pr, f, g, (hipStream_t)stream, opts, workspace, workspace_bytes, result_dev);
}

fs_status fs_sinkhorn_dense_batched(const float *C, const float *a, const float *b, int batch, int n, int m,
                                    float eps, int max_iter, float tol, float *f, float *g, fs_stream stream,
                                    const fs_options *opts, fs_result *result_dev) {
    if (!C) { set_err("C must be non-null"); return FS_ERR_INVALID_ARG; }
    if (batch < 1) { set_err("batch must be >= 1 (got %d)", batch); return FS_ERR_INVALID_ARG; }
    Problem pr{C, nullptr, nullptr, a, b, 0, n, m, eps, max_iter, tol};
    fs_status v = validate(pr, f, g);
    if (v != FS_OK) return v;
    if (n > FS_SMALL_MAX || m > FS_SMALL_MAX) {
        set_err("batched solves need n, m <= %d (got %d, %d)", FS_SMALL_MAX, n, m);
        return FS_ERR_UNSUPPORTED;
    }
    if (opts && opts->kernel_mode != 0 && opts->kernel_mode != 3) { set_err("batched solves have one kernel (kernel_mode 0 or 3)"); return FS_ERR_INVALID_ARG; }
    v = check_options(pr, opts);
    if (v != FS_OK) return v;
    SmallArgs A;
    v = small_args(pr, batch, opts, f, g, &A);
    if (v != FS_OK) return v;
    A.result = (ResultRecord *)result_dev;
    FS_HIP(launch_small((hipStream_t)stream, A));
    return FS_OK;
}

fs_status fs_plan(const float *C, const float *X, const float *Y, int d, const float *a, const float *b, int n,
                  int m, float eps, const float *f, const float *g, float *P, fs_stream stream) {
    if (!P) { set_err("P must be non-null"); return FS_ERR_INVALID_ARG; }
    if (!f || !g) { set_err("f and g must be non-null"); return FS_ERR_INVALID_ARG; }
    return plan_or_cost(C, X, Y, d, a, b, n, m, eps, f, g, nullptr, nullptr, P, nullptr, (hipStream_t)stream);
}

fs_status fs_cost(const float *C, const float *X, const float *Y, int d, const float *a, const float *b, int n,
                  int m, float eps, const float *f, const float *g, double *cost_dev, fs_stream stream) {
    if (!cost_dev) { set_err("cost_dev must be non-null"); return FS_ERR_INVALID_ARG; }
    if (!f || !g) { set_err("f and g must be non-null"); return FS_ERR_INVALID_ARG; }
    return plan_or_cost(C, X, Y, d, a, b, n, m, eps, f, g, nullptr, nullptr, nullptr, cost_dev, (hipStream_t)stream);
}

fs_status fs_plan_f64(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *f64, const double *g64, float *P, fs_stream stream) {
    if (!P) { set_err("P must be non-null"); return FS_ERR_INVALID_ARG; }
    if (!f64 || !g64) { set_err("f64 and g64 must be non-null"); return FS_ERR_INVALID_ARG; }
    return plan_or_cost(C, X, Y, d, a, b, n, m, eps, nullptr, nullptr, f64, g64, P, nullptr, (hipStream_t)stream);
}

fs_status fs_cost_f64(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *f64, const double *g64, double *cost_dev,
                      fs_stream stream) {
    if (!cost_dev) { set_err("cost_dev must be non-null"); return FS_ERR_INVALID_ARG; }
    if (!f64 || !g64) { set_err("f64 and g64 must be non-null"); return FS_ERR_INVALID_ARG; }
    return plan_or_cost(C, X, Y, d, a, b, n, m, eps, nullptr, nullptr, f64, g64, nullptr, cost_dev, (hipStream_t)stream);
}

fs_status fs_diagnostics(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                         int n, int m, float eps, const float *f, const float *g, const double *f64,
                         const double *g64, double *out_dev, double *row_marginal_dev, double *col_marginal_dev,
                         fs_stream stream) {
    return diagnostics(C, X, Y, d, a, b, n, m, eps, f, g, f64, g64, out_dev, row_marginal_dev, col_marginal_dev,
                       (hipStream_t)stream);
}

fs_status fs_barycentric(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                         int n, int m, float eps, const float *f, const float *g, const double *f64,
                         const double *g64, const float *Z, int dz, float *T, fs_stream stream) {
    return barycentric(C, X, Y, d, a, b, n, m, eps, f, g, f64, g64, Z, dz, T, (hipStream_t)stream);
}

fs_status fs_update_f(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *g64, double *f64_out, fs_stream stream) {
    if (!g64 || !f64_out) { set_err("g64 and f64_out must be non-null"); return FS_ERR_INVALID_ARG; }
    return half_step(true, C, X, Y, d, a, b, n, m, eps, g64, f64_out, (hipStream_t)stream);
}

fs_status fs_update_g(const float *C, const float *X, const float *Y, int d, const float *a, const float *b,
                      int n, int m, float eps, const double *f64, double *g64_out, fs_stream stream) {
    if (!f64 || !g64_out) { set_err("f64 and g64_out must be non-null"); return FS_ERR_INVALID_ARG; }
    return half_step(false, C, X, Y, d, a, b, n, m, eps, f64, g64_out, (hipStream_t)stream);
}

}  // extern "C"
