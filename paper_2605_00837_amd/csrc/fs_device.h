// Device-side building blocks shared by the gfx950 kernels: wave64 reductions
// (DPP inside a row of 16 lanes, v_permlane16_swap / v_permlane32_swap across rows), the
// fp32 exp2/log2 hardware instructions, the online (max, sum) LogSumExp update
// and the device-resident solver state.
//
// Arithmetic convention of every kernel.  With s = log2(e)/eps the potentials
// are carried as F_i = -s f_i and G_j = -s g_j in double precision, together
// with U_i = log2 a_i - F_i and V_j = log2 b_j - G_j.  One half-step of the
// paper's Eq. 9 is then F_i = LSE2_j( V_j - s C_ij ), and Eq. 10 is
// G_j = LSE2_i( U_i - s C_ij ), where LSE2 is the base-2 LogSumExp of Eq. 8.
// The argument of every exponential is formed in fp64 and only the difference
// to the running maximum is rounded to fp32 for v_exp_f32.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace fs {

constexpr double kNegHuge = -1.0e300;   // finite stand-in for "-inf" as a running maximum

// ---------------------------------------------------------------- state
// Lives in device memory (first 256 bytes of the workspace).  Written only by
// the init kernel, by the single "advance" thread after each iteration and by
// the finalize kernels.
struct alignas(256) State {
    int32_t k;            // iterations completed
    int32_t flags;        // bit 0: stop flag (every later kernel of the solve returns at once);
                          // bit 1: pace hint for the next iteration, 1 = the potentials move slowly (FAST)
    int32_t iters;        // result: iterations whose potentials are returned
    int32_t converged;
    int32_t nonfinite;
    int32_t err_valid;
    double err;           // err after `iters`
    // Closing word of the iteration in progress, updated with ONE atomic per workgroup: bits 0..13
    // count the workgroups that have reported (the ticket), bits 14..62 hold the fixed-point sum of
    // their error terms, bit 63 says that some share was not a number (or that the sum left its range).
    // Returns to 0 after every use.
    unsigned long long err_acc;
    uint32_t big_acc[2];  // columns that moved by more than the FAST-mode threshold, by parity of the iteration
    uint32_t fin_ticket;  // workgroups of the finalize kernel that are through (the last one writes the result record)
};

constexpr int kHintRing = 256;        // slots of the host-visible ring of pace hints (index: iteration mod ring)

// Constant description of one solve, passed by value to the kernels.
struct Ctl {
    State *st;
    int32_t max_iter;
    int32_t check_every;
    double tol;               // <= 0: fixed iteration count
    float *err_history;       // device, may be null
    int32_t err_history_len;
    int32_t phase;            // 0: iteration kernel, 1: trailing error pass
    volatile int32_t *host_flag;   // pinned host mirror of {done, mode hint}, may be null
    int32_t force_fast;       // 1: kernels that follow the device's pace hint take the FAST variant regardless
};

// The iteration counter and the stop flag sit side by side and are fetched with ONE 8-byte load (a
// relaxed atomic: it is neither split nor repeated, and nothing waits for it until its value is used,
// so loads issued after it overlap with it).
__device__ __forceinline__ unsigned long long load_counter(const Ctl &c) {
    static_assert(offsetof(State, k) == 0 && offsetof(State, flags) == 4, "k and the flags are read as one word");
    return __hip_atomic_load(reinterpret_cast<const unsigned long long *>(c.st), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
}
// Does this launch have work to do?  Iteration kernels run while k < max_iter, the trailing error
// pass runs only when k == max_iter; nothing runs once done.
constexpr int kFlagDone = 1, kFlagFast = 2;
__device__ __forceinline__ bool counter_active(const Ctl &c, unsigned long long kd, int &k, bool *fast_hint = nullptr) {
    // the same value in every lane; readfirstlane tells the compiler so (scalar control flow and
    // scalar addressing everywhere downstream)
    k = __builtin_amdgcn_readfirstlane((int)(unsigned)kd);
    const int flags = __builtin_amdgcn_readfirstlane((int)(unsigned)(kd >> 32));
    if (fast_hint) *fast_hint = (flags & kFlagFast) != 0 || c.force_fast != 0;
    if (flags & kFlagDone) return false;
    return c.phase == 0 ? (k < c.max_iter) : (k == c.max_iter);
}
__device__ __forceinline__ bool launch_active(const Ctl &c, int &k) { return counter_active(c, load_counter(c), k); }

// ---------------------------------------------------------------- math
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }    // v_log_f32

// log2 of a positive fp32 sum as a double, accurate to ~1e-7 absolute whatever the magnitude of
// the sum: the exponent is taken exactly (v_frexp_exp), v_log_f32 only sees the mantissa in
// [0.5, 1).  log2(0) = -inf, log2(inf) = +inf, NaN stays NaN.
__device__ __forceinline__ double log2_sum(float s) {
    const int e = __builtin_amdgcn_frexp_expf(s);
    const float mant = __builtin_amdgcn_frexp_mantf(s);
    return (double)e + (double)__builtin_amdgcn_logf(mant);
}

// same for a sum held in double precision (it may lie below the fp32 range)
__device__ __forceinline__ double log2_sum(double s) {
    const int e = __builtin_amdgcn_frexp_exp(s);
    const float mant = (float)__builtin_amdgcn_frexp_mant(s);
    return (double)e + (double)__builtin_amdgcn_logf(mant);
}

__device__ __forceinline__ double dmax(double a, double b) { return fmax(a, b); }

// log2 of an fp32 weight in double precision; zero (or negative) weight -> -inf.
__device__ __forceinline__ double log2_weight(float w) {
    return w > 0.0f ? log2((double)w) : -__builtin_huge_val();
}

// A cost entry stored in 2 bytes, from its bits: DT = 1 IEEE half precision, DT = 2 bfloat16.
template <int DT>
__device__ __forceinline__ float cost_from_bits(unsigned bits16) {
    if constexpr (DT == 1) {
        return (float)__builtin_bit_cast(_Float16, (unsigned short)bits16);
    } else {
        return __uint_as_float(bits16 << 16);
    }
}

// Entry `idx` of a cost matrix stored as fp32 (dtype 0), fp16 (1) or bfloat16 (2).
__device__ __forceinline__ float cost_entry(const float *C, int dtype, size_t idx) {
    if (dtype == 0) return C[idx];
    const unsigned bits = reinterpret_cast<const unsigned short *>(C)[idx];
    return dtype == 1 ? cost_from_bits<1>(bits) : cost_from_bits<2>(bits);
}

// 2^d - 1 with a relative error below 2e-6 and few registers (the library's expm1 costs about a hundred
// instructions and, in the kernels whose lanes hold a tile of the cost matrix, much of their register
// budget): a 6-term series where the result is small, v_exp_f32 elsewhere.
__device__ __forceinline__ double exp2m1(double d) {
    const double t = d * 0.6931471805599453094;
    if (fabs(t) < 0.0625)
        return t * (1.0 + t * (0.5 + t * (1.0 / 6.0 + t * (1.0 / 24.0 + t * (1.0 / 120.0 + t * (1.0 / 720.0))))));
    return (double)fast_exp2((float)d) - 1.0;
}

// A cost entry held in a register for a whole solve, as an fp64 value, through a compiler barrier: every
// use converts its 4-byte register afresh.  Without it the compiler keeps all converted values of a lane's
// tile alive (twice the registers) across the two half-steps, or hoists them out of the iteration loop,
// and spills.
__device__ __forceinline__ double cost_f64(float &c) {       // by reference: the barrier acts on the register itself
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+v"(c));
#endif
    return (double)c;
}
__device__ __forceinline__ double cost_f64(double c) { return c; }

// Four adjacent fp32 values at any 4-byte boundary (rows of a matrix whose width is not a multiple of
// 4 start anywhere): one 16-byte access, the hardware's unaligned access mode does the rest.
typedef float float4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// ---------------------------------------------------------------- DPP / swizzle moves
// dpp_ctrl encodings: row_ror:n = 0x120 + n (rotate inside a row of 16 lanes).
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(dpp_i32<CTRL>(__float_as_int(v)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    int lo = dpp_i32<CTRL>(__double2loint(v));
    int hi = dpp_i32<CTRL>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}
// The two exchanges across the rows of 16 lanes go through the vector ALU, with the lane swaps of this device:
// v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second, v_permlane32_swap
// the upper half of the first with the lower half of the second (checked on the device).  With the same value v in
// both operands the results are a = [v.row0, v.row0, v.row2, v.row2] and b = [v.row1, v.row1, v.row3, v.row3]
// (resp. a = [v.lower, v.lower], b = [v.upper, v.upper]): every lane finds its own and its partner's value in them.
// (ds_swizzle / ds_bpermute do the same through the LDS crossbar: two round trips of its latency in front of every
// barrier that follows a row sum; 32768 x 2048 ran 9 % slower per iteration with them.)
__device__ __forceinline__ void rows16_i32(int v, int &a, int &b) {
    const auto p = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
    a = (int)p[0];
    b = (int)p[1];
}
__device__ __forceinline__ void halves32_i32(int v, int &a, int &b) {
    const auto p = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    a = (int)p[0];
    b = (int)p[1];
}
// the value of lane ^ 16
__device__ __forceinline__ int swz16_i32(int v) {
    int a, b;
    rows16_i32(v, a, b);
    return (__lane_id() & 16) ? a : b;
}
// the value of lane ^ 32
__device__ __forceinline__ int xor32_i32(int v) {
    int a, b;
    halves32_i32(v, a, b);
    return (__lane_id() & 32) ? a : b;
}
__device__ __forceinline__ float swz16_f32(float v) { return __int_as_float(swz16_i32(__float_as_int(v))); }
__device__ __forceinline__ float xor32_f32(float v) { return __int_as_float(xor32_i32(__float_as_int(v))); }
__device__ __forceinline__ double swz16_f64(double v) {
    return __hiloint2double(swz16_i32(__double2hiint(v)), swz16_i32(__double2loint(v)));
}
__device__ __forceinline__ double xor32_f64(double v) {
    return __hiloint2double(xor32_i32(__double2hiint(v)), xor32_i32(__double2loint(v)));
}

// the value lane `src_lane` (wave-uniform) holds, in every lane
__device__ __forceinline__ double bcast_f64(double x, int src_lane) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), src_lane),
                            __builtin_amdgcn_readlane(__double2loint(x), src_lane));
}
__device__ __forceinline__ float bcast_f32(float x, int src_lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src_lane));
}

// All-reduce over the 64 lanes of a wave; every lane must be active.
__device__ __forceinline__ double wave_max_f64(double v) {
    v = dmax(v, dpp_f64<0x128>(v));   // row_ror:8
    v = dmax(v, dpp_f64<0x124>(v));   // row_ror:4
    v = dmax(v, dpp_f64<0x122>(v));   // row_ror:2
    v = dmax(v, dpp_f64<0x121>(v));   // row_ror:1
    int ah, bh, al, bl;
    rows16_i32(__double2hiint(v), ah, bh);
    rows16_i32(__double2loint(v), al, bl);
    v = dmax(__hiloint2double(ah, al), __hiloint2double(bh, bl));
    halves32_i32(__double2hiint(v), ah, bh);
    halves32_i32(__double2loint(v), al, bl);
    return dmax(__hiloint2double(ah, al), __hiloint2double(bh, bl));
}
__device__ __forceinline__ float wave_sum_f32(float v) {
    v += dpp_f32<0x128>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x122>(v);
    v += dpp_f32<0x121>(v);
    // (the same two values are added in every lane as with v += value of lane ^ 16, then lane ^ 32)
    int a, b;
    rows16_i32(__float_as_int(v), a, b);
    v = __int_as_float(a) + __int_as_float(b);
    halves32_i32(__float_as_int(v), a, b);
    return __int_as_float(a) + __int_as_float(b);
}
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_f64<0x128>(v);
    v += dpp_f64<0x124>(v);
    v += dpp_f64<0x122>(v);
    v += dpp_f64<0x121>(v);
    int ah, bh, al, bl;
    rows16_i32(__double2hiint(v), ah, bh);
    rows16_i32(__double2loint(v), al, bl);
    v = __hiloint2double(ah, al) + __hiloint2double(bh, bl);
    halves32_i32(__double2hiint(v), ah, bh);
    halves32_i32(__double2loint(v), al, bl);
    return __hiloint2double(ah, al) + __hiloint2double(bh, bl);
}

// The sums over the 64 lanes of a wave of N values per lane (N rows of a panel), each stored by one lane to
// dst[row * stride].  Two rows at a time: v_permlane32_swap of two registers puts the lower halves of both into one
// and the upper halves into the other, so ONE exchange and one addition halve two rows at once (a wave sum per row
// takes two exchanges and two additions for these two steps); the same with v_permlane16_swap across the rows of 16
// lanes; the last four steps (inside 16 lanes) are DPP rotations of the N / 4 registers that are left.  For N = 8:
// 20 instructions instead of 64.  Row 4 i + k ends up in lanes 16 k' ... of register i with k = {0, 2, 1, 3}[k'].
template <int N>
__device__ __forceinline__ void rows_sum_store(const float (&acc)[N], float *dst, int stride, int lane) {
    static_assert(N == 1 || N == 2 || N == 4 || N == 8, "rows per row group of a panel");
    auto rot16 = [](float x) {
        x += dpp_f32<0x128>(x);
        x += dpp_f32<0x124>(x);
        x += dpp_f32<0x122>(x);
        x += dpp_f32<0x121>(x);
        return x;
    };
    if constexpr (N == 1) {
        const float t = wave_sum_f32(acc[0]);
        if (lane == 0) dst[0] = t;
    } else {
        float p[N / 2];                        // lanes 0 .. 31: row 2 i, lanes 32 .. 63: row 2 i + 1
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
            const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[2 * i]), __float_as_uint(acc[2 * i + 1]),
                                                            false, false);
            p[i] = __uint_as_float(h[0]) + __uint_as_float(h[1]);
        }
        if constexpr (N == 2) {
            const auto h = __builtin_amdgcn_permlane16_swap(__float_as_uint(p[0]), __float_as_uint(p[0]), false, false);
            const float t = rot16(__uint_as_float(h[0]) + __uint_as_float(h[1]));
            if ((lane & 31) == 0) dst[(lane >> 5) * stride] = t;
        } else {
#pragma unroll
            for (int i = 0; i < N / 4; ++i) {
                const auto h = __builtin_amdgcn_permlane16_swap(__float_as_uint(p[2 * i]), __float_as_uint(p[2 * i + 1]),
                                                                false, false);
                const float t = rot16(__uint_as_float(h[0]) + __uint_as_float(h[1]));
                const int kq = lane >> 4;      // lanes 16 kq ...: row 4 i + {0, 2, 1, 3}[kq]
                if ((lane & 15) == 0) dst[(4 * i + ((kq & 1) << 1) + (kq >> 1)) * stride] = t;
            }
        }
    }
}

// ---------------------------------------------------------------- barriers and waits around LDS-DMA prefetch
// A workgroup barrier that waits for this wave's LDS traffic only.  __syncthreads() carries a fence that also
// waits for every vector-memory operation in flight, i.e. for an asynchronous HBM -> LDS prefetch.
__device__ __forceinline__ void lds_only_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xc07f);            // lgkmcnt(0): this wave's LDS writes are done
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#endif
}

constexpr int waitcnt_vm(int n) { return 0x0f70 | (n & 15) | ((n >> 4) << 14); }   // s_waitcnt vmcnt(n) only

// ---------------------------------------------------------------- online LSE
// Running base-2 LogSumExp as (M, s): value = M + log2(s), s = sum 2^(x - M).
struct Lse {
    double M;
    float s;
    __device__ __forceinline__ void init() { M = kNegHuge; s = 0.0f; }
    // fold a chunk of N arguments; one rescale per chunk
    template <int N>
    __device__ __forceinline__ void add(const double (&x)[N]) {
        double cm = x[0];
#pragma unroll
        for (int e = 1; e < N; ++e) cm = dmax(cm, x[e]);
        const double Mn = dmax(M, cm);
        float acc = s * fast_exp2((float)(M - Mn));
#pragma unroll
        for (int e = 0; e < N; ++e) acc += fast_exp2((float)(x[e] - Mn));
        s = acc;
        M = Mn;
    }
    // merge another running pair
    __device__ __forceinline__ void merge(double M2, float s2) {
        const double Mn = dmax(M, M2);
        s = s * fast_exp2((float)(M - Mn)) + s2 * fast_exp2((float)(M2 - Mn));
        M = Mn;
    }
    // all lanes of the wave end up with the wave's pair
    __device__ __forceinline__ void wave_reduce() {
        const double Mw = wave_max_f64(M);
        s = wave_sum_f32(s * fast_exp2((float)(M - Mw)));
        M = Mw;
    }
    __device__ __forceinline__ double value() const { return M + log2_sum(s); }
};

// ---------------------------------------------------------------- last workgroup finishes
// What one workgroup hands to the workgroup that finishes the call (whichever arrives last): stores and loads at
// agent scope, which pass the per-die caches, and an arrival counter that returns to 0 after use.
__device__ __forceinline__ void agent_store_f64(double *p, double v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double agent_load_f64(const double *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void agent_store_f32(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float agent_load_f32(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Called by every thread of a workgroup after thread 0 has published the workgroup's record: true (for all
// threads) in the workgroup that arrives last of `total`.
__device__ __forceinline__ bool last_to_arrive(unsigned int *ticket, unsigned int total, int *lds_flag) {
    if (threadIdx.x == 0) {
        __builtin_amdgcn_s_waitcnt(0);                 // this workgroup's record has been acknowledged
        const unsigned int t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = t == total - 1u;
        if (last) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *lds_flag = last;
    }
    __syncthreads();
    return *lds_flag != 0;
}


// ---------------------------------------------------------------- advance
// Runs in ONE thread after the g-update of an iteration (or after the trailing
// error pass).  `err` is the row-marginal error of the iterate the launch
// started from, i.e. err_k for k = st->k (Alg. 1: checked when k mod c == 0).
__device__ __forceinline__ void advance_state(const Ctl &c, int k, double err, double big_cols) {
    State *st = c.st;
    // hint for the driver: at most 128 columns moved by more than 40 (base 2) this time
    const int hint = (big_cols <= 128.0) ? 1 : 0;
    if (c.host_flag) {                            // made visible by the completion of this kernel
        c.host_flag[1] = hint;
        c.host_flag[2 + ((k + 1) & (kHintRing - 1))] = hint;
    }
    if (c.err_history && k >= 1 && k - 1 < c.err_history_len) c.err_history[k - 1] = (float)err;
    const bool checked = (c.tol > 0.0) && (k >= 1) && (k % c.check_every == 0);
    bool stop = false;
    if (c.phase == 1) {                 // trailing pass: k == max_iter, nothing left to run
        stop = true;
        st->converged = (checked && err < c.tol) ? 1 : 0;
    } else if (checked && err < c.tol) {
        stop = true;
        st->converged = 1;
    }
    if (stop) {
        st->iters = k;
        st->err = err;
        st->err_valid = 1;
        __threadfence();
        st->flags = kFlagDone | (hint ? kFlagFast : 0);
        if (c.host_flag) {
            *c.host_flag = 1;
            __threadfence_system();
        }
    } else {
        st->flags = hint ? kFlagFast : 0;
        st->k = k + 1;
    }
}

}  // namespace fs
