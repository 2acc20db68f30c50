// Grid-wide exchange of the persistent kernels (fs_persist.hip, fs_resident.hip): agent-scope stores and loads of
// what the workgroups publish to one another, and the bounded grid-wide wait on the counters of PersistSync.
#pragma once

#include "fs_kernels.h"

namespace fs {
namespace {

__device__ __forceinline__ void pub_f64(double *p, double v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double get_f64(const double *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float get_f32(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// two adjacent floats at an 8-byte boundary as one store
__device__ __forceinline__ void pub_f32x2(float *p, float x, float y) {
    const unsigned long long v = (unsigned long long)__float_as_uint(x) | ((unsigned long long)__float_as_uint(y) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Grid-wide wait number `gen`, in two halves called by all 64 lanes of ONE wave while the others are parked at
// barriers, after every wave's published stores have been acknowledged.
//   grid_arrive  lane 0 counts the workgroup into its group's counter (the value comes back later);
//   grid_wait    the workgroup that completed its group writes `gen` into the group's word of every copy of the
//                `done` line (one store instruction); lanes 0..7 watch one word each of the copy this workgroup is
//                assigned and lane 8 the abort flag next to them, with ONE load instruction per poll, one poll at
//                a time (more polls in flight, or more pollers per line, delay the store they wait for).
//                Everything only grows.
// grid_wait returns 0 when the wait was abandoned (by this workgroup or by another).
__device__ __forceinline__ unsigned long long grid_arrive(PersistSync *sy) {
    unsigned long long old = 0ull;
    if ((threadIdx.x & 63) == 0)
        old = __hip_atomic_fetch_add(&sy->grp[blockIdx.x % kSyncGroups].v, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return old;
}
__device__ __forceinline__ int grid_wait(PersistSync *sy, unsigned long long old, unsigned long long gen, int W,
                                         int spin_limit) {
    const int lane = threadIdx.x & 63;
    const int grp = blockIdx.x % kSyncGroups;
    int last = 0;
    if (lane == 0) {
        const unsigned long long members = (unsigned long long)((W - grp + kSyncGroups - 1) / kSyncGroups);
        last = old + 1ull == gen * members;
    }
    if (__builtin_amdgcn_readfirstlane(last)) {
        // the workgroup that completed its group says so in every copy of the line: one store instruction
        if (lane == 0) __hip_atomic_store(&sy->done[grp], gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int q = lane; q < kSyncCopies; q += 64)
            __hip_atomic_store(&sy->copy[q][grp], gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const int groups = W < kSyncGroups ? W : kSyncGroups;
    const unsigned long long *watch = &sy->copy[blockIdx.x & (kSyncCopies - 1)][lane < kSyncGroups ? lane : kSyncGroups];
    int good = 1, spins = 0;
    for (;;) {
        unsigned long long v = 0ull;
        if (lane <= kSyncGroups) v = __hip_atomic_load(watch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool reached = lane < groups ? v >= gen : true;
        const bool aborted = lane == kSyncGroups && v != 0ull;
        if (__any(aborted) || ++spins > spin_limit) {
            good = 0;
            for (int q = lane; q < kSyncCopies; q += 64)
                __hip_atomic_store(&sy->copy[q][kSyncGroups], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) __hip_atomic_store(&sy->abort_flag, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
        if (__all(reached)) break;
        __builtin_amdgcn_s_sleep(1);
    }
    return good;
}

constexpr int kWgPartLd = 512;          // slots of the per-workgroup exchange array
constexpr int kAgent = 16;              // cache policy of a buffer load / store that other workgroups must see: sc1
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

}  // namespace
}  // namespace fs

// Debug builds (-DFS_PERSIST_TRACE) stamp the phases of one iteration per workgroup with the 100 MHz clock.
#ifdef FS_PERSIST_TRACE
#define FS_TRACE(slot) do { if (lane == 0 && X.trace) { \
        const long long now_ = (long long)__builtin_amdgcn_s_memrealtime(); \
        if (X.trace[65536 + 8191] < 0 ? k == 0 : k == k_end - 2) X.trace[(w * 16 + wave) * 8 + (slot)] = now_; \
        if ((slot) <= 1 && wave == 0 && (w == 0 || w == 100) && k < 2000) X.trace[65536 + (w ? 4096 : 0) + 2 * k + (slot)] = now_; } } while (0)
#else
#define FS_TRACE(slot) do { } while (0)
#endif
