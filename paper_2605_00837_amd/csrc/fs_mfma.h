// Point clouds on the fp64 matrix cores: the walk over 16 x 16 tiles of dot products shared by the
// kernels that evaluate the plan of Eq. 5 for point-cloud inputs (diagnostics, barycentric mapping,
// plan).  v_mfma_f64_16x16x4f64 computes a 16 x 16 tile over 4 coordinates per instruction:
//   A: lane l holds x[row l % 16][k = l / 16];  B: lane l holds y'[col l % 16][k = l / 16];
//   result register r of lane l is entry (row l / 16 + 4 r, col l % 16).
// Products of fp32 coordinates are exact in fp64 and the accumulation is fp64.
#pragma once
#include "fs_device.h"

namespace fs {

constexpr int kTileJ = 64;            // columns staged in LDS at a time
constexpr int kTileRT = 2;            // row tiles (16 rows each) per wave
constexpr int kTileRows = 4 * kTileRT * 16;      // rows per workgroup of 4 waves (256 threads)

typedef double double4_m __attribute__((ext_vector_type(4)));

constexpr int mfma_d4(int d) { return d <= 4 ? 1 : d <= 8 ? 2 : d <= 16 ? 4 : d <= 32 ? 8 : 16; }

__device__ __forceinline__ float row16_sum(float v) {             // all-reduce over a DPP row of 16 lanes
    v += dpp_f32<0x128>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x122>(v);
    v += dpp_f32<0x121>(v);
    return v;
}
__device__ __forceinline__ double row16_sum(double v) {
    v += dpp_f64<0x128>(v);
    v += dpp_f64<0x124>(v);
    v += dpp_f64<0x122>(v);
    v += dpp_f64<0x121>(v);
    return v;
}

// The row side of a wave: A operands of its kTileRT row tiles, zero beyond nr and beyond d.
template <int D4>
struct RowTiles {
    double a[kTileRT][D4];
    int row0;                          // first row of the wave
    __device__ __forceinline__ void load(const double *rows, int nr, int d) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int lj = lane & 15, lk = lane >> 4;
        row0 = blockIdx.x * kTileRows + wave * (kTileRT * 16);
#pragma unroll
        for (int rt = 0; rt < kTileRT; ++rt) {
            const int row = row0 + rt * 16 + lj;
#pragma unroll
            for (int ks = 0; ks < D4; ++ks) {
                const int t = 4 * ks + lk;
                a[rt][ks] = (row < nr && t < d) ? rows[(size_t)row * d + t] : 0.0;
            }
        }
    }
    // the row that result register r of row tile rt belongs to, in this lane
    __device__ __forceinline__ int result_row(int rt, int r) const {
        return row0 + rt * 16 + ((threadIdx.x & 63) >> 4) + 4 * r;
    }
};

// Walks the columns [j0, j1) in LDS tiles of kTileJ.  `tile` is the workgroup's LDS buffer
// [kTileJ][4 * D4 + 1].  stage(jt) is called by all threads after the coordinates of the tile
// starting at column jt have been requested and before the barrier (to stage per-column extras);
// init(ct, rt, r) gives the start value of the accumulator; done(jt, ct, rt, acc) consumes the 4
// results of row tile rt against columns jt + 16 ct + (lane % 16).
template <int D4, class Stage, class Init, class Done>
__device__ __forceinline__ void mfma_walk(const RowTiles<D4> &R, double (*tile)[4 * D4 + 1], const double *cols2s,
                                          int d, int j0, int j1, Stage stage, Init init, Done done) {
#if defined(__HIP_DEVICE_COMPILE__)
    const int tid = threadIdx.x, lane = tid & 63;
    const int lj = lane & 15, lk = lane >> 4;
    for (int jt = j0; jt < j1; jt += kTileJ) {
        __syncthreads();                                   // previous tile fully consumed
        for (int e = tid; e < kTileJ * 4 * D4; e += 256) {
            const int jj = e / (4 * D4), t = e % (4 * D4);
            const int j = jt + jj;
            tile[jj][t] = (j < j1 && t < d) ? cols2s[(size_t)j * d + t] : 0.0;
        }
        stage(jt);
        __syncthreads();
#pragma unroll
        for (int ct = 0; ct < kTileJ / 16; ++ct) {
            double b[D4];
#pragma unroll
            for (int ks = 0; ks < D4; ++ks) b[ks] = tile[ct * 16 + lj][4 * ks + lk];
            double4_m acc[kTileRT];
#pragma unroll
            for (int rt = 0; rt < kTileRT; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[rt][r] = init(ct, rt, r);
#pragma unroll
            for (int ks = 0; ks < D4; ++ks)
#pragma unroll
                for (int rt = 0; rt < kTileRT; ++rt)
                    acc[rt] = __builtin_amdgcn_mfma_f64_16x16x4f64(R.a[rt][ks], b[ks], acc[rt], 0, 0, 0);
#pragma unroll
            for (int rt = 0; rt < kTileRT; ++rt) done(jt, ct, rt, acc[rt]);
        }
    }
#endif
}

}  // namespace fs
