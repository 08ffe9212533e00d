// Register tile of the dense row-major kernels: how a wavefront covers rows and columns of X.
#pragma once

#include "device_util.h"

namespace tron {

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

template <int E, int L, int U, bool VEC>
struct Tile {
    static constexpr int RW = kWave / L;     // rows per step
    static constexpr int RT = U * RW;        // rows per wave tile

    // load the U x E block of this lane; out-of-range rows / columns read as zero.  rows: bit i clear = row row0 + i
    // is not needed (its coefficient is zero) and is not read at all
    __device__ static __forceinline__ void load(const double *__restrict__ X, int64_t n, int64_t d, int64_t row0,
                                                int lane, double (&x)[U][E], uint64_t rows = ~0ull)
    {
        const int q = lane % L, rl = lane / L;
        const int c0 = q * E;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = row0 + u * RW + rl;
            const bool rok = row < n && ((rows >> (u * RW + rl)) & 1u);
            const double *p = X + row * d + c0;
            if (VEC) {
#pragma unroll
                for (int e = 0; e < E; e += 2) {
                    double2 t = make_double2(0.0, 0.0);
                    if (rok && c0 + e < d) t = *reinterpret_cast<const double2 *>(p + e);
                    x[u][e] = t.x;
                    x[u][e + 1] = t.y;
                }
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) x[u][e] = (rok && c0 + e < d) ? p[e] : 0.0;
            }
        }
    }

    // t[u] = x_row . vec for the row this lane helps with in step u (all L lanes of the row get it)
    __device__ static __forceinline__ void row_dots(const double (&x)[U][E], const double (&vec)[E], double (&t)[U])
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            double s = 0.0;
#pragma unroll
            for (int e = 0; e < E; ++e) s = fma(x[u][e], vec[e], s);
            if (L == 2) s = sum2(s);
            else if (L == 4) s = sum4(s);
            else if (L == 8) s = sum8(s);
            else if (L >= 16) {
                s = sum16(s);
#pragma unroll
                for (int m = 16; m < L; m <<= 1) s += __shfl_xor(s, m, kWave);
            }
            t[u] = s;
        }
    }

    // lane i (< RT) receives the value of tile row i
    __device__ static __forceinline__ double to_row_owner(const double (&t)[U], int lane)
    {
        double mine = 0.0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const double got = __shfl(t[u], (lane % RW) * L, kWave);
            if (lane / RW == u) mine = got;
        }
        return mine;
    }

    // every lane receives, for step u, the value owned by the lane of its row
    __device__ static __forceinline__ void from_row_owner(double mine, int lane, double (&c)[U])
    {
#pragma unroll
        for (int u = 0; u < U; ++u) c[u] = __shfl(mine, u * RW + lane / L, kWave);
    }

    // acc[e] summed over the lanes that hold the same columns, then over the workgroup's wavefronts,
    // written to partials[(col) * grid + block]
    __device__ static __forceinline__ void flush(double (&acc)[E], int64_t d, int lane, int wv, double *lds /*4*E*L*/,
                                                 double *__restrict__ partials)
    {
#pragma unroll
        for (int e = 0; e < E; ++e) {
#pragma unroll
            for (int m = L; m < kWave; m <<= 1) acc[e] += __shfl_xor(acc[e], m, kWave);
        }
        if (lane < L) {
#pragma unroll
            for (int e = 0; e < E; ++e) lds[wv * (E * L) + lane * E + e] = acc[e];
        }
        __syncthreads();
        for (int c = threadIdx.x; c < d; c += kBlock) {
            double s = 0.0;
#pragma unroll
            for (int k = 0; k < kWavesPerBlock; ++k) s += lds[k * (E * L) + c];
            partials[(int64_t)c * gridDim.x + blockIdx.x] = s;
        }
    }
};

struct Shape { int E, L; };

// smallest L in {1,2,4,...,64} with E = ceil(d/L) <= 8; for even d an odd E is rounded up, so that every lane can
// use 16-byte loads (the columns past d are masked: d = 18 runs as 4 lanes x 6 columns, d = 28 as 4 x 8)
inline bool pick_shape(int64_t d, Shape &s)
{
    for (int L = 1; L <= kWave; L *= 2) {
        int64_t E = (d + L - 1) / L;
        if (E <= 8) {
            if (L > 1 && d % 2 == 0 && E % 2 == 1) E += 1;
            s.E = (int)E;
            s.L = L;
            return true;
        }
    }
    return false;
}

constexpr int pick_U(int E, int L) { return (L < 4 ? L : 4); }

}  // namespace tron
