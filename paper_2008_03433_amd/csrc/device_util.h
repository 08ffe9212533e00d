// Device-side helpers: wavefront / workgroup sums and the per-instance loss terms.
#pragma once

#include "common.h"

namespace tron {

// Sum over the 64 lanes of a wavefront; every lane receives the total.  Fixed butterfly order.
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// Sum over aligned groups of `g` consecutive lanes (g a power of two <= 64).
__device__ __forceinline__ double group_sum(double v, int g)
{
    for (int m = g >> 1; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// Sum over the workgroup (kBlock threads); valid in thread 0.  `lds` holds kWavesPerBlock doubles
// and may be reused right after the call returns (the trailing barrier orders it).
__device__ __forceinline__ double block_sum(double v, double *lds)
{
    v = wave_sum(v);
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    if (lane == 0) lds[wv] = v;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) t += lds[k];
    }
    __syncthreads();
    return t;
}

// Per-instance terms at margin z with label y (Table 1 and Appendix E of the paper):
//   logistic:  t = y z, h = 1/(1+exp(-t));  alpha = log(1+exp(-t)),  zhat = (h-1) y,  D = h (1-h)
//   L2-SVM:    m = 1 - y z;  active iff m > 0;  alpha = max(0,m)^2,  zhat = 2 (z-y) [active],  D = 2 [active]
// The exponential is only taken of a non-positive argument, and 1-h is formed without cancellation.
template <int LOSS>
__device__ __forceinline__ void loss_terms_dev(double z, double y, double &alpha, double &zhat, double &D)
{
    if (LOSS == TRON_LOSS_LR) {
        const double t = y * z;
        const double e = exp(-fabs(t));
        const double inv = 1.0 / (1.0 + e);
        const double big = inv, small = e * inv;   // h and 1-h in some order
        const double omh = (t >= 0.0) ? small : big;
        const double h = (t >= 0.0) ? big : small;
        alpha = log1p(e) + ((t >= 0.0) ? 0.0 : -t);
        zhat = -omh * y;
        D = h * omh;
    } else {
        const double m = 1.0 - y * z;
        const bool act = m > 0.0;
        alpha = act ? m * m : 0.0;
        zhat = act ? 2.0 * (z - y) : 0.0;
        D = act ? 2.0 : 0.0;
    }
}

}  // namespace tron
