// Device-side helpers: wavefront / workgroup sums and the per-instance loss terms.
#pragma once

#include "common.h"

namespace tron {

// Cross-lane moves through the DPP data path (a few cycles) instead of ds_bpermute (an LDS round trip):
//   0xB1 = quad_perm [1,0,3,2] (lane ^ 1), 0x4E = quad_perm [2,3,0,1] (lane ^ 2),
//   0x141 = row_half_mirror (lane i <-> 7-i inside each group of 8), 0x140 = row_mirror (i <-> 15-i inside 16).
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// Sum over aligned groups of 2 / 4 / 8 / 16 consecutive lanes; every lane of a group receives its total.
__device__ __forceinline__ double sum2(double v) { return v + dpp_move<0xB1>(v); }
__device__ __forceinline__ double sum4(double v) { v = sum2(v); return v + dpp_move<0x4E>(v); }
__device__ __forceinline__ double sum8(double v) { v = sum4(v); return v + dpp_move<0x141>(v); }
__device__ __forceinline__ double sum16(double v) { v = sum8(v); return v + dpp_move<0x140>(v); }

// Sum over the 64 lanes of a wavefront; every lane receives the total.  Fixed order.
__device__ __forceinline__ double wave_sum(double v)
{
    v = sum16(v);
    return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}

// Sum over aligned groups of `g` consecutive lanes (g a power of two <= 64); every lane of a group gets its total.
__device__ __forceinline__ double group_sum(double v, int g)
{
    if (g == 1) return v;
    if (g == 2) return sum2(v);
    if (g == 4) return sum4(v);
    if (g == 8) return sum8(v);
    v = sum16(v);
    if (g == 16) return v;
    if (g == 32) return v + __shfl_xor(v, 16, kWave);
    return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}

// ---- inclusive scans over the 64 lanes of a wavefront, through DPP (no LDS).
// Steps: row_shr 1, 2, 4, 8 inside each row of 16 lanes, then row_bcast:15 into rows 1 and 3 (lane 15 of the row
// before), then row_bcast:31 into rows 2 and 3.  A lane that has no source in a step keeps the identity it passes in.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_int(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xf, false);
    return __hiloint2double(hi, lo);
}

// c := c[0] + ... + c[lane]
__device__ __forceinline__ int wave_scan_add(int c)
{
    c += dpp_int<0x111, 0xf>(c);
    c += dpp_int<0x112, 0xf>(c);
    c += dpp_int<0x114, 0xf>(c);
    c += dpp_int<0x118, 0xf>(c);
    c += dpp_int<0x142, 0xa>(c);
    c += dpp_int<0x143, 0xc>(c);
    return c;
}

// Segmented sum: every lane holds (t, h) = (sum of the open run at its end, whether a run ended inside it).
// Afterwards t = t[lane] + the t of the lanes before it back to, and including, the nearest one with h set, and
// h = whether any lane up to this one had h set.  The operator (ta,ha)+(tb,hb) = (hb ? tb : ta+tb, ha|hb) is
// associative, so the tree order above applies.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void seg_scan_step(double &t, int &h)
{
    // h is 0 or 1: the mask keeps the incoming sum only while no run has ended up to this lane (t + 0.0 is t)
    const int open = h - 1;
    const int lo = dpp_int<CTRL, ROW_MASK>(__double2loint(t)) & open;
    const int hi = dpp_int<CTRL, ROW_MASK>(__double2hiint(t)) & open;
    const int sh = dpp_int<CTRL, ROW_MASK>(h);
    t += __hiloint2double(hi, lo);
    h |= sh;
}

__device__ __forceinline__ void wave_seg_scan(double &t, int &h)
{
    seg_scan_step<0x111, 0xf>(t, h);
    seg_scan_step<0x112, 0xf>(t, h);
    seg_scan_step<0x114, 0xf>(t, h);
    seg_scan_step<0x118, 0xf>(t, h);
    seg_scan_step<0x142, 0xa>(t, h);
    seg_scan_step<0x143, 0xc>(t, h);
}

// value of the lane before (lane 0 receives 0): wave_shr:1
__device__ __forceinline__ double lane_before(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), 0x138, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), 0x138, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ int lane_before(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x138, 0xf, 0xf, false); }

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

// Second reduction stage inside the producing kernel (see Finish in common.h).  Every thread of every workgroup calls it
// after thread 0 has written the workgroup's partial sums (NSLOTS of them, `stride` apart).  The workgroup that draws
// the last ticket adds the partial sums of all workgroups -- in the order and with the arithmetic of k_reduce_final, so
// the result does not depend on which workgroup that is -- writes the scalars and clears the counter for the next
// kernel on the stream.  The counter is the only thing touched atomically; no sum goes through an atomic.
template <int NSLOTS>
__device__ __forceinline__ void finish_partials(const Finish &f, const double *partials, int stride, double *lds)
{
    if (!f.ticket) return;
    __shared__ int is_last;
    if (threadIdx.x == 0) {
        __threadfence();   // the partial sums above are visible device-wide before the ticket is
        is_last = (atomicAdd(f.ticket, 1u) == gridDim.x - 1) ? 1 : 0;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();       // and the other workgroups' partial sums are visible here
    const int count = (int)gridDim.x;
#pragma unroll
    for (int s = 0; s < NSLOTS; ++s) {
        const double *p = partials + (int64_t)s * stride;
        double acc = 0.0;
        for (int b = threadIdx.x; b < count; b += kBlock) acc += __builtin_nontemporal_load(p + b);
        acc = block_sum(acc, lds);
        if (threadIdx.x == 0) {
            f.scal[f.first + s] = acc;
            f.scal_copy[f.first + s] = acc;
        }
    }
    if (threadIdx.x == 0) *f.ticket = 0u;
}

// log(1 + e) for 0 <= e <= 1, as 2 atanh(u) with u = e / (2 + e) <= 1/3: the odd series in u up to u^31 (the first
// term left out is below 2e-17 of the sum).  Within 2 ulp of the exact value (4.2e-16 relative at worst over 2.6M
// arguments e = exp(-t), t in [0, 600], against extended precision on the host; the library's general-argument routine:
// 1.2e-16) at about a third of that routine's instructions -- in the multi-problem logistic function/gradient pass, which
// evaluates it once per row and problem, the general routine alone took a quarter of the time.
__device__ __forceinline__ double log1p_unit(double e)
{
    const double u = e / (2.0 + e), w = u * u;
    double p = 1.0 / 31.0;
    p = fma(p, w, 1.0 / 29.0);
    p = fma(p, w, 1.0 / 27.0);
    p = fma(p, w, 1.0 / 25.0);
    p = fma(p, w, 1.0 / 23.0);
    p = fma(p, w, 1.0 / 21.0);
    p = fma(p, w, 1.0 / 19.0);
    p = fma(p, w, 1.0 / 17.0);
    p = fma(p, w, 1.0 / 15.0);
    p = fma(p, w, 1.0 / 13.0);
    p = fma(p, w, 1.0 / 11.0);
    p = fma(p, w, 1.0 / 9.0);
    p = fma(p, w, 1.0 / 7.0);
    p = fma(p, w, 1.0 / 5.0);
    p = fma(p, w, 1.0 / 3.0);
    p = fma(p, w, 1.0);
    return 2.0 * u * p;
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
        alpha = log1p_unit(e) + ((t >= 0.0) ? 0.0 : -t);
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
