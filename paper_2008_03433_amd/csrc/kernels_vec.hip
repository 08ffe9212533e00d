// Elementwise and reduction kernels over the length-n and length-d vectors: per-instance loss
// terms (Appendix E of the paper), dot products / norms, the conjugate-gradient vector updates
// and the second reduction stage.  All reductions are two-stage: each workgroup writes one partial
// per quantity, a single workgroup then adds the partials in a fixed order (no atomics).
#include "device_util.h"

namespace tron {

// ------------------------------------------------------------------ second stage
// scal[first + s] = sum_{b < count} partials[s*stride + b]; scal is the host's copy (mapped pinned memory), scal_copy the
// device's
__global__ __launch_bounds__(kBlock) void k_reduce_final(const double *__restrict__ partials, int count, int stride,
                                                         double *__restrict__ scal, double *__restrict__ scal_copy, int first)
{
    __shared__ double lds[kWavesPerBlock];
    const int s = blockIdx.x;
    const double *p = partials + (int64_t)s * stride;
    double acc = 0.0;
    for (int b = threadIdx.x; b < count; b += kBlock) acc += p[b];
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        scal[first + s] = acc;
        scal_copy[first + s] = acc;
    }
}

// Automatic rule: only launches of up to kFuseMaxGrid workgroups complete their own reduction.  Every workgroup pays a
// device-wide fence and a ticket (a few microseconds, overlapped only if there are few of them); measured: with 5
// workgroups a solve of the smallest sparse configuration takes 0.42 instead of 0.49 ms, with 47 nothing is gained, with
// 2048 a combine kernel takes 65 instead of 36 us.
constexpr int kFuseMaxGrid = 32;
Finish finish_for(tron_dataset *ds, int first_scalar, int grid)
{
    const bool fuse = ds->ticket && first_scalar >= 0 &&
                      (g_tuning.fuse_reductions > 0 || (g_tuning.fuse_reductions < 0 && grid <= kFuseMaxGrid));
    ds->finish_done = fuse;
    return Finish{fuse ? ds->ticket : nullptr, ds->scal_dev, ds->scal_copy, first_scalar};
}

int reduce_final(tron_dataset *ds, int nslots, int count, int stride, int first_scalar)
{
    if (ds->finish_done) {   // the kernel that produced the partial sums has added them already
        ds->finish_done = false;
        return TRON_OK;
    }
    ProfScope ps(ds, SLOT_REDUCE_FINAL);
    hipLaunchKernelGGL(k_reduce_final, dim3(nslots), dim3(kBlock), 0, ds->stream, ds->partials, count, stride,
                       ds->scal_dev, ds->scal_copy, first_scalar);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

int reduce_cg_regions(tron_dataset *ds, int region, int nregions, int count, int first_scalar)
{
    ProfScope ps(ds, SLOT_REDUCE_FINAL);
    hipLaunchKernelGGL(k_reduce_final, dim3(nregions), dim3(kBlock), 0, ds->stream, ds->cg_partials + (size_t)region * kMaxGrid, count, kMaxGrid,
                       ds->scal_dev, ds->scal_copy, first_scalar);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

int read_scalars(tron_dataset *ds, int count)
{
    (void)count;   // scal_dev is the device address of scal_host: the kernels have written the scalars in place
    TRON_HIP(hipStreamSynchronize(ds->stream));
    return TRON_OK;
}

static inline int vec_grid(int64_t m)
{
    int64_t g = (m + kBlock * 4 - 1) / (kBlock * 4);
    if (g < 1) g = 1;
    if (g > kMaxGrid) g = kMaxGrid;
    return (int)g;
}

// ------------------------------------------------------------------ dots
template <int K>
__global__ __launch_bounds__(kBlock) void k_dots(int64_t m, const double *__restrict__ a0, const double *__restrict__ b0,
                                                 const double *__restrict__ a1, const double *__restrict__ b1,
                                                 const double *__restrict__ a2, const double *__restrict__ b2,
                                                 double *__restrict__ partials, int stride, Finish fin)
{
    __shared__ double lds[kWavesPerBlock];
    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < m; i += (int64_t)gridDim.x * kBlock) {
        s0 += a0[i] * b0[i];
        if (K > 1) s1 += a1[i] * b1[i];
        if (K > 2) s2 += a2[i] * b2[i];
    }
    s0 = block_sum(s0, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = s0;
    if (K > 1) {
        s1 = block_sum(s1, lds);
        if (threadIdx.x == 0) partials[stride + blockIdx.x] = s1;
    }
    if (K > 2) {
        s2 = block_sum(s2, lds);
        if (threadIdx.x == 0) partials[2 * stride + blockIdx.x] = s2;
    }
    finish_partials<K>(fin, partials, stride, lds);
}

int dot_partials(tron_dataset *ds, int64_t m, const double *a0, const double *b0, const double *a1, const double *b1,
                 const double *a2, const double *b2, int first)
{
    ProfScope ps(ds, SLOT_DOT);
    const int g = vec_grid(m);
    const Finish fin = finish_for(ds, first, g);
    if (a2)
        hipLaunchKernelGGL(k_dots<3>, dim3(g), dim3(kBlock), 0, ds->stream, m, a0, b0, a1, b1, a2, b2, ds->partials, kMaxGrid, fin);
    else if (a1)
        hipLaunchKernelGGL(k_dots<2>, dim3(g), dim3(kBlock), 0, ds->stream, m, a0, b0, a1, b1, a2, b2, ds->partials, kMaxGrid, fin);
    else
        hipLaunchKernelGGL(k_dots<1>, dim3(g), dim3(kBlock), 0, ds->stream, m, a0, b0, a1, b1, a2, b2, ds->partials, kMaxGrid, fin);
    TRON_HIP(hipGetLastError());
    return g;
}

// ------------------------------------------------------------------ per-instance loss terms
// z -> zhat, D and the partial loss sums (partial slot 0).
template <int LOSS>
__global__ __launch_bounds__(kBlock) void k_loss_terms(int64_t n, const double *__restrict__ z, const double *__restrict__ y,
                                                       double *__restrict__ zhat, double *__restrict__ D,
                                                       double *__restrict__ partials, Finish fin)
{
    __shared__ double lds[kWavesPerBlock];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        double a, zh, Di;
        loss_terms_dev<LOSS>(z[i], y[i], a, zh, Di);
        zhat[i] = zh;
        D[i] = Di;
        acc += a;
    }
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = acc;
    finish_partials<1>(fin, partials, 0, lds);
}

int loss_terms(tron_dataset *ds, int loss, const double *z, double *zhat, double *D, int first)
{
    ProfScope ps(ds, SLOT_LOSS_TERMS);
    const int g = vec_grid(ds->n);
    const Finish fin = finish_for(ds, first, g);
    if (loss == TRON_LOSS_LR)
        hipLaunchKernelGGL(k_loss_terms<TRON_LOSS_LR>, dim3(g), dim3(kBlock), 0, ds->stream, ds->n, z, ds->y, zhat, D, ds->partials, fin);
    else
        hipLaunchKernelGGL(k_loss_terms<TRON_LOSS_L2SVM>, dim3(g), dim3(kBlock), 0, ds->stream, ds->n, z, ds->y, zhat, D, ds->partials, fin);
    TRON_HIP(hipGetLastError());
    return g;
}

// ------------------------------------------------------------------ conjugate-gradient vector updates
// PRE = preconditioned by the diagonal M (the trust region is then measured in the M-norm): z = r / M takes the
// place of r in the direction, r.z of r.r, and the three dot products that locate the boundary are M-weighted.
// Without PRE the arithmetic is exactly that of plain CG (M is not read).

// s = 0, r = -g, p = r (PRE: p = r / M; partial slot 0 = r.p)
template <bool PRE>
__global__ __launch_bounds__(kBlock) void k_cg_init(int64_t d, const double *__restrict__ g, const double *__restrict__ M,
                                                    double *__restrict__ s, double *__restrict__ r, double *__restrict__ p,
                                                    double *__restrict__ partials, Finish fin, double rr0, double *__restrict__ scal,
                                                    double *__restrict__ scal_copy)
{
    __shared__ double lds[kWavesPerBlock];
    if (rr0 >= 0.0 && blockIdx.x == 0 && threadIdx.x == 0) {
        scal[kScalRR] = rr0;
        scal_copy[kScalRR] = rr0;
        for (int q = 0; q < 2; ++q) {
            scal[kScalFlag + q] = 0.0;
            scal_copy[kScalFlag + q] = 0.0;
        }
    }
    double acc = 0.0;
    for (int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x; j < d; j += (int64_t)gridDim.x * kBlock) {
        const double t = -g[j];
        const double z = PRE ? t / M[j] : t;
        s[j] = 0.0;
        r[j] = t;
        p[j] = z;
        acc += t * z;
    }
    if (PRE) {
        acc = block_sum(acc, lds);
        if (threadIdx.x == 0) partials[blockIdx.x] = acc;
        finish_partials<1>(fin, partials, 0, lds);
    }
}

int cg_init(tron_dataset *ds, const double *g, const double *M, double *s, double *r, double *p, int first, double rr0)
{
    ProfScope ps(ds, SLOT_CG_VEC);
    const int gr = vec_grid(ds->d);
    const Finish fin = finish_for(ds, M ? first : -1, gr);   // without M the kernel produces no sum
    if (M) hipLaunchKernelGGL(k_cg_init<true>, dim3(gr), dim3(kBlock), 0, ds->stream, ds->d, g, M, s, r, p, ds->partials, fin, rr0, ds->scal_dev, ds->scal_copy);
    else hipLaunchKernelGGL(k_cg_init<false>, dim3(gr), dim3(kBlock), 0, ds->stream, ds->d, g, M, s, r, p, ds->partials, fin, rr0, ds->scal_dev, ds->scal_copy);
    TRON_HIP(hipGetLastError());
    return gr;
}

// Whether the CG run had ended before iteration c.it: the iteration before went to the boundary or left
// sqrt(r.r) <= tol (the comparison the host makes).  The same in every thread of the launch.
__device__ __forceinline__ bool cg_run_ended(const CgStepCtl &c, const double *__restrict__ sc)
{
    if (c.it == 0) return false;
    return sc[kScalFlag + ((c.it - 1) & 1)] != 0.0 || sqrt(sc[kScalRR + (c.it & 1)]) <= c.tol;
}

// The step length of a CG iteration from the device copy of the scalars (see CgStepCtl), in the operations and the
// order the host used to take (no contraction into fused multiply-adds), the same in every thread.
__device__ __forceinline__ double cg_step_length(const CgStepCtl &c, const double *__restrict__ sc, double pHp, double pp, double sp, double ss, bool &boundary)
{
    const double rr = sc[kScalRR + (c.it & 1)];
    if (c.it == 0) { pp = rr; sp = 0.0; ss = 0.0; }
    const double alpha = rr / pHp;
    // |s + alpha p|^2 from the three dot products kept alongside the vectors
    const double len2 = __dadd_rn(ss, __dmul_rn(alpha, __dadd_rn(__dmul_rn(2.0, sp), __dmul_rn(alpha, pp))));
    boundary = sqrt(len2) >= c.delta;
    if (!boundary) return alpha;
    const double gap = __dadd_rn(__dmul_rn(c.delta, c.delta), -ss);
    const double rad = sqrt(__dadd_rn(__dmul_rn(sp, sp), __dmul_rn(pp, gap)));
    return (sp >= 0.0) ? gap / __dadd_rn(sp, rad) : __dadd_rn(rad, -sp) / pp;
}

// The sum of `count` <= kCgDirectGrid per-workgroup partial sums with the order and arithmetic of k_reduce_final, formed
// by every wavefront on its own: each lane plays its thread of each of that kernel's wavefronts in turn.  No barrier, no
// LDS, and the loads of several such sums can be in flight together.
static_assert(kCgDirectGrid <= 2 * kBlock, "two partial sums per thread of the second-stage kernel at most");
__device__ __forceinline__ double sum_of_partials(const double *__restrict__ p, int count)
{
    const int lane = threadIdx.x & (kWave - 1);
    double a[kWavesPerBlock];
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        const int b = w * kWave + lane;
        const double x = p[b < count ? b : 0], y = p[b + kBlock < count ? b + kBlock : 0];
        a[w] = (0.0 + (b < count ? x : 0.0)) + (b + kBlock < count ? y : 0.0);
    }
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) t += wave_sum(a[w]);
    return t;
}

// s += a p;  r -= a Hp with a = the step length above;  region CGP_RR = partial sums of r.r (PRE: r.(r / M));  scalar 4 = a,
// the iteration's flag slot = whether the step went to the boundary.  Nothing at all if the run had ended.
template <bool PRE>
__global__ __launch_bounds__(kBlock) void k_cg_step(int64_t d, CgStepCtl ctl, int n_dir, int n_php, const double *__restrict__ php, const double *__restrict__ sc, const double *__restrict__ p,
                                                    const double *__restrict__ Hp, const double *__restrict__ M,
                                                    double *__restrict__ s, double *__restrict__ r, double *__restrict__ cgp,
                                                    double *__restrict__ scal, double *__restrict__ scal_copy)
{
    __shared__ double lds[kWavesPerBlock];
    if (cg_run_ended(ctl, sc)) return;
    double pp = 0.0, sp = 0.0, ss = 0.0;
    if (ctl.it > 0 && n_dir > 0) {   // what the direction kernel before left, one partial sum per workgroup
        pp = sum_of_partials(cgp + (size_t)CGP_PP * kMaxGrid, n_dir);
        sp = sum_of_partials(cgp + (size_t)CGP_SP * kMaxGrid, n_dir);
        ss = sum_of_partials(cgp + (size_t)CGP_SS * kMaxGrid, n_dir);
    } else if (ctl.it > 0) {   // added up by a launch in between
        pp = sc[1];
        sp = sc[2];
        ss = sc[3];
    }
    const double pHp = n_php > 0 ? sum_of_partials(php, n_php) : sc[0];   // left by the product's last kernel, or added up by a launch
    bool boundary;
    const double alpha = cg_step_length(ctl, sc, pHp, pp, sp, ss, boundary);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        scal[4] = alpha;
        scal[kScalFlag + (ctl.it & 1)] = boundary ? 1.0 : 0.0;
        scal_copy[kScalFlag + (ctl.it & 1)] = boundary ? 1.0 : 0.0;   // read by the kernels after this one only
    }
    double acc = 0.0;
    for (int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x; j < d; j += (int64_t)gridDim.x * kBlock) {
        s[j] = fma(alpha, p[j], s[j]);
        const double rj = fma(-alpha, Hp[j], r[j]);
        r[j] = rj;
        acc += rj * (PRE ? rj / M[j] : rj);
    }
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) cgp[(size_t)CGP_RR * kMaxGrid + blockIdx.x] = acc;
}

int vec_workgroups(int64_t m) { return vec_grid(m); }

// The step and direction kernels run with at most kCgDirectGrid workgroups, so that each can add up the other's partial
// sums itself whatever d is (longer loops per thread instead of more workgroups).
static inline int cg_grid(int64_t m)
{
    const int g = vec_grid(m);
    return g < kCgDirectGrid ? g : kCgDirectGrid;
}

int cg_step(tron_dataset *ds, const CgStepCtl &ctl, int n_dir, int n_php, const double *p, const double *Hp, const double *M, double *s, double *r)
{
    ProfScope ps(ds, SLOT_CG_VEC);
    const int g = cg_grid(ds->d);
    if (M) hipLaunchKernelGGL(k_cg_step<true>, dim3(g), dim3(kBlock), 0, ds->stream, ds->d, ctl, n_dir, n_php, ds->partials, ds->scal_copy, p, Hp, M, s, r, ds->cg_partials, ds->scal_dev, ds->scal_copy);
    else hipLaunchKernelGGL(k_cg_step<false>, dim3(g), dim3(kBlock), 0, ds->stream, ds->d, ctl, n_dir, n_php, ds->partials, ds->scal_copy, p, Hp, M, s, r, ds->cg_partials, ds->scal_dev, ds->scal_copy);
    TRON_HIP(hipGetLastError());
    return g;
}

// p = r + beta p (PRE: r / M + beta p) with beta = (the new r.r) / (the old r.r): the new one is added up here from the
// step kernel's partial sums and left in its scalar slot for the host and the next step; regions CGP_PP, CGP_SP, CGP_SS =
// partial sums of p.p, s.p, s.s (PRE: M-weighted).  Nothing at all if the run had ended before this iteration; only the
// new r.r if it ends with it.
template <bool PRE>
__global__ __launch_bounds__(kBlock) void k_cg_dir(int64_t d, CgStepCtl ctl, int n_step, const double *__restrict__ sc, const double *__restrict__ r,
                                                   const double *__restrict__ s, const double *__restrict__ M,
                                                   double *__restrict__ p, double *__restrict__ cgp, double *__restrict__ scal,
                                                   double *__restrict__ scal_copy)
{
    __shared__ double lds[kWavesPerBlock];
    if (cg_run_ended(ctl, sc)) return;
    const double rr_old = sc[kScalRR + (ctl.it & 1)];
    const double rr_new = n_step > 0 ? sum_of_partials(cgp + (size_t)CGP_RR * kMaxGrid, n_step) : sc[kScalRR + ((ctl.it + 1) & 1)];
    if (n_step > 0 && blockIdx.x == 0 && threadIdx.x == 0) {   // read by the kernels after this one only (this one reads the other slot)
        scal[kScalRR + ((ctl.it + 1) & 1)] = rr_new;
        scal_copy[kScalRR + ((ctl.it + 1) & 1)] = rr_new;
    }
    if (sc[kScalFlag + (ctl.it & 1)] != 0.0 || sqrt(rr_new) <= ctl.tol) return;
    const double beta = rr_new / rr_old;
    double pp = 0.0, sp = 0.0, ss = 0.0;
    for (int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x; j < d; j += (int64_t)gridDim.x * kBlock) {
        const double m = PRE ? M[j] : 1.0;
        const double pj = fma(beta, p[j], PRE ? r[j] / m : r[j]);
        const double sj = s[j];
        p[j] = pj;
        if (PRE) {
            pp += m * pj * pj;
            sp += m * sj * pj;
            ss += m * sj * sj;
        } else {
            pp += pj * pj;
            sp += sj * pj;
            ss += sj * sj;
        }
    }
    pp = block_sum(pp, lds);
    if (threadIdx.x == 0) cgp[(size_t)CGP_PP * kMaxGrid + blockIdx.x] = pp;
    sp = block_sum(sp, lds);
    if (threadIdx.x == 0) cgp[(size_t)CGP_SP * kMaxGrid + blockIdx.x] = sp;
    ss = block_sum(ss, lds);
    if (threadIdx.x == 0) cgp[(size_t)CGP_SS * kMaxGrid + blockIdx.x] = ss;
}

int cg_dir(tron_dataset *ds, const CgStepCtl &ctl, int n_step, const double *r, const double *s, const double *M, double *p)
{
    ProfScope ps(ds, SLOT_CG_VEC);
    const int g = cg_grid(ds->d);
    if (M) hipLaunchKernelGGL(k_cg_dir<true>, dim3(g), dim3(kBlock), 0, ds->stream, ds->d, ctl, n_step, ds->scal_copy, r, s, M, p, ds->cg_partials, ds->scal_dev, ds->scal_copy);
    else hipLaunchKernelGGL(k_cg_dir<false>, dim3(g), dim3(kBlock), 0, ds->stream, ds->d, ctl, n_step, ds->scal_copy, r, s, M, p, ds->cg_partials, ds->scal_dev, ds->scal_copy);
    TRON_HIP(hipGetLastError());
    return g;
}

// wnew = w + s;  partial slots: 0 = g.s, 1 = s.r, 2 = s.s (PRE: s.Ms)
template <bool PRE>
__global__ __launch_bounds__(kBlock) void k_trial_point(int64_t d, const double *__restrict__ w, const double *__restrict__ s,
                                                        const double *__restrict__ g, const double *__restrict__ r,
                                                        const double *__restrict__ M, double *__restrict__ wnew,
                                                        double *__restrict__ partials, int stride, Finish fin)
{
    __shared__ double lds[kWavesPerBlock];
    double gs = 0.0, sr = 0.0, ss = 0.0;
    for (int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x; j < d; j += (int64_t)gridDim.x * kBlock) {
        const double sj = s[j];
        wnew[j] = w[j] + sj;
        gs += g[j] * sj;
        sr += sj * r[j];
        ss += PRE ? M[j] * sj * sj : sj * sj;
    }
    gs = block_sum(gs, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = gs;
    sr = block_sum(sr, lds);
    if (threadIdx.x == 0) partials[stride + blockIdx.x] = sr;
    ss = block_sum(ss, lds);
    if (threadIdx.x == 0) partials[2 * stride + blockIdx.x] = ss;
    finish_partials<3>(fin, partials, stride, lds);
}

int trial_point(tron_dataset *ds, const double *w, const double *s, const double *g, const double *r, const double *M,
                double *wnew, int first)
{
    ProfScope ps(ds, SLOT_CG_VEC);
    const int gr = vec_grid(ds->d);
    const Finish fin = finish_for(ds, first, gr);
    if (M) hipLaunchKernelGGL(k_trial_point<true>, dim3(gr), dim3(kBlock), 0, ds->stream, ds->d, w, s, g, r, M, wnew, ds->partials, kMaxGrid, fin);
    else hipLaunchKernelGGL(k_trial_point<false>, dim3(gr), dim3(kBlock), 0, ds->stream, ds->d, w, s, g, r, M, wnew, ds->partials, kMaxGrid, fin);
    TRON_HIP(hipGetLastError());
    return gr;
}

// ------------------------------------------------------------------ streaming-read probe
// Every wavefront reads blocks of 12 KiB of consecutive bytes -- twelve 16-byte loads per lane in flight, each instruction
// covering 1 KiB -- the access pattern of the dense kernels (block w, w + W, ... for wavefront w of W).
__global__ __launch_bounds__(kBlock) void k_probe_sum(const double2 *__restrict__ src, int64_t count2, double *__restrict__ out)
{
    __shared__ double lds[kWavesPerBlock];
    constexpr int kInFlight = 12;
    constexpr int64_t kPerBlock = (int64_t)kInFlight * kWave;   // double2 elements per 12 KiB block
    double a = 0.0, b = 0.0;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    const int64_t nblocks = count2 / kPerBlock;
    for (int64_t blk = wave; blk < nblocks; blk += nwaves) {
        const double2 *p = src + blk * kPerBlock + lane;
        double2 x[kInFlight];
#pragma unroll
        for (int m = 0; m < kInFlight; ++m) x[m] = p[m * kWave];
#pragma unroll
        for (int m = 0; m < kInFlight; ++m) {
            a += x[m].x;
            b += x[m].y;
        }
    }
    for (int64_t i = nblocks * kPerBlock + (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count2; i += (int64_t)gridDim.x * kBlock) {
        const double2 x0 = src[i];
        a += x0.x;
        b += x0.y;
    }
    a = block_sum(a + b, lds);
    if (threadIdx.x == 0) out[blockIdx.x] = a;
}

__global__ __launch_bounds__(kBlock) void k_probe_copy(double2 *__restrict__ dst, const double2 *__restrict__ src, int64_t count2)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count2; i += stride) dst[i] = src[i];
}

int probe_copy(double *dst, const double *src, int64_t count, int reps, hipStream_t st, double *ms)
{
    if (!src || !dst || count < 2 || reps < 1 || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15)) {
        set_error("tron_probe_copy_bandwidth: need 16-byte aligned device pointers, count >= 2, reps >= 1");
        return TRON_EINVAL;
    }
    hipEvent_t e0, e1;
    TRON_HIP(hipEventCreate(&e0));
    TRON_HIP(hipEventCreate(&e1));
    hipLaunchKernelGGL(k_probe_copy, dim3(kMaxGrid), dim3(kBlock), 0, st, reinterpret_cast<double2 *>(dst),
                       reinterpret_cast<const double2 *>(src), count / 2);
    TRON_HIP(hipEventRecord(e0, st));
    for (int r = 0; r < reps; ++r)
        hipLaunchKernelGGL(k_probe_copy, dim3(kMaxGrid), dim3(kBlock), 0, st, reinterpret_cast<double2 *>(dst),
                           reinterpret_cast<const double2 *>(src), count / 2);
    TRON_HIP(hipEventRecord(e1, st));
    TRON_HIP(hipEventSynchronize(e1));
    float t = 0.f;
    TRON_HIP(hipEventElapsedTime(&t, e0, e1));
    if (ms) *ms = (double)t / reps;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    return TRON_OK;
}

int probe_read(const double *src, int64_t count, int reps, hipStream_t st, double *ms, double *checksum)
{
    if (!src || count < 2 || reps < 1 || (reinterpret_cast<uintptr_t>(src) & 15)) {
        set_error("tron_probe_read_bandwidth: need a 16-byte aligned device pointer, count >= 2, reps >= 1");
        return TRON_EINVAL;
    }
    const int grid = kMaxGrid;
    double *out = nullptr;
    TRON_HIP(hipMalloc(&out, sizeof(double) * grid));
    hipEvent_t e0, e1;
    TRON_HIP(hipEventCreate(&e0));
    TRON_HIP(hipEventCreate(&e1));
    hipLaunchKernelGGL(k_probe_sum, dim3(grid), dim3(kBlock), 0, st, reinterpret_cast<const double2 *>(src), count / 2, out);
    TRON_HIP(hipEventRecord(e0, st));
    for (int r = 0; r < reps; ++r)
        hipLaunchKernelGGL(k_probe_sum, dim3(grid), dim3(kBlock), 0, st, reinterpret_cast<const double2 *>(src), count / 2, out);
    TRON_HIP(hipEventRecord(e1, st));
    TRON_HIP(hipEventSynchronize(e1));
    float t = 0.f;
    TRON_HIP(hipEventElapsedTime(&t, e0, e1));
    std::vector<double> h(grid);
    TRON_HIP(hipMemcpy(h.data(), out, sizeof(double) * grid, hipMemcpyDeviceToHost));
    double cs = 0.0;
    for (double x : h) cs += x;
    if (ms) *ms = (double)t / reps;
    if (checksum) *checksum = cs;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    hipFree(out);
    return TRON_OK;
}

}  // namespace tron
