// Host driver: function / gradient / Hessian-vector evaluation on top of the kernels, the
// conjugate-gradient inner solver and the trust-region outer loop (Algorithm 1 of the paper).
// All vectors stay in device memory; per CG iteration the host reads back a handful of scalars.
#include <cmath>
#include <cstring>

#include "common.h"

namespace tron {

// f(w) for the sparse layout: z = X w, loss terms (zhat, D into Dbuf[Dslot]), f = 1/2 w.w + C sum loss.
// The dense layout computes the same together with the gradient sums in one fused pass.
int fun_enqueue(tron_dataset *ds, int loss, const double *w, int Dslot)   // scalar 0 = sum of the loss terms, scalar 1 = w.w
{
    // with unit plans zhat is stored already multiplied by the instances' values, as the transposed plan gathers it
    const int gl = spmv_loss(ds, ds->fwd, SLOT_SPMV_FWD, loss, w, ds->z, ds->zhat, ds->Dbuf[Dslot], ds->bwd.col_scale, 0);
    TRON_TRY(gl);
    TRON_TRY(reduce_final(ds, 1, gl, 0, 0));
    const int gw = dot_partials(ds, ds->d, w, w, nullptr, nullptr, nullptr, nullptr, 1);
    TRON_TRY(gw);
    TRON_TRY(reduce_final(ds, 1, gw, 0, 1));
    return TRON_OK;
}

int fun_eval(tron_dataset *ds, int loss, double C, const double *w, int Dslot, double *f_out)
{
    TRON_TRY(fun_enqueue(ds, loss, w, Dslot));
    TRON_TRY(read_scalars(ds, 2));
    *f_out = 0.5 * ds->scal_host[1] + C * ds->scal_host[0];
    return TRON_OK;
}

// g = w + C X^T zhat (zhat from the preceding fun_enqueue); scalar `scalar` = g.g
int grad_enqueue(tron_dataset *ds, double C, const double *w, double *g, int scalar)
{
    const int gg = spmv_axpy(ds, ds->bwd, SLOT_SPMV_BWD, ds->zhat, w, C, true, g, false, ds->bwd.col_scale != nullptr, scalar);
    TRON_TRY(gg);
    TRON_TRY(reduce_final(ds, 1, gg, 0, scalar));
    return TRON_OK;
}

int grad_eval(tron_dataset *ds, double C, const double *w, double *g, double *gnorm_out)
{
    TRON_TRY(grad_enqueue(ds, C, w, g, 0));
    TRON_TRY(read_scalars(ds, 1));
    *gnorm_out = std::sqrt(ds->scal_host[0]);
    return TRON_OK;
}

// Hv = v + C X^T (D (X v)) with D = Dbuf[Dcur]; scal_dev[0] = v.Hv.  Enqueue only.
// vhv_partials not null: a caller whose next kernel can add up the per-workgroup partial sums of v.Hv itself (they lie at
// the start of ds->partials); where there are few enough of them their number comes back there and scalar 0 is not
// formed, otherwise 0 comes back and scalar 0 is.
int hv_enqueue(tron_dataset *ds, double C, const double *v, double *Hv, int *vhv_partials)
{
    if (vhv_partials) *vhv_partials = 0;
    if (ds->dense) return dense_hv(ds, C, ds->Dcur, v, Hv);
    const double *D = ds->Dbuf[ds->Dcur];
    TRON_TRY(spmv_scale(ds, ds->fwd, SLOT_SPMV_FWD, v, D, ds->z, ds->bwd.col_scale));   // a1 = D (X v)
    const bool direct = vhv_partials && vec_workgroups(ds->d) <= kCgDirectGrid;
    const int g = spmv_axpy(ds, ds->bwd, SLOT_SPMV_BWD, ds->z, v, C, false, Hv, false, ds->bwd.col_scale != nullptr, direct ? -1 : 0);  // Hv = v + C X^T a1
    TRON_TRY(g);
    if (direct && g <= kCgDirectGrid) {
        *vhv_partials = g;
        return TRON_OK;
    }
    TRON_TRY(reduce_final(ds, 1, g, 0, 0));
    return TRON_OK;
}

// out = 1 + C sum_i D_i x_ij^2  (diagonal of the Hessian of Appendix B when C is the solver's C)
int hess_diag_enqueue(tron_dataset *ds, double C, int Dslot, double *out)
{
    if (ds->dense) return dense_hess_diag(ds, C, Dslot, out);
    const int g = spmv_axpy(ds, ds->bwd, SLOT_SPMV_BWD, ds->Dbuf[Dslot], nullptr, C, false, out, true);
    return g < 0 ? g : TRON_OK;
}

namespace {

enum { V_W = 0, V_WNEW, V_G, V_GNEW, V_S, V_R, V_P, V_HP, V_M, V_COUNT };

int ensure_solver_vectors(tron_dataset *ds, bool precond)
{
    for (int k = 0; k < V_COUNT; ++k)
        if (!ds->sv[k] && (k != V_M || precond)) TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->sv[k]), sizeof(double) * ds->d));
    if (!ds->cg_partials) TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->cg_partials), sizeof(double) * kCgRegions * kMaxGrid));
    return TRON_OK;
}

// Scalar slots of the outer loop, apart from 0..3 of the evaluation: what one wait of the host brings back together.
constexpr int kScalGG = 2;      // g.g of the sparse gradient (the dense pass leaves it there as well)
constexpr int kScalTrial = 10;  // g.s, s.r, s.s of the trial point
constexpr int kScalW0 = 13;     // w0.w0

// Whether a product with X is cheap enough to be spent on a guess (kernels enqueued before the host knows that their
// result is wanted), as against one idle gap of the device per wait of the host.
bool products_cheap(const tron_dataset *ds)
{
    const double hv_bytes = ds->dense ? 8.0 * (double)ds->n * (double)ds->d : 24.0 * (double)ds->fwd.nnz;
    return hv_bytes <= 64e6;
}

// f at w, D into Dbuf[Dslot], and -- dense always, sparse if with_grad -- the gradient into gout.  Enqueue only.
int eval_enqueue(tron_dataset *ds, const tron_params &P, const double *w, int Dslot, double *gout, bool with_grad)
{
    if (ds->dense) return dense_fun_grad(ds, P.loss, P.C, w, Dslot, gout);
    TRON_TRY(fun_enqueue(ds, P.loss, w, Dslot));
    if (with_grad) TRON_TRY(grad_enqueue(ds, P.C, w, gout, kScalGG));
    return TRON_OK;
}

// What eval_enqueue's kernels left, after a wait; *gnorm only where the gradient was formed.
void eval_result(tron_dataset *ds, const tron_params &P, int Dslot, bool with_grad, double *f, double *gnorm)
{
    *f = 0.5 * ds->scal_host[1] + P.C * ds->scal_host[0];
    if (ds->dense) {
        ds->active_frac[Dslot] = ds->scal_host[3] / (double)ds->n;
        ds->active_count[Dslot] = (int64_t)ds->scal_host[3];
    }
    if (ds->dense || with_grad) *gnorm = std::sqrt(ds->scal_host[kScalGG]);
}

// Steihaug-Toint truncated CG on q(s) = g.s + 1/2 s.H s inside |s| <= delta.
//   s = 0, r = p = -g;  loop: stop when |r| <= xi |g|;  alpha = r.r / p.Hp;  if |s + alpha p| >= delta go to
//   the boundary along p and stop;  s += alpha p, r -= alpha Hp, beta = r'.r'/r.r, p = r + beta p.
// With a diagonal preconditioner M (not null): z = r / M replaces r in p and in the dot products r.r, and the lengths
// are M-norms (the iteration is plain CG in the variables M^(1/2) s); gscaled = sqrt(g.M^-1 g) takes the place of |g|.
// One wait per iteration: the step kernel forms alpha (or the step to the boundary) from the scalars the device keeps,
// the direction kernel forms beta, and the host reads the new r.r and the boundary flag of iteration k once its kernels
// have run.  Where a product is cheap the kernels of iteration k + 1 are enqueued before that wait, so the device never
// idles while the host decides; if iteration k turns out to be the last, those kernels find that out by themselves and
// leave s and r alone (see CgStepCtl) -- one product computed for nothing per run, against one idle gap per iteration.
int cg_solve(tron_dataset *ds, const tron_params &P, const double *M, double delta, double gscaled, int *n_hv, int *on_boundary)
{
    double *g = ds->sv[V_G], *s = ds->sv[V_S], *r = ds->sv[V_R], *p = ds->sv[V_P], *Hp = ds->sv[V_HP];
    const double rr0 = gscaled * gscaled;   // p = z = -g / M at the start: p.Mp = r.z
    const double tol = P.cg_xi * gscaled;
    *on_boundary = 0;
    *n_hv = 0;
    for (hipEvent_t &e : ds->cg_event)
        if (!e) TRON_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    TRON_TRY(cg_init(ds, g, M, s, r, p, -1, rr0));
    if (std::sqrt(rr0) <= tol) return TRON_OK;
    const bool ahead = g_tuning.cg_speculate > 0 || (g_tuning.cg_speculate < 0 && products_cheap(ds));
    int n_dir = 0;   // workgroups of the direction kernel enqueued last
    auto enqueue = [&](int it) -> int {
        int n_php = 0;   // per-workgroup partial sums of p.Hp left for the step kernel (0: the sum is in scalar 0)
        TRON_TRY(hv_enqueue(ds, P.C, p, Hp, &n_php));
        const CgStepCtl ctl{tol, delta, it};
        const int g1 = cg_step(ds, ctl, n_dir, n_php, p, Hp, M, s, r);
        TRON_TRY(g1);
        const bool direct = g1 <= kCgDirectGrid;   // the consumer adds up the partial sums itself
        const bool last = it + 1 >= P.max_cg;      // the last iteration allowed: no direction after it
        if (!direct || last) TRON_TRY(reduce_cg_regions(ds, CGP_RR, 1, g1, kScalRR + ((it + 1) & 1)));
        if (!last) {
            const int g2 = cg_dir(ds, ctl, direct ? g1 : 0, r, s, M, p);
            TRON_TRY(g2);
            if (!direct) TRON_TRY(reduce_cg_regions(ds, CGP_PP, 3, g2, 1));
            n_dir = direct ? g2 : 0;
        }
        TRON_HIP(hipEventRecord(ds->cg_event[it & 1], ds->stream));
        return TRON_OK;
    };
    TRON_TRY(enqueue(0));
    for (int it = 0;; ++it) {
        const bool more = it + 1 < P.max_cg;
        if (ahead && more) TRON_TRY(enqueue(it + 1));
        TRON_HIP(hipEventSynchronize(ds->cg_event[it & 1]));
        *n_hv = it + 1;
        if (ds->scal_host[kScalFlag + (it & 1)] != 0.0) {
            *on_boundary = 1;
            break;
        }
        const double rr = ds->scal_host[kScalRR + ((it + 1) & 1)];
        if (!more || std::sqrt(rr) <= tol) break;
        if (!ahead) TRON_TRY(enqueue(it + 1));
    }
    return TRON_OK;
}

// M = (1 - blend) I + blend diag(H) at the point whose D is in Dbuf[Dslot], and sqrt(g.M^-1 g)
int build_preconditioner(tron_dataset *ds, const tron_params &P, int Dslot, const double *g, double *M, double *gscaled)
{
    TRON_TRY(hess_diag_enqueue(ds, P.precond_blend * P.C, Dslot, M));   // 1 + blend C sum D x^2
    // g.(g / M) with the CG start-up kernel (s, r, p are scratch here: the inner solver initialises them again)
    const int gr = cg_init(ds, g, M, ds->sv[V_S], ds->sv[V_R], ds->sv[V_P], 0);
    TRON_TRY(gr);
    TRON_TRY(reduce_final(ds, 1, gr, 0, 0));
    TRON_TRY(read_scalars(ds, 1));
    *gscaled = std::sqrt(ds->scal_host[0]);
    return TRON_OK;
}

}  // namespace
}  // namespace tron

using namespace tron;

extern "C" int tron_solve(tron_dataset *ds, const tron_params *params, double *w_dev, tron_result *res)
{
    if (!ds || !params || !w_dev || !res) { set_error("tron_solve: null argument"); return TRON_EINVAL; }
    const tron_params P = *params;
    if ((P.loss != TRON_LOSS_LR && P.loss != TRON_LOSS_L2SVM) || !(P.C > 0.0) || !std::isfinite(P.C) || !(P.eps > 0.0) ||
        P.max_outer < 1 || P.max_cg < 1 || !(P.cg_xi > 0.0) || !(P.cg_xi < 1.0) || !(P.precond_blend >= 0.0) ||
        !(P.precond_blend <= 1.0) || res->trace_cap < 0 || (res->trace_cap > 0 && !res->trace)) {
        set_error("tron_solve: bad parameter (loss, C > 0, eps > 0, max_outer >= 1, max_cg >= 1, 0 < cg_xi < 1, "
                  "0 <= precond_blend <= 1, trace)");
        return TRON_EINVAL;
    }
    // Dense matrices with d <= 32: the solve can be driven from the device (batch.hip), which saves the host's waits for
    // scalars inside every iteration.  Measured: 0.31 ms against 0.40 ms on the 1M x 24 L2-SVM configuration; no gain
    // for the logistic loss (its multi-problem pass is slower than the single-problem kernels) or for large matrices
    // (there the waits are small next to the passes).  So by default: the L2-SVM up to 1 GB.
    if (ds->dense && ds->d <= TRON_BATCH_MAX_D && P.precond_blend == 0.0 && g_tuning.dense_device_driver != 0) {
        const double bytes = (double)ds->n * (double)ds->d * 8.0;
        if (g_tuning.dense_device_driver > 0 || (P.loss == TRON_LOSS_L2SVM && bytes <= 1e9)) return dense_device_solve(ds, P, w_dev, res);
    }
    const double eta0 = 1e-4, eta1 = 0.25, eta2 = 0.75, sig2 = 0.5, sig3 = 4.0;
    tron_trace_rec *trace = res->trace;
    const int trace_cap = res->trace_cap;
    res->f = res->gnorm = res->gnorm0 = 0.0;
    res->outer_iters = res->cg_iters_total = res->n_fun = res->n_grad = res->n_hv = res->converged = 0;
    res->trace_len = 0;

    const bool precond = P.precond_blend > 0.0;
    TRON_TRY(ensure_solver_vectors(ds, precond));
    double *M = precond ? ds->sv[V_M] : nullptr;
    const size_t dbytes = sizeof(double) * ds->d;
    double *&w = ds->sv[V_W], *&wnew = ds->sv[V_WNEW], *&g = ds->sv[V_G], *&gnew = ds->sv[V_GNEW];
    double *s = ds->sv[V_S], *r = ds->sv[V_R];
    TRON_HIP(hipMemcpyAsync(w, w_dev, dbytes, hipMemcpyDeviceToDevice, ds->stream));

    // f and the gradient at w0, and whether w0 = 0, behind one wait
    ds->Dcur = 0;
    ds->have_D = false;
    double f, gnorm = 0.0;
    {
        const int gz = dot_partials(ds, ds->d, w, w, nullptr, nullptr, nullptr, nullptr, kScalW0);
        TRON_TRY(gz);
        TRON_TRY(reduce_final(ds, 1, gz, 0, kScalW0));
    }
    TRON_TRY(eval_enqueue(ds, P, w, ds->Dcur, g, true));
    TRON_TRY(read_scalars(ds, kScalars));
    eval_result(ds, P, ds->Dcur, true, &f, &gnorm);
    ds->have_D = true;
    res->n_fun++;
    res->n_grad++;
    // |grad f(0)|: the reference of the stopping test.  When w0 = 0 it is the first gradient itself; otherwise one more
    // evaluation, whose D goes to the buffer of the trial points.
    if (ds->scal_host[kScalW0] != 0.0) {
        double f0, gn0 = 0.0;
        TRON_HIP(hipMemsetAsync(wnew, 0, dbytes, ds->stream));
        TRON_TRY(eval_enqueue(ds, P, wnew, 1 - ds->Dcur, gnew, true));
        TRON_TRY(read_scalars(ds, kScalars));
        eval_result(ds, P, 1 - ds->Dcur, true, &f0, &gn0);
        res->gnorm0 = gn0;
        res->n_fun++;
        res->n_grad++;
    }
    // L2-SVM with a small active set (a warm start far along): Hessian-vector products over a compacted copy of the active rows
    if (ds->dense && dense_compact_wanted(ds, ds->Dcur, g_tuning.dense_compact > 0 ? 0 : P.max_cg)) TRON_TRY(dense_compact_build(ds, ds->Dcur));
    if (res->gnorm0 == 0.0) res->gnorm0 = gnorm;
    // gscaled: the length of the gradient the inner solver measures its residual against (|g|, or sqrt(g.M^-1 g))
    double gscaled = gnorm;
    if (precond) TRON_TRY(build_preconditioner(ds, P, ds->Dcur, g, M, &gscaled));
    double delta = gscaled;
    int status = TRON_EMAXITER;
    if (gnorm <= P.eps * res->gnorm0) { status = TRON_OK; res->converged = 1; }

    for (int k = 1; status == TRON_EMAXITER && k <= P.max_outer; ++k) {
        int ncg = 0, onb = 0;
        TRON_TRY(cg_solve(ds, P, M, delta, gscaled, &ncg, &onb));
        res->n_hv += ncg;
        res->cg_iters_total += ncg;
        // The trial point, the model reduction  pred = -q(s) = -1/2 (g.s - s.r)  and f at the trial point behind one wait.
        // Where products are cheap the sparse gradient at the trial point is formed on the guess that the step will be
        // accepted (a rejected step leaves it unused; n_grad counts the gradients of accepted steps either way).
        const int gt = trial_point(ds, w, s, g, r, M, wnew, kScalTrial);
        TRON_TRY(gt);
        TRON_TRY(reduce_final(ds, 3, gt, kMaxGrid, kScalTrial));
        const int trial_slot = 1 - ds->Dcur;   // D of the trial point goes to the other buffer
        const bool grad_ahead = !ds->dense && g_tuning.cg_speculate != 0 && (g_tuning.cg_speculate > 0 || products_cheap(ds));
        TRON_TRY(eval_enqueue(ds, P, wnew, trial_slot, gnew, grad_ahead));
        TRON_TRY(read_scalars(ds, kScalars));
        const double gs = ds->scal_host[kScalTrial], sr = ds->scal_host[kScalTrial + 1];
        const double snorm = std::sqrt(ds->scal_host[kScalTrial + 2]);
        const double pred = -0.5 * (gs - sr);
        double fnew, gnorm_new = 0.0;
        eval_result(ds, P, trial_slot, grad_ahead, &fnew, &gnorm_new);
        res->n_fun++;
        const double ared = f - fnew;
        const bool noise = std::fabs(ared) <= 1e-12 * std::fabs(f) && pred <= 1e-12 * std::fabs(f);
        const double sigma = noise ? 1.0 : ared / pred;
        const double gnorm_before = gnorm;
        if (sigma < eta1) delta = sig2 * std::fmin(snorm, delta);
        else if (sigma < eta2) { /* unchanged */ }
        else delta = std::fmin(sig3 * delta, std::fmax(delta, sig3 * snorm));
        int accepted = 0;
        if (sigma > eta0) {
            accepted = 1;
            if (!ds->dense && !grad_ahead) TRON_TRY(grad_eval(ds, P.C, wnew, gnew, &gnorm_new));
            std::swap(w, wnew);
            std::swap(g, gnew);
            ds->Dcur = trial_slot;   // the Hessian now uses D at the accepted point
            f = fnew;
            gnorm = gnorm_new;
            gscaled = gnorm;
            res->n_grad++;
            // the active set changed with the iterate: rebuild the compacted copy if it is worth having (judged by the
            // number of products the inner solve just took)
            if (ds->dense && gnorm > P.eps * res->gnorm0 && dense_compact_wanted(ds, ds->Dcur, ncg)) TRON_TRY(dense_compact_build(ds, ds->Dcur));
            if (precond && gnorm > P.eps * res->gnorm0) TRON_TRY(build_preconditioner(ds, P, ds->Dcur, g, M, &gscaled));
        }
        res->outer_iters = k;
        if (trace && res->trace_len < trace_cap) {
            tron_trace_rec &t = trace[res->trace_len++];
            t.iter = k; t.cg_iters = ncg; t.accepted = accepted; t.on_boundary = onb;
            t.f = f; t.gnorm = gnorm; t.delta = delta; t.ared = ared; t.pred = pred; t.snorm = snorm;
        }
        if (accepted && gnorm <= P.eps * res->gnorm0) { status = TRON_OK; res->converged = 1; break; }
        if (pred <= 0.0 || (noise && gnorm >= gnorm_before)) break;
    }
    res->f = f;
    res->gnorm = gnorm;
    TRON_HIP(hipMemcpyAsync(w_dev, w, dbytes, hipMemcpyDeviceToDevice, ds->stream));
    TRON_HIP(hipStreamSynchronize(ds->stream));
    return status;
}

extern "C" int tron_hess_diag(tron_dataset *ds, double C, double *hd_dev)
{
    if (!ds || !hd_dev) { set_error("tron_hess_diag: null argument"); return TRON_EINVAL; }
    if (!(C > 0.0) || !std::isfinite(C)) { set_error("tron_hess_diag: C must be positive and finite"); return TRON_EINVAL; }
    if (!ds->have_D) { set_error("tron_hess_diag: no D cached; call tron_fun_grad first"); return TRON_ESTATE; }
    TRON_TRY(hess_diag_enqueue(ds, C, ds->Dcur, hd_dev));
    TRON_HIP(hipStreamSynchronize(ds->stream));
    return TRON_OK;
}
