/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded fp64 implementation of trust-region Newton (TRON)
 * training for L2-regularised logistic regression and the L2-loss SVM, written from
 * the paper (Halloran & Rocke, "GPU-Accelerated Primal Learning for Extremely Fast
 * Large-Scale Classification", Section 3, Table 1, Algorithm 1, Appendices B, D, E).
 *
 * It exists to check the GPU library and to be timed beside it.  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it; the product
 * path never does, and the two share no code.
 *
 * Notation: n = number of instances (rows of X), d = number of features, so
 * X is n-by-d, z = X w has length n, and w, g, v, Hv have length d.  (The paper
 * writes l for instances and n for features.)
 *
 * Every sum -- row dot products, the loss sum, the d scatter accumulators, the
 * conjugate-gradient dot products -- is accumulated in long double, so the oracle's
 * own rounding stays far below the 1e-10 parity gate even for 2.3e8-term sums.
 *
 * Readings of the paper taken here (it is silent or inconsistent on them):
 *   - z = X w (the paper also writes X^T w; only X w is dimensionally valid for
 *     X = [x_1 ... x_l]^T, Section 3);
 *   - gradient  g = w + C X^T zhat  (the sum forms in Table 1 / Appendix B decide);
 *   - L2-SVM loss  max(0, 1 - y z)^2  (Section 3, Eq. 1 text), active set strict:
 *     i in I  iff  1 - y_i z_i > 0  (Table 1);
 *   - Hessian-vector product  Hv = v + C X^T (D (X v)), with the L2-SVM written in
 *     the same form through D_ii = 2 * [i in I]  (Appendix B: I + 2C X_I^T X_I);
 *   - the trust-region constants, the CG stopping rule and the convergence test are
 *     not given by the paper: see orc_tron / orc_cg below.  PARITY UNPINNED against
 *     the paper for those constants; they are pinned by convergence to the
 *     brute-force minimiser only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_API __attribute__((visibility("default")))

/* Accumulator type of every sum.  The oracle proper uses long double; building with -DORC_ACC_DOUBLE gives a plain
 * fp64 twin that the tests use only to measure how far rounding alone can move a trust-region trajectory. */
#ifdef ORC_ACC_DOUBLE
typedef double acc_t;
#define ORC_SQRT sqrt
#else
typedef long double acc_t;
#define ORC_SQRT sqrtl
#endif

enum { ORC_LOSS_LR = 0, ORC_LOSS_L2SVM = 1 };

typedef struct {
    int64_t n, d;
    /* CSR (used when X == NULL) */
    const int64_t *rowptr;
    const int32_t *col;
    const double *val;
    /* dense row-major n*d (used when non-NULL) */
    const double *X;
    const double *y;
} orc_data;

/* ---- row access: the only place the storage format matters ---- */

/* x_i . u */
static acc_t row_dot(const orc_data *A, int64_t i, const double *u)
{
    acc_t acc = (acc_t)0;
    if (A->X) {
        const double *x = A->X + i * A->d;
        for (int64_t j = 0; j < A->d; ++j) acc += (acc_t)x[j] * (acc_t)u[j];
    } else {
        for (int64_t k = A->rowptr[i]; k < A->rowptr[i + 1]; ++k)
            acc += (acc_t)A->val[k] * (acc_t)u[A->col[k]];
    }
    return acc;
}

/* acc += c * x_i */
static void row_axpy(const orc_data *A, int64_t i, acc_t c, acc_t *acc)
{
    if (A->X) {
        const double *x = A->X + i * A->d;
        for (int64_t j = 0; j < A->d; ++j) acc[j] += c * (acc_t)x[j];
    } else {
        for (int64_t k = A->rowptr[i]; k < A->rowptr[i + 1]; ++k)
            acc[A->col[k]] += c * (acc_t)A->val[k];
    }
}

static acc_t vdot(int64_t m, const double *a, const double *b)
{
    acc_t acc = (acc_t)0;
    for (int64_t j = 0; j < m; ++j) acc += (acc_t)a[j] * (acc_t)b[j];
    return acc;
}

/* ---- per-instance loss terms (Appendix E: alpha, zhat, D; Table 1) ---- */

/*
 * Logistic loss at margin t = y z, with h(t) = 1/(1+exp(-t)):
 *   alpha = log(1/h(t)) = log(1+exp(-t)),  zhat = (h(t)-1) y,  D = h(t)(1-h(t)).
 * Evaluated with exp of a non-positive argument only, so nothing overflows and
 * 1-h is formed without cancellation.
 */
static void lr_terms(double t, double yi, double *alpha, double *zhat, double *D)
{
    double e, h, omh; /* e = exp(-|t|), h = h(t), omh = 1 - h(t) */
    if (t >= 0.0) {
        e = exp(-t);
        h = 1.0 / (1.0 + e);
        omh = e / (1.0 + e);
        *alpha = log1p(e);
    } else {
        e = exp(t);
        h = e / (1.0 + e);
        omh = 1.0 / (1.0 + e);
        *alpha = -t + log1p(e);
    }
    *zhat = -omh * yi;
    *D = h * omh;
}

/*
 * L2-SVM at margin slack m = 1 - y z: active iff m > 0 (strict);
 *   alpha = max(0,m)^2,  zhat = 2 (z - y) on the active set (else 0),  D = 2 on the
 *   active set (else 0), so that g = w + C X^T zhat and Hv = v + C X^T D X v
 *   reproduce  w + 2C X_I^T (z_I - y_I)  and  v + 2C X_I^T X_I v.
 */
static void svm_terms(double z, double yi, double *alpha, double *zhat, double *D)
{
    const double m = 1.0 - yi * z;
    if (m > 0.0) {
        *alpha = m * m;
        *zhat = 2.0 * (z - yi);
        *D = 2.0;
    } else {
        *alpha = 0.0;
        *zhat = 0.0;
        *D = 0.0;
    }
}

/*
 * Function value (Section 3 Eq. 1 with the 1/2 w.w regulariser of Appendix B):
 *   f(w) = 1/2 w.w + C sum_i loss_i,   z = X w.
 * Also returns, per instance, z (optional), zhat and D at this w -- the quantities the
 * gradient and the Hessian-vector product reuse (Section 4.2, Appendix D).
 */
ORC_API int orc_fun(const orc_data *A, int loss, double C, const double *w, double *f_out, double *z_out,
                    double *zhat, double *D)
{
    acc_t sum = (acc_t)0;
    for (int64_t i = 0; i < A->n; ++i) {
        const double z = (double)row_dot(A, i, w);
        double a, zh, Di;
        if (loss == ORC_LOSS_LR)
            lr_terms(A->y[i] * z, A->y[i], &a, &zh, &Di);
        else
            svm_terms(z, A->y[i], &a, &zh, &Di);
        sum += (acc_t)a;
        if (z_out) z_out[i] = z;
        if (zhat) zhat[i] = zh;
        if (D) D[i] = Di;
    }
    *f_out = (double)((acc_t)0.5 * vdot(A->d, w, w) + (acc_t)C * sum);
    return 0;
}

/* Gradient (Table 1, Appendix B):  g = w + C sum_i zhat_i x_i. */
ORC_API int orc_grad(const orc_data *A, double C, const double *w, const double *zhat, double *g)
{
    acc_t *acc = (acc_t *)calloc((size_t)A->d, sizeof(acc_t));
    if (!acc) return -2;
    for (int64_t i = 0; i < A->n; ++i)
        if (zhat[i] != 0.0) row_axpy(A, i, (acc_t)zhat[i], acc);
    for (int64_t j = 0; j < A->d; ++j) g[j] = (double)((acc_t)w[j] + (acc_t)C * acc[j]);
    free(acc);
    return 0;
}

/* Hessian-vector product (Table 1, Appendix B, D):  Hv = v + C sum_i D_i (x_i.v) x_i. */
ORC_API int orc_hv(const orc_data *A, double C, const double *D, const double *v, double *Hv)
{
    acc_t *acc = (acc_t *)calloc((size_t)A->d, sizeof(acc_t));
    if (!acc) return -2;
    for (int64_t i = 0; i < A->n; ++i) {
        if (D[i] == 0.0) continue;
        const acc_t a0 = row_dot(A, i, v);         /* a0 = X v      */
        const acc_t a1 = (acc_t)D[i] * a0;   /* a1 = D a0     */
        row_axpy(A, i, a1, acc);                         /* X^T a1        */
    }
    for (int64_t j = 0; j < A->d; ++j) Hv[j] = (double)((acc_t)v[j] + (acc_t)C * acc[j]);
    free(acc);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Truncated Newton step: conjugate gradients inside the trust region  */
/* (Algorithm 1 line 4; Appendix B Eq. "min q(d) s.t. |d| <= Delta").   */
/* ------------------------------------------------------------------ */
/*
 * The paper only names "a conjugate gradient procedure"; the reading taken is the
 * textbook Steihaug-Toint iteration on  q(s) = g.s + 1/2 s.H s:
 *   s = 0, r = -g, p = r
 *   repeat (at most max_cg products):
 *     stop if |r| <= xi |g|
 *     alpha = r.r / p.Hp
 *     if |s + alpha p| >= Delta: move to the boundary along p (tau >= 0 with
 *         |s + tau p| = Delta), update r, stop
 *     s += alpha p;  r -= alpha Hp;  beta = r_new.r_new / r.r;  p = r + beta p
 * H >= I for both losses (Appendix B), so p.Hp > 0 always.
 * Outputs s, r (= -g - H s), the number of Hessian-vector products and whether the
 * step ended on the boundary.
 */
ORC_API int orc_cg(const orc_data *A, double C, const double *D, const double *g, double delta, double xi,
                   int max_cg, double *s, double *r, int *n_hv, int *on_boundary)
{
    const int64_t d = A->d;
    double *p = (double *)malloc(sizeof(double) * (size_t)d);
    double *Hp = (double *)malloc(sizeof(double) * (size_t)d);
    if (!p || !Hp) { free(p); free(Hp); return -2; }
    for (int64_t j = 0; j < d; ++j) { s[j] = 0.0; r[j] = -g[j]; p[j] = r[j]; }
    acc_t rr = vdot(d, r, r);
    const acc_t gnorm = ORC_SQRT(vdot(d, g, g));
    int it = 0;
    *on_boundary = 0;
    while (it < max_cg) {
        if (ORC_SQRT(rr) <= (acc_t)xi * gnorm) break;
        orc_hv(A, C, D, p, Hp);
        ++it;
        const acc_t pHp = vdot(d, p, Hp);
        const double alpha = (double)(rr / pHp);
        /* length of the tentative iterate s + alpha p */
        acc_t len2 = (acc_t)0;
        for (int64_t j = 0; j < d; ++j) {
            const acc_t t = (acc_t)s[j] + (acc_t)alpha * (acc_t)p[j];
            len2 += t * t;
        }
        if (ORC_SQRT(len2) >= (acc_t)delta) {
            /* positive root of |s + tau p|^2 = Delta^2, in the cancellation-free form */
            const acc_t ss = vdot(d, s, s), sp = vdot(d, s, p), pp = vdot(d, p, p);
            const acc_t gap = (acc_t)delta * (acc_t)delta - ss;
            const acc_t rad = ORC_SQRT(sp * sp + pp * gap);
            const double tau = (double)((sp >= (acc_t)0) ? gap / (sp + rad) : (rad - sp) / pp);
            for (int64_t j = 0; j < d; ++j) {
                s[j] = (double)((acc_t)s[j] + (acc_t)tau * (acc_t)p[j]);
                r[j] = (double)((acc_t)r[j] - (acc_t)tau * (acc_t)Hp[j]);
            }
            *on_boundary = 1;
            break;
        }
        for (int64_t j = 0; j < d; ++j) {
            s[j] = (double)((acc_t)s[j] + (acc_t)alpha * (acc_t)p[j]);
            r[j] = (double)((acc_t)r[j] - (acc_t)alpha * (acc_t)Hp[j]);
        }
        const acc_t rr_new = vdot(d, r, r);
        const double beta = (double)(rr_new / rr);
        for (int64_t j = 0; j < d; ++j) p[j] = (double)((acc_t)r[j] + (acc_t)beta * (acc_t)p[j]);
        rr = rr_new;
    }
    *n_hv = it;
    free(p);
    free(Hp);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Diagonal preconditioner (the paper only names it: Sections 2 and 4.3, */
/* Appendix D say that D is kept for "preconditioning computations" and   */
/* cite Hsia, Chiang and Lin 2018; no formula is given).                  */
/* PARITY UNPINNED against the paper; the reading below is the method of  */
/* the cited work in this oracle's own rules.                             */
/* ------------------------------------------------------------------ */
/* Diagonal of the Hessian of Appendix B:  diag(H)_j = 1 + C sum_i D_i x_ij^2. */
ORC_API int orc_hess_diag(const orc_data *A, double C, const double *D, double *hd)
{
    acc_t *acc = (acc_t *)calloc((size_t)A->d, sizeof(acc_t));
    if (!acc) return -2;
    for (int64_t i = 0; i < A->n; ++i) {
        if (D[i] == 0.0) continue;
        if (A->X) {
            const double *x = A->X + i * A->d;
            for (int64_t j = 0; j < A->d; ++j) acc[j] += (acc_t)D[i] * (acc_t)x[j] * (acc_t)x[j];
        } else {
            for (int64_t k = A->rowptr[i]; k < A->rowptr[i + 1]; ++k)
                acc[A->col[k]] += (acc_t)D[i] * (acc_t)A->val[k] * (acc_t)A->val[k];
        }
    }
    for (int64_t j = 0; j < A->d; ++j) hd[j] = (double)((acc_t)1 + (acc_t)C * acc[j]);
    free(acc);
    return 0;
}

/* u . (M v) for a diagonal M */
static acc_t mdot(int64_t m, const double *M, const double *a, const double *b)
{
    acc_t t = (acc_t)0;
    for (int64_t j = 0; j < m; ++j) t += (acc_t)M[j] * (acc_t)a[j] * (acc_t)b[j];
    return t;
}

/*
 * Preconditioned Steihaug-Toint iteration with a diagonal M > 0: the trust region is
 * measured in the M-norm |s|_M = sqrt(s.Ms), which makes it plain CG on the variables
 * M^(1/2) s:
 *   s = 0, r = -g, z = M^-1 r, p = z
 *   repeat (at most max_cg products):
 *     stop if sqrt(r.z) <= xi sqrt(g.M^-1 g)
 *     alpha = r.z / p.Hp
 *     if |s + alpha p|_M >= Delta: tau >= 0 with |s + tau p|_M = Delta, update r, stop
 *     s += alpha p;  r -= alpha Hp;  z = M^-1 r;  beta = r_new.z_new / r.z;  p = z + beta p
 * With M = I this is orc_cg step for step.
 */
ORC_API int orc_pcg(const orc_data *A, double C, const double *D, const double *g, const double *M, double delta,
                    double xi, int max_cg, double *s, double *r, int *n_hv, int *on_boundary)
{
    const int64_t d = A->d;
    double *p = (double *)malloc(sizeof(double) * (size_t)d);
    double *z = (double *)malloc(sizeof(double) * (size_t)d);
    double *Hp = (double *)malloc(sizeof(double) * (size_t)d);
    if (!p || !z || !Hp) { free(p); free(z); free(Hp); return -2; }
    for (int64_t j = 0; j < d; ++j) { s[j] = 0.0; r[j] = -g[j]; z[j] = r[j] / M[j]; p[j] = z[j]; }
    acc_t rz = vdot(d, r, z);
    const acc_t gnorm = ORC_SQRT(rz);
    int it = 0;
    *on_boundary = 0;
    while (it < max_cg) {
        if (ORC_SQRT(rz) <= (acc_t)xi * gnorm) break;
        orc_hv(A, C, D, p, Hp);
        ++it;
        const acc_t pHp = vdot(d, p, Hp);
        const double alpha = (double)(rz / pHp);
        acc_t len2 = (acc_t)0;
        for (int64_t j = 0; j < d; ++j) {
            const acc_t t = (acc_t)s[j] + (acc_t)alpha * (acc_t)p[j];
            len2 += (acc_t)M[j] * t * t;
        }
        if (ORC_SQRT(len2) >= (acc_t)delta) {
            const acc_t ss = mdot(d, M, s, s), sp = mdot(d, M, s, p), pp = mdot(d, M, p, p);
            const acc_t gap = (acc_t)delta * (acc_t)delta - ss;
            const acc_t rad = ORC_SQRT(sp * sp + pp * gap);
            const double tau = (double)((sp >= (acc_t)0) ? gap / (sp + rad) : (rad - sp) / pp);
            for (int64_t j = 0; j < d; ++j) {
                s[j] = (double)((acc_t)s[j] + (acc_t)tau * (acc_t)p[j]);
                r[j] = (double)((acc_t)r[j] - (acc_t)tau * (acc_t)Hp[j]);
            }
            *on_boundary = 1;
            break;
        }
        for (int64_t j = 0; j < d; ++j) {
            s[j] = (double)((acc_t)s[j] + (acc_t)alpha * (acc_t)p[j]);
            r[j] = (double)((acc_t)r[j] - (acc_t)alpha * (acc_t)Hp[j]);
            z[j] = r[j] / M[j];
        }
        const acc_t rz_new = vdot(d, r, z);
        const double beta = (double)(rz_new / rz);
        for (int64_t j = 0; j < d; ++j) p[j] = (double)((acc_t)z[j] + (acc_t)beta * (acc_t)p[j]);
        rz = rz_new;
    }
    *n_hv = it;
    free(p);
    free(z);
    free(Hp);
    return 0;
}

/* ------------------------------------------------------------------ */
/* TRON outer loop (Algorithm 1)                                        */
/* ------------------------------------------------------------------ */
typedef struct {
    int iter;          /* outer iteration, from 1 */
    int cg_iters;      /* Hessian-vector products in this iteration's CG */
    int accepted;      /* step taken (sigma > sigma_0) */
    int on_boundary;   /* CG stopped on the trust-region boundary */
    double f;          /* objective after this iteration (at the current w) */
    double gnorm;      /* |grad f| at the current w */
    double delta;      /* trust-region radius after the update */
    double ared;       /* f(w) - f(w+s) */
    double pred;       /* -q(s) */
    double snorm;      /* |s| */
} orc_trace_rec;

typedef struct {
    double f, gnorm, gnorm0;
    int outer_iters, cg_iters_total, n_fun, n_grad, n_hv, converged;
} orc_result;

/* Optional observer, called with the record of every finished outer iteration (a long solve can report where it
 * is); it sees the values and changes nothing. */
typedef void (*orc_progress_fn)(const orc_trace_rec *);
static orc_progress_fn progress_fn = NULL;
ORC_API void orc_set_progress(orc_progress_fn fn) { progress_fn = fn; }

/*
 * Algorithm 1 with the blanks filled in as follows (the paper names sigma_0 only):
 *   - Delta_0 = |grad f(w_0)|;
 *   - converged when |grad f(w)| <= eps |grad f(0)|;
 *   - sigma = ared/pred with ared = f(w) - f(w+s), pred = -q(s) = -1/2 (g.s - s.r)
 *     (the paper's sigma = (f(w+d)-f(w))/q(d) is the same ratio);
 *   - accept the step iff sigma > sigma_0 = 1e-4;
 *   - radius:  sigma < 1/4  -> Delta = 1/2 min(|s|, Delta);
 *              sigma < 3/4  -> unchanged;
 *              otherwise    -> Delta = min(4 Delta, max(Delta, 4 |s|));
 *   - when |ared| and pred are both below 1e-12 |f| the measured reduction is rounding
 *     noise of f, so the model is trusted: sigma is taken as 1;
 *   - stop (not converged) when pred <= 0, when such a noise-level step fails to
 *     reduce |grad f|, or after max_outer iterations.
 * The Hessian-vector products of an iteration use D at the current (accepted) w: a
 * rejected trial point never replaces it.
 * Status: 0 converged, 1 iteration/stall limit, <0 error.
 */
static int tron_impl(const orc_data *A, int loss, double C, double eps, int max_outer, int max_cg, double xi, int precond,
                     double blend, double *w, orc_result *res, orc_trace_rec *trace, int trace_cap, int *trace_len)
{
    const int64_t n = A->n, d = A->d;
    double *M = precond ? (double *)malloc(sizeof(double) * (size_t)d) : NULL;
    const double eta0 = 1e-4, eta1 = 0.25, eta2 = 0.75, sig2 = 0.5, sig3 = 4.0;
    double *g = (double *)malloc(sizeof(double) * (size_t)d);
    double *s = (double *)malloc(sizeof(double) * (size_t)d);
    double *r = (double *)malloc(sizeof(double) * (size_t)d);
    double *wnew = (double *)malloc(sizeof(double) * (size_t)d);
    double *zhat = (double *)malloc(sizeof(double) * (size_t)n);
    double *Dcur = (double *)malloc(sizeof(double) * (size_t)n);
    double *Dnew = (double *)malloc(sizeof(double) * (size_t)n);
    int status = 1, tl = 0;
    memset(res, 0, sizeof(*res));
    if (!g || !s || !r || !wnew || !zhat || !Dcur || !Dnew || (precond && !M)) { status = -2; goto done; }

    /* |grad f(0)|, the reference for the stopping test */
    {
        int w_is_zero = 1;
        for (int64_t j = 0; j < d; ++j) if (w[j] != 0.0) { w_is_zero = 0; break; }
        if (!w_is_zero) {
            double f0;
            memset(wnew, 0, sizeof(double) * (size_t)d);
            orc_fun(A, loss, C, wnew, &f0, NULL, zhat, Dnew);
            orc_grad(A, C, wnew, zhat, g);
            res->gnorm0 = (double)ORC_SQRT(vdot(d, g, g));
            res->n_fun++; res->n_grad++;
        }
    }
    double f;
    orc_fun(A, loss, C, w, &f, NULL, zhat, Dcur);
    orc_grad(A, C, w, zhat, g);
    res->n_fun++; res->n_grad++;
    double gnorm = (double)ORC_SQRT(vdot(d, g, g));
    if (res->gnorm0 == 0.0) res->gnorm0 = gnorm;
    double delta = gnorm;
    if (precond) {
        /* M = (1 - blend) I + blend diag(H) at the current w;  Delta_0 = |M^-1 g|_M = sqrt(g.M^-1 g) */
        orc_hess_diag(A, C, Dcur, M);
        acc_t t = (acc_t)0;
        for (int64_t j = 0; j < d; ++j) {
            M[j] = (1.0 - blend) + blend * M[j];
            t += (acc_t)g[j] * (acc_t)g[j] / (acc_t)M[j];
        }
        delta = (double)ORC_SQRT(t);
    }
    if (gnorm <= eps * res->gnorm0) { status = 0; res->converged = 1; }

    for (int k = 1; status == 1 && k <= max_outer; ++k) {
        int ncg = 0, onb = 0;
        if (precond) orc_pcg(A, C, Dcur, g, M, delta, xi, max_cg, s, r, &ncg, &onb);
        else orc_cg(A, C, Dcur, g, delta, xi, max_cg, s, r, &ncg, &onb);
        res->n_hv += ncg; res->cg_iters_total += ncg;
        const double snorm = (double)ORC_SQRT(precond ? mdot(d, M, s, s) : vdot(d, s, s));
        const double pred = (double)(-(acc_t)0.5 * (vdot(d, g, s) - vdot(d, s, r)));
        for (int64_t j = 0; j < d; ++j) wnew[j] = w[j] + s[j];
        double fnew;
        orc_fun(A, loss, C, wnew, &fnew, NULL, zhat, Dnew);
        res->n_fun++;
        const double ared = f - fnew;
        const int noise = fabs(ared) <= 1e-12 * fabs(f) && pred <= 1e-12 * fabs(f);
        const double sigma = noise ? 1.0 : ared / pred;
        const double gnorm_before = gnorm;
        if (sigma < eta1) delta = sig2 * fmin(snorm, delta);
        else if (sigma < eta2) { /* unchanged */ }
        else delta = fmin(sig3 * delta, fmax(delta, sig3 * snorm));
        int accepted = 0;
        if (sigma > eta0) {
            accepted = 1;
            memcpy(w, wnew, sizeof(double) * (size_t)d);
            f = fnew;
            orc_grad(A, C, w, zhat, g);
            res->n_grad++;
            { double *t = Dcur; Dcur = Dnew; Dnew = t; }
            gnorm = (double)ORC_SQRT(vdot(d, g, g));
            if (precond) {
                orc_hess_diag(A, C, Dcur, M);
                for (int64_t j = 0; j < d; ++j) M[j] = (1.0 - blend) + blend * M[j];
            }
        }
        res->outer_iters = k;
        {
            const orc_trace_rec rec = { k, ncg, accepted, onb, f, gnorm, delta, ared, pred, snorm };
            if (trace && tl < trace_cap) trace[tl++] = rec;
            if (progress_fn) progress_fn(&rec);
        }
        if (accepted && gnorm <= eps * res->gnorm0) { status = 0; res->converged = 1; break; }
        if (pred <= 0.0 || (noise && gnorm >= gnorm_before)) break;
    }
    res->f = f;
    res->gnorm = gnorm;
done:
    if (trace_len) *trace_len = tl;
    free(g); free(s); free(r); free(wnew); free(zhat); free(Dcur); free(Dnew); free(M);
    return status;
}

ORC_API int orc_tron(const orc_data *A, int loss, double C, double eps, int max_outer, int max_cg, double xi,
                     double *w, orc_result *res, orc_trace_rec *trace, int trace_cap, int *trace_len)
{
    return tron_impl(A, loss, C, eps, max_outer, max_cg, xi, 0, 0.0, w, res, trace, trace_cap, trace_len);
}

/*
 * The same outer loop with the diagonally preconditioned inner solver: M = (1 - blend) I + blend diag(H(w)) is
 * rebuilt at every accepted iterate, the trust region and the step length |s| of the radius rules are measured in
 * the M-norm of the iteration, Delta_0 = sqrt(g.M^-1 g); the convergence test is unchanged (2-norm of the gradient).
 * blend = 0.01 is the value recommended by the cited work.  Own rules: PARITY UNPINNED against the paper.
 */
ORC_API int orc_tron_pcg(const orc_data *A, int loss, double C, double eps, int max_outer, int max_cg, double xi, double blend,
                         double *w, orc_result *res, orc_trace_rec *trace, int trace_cap, int *trace_len)
{
    return tron_impl(A, loss, C, eps, max_outer, max_cg, xi, 1, blend, w, res, trace, trace_cap, trace_len);
}
