/*
 * tron.h -- C ABI of the MI355X (gfx950) trust-region Newton hot path for
 * L2-regularised logistic regression and the L2-loss SVM.
 *
 * Method: Halloran & Rocke, "GPU-Accelerated Primal Learning for Extremely Fast
 * Large-Scale Classification" (Section 3, Table 1, Algorithm 1, Appendices B, D, E).
 *
 * Notation used throughout: n = instances (rows of X), d = features, X is n-by-d,
 * y in {-1,+1}^n, z = X w.  (The paper writes l for instances and n for features.)
 *
 *   f(w)  = 1/2 w.w + C sum_i loss(y_i z_i)                 (Section 3, Eq. 1; Appendix B)
 *   g(w)  = w + C X^T zhat                                  (Table 1)
 *   H(w)v = v + C X^T ( D (X v) )                           (Table 1, Appendix B, D)
 *
 *   logistic: loss = log(1+exp(-y z)), zhat_i = (h(y_i z_i)-1) y_i, D_ii = h(1-h),
 *             h(t) = 1/(1+exp(-t))                          (Appendix E)
 *   L2-SVM:   loss = max(0, 1-y z)^2, I = {i : 1 - y_i z_i > 0} (strict),
 *             zhat_i = 2 (z_i - y_i) on I else 0, D_ii = 2 on I else 0, which is the
 *             paper's  w + 2C X_I^T (z_I - y_I)  and  v + 2C X_I^T X_I v.
 *
 * General rules
 *   - Every function returns an int status: TRON_OK (0), a negative error, or the
 *     positive soft status TRON_EMAXITER.  Nothing throws or aborts across the ABI.
 *     After an error, tron_last_error() (thread-local) describes it.
 *   - "device pointer" = HIP device memory on the handle's GPU, caller-owned, fp64,
 *     never retained after the call returns.  "host pointer" = ordinary host memory.
 *   - All GPU work is enqueued on the hipStream_t given at dataset creation (pass the
 *     stream as void*; NULL = the default stream).  A call that returns a host scalar
 *     synchronises that stream before returning; one that does not, does not.
 *   - A handle is not thread-safe; distinct handles are independent.
 *   - All arithmetic is fp64.  Reductions are two-stage and atomic-free, so repeated
 *     calls with the same inputs return bit-identical results.
 *   - There is no CPU fallback: without a usable GPU every call returns TRON_EDEVICE.
 */
#ifndef TRON_H_
#define TRON_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TRON_API __attribute__((visibility("default")))

typedef struct tron_dataset tron_dataset; /* opaque: device copies of X (and X^T for CSR), y, cached D, work space */

enum { TRON_LOSS_LR = 0, TRON_LOSS_L2SVM = 1 };
enum {
    TRON_OK = 0,
    TRON_EINVAL = -1,   /* bad argument or malformed input */
    TRON_ENOMEM = -2,   /* host or device allocation failed */
    TRON_EDEVICE = -3,  /* HIP runtime error / no device */
    TRON_ESTATE = -4,   /* call order violated (e.g. tron_hv before tron_fun_grad) */
    TRON_EMAXITER = 1   /* soft: iteration limit or stall; outputs hold the last iterate */
};
enum { TRON_MEM_HOST = 0, TRON_MEM_DEVICE = 1 };

/* ------------------------------------------------------------------------------------------
 * Dataset handles (the problem statement of Section 3: X = [x_1 ... x_l]^T and y).
 * The library copies X and y (the caller may free its buffers on return) and, for CSR,
 * builds the explicit transposed copy used by X^T products (Table 1: X^T zhat, X^T(D(Xv))).
 * ------------------------------------------------------------------------------------------ */

/*
 * CSR input: rowptr int64[n+1] (rowptr[0] = 0, non-decreasing, rowptr[n] = nnz), col int32[nnz]
 * (inside each row strictly increasing and in [0,d)), val fp64[nnz] (finite), y fp64[n]
 * (exactly +1.0 or -1.0).  mem says whether the four arrays are host or device pointers (all
 * alike).  Validation failures return TRON_EINVAL and create nothing.  1 <= n, d < 2^29; nnz may be 0;
 * empty rows and columns are allowed.
 */
TRON_API int tron_dataset_create_csr(int64_t n, int64_t d, const int64_t *rowptr, const int32_t *col,
                                     const double *val, const double *y, int mem, void *hip_stream,
                                     tron_dataset **out);

/* Dense input: X row-major n*d fp64 with leading dimension d (finite), y fp64[n] exactly +1.0 or -1.0; host or device
 * pointers per mem, checked either way (device input by a kernel): TRON_EINVAL and nothing created otherwise. */
TRON_API int tron_dataset_create_dense(int64_t n, int64_t d, const double *X_rowmajor, const double *y, int mem,
                                       void *hip_stream, tron_dataset **out);

/*
 * Dense dataset filled in row chunks (for matrices too large to stage on the host at once):
 * create_dense_empty allocates n*d on the device with undefined contents; write_rows copies
 * nrows rows starting at row0 (X_chunk row-major nrows*d, y_chunk nrows; host or device per mem).  A chunk with a
 * label other than +1 / -1 or a non-finite entry returns TRON_EINVAL and writes nothing.
 * Every row must be written once before the first compute call; this is not checked.
 */
TRON_API int tron_dataset_create_dense_empty(int64_t n, int64_t d, void *hip_stream, tron_dataset **out);
TRON_API int tron_dataset_write_rows(tron_dataset *ds, int64_t row0, int64_t nrows, const double *X_chunk,
                                     const double *y_chunk, int mem);

/* Frees the device memory.  NULL is ignored. */
TRON_API void tron_dataset_destroy(tron_dataset *ds);

/* Shape query: any output pointer may be NULL.  nnz = n*d for dense handles. */
TRON_API int tron_dataset_shape(const tron_dataset *ds, int64_t *n, int64_t *d, int64_t *nnz, int *is_dense);

/*
 * Layout statistics of a handle (what the library built from the input), by name:
 *   "fwd_parts", "bwd_parts"   column partitions of the forward / transposed CSR layouts (0 for dense)
 *   "fwd_segmented", "bwd_segmented"  1 when that layout stores row segments + flag bits (every partitioned layout, and
 *                              unpartitioned ones whose chunks mix long and short rows), 0 for plain CSR
 *   "fwd_csr_nnz", "bwd_csr_nnz"  nonzeros held in those CSR layouts
 *   "fwd_head_nnz"             of fwd_csr_nnz, the nonzeros of the head partition (the most frequent columns)
 *   "bwd_tile_nnz", "bwd_tile_rows", "bwd_tiles"  nonzeros, features and tiles of the hot-row tiles
 *   "fwd_lds_columns"          columns served from LDS tables in the forward pass
 *   "dense_grid"               workgroups of the dense kernels
 *   "dense_compact_rows"       rows of the compacted copy of the active rows the next tron_hv would run over (0: none)
 *   "unit_values"              1 when the sparse layouts keep no values (every instance's entries share one value)
 *   "fwd_bytes_gather", "fwd_bytes_head", "fwd_bytes_ranges", "fwd_bytes_combine",
 *   "bwd_bytes_tiles", "bwd_bytes_tile_reduce", "bwd_bytes_ranges", "bwd_bytes_combine"
 *                              bytes one launch of that kernel of the forward / transposed product has to move in the
 *                              format the handle stores (index and value streams, flag bits, tables, each needed vector
 *                              element once, partial sums and results written); 0 for dense handles and absent parts
 *   "hv_bytes", "fun_grad_bytes"  the same for a whole tron_hv / tron_fun_grad call with the currently cached D (dense:
 *                              X once -- only the active rows when the pass skips the others -- plus D or the
 *                              active-set bits); these are the denominators of the reported HBM fractions
 * Unknown names return TRON_EINVAL.
 */
TRON_API int tron_dataset_stat(const tron_dataset *ds, const char *name, int64_t *value);

/* ------------------------------------------------------------------------------------------
 * The three callbacks of Table 1.
 * ------------------------------------------------------------------------------------------ */

/*
 * Function value and gradient at w (Algorithm 1 lines 2, 5, 7; Section 4.2; Appendix E):
 *   z = X w;  per-instance loss, zhat, D;  *f_host = 1/2 w.w + C sum loss;  g = w + C X^T zhat.
 * w_dev: device pointer, d doubles.  f_host: host pointer (required).  g_dev: device pointer to d
 * doubles, or NULL for the function value only.  Side effect: D at w is cached in the handle and
 * is what tron_hv uses until the next tron_fun_grad / tron_solve.  Synchronises the stream.
 */
TRON_API int tron_fun_grad(tron_dataset *ds, int loss, double C, const double *w_dev, double *f_host,
                           double *g_dev);

/*
 * Hessian-vector product at the w of the last tron_fun_grad (Table 1; Appendix D):
 *   a0 = X v;  a1 = D a0;  Hv = v + C X^T a1;  optionally *vHv_host = v.Hv (Appendix D: the
 *   curvature scalar is reduced on the device).
 * v_dev, Hv_dev: device pointers, d doubles, must not alias.  vHv_host: host pointer or NULL; when
 * NULL the call only enqueues work and does not synchronise.  C must be the value the cached D
 * belongs with (D itself does not depend on C).  TRON_ESTATE if no D is cached.
 */
TRON_API int tron_hv(tron_dataset *ds, double C, const double *v_dev, double *Hv_dev, double *vHv_host);

/*
 * tron_hv for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same product, same kernels and same results as tron_hv on a dense handle, but the
 * kernels' work space (per-workgroup column sums, column products, the curvature scalar) is a static device array of
 * TRON_HV_STATIC_MAX_DOUBLES doubles (2 MiB, held by every GPU the library runs on until the process ends) instead of
 * the handle's allocation, and the call itself allocates nothing and never synchronises: it only enqueues on the
 * handle's stream.  vHv_dev: DEVICE pointer to one double that receives v.Hv, or NULL.
 * Dense handles only.  TRON_EINVAL when d * (workgroups of the dense kernels, at most 2048; tron_dataset_stat
 * "dense_grid") + d + 1 exceeds TRON_HV_STATIC_MAX_DOUBLES (any n for d <= 127), when the handle is sparse, or when
 * the current device is not the handle's; TRON_ESTATE if no D is cached.
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams or
 * threads) race; calls on one stream are ordered and safe.  The array keeps the last call's contents; no call relies
 * on them.
 */
#define TRON_HV_STATIC_MAX_DOUBLES 262144
TRON_API int tron_hv_static(tron_dataset *ds, double C, const double *v_dev, double *Hv_dev, double *vHv_dev);

/*
 * Diagonal of the Hessian at the w of the last tron_fun_grad (Appendix B: H = I + C X^T D X):
 *   hd_j = 1 + C sum_i D_i x_ij^2.
 * hd_dev: device pointer, d doubles.  Synchronises the stream.  TRON_ESTATE if no D is cached.
 */
TRON_API int tron_hess_diag(tron_dataset *ds, double C, double *hd_dev);

/* ------------------------------------------------------------------------------------------
 * Full solve: Algorithm 1 with the conjugate-gradient inner solver, all vectors on the device;
 * only scalars reach the host.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int loss;       /* TRON_LOSS_* */
    double C;       /* > 0 */
    double eps;     /* > 0: stop when |grad f(w)| <= eps |grad f(0)| */
    int max_outer;  /* > 0 */
    int max_cg;     /* > 0: cap on Hessian-vector products per outer iteration */
    double cg_xi;   /* in (0,1): CG stops when |r| <= cg_xi |g| */
    double precond_blend; /* 0: plain CG.  a in (0,1]: CG preconditioned by the diagonal M = (1-a) I + a diag(H) */
} tron_params;

typedef struct {
    int iter;         /* outer iteration, from 1 */
    int cg_iters;     /* Hessian-vector products of this iteration */
    int accepted;     /* step taken */
    int on_boundary;  /* CG ended on the trust-region boundary */
    double f;         /* objective at the current w after this iteration */
    double gnorm;     /* |grad f| at the current w */
    double delta;     /* radius after the update */
    double ared;      /* f(w) - f(w+s) */
    double pred;      /* -q(s) */
    double snorm;     /* |s| (with a preconditioner: the M-norm sqrt(s.Ms)) */
} tron_trace_rec;

typedef struct {
    double f, gnorm, gnorm0;
    int outer_iters, cg_iters_total, n_fun, n_grad, n_hv, converged;
    int trace_cap;          /* in: capacity of trace (0 = none) */
    int trace_len;          /* out: records written */
    tron_trace_rec *trace;  /* in: host array of trace_cap records, or NULL */
} tron_result;

/*
 * w_dev: device pointer, d doubles; in: starting point w0, out: final iterate.
 * res_host: host pointer; set trace/trace_cap before the call.
 * Rules (the paper names sigma_0 only; these are this library's reading of Algorithm 1):
 *   Delta_0 = |g(w0)|;  accept iff sigma = ared/pred > 1e-4;  sigma < 1/4: Delta = min(|s|,Delta)/2;
 *   sigma < 3/4: unchanged;  else Delta = min(4 Delta, max(Delta, 4|s|));  when |ared| and pred are
 *   both below 1e-12 |f| sigma is taken as 1;  CG is Steihaug's truncated iteration.
 * With precond_blend = a > 0 the inner solver is preconditioned by M = (1-a) I + a diag(H(w)), rebuilt at every
 * accepted iterate: the trust region and |s| are then measured in the M-norm, Delta_0 = sqrt(g.M^-1 g), CG stops when
 * sqrt(r.M^-1 r) <= cg_xi sqrt(g.M^-1 g).  (The paper names a preconditioner -- Sections 2, 4.3, Appendix D -- without
 * giving it; this is the diagonal one of the work it cites, a = 0.01 being that work's choice.)
 * Returns TRON_OK when converged, TRON_EMAXITER when max_outer was reached or progress stalled.
 * On return the handle caches D at the final iterate (so tron_hv may follow).
 * Small dense L2-SVM problems (d <= 32, no preconditioner) are driven from the device, like tron_batch_solve with one
 * problem over all rows: same rules, same results up to summation order (knob "dense_device_driver").
 */
TRON_API int tron_solve(tron_dataset *ds, const tron_params *params, double *w_dev, tron_result *res_host);

/* ------------------------------------------------------------------------------------------
 * Several problems over one resident matrix.
 * Section 2.1: Percolator trains its SVMs under three-fold cross-validation with a nested
 * cross-validation inside every fold, i.e. many problems of Section 3 that differ only in the
 * subset of instances they train on and in C.  A batch runs up to TRON_BATCH_MAX such problems in
 * lock-step: one pass over X serves every problem's pending product -- X^T(D(Xv)) for those inside
 * CG, the function/gradient pass for those at a trial point -- so X is read once per round, not once
 * per problem.  Problem k is exactly the problem of Section 3 over the instances {i : bit k of
 * member[i] is set}: the rows outside it contribute nothing to f, g or Hv.
 * Dense handles with d <= TRON_BATCH_MAX_D only (sparse handles and wider matrices: one tron_solve per problem).
 * Per tile of 64 instances the pass is two skinny matrix products (64 x d by d x K, and d x 64 by 64 x K).  They run
 * on the vector units, or as fp64 matrix instructions with the problems as the sixteen result columns: always above
 * eight problems, below that per loss where measured faster (L2-SVM: eight problems, logistic loss: five and more);
 * knob "batch_mfma".  Same results up to summation order.
 * ------------------------------------------------------------------------------------------ */
typedef struct tron_batch tron_batch; /* opaque: membership bits, per-problem D, solver state, work space */

#define TRON_BATCH_MAX 16
#define TRON_BATCH_MAX_D 32

/*
 * K in [1, TRON_BATCH_MAX].  member: n words, host or device per mem; bit k (k < K) of member[i] says
 * whether instance i belongs to problem k; higher bits must be zero.  The words are copied.  The batch
 * uses the dataset's matrix, labels, stream and profiler: ds must stay alive, and must not be used by
 * another thread, while the batch exists.  A problem with no instance is allowed (f = 1/2 w.w).
 */
TRON_API int tron_batch_create(tron_dataset *ds, int K, const uint32_t *member, int mem, tron_batch **out);

/* Frees the batch (not the dataset).  NULL is ignored. */
TRON_API void tron_batch_destroy(tron_batch *b);

/*
 * tron_fun_grad for every problem in one pass.  C_host: K values > 0 (host).  W_dev: K*d doubles,
 * problem k's w at W_dev + k*d (device).  f_host: K doubles (host).  G_dev: K*d doubles (device) or
 * NULL.  D of every problem at its w is cached in the batch for tron_batch_hv.  Synchronises.
 */
TRON_API int tron_batch_fun_grad(tron_batch *b, int loss, const double *C_host, const double *W_dev, double *f_host,
                                 double *G_dev);

/*
 * tron_hv for every problem in one pass, with the D cached by the last tron_batch_fun_grad or
 * tron_batch_solve.  V_dev, HV_dev: K*d doubles each (device), must not alias.  vHv_host: K doubles
 * (host) or NULL.  Synchronises.  TRON_ESTATE if no D is cached.
 */
TRON_API int tron_batch_hv(tron_batch *b, const double *C_host, const double *V_dev, double *HV_dev, double *vHv_host);

/*
 * tron_solve for every problem, in lock-step rounds of one pass over X each.  params: loss, eps,
 * max_outer, max_cg, cg_xi, precond_blend apply to every problem; params->C is ignored (C_host[k] is problem k's C).
 * With precond_blend > 0 every problem runs the preconditioned inner solver described for tron_solve; the Hessian
 * diagonal of a problem's new iterate takes one more pass over X (a round of its own, shared with whatever the other
 * problems have pending).  W_dev: K*d doubles, in: starting points, out: final iterates.
 * res_host: K results, each with its own trace / trace_cap set before the call.  Every problem follows
 * the rules stated for tron_solve; the whole trust-region and CG logic runs on the device (the vectors
 * have d <= 32 entries), the host only learns which problems are still running.
 * Returns TRON_OK when every problem converged, TRON_EMAXITER when some problem stopped at its
 * iteration limit or stalled (status_host[k], if not NULL, receives each problem's own status).
 */
TRON_API int tron_batch_solve(tron_batch *b, const tron_params *params, const double *C_host, double *W_dev,
                              tron_result *res_host, int *status_host);

/* ------------------------------------------------------------------------------------------
 * Diagnostics.
 * ------------------------------------------------------------------------------------------ */

/* Message for the calling thread's most recent failure ("" if none).  Static storage. */
TRON_API const char *tron_last_error(void);

/*
 * Per-kernel timing with HIP events on the handle's stream.  While enabled, every kernel the
 * library launches for this handle is bracketed by an event pair.  tron_profile_read synchronises,
 * adds up the elapsed time per kernel slot since the last reset, and fills up to `cap` entries of
 * names[] (static strings), ms[] (total milliseconds) and calls[] (launch counts); it returns the
 * number of slots in *count and resets the totals.
 */
TRON_API int tron_profile_enable(tron_dataset *ds, int on);
TRON_API int tron_profile_read(tron_dataset *ds, int cap, const char **names, double *ms, int64_t *calls,
                               int *count);

/*
 * Streaming-read probe: sums `count` doubles at src_dev, every wavefront reading 12 KiB blocks of
 * consecutive bytes with twelve 16-byte loads per lane in flight (the access pattern of the dense
 * kernels), `reps` launches back to back, and returns the average milliseconds per launch measured
 * with HIP events.  Used to report the attainable HBM read rate next to the nominal peak.
 */
TRON_API int tron_probe_read_bandwidth(const double *src_dev, int64_t count, int reps, void *hip_stream,
                                       double *ms_per_launch, double *checksum);

/*
 * Process-wide tuning knobs, read when a dataset is created.  Results do not depend on them beyond
 * floating-point summation order.
 *   "csr_parts": column partitions of the two CSR layouts: 0 = automatic (8 when the gathered
 *                vector would not stay resident in one L2, else 1), 1 = never partition, 8 = always.
 *   "csr_segmented" (-1/0/1): unpartitioned layouts as row segments + flag bits (summed by scans) instead of plain CSR
 *                (one lane group per row): 0 never, 1 always, -1 (default) when some chunk of the plain layout would
 *                leave a single thread a row of about a hundred entries or more.
 * Partitioned layouts only:
 *   "csr_hot" (0/1): LDS tables of frequent columns in the forward layout;
 *   "csr_head" (0/1): a head partition for the most frequent columns of the whole matrix (needs csr_hot);
 *   "csr_range_slots" (2..4096): LDS table entries per column range;
 *   "csr_tiles" (0/1): hot-row tiles for the transposed product;
 *   "csr_unit" (0/1): layouts without a value stream when every instance's entries share one value;
 *   "csr_sell" (0/1), "csr_sell_blocks" (1..4096): such a layout keeps its head partition as sorted slices of 64 rows,
 *                one row per lane, over the 16384 most frequent columns (0: as chunks like the other partitions, over
 *                4096 columns); a quarter of the number of wavefronts the slices are dealt to;
 *   "csr_hot_blocks_per_part", "csr_range_blocks_per_part", "csr_blocks_per_part",
 *   "csr_tile_blocks_per_slice": persistent workgroups of the head, table, table-less and tile kernels.
 * "cg_speculate" (-1/0/1), read at every solve: the host-driven CG loop enqueues the kernels of iteration k + 1 before it
 *                has read the scalars of iteration k (1), or only after (0); -1: ahead when a Hessian-vector product moves
 *                at most 64 MB.  Same iterates either way: the kernels of an iteration that turns out not to exist change nothing.
 *                Under the same setting the outer loop forms the sparse gradient at a trial point before it knows whether
 *                the step is accepted (a rejected step leaves it unused; n_grad counts accepted steps' gradients only).
 * "fuse_reductions" (-1/0/1), read at every call: the second stage of every two-stage reduction (sum of the
 *   per-workgroup partial sums) is done by the workgroup of the producing kernel that finishes last (found through a ticket
 *   counter; the sums themselves are added in a fixed order, so results do not change) instead of by a launch of its own:
 *   0 never, 1 always, -1 (default) for launches of up to 32 workgroups (vectors of up to 32768 elements).
 *   (The step and direction kernels of the CG loop are outside this setting: with up to 512 workgroups each adds up the
 *   other's partial sums itself, in that same order; above, a launch does it.)
 * "dense_compact" (-1/0/1): L2-SVM on a dense matrix with d <= 32: Hessian-vector products run over a compacted copy of the
 *   active rows, X_I of Section 5 of the paper, built on the device (up to n*d more doubles of device memory): 0 never (the
 *   pass over X skips inactive rows instead), 1 whenever some rows are inactive (tron_fun_grad then builds the copy for the
 *   tron_hv calls that follow), -1 (default) inside tron_solve when at most 60% of the rows are active and the last inner
 *   solve took at least ten products.  Read at call time, not at creation.
 * "dense_device_driver" (-1/0/1): tron_solve on a dense matrix with d <= 32 and no preconditioner runs its trust-region and
 *   CG steps on the device (as tron_batch_solve does): 0 never, 1 always, -1 (default) for the L2-SVM on matrices up to 1 GB.
 * "batch_grid" (0..4096): workgroups of the multi-problem pass (0 = as many as are resident at once).
 * "batch_mfma_rows" (0/32/64): rows of X a wavefront of the matrix-unit pass keeps in LDS at a time (0: 32, except 64
 *                in the L2-SVM's rounds without function / gradient requests).
 * "batch_lean" (0/1, default 1): batches created afterwards run a round of the matrix-unit pass in which no problem asks
 *                for function and gradient (the Hessian-vector calls; inside tron_batch_solve the rounds right after the
 *                host has looked at the problems' requests) with a kernel compiled without the loss terms of such
 *                requests: fewer registers, so more wavefronts per SIMD.
 * "batch_mfma" (-1/0/1): batches created afterwards run the multi-problem pass on the fp64 matrix units (1), or on the
 *                vector units where those can hold the batch, i.e. up to eight problems (0); -1 (default): per loss,
 *                the matrix units from eight problems on for the L2-SVM and from five on for the logistic loss.
 * Unknown names or values return TRON_EINVAL.
 */
TRON_API int tron_tuning_set(const char *name, int64_t value);

/*
 * Plain copy probe: dst[i] = src[i] for `count` doubles, `reps` launches, average milliseconds per
 * launch.  A kernel of known read and write size: the yardstick the hardware byte counters
 * (FETCH_SIZE / WRITE_SIZE) are scaled with.
 */
TRON_API int tron_probe_copy_bandwidth(double *dst_dev, const double *src_dev, int64_t count, int reps,
                                       void *hip_stream, double *ms_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* TRON_H_ */
