// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/tron.h"

namespace tron {

// ---------------------------------------------------------------- errors
void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
int hip_fail(hipError_t e, const char *what, const char *file, int line);

#define TRON_HIP(expr)                                                        \
    do {                                                                      \
        hipError_t e__ = (expr);                                              \
        if (e__ != hipSuccess) return ::tron::hip_fail(e__, #expr, __FILE__, __LINE__); \
    } while (0)

#define TRON_TRY(expr)            \
    do {                          \
        int rc__ = (expr);        \
        if (rc__ < 0) return rc__; \
    } while (0)

// ---------------------------------------------------------------- launch geometry
constexpr int kBlock = 256;          // threads per workgroup everywhere (4 wavefronts of 64)
constexpr int kWave = 64;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxGrid = 2048;       // 256 CUs x 8 resident workgroups: grid-stride kernels use at most this
constexpr int kChunk = 2048;         // nonzeros per workgroup in the CSR kernels (256 threads x 8)
constexpr int kScalars = 16;         // scalar slots shared by the reductions

// ---------------------------------------------------------------- profiling slots
enum Slot {
    SLOT_SPMV_FWD_Z = 0,   // z = X w
    SLOT_SPMV_FWD_A1,      // a1 = D .* (X v)
    SLOT_SPMV_BWD_G,       // g = w + C X^T zhat
    SLOT_SPMV_BWD_HV,      // Hv = v + C X^T a1
    SLOT_SPMV_FIXUP,       // rows split across workgroups
    SLOT_LOSS_TERMS,       // zhat, D, sum loss from z
    SLOT_DENSE_FUN_GRAD,   // fused dense z / loss / D / X^T zhat
    SLOT_DENSE_HV,         // fused dense X^T (D (X v))
    SLOT_DENSE_FINALIZE,   // column sums of per-workgroup partials
    SLOT_DOT,              // dot products / norms (first stage)
    SLOT_REDUCE_FINAL,     // second reduction stage -> scalars
    SLOT_CG_VEC,           // CG vector updates
    SLOT_COUNT
};
extern const char *const kSlotNames[SLOT_COUNT];

struct Profiler {
    bool on = false;
    struct Rec { hipEvent_t a, b; int slot; };
    std::vector<Rec> pool;     // created lazily, reused
    size_t used = 0;
    double ms[SLOT_COUNT] = {0};
    int64_t calls[SLOT_COUNT] = {0};
    int begin(int slot, hipStream_t st);   // returns index or -1
    void end(int idx, hipStream_t st);
    int drain();                            // sync events, accumulate, reset used
    void destroy();
};

// ---------------------------------------------------------------- CSR work partition
// One orientation of the sparse matrix (rows x cols) with the nnz-balanced partition the SpMV
// kernel uses: workgroup b streams nonzeros [b*kChunk, (b+1)*kChunk) and owns the rows that
// *start* in that range, rows [row_lo[b], row_lo[b+1]).  A row that continues into later chunks
// gets the remainder through `carry` and the fix-up list.
struct CsrPlan {
    int64_t rows = 0, cols = 0, nnz = 0;
    int64_t *rowptr = nullptr;   // device, rows+1
    int32_t *col = nullptr;      // device, nnz
    double *val = nullptr;       // device, nnz
    int nblocks = 0;
    int32_t *row_lo = nullptr;   // device, nblocks+1
    double *carry = nullptr;     // device, nblocks: partial sum of the row entering chunk b from before
    int nfix = 0;                // number of split rows
    int32_t *fix_row = nullptr;  // device, nfix: the split row
    int32_t *fix_b0 = nullptr;   // device, nfix: first chunk holding a continuation of it
    int32_t *fix_cnt = nullptr;  // device, nfix: number of consecutive chunks that do
    void release();
};

}  // namespace tron

// ---------------------------------------------------------------- the handle
struct tron_dataset {
    int64_t n = 0, d = 0;
    bool dense = false;
    hipStream_t stream = nullptr;
    int device = 0;

    // dense
    double *X = nullptr;
    // sparse: forward (n x d) and explicit transposed (d x n) copies
    tron::CsrPlan fwd, bwd;

    double *y = nullptr;         // n
    double *z = nullptr;         // n   (sparse: margins X w; also a0 / a1 work space for Hv)
    double *zhat = nullptr;      // n   (sparse only; dense folds it into the fused pass)
    double *Dbuf[2] = {nullptr, nullptr};  // n each: D at the accepted w and at the trial point
    int Dcur = 0;
    bool have_D = false;

    // reductions
    double *partials = nullptr;  // device scratch for first-stage partial sums
    int64_t partials_len = 0;
    double *scal_dev = nullptr;  // kScalars device scalars
    double *scal_host = nullptr; // kScalars pinned host scalars
    int dense_grid = 0;          // workgroups of the dense kernels
    int vec_grid_n = 0, vec_grid_d = 0;  // workgroups of elementwise kernels over n / d

    // solver vectors (d each), allocated on first tron_solve
    double *sv[8] = {nullptr};

    tron::Profiler prof;
};

namespace tron {

// RAII bracket used by the launch helpers
struct ProfScope {
    tron_dataset *ds; int idx;
    ProfScope(tron_dataset *d, int slot) : ds(d), idx(d->prof.on ? d->prof.begin(slot, d->stream) : -1) {}
    ~ProfScope() { if (idx >= 0) ds->prof.end(idx, ds->stream); }
};

// ---- kernels_vec.hip
// out_scal[s] = sum of partials[s*stride .. s*stride+count) for s < nslots (second stage)
int reduce_final(tron_dataset *ds, int nslots, int count, int stride, int first_scalar);
// partial sums of a.b (and optionally c.e, f.h) into partial slots 0..k-1; returns #partials per slot
int dot_partials(tron_dataset *ds, int64_t m, const double *a0, const double *b0, const double *a1, const double *b1,
                 const double *a2, const double *b2);
int loss_terms(tron_dataset *ds, int loss, const double *z, double *zhat, double *D);  // partial slot 0 = sum loss
int read_scalars(tron_dataset *ds, int count);  // D2H of scal_dev[0..count) + stream sync
// CG vector kernels (see solver.hip)
int cg_init(tron_dataset *ds, const double *g, double *s, double *r, double *p);
int cg_step(tron_dataset *ds, double alpha, const double *p, const double *Hp, double *s, double *r);  // slot0 = r.r
int cg_dir(tron_dataset *ds, double beta, const double *r, const double *s, double *p);  // slots: p.p, s.p, s.s
int trial_point(tron_dataset *ds, const double *w, const double *s, const double *g, const double *r,
                double *wnew);  // wnew = w+s; slots: g.s, s.r, s.s
int probe_read(const double *src, int64_t count, int reps, hipStream_t st, double *ms, double *checksum);

// ---- kernels_csr.hip
int csr_plan_build(CsrPlan &P, int64_t rows, int64_t cols, const int64_t *h_rowptr, const int32_t *h_col,
                   const double *h_val, hipStream_t st);
enum { EPI_PLAIN = 0, EPI_SCALE = 1, EPI_AXPY = 2 };
// y[r] = epilogue( sum_k val[k] x[col[k]] ):  PLAIN: sum;  SCALE: scale[r]*sum;  AXPY: add[r] + alpha*sum
int csr_spmv(tron_dataset *ds, const CsrPlan &P, int slot, int epi, const double *x, double *yout,
             const double *scale_or_add, double alpha);

// ---- kernels_dense.hip
bool dense_supported(int64_t d);
int dense_grid_for(int64_t n, int64_t d);
int64_t dense_partials_needed(int64_t n, int64_t d);
// fused pass: z = X w, loss terms, D -> Dout, partial sums of X^T zhat and of the loss;
// then g = w + C (column sums) (if g != null), scalars[0] = sum loss, [1] = w.w, [2] = g.g
int dense_fun_grad(tron_dataset *ds, int loss, double C, const double *w, double *Dout, double *g);
// Hv = v + C X^T (D (X v)); scalars[0] = v.Hv
int dense_hv(tron_dataset *ds, double C, const double *D, const double *v, double *Hv);

// ---- solver.hip
int fun_eval(tron_dataset *ds, int loss, double C, const double *w, int Dslot, double *f_out);  // syncs
int grad_eval(tron_dataset *ds, double C, const double *w, double *g, double *gnorm_out);        // syncs
int hv_enqueue(tron_dataset *ds, double C, const double *v, double *Hv);                         // scalars[0]=v.Hv, no sync

}  // namespace tron
