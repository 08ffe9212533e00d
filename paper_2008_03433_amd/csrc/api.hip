// C ABI entry points: dataset handles, argument checking, profiling, error text.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <exception>
#include <new>
#include <thread>

#include "common.h"

namespace tron {

Tuning g_tuning;

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char *what, const char *file, int line)
{
    const char *base = strrchr(file, '/');
    set_error("HIP error %d (%s) in %s at %s:%d", (int)e, hipGetErrorString(e), what, base ? base + 1 : file, line);
    return (e == hipErrorOutOfMemory) ? TRON_ENOMEM : TRON_EDEVICE;
}

// ------------------------------------------------------------------ profiler
const char *const kSlotNames[SLOT_COUNT] = {
    "spmv_fwd", "spmv_bwd", "spmv_head", "spmv_tiles", "spmv_tile_reduce", "spmv_gather", "spmv_fixup", "spmv_combine", "loss_terms",
    "dense_fun_grad", "dense_hv", "dense_finalize", "dense_compact", "dot", "reduce_final", "cg_vec", "batch_pass", "batch_advance"};

int Profiler::begin(int slot, hipStream_t st)
{
    if (used == pool.size()) {
        Rec r;
        if (hipEventCreate(&r.a) != hipSuccess) return -1;
        if (hipEventCreate(&r.b) != hipSuccess) { hipEventDestroy(r.a); return -1; }
        r.slot = slot;
        pool.push_back(r);
    }
    Rec &r = pool[used];
    r.slot = slot;
    if (hipEventRecord(r.a, st) != hipSuccess) return -1;
    return (int)used++;
}

void Profiler::end(int idx, hipStream_t st) { hipEventRecord(pool[idx].b, st); }

int Profiler::drain()
{
    for (size_t i = 0; i < used; ++i) {
        Rec &r = pool[i];
        TRON_HIP(hipEventSynchronize(r.b));
        float t = 0.f;
        TRON_HIP(hipEventElapsedTime(&t, r.a, r.b));
        ms[r.slot] += t;
        calls[r.slot] += 1;
    }
    used = 0;
    return TRON_OK;
}

void Profiler::destroy()
{
    for (auto &r : pool) { hipEventDestroy(r.a); hipEventDestroy(r.b); }
    pool.clear();
    used = 0;
}

// ------------------------------------------------------------------ helpers
static int check_device()
{
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || count < 1) {
        set_error("no usable HIP device (%s); this library has no CPU fallback", hipGetErrorString(e));
        (void)hipGetLastError();
        return TRON_EDEVICE;
    }
    return TRON_OK;
}

static int vec_grid_for(int64_t m)
{
    int64_t g = (m + kBlock * 4 - 1) / (kBlock * 4);
    if (g < 1) g = 1;
    if (g > kMaxGrid) g = kMaxGrid;
    return (int)g;
}

static int alloc_common(tron_dataset *ds)
{
    const int64_t n = ds->n;
    TRON_HIP(hipGetDevice(&ds->device));
    if (ds->dense) TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->y8), (size_t)n));
    else TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->y), sizeof(double) * n));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->Dbuf[0]), sizeof(double) * n));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->Dbuf[1]), sizeof(double) * n));
    if (!ds->dense) {
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->z), sizeof(double) * n));
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->zhat), sizeof(double) * n));
    }
    int64_t need = 4 * (int64_t)kMaxGrid;
    if (ds->dense) {
        ds->dense_grid = dense_grid_for(ds->n, ds->d);
        const int64_t dn = dense_partials_needed(ds->n, ds->d);
        if (dn > need) need = dn;
    }
    ds->partials_len = need;
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->partials), sizeof(double) * need));
    // The scalars the host steers by live in pinned host memory that the kernels write directly: they are there when
    // the stream has drained, without a copy operation between the last kernel and the host's wait.
    TRON_HIP(hipHostMalloc(reinterpret_cast<void **>(&ds->scal_host), sizeof(double) * kScalars, hipHostMallocMapped));
    TRON_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&ds->scal_dev), ds->scal_host, 0));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->scal_copy), sizeof(double) * kScalars));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->ticket), 64));
    TRON_HIP(hipMemset(ds->ticket, 0, 64));
    ds->vec_grid_n = vec_grid_for(ds->n);
    ds->vec_grid_d = vec_grid_for(ds->d);
    return TRON_OK;
}

static int check_labels(const double *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        if (!(y[i] == 1.0 || y[i] == -1.0)) {
            set_error("y[%lld] = %g is not +1 or -1", (long long)i, y[i]);
            return TRON_EINVAL;
        }
    return TRON_OK;
}

// host copies of caller arrays (from host or device memory)
template <typename T>
static int fetch(std::vector<T> &dst, const T *src, size_t count, int mem)
{
    try {
        dst.resize(count);
    } catch (const std::bad_alloc &) {
        set_error("out of host memory staging %zu elements", count);
        return TRON_ENOMEM;
    }
    if (!count) return TRON_OK;
    if (mem == TRON_MEM_DEVICE)
        TRON_HIP(hipMemcpy(dst.data(), src, sizeof(T) * count, hipMemcpyDeviceToHost));
    else
        memcpy(dst.data(), src, sizeof(T) * count);
    return TRON_OK;
}

}  // namespace tron

using namespace tron;

// =================================================================== ABI
extern "C" {

const char *tron_last_error(void) { return g_err; }

void tron_dataset_destroy(tron_dataset *ds)
{
    if (!ds) return;
    hipStreamSynchronize(ds->stream);
    dense_device_release(ds);
    dense_compact_release(ds);
    hipFree(ds->X);
    ds->fwd.release();
    ds->bwd.release();
    hipFree(ds->y); hipFree(ds->y8); hipFree(ds->z); hipFree(ds->zhat); hipFree(ds->Dbuf[0]); hipFree(ds->Dbuf[1]);
    hipFree(ds->partials); hipFree(ds->row_partials); hipFree(ds->unit_scale); hipFree(ds->scal_copy); hipFree(ds->ticket);
    if (ds->scal_host) hipHostFree(ds->scal_host);
    for (double *p : ds->sv) hipFree(p);
    for (hipEvent_t e : ds->cg_event)
        if (e) hipEventDestroy(e);
    hipFree(ds->cg_partials);
    ds->prof.destroy();
    delete ds;
}

int tron_dataset_create_csr(int64_t n, int64_t d, const int64_t *rowptr, const int32_t *col, const double *val,
                            const double *y, int mem, void *hip_stream, tron_dataset **out)
{
    if (out) *out = nullptr;
    // the sparse kernels address the gathered vectors through 32-bit byte offsets: n, d < 2^29
    if (!out || !rowptr || !y || n < 1 || d < 1 || n >= (1 << 29) || d >= (1 << 29) ||
        (mem != TRON_MEM_HOST && mem != TRON_MEM_DEVICE)) {
        set_error("tron_dataset_create_csr: bad argument (need 1 <= n,d < 2^29, non-null rowptr/y/out, mem in {0,1})");
        return TRON_EINVAL;
    }
    TRON_TRY(check_device());
    std::vector<int64_t> h_rowptr;
    TRON_TRY(fetch(h_rowptr, rowptr, (size_t)n + 1, mem));
    if (h_rowptr[0] != 0) { set_error("rowptr[0] = %lld, expected 0", (long long)h_rowptr[0]); return TRON_EINVAL; }
    for (int64_t i = 0; i < n; ++i)
        if (h_rowptr[i + 1] < h_rowptr[i]) { set_error("rowptr decreases at row %lld", (long long)i); return TRON_EINVAL; }
    const int64_t nnz = h_rowptr[n];
    if (nnz > 0 && (!col || !val)) { set_error("col/val are null but nnz = %lld", (long long)nnz); return TRON_EINVAL; }
    std::vector<int32_t> h_col;
    std::vector<double> h_val, h_y;
    TRON_TRY(fetch(h_col, col, (size_t)nnz, mem));
    TRON_TRY(fetch(h_val, val, (size_t)nnz, mem));
    TRON_TRY(fetch(h_y, y, (size_t)n, mem));
    TRON_TRY(check_labels(h_y.data(), n));
    // columns strictly increasing inside each row and in range; values finite; count per column
    std::vector<int64_t> t_rowptr;
    try {
        t_rowptr.assign((size_t)d + 1, 0);
    } catch (const std::bad_alloc &) { set_error("out of host memory"); return TRON_ENOMEM; }
    for (int64_t i = 0; i < n; ++i) {
        int64_t prev = -1;
        for (int64_t k = h_rowptr[i]; k < h_rowptr[i + 1]; ++k) {
            const int64_t c = h_col[k];
            if (c <= prev || c >= d) {
                set_error("row %lld: column index %lld out of order or out of range [0,%lld)", (long long)i, (long long)c, (long long)d);
                return TRON_EINVAL;
            }
            if (!std::isfinite(h_val[k])) { set_error("row %lld: non-finite value", (long long)i); return TRON_EINVAL; }
            prev = c;
            t_rowptr[c + 1] += 1;
        }
    }
    // Unit plans: when both layouts are partitioned and every instance's entries share one value r_i (binary features,
    // optionally scaled per instance, e.g. normalised to unit length), X = diag(r) B with B binary: the layouts keep no
    // values, the row sums of X are multiplied by r afterwards and X^T gathers from r .* (its vector).
    const bool fwd_partitioned = g_tuning.csr_parts == kColParts ||
                                 (g_tuning.csr_parts == 0 && d * (int64_t)sizeof(double) > (3 << 19) && nnz >= (1 << 22));
    const bool bwd_partitioned = g_tuning.csr_parts == kColParts ||
                                 (g_tuning.csr_parts == 0 && n * (int64_t)sizeof(double) > (3 << 19) && nnz >= (1 << 22));
    bool unit = g_tuning.csr_unit != 0 && fwd_partitioned && bwd_partitioned;
    std::vector<double> row_value;
    if (unit) {
        try {
            row_value.assign((size_t)n, 1.0);
        } catch (const std::bad_alloc &) { set_error("out of host memory"); return TRON_ENOMEM; }
        for (int64_t i = 0; i < n && unit; ++i) {
            const int64_t k0 = h_rowptr[i], k1 = h_rowptr[i + 1];
            if (k1 > k0) row_value[i] = h_val[k0];
            for (int64_t k = k0 + 1; k < k1; ++k)
                if (h_val[k] != h_val[k0]) { unit = false; break; }
        }
    }
    // Hot-row tiles for the transposed product of large matrices: the features with the most entries (rank r by
    // count -> slice r % 8, slot r / 8) leave the transposed CSR copy and are stored as tiles instead.
    std::vector<int32_t> slot_code;
    int nhot = 0;
    const bool partitioned = bwd_partitioned;
    if (g_tuning.csr_tiles && partitioned) {
        std::vector<std::pair<int64_t, int32_t>> cand;
        for (int64_t j = 0; j < d; ++j)
            if (t_rowptr[j + 1] >= kTileMinCount) cand.emplace_back(-t_rowptr[j + 1], (int32_t)j);
        size_t keep = std::min<size_t>(cand.size(), (size_t)kTileSlices * kTileSlots);
        std::partial_sort(cand.begin(), cand.begin() + keep, cand.end());
        // A tile spans at most kTileWindow instances, so a slice has about n / kTileWindow of them however few entries
        // they hold, and a tile costs the kernel about as much as 400 entries cost the range kernels: where there are
        // many tiles they must be at least a quarter full on average, or the features stay in the CSR copy.
        {
            int64_t entries = 0;
            for (size_t r = 0; r < keep; ++r) entries -= cand[r].first;
            const int64_t windows = (n + kTileWindow - 1) / kTileWindow * kTileSlices;
            if (windows > 4096 && entries < windows * (kChunk / 4)) keep = 0;
        }
        if (keep > 0) {
            slot_code.assign((size_t)d, -1);
            for (size_t r = 0; r < keep; ++r) {
                slot_code[cand[r].second] = (int32_t)((r % kTileSlices) * kTileSlots + r / kTileSlices);
                t_rowptr[cand[r].second + 1] = 0;   // no entries of this feature in the CSR copy
            }
            nhot = (int)keep;
        }
    }
    // explicit transposed copy (d x n): counting sort by column keeps rows ascending inside each column
    for (int64_t j = 0; j < d; ++j) t_rowptr[j + 1] += t_rowptr[j];
    const int64_t t_nnz = t_rowptr[d];
    std::vector<int32_t> t_col;
    std::vector<double> t_val;
    std::vector<int64_t> cursor;
    try {
        t_col.resize((size_t)t_nnz);
        if (!unit) t_val.resize((size_t)t_nnz);
        cursor.assign(t_rowptr.begin(), t_rowptr.end() - 1);
    } catch (const std::bad_alloc &) { set_error("out of host memory building the transposed copy"); return TRON_ENOMEM; }
    {
        // One host thread per range of features (equal shares of the copy's entries): every thread walks the whole matrix
        // and places the entries of its own features, so the instances stay in ascending order inside a feature and no
        // two threads touch the same cursor.
        unsigned T = std::max(1u, std::min(8u, std::thread::hardware_concurrency()));
        if (t_nnz < (1 << 20)) T = 1;
        std::vector<int64_t> bound(T + 1, d);
        bound[0] = 0;
        for (unsigned t = 1; t < T; ++t)
            bound[t] = std::lower_bound(t_rowptr.begin(), t_rowptr.end(), t_nnz / T * t) - t_rowptr.begin();
        for (unsigned t = 1; t <= T; ++t) bound[t] = std::min<int64_t>(d, std::max(bound[t], bound[t - 1]));
        bound[T] = d;
        auto place = [&](int64_t c0, int64_t c1) {
            if (c0 >= c1) return;
            for (int64_t i = 0; i < n; ++i)
                for (int64_t k = h_rowptr[i]; k < h_rowptr[i + 1]; ++k) {
                    const int64_t c = h_col[k];
                    if (c < c0) continue;
                    if (c >= c1) break;   // columns ascend inside a row
                    if (nhot && slot_code[c] >= 0) continue;
                    const int64_t pos = cursor[c]++;
                    t_col[pos] = (int32_t)i;
                    if (!unit) t_val[pos] = h_val[k];
                }
        };
        std::vector<std::thread> workers;
        unsigned started = 0;
        try {
            for (unsigned t = 1; t < T; ++t) { workers.emplace_back(place, bound[t], bound[t + 1]); ++started; }
        } catch (const std::exception &) {
            // no more threads to be had: the remaining ranges run below
        }
        place(bound[0], bound[1]);
        for (unsigned t = 1 + started; t < T; ++t) place(bound[t], bound[t + 1]);
        for (std::thread &w : workers) w.join();
    }

    tron_dataset *ds = new (std::nothrow) tron_dataset();
    if (!ds) { set_error("out of host memory"); return TRON_ENOMEM; }
    ds->n = n; ds->d = d; ds->dense = false; ds->stream = reinterpret_cast<hipStream_t>(hip_stream);
    int rc = alloc_common(ds);
    if (rc >= 0) rc = csr_plan_build(ds->fwd, n, d, h_rowptr.data(), h_col.data(), unit ? nullptr : h_val.data(),
                                     fwd_partitioned ? kColParts : 1, g_tuning.csr_hot != 0, unit, ds->stream);
    if (rc >= 0) rc = csr_plan_build(ds->bwd, d, n, t_rowptr.data(), t_col.data(), unit ? nullptr : t_val.data(), partitioned ? kColParts : 1,
                                     false, unit, ds->stream);
    if (rc >= 0 && nhot) rc = hot_tiles_build(ds->bwd, h_rowptr.data(), h_col.data(), h_val.data(), slot_code, nhot, ds->stream);
    if (rc >= 0 && unit) {
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&ds->unit_scale), sizeof(double) * (size_t)n);
        if (e == hipSuccess) e = hipMemcpyAsync(ds->unit_scale, row_value.data(), sizeof(double) * (size_t)n, hipMemcpyHostToDevice, ds->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ds->stream);
        if (e != hipSuccess) rc = hip_fail(e, "copy the instances' values", __FILE__, __LINE__);
        ds->fwd.row_scale = ds->unit_scale;
        ds->bwd.col_scale = ds->unit_scale;
    }
    if (rc >= 0) {
        int64_t need = 0;
        if (!ds->fwd.plain) need = std::max<int64_t>(need, ds->fwd.nseg_total);   // one partial sum per segment
        if (!ds->bwd.plain) need = std::max<int64_t>(need, ds->bwd.nseg_total);
        if (need > 0) {
            hipError_t e = hipMalloc(reinterpret_cast<void **>(&ds->row_partials), sizeof(double) * need);
            if (e != hipSuccess) rc = hip_fail(e, "allocate row partials", __FILE__, __LINE__);
        }
    }
    if (rc >= 0) {
        hipError_t e = hipMemcpyAsync(ds->y, h_y.data(), sizeof(double) * n, hipMemcpyHostToDevice, ds->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ds->stream);
        if (e != hipSuccess) rc = hip_fail(e, "copy y", __FILE__, __LINE__);
    }
    if (rc < 0) { tron_dataset_destroy(ds); return rc; }
    *out = ds;
    return TRON_OK;
}

int tron_dataset_create_dense_empty(int64_t n, int64_t d, void *hip_stream, tron_dataset **out)
{
    if (out) *out = nullptr;
    if (!out || n < 1 || d < 1 || n > 0x7ffffff0) {
        set_error("tron_dataset_create_dense_empty: bad argument (need 1 <= n < 2^31, d >= 1, non-null out)");
        return TRON_EINVAL;
    }
    if (!dense_supported(d)) { set_error("dense d = %lld not supported (1 <= d <= 512)", (long long)d); return TRON_EINVAL; }
    TRON_TRY(check_device());
    tron_dataset *ds = new (std::nothrow) tron_dataset();
    if (!ds) { set_error("out of host memory"); return TRON_ENOMEM; }
    ds->n = n; ds->d = d; ds->dense = true; ds->stream = reinterpret_cast<hipStream_t>(hip_stream);
    int rc = alloc_common(ds);
    if (rc >= 0) {
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&ds->X), sizeof(double) * (size_t)n * (size_t)d);
        if (e != hipSuccess) rc = hip_fail(e, "allocate X", __FILE__, __LINE__);
    }
    if (rc < 0) { tron_dataset_destroy(ds); return rc; }
    *out = ds;
    return TRON_OK;
}

int tron_dataset_write_rows(tron_dataset *ds, int64_t row0, int64_t nrows, const double *X_chunk, const double *y_chunk, int mem)
{
    if (!ds || !ds->dense || !X_chunk || !y_chunk || row0 < 0 || nrows < 0 || row0 + nrows > ds->n ||
        (mem != TRON_MEM_HOST && mem != TRON_MEM_DEVICE)) {
        set_error("tron_dataset_write_rows: bad argument");
        return TRON_EINVAL;
    }
    if (nrows == 0) return TRON_OK;
    if (mem == TRON_MEM_HOST) {
        TRON_TRY(check_labels(y_chunk, nrows));
        for (int64_t k = 0; k < nrows * ds->d; ++k)
            if (!std::isfinite(X_chunk[k])) { set_error("X has a non-finite entry in row %lld", (long long)(row0 + k / ds->d)); return TRON_EINVAL; }
    } else {
        // the same checks on the device, before anything is copied
        int what = 0;
        TRON_TRY(dense_validate_device(ds, nrows, X_chunk, y_chunk, &what));
        if (what == 1) { set_error("a label in rows [%lld, %lld) is not +1 or -1", (long long)row0, (long long)(row0 + nrows)); return TRON_EINVAL; }
        if (what == 2) { set_error("X has a non-finite entry in rows [%lld, %lld)", (long long)row0, (long long)(row0 + nrows)); return TRON_EINVAL; }
    }
    const hipMemcpyKind kind = (mem == TRON_MEM_HOST) ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice;
    TRON_HIP(hipMemcpyAsync(ds->X + row0 * ds->d, X_chunk, sizeof(double) * (size_t)nrows * (size_t)ds->d, kind, ds->stream));
    std::vector<int8_t> y8;
    if (mem == TRON_MEM_HOST) {
        y8.resize((size_t)nrows);
        for (int64_t i = 0; i < nrows; ++i) y8[i] = (y_chunk[i] > 0.0) ? 1 : -1;
        TRON_HIP(hipMemcpyAsync(ds->y8 + row0, y8.data(), (size_t)nrows, hipMemcpyHostToDevice, ds->stream));
    } else {
        TRON_TRY(dense_labels_from_device(ds, row0, nrows, y_chunk));
    }
    TRON_HIP(hipStreamSynchronize(ds->stream));  // the caller may reuse its buffers on return
    ds->have_D = false;
    return TRON_OK;
}

int tron_dataset_create_dense(int64_t n, int64_t d, const double *X_rowmajor, const double *y, int mem, void *hip_stream,
                              tron_dataset **out)
{
    if (out) *out = nullptr;
    if (!out || !X_rowmajor || !y) { set_error("tron_dataset_create_dense: null argument"); return TRON_EINVAL; }
    tron_dataset *ds = nullptr;
    TRON_TRY(tron_dataset_create_dense_empty(n, d, hip_stream, &ds));
    int rc = tron_dataset_write_rows(ds, 0, n, X_rowmajor, y, mem);
    if (rc < 0) { tron_dataset_destroy(ds); return rc; }
    *out = ds;
    return TRON_OK;
}

int tron_dataset_shape(const tron_dataset *ds, int64_t *n, int64_t *d, int64_t *nnz, int *is_dense)
{
    if (!ds) { set_error("tron_dataset_shape: null handle"); return TRON_EINVAL; }
    if (n) *n = ds->n;
    if (d) *d = ds->d;
    if (nnz) *nnz = ds->dense ? ds->n * ds->d : ds->fwd.nnz;
    if (is_dense) *is_dense = ds->dense ? 1 : 0;
    return TRON_OK;
}

int tron_dataset_stat(const tron_dataset *ds, const char *name, int64_t *value)
{
    if (!ds || !name || !value) { set_error("tron_dataset_stat: null argument"); return TRON_EINVAL; }
    // bytes per launch in the stored format (see PlanBytes); the Hessian-vector call adds the vectors of the call itself
    PlanBytes fb{0, 0, 0, 0, 0, 0}, bb{0, 0, 0, 0, 0, 0};
    int64_t hv_bytes = 0, fun_grad_bytes = 0;
    if (ds->dense) {
        // X once (the active rows only when the pass skips the others), D or the active-set bits / bytes, per-workgroup sums
        const int slot = ds->Dcur;
        const bool mask = ds->have_D && ds->D_is_mask[slot];
        const double frac = (mask && ds->active_frac[slot] < 0.95) ? ds->active_frac[slot] : 1.0;
        const int64_t dbytes = !mask ? 8 * ds->n : (ds->d <= 32 ? ds->n / 8 : ds->n);
        hv_bytes = (int64_t)(8.0 * frac * (double)ds->n * (double)ds->d) + dbytes + 8 * ds->d * ds->dense_grid;
        if (ds->have_D && ds->hat_slot == slot)   // the pass runs over the compacted copy
            hv_bytes = 8 * ds->hat_rows * ds->d + ds->hat_rows / 8 + 8 * ds->d * dense_grid_for(ds->hat_rows, ds->d);
        fun_grad_bytes = 8 * ds->n * ds->d + ds->n /* labels */ + dbytes + 8 * ds->d * ds->dense_grid;
    } else {
        fb = plan_bytes(ds->fwd);
        bb = plan_bytes(ds->bwd);
        hv_bytes = fb.gather + fb.head + fb.ranges + fb.combine + 8 * ds->n /* D */ +
                   bb.tiles + bb.tile_reduce + bb.ranges + bb.combine + 8 * ds->d /* v as addend */;
        fun_grad_bytes = hv_bytes + 8 * ds->n /* y */ + 8 * ds->n /* zhat and D both written */;
    }
    struct { const char *k; int64_t v; } tab[] = {
        {"fwd_bytes_gather", fb.gather}, {"fwd_bytes_head", fb.head}, {"fwd_bytes_ranges", fb.ranges}, {"fwd_bytes_combine", fb.combine},
        {"bwd_bytes_tiles", bb.tiles}, {"bwd_bytes_tile_reduce", bb.tile_reduce}, {"bwd_bytes_ranges", bb.ranges},
        {"bwd_bytes_combine", bb.combine}, {"hv_bytes", hv_bytes}, {"fun_grad_bytes", fun_grad_bytes},
        {"fwd_parts", ds->dense ? 0 : ds->fwd.P},
        {"bwd_parts", ds->dense ? 0 : ds->bwd.P},
        {"fwd_segmented", (ds->dense || ds->fwd.plain) ? 0 : 1},
        {"bwd_segmented", (ds->dense || ds->bwd.plain) ? 0 : 1},
        {"fwd_csr_nnz", ds->dense ? 0 : ds->fwd.nnz},
        {"fwd_head_nnz", (ds->dense || ds->fwd.head < 0) ? 0 : ds->fwd.part_nnz[ds->fwd.head]},
        {"bwd_csr_nnz", ds->dense ? 0 : ds->bwd.nnz},
        {"bwd_tile_nnz", ds->dense ? 0 : ds->bwd.hot.nnz},
        {"bwd_tile_rows", ds->dense ? 0 : ds->bwd.hot.nhot},
        {"bwd_tiles", ds->dense ? 0 : ds->bwd.hot.ntiles_total},
        {"fwd_lds_columns", ds->dense ? 0 : [&] { int64_t t = 0; for (int x = 0; x < kMaxParts; ++x) t += ds->fwd.part_nhot[x]; return t; }()},
        {"dense_grid", ds->dense_grid},
        {"dense_compact_rows", (ds->dense && ds->have_D && ds->hat_slot == ds->Dcur) ? ds->hat_rows : 0},
        {"unit_values", (!ds->dense && ds->fwd.unit) ? 1 : 0},
    };
    for (auto &e : tab)
        if (strcmp(e.k, name) == 0) { *value = e.v; return TRON_OK; }
    set_error("tron_dataset_stat: unknown name '%s'", name);
    return TRON_EINVAL;
}

int tron_fun_grad(tron_dataset *ds, int loss, double C, const double *w_dev, double *f_host, double *g_dev)
{
    if (!ds || !w_dev || !f_host || (loss != TRON_LOSS_LR && loss != TRON_LOSS_L2SVM) || !(C > 0.0) || !std::isfinite(C)) {
        set_error("tron_fun_grad: bad argument (null handle/w/f, unknown loss, or C <= 0)");
        return TRON_EINVAL;
    }
    const int slot = ds->have_D ? 1 - ds->Dcur : ds->Dcur;
    if (ds->dense) {
        TRON_TRY(dense_fun_grad(ds, loss, C, w_dev, slot, g_dev));
        TRON_TRY(read_scalars(ds, 4));
        ds->active_frac[slot] = ds->scal_host[3] / (double)ds->n;
        ds->active_count[slot] = (int64_t)ds->scal_host[3];
        *f_host = 0.5 * ds->scal_host[1] + C * ds->scal_host[0];
        // stand-alone calls: the compacted copy of the active rows only when the knob forces it
        if (g_tuning.dense_compact > 0 && dense_compact_wanted(ds, slot, 0)) TRON_TRY(dense_compact_build(ds, slot));
    } else {
        TRON_TRY(fun_eval(ds, loss, C, w_dev, slot, f_host));
        if (g_dev) {
            double gn;
            TRON_TRY(grad_eval(ds, C, w_dev, g_dev, &gn));
        }
    }
    ds->Dcur = slot;
    ds->have_D = true;
    return TRON_OK;
}

int tron_hv(tron_dataset *ds, double C, const double *v_dev, double *Hv_dev, double *vHv_host)
{
    if (!ds || !v_dev || !Hv_dev || v_dev == Hv_dev || !(C > 0.0) || !std::isfinite(C)) {
        set_error("tron_hv: bad argument (null handle/v/Hv, v aliases Hv, or C <= 0)");
        return TRON_EINVAL;
    }
    if (!ds->have_D) { set_error("tron_hv: no cached D; call tron_fun_grad first"); return TRON_ESTATE; }
    TRON_TRY(hv_enqueue(ds, C, v_dev, Hv_dev));
    if (vHv_host) {
        TRON_TRY(read_scalars(ds, 1));
        *vHv_host = ds->scal_host[0];
    }
    return TRON_OK;
}

int tron_profile_enable(tron_dataset *ds, int on)
{
    if (!ds) { set_error("tron_profile_enable: null handle"); return TRON_EINVAL; }
    TRON_HIP(hipStreamSynchronize(ds->stream));
    TRON_TRY(ds->prof.drain());
    ds->prof.on = on != 0;
    for (int s = 0; s < SLOT_COUNT; ++s) { ds->prof.ms[s] = 0; ds->prof.calls[s] = 0; }
    return TRON_OK;
}

int tron_profile_read(tron_dataset *ds, int cap, const char **names, double *ms, int64_t *calls, int *count)
{
    if (!ds || cap < 0) { set_error("tron_profile_read: bad argument"); return TRON_EINVAL; }
    TRON_HIP(hipStreamSynchronize(ds->stream));
    TRON_TRY(ds->prof.drain());
    for (int s = 0; s < SLOT_COUNT && s < cap; ++s) {
        if (names) names[s] = kSlotNames[s];
        if (ms) ms[s] = ds->prof.ms[s];
        if (calls) calls[s] = ds->prof.calls[s];
    }
    if (count) *count = SLOT_COUNT;
    for (int s = 0; s < SLOT_COUNT; ++s) { ds->prof.ms[s] = 0; ds->prof.calls[s] = 0; }
    return TRON_OK;
}

int tron_probe_read_bandwidth(const double *src_dev, int64_t count, int reps, void *hip_stream, double *ms_per_launch,
                              double *checksum)
{
    TRON_TRY(check_device());
    return probe_read(src_dev, count, reps, reinterpret_cast<hipStream_t>(hip_stream), ms_per_launch, checksum);
}

int tron_tuning_set(const char *name, int64_t value)
{
    if (name && strcmp(name, "csr_parts") == 0 && (value == 0 || value == 1 || value == kColParts)) {
        g_tuning.csr_parts = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_hot") == 0 && (value == 0 || value == 1)) {
        g_tuning.csr_hot = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_hot_blocks_per_part") == 0 && value >= 1 && value <= 4096) {
        g_tuning.csr_hot_blocks_per_part = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_range_slots") == 0 && value >= 2 && value <= kHotSlots) {
        g_tuning.csr_range_slots = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_range_blocks_per_part") == 0 && value >= 1 && value <= 1024) {
        g_tuning.csr_range_blocks_per_part = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_head") == 0 && (value == 0 || value == 1)) {
        g_tuning.csr_head = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_tiles") == 0 && (value == 0 || value == 1)) {
        g_tuning.csr_tiles = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_tile_blocks_per_slice") == 0 && value >= 0 && value <= 1024) {
        g_tuning.csr_tile_blocks_per_slice = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_blocks_per_part") == 0 && value >= 1 && value <= 4096) {
        g_tuning.csr_blocks_per_part = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_sell") == 0 && (value == 0 || value == 1)) {
        g_tuning.csr_sell = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_sell_blocks") == 0 && value >= 1 && value <= 4096) {
        g_tuning.csr_sell_blocks = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_segmented") == 0 && value >= -1 && value <= 1) {
        g_tuning.csr_segmented = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "csr_unit") == 0 && (value == 0 || value == 1)) {
        g_tuning.csr_unit = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "cg_speculate") == 0 && value >= -1 && value <= 1) {
        g_tuning.cg_speculate = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "fuse_reductions") == 0 && value >= -1 && value <= 1) {
        g_tuning.fuse_reductions = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "dense_compact") == 0 && value >= -1 && value <= 1) {
        g_tuning.dense_compact = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "dense_device_driver") == 0 && value >= -1 && value <= 1) {
        g_tuning.dense_device_driver = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "batch_grid") == 0 && value >= 0 && value <= 4096) {
        g_tuning.batch_grid = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "batch_mfma_rows") == 0 && (value == 0 || value == 32 || value == 64)) {
        g_tuning.batch_mfma_rows = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "batch_lean") == 0 && value >= 0 && value <= 1) {
        g_tuning.batch_lean = value;
        return TRON_OK;
    }
    if (name && strcmp(name, "batch_mfma") == 0 && value >= -1 && value <= 1) {
        g_tuning.batch_mfma = value;
        return TRON_OK;
    }
    set_error("tron_tuning_set: unknown knob or value out of range");
    return TRON_EINVAL;
}

int tron_probe_copy_bandwidth(double *dst_dev, const double *src_dev, int64_t count, int reps, void *hip_stream,
                              double *ms_per_launch)
{
    TRON_TRY(check_device());
    return probe_copy(dst_dev, src_dev, count, reps, reinterpret_cast<hipStream_t>(hip_stream), ms_per_launch);
}

}  // extern "C"
