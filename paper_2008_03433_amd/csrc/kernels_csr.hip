// CSR sparse matrix-vector products for both orientations (X and the explicit X^T copy):
//   z = X w,  a1 = D .* (X v)          (Table 1 / Appendix D of the paper: a0 = X v, a1 = D a0)
//   g = w + C X^T zhat,  Hv = v + C X^T a1   (a2 = C X^T a1)
//
// Work is split by nonzeros, not by rows, because row lengths are heavily skewed (Zipf-distributed
// features give the transposed copy rows of length ~n next to millions of length 0/1): workgroup b
// streams nonzeros [b*kChunk, (b+1)*kChunk) with fully coalesced 16-byte loads, multiplies them by the
// gathered vector entries and parks the products in LDS; the rows that start inside the chunk are then
// summed from LDS by lane groups sized to the number of such rows.  A row that runs past the end of
// its chunk receives the rest from the `carry` of the following chunks in a small fix-up kernel, in a
// fixed order -- no atomics anywhere, so results are bit-reproducible.
#include <algorithm>

#include "device_util.h"

namespace tron {

void CsrPlan::release()
{
    hipFree(rowptr); hipFree(col); hipFree(val); hipFree(row_lo); hipFree(carry);
    hipFree(fix_row); hipFree(fix_b0); hipFree(fix_cnt);
    *this = CsrPlan();
}

template <typename T>
static int upload(T **dst, const T *src, size_t count, hipStream_t st)
{
    *dst = nullptr;
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(dst), sizeof(T) * std::max<size_t>(count, 1)));
    if (count) TRON_HIP(hipMemcpyAsync(*dst, src, sizeof(T) * count, hipMemcpyHostToDevice, st));
    return TRON_OK;
}

int csr_plan_build(CsrPlan &P, int64_t rows, int64_t cols, const int64_t *h_rowptr, const int32_t *h_col,
                   const double *h_val, hipStream_t st)
{
    P.rows = rows;
    P.cols = cols;
    P.nnz = h_rowptr[rows];
    const int64_t nb64 = std::max<int64_t>(1, (P.nnz + kChunk - 1) / kChunk);
    if (nb64 > 0x7fffffff) { set_error("matrix too large: %lld chunks", (long long)nb64); return TRON_EINVAL; }
    P.nblocks = (int)nb64;

    // row_lo[b] = first row r with rowptr[r] >= b*kChunk; row_lo[nblocks] = rows
    std::vector<int32_t> row_lo(P.nblocks + 1);
    {
        int64_t r = 0;
        for (int b = 0; b < P.nblocks; ++b) {
            const int64_t start = (int64_t)b * kChunk;
            while (r < rows && h_rowptr[r] < start) ++r;
            row_lo[b] = (int32_t)r;
        }
        row_lo[0] = 0;
        row_lo[P.nblocks] = (int32_t)rows;
    }
    // split rows: chunk b (b >= 1) begins inside row row_lo[b]-1 iff rowptr[row_lo[b]] > b*kChunk
    std::vector<int32_t> fix_row, fix_b0, fix_cnt;
    for (int b = 1; b < P.nblocks; ++b) {
        const int64_t start = (int64_t)b * kChunk;
        const int64_t next_row_start = h_rowptr[row_lo[b]];  // rowptr[rows] = nnz when row_lo[b] == rows
        if (row_lo[b] >= 1 && next_row_start > start) {
            const int32_t row = row_lo[b] - 1;
            if (!fix_row.empty() && fix_row.back() == row) {
                fix_cnt.back() += 1;
            } else {
                fix_row.push_back(row);
                fix_b0.push_back(b);
                fix_cnt.push_back(1);
            }
        }
    }
    P.nfix = (int)fix_row.size();

    TRON_TRY(upload(&P.rowptr, h_rowptr, (size_t)rows + 1, st));
    TRON_TRY(upload(&P.col, h_col, (size_t)P.nnz, st));
    TRON_TRY(upload(&P.val, h_val, (size_t)P.nnz, st));
    TRON_TRY(upload(&P.row_lo, row_lo.data(), row_lo.size(), st));
    TRON_TRY(upload(&P.fix_row, fix_row.data(), fix_row.size(), st));
    TRON_TRY(upload(&P.fix_b0, fix_b0.data(), fix_b0.size(), st));
    TRON_TRY(upload(&P.fix_cnt, fix_cnt.data(), fix_cnt.size(), st));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&P.carry), sizeof(double) * P.nblocks));
    TRON_HIP(hipMemsetAsync(P.carry, 0, sizeof(double) * P.nblocks, st));
    TRON_HIP(hipStreamSynchronize(st));  // the host vectors above go out of scope
    return TRON_OK;
}

// ------------------------------------------------------------------ main kernel
template <int EPI>
__device__ __forceinline__ double epilogue(double sum, int64_t r, const double *__restrict__ aux, double alpha)
{
    if (EPI == EPI_PLAIN) return sum;
    if (EPI == EPI_SCALE) return aux[r] * sum;
    return fma(alpha, sum, aux[r]);
}

template <int EPI>
__global__ __launch_bounds__(kBlock) void k_csr_spmv(int64_t rows, int64_t nnz, const int64_t *__restrict__ rowptr,
                                                     const int32_t *__restrict__ col, const double *__restrict__ val,
                                                     const int32_t *__restrict__ row_lo, const double *__restrict__ x,
                                                     double *__restrict__ yout, const double *__restrict__ aux,
                                                     double alpha, double *__restrict__ carry)
{
    __shared__ __align__(16) double prod[kChunk];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t start = (int64_t)b * kChunk;
    const int64_t end = (start + kChunk < nnz) ? start + kChunk : nnz;  // this chunk is [start, end)

    // ---- phase 1: products into LDS (two passes of 1024 nonzeros, 4 per thread per pass)
    if (end - start == kChunk) {
        int4 c[2];
        double2 v[2][2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t k = start + j * (kChunk / 2) + tid * 4;
            c[j] = *reinterpret_cast<const int4 *>(col + k);
            v[j][0] = *reinterpret_cast<const double2 *>(val + k);
            v[j][1] = *reinterpret_cast<const double2 *>(val + k + 2);
        }
        double xg[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            xg[j][0] = x[c[j].x];
            xg[j][1] = x[c[j].y];
            xg[j][2] = x[c[j].z];
            xg[j][3] = x[c[j].w];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            double2 p0, p1;
            p0.x = v[j][0].x * xg[j][0];
            p0.y = v[j][0].y * xg[j][1];
            p1.x = v[j][1].x * xg[j][2];
            p1.y = v[j][1].y * xg[j][3];
            double2 *dst = reinterpret_cast<double2 *>(prod + j * (kChunk / 2) + tid * 4);
            dst[0] = p0;
            dst[1] = p1;
        }
    } else {
        for (int k = tid; k < kChunk; k += kBlock) {
            const int64_t kk = start + k;
            prod[k] = (kk < end) ? val[kk] * x[col[kk]] : 0.0;
        }
    }
    __syncthreads();

    const int lo = row_lo[b], hi = row_lo[b + 1];

    // ---- carry: the part of row lo-1 that lies in this chunk (wavefront 0)
    if (b > 0 && tid < kWave) {
        const int64_t next_start = rowptr[lo];  // rowptr[rows] == nnz
        if (next_start > start) {
            const int len = (int)(((next_start < end) ? next_start : end) - start);
            double s = 0.0;
            for (int k = tid; k < len; k += kWave) s += prod[k];
            s = wave_sum(s);
            if (tid == 0) carry[b] = s;
        }
    }

    // ---- rows that start in this chunk: groups of g lanes per row, g = 256 / (number of rows) rounded
    //      down to a power of two (so one pass covers them whenever there are at most 256 rows)
    const int nrows = hi - lo;
    if (nrows <= 0) return;
    int g = 1;
    while (g < kWave && nrows * (g * 2) <= kBlock) g *= 2;
    const int sub = tid & (g - 1);
    const int rows_per_pass = kBlock / g;
    for (int base = 0; base < nrows; base += rows_per_pass) {
        const int ri = base + tid / g;
        double s = 0.0;
        int64_t r = 0;
        if (ri < nrows) {
            r = (int64_t)lo + ri;
            const int64_t rs = rowptr[r], re = rowptr[r + 1];
            const int k0 = (int)(rs - start);
            const int k1 = (int)(((re < end) ? re : end) - start);
            for (int k = k0 + sub; k < k1; k += g) s += prod[k];
        }
        s = group_sum(s, g);
        if (ri < nrows && sub == 0) yout[r] = epilogue<EPI>(s, r, aux, alpha);
    }
}

// ------------------------------------------------------------------ fix-up of split rows
// One wavefront per split row: y[row] += factor * (carry[b0] + ... + carry[b0+cnt-1]).
template <int EPI>
__global__ __launch_bounds__(kBlock) void k_csr_fixup(int nfix, const int32_t *__restrict__ fix_row,
                                                      const int32_t *__restrict__ fix_b0, const int32_t *__restrict__ fix_cnt,
                                                      const double *__restrict__ carry, double *__restrict__ yout,
                                                      const double *__restrict__ aux, double alpha)
{
    const int m = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (m >= nfix) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int b0 = fix_b0[m], cnt = fix_cnt[m];
    double s = 0.0;
    for (int k = lane; k < cnt; k += kWave) s += carry[b0 + k];
    s = wave_sum(s);
    if (lane == 0) {
        const int64_t r = fix_row[m];
        double factor = 1.0;
        if (EPI == EPI_SCALE) factor = aux[r];
        if (EPI == EPI_AXPY) factor = alpha;
        yout[r] = fma(factor, s, yout[r]);
    }
}

template <int EPI>
static int launch_spmv(tron_dataset *ds, const CsrPlan &P, int slot, const double *x, double *yout, const double *aux,
                       double alpha)
{
    {
        ProfScope ps(ds, slot);
        hipLaunchKernelGGL(k_csr_spmv<EPI>, dim3(P.nblocks), dim3(kBlock), 0, ds->stream, P.rows, P.nnz, P.rowptr, P.col,
                           P.val, P.row_lo, x, yout, aux, alpha, P.carry);
        TRON_HIP(hipGetLastError());
    }
    if (P.nfix > 0) {
        ProfScope ps(ds, SLOT_SPMV_FIXUP);
        const int grid = (P.nfix + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(k_csr_fixup<EPI>, dim3(grid), dim3(kBlock), 0, ds->stream, P.nfix, P.fix_row, P.fix_b0,
                           P.fix_cnt, P.carry, yout, aux, alpha);
        TRON_HIP(hipGetLastError());
    }
    return TRON_OK;
}

int csr_spmv(tron_dataset *ds, const CsrPlan &P, int slot, int epi, const double *x, double *yout,
             const double *scale_or_add, double alpha)
{
    switch (epi) {
    case EPI_PLAIN: return launch_spmv<EPI_PLAIN>(ds, P, slot, x, yout, scale_or_add, alpha);
    case EPI_SCALE: return launch_spmv<EPI_SCALE>(ds, P, slot, x, yout, scale_or_add, alpha);
    default: return launch_spmv<EPI_AXPY>(ds, P, slot, x, yout, scale_or_add, alpha);
    }
}

}  // namespace tron
