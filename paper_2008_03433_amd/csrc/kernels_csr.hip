// CSR sparse matrix-vector products for both orientations (X and the explicit X^T copy):
//   z = X w,  a1 = D .* (X v)               (Table 1 / Appendix D of the paper: a0 = X v, a1 = D a0)
//   g = w + C X^T zhat,  Hv = v + C X^T a1   (a2 = C X^T a1)
//
// Work is split by nonzeros, not by rows, because row lengths are heavily skewed (Zipf-distributed
// features give the transposed copy rows of length ~n next to millions of length 0/1): a workgroup
// streams one chunk of kChunk nonzeros with coalesced 16-byte non-temporal loads, multiplies them by
// the gathered vector entries and parks the products in LDS; the rows that start inside the chunk are
// then summed from LDS by lane groups sized to the number of such rows.  A row that runs past the end
// of its chunk receives the rest from the `carry` of the following chunks in a small fix-up kernel, in
// a fixed order -- no atomics anywhere, so results are bit-reproducible.
//
// The gathers decide the speed: every L2 miss pulls a 128-byte line for 8 useful bytes.  For vectors
// that do not fit one XCD's L2 the matrix is therefore stored in P = 8 column partitions (see CsrPlan)
// and workgroup b handles partition b % 8, so that each XCD gathers from its own slice only; the
// partial row sums of the partitions are added by a combine kernel that also applies the epilogue
// (loss terms, D scaling, v + C * sum) and the first stage of the scalar reductions.
#include <algorithm>
#include <cstring>

#include "device_util.h"

namespace tron {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));

constexpr int64_t kGatherBytesForPartitioning = 3 << 19;  // 1.5 MiB: larger gather vectors get partitioned
constexpr int64_t kMinNnzForPartitioning = 1 << 22;
constexpr int kHotMinCount = 8;   // columns with fewer entries are not worth an LDS slot

void CsrPlan::release()
{
    hipFree(rowptr); hipFree(rowptr32); hipFree(col); hipFree(val); hipFree(row_lo); hipFree(carry);
    hipFree(hot_ids); hipFree(fix_row); hipFree(fix_part); hipFree(fix_b0); hipFree(fix_cnt);
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

// row_lo / fix-up lists of one partition (or of the whole matrix when P == 1).
// rp[r] = position of row r's first entry relative to the partition start; rp[rows] = nnz_x.
template <typename RP>
static void plan_chunks(const RP *rp, int64_t rows, int64_t nnz_x, int nchunks, int chunk0, int part,
                        std::vector<int32_t> &row_lo, std::vector<int32_t> &fix_row, std::vector<int32_t> &fix_part,
                        std::vector<int32_t> &fix_b0, std::vector<int32_t> &fix_cnt)
{
    // row_lo[c] = first row r with rp[r] >= c*kChunk; row_lo[nchunks] = rows
    const size_t off = row_lo.size();
    row_lo.resize(off + nchunks + 1);
    int64_t r = 0;
    for (int c = 0; c < nchunks; ++c) {
        const int64_t start = (int64_t)c * kChunk;
        while (r < rows && (int64_t)rp[r] < start) ++r;
        row_lo[off + c] = (int32_t)r;
    }
    row_lo[off] = 0;
    row_lo[off + nchunks] = (int32_t)rows;
    // chunk c >= 1 begins inside row row_lo[c]-1 iff rp[row_lo[c]] > c*kChunk  (rp[rows] = nnz_x)
    for (int c = 1; c < nchunks; ++c) {
        const int64_t start = (int64_t)c * kChunk;
        const int32_t lo = row_lo[off + c];
        if (lo >= 1 && (int64_t)rp[lo] > start) {
            const int32_t row = lo - 1;
            if (!fix_row.empty() && fix_row.back() == row && fix_part.back() == part) {
                fix_cnt.back() += 1;
            } else {
                fix_row.push_back(row);
                fix_part.push_back(part);
                fix_b0.push_back(chunk0 + c);
                fix_cnt.push_back(1);
            }
        }
    }
    (void)nnz_x;
}

int csr_plan_build(CsrPlan &A, int64_t rows, int64_t cols, const int64_t *h_rowptr, const int32_t *h_col,
                   const double *h_val, int parts, bool hot, hipStream_t st)
{
    A.rows = rows;
    A.cols = cols;
    A.nnz = h_rowptr[rows];
    if (parts <= 0)
        parts = (cols * (int64_t)sizeof(double) > kGatherBytesForPartitioning && A.nnz >= kMinNnzForPartitioning) ? kMaxParts : 1;
    if (parts > kMaxParts) parts = kMaxParts;
    A.P = parts;
    std::vector<int32_t> row_lo, fix_row, fix_part, fix_b0, fix_cnt;

    if (A.P == 1) {
        const int64_t nb64 = std::max<int64_t>(1, (A.nnz + kChunk - 1) / kChunk);
        if (nb64 > 0x7ffffff0) { set_error("matrix too large: %lld chunks", (long long)nb64); return TRON_EINVAL; }
        A.nblocks = (int)nb64;
        A.part_base[0] = 0; A.part_nnz[0] = A.nnz; A.part_chunk0[0] = 0; A.part_nchunks[0] = A.nblocks;
        A.max_chunks = A.nblocks;
        plan_chunks(h_rowptr, rows, A.nnz, A.nblocks, 0, 0, row_lo, fix_row, fix_part, fix_b0, fix_cnt);
        TRON_TRY(upload(&A.rowptr, h_rowptr, (size_t)rows + 1, st));
        TRON_TRY(upload(&A.col, h_col, (size_t)A.nnz, st));
        TRON_TRY(upload(&A.val, h_val, (size_t)A.nnz, st));
    } else {
        const int P = A.P;
        // column ranges with equal nonzero counts: bound[x] = first column of range x
        std::vector<int64_t> colcount((size_t)cols + 1, 0);
        for (int64_t k = 0; k < A.nnz; ++k) colcount[h_col[k] + 1]++;
        for (int64_t j = 0; j < cols; ++j) colcount[j + 1] += colcount[j];
        std::vector<int64_t> bound(P + 1, cols);
        bound[0] = 0;
        for (int x = 1; x < P; ++x) {
            const int64_t target = A.nnz / P * x;
            bound[x] = std::lower_bound(colcount.begin(), colcount.end(), target) - colcount.begin();
            if (bound[x] > cols) bound[x] = cols;
            if (bound[x] < bound[x - 1]) bound[x] = bound[x - 1];
        }
        std::vector<uint8_t> part_of((size_t)cols);
        for (int x = 0; x < P; ++x)
            for (int64_t j = bound[x]; j < bound[x + 1]; ++j) part_of[j] = (uint8_t)x;
        for (int x = 0; x < P; ++x) {
            A.part_nnz[x] = colcount[bound[x + 1]] - colcount[bound[x]];
            if (A.part_nnz[x] > 0x7ffffff0) { set_error("partition too large for 32-bit row offsets"); return TRON_EINVAL; }
        }
        std::vector<int32_t> colcnt;
        if (hot) {
            colcnt.resize((size_t)cols);
            for (int64_t j = 0; j < cols; ++j) colcnt[j] = (int32_t)std::min<int64_t>(colcount[j + 1] - colcount[j], 0x7fffffff);
        }
        std::vector<int64_t>().swap(colcount);
        // per-partition row offsets
        std::vector<int32_t> rp32((size_t)P * (rows + 1), 0);
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t k = h_rowptr[r]; k < h_rowptr[r + 1]; ++k) rp32[(size_t)part_of[h_col[k]] * (rows + 1) + r + 1]++;
        int64_t pos = 0;
        int chunk = 0;
        A.max_chunks = 0;
        for (int x = 0; x < P; ++x) {
            int32_t *rp = rp32.data() + (size_t)x * (rows + 1);
            for (int64_t r = 0; r < rows; ++r) rp[r + 1] += rp[r];
            A.part_base[x] = pos;
            A.part_chunk0[x] = chunk;
            A.part_nchunks[x] = (int)std::max<int64_t>(1, (A.part_nnz[x] + kChunk - 1) / kChunk);
            A.max_chunks = std::max(A.max_chunks, A.part_nchunks[x]);
            chunk += A.part_nchunks[x];
            pos += (int64_t)A.part_nchunks[x] * kChunk;
        }
        A.nblocks = chunk;
        // LDS-resident columns: in each range the kHotSlots most frequent columns with at least kHotMinCount entries
        std::vector<int32_t> slot_of;
        std::vector<int32_t> hot_ids;
        if (hot) {
            slot_of.assign((size_t)cols, -1);
            hot_ids.assign((size_t)P * kHotSlots, 0);
            std::vector<std::pair<int64_t, int32_t>> cand;
            for (int x = 0; x < P; ++x) {
                cand.clear();
                for (int64_t j = bound[x]; j < bound[x + 1]; ++j)
                    if (colcnt[j] >= kHotMinCount) cand.emplace_back(-colcnt[j], (int32_t)j);
                const size_t keep = std::min<size_t>(cand.size(), kHotSlots);
                std::partial_sort(cand.begin(), cand.begin() + keep, cand.end());
                A.part_nhot[x] = (int)keep;
                for (size_t k = 0; k < keep; ++k) {
                    slot_of[cand[k].second] = (int32_t)k;
                    hot_ids[(size_t)x * kHotSlots + k] = cand[k].second;
                }
            }
        }
        // entries partition-major; inside a row the entries of one range are contiguous and stay ordered
        std::vector<int32_t> pcol((size_t)pos, 0);
        std::vector<double> pval((size_t)pos, 0.0);
        std::vector<int64_t> cursor(P);
        for (int64_t r = 0; r < rows; ++r) {
            for (int x = 0; x < P; ++x) cursor[x] = A.part_base[x] + rp32[(size_t)x * (rows + 1) + r];
            for (int64_t k = h_rowptr[r]; k < h_rowptr[r + 1]; ++k) {
                const int64_t q = cursor[part_of[h_col[k]]]++;
                pcol[q] = (hot && slot_of[h_col[k]] >= 0) ? ~slot_of[h_col[k]] : h_col[k];
                pval[q] = h_val[k];
            }
        }
        for (int x = 0; x < P; ++x)
            plan_chunks(rp32.data() + (size_t)x * (rows + 1), rows, A.part_nnz[x], A.part_nchunks[x], A.part_chunk0[x], x,
                        row_lo, fix_row, fix_part, fix_b0, fix_cnt);
        if (hot) TRON_TRY(upload(&A.hot_ids, hot_ids.data(), hot_ids.size(), st));
        TRON_TRY(upload(&A.rowptr32, rp32.data(), rp32.size(), st));
        TRON_TRY(upload(&A.col, pcol.data(), pcol.size(), st));
        TRON_TRY(upload(&A.val, pval.data(), pval.size(), st));
        TRON_HIP(hipStreamSynchronize(st));
    }
    A.nfix = (int)fix_row.size();
    TRON_TRY(upload(&A.row_lo, row_lo.data(), row_lo.size(), st));
    TRON_TRY(upload(&A.fix_row, fix_row.data(), fix_row.size(), st));
    TRON_TRY(upload(&A.fix_part, fix_part.data(), fix_part.size(), st));
    TRON_TRY(upload(&A.fix_b0, fix_b0.data(), fix_b0.size(), st));
    TRON_TRY(upload(&A.fix_cnt, fix_cnt.data(), fix_cnt.size(), st));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&A.carry), sizeof(double) * A.nblocks));
    TRON_HIP(hipMemsetAsync(A.carry, 0, sizeof(double) * A.nblocks, st));
    TRON_HIP(hipStreamSynchronize(st));  // the host vectors above go out of scope
    return TRON_OK;
}

// ------------------------------------------------------------------ chunk kernel
enum { EPI_PLAIN = 0, EPI_SCALE = 1, EPI_AXPY = 2 };

template <int EPI>
__device__ __forceinline__ double epilogue(double sum, int64_t r, const double *__restrict__ aux, double alpha)
{
    if (EPI == EPI_PLAIN) return sum;
    if (EPI == EPI_SCALE) return aux[r] * sum;
    return fma(alpha, sum, aux[r]);
}

// One chunk: nonzeros [start, end) of a (sub)matrix whose row offsets are rp (relative to col/val),
// chunk-local tables row_lo[0..1] and carry slot *carry_out.
// With HOT, a negative stored column c means "entry ~c of the workgroup's LDS table" (the most frequent
// columns of the partition, copied from x once per workgroup).
template <bool HOT>
__device__ __forceinline__ double gather(const double *__restrict__ x, const double *table, int c)
{
    if (HOT && c < 0) return table[~c];
    return x[c];
}

template <int EPI, typename RP, bool HOT = false>
__device__ __forceinline__ void chunk_body(double *prod, const double *table, int64_t start, int64_t end, bool first_chunk,
                                           const RP *__restrict__ rp, const int32_t *__restrict__ col,
                                           const double *__restrict__ val, const int32_t *__restrict__ row_lo,
                                           const double *__restrict__ x, double *__restrict__ yout,
                                           const double *__restrict__ aux, double alpha, double *__restrict__ carry_out)
{
    const int tid = threadIdx.x;
    // ---- phase 1: products into LDS (two passes of 1024 nonzeros, 4 per thread per pass)
    if (end - start == kChunk) {
        v4i c[2];
        v2d v[2][2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t k = start + j * (kChunk / 2) + tid * 4;
            c[j] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(col + k));
            v[j][0] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(val + k));
            v[j][1] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(val + k + 2));
        }
        double xg[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            xg[j][0] = gather<HOT>(x, table, c[j].x);
            xg[j][1] = gather<HOT>(x, table, c[j].y);
            xg[j][2] = gather<HOT>(x, table, c[j].z);
            xg[j][3] = gather<HOT>(x, table, c[j].w);
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
            prod[k] = (kk < end) ? val[kk] * gather<HOT>(x, table, col[kk]) : 0.0;
        }
    }
    __syncthreads();

    const int lo = row_lo[0], hi = row_lo[1];

    // ---- carry: the part of row lo-1 that lies in this chunk (wavefront 0)
    if (!first_chunk && tid < kWave) {
        const int64_t next_start = (int64_t)rp[lo];  // rp[rows] == nnz of this (sub)matrix
        if (next_start > start) {
            const int len = (int)(((next_start < end) ? next_start : end) - start);
            double s = 0.0;
            for (int k = tid; k < len; k += kWave) s += prod[k];
            s = wave_sum(s);
            if (tid == 0) *carry_out = s;
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
            const int64_t rs = (int64_t)rp[r], re = (int64_t)rp[r + 1];
            const int k0 = (int)(rs - start);
            const int k1 = (int)(((re < end) ? re : end) - start);
            for (int k = k0 + sub; k < k1; k += g) s += prod[k];
        }
        s = group_sum(s, g);
        if (ri < nrows && sub == 0) yout[r] = epilogue<EPI>(s, r, aux, alpha);
    }
}

// unpartitioned: y = epilogue(A x) directly
template <int EPI>
__global__ __launch_bounds__(kBlock) void k_csr_spmv(int64_t nnz, const int64_t *__restrict__ rowptr,
                                                     const int32_t *__restrict__ col, const double *__restrict__ val,
                                                     const int32_t *__restrict__ row_lo, const double *__restrict__ x,
                                                     double *__restrict__ yout, const double *__restrict__ aux,
                                                     double alpha, double *__restrict__ carry)
{
    __shared__ __align__(16) double prod[kChunk];
    const int b = blockIdx.x;
    const int64_t start = (int64_t)b * kChunk;
    const int64_t end = (start + kChunk < nnz) ? start + kChunk : nnz;
    chunk_body<EPI>(prod, nullptr, start, end, b == 0, rowptr, col, val, row_lo + b, x, yout, aux, alpha, carry + b);
}

struct PartArgs {
    int64_t base[kMaxParts];
    int64_t nnz[kMaxParts];
    int chunk0[kMaxParts];
    int nchunks[kMaxParts];
    int nhot[kMaxParts];
    int P;
};

// partitioned: partial[x*rows + r] = sum over the entries of row r in column range x
__global__ __launch_bounds__(kBlock) void k_csr_spmv_part(PartArgs pa, int64_t rows, const int32_t *__restrict__ rowptr32,
                                                          const int32_t *__restrict__ col, const double *__restrict__ val,
                                                          const int32_t *__restrict__ row_lo, const double *__restrict__ x,
                                                          double *__restrict__ partial, double *__restrict__ carry)
{
    __shared__ __align__(16) double prod[kChunk];
    const int xp = blockIdx.x % pa.P;      // partition; with round-robin dispatch also the XCD
    const int c = blockIdx.x / pa.P;       // chunk inside the partition
    if (c >= pa.nchunks[xp]) return;
    const int64_t start = (int64_t)c * kChunk;
    const int64_t nnz = pa.nnz[xp];
    const int64_t end = (start + kChunk < nnz) ? start + kChunk : nnz;
    const int gc = pa.chunk0[xp] + c;      // global chunk id
    chunk_body<EPI_PLAIN>(prod, nullptr, start, end, c == 0, rowptr32 + (int64_t)xp * (rows + 1), col + pa.base[xp],
                          val + pa.base[xp], row_lo + gc + xp, x, partial + (int64_t)xp * rows, nullptr, 0.0, carry + gc);
}

// partitioned with an LDS table of the partition's most frequent columns: persistent workgroups, each
// loads the table once and then walks chunks q, q + Q, q + 2Q, ... of its partition (Q = gridDim / P)
__global__ __launch_bounds__(kBlock) void k_csr_spmv_part_hot(PartArgs pa, int64_t rows, const int32_t *__restrict__ rowptr32,
                                                              const int32_t *__restrict__ col, const double *__restrict__ val,
                                                              const int32_t *__restrict__ row_lo, const int32_t *__restrict__ hot_ids,
                                                              const double *__restrict__ x, double *__restrict__ partial,
                                                              double *__restrict__ carry)
{
    __shared__ __align__(16) double prod[kChunk];
    __shared__ double table[kHotSlots];
    const int xp = blockIdx.x % pa.P;
    const int q = blockIdx.x / pa.P, Q = gridDim.x / pa.P;
    const int nhot = pa.nhot[xp];
    for (int k = threadIdx.x; k < nhot; k += kBlock) table[k] = x[hot_ids[xp * kHotSlots + k]];
    __syncthreads();
    const int64_t nnz = pa.nnz[xp];
    for (int c = q; c < pa.nchunks[xp]; c += Q) {
        const int64_t start = (int64_t)c * kChunk;
        const int64_t end = (start + kChunk < nnz) ? start + kChunk : nnz;
        const int gc = pa.chunk0[xp] + c;
        chunk_body<EPI_PLAIN, int32_t, true>(prod, table, start, end, c == 0, rowptr32 + (int64_t)xp * (rows + 1),
                                             col + pa.base[xp], val + pa.base[xp], row_lo + gc + xp, x,
                                             partial + (int64_t)xp * rows, nullptr, 0.0, carry + gc);
        __syncthreads();  // prod is reused by the next chunk
    }
}

// ------------------------------------------------------------------ fix-up of split rows
// One wavefront per split row: y[row] += factor * (carry[b0] + ... + carry[b0+cnt-1]).
template <int EPI>
__global__ __launch_bounds__(kBlock) void k_csr_fixup(int nfix, int64_t rows, const int32_t *__restrict__ fix_row,
                                                      const int32_t *__restrict__ fix_part, const int32_t *__restrict__ fix_b0,
                                                      const int32_t *__restrict__ fix_cnt, const double *__restrict__ carry,
                                                      double *__restrict__ yout, const double *__restrict__ aux, double alpha)
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
        double *dst = yout + (int64_t)fix_part[m] * rows + r;   // fix_part is 0 when unpartitioned
        *dst = fma(factor, s, *dst);
    }
}

// ------------------------------------------------------------------ combine kernels (partitioned layout)
template <int P>
__device__ __forceinline__ double sum_parts(const double *__restrict__ partial, int64_t rows, int64_t r)
{
    double s = partial[r];
#pragma unroll
    for (int x = 1; x < P; ++x) s += partial[(int64_t)x * rows + r];
    return s;
}

__device__ __forceinline__ double sum_parts_rt(const double *__restrict__ partial, int64_t rows, int64_t r, int P)
{
    if (P == 8) return sum_parts<8>(partial, rows, r);
    double s = partial[r];
    for (int x = 1; x < P; ++x) s += partial[(int64_t)x * rows + r];
    return s;
}

// z = sum of partials; loss terms; partial slot 0 = sum loss
template <int LOSS>
__global__ __launch_bounds__(kBlock) void k_combine_loss(int64_t n, int P, const double *__restrict__ partial,
                                                         const double *__restrict__ y, double *__restrict__ zhat,
                                                         double *__restrict__ D, double *__restrict__ red)
{
    __shared__ double lds[kWavesPerBlock];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        const double z = sum_parts_rt(partial, n, i, P);
        double a, zh, Di;
        loss_terms_dev<LOSS>(z, y[i], a, zh, Di);
        zhat[i] = zh;
        D[i] = Di;
        acc += a;
    }
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) red[blockIdx.x] = acc;
}

// out = scale .* sum of partials
__global__ __launch_bounds__(kBlock) void k_combine_scale(int64_t rows, int P, const double *__restrict__ partial,
                                                          const double *__restrict__ scale, double *__restrict__ out)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < rows; i += (int64_t)gridDim.x * kBlock)
        out[i] = scale[i] * sum_parts_rt(partial, rows, i, P);
}

// out = add + alpha * sum of partials; partial slot 0 = out . (SELF ? out : add)
template <bool SELF>
__global__ __launch_bounds__(kBlock) void k_combine_axpy(int64_t rows, int P, const double *__restrict__ partial,
                                                         const double *__restrict__ add, double alpha,
                                                         double *__restrict__ out, double *__restrict__ red)
{
    __shared__ double lds[kWavesPerBlock];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < rows; i += (int64_t)gridDim.x * kBlock) {
        const double a = add[i];
        const double o = fma(alpha, sum_parts_rt(partial, rows, i, P), a);
        out[i] = o;
        acc += o * (SELF ? o : a);
    }
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) red[blockIdx.x] = acc;
}

// ------------------------------------------------------------------ launchers
static inline int vec_grid(int64_t m)
{
    int64_t g = (m + kBlock * 4 - 1) / (kBlock * 4);
    if (g < 1) g = 1;
    if (g > kMaxGrid) g = kMaxGrid;
    return (int)g;
}

template <int EPI>
static int launch_plain(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, double *yout, const double *aux,
                        double alpha)
{
    {
        ProfScope ps(ds, slot);
        hipLaunchKernelGGL(k_csr_spmv<EPI>, dim3(A.nblocks), dim3(kBlock), 0, ds->stream, A.nnz, A.rowptr, A.col, A.val,
                           A.row_lo, x, yout, aux, alpha, A.carry);
        TRON_HIP(hipGetLastError());
    }
    if (A.nfix > 0) {
        ProfScope ps(ds, SLOT_SPMV_FIXUP);
        const int grid = (A.nfix + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(k_csr_fixup<EPI>, dim3(grid), dim3(kBlock), 0, ds->stream, A.nfix, A.rows, A.fix_row, A.fix_part,
                           A.fix_b0, A.fix_cnt, A.carry, yout, aux, alpha);
        TRON_HIP(hipGetLastError());
    }
    return TRON_OK;
}

// partial row sums of all partitions into ds->row_partials (with split rows fixed up)
static int launch_partials(tron_dataset *ds, const CsrPlan &A, int slot, const double *x)
{
    PartArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    pa.P = A.P;
    for (int i = 0; i < A.P; ++i) {
        pa.base[i] = A.part_base[i];
        pa.nnz[i] = A.part_nnz[i];
        pa.chunk0[i] = A.part_chunk0[i];
        pa.nchunks[i] = A.part_nchunks[i];
        pa.nhot[i] = A.part_nhot[i];
    }
    {
        ProfScope ps(ds, slot);
        if (A.hot_ids) {
            int per_part = std::min(A.max_chunks, (int)g_tuning.csr_hot_blocks_per_part);
            hipLaunchKernelGGL(k_csr_spmv_part_hot, dim3(per_part * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows, A.rowptr32,
                               A.col, A.val, A.row_lo, A.hot_ids, x, ds->row_partials, A.carry);
        } else {
            hipLaunchKernelGGL(k_csr_spmv_part, dim3(A.max_chunks * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows, A.rowptr32,
                               A.col, A.val, A.row_lo, x, ds->row_partials, A.carry);
        }
        TRON_HIP(hipGetLastError());
    }
    if (A.nfix > 0) {
        ProfScope ps(ds, SLOT_SPMV_FIXUP);
        const int grid = (A.nfix + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(k_csr_fixup<EPI_PLAIN>, dim3(grid), dim3(kBlock), 0, ds->stream, A.nfix, A.rows, A.fix_row,
                           A.fix_part, A.fix_b0, A.fix_cnt, A.carry, ds->row_partials, (const double *)nullptr, 0.0);
        TRON_HIP(hipGetLastError());
    }
    return TRON_OK;
}

int spmv_loss(tron_dataset *ds, const CsrPlan &A, int slot, int loss, const double *x, double *zwork, double *zhat, double *D)
{
    if (A.P == 1) {
        TRON_TRY(launch_plain<EPI_PLAIN>(ds, A, slot, x, zwork, nullptr, 0.0));
        return loss_terms(ds, loss, zwork, zhat, D);
    }
    TRON_TRY(launch_partials(ds, A, slot, x));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    const int g = vec_grid(A.rows);
    if (loss == TRON_LOSS_LR)
        hipLaunchKernelGGL(k_combine_loss<TRON_LOSS_LR>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, A.P, ds->row_partials, ds->y, zhat, D, ds->partials);
    else
        hipLaunchKernelGGL(k_combine_loss<TRON_LOSS_L2SVM>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, A.P, ds->row_partials, ds->y, zhat, D, ds->partials);
    TRON_HIP(hipGetLastError());
    return g;
}

int spmv_scale(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, const double *scale, double *out)
{
    if (A.P == 1) return launch_plain<EPI_SCALE>(ds, A, slot, x, out, scale, 0.0);
    TRON_TRY(launch_partials(ds, A, slot, x));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    hipLaunchKernelGGL(k_combine_scale, dim3(vec_grid(A.rows)), dim3(kBlock), 0, ds->stream, A.rows, A.P, ds->row_partials, scale, out);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

int spmv_axpy(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, const double *add, double alpha, bool dot_self,
              double *out)
{
    if (A.P == 1) {
        TRON_TRY(launch_plain<EPI_AXPY>(ds, A, slot, x, out, add, alpha));
        return dot_partials(ds, A.rows, out, dot_self ? out : add, nullptr, nullptr, nullptr, nullptr);
    }
    TRON_TRY(launch_partials(ds, A, slot, x));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    const int g = vec_grid(A.rows);
    if (dot_self)
        hipLaunchKernelGGL(k_combine_axpy<true>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, A.P, ds->row_partials, add, alpha, out, ds->partials);
    else
        hipLaunchKernelGGL(k_combine_axpy<false>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, A.P, ds->row_partials, add, alpha, out, ds->partials);
    TRON_HIP(hipGetLastError());
    return g;
}

}  // namespace tron
