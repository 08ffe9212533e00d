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

void HotTiles::release()
{
    hipFree(val); hipFree(iloc); hipFree(hdr); hipFree(seg_desc); hipFree(slot_of_row);
    hipFree(wg_acc); hipFree(sums);
    *this = HotTiles();
}

void CsrPlan::release()
{
    hot.release();
    hipFree(rowptr); hipFree(col); hipFree(val); hipFree(row_lo); hipFree(carry);
    hipFree(hot_ids); hipFree(seg_row); hipFree(chunk_tab); hipFree(seg_end); hipFree(row_mask);
    hipFree(fix_row); hipFree(fix_part); hipFree(fix_b0); hipFree(fix_cnt);
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
            if (A.part_nnz[x] > 0x7ffffff0) { set_error("partition too large for 32-bit offsets"); return TRON_EINVAL; }
        }
        // LDS-resident columns: in each range the kHotSlots most frequent columns with at least kHotMinCount entries
        std::vector<int32_t> slot_of, hot_ids;
        if (hot) {
            slot_of.assign((size_t)cols, -1);
            hot_ids.assign((size_t)P * kHotSlots, 0);
            std::vector<std::pair<int64_t, int32_t>> cand;
            for (int x = 0; x < P; ++x) {
                cand.clear();
                for (int64_t j = bound[x]; j < bound[x + 1]; ++j) {
                    const int64_t cnt = colcount[j + 1] - colcount[j];
                    if (cnt >= kHotMinCount) cand.emplace_back(-cnt, (int32_t)j);
                }
                const size_t keep = std::min<size_t>(cand.size(), kHotSlots);
                std::partial_sort(cand.begin(), cand.begin() + keep, cand.end());
                A.part_nhot[x] = (int)keep;
                for (size_t k = 0; k < keep; ++k) {
                    slot_of[cand[k].second] = (int32_t)k;
                    hot_ids[(size_t)x * kHotSlots + k] = cand[k].second;
                }
            }
        }
        std::vector<int64_t>().swap(colcount);
        // per-(partition,row) entry counts -> offsets; non-empty pairs are the segments
        std::vector<int32_t> rp32((size_t)P * (rows + 1), 0);
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t k = h_rowptr[r]; k < h_rowptr[r + 1]; ++k) rp32[(size_t)part_of[h_col[k]] * (rows + 1) + r + 1]++;
        std::vector<uint8_t> mask((size_t)rows, 0);
        int64_t pos = 0, nseg_total = 0;
        int chunk = 0;
        A.max_chunks = 0;
        for (int x = 0; x < P; ++x) {
            int32_t *rp = rp32.data() + (size_t)x * (rows + 1);
            int64_t nseg = 0;
            for (int64_t r = 0; r < rows; ++r) {
                if (rp[r + 1] > 0) { mask[r] |= (uint8_t)(1u << x); ++nseg; }
                rp[r + 1] += rp[r];
            }
            A.part_base[x] = pos;
            A.part_seg0[x] = nseg_total;
            A.part_chunk0[x] = chunk;
            A.part_nchunks[x] = (int)std::max<int64_t>(1, (A.part_nnz[x] + kChunk - 1) / kChunk);
            A.max_chunks = std::max(A.max_chunks, A.part_nchunks[x]);
            chunk += A.part_nchunks[x];
            pos += (int64_t)A.part_nchunks[x] * kChunk;
            nseg_total += nseg;
        }
        A.nblocks = chunk;
        if (nseg_total + 8 * (int64_t)chunk > 0x7ffffff0) { set_error("too many row segments for 32-bit indexing"); return TRON_EINVAL; }
        // entries partition-major; inside a row the entries of one range are contiguous and stay ordered
        std::vector<int32_t> pcol((size_t)pos, 0);
        std::vector<double> pval((size_t)pos, 0.0);
        {
            std::vector<int64_t> cursor(P);
            for (int64_t r = 0; r < rows; ++r) {
                for (int x = 0; x < P; ++x) cursor[x] = A.part_base[x] + rp32[(size_t)x * (rows + 1) + r];
                for (int64_t k = h_rowptr[r]; k < h_rowptr[r + 1]; ++k) {
                    const int64_t q = cursor[part_of[h_col[k]]]++;
                    pcol[q] = (hot && slot_of[h_col[k]] >= 0) ? ~slot_of[h_col[k]] : h_col[k];
                    pval[q] = h_val[k];
                }
            }
        }
        // segment tables
        std::vector<int32_t> seg_row((size_t)std::max<int64_t>(nseg_total, 1));
        std::vector<int4> tab((size_t)chunk);
        std::vector<uint16_t> seg_end;
        seg_end.reserve((size_t)(nseg_total + 8 * (int64_t)chunk));
        for (int x = 0; x < P; ++x) {
            const int32_t *rp = rp32.data() + (size_t)x * (rows + 1);
            const int nch = A.part_nchunks[x];
            // the segments of this partition, in row order, with start/end positions relative to the partition
            int64_t m = 0;               // segment counter (partition-relative)
            int c = 0;                   // chunk that owns the segments being emitted
            int4 t = make_int4(0, 0, 0, (int)seg_end.size());
            auto close_chunk = [&](int next_first_seg, int64_t next_seg_start) {
                tab[A.part_chunk0[x] + c] = t;
                while (seg_end.size() % 8) seg_end.push_back(0);
                ++c;
                const int64_t cstart = (int64_t)c * kChunk;
                const int64_t off = std::min<int64_t>(std::max<int64_t>(next_seg_start - cstart, 0), kChunk);
                t = make_int4(next_first_seg, 0, (int)off, (int)seg_end.size());
            };
            for (int64_t r = 0; r < rows; ++r) {
                const int64_t rs = rp[r], re = rp[r + 1];
                if (re == rs) continue;
                while (rs >= (int64_t)(c + 1) * kChunk) close_chunk((int)m, rs);   // this segment starts in a later chunk
                seg_row[A.part_seg0[x] + m] = (int32_t)r;
                const int64_t cstart = (int64_t)c * kChunk;
                seg_end.push_back((uint16_t)std::min<int64_t>(re - cstart, kChunk));
                t.y += 1;
                // continuation chunks of a split row: fix-up list
                const int c_last = (int)((re - 1) / kChunk);
                if (c_last > c) {
                    fix_row.push_back((int32_t)r);
                    fix_part.push_back(x);
                    fix_b0.push_back(A.part_chunk0[x] + c + 1);
                    fix_cnt.push_back(c_last - c);
                }
                ++m;
            }
            while (c < nch - 1) close_chunk((int)m, (int64_t)A.part_nnz[x]);
            tab[A.part_chunk0[x] + c] = t;
            while (seg_end.size() % 8) seg_end.push_back(0);
        }
        // first_off of a chunk inside or at the end of a split row: the chunk-relative end of that row
        // (set above from the start of the next segment; for chunks wholly inside one row that start lies
        // beyond the chunk and clips to kChunk, which is right)
        if (hot) TRON_TRY(upload(&A.hot_ids, hot_ids.data(), hot_ids.size(), st));
        TRON_TRY(upload(&A.col, pcol.data(), pcol.size(), st));
        TRON_TRY(upload(&A.val, pval.data(), pval.size(), st));
        TRON_TRY(upload(&A.seg_row, seg_row.data(), seg_row.size(), st));
        TRON_TRY(upload(&A.chunk_tab, tab.data(), tab.size(), st));
        TRON_TRY(upload(&A.seg_end, seg_end.data(), seg_end.size(), st));
        TRON_TRY(upload(&A.row_mask, mask.data(), mask.size(), st));
        TRON_HIP(hipStreamSynchronize(st));
    }
    A.nfix = (int)fix_row.size();
    if (A.P == 1) TRON_TRY(upload(&A.row_lo, row_lo.data(), row_lo.size(), st));
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
// x[c] through a 32-bit byte offset (c < 2^28 is guaranteed by the plan builder's size checks)
__device__ __forceinline__ double load_elem(const double *__restrict__ x, int c)
{
    return *reinterpret_cast<const double *>(reinterpret_cast<const char *>(x) + (size_t)((uint32_t)c << 3));
}

template <bool HOT>
__device__ __forceinline__ double gather(const double *__restrict__ x, const double *table, int c)
{
    if (!HOT) return load_elem(x, c);
    // two separate accesses (an LDS read and a lane-masked global load), not one flat load of a selected address
    const double hot = table[(c < 0) ? ~c : 0];
    double cold = 0.0;
    if (c >= 0) cold = load_elem(x, c);
    return (c < 0) ? hot : cold;
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
    int64_t seg0[kMaxParts];
    int chunk0[kMaxParts];
    int nchunks[kMaxParts];
    int nhot[kMaxParts];
    int P;
};

// Partitioned layout, persistent workgroups: workgroup (partition xp, q) walks chunks q, q + Q, ... of its
// partition (Q = gridDim / P).  Everything the next chunk needs -- the col/val stream, the chunk's table entry,
// its segment end offsets and the row ids this thread will write -- is fetched into registers while the current
// chunk is being reduced, so HBM latency is paid once per workgroup, not once per chunk.
// With HOT the partition's most frequent columns are first copied from x into an LDS table; entries of those
// columns are stored as ~slot and never touch the vector cache.
struct StreamRegs {
    v4i c[2];
    v2d v[2][2];
};

__device__ __forceinline__ StreamRegs load_stream(const int32_t *__restrict__ col, const double *__restrict__ val, int64_t start)
{
    StreamRegs s;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int64_t k = start + j * (kChunk / 2) + threadIdx.x * 4;
        s.c[j] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(col + k));
        s.v[j][0] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(val + k));
        s.v[j][1] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(val + k + 2));
    }
    return s;
}

// lanes per segment: 256 / (number of segments) rounded down to a power of two, at most 64, at least 1
__device__ __forceinline__ int lanes_per_segment(int nseg)
{
    int g = 1;
    while (g < kWave && nseg * (g * 2) <= kBlock) g *= 2;
    return g;
}

constexpr int kSegPasses = kChunk / kBlock;   // a chunk owns at most kChunk segments: 8 passes of 256

struct SegRegs {
    uint4 ends;             // 8 x uint16 end offsets: segments 8*tid .. 8*tid+7 of the chunk
    int rid[kSegPasses];    // row ids of the segments this thread writes: (tid / g) + 256 j
};

__device__ __forceinline__ SegRegs load_segs(const int4 tab, const uint16_t *__restrict__ seg_end,
                                             const int32_t *__restrict__ seg_row /* of this partition */)
{
    SegRegs s;
    const int nseg = tab.y;
    s.ends = make_uint4(0, 0, 0, 0);
    if (8 * (int)threadIdx.x < nseg) s.ends = *reinterpret_cast<const uint4 *>(seg_end + tab.w + 8 * threadIdx.x);
    const int g = lanes_per_segment(nseg);
    const int first = threadIdx.x / g;
#pragma unroll
    for (int j = 0; j < kSegPasses; ++j) {
        const int sidx = first + kBlock * j;
        s.rid[j] = (sidx < nseg && (g == 1 || j == 0)) ? seg_row[tab.x + sidx] : 0;
    }
    return s;
}

template <bool HOT>
__global__ __launch_bounds__(kBlock) void k_csr_spmv_part(PartArgs pa, int64_t rows, const int32_t *__restrict__ col_all,
                                                          const double *__restrict__ val_all, const int4 *__restrict__ chunk_tab,
                                                          const uint16_t *__restrict__ seg_end, const int32_t *__restrict__ seg_row_all,
                                                          const int32_t *__restrict__ hot_ids, const double *__restrict__ x,
                                                          double *__restrict__ partial_all, double *__restrict__ carry_all)
{
    __shared__ __align__(16) double prod[kChunk];
    __shared__ __align__(16) uint16_t ends[kChunk];
    __shared__ double table[HOT ? kHotSlots : 1];
    const int tid = threadIdx.x;
    const int xp = blockIdx.x % pa.P;
    const int q = blockIdx.x / pa.P, Q = gridDim.x / pa.P;
    const int nchunks = pa.nchunks[xp];
    if (q >= nchunks) return;
    if (HOT) {
        const int nhot = pa.nhot[xp];
        for (int k = tid; k < nhot; k += kBlock) table[k] = x[hot_ids[xp * kHotSlots + k]];
        if (tid == 0 && nhot == 0) table[0] = 0.0;
        __syncthreads();
    }
    const int32_t *col = col_all + pa.base[xp];     // padded to whole chunks (zeros)
    const double *val = val_all + pa.base[xp];
    const int4 *tabs = chunk_tab + pa.chunk0[xp];
    const int32_t *seg_row = seg_row_all + pa.seg0[xp];
    double *partial = partial_all + (int64_t)xp * rows;
    double *carry = carry_all + pa.chunk0[xp];

    int c = q;
    int4 tab = tabs[c];
    int4 tab_n = tabs[(c + Q < nchunks) ? c + Q : c];
    StreamRegs cur = load_stream(col, val, (int64_t)c * kChunk);
    SegRegs seg = load_segs(tab, seg_end, seg_row);

    for (; c < nchunks; c += Q) {
        const int nseg = tab.y, first_off = tab.z;
        if (8 * tid < nseg) *reinterpret_cast<uint4 *>(ends + 8 * tid) = seg.ends;
        // products of this chunk into LDS
        double xg[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            xg[j][0] = gather<HOT>(x, table, cur.c[j].x);
            xg[j][1] = gather<HOT>(x, table, cur.c[j].y);
            xg[j][2] = gather<HOT>(x, table, cur.c[j].z);
            xg[j][3] = gather<HOT>(x, table, cur.c[j].w);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            double2 p0, p1;
            p0.x = cur.v[j][0].x * xg[j][0];
            p0.y = cur.v[j][0].y * xg[j][1];
            p1.x = cur.v[j][1].x * xg[j][2];
            p1.y = cur.v[j][1].y * xg[j][3];
            double2 *dst = reinterpret_cast<double2 *>(prod + j * (kChunk / 2) + tid * 4);
            dst[0] = p0;
            dst[1] = p1;
        }
        // Only now fetch the next chunk (clamped index: always the same loads): nothing below waits for these
        // registers, so they stay in flight during the barrier and the segment sums and are waited for at the
        // top of the next iteration.
        __builtin_amdgcn_sched_barrier(0);
        const int cn = (c + Q < nchunks) ? c + Q : c;
        const int cnn = (cn + Q < nchunks) ? cn + Q : cn;
        const StreamRegs nxt = load_stream(col, val, (int64_t)cn * kChunk);
        const SegRegs seg_n = load_segs(tab_n, seg_end, seg_row);
        const int4 tab_nn = tabs[cnn];
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();

        // carry: the part of the row entering this chunk from before (wavefront 0)
        if (c > 0 && tid < kWave && first_off > 0) {
            double sacc = 0.0;
            for (int k = tid; k < first_off; k += kWave) sacc += prod[k];
            sacc = wave_sum(sacc);
            if (tid == 0) carry[c] = sacc;
        }
        // segments that start in this chunk: g lanes each
        const int g = lanes_per_segment(nseg);
        const int sub = tid & (g - 1);
        const int first = tid / g;
#pragma unroll
        for (int j = 0; j < kSegPasses; ++j) {
            if (j * kBlock < nseg && (g == 1 || j == 0)) {   // uniform over the workgroup
                const int sidx = first + kBlock * j;
                double sacc = 0.0;
                if (sidx < nseg) {
                    const int k0 = (sidx == 0) ? first_off : (int)ends[sidx - 1];
                    const int k1 = (int)ends[sidx];
                    for (int k = k0 + sub; k < k1; k += g) sacc += prod[k];
                }
                sacc = group_sum(sacc, g);
                if (sidx < nseg && sub == 0) partial[seg.rid[j]] = sacc;
            }
        }
        __syncthreads();  // prod / ends are reused by the next chunk
        cur = nxt;
        seg = seg_n;
        tab = tab_n;
        tab_n = tab_nn;
    }
}

// One chunk per workgroup (no LDS table): few registers, so eight workgroups fit on a CU and the memory latency of
// one is hidden by the others.  Loads are issued in two waves: {col/val stream, chunk table entry}, then
// {gathers, segment end offsets, row ids}.
__global__ __launch_bounds__(kBlock) void k_csr_spmv_part_np(PartArgs pa, int64_t rows, const int32_t *__restrict__ col_all,
                                                             const double *__restrict__ val_all, const int4 *__restrict__ chunk_tab,
                                                             const uint16_t *__restrict__ seg_end, const int32_t *__restrict__ seg_row_all,
                                                             const double *__restrict__ x, double *__restrict__ partial_all,
                                                             double *__restrict__ carry_all)
{
    __shared__ __align__(16) double prod[kChunk];
    __shared__ __align__(16) uint16_t ends[kChunk];
    const int tid = threadIdx.x;
    const int xp = blockIdx.x % pa.P;
    const int c = blockIdx.x / pa.P;
    if (c >= pa.nchunks[xp]) return;
    const int32_t *col = col_all + pa.base[xp];
    const double *val = val_all + pa.base[xp];
    const int32_t *seg_row = seg_row_all + pa.seg0[xp];
    double *partial = partial_all + (int64_t)xp * rows;

    const StreamRegs cur = load_stream(col, val, (int64_t)c * kChunk);   // col/val are padded to whole chunks
    const int4 tab = chunk_tab[pa.chunk0[xp] + c];
    const int nseg = tab.y, first_off = tab.z;
    double xg[2][4];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        xg[j][0] = load_elem(x, cur.c[j].x);
        xg[j][1] = load_elem(x, cur.c[j].y);
        xg[j][2] = load_elem(x, cur.c[j].z);
        xg[j][3] = load_elem(x, cur.c[j].w);
    }
    const SegRegs seg = load_segs(tab, seg_end, seg_row);
    if (8 * tid < nseg) *reinterpret_cast<uint4 *>(ends + 8 * tid) = seg.ends;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        double2 p0, p1;
        p0.x = cur.v[j][0].x * xg[j][0];
        p0.y = cur.v[j][0].y * xg[j][1];
        p1.x = cur.v[j][1].x * xg[j][2];
        p1.y = cur.v[j][1].y * xg[j][3];
        double2 *dst = reinterpret_cast<double2 *>(prod + j * (kChunk / 2) + tid * 4);
        dst[0] = p0;
        dst[1] = p1;
    }
    __syncthreads();
    if (c > 0 && tid < kWave && first_off > 0) {
        double sacc = 0.0;
        for (int k = tid; k < first_off; k += kWave) sacc += prod[k];
        sacc = wave_sum(sacc);
        if (tid == 0) carry_all[pa.chunk0[xp] + c] = sacc;
    }
    const int g = lanes_per_segment(nseg);
    const int sub = tid & (g - 1);
    const int first = tid / g;
#pragma unroll
    for (int j = 0; j < kSegPasses; ++j) {
        if (j * kBlock < nseg && (g == 1 || j == 0)) {
            const int sidx = first + kBlock * j;
            double sacc = 0.0;
            if (sidx < nseg) {
                const int k0 = (sidx == 0) ? first_off : (int)ends[sidx - 1];
                const int k1 = (int)ends[sidx];
                for (int k = k0 + sub; k < k1; k += g) sacc += prod[k];
            }
            sacc = group_sum(sacc, g);
            if (sidx < nseg && sub == 0) partial[seg.rid[j]] = sacc;
        }
    }
}

// ------------------------------------------------------------------ hot-row tiles (see HotTiles)
constexpr int kLongSegment = 64;   // segments at least this long are summed by a whole wavefront,
constexpr int kMidSegment = 8;     // at least this long by 8 lanes, shorter ones by one thread

int hot_tiles_build(CsrPlan &A, const int64_t *t_rowptr, const int32_t *t_col, const double *t_val,
                    const std::vector<int32_t> &slot_code, int nhot, hipStream_t st)
{
    HotTiles &H = A.hot;
    H.nhot = nhot;
    struct Entry { uint16_t slot, iloc; double val; };
    std::vector<Entry> cur[kTileSlices];
    int64_t base[kTileSlices] = {0};
    std::vector<double> tval[kTileSlices];
    std::vector<uint16_t> tiloc[kTileSlices];
    std::vector<uint32_t> sdesc[kTileSlices];
    std::vector<int4> hdrs[kTileSlices];
    std::vector<int> seglen(kTileSlots);
    std::vector<Entry> sorted;

    auto close_tile = [&](int s) {
        std::vector<Entry> &e = cur[s];
        if (e.empty()) return;
        // long segments first, then by slot; entries of a slot keep their column order
        for (const Entry &x : e) seglen[x.slot]++;
        sorted = e;
        auto cls = [&](int slot) { return seglen[slot] >= kLongSegment ? 0 : (seglen[slot] >= kMidSegment ? 1 : 2); };
        std::stable_sort(sorted.begin(), sorted.end(), [&](const Entry &a, const Entry &b) {
            const int ca = cls(a.slot), cb = cls(b.slot);
            if (ca != cb) return ca < cb;
            // inside the medium and short classes by length (the lanes of a wavefront then loop equally long)
            if (ca != 0 && seglen[a.slot] != seglen[b.slot]) return seglen[a.slot] > seglen[b.slot];
            return a.slot < b.slot;
        });
        int4 h = make_int4((int)base[s], 0, 0, (int)sdesc[s].size());
        const size_t off = tval[s].size();
        tval[s].resize(off + kChunk, 0.0);
        tiloc[s].resize(off + kChunk, 0);
        for (size_t k = 0; k < sorted.size(); ++k) {
            tval[s][off + k] = sorted[k].val;
            tiloc[s][off + k] = sorted[k].iloc;
            if (k + 1 == sorted.size() || sorted[k + 1].slot != sorted[k].slot) {
                sdesc[s].push_back((uint32_t)(k + 1) | ((uint32_t)sorted[k].slot << 16));
                h.y += 1;
                if (cls(sorted[k].slot) == 0) h.z += 1;          // low 16 bits: long segments
                if (cls(sorted[k].slot) == 1) h.z += 1 << 16;    // high 16 bits: medium segments
            }
        }
        while (sdesc[s].size() % 4) sdesc[s].push_back(0);
        hdrs[s].push_back(h);
        for (const Entry &x : e) seglen[x.slot] = 0;
        e.clear();
    };

    int cnt[kTileSlices];
    for (int64_t i = 0; i < A.cols; ++i) {
        for (int s = 0; s < kTileSlices; ++s) cnt[s] = 0;
        for (int64_t k = t_rowptr[i]; k < t_rowptr[i + 1]; ++k) {
            const int32_t code = slot_code[t_col[k]];
            if (code >= 0) cnt[code / kTileSlots]++;
        }
        for (int s = 0; s < kTileSlices; ++s) {
            if (!cnt[s]) continue;
            if ((int)cur[s].size() + cnt[s] > kChunk || (!cur[s].empty() && i - base[s] > 65535)) close_tile(s);
            if (cur[s].empty()) base[s] = i;
        }
        for (int64_t k = t_rowptr[i]; k < t_rowptr[i + 1]; ++k) {
            const int32_t code = slot_code[t_col[k]];
            if (code >= 0) H.nnz++;
            if (code >= 0) cur[code / kTileSlots].push_back({(uint16_t)(code % kTileSlots), (uint16_t)(i - base[code / kTileSlots]), t_val[k]});
        }
    }
    for (int s = 0; s < kTileSlices; ++s) close_tile(s);

    // concatenate the slices; segment offsets become global
    int64_t ntiles = 0, nseg = 0;
    for (int s = 0; s < kTileSlices; ++s) {
        H.tile0[s] = ntiles;
        H.ntiles[s] = (int64_t)hdrs[s].size();
        for (int4 &h : hdrs[s]) h.w += (int)nseg;
        ntiles += H.ntiles[s];
        nseg += (int64_t)sdesc[s].size();
    }
    H.ntiles_total = ntiles;
    if (ntiles == 0) return TRON_OK;
    if (nseg > 0x7ffffff0 || ntiles > 0x7ffffff0 / kChunk * 1024) { set_error("hot tiles too large"); return TRON_EINVAL; }
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.val), sizeof(double) * ntiles * kChunk));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.iloc), sizeof(uint16_t) * ntiles * kChunk));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.hdr), sizeof(int4) * ntiles));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.seg_desc), sizeof(uint32_t) * std::max<int64_t>(nseg, 4)));
    int64_t segpos = 0;
    for (int s = 0; s < kTileSlices; ++s) {
        const int64_t t0 = H.tile0[s];
        if (H.ntiles[s] == 0) continue;
        TRON_HIP(hipMemcpyAsync(H.val + t0 * kChunk, tval[s].data(), sizeof(double) * tval[s].size(), hipMemcpyHostToDevice, st));
        TRON_HIP(hipMemcpyAsync(H.iloc + t0 * kChunk, tiloc[s].data(), sizeof(uint16_t) * tiloc[s].size(), hipMemcpyHostToDevice, st));
        TRON_HIP(hipMemcpyAsync(H.hdr + t0, hdrs[s].data(), sizeof(int4) * hdrs[s].size(), hipMemcpyHostToDevice, st));
        TRON_HIP(hipMemcpyAsync(H.seg_desc + segpos, sdesc[s].data(), sizeof(uint32_t) * sdesc[s].size(), hipMemcpyHostToDevice, st));
        segpos += (int64_t)sdesc[s].size();
    }
    TRON_TRY(upload(&H.slot_of_row, slot_code.data(), slot_code.size(), st));
    int64_t maxt = 0;
    for (int s = 0; s < kTileSlices; ++s) maxt = std::max(maxt, H.ntiles[s]);
    H.blocks_per_slice = (int)std::max<int64_t>(1, std::min<int64_t>(maxt, g_tuning.csr_tile_blocks_per_slice));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.wg_acc), sizeof(double) * kTileSlices * H.blocks_per_slice * kTileSlots));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.sums), sizeof(double) * kTileSlices * kTileSlots));
    TRON_HIP(hipStreamSynchronize(st));
    return TRON_OK;
}

struct TileArgs {
    int64_t tile0[kTileSlices];
    int64_t ntiles[kTileSlices];
};

struct TileRegs {
    v2d v[4];
    uint32_t il[4];     // two 16-bit local column offsets each
    uint4 desc[2];      // segment descriptors 8*tid .. 8*tid+7: end offset | slot << 16
    int4 hdr;
};

// data of tile T whose header h is already in registers
__device__ __forceinline__ TileRegs load_tile(const double *__restrict__ val, const uint16_t *__restrict__ iloc, int4 h,
                                              const uint32_t *__restrict__ seg_desc, int64_t T)
{
    TileRegs r;
    r.hdr = h;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int64_t k = T * kChunk + m * (kChunk / 4) + threadIdx.x * 2;
        r.v[m] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(val + k));
        r.il[m] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(iloc + k));
    }
    // descriptor blocks are padded to a multiple of 4; threads beyond the tile's segments re-read its first block
    const int nseg = h.y;
    const int64_t d0 = (int64_t)h.w + ((8 * (int)threadIdx.x < nseg) ? 8 * (int)threadIdx.x : 0);
    const int64_t d1 = (int64_t)h.w + ((8 * (int)threadIdx.x + 4 < nseg) ? 8 * (int)threadIdx.x + 4 : 0);
    r.desc[0] = *reinterpret_cast<const uint4 *>(seg_desc + d0);
    r.desc[1] = *reinterpret_cast<const uint4 *>(seg_desc + d1);
    return r;
}

// Persistent workgroup (slice s, q): tiles q, q + B, ... of the slice; LDS accumulators for the slice's hot rows.
// Software pipeline: while tile t is reduced, the data of tiles t + B and t + 2B and the header of tile t + 3B are
// in flight (all indices clamped to the last tile, so every iteration issues the same loads).
// Segment sums: the segments of a tile are ordered long (>= 64 entries: one wavefront each), medium (>= 8: eight
// lanes each), short (one thread each, all seven possible reads issued together).  Slots inside a tile are
// distinct, so the accumulator updates of different segments never collide.
__global__ __launch_bounds__(kBlock) void k_hot_tiles(TileArgs ta, int B, const double *__restrict__ val,
                                                      const uint16_t *__restrict__ iloc, const int4 *__restrict__ hdr,
                                                      const uint32_t *__restrict__ seg_desc,
                                                      const double *__restrict__ x, double *__restrict__ wg_acc)
{
    __shared__ __align__(16) double prod[kChunk];
    __shared__ __align__(16) uint32_t desc[kChunk];
    __shared__ double acc[kTileSlots];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int s = blockIdx.x % kTileSlices;
    const int q = blockIdx.x / kTileSlices;
    for (int k = tid; k < kTileSlots; k += kBlock) acc[k] = 0.0;
    const int64_t nt = ta.ntiles[s];
    if (q < nt) {
        const int64_t T0 = ta.tile0[s];
        const int64_t last = nt - 1;
        auto clampt = [&](int64_t t) { return T0 + (t < last ? t : last); };
        TileRegs cur = load_tile(val, iloc, hdr[clampt(q)], seg_desc, clampt(q));
        TileRegs nxt = load_tile(val, iloc, hdr[clampt(q + B)], seg_desc, clampt(q + B));
        int4 hdr2 = hdr[clampt(q + 2 * (int64_t)B)];
        for (int64_t t = q; t < nt; t += B) {
            const int nseg = cur.hdr.y, nlong = cur.hdr.z & 0xffff, nmid = (unsigned)cur.hdr.z >> 16;
            const double *xt = x + cur.hdr.x;   // the tile's first column
            // gathers: a few consecutive cache lines of x per tile
            double xg[4][2];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                xg[m][0] = xt[cur.il[m] & 0xffffu];
                xg[m][1] = xt[cur.il[m] >> 16];
            }
            if (8 * tid < nseg) *reinterpret_cast<uint4 *>(desc + 8 * tid) = cur.desc[0];
            if (8 * tid + 4 < nseg) *reinterpret_cast<uint4 *>(desc + 8 * tid + 4) = cur.desc[1];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                double2 p;
                p.x = cur.v[m].x * xg[m][0];
                p.y = cur.v[m].y * xg[m][1];
                *reinterpret_cast<double2 *>(prod + m * (kChunk / 4) + tid * 2) = p;
            }
            __builtin_amdgcn_sched_barrier(0);
            const TileRegs nn = load_tile(val, iloc, hdr2, seg_desc, clampt(t + 2 * (int64_t)B));
            const int4 hdr3 = hdr[clampt(t + 3 * (int64_t)B)];
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            // long segments: one wavefront each
            for (int sg = tid / kWave; sg < nlong; sg += kWavesPerBlock) {
                const int k0 = sg ? (int)(desc[sg - 1] & 0xffffu) : 0;
                const uint32_t dsc = desc[sg];
                const int k1 = (int)(dsc & 0xffffu);
                double sacc = 0.0;
                for (int k = k0 + lane; k < k1; k += kWave) sacc += prod[k];
                sacc = wave_sum(sacc);
                if (lane == 0) acc[dsc >> 16] += sacc;
            }
            // LDS bandwidth is what these sums cost, so each lane reads exactly the entries it needs; segments of
            // the medium and short classes are ordered by length, so the lanes of a wavefront loop equally long.
            // medium segments (8..63 entries): eight lanes each
            {
                const int sub = lane & 7;
                const int mid_end = nlong + nmid;
                for (int sg = nlong + tid / 8; sg < mid_end; sg += kBlock / 8) {
                    const int k0 = sg ? (int)(desc[sg - 1] & 0xffffu) : 0;
                    const uint32_t dsc = desc[sg];
                    const int k1 = (int)(dsc & 0xffffu);
                    double sacc = 0.0;
                    for (int k = k0 + sub; k < k1; k += 8) sacc += prod[k];
                    sacc = sum8(sacc);
                    if (sub == 0) acc[dsc >> 16] += sacc;
                }
            }
            // short segments (1..7 entries): one thread each
            for (int sg = nlong + nmid + tid; sg < nseg; sg += kBlock) {
                const int k0 = sg ? (int)(desc[sg - 1] & 0xffffu) : 0;
                const uint32_t dsc = desc[sg];
                const int k1 = (int)(dsc & 0xffffu);
                double sacc = prod[k0];
                for (int k = k0 + 1; k < k1; ++k) sacc += prod[k];
                acc[dsc >> 16] += sacc;
            }
            __syncthreads();
            cur = nxt;
            nxt = nn;
            hdr2 = hdr3;
        }
    }
    __syncthreads();
    double *out = wg_acc + ((int64_t)s * B + q) * kTileSlots;
    for (int k = tid; k < kTileSlots; k += kBlock) out[k] = acc[k];
}

// sums[s*K + k] = sum over the B workgroups of slice s, in workgroup order
__global__ __launch_bounds__(kBlock) void k_hot_reduce(int B, const double *__restrict__ wg_acc, double *__restrict__ sums)
{
    const int idx = blockIdx.x * kBlock + threadIdx.x;   // s*K + k
    if (idx >= kTileSlices * kTileSlots) return;
    const int s = idx / kTileSlots, k = idx % kTileSlots;
    const double *p = wg_acc + (int64_t)s * B * kTileSlots + k;
    double a = 0.0;
    for (int q = 0; q < B; ++q) a += p[(int64_t)q * kTileSlots];
    sums[idx] = a;
}

static int launch_hot_tiles(tron_dataset *ds, const CsrPlan &A, const double *x)
{
    const HotTiles &H = A.hot;
    TileArgs ta;
    for (int s = 0; s < kTileSlices; ++s) { ta.tile0[s] = H.tile0[s]; ta.ntiles[s] = H.ntiles[s]; }
    // The tiles stream from HBM, the CSR remainder waits on gather misses: they run side by side on two streams.
    hipStream_t st = g_tuning.csr_two_streams ? ds->side : ds->stream;
    if (st != ds->stream) {
        TRON_HIP(hipEventRecord(ds->ev_fork, ds->stream));
        TRON_HIP(hipStreamWaitEvent(st, ds->ev_fork, 0));
    }
    {
        ProfScope ps(ds, SLOT_SPMV_TILES, st);
        hipLaunchKernelGGL(k_hot_tiles, dim3(kTileSlices * H.blocks_per_slice), dim3(kBlock), 0, st, ta, H.blocks_per_slice,
                           H.val, H.iloc, H.hdr, H.seg_desc, x, H.wg_acc);
        hipLaunchKernelGGL(k_hot_reduce, dim3(kTileSlices * kTileSlots / kBlock), dim3(kBlock), 0, st, H.blocks_per_slice,
                           H.wg_acc, H.sums);
        TRON_HIP(hipGetLastError());
    }
    if (st != ds->stream) TRON_HIP(hipEventRecord(ds->ev_join, st));
    return TRON_OK;
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
// sum over the partitions in which row r has entries (bit x of mask), in partition order
struct HotRef {
    const int32_t *slot_of_row;   // null: no hot rows
    const double *sums;
};

__device__ __forceinline__ double sum_parts(const double *__restrict__ partial, const uint8_t *__restrict__ mask, int64_t rows, int64_t r,
                                            HotRef hot = HotRef{nullptr, nullptr})
{
    const unsigned m = mask[r];
    double s = 0.0;
    if (hot.slot_of_row) {
        const int hs = hot.slot_of_row[r];
        if (hs >= 0) s = hot.sums[hs];
    }
#pragma unroll
    for (int x = 0; x < kMaxParts; ++x)
        if (m & (1u << x)) s += partial[(int64_t)x * rows + r];
    return s;
}

// z = sum of partials; loss terms; partial slot 0 = sum loss
template <int LOSS>
__global__ __launch_bounds__(kBlock) void k_combine_loss(int64_t n, const double *__restrict__ partial, const uint8_t *__restrict__ mask,
                                                         const double *__restrict__ y, double *__restrict__ zhat,
                                                         double *__restrict__ D, double *__restrict__ red)
{
    __shared__ double lds[kWavesPerBlock];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        const double z = sum_parts(partial, mask, n, i);
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
__global__ __launch_bounds__(kBlock) void k_combine_scale(int64_t rows, const double *__restrict__ partial, const uint8_t *__restrict__ mask,
                                                          const double *__restrict__ scale, double *__restrict__ out)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < rows; i += (int64_t)gridDim.x * kBlock)
        out[i] = scale[i] * sum_parts(partial, mask, rows, i);
}

// out = add + alpha * sum of partials; partial slot 0 = out . (SELF ? out : add)
template <bool SELF>
__global__ __launch_bounds__(kBlock) void k_combine_axpy(int64_t rows, const double *__restrict__ partial, const uint8_t *__restrict__ mask,
                                                         const double *__restrict__ add, double alpha,
                                                         double *__restrict__ out, double *__restrict__ red, HotRef hot)
{
    __shared__ double lds[kWavesPerBlock];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < rows; i += (int64_t)gridDim.x * kBlock) {
        const double a = add[i];
        const double o = fma(alpha, sum_parts(partial, mask, rows, i, hot), a);
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
        pa.seg0[i] = A.part_seg0[i];
        pa.chunk0[i] = A.part_chunk0[i];
        pa.nchunks[i] = A.part_nchunks[i];
        pa.nhot[i] = A.part_nhot[i];
    }
    {
        ProfScope ps(ds, slot);
        const int want = (int)(A.hot_ids ? g_tuning.csr_hot_blocks_per_part : g_tuning.csr_blocks_per_part);
        const int per_part = std::max(1, std::min(A.max_chunks, want));
        if (A.hot_ids)
            hipLaunchKernelGGL(k_csr_spmv_part<true>, dim3(per_part * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows, A.col, A.val,
                               A.chunk_tab, A.seg_end, A.seg_row, A.hot_ids, x, ds->row_partials, A.carry);
        else if (g_tuning.csr_blocks_per_part > 0)
            hipLaunchKernelGGL(k_csr_spmv_part<false>, dim3(per_part * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows, A.col, A.val,
                               A.chunk_tab, A.seg_end, A.seg_row, (const int32_t *)nullptr, x, ds->row_partials, A.carry);
        else
            hipLaunchKernelGGL(k_csr_spmv_part_np, dim3(A.max_chunks * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows, A.col, A.val,
                               A.chunk_tab, A.seg_end, A.seg_row, x, ds->row_partials, A.carry);
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
        hipLaunchKernelGGL(k_combine_loss<TRON_LOSS_LR>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, ds->row_partials, A.row_mask, ds->y, zhat, D, ds->partials);
    else
        hipLaunchKernelGGL(k_combine_loss<TRON_LOSS_L2SVM>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, ds->row_partials, A.row_mask, ds->y, zhat, D, ds->partials);
    TRON_HIP(hipGetLastError());
    return g;
}

int spmv_scale(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, const double *scale, double *out)
{
    if (A.P == 1) return launch_plain<EPI_SCALE>(ds, A, slot, x, out, scale, 0.0);
    TRON_TRY(launch_partials(ds, A, slot, x));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    hipLaunchKernelGGL(k_combine_scale, dim3(vec_grid(A.rows)), dim3(kBlock), 0, ds->stream, A.rows, ds->row_partials, A.row_mask, scale, out);
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
    HotRef hot{nullptr, nullptr};
    if (A.hot.ntiles_total > 0) {
        TRON_TRY(launch_hot_tiles(ds, A, x));
        hot.slot_of_row = A.hot.slot_of_row;
        hot.sums = A.hot.sums;
    }
    TRON_TRY(launch_partials(ds, A, slot, x));
    if (hot.sums && g_tuning.csr_two_streams) TRON_HIP(hipStreamWaitEvent(ds->stream, ds->ev_join, 0));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    const int g = vec_grid(A.rows);
    if (dot_self)
        hipLaunchKernelGGL(k_combine_axpy<true>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, ds->row_partials, A.row_mask, add, alpha, out, ds->partials, hot);
    else
        hipLaunchKernelGGL(k_combine_axpy<false>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, ds->row_partials, A.row_mask, add, alpha, out, ds->partials, hot);
    TRON_HIP(hipGetLastError());
    return g;
}

}  // namespace tron
