// Sparse matrix-vector products for both orientations (X and the explicit X^T copy):
//   z = X w,  a1 = D .* (X v)               (Table 1 / Appendix D of the paper: a0 = X v, a1 = D a0)
//   g = w + C X^T zhat,  Hv = v + C X^T a1   (a2 = C X^T a1)
//
// Work is split by nonzeros, not by rows, because row lengths are heavily skewed (Zipf-distributed
// features give the transposed copy rows of length ~n next to millions of length 0/1): a workgroup
// streams one chunk of kChunk nonzeros with 16-byte non-temporal loads that cover whole cache lines,
// multiplies them by the gathered vector entries and parks the products in LDS; the sums of the row
// pieces ("segments") of the chunk come out of a segmented scan (see chunk_runs).  Rows and segments that fit
// into a chunk are stored so that they never cross a chunk boundary; one longer than a chunk receives the rest
// from the `carry` of the following chunks in a small fix-up kernel, in a fixed order -- nothing is ever added in
// an order that depends on timing, so results are bit-reproducible (the one atomic instruction in use, the LDS
// add of the unit tile kernel, has a fixed order too).
//
// The gathers decide the speed.  A gather that misses the vector L1 costs an L2 request of its own, and
// a CU keeps only ~100 of them in flight; one that misses L2 as well pulls a 64-byte sector for 8 useful
// bytes.  Large matrices are therefore regrouped by where the gathered element can be kept:
//   - forward orientation: a head partition (the most frequent columns of the whole matrix, served from
//     one LDS table, 16-bit slots, whole rows) and 8 column ranges, workgroup b on range b % 8 so that
//     each XCD's L2 gathers from its own slice of the vector; each range has an LDS table of its own;
//   - transposed orientation: hot-row tiles (see HotTiles: LDS accumulators, gathers from a copy of the tile's
//     columns in LDS) and 8 column ranges for the rest.
// Partitions write one partial sum per segment; combine kernels add a row's partial sums in a fixed
// order and apply the epilogue (loss terms, D scaling, v + C * sum) and the first stage of the scalar
// reductions.
#include <algorithm>
#include <cstring>
#include <exception>
#include <thread>

#include "device_util.h"

namespace tron {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef double v2d __attribute__((ext_vector_type(2)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

constexpr int64_t kGatherBytesForPartitioning = 3 << 19;  // 1.5 MiB: larger gather vectors get partitioned
constexpr int64_t kMinNnzForPartitioning = 1 << 22;
constexpr int kHotMinCount = 8;   // columns with fewer entries are not worth an LDS slot

void HotTiles::release()
{
    hipFree(val); hipFree(iloc); hipFree(flags); hipFree(hdr); hipFree(seg_slot); hipFree(slot_of_row);
    hipFree(wg_acc); hipFree(sums);
    *this = HotTiles();
}

void SellHead::release()
{
    hipFree(wave_off); hipFree(data); hipFree(sums); hipFree(pos);
    *this = SellHead();
}

void CsrPlan::release()
{
    hot.release();
    sell.release();
    hipFree(rowptr); hipFree(col); hipFree(col16); hipFree(val); hipFree(row_lo); hipFree(carry);
    hipFree(xs); hipFree(hot_ids); hipFree(hot_x); hipFree(group_base); hipFree(chunk_tab); hipFree(flags); hipFree(row_mask);
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

// fn(first, last) over [0, n) cut into equal ranges, one host thread per range (at most eight; small n: the caller's
// thread alone).  fn must not throw and must write only what belongs to its own range.
template <class F>
static void parallel_ranges(int64_t n, F &&fn)
{
    unsigned T = std::thread::hardware_concurrency();
    T = std::max(1u, std::min(8u, T));
    if (n < (1 << 16)) T = 1;
    const int64_t per = (n + T - 1) / T;
    std::vector<std::thread> workers;
    unsigned started = 0;
    try {
        for (unsigned t = 1; t < T; ++t) {
            workers.emplace_back(fn, std::min<int64_t>(n, (int64_t)t * per), std::min<int64_t>(n, (int64_t)(t + 1) * per));
            ++started;
        }
    } catch (const std::exception &) {
        // no more threads to be had: the remaining ranges run below
    }
    fn((int64_t)0, std::min<int64_t>(n, per));
    for (unsigned t = 1 + started; t < T; ++t) fn(std::min<int64_t>(n, (int64_t)t * per), std::min<int64_t>(n, (int64_t)(t + 1) * per));
    for (std::thread &w : workers) w.join();
}

int csr_plan_build(CsrPlan &A, int64_t rows, int64_t cols, const int64_t *h_rowptr, const int32_t *h_col,
                   const double *h_val, int parts, bool hot, bool unit, hipStream_t st)
{
    A.rows = rows;
    A.cols = cols;
    A.nnz = h_rowptr[rows];
    A.unit = unit;
    if (parts <= 0)
        parts = (cols * (int64_t)sizeof(double) > kGatherBytesForPartitioning && A.nnz >= kMinNnzForPartitioning) ? kColParts : 1;
    if (parts > kColParts) parts = kColParts;
    A.P = parts;
    A.plain = (parts == 1);
    std::vector<int32_t> row_lo, fix_row, fix_part, fix_b0, fix_cnt;

    if (A.unit && A.P == 1) { set_error("internal: unit plan without partitions"); return TRON_EINVAL; }
    if (A.plain && g_tuning.csr_segmented != 0) {
        // The plain kernel gives a chunk's rows groups of g = 256 / (rows starting in the chunk) lanes, one thread per row
        // when there are more than 128: a row of hundreds of entries among many short ones (the middle of a Zipf
        // distribution, in the transposed copy) then keeps one thread adding for tens of microseconds.  Count, per chunk,
        // the additions the busiest thread would make; beyond 96 the segment layout (scans, no per-row loops) is used.
        bool segmented = g_tuning.csr_segmented > 0;
        int64_t r = 0;
        const int64_t nchunks = (A.nnz + kChunk - 1) / kChunk;
        for (int64_t c = 0; c < nchunks && !segmented; ++c) {
            const int64_t start = c * kChunk, end = std::min<int64_t>(A.nnz, start + kChunk);
            while (r < rows && h_rowptr[r] < start) ++r;
            int64_t nrows = 0, longest = 0;
            for (int64_t q = r; q < rows && h_rowptr[q] < end; ++q) {
                ++nrows;
                longest = std::max<int64_t>(longest, std::min<int64_t>(h_rowptr[q + 1], end) - h_rowptr[q]);
            }
            int64_t g = 1;
            while (g < kWave && nrows * (g * 2) <= kBlock) g *= 2;
            if ((longest + g - 1) / g > 96) segmented = true;
        }
        if (segmented) A.plain = false;
    }
    hot = hot && A.P > 1;   // LDS tables belong to the column ranges of large matrices
    if (A.plain) {
        // A row that fits into a chunk never straddles a chunk boundary: one that would is moved to the start of the next
        // chunk.  The gap it leaves is counted to the row before, filled with zeros at that row's last column (they add
        // 0 times an entry of the vector the row reads anyway).  Only rows longer than a chunk are still completed by the
        // fix-up kernel; for matrices of short rows that launch disappears.
        std::vector<int64_t> rp((size_t)rows + 1);
        int64_t at = 0;
        for (int64_t r = 0; r < rows; ++r) {
            const int64_t len = h_rowptr[r + 1] - h_rowptr[r];
            if (len > 0 && len <= kChunk && at % kChunk + len > kChunk) at = (at / kChunk + 1) * kChunk;
            rp[r] = at;
            at += len;
        }
        rp[rows] = at;
        const int64_t stored = at;
        std::vector<int32_t> pcol((size_t)stored);
        std::vector<double> pval((size_t)stored);
        {
            int64_t filled = 0;
            int32_t last_col = 0;
            for (int64_t r = 0; r < rows; ++r) {
                for (; filled < rp[r]; ++filled) { pcol[filled] = last_col; pval[filled] = 0.0; }
                for (int64_t k = h_rowptr[r]; k < h_rowptr[r + 1]; ++k, ++filled) { pcol[filled] = h_col[k]; pval[filled] = h_val[k]; }
                if (h_rowptr[r + 1] > h_rowptr[r]) last_col = h_col[h_rowptr[r + 1] - 1];
            }
        }
        const int64_t nb64 = std::max<int64_t>(1, (stored + kChunk - 1) / kChunk);
        if (nb64 > 0x7ffffff0) { set_error("matrix too large: %lld chunks", (long long)nb64); return TRON_EINVAL; }
        A.nblocks = (int)nb64;
        A.part_base[0] = 0; A.part_nnz[0] = stored; A.part_chunk0[0] = 0; A.part_nchunks[0] = A.nblocks;
        A.max_chunks = A.nblocks;
        plan_chunks(rp.data(), rows, stored, A.nblocks, 0, 0, row_lo, fix_row, fix_part, fix_b0, fix_cnt);
        TRON_TRY(upload(&A.rowptr, rp.data(), (size_t)rows + 1, st));
        TRON_TRY(upload(&A.col, pcol.data(), (size_t)stored, st));
        TRON_TRY(upload(&A.val, pval.data(), (size_t)stored, st));
        TRON_HIP(hipStreamSynchronize(st));   // the staging vectors go out of scope
    } else {
        const int P = A.P;
        std::vector<int64_t> colcount((size_t)cols + 1, 0);
        for (int64_t k = 0; k < A.nnz; ++k) colcount[h_col[k] + 1]++;
        // Head partition: the kHotSlots most frequent columns of the whole matrix, when they hold a good part of
        // the nonzeros.  Their entries need no locality in L2 (one LDS table serves them all), so they are not
        // split by column range: one segment per row instead of one per row and range.
        std::vector<uint8_t> part_of((size_t)cols, 0);
        std::vector<int32_t> slot_of, hot_ids;
        std::vector<std::pair<int64_t, int32_t>> cand;
        int64_t head_nnz = 0;
        // unit plans keep the head partition as sorted slices (SellHead) instead of chunks, with a larger table
        const bool want_sell = A.unit && g_tuning.csr_sell != 0;
        A.head_slots = want_sell ? kSellSlots : kHotSlots;
        if (hot) {
            A.range_slots = (int)std::min<int64_t>(kHotSlots, std::max<int64_t>(2, g_tuning.csr_range_slots / 2 * 2));
            slot_of.assign((size_t)cols, -1);
            hot_ids.assign((size_t)P * kHotSlots + A.head_slots, 0);
        }
        if (hot && g_tuning.csr_head) {
            for (int64_t j = 0; j < cols; ++j)
                if (colcount[j + 1] >= kHotMinCount) cand.emplace_back(-colcount[j + 1], (int32_t)j);
            const size_t keep = std::min<size_t>(cand.size(), (size_t)A.head_slots);
            std::partial_sort(cand.begin(), cand.begin() + keep, cand.end());
            for (size_t k = 0; k < keep; ++k) head_nnz -= cand[k].first;
            if (head_nnz * 4 >= A.nnz) {
                A.head = P;
                A.part_nhot[P] = (int)keep;
                A.part_nnz[P] = head_nnz;
                for (size_t k = 0; k < keep; ++k) {
                    part_of[cand[k].second] = (uint8_t)P;
                    slot_of[cand[k].second] = (int32_t)k;
                    hot_ids[(size_t)P * kHotSlots + k] = cand[k].second;
                    colcount[cand[k].second + 1] = 0;   // not counted in the ranges below
                }
            }
        }
        const bool sell = want_sell && A.head >= 0;
        const int NP = (A.head >= 0 && !sell) ? P + 1 : P;   // chunked partitions in all
        const int64_t range_nnz = A.nnz - ((A.head >= 0) ? head_nnz : 0);
        // column ranges with equal nonzero counts (head columns excluded): bound[x] = first column of range x
        for (int64_t j = 0; j < cols; ++j) colcount[j + 1] += colcount[j];
        std::vector<int64_t> bound(P + 1, cols);
        bound[0] = 0;
        for (int x = 1; x < P; ++x) {
            const int64_t target = range_nnz / P * x;
            bound[x] = std::lower_bound(colcount.begin(), colcount.end(), target) - colcount.begin();
            if (bound[x] > cols) bound[x] = cols;
            if (bound[x] < bound[x - 1]) bound[x] = bound[x - 1];
        }
        for (int x = 0; x < P; ++x)
            for (int64_t j = bound[x]; j < bound[x + 1]; ++j)
                if (part_of[j] != P || A.head < 0) part_of[j] = (uint8_t)x;
        for (int x = 0; x < P; ++x) A.part_nnz[x] = colcount[bound[x + 1]] - colcount[bound[x]];
        for (int x = 0; x < NP; ++x)
            if (A.part_nnz[x] > 0x7ffffff0) { set_error("partition too large for 32-bit offsets"); return TRON_EINVAL; }
        // LDS-resident columns of a range: its kHotSlots most frequent columns with at least kHotMinCount entries
        if (hot) {
            for (int x = 0; x < P; ++x) {
                cand.clear();
                for (int64_t j = bound[x]; j < bound[x + 1]; ++j) {
                    const int64_t cnt = colcount[j + 1] - colcount[j];   // 0 for head columns
                    if (cnt >= kHotMinCount) cand.emplace_back(-cnt, (int32_t)j);
                }
                const size_t keep = std::min<size_t>(cand.size(), (size_t)A.range_slots);
                std::partial_sort(cand.begin(), cand.begin() + keep, cand.end());
                A.part_nhot[x] = (int)keep;
                for (size_t k = 0; k < keep; ++k) {
                    slot_of[cand[k].second] = (int32_t)k;
                    hot_ids[(size_t)x * kHotSlots + k] = cand[k].second;
                }
            }
        }
        for (int64_t j = 0; j < cols; ++j)   // head columns have count 0 here
            if (colcount[j + 1] > colcount[j] && !(hot && slot_of[j] >= 0)) A.cold_cols++;
        std::vector<int64_t>().swap(colcount);
        // per-(partition,row) entry counts -> offsets; non-empty pairs are the segments.  A segment that would straddle a
        // chunk boundary is moved to the start of the next chunk (the gap it leaves is padding that reaches no sum), so
        // that a chunk never continues a row of the chunk before and no carry / fix-up pass is needed; only a segment
        // longer than a whole chunk is still split.
        std::vector<int32_t> rp32((size_t)NP * (rows + 1), 0);    // start of (x, r) relative to the partition
        std::vector<int32_t> len32((size_t)NP * rows, 0);         // its number of entries
        std::vector<int32_t> head_cnt(sell ? (size_t)rows : 0, 0);   // entries of the row in a head kept as sorted slices
        // one table for the passes over the entries below: partition in the upper half, LDS slot + 1 (0: none) in the lower
        std::vector<int32_t> code_of((size_t)cols);
        for (int64_t j = 0; j < cols; ++j) code_of[j] = ((int32_t)part_of[j] << 16) | ((hot && slot_of[j] >= 0) ? slot_of[j] + 1 : 0);
        parallel_ranges(rows, [&](int64_t r0, int64_t r1) {
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t k = h_rowptr[r]; k < h_rowptr[r + 1]; ++k) {
                    const int x = code_of[h_col[k]] >> 16;
                    if (x < NP) len32[(size_t)x * rows + r]++;
                    else if (sell && x == P) head_cnt[r]++;
                }
        });
        // a head kept as sorted slices: the slots of a row's head entries, row after row (filled with the ranges below)
        std::vector<int64_t> head_off(sell ? (size_t)rows + 1 : 0, 0);
        for (int64_t r = 0; sell && r < rows; ++r) head_off[r + 1] = head_off[r] + head_cnt[r];
        std::vector<uint16_t> head_slot(sell ? (size_t)head_off[rows] : 0);
        std::vector<uint16_t> mask((size_t)rows, 0);
        int64_t pos = 0, nseg_total = 0;
        int chunk = 0;
        A.max_chunks = 0;
        for (int x = 0; x < NP; ++x) {
            int32_t *rp = rp32.data() + (size_t)x * (rows + 1);
            const int32_t *ln = len32.data() + (size_t)x * rows;
            int64_t nseg = 0, at = 0;
            for (int64_t r = 0; r < rows; ++r) {
                const int64_t len = ln[r];
                if (len > 0) {
                    mask[r] |= (uint16_t)(1u << x);
                    ++nseg;
                    if (len <= kChunk && at % kChunk + len > kChunk) at = (at / kChunk + 1) * kChunk;
                }
                rp[r] = (int32_t)at;
                at += len;
                if (at > 0x7ffffff0) { set_error("partition too large for 32-bit offsets"); return TRON_EINVAL; }
            }
            rp[rows] = (int32_t)at;
            A.part_base[x] = pos;
            A.part_seg0[x] = nseg_total;
            A.part_chunk0[x] = chunk;
            A.part_nchunks[x] = (int)std::max<int64_t>(1, (at + kChunk - 1) / kChunk);
            if (x < P) A.max_chunks = std::max(A.max_chunks, A.part_nchunks[x]);
            chunk += A.part_nchunks[x];
            pos += (int64_t)A.part_nchunks[x] * kChunk;
            nseg_total += nseg;
        }
        A.nblocks = chunk;
        if (nseg_total > 0x7ffffff0) { set_error("too many row segments for 32-bit indexing"); return TRON_EINVAL; }
        // entries partition-major; inside a row the entries of one range are contiguous and stay ordered
        std::vector<int32_t> pcol((size_t)pos, 0);
        std::vector<double> pval(A.unit ? 0 : (size_t)pos, 0.0);
        parallel_ranges(rows, [&](int64_t r0, int64_t r1) {   // a row's places belong to that row alone
            int64_t cursor[kMaxParts + 1];
            for (int64_t r = r0; r < r1; ++r) {
                for (int x = 0; x < NP; ++x) cursor[x] = A.part_base[x] + rp32[(size_t)x * (rows + 1) + r];
                int64_t hq = sell ? head_off[r] : 0;
                for (int64_t k = h_rowptr[r]; k < h_rowptr[r + 1]; ++k) {
                    const int32_t code = code_of[h_col[k]];
                    const int x = code >> 16, slot1 = code & 0xffff;
                    if (x >= NP) {   // head entries of a plan with sorted slices
                        if (sell && x == P) head_slot[hq++] = (uint16_t)(slot1 - 1);
                        continue;
                    }
                    const int64_t q = cursor[x]++;
                    pcol[q] = slot1 ? ~(slot1 - 1) : h_col[k];   // the head's become 16-bit slots below
                    if (!A.unit) pval[q] = h_val[k];
                }
            }
        });
        // segment tables
        std::vector<int32_t> seg_row((size_t)std::max<int64_t>(nseg_total, 1));
        std::vector<int4> tab((size_t)chunk);
        std::vector<uint8_t> flags((size_t)chunk * kBlock, 0);   // per chunk: one bit per entry, set on the last entry of a segment
        for (int x = 0; x < NP; ++x) {
            const int32_t *rp = rp32.data() + (size_t)x * (rows + 1);
            const int32_t *ln = len32.data() + (size_t)x * rows;
            const int nch = A.part_nchunks[x];
            // the segments of this partition, in row order, with start/end positions relative to the partition
            int64_t m = 0;               // segment counter (partition-relative)
            int c = 0;                   // chunk that owns the segments being emitted
            int4 t = make_int4(0, 0, 0, 0);
            auto close_chunk = [&](int next_first_seg, int64_t next_seg_start) {
                tab[A.part_chunk0[x] + c] = t;
                ++c;
                const int64_t cstart = (int64_t)c * kChunk;
                const int64_t off = std::min<int64_t>(std::max<int64_t>(next_seg_start - cstart, 0), kChunk);
                t = make_int4(next_first_seg, 0, (int)off, 0);
            };
            for (int64_t r = 0; r < rows; ++r) {
                const int64_t rs = rp[r], re = rs + ln[r];
                if (re == rs) continue;
                while (rs >= (int64_t)(c + 1) * kChunk) close_chunk((int)m, rs);   // this segment starts in a later chunk
                seg_row[A.part_seg0[x] + m] = (int32_t)r;
                t.y += 1;
                // the row's piece in each chunk it touches ends with a flag; continuation chunks go to the fix-up list
                const int c_last = (int)((re - 1) / kChunk);
                for (int ck = c; ck <= c_last; ++ck) {
                    const int64_t pe = std::min<int64_t>(re, (int64_t)(ck + 1) * kChunk) - 1 - (int64_t)ck * kChunk;
                    flags[((size_t)A.part_chunk0[x] + ck) * kBlock + pe / 8] |= (uint8_t)(1u << (pe % 8));
                }
                if (c_last > c) {
                    fix_row.push_back((int32_t)(A.part_seg0[x] + m));   // partitioned plans: the segment's slot in the partial sums
                    fix_part.push_back(0);
                    fix_b0.push_back(A.part_chunk0[x] + c + 1);
                    fix_cnt.push_back(c_last - c);
                }
                ++m;
            }
            while (c < nch - 1) close_chunk((int)m, (int64_t)rp[rows]);
            tab[A.part_chunk0[x] + c] = t;
        }
        // first_off of a chunk inside or at the end of a split row: the chunk-relative end of that row
        // (set above from the start of the next segment; for chunks wholly inside one row that start lies
        // beyond the chunk and clips to kChunk, which is right)
        if (hot) {
            TRON_TRY(upload(&A.hot_ids, hot_ids.data(), hot_ids.size(), st));   // unused slots: column 0
            TRON_HIP(hipMalloc(reinterpret_cast<void **>(&A.hot_x), sizeof(double) * hot_ids.size()));
        }
        if (sell) {
            // ---- sorted slices of the head partition
            const std::vector<int32_t> &cnt = head_cnt;   // counted with the segment lengths above
            struct Slice { int32_t len8; int64_t first; };   // first: position of its 64 rows in `order`
            std::vector<int32_t> order((size_t)rows);
            std::vector<Slice> slices;
            for (int64_t w0 = 0; w0 < rows; w0 += kSellWindow) {
                const int64_t w1 = std::min<int64_t>(rows, w0 + kSellWindow);
                for (int64_t r = w0; r < w1; ++r) order[r] = (int32_t)r;
                std::stable_sort(order.begin() + w0, order.begin() + w1, [&](int32_t a, int32_t b) { return cnt[a] > cnt[b]; });
                for (int64_t s0 = w0; s0 < w1; s0 += kWave) {
                    const int32_t longest = cnt[order[s0]];
                    if (longest == 0) break;   // the rest of the window has no head entries
                    slices.push_back({(longest + 7) / 8, s0});
                }
            }
            std::stable_sort(slices.begin(), slices.end(), [](const Slice &a, const Slice &b) { return a.len8 > b.len8; });
            SellHead &S = A.sell;
            S.on = true;
            S.nslices = (int)slices.size();
            S.nwaves = (int)std::max<int64_t>(1, std::min<int64_t>(g_tuning.csr_sell_blocks, 4096)) * kWavesPerBlock;
            // longest first, each slice to the wavefront with the least work so far (ties: the lower wavefront)
            std::vector<std::vector<int32_t>> mine((size_t)S.nwaves);
            {
                std::vector<std::pair<int64_t, int32_t>> heap;   // (-load, -wave): the top is the least loaded, lowest wave
                for (int w = 0; w < S.nwaves; ++w) heap.emplace_back(0, -w);
                std::make_heap(heap.begin(), heap.end());
                for (size_t i = 0; i < slices.size(); ++i) {
                    std::pop_heap(heap.begin(), heap.end());
                    auto &top = heap.back();
                    mine[(size_t)(-top.second)].push_back((int32_t)i);
                    top.first -= slices[i].len8;
                    std::push_heap(heap.begin(), heap.end());
                }
            }
            std::vector<int64_t> wave_off((size_t)S.nwaves + 1);
            std::vector<int64_t> goff(slices.size());    // header group of each slice (in stored order)
            std::vector<int32_t> stored(slices.size());  // stored position -> index into slices
            int64_t groups = 0;
            int32_t sl = 0;
            std::vector<int64_t> null_groups;   // padding of every stream to a whole number of kSellAhead groups
            for (int w = 0; w < S.nwaves; ++w) {
                wave_off[w] = groups;
                for (int32_t i : mine[(size_t)w]) {
                    stored[sl] = i;
                    goff[sl] = groups;
                    groups += 1 + slices[i].len8;
                    ++sl;
                }
                while ((groups - wave_off[w]) % kSellAhead) null_groups.push_back(groups++);
            }
            wave_off[S.nwaves] = groups;
            S.ngroups = groups;
            for (int64_t r = 0; r < rows; ++r) S.nrows_with_entries += cnt[r] > 0;
            std::vector<uint16_t> data((size_t)std::max<int64_t>(groups, 1) * kWave * 8, (uint16_t)kSellSlots);
            for (int64_t gpad : null_groups)
                for (int l = 0; l < kWave; ++l) {
                    const int32_t hdr[4] = {-1, 0, 0, 0};   // a header of a slice without groups
                    std::memcpy(&data[((size_t)gpad * kWave + l) * 8], hdr, sizeof(hdr));
                }
            parallel_ranges((int64_t)slices.size(), [&](int64_t p0, int64_t p1) {   // a slice's groups belong to it alone
            for (int64_t p = p0; p < p1; ++p) {
                const Slice &sc = slices[stored[p]];
                const int64_t w1 = std::min<int64_t>(rows, (sc.first / kSellWindow + 1) * (int64_t)kSellWindow);
                for (int l = 0; l < kWave; ++l) {
                    int32_t hdr[4] = {-1, sc.len8, 0, 0};
                    const int64_t pos = sc.first + l;
                    const int32_t r = (pos < w1) ? order[pos] : -1;
                    if (r >= 0 && cnt[r] > 0) {
                        hdr[0] = (int32_t)pos;   // sums are kept in sorted order
                        // entry j of the row: group 1 + j / 8 of the slice, lane l, place j % 8
                        const uint16_t *hs = head_slot.data() + head_off[r];
                        for (int j = 0; j < cnt[r]; ++j) data[((size_t)(goff[p] + 1 + j / 8) * kWave + l) * 8 + j % 8] = hs[j];
                    }
                    std::memcpy(&data[((size_t)goff[p] * kWave + l) * 8], hdr, sizeof(hdr));
                }
            }
            });
            {
                std::vector<int32_t> pos_of((size_t)rows);
                for (int64_t q = 0; q < rows; ++q) pos_of[order[q]] = (int32_t)q;
                TRON_TRY(upload(&S.pos, pos_of.data(), pos_of.size(), st));
                TRON_HIP(hipStreamSynchronize(st));
            }
            TRON_TRY(upload(&S.wave_off, wave_off.data(), wave_off.size(), st));
            TRON_TRY(upload(&S.data, data.data(), data.size(), st));
            TRON_HIP(hipMalloc(reinterpret_cast<void **>(&S.sums), sizeof(double) * (size_t)rows));
            TRON_HIP(hipMemsetAsync(S.sums, 0, sizeof(double) * (size_t)rows, st));
            TRON_HIP(hipStreamSynchronize(st));
        } else if (A.head >= 0) {
            // the head partition is the last one: its columns go to col16, the ranges' stay in col
            const size_t h0 = (size_t)A.part_base[A.head];
            std::vector<uint16_t> c16(pcol.size() - h0, 0);
            // padding: slot 0 (value 0; in a unit plan the padding lies behind the last flagged entry of the partition, and
            // what follows the last flag of a chunk never reaches a sum)
            for (size_t k = h0; k < pcol.size(); ++k) c16[k - h0] = (uint16_t)(pcol[k] < 0 ? ~pcol[k] : 0);
            TRON_TRY(upload(&A.col16, c16.data(), c16.size(), st));
            TRON_HIP(hipStreamSynchronize(st));
            pcol.resize(h0);
        }
        TRON_TRY(upload(&A.col, pcol.data(), pcol.size(), st));
        if (!A.unit) TRON_TRY(upload(&A.val, pval.data(), pval.size(), st));
        else TRON_HIP(hipMalloc(reinterpret_cast<void **>(&A.xs), sizeof(double) * (size_t)(cols + 1)));
        // group_base[G].first[x] = first segment of partition x whose row is >= 64 G (see sum_parts)
        A.ngroups = (rows + kWave - 1) / kWave;
        A.nseg_total = nseg_total;
        std::vector<GroupBase> gbase((size_t)A.ngroups);
        std::memset(gbase.data(), 0, sizeof(GroupBase) * gbase.size());
        for (int x = 0; x < NP; ++x) {
            const int64_t s0 = A.part_seg0[x], s1 = (x + 1 < NP) ? A.part_seg0[x + 1] : nseg_total;
            int64_t m = s0;
            for (int64_t G = 0; G < A.ngroups; ++G) {
                while (m < s1 && seg_row[m] < G * kWave) ++m;
                gbase[(size_t)G].first[x] = (int32_t)m;
            }
        }
        TRON_TRY(upload(&A.group_base, gbase.data(), gbase.size(), st));
        TRON_TRY(upload(&A.chunk_tab, tab.data(), tab.size(), st));
        TRON_TRY(upload(&A.flags, flags.data(), flags.size(), st));
        TRON_TRY(upload(&A.row_mask, mask.data(), mask.size(), st));
        TRON_HIP(hipStreamSynchronize(st));
    }
    A.nfix = (int)fix_row.size();
    A.fix_max_cnt = 0;
    for (int32_t c : fix_cnt) A.fix_max_cnt = std::max(A.fix_max_cnt, (int)c);
    if (A.plain) TRON_TRY(upload(&A.row_lo, row_lo.data(), row_lo.size(), st));
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
    return fma(alpha, sum, aux ? aux[r] : 1.0);   // no addend vector: add 1 (the Hessian diagonal)
}

// One chunk: nonzeros [start, end) of a (sub)matrix whose row offsets are rp (relative to col/val),
// chunk-local tables row_lo[0..1] and carry slot *carry_out.
// With HOT, a negative stored column c means "entry ~c of the workgroup's LDS table" (the most frequent
// columns of the partition, copied from x once per workgroup).
// x[c] through a 32-bit byte offset (tron_dataset_create_csr accepts n, d < 2^29 only)
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

template <int EPI, typename RP, bool HOT = false, bool SQ = false>
__device__ __forceinline__ void chunk_body(double *prod, const double *table, int64_t start, int64_t end, bool first_chunk,
                                           const RP *__restrict__ rp, const int32_t *__restrict__ col,
                                           const double *__restrict__ val, const int32_t *__restrict__ row_lo,
                                           const double *__restrict__ x, double *__restrict__ yout,
                                           const double *__restrict__ aux, double alpha, double *__restrict__ carry_out)
{
    const int tid = threadIdx.x;
    // ---- phase 1: products into LDS (two passes of 1024 nonzeros, 4 per thread per pass)
    if (end - start == kChunk) {
        // thread t takes entries m*512 + 2t, m*512 + 2t + 1: every load instruction covers whole cache lines
        v2i c[4];
        v2d v[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int64_t k = start + m * (kChunk / 4) + tid * 2;
            c[m] = __builtin_nontemporal_load(reinterpret_cast<const v2i *>(col + k));
            v[m] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(val + k));
        }
        double xg[4][2];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            xg[m][0] = gather<HOT>(x, table, c[m].x);
            xg[m][1] = gather<HOT>(x, table, c[m].y);
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            double2 p;
            p.x = (SQ ? v[m].x * v[m].x : v[m].x) * xg[m][0];
            p.y = (SQ ? v[m].y * v[m].y : v[m].y) * xg[m][1];
            *reinterpret_cast<double2 *>(prod + m * (kChunk / 4) + tid * 2) = p;
        }
    } else {
        for (int k = tid; k < kChunk; k += kBlock) {
            const int64_t kk = start + k;
            prod[k] = (kk < end) ? (SQ ? val[kk] * val[kk] : val[kk]) * gather<HOT>(x, table, col[kk]) : 0.0;
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
    if (g == 1 && nrows > kBlock) {
        // Many short rows (the tail of a Zipf-distributed transposed copy: a thousand rows of one or two entries in a
        // chunk): one thread per row, and the row offsets of eight passes are fetched together -- a pass that waited
        // for its own two offsets first cost a memory round trip each, eight or more per chunk.
        constexpr int kBatch = 8;
        for (int base = 0; base < nrows; base += kBatch * kBlock) {
            int64_t rs[kBatch], re[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int ri = base + j * kBlock + tid;
                const int64_t r = (int64_t)lo + (ri < nrows ? ri : nrows - 1);
                rs[j] = (int64_t)rp[r];
                re[j] = (int64_t)rp[r + 1];
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int ri = base + j * kBlock + tid;
                if (ri < nrows) {
                    const int64_t r = (int64_t)lo + ri;
                    const int k0 = (int)(rs[j] - start);
                    const int k1 = (int)(((re[j] < end) ? re[j] : end) - start);
                    double s = 0.0;
                    for (int k = k0; k < k1; ++k) s += prod[k];
                    yout[r] = epilogue<EPI>(s, r, aux, alpha);
                }
            }
        }
        return;
    }
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
template <int EPI, bool SQ>
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
    chunk_body<EPI, int64_t, false, SQ>(prod, nullptr, start, end, b == 0, rowptr, col, val, row_lo + b, x, yout, aux, alpha, carry + b);
}

struct PartArgs {
    int64_t base[kMaxParts];
    int64_t nnz[kMaxParts];
    int64_t seg0[kMaxParts];
    int chunk0[kMaxParts];
    int nchunks[kMaxParts];
    int nhot[kMaxParts];
    int P;
    int slots;   // LDS table entries per workgroup (a multiple of 2; the tables are stored kHotSlots apart)
};

// Partitioned layout, persistent workgroups: workgroup (partition xp, q) walks chunks q, q + Q, ... of its
// partition (Q = gridDim / P).  Everything the next chunk needs -- the col/val stream, the chunk's table entry,
// its segment end offsets and the row ids this thread will write -- is fetched into registers while the current
// chunk is being reduced, so HBM latency is paid once per workgroup, not once per chunk.
// With HOT the partition's most frequent columns are first copied from x into an LDS table; entries of those
// columns are stored as ~slot and never touch the vector cache.
// Stream registers of one chunk: thread t holds entries m*512 + 2t, m*512 + 2t + 1 (m = 0..3), so that every load
// instruction of a wavefront covers whole consecutive cache lines (a wavefront that reads 16 of every 32 bytes is
// served in 64-byte requests, twice as many, and the number of requests a CU keeps in flight is what bounds it).
constexpr int kQuarter = kChunk / 4;

template <bool HEAD>
struct StreamRegs {
    v2i c[4];
    v2d v[4];
};
template <>
struct StreamRegs<true> {
    uint32_t c[4];   // two 16-bit LDS slots each
    v2d v[4];
};

// UNIT: the entries carry no values (see CsrPlan::unit); v stays unset and unused
template <bool HEAD, bool UNIT>
__device__ __forceinline__ StreamRegs<HEAD> load_stream(const void *__restrict__ col, const double *__restrict__ val, int64_t start)
{
    StreamRegs<HEAD> s;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int64_t k = start + m * kQuarter + threadIdx.x * 2;
        if constexpr (HEAD)
            s.c[m] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(static_cast<const uint16_t *>(col) + k));
        else
            s.c[m] = __builtin_nontemporal_load(reinterpret_cast<const v2i *>(static_cast<const int32_t *>(col) + k));
        if constexpr (!UNIT) s.v[m] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(val + k));
    }
    return s;
}

// the two gathered vector entries of quarter m
template <bool HOT, bool HEAD>
__device__ __forceinline__ void gather2(const StreamRegs<HEAD> &r, int m, const double *__restrict__ x, const double *table, double *out)
{
    if constexpr (HEAD) {
        out[0] = table[r.c[m] & 0xffffu];
        out[1] = table[r.c[m] >> 16];
    } else {
        out[0] = gather<HOT>(x, table, r.c[m].x);
        out[1] = gather<HOT>(x, table, r.c[m].y);
    }
}

// ------------------------------------------------------------------ segment sums of a chunk
// The entries of a chunk are in segment order (a segment = the entries of one row inside the chunk) and a flag bit
// marks the last entry of every segment.  Products are written to LDS in load order and read back so that thread
// t owns entries 8t .. 8t+7; the thread sums its own runs in registers, the open run at its end is carried to the
// following threads by a segmented scan over the wavefront (DPP) and across the four wavefronts through LDS.
// No loop depends on how long the segments are.
//
// LDS layout of the products: blocks of 8 entries padded to 10 doubles, so that the 128-bit reads of a wavefront
// (80-byte lane stride) fall into distinct banks; the padding of the first four blocks holds the wavefront totals.
constexpr int kProdDoubles = kChunk / 8 * 10;   // 2560 doubles = 20 KiB
constexpr int kOutOffset = 40;                  // segment sums are parked at prod[kOutOffset ...] (behind the totals)
constexpr int kSegPasses = kChunk / kBlock;     // a chunk holds at most kChunk segments: 8 passes of 256

__device__ __forceinline__ int prod_pos(int e) { return e + 2 * (e >> 3); }

// products of the chunk in `r` into LDS
template <bool HOT, bool HEAD, bool SQ, bool UNIT>
__device__ __forceinline__ void products_to_lds(const StreamRegs<HEAD> &r, const double *__restrict__ x, const double *table, double *prod)
{
    double xg[4][2];
#pragma unroll
    for (int m = 0; m < 4; ++m) gather2<HOT, HEAD>(r, m, x, table, xg[m]);
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        double2 p;
        if constexpr (UNIT) {
            p.x = xg[m][0];
            p.y = xg[m][1];
        } else {
            p.x = (SQ ? r.v[m].x * r.v[m].x : r.v[m].x) * xg[m][0];
            p.y = (SQ ? r.v[m].y * r.v[m].y : r.v[m].y) * xg[m][1];
        }
        *reinterpret_cast<double2 *>(prod + prod_pos(m * kQuarter + threadIdx.x * 2)) = p;   // an even entry: the pair stays together
    }
}

// Call after the barrier that follows the product writes.  f = the thread's 8 flag bits.
// p[e] in: the product of entry 8 * tid + e.  On return p[e] = sum of the thread's entries from the start of the run
// containing e up to e, cin = what the entries before the thread add to its first run, idx0 = number of flags in the
// threads before it.  Uses prod[8..39] for the wavefront totals; contains one barrier.
__device__ __forceinline__ void runs_from_regs(double *prod, const unsigned f, double (&p)[8], double &cin, int &idx0)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    double run = 0.0;
    const unsigned nf = ~f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        run += p[e];
        p[e] = run;
        const int keep = (int)(nf << (31 - e)) >> 31;   // all ones unless entry e ends a segment
        run = __hiloint2double(__double2hiint(run) & keep, __double2loint(run) & keep);
    }
    const int cnt = __popc(f);
    double t = run;
    int h = (f != 0u);
    wave_seg_scan(t, h);
    const int ci = wave_scan_add(cnt);
    const double ext = lane_before(t);
    const int exh = lane_before(h);
    if (lane == kWave - 1) {
        prod[10 * wv + 8] = t;
        *reinterpret_cast<int2 *>(prod + 10 * wv + 9) = make_int2(h, ci);
    }
    __syncthreads();
    double ct = 0.0;
    int cb = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock - 1; ++w) {
        if (w < wv) {
            const double wt = prod[10 * w + 8];
            const int2 hc = *reinterpret_cast<const int2 *>(prod + 10 * w + 9);
            ct = hc.x ? wt : ct + wt;
            cb += hc.y;
        }
    }
    cin = exh ? ext : ct + ext;
    idx0 = cb + ci - cnt;
}

// The same with the products taken from LDS (call after the barrier that follows the product writes).  After the barrier
// inside, the product area may be overwritten (the totals at prod[8..39] may not).
__device__ __forceinline__ void chunk_runs(double *prod, const unsigned f, double (&p)[8], double &cin, int &idx0)
{
    const double2 *src = reinterpret_cast<const double2 *>(prod + 10 * threadIdx.x);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const double2 d = src[q];
        p[2 * q] = d.x;
        p[2 * q + 1] = d.y;
    }
    runs_from_regs(prod, f, p, cin, idx0);
}

// flag byte of the calling thread: bit e = entry 8*tid + e is the last of its segment
__device__ __forceinline__ unsigned load_flags(const uint8_t *__restrict__ flags /* of this chunk */)
{
    return flags[threadIdx.x];
}

// Segment sums of the chunk whose products are in LDS: the sums of the owned segments go to out[0 .. nseg) in segment
// order (one coalesced store per 64 segments; the partial sums of a plan are stored segment by segment, not by row:
// see sum_parts), the piece of a row that started in an earlier chunk to *carry_slot.  Three barriers; the caller
// adds one before it reuses `prod`.
// FROM_REGS: p holds the products of the thread's own 8 entries (nothing is read from the product area)
template <bool FROM_REGS = false>
__device__ __forceinline__ void chunk_segments(double *prod, const unsigned flags, const int nseg, const bool continued,
                                               double *__restrict__ out, double *__restrict__ carry_slot, double *regs = nullptr)
{
    double p[8], cin;
    int idx0;
    if constexpr (FROM_REGS) {
#pragma unroll
        for (int e = 0; e < 8; ++e) p[e] = regs[e];
        runs_from_regs(prod, flags, p, cin, idx0);
    } else {
        chunk_runs(prod, flags, p, cin, idx0);
    }
    double *outv = prod + kOutOffset;
    int i = idx0 - (continued ? 1 : 0);
    bool first = true;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if ((flags >> e) & 1u) {
            const double v = first ? p[e] + cin : p[e];
            if (i < 0) *carry_slot = v;
            else outv[i] = v;
            first = false;
            ++i;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSegPasses; ++j) {
        const int sidx = (int)threadIdx.x + kBlock * j;
        if (j * kBlock < nseg && sidx < nseg) out[sidx] = outv[sidx];
    }
}

// hot_x[k] = x[hot_ids[k]]: the LDS tables of all partitions, so that a workgroup fills its table with 128 line
// requests instead of 4096 gathers
__global__ __launch_bounds__(kBlock) void k_gather_hot(int n, const int32_t *__restrict__ hot_ids, const double *__restrict__ x,
                                                       double *__restrict__ hot_x)
{
    const int k = blockIdx.x * kBlock + threadIdx.x;
    if (k < n) hot_x[k] = x[hot_ids[k]];
}

// A table entry that every thread of the workgroup needs, fetched with a vector load.  A scalar load would be counted
// by the same counter as the LDS operations, so the wait for LDS before the next barrier would also wait for it --
// a full memory latency in every iteration of the persistent loops, which prefetch these entries two chunks ahead.
__device__ __forceinline__ int4 load_uniform(const int4 *__restrict__ p)
{
    int zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));   // a lane-dependent zero as far as the compiler can tell
    return p[zero];
}

struct PartPtrs {   // device arrays of one partitioned plan (or of its head partition, pre-offset where noted)
    const void *col;           // int32 columns of the ranges, or the head's 16-bit slots
    const double *val;
    const int4 *chunk_tab;
    const uint8_t *flags;
    const double *hot_x;       // x at the LDS-resident columns, kHotSlots per partition (null without LDS tables)
    double *partial;           // partial sums, one per segment of the plan
    double *carry;
};

// Partitioned layout, persistent workgroups: workgroup (partition xp, q) walks chunks q, q + Q, ... of its
// partition.  Everything the next chunk needs -- the col/val stream, the chunk's table entry, its flags and the row
// ids this thread will write -- is fetched into registers while the current chunk is being reduced, so HBM latency
// is paid once per workgroup, not once per chunk.
// SQ: the values are squared (sum_i x_ij^2 a_i, for the diagonal of the Hessian)
template <bool HOT, bool HEAD, bool SQ, bool UNIT>
__device__ __forceinline__ void part_body(double *prod, double *table, const PartArgs &pa, const int xp, const int q, const int Q,
                                          const int64_t rows, const PartPtrs &pp, const double *__restrict__ x)
{
    const int tid = threadIdx.x;
    const int nchunks = pa.nchunks[xp];
    if (q >= nchunks) return;
    if (HOT) {
        // the vector entries of this partition's LDS-resident columns, gathered once per call by k_gather_hot
        const double2 *__restrict__ src = reinterpret_cast<const double2 *>(pp.hot_x + (size_t)xp * kHotSlots);
        for (int k = tid; k < pa.slots / 2; k += kBlock) reinterpret_cast<double2 *>(table)[k] = src[k];
        __syncthreads();
    }
    // col/val are padded to whole chunks (zeros)
    const void *col = HEAD ? static_cast<const void *>(static_cast<const uint16_t *>(pp.col) + pa.base[xp])
                           : static_cast<const void *>(static_cast<const int32_t *>(pp.col) + pa.base[xp]);
    const double *val = UNIT ? nullptr : pp.val + pa.base[xp];
    const int4 *__restrict__ tabs = pp.chunk_tab + pa.chunk0[xp];
    const uint8_t *__restrict__ flags = pp.flags + (int64_t)pa.chunk0[xp] * kBlock;
    double *partial = pp.partial + pa.seg0[xp];
    double *carry = pp.carry + pa.chunk0[xp];

    int c = q;
    int4 tab = load_uniform(tabs + c);
    int4 tab_n = load_uniform(tabs + ((c + Q < nchunks) ? c + Q : c));
    StreamRegs<HEAD> cur = load_stream<HEAD, UNIT>(col, val, (int64_t)c * kChunk);
    unsigned fl = load_flags(flags + (int64_t)c * kBlock);

    for (; c < nchunks; c += Q) {
        products_to_lds<HOT, HEAD, SQ, UNIT>(cur, x, table, prod);
        // Only now fetch the next chunk (clamped index: always the same loads): nothing below waits for these
        // registers, so they stay in flight during the segment sums and are waited for at the top of the next
        // iteration.
        __builtin_amdgcn_sched_barrier(0);
        const int cn = (c + Q < nchunks) ? c + Q : c;
        const int cnn = (cn + Q < nchunks) ? cn + Q : cn;
        const StreamRegs<HEAD> nxt = load_stream<HEAD, UNIT>(col, val, (int64_t)cn * kChunk);
        const unsigned fl_n = load_flags(flags + (int64_t)cn * kBlock);
        const int4 tab_nn = load_uniform(tabs + cnn);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        chunk_segments(prod, fl, tab.y, tab.z > 0, partial + tab.x, carry + c);
        __syncthreads();  // prod is reused by the next chunk
        cur = nxt;
        fl = fl_n;
        tab = tab_n;
        tab_n = tab_nn;
    }
}

// The head partition of a unit plan: an entry is a 16-bit slot of the LDS table and nothing else, so thread t loads the
// slots of entries 8t .. 8t+7 with one 16-byte load and gathers their table values straight into the registers the
// segment sums start from -- no trip of the products through LDS.
__device__ __forceinline__ void head_unit_body(double *prod, double *table, const PartArgs &pa, const int q, const int Q,
                                               const PartPtrs &pp)
{
    const int tid = threadIdx.x;
    const int nchunks = pa.nchunks[0];
    if (q >= nchunks) return;
    {
        const double2 *__restrict__ src = reinterpret_cast<const double2 *>(pp.hot_x);
        for (int k = tid; k < pa.slots / 2; k += kBlock) reinterpret_cast<double2 *>(table)[k] = src[k];
        __syncthreads();
    }
    const uint16_t *col = static_cast<const uint16_t *>(pp.col) + pa.base[0];
    const int4 *__restrict__ tabs = pp.chunk_tab + pa.chunk0[0];
    const uint8_t *__restrict__ flags = pp.flags + (int64_t)pa.chunk0[0] * kBlock;
    double *partial = pp.partial + pa.seg0[0];
    double *carry = pp.carry + pa.chunk0[0];
    auto load8 = [&](int c) { return __builtin_nontemporal_load(reinterpret_cast<const v4i *>(col + (int64_t)c * kChunk + 8 * tid)); };

    int c = q;
    int4 tab = load_uniform(tabs + c);
    int4 tab_n = load_uniform(tabs + ((c + Q < nchunks) ? c + Q : c));
    v4i cur = load8(c);
    unsigned fl = load_flags(flags + (int64_t)c * kBlock);
    for (; c < nchunks; c += Q) {
        double p[8];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const unsigned two = (unsigned)cur[m];
            p[2 * m] = table[two & 0xffffu];
            p[2 * m + 1] = table[two >> 16];
        }
        __builtin_amdgcn_sched_barrier(0);
        const int cn = (c + Q < nchunks) ? c + Q : c;
        const int cnn = (cn + Q < nchunks) ? cn + Q : cn;
        const v4i nxt = load8(cn);
        const unsigned fl_n = load_flags(flags + (int64_t)cn * kBlock);
        const int4 tab_nn = load_uniform(tabs + cnn);
        __builtin_amdgcn_sched_barrier(0);
        chunk_segments<true>(prod, fl, tab.y, tab.z > 0, partial + tab.x, carry + c, p);
        __syncthreads();  // the totals and the parked sums are reused by the next chunk
        cur = nxt;
        fl = fl_n;
        tab = tab_n;
        tab_n = tab_nn;
    }
}

__global__ __launch_bounds__(kBlock) void k_csr_head_unit(PartArgs pa, PartPtrs pp)
{
    __shared__ __align__(16) double prod[kOutOffset + kChunk];
    extern __shared__ __align__(16) double table[];   // pa.slots doubles
    head_unit_body(prod, table, pa, blockIdx.x, gridDim.x, pp);
}

// Head partition of a unit plan stored as sorted slices (see SellHead).  A wavefront reads its own contiguous stream of
// groups (64 lanes x 16 bytes = eight 16-bit slots per lane); lane l sums row l of the current slice and writes the
// sum when the slice ends.  The loads of the next kSellAhead groups are always in flight, also across the ends of
// slices (they are short: the pipeline must not drain there); a slice's row ids and length come in its header group.  No barrier after the table is filled, no segment bookkeeping.  The sum of a row is
// (entries 0, 2, 4, ...) + (entries 1, 3, 5, ...), each in storage order.
__device__ __forceinline__ int64_t uniform64(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

__global__ __launch_bounds__(kSellBlock) void k_head_sell(int nwaves, const int64_t *__restrict__ wave_off, const uint16_t *__restrict__ data,
                                                         const double *__restrict__ hot_x, double *__restrict__ sums)
{
    __shared__ __align__(16) double table[kSellSlots + 2];
    {
        const double2 *__restrict__ src = reinterpret_cast<const double2 *>(hot_x);
        for (int k = threadIdx.x; k < kSellSlots / 2; k += kSellBlock) reinterpret_cast<double2 *>(table)[k] = src[k];
        if (threadIdx.x == 0) table[kSellSlots] = 0.0;   // the padding slot
        __syncthreads();
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int w = blockIdx.x * (kSellBlock / kWave) + threadIdx.x / kWave;
    if (w >= nwaves) return;
    // everything that steers the loop is kept in scalar registers: a branch on a vector condition would make the compiler
    // wait for every load in flight where the paths join
    const int64_t g0 = uniform64(wave_off[w]);
    const int64_t total = uniform64(wave_off[w + 1]) - g0;   // a multiple of kSellAhead
    if (total <= 0) return;
    const v4i *__restrict__ p = reinterpret_cast<const v4i *>(data) + g0 * kWave + lane;
    v4i buf[kSellAhead];
#pragma unroll
    for (int a = 0; a < kSellAhead; ++a) buf[a] = __builtin_nontemporal_load(p + (int64_t)a * kWave);
    int left = 0;    // groups left in the current slice (0: the next group is a header)
    int row = -1;
    double e0 = 0.0, e1 = 0.0;
    // buffer a holds group g + a: the body is unrolled over the buffers, so no buffer is ever copied (a copy would have to
    // wait for the load that fills its source); everything a slice needs arrives through this one stream, in order
    for (int64_t g = 0; g < total; g += kSellAhead) {
#pragma unroll
        for (int a = 0; a < kSellAhead; ++a) {
            const v4i cur = buf[a];
            const int64_t nx = g + a + kSellAhead;
            buf[a] = __builtin_nontemporal_load(p + ((nx < total) ? nx : total - 1) * kWave);
            if (left == 0) {   // a header (a slice without groups is padding)
                row = cur[0];
                left = __builtin_amdgcn_readfirstlane(cur[1]);
            } else {
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const unsigned two = (unsigned)cur[m];
                    e0 += table[two & 0xffffu];
                    e1 += table[two >> 16];
                }
                if (--left == 0) {   // the slice ends
                    if (row >= 0) sums[row] = e0 + e1;
                    e0 = 0.0;
                    e1 = 0.0;
                }
            }
        }
    }
}

template <bool HOT, bool HEAD, bool SQ, bool UNIT>
__global__ __launch_bounds__(kBlock) void k_csr_spmv_part(PartArgs pa, int64_t rows, PartPtrs pp, const double *__restrict__ x)
{
    __shared__ __align__(16) double prod[kProdDoubles];
    extern __shared__ __align__(16) double table[];   // pa.slots doubles (none without HOT)
    part_body<HOT, HEAD, SQ, UNIT>(prod, table, pa, blockIdx.x % pa.P, blockIdx.x / pa.P, gridDim.x / pa.P, rows, pp, x);
}

// ------------------------------------------------------------------ hot-row tiles (see HotTiles)
constexpr int kMaxTileBlocks = 256;   // workgroups per slice

int hot_tiles_build(CsrPlan &A, const int64_t *t_rowptr, const int32_t *t_col, const double *t_val,
                    const std::vector<int32_t> &slot_code, int nhot, hipStream_t st)
{
    HotTiles &H = A.hot;
    H.nhot = nhot;
    struct Entry { uint16_t slot, iloc; double val; };
    std::vector<Entry> cur[kTileSlices];
    int64_t base[kTileSlices] = {0};
    const bool unit = A.unit;
    std::vector<double> tval[kTileSlices];
    std::vector<uint16_t> tiloc[kTileSlices];
    std::vector<uint8_t> tflags[kTileSlices];
    std::vector<uint16_t> sslot[kTileSlices];
    std::vector<int4> hdrs[kTileSlices];

    std::vector<Entry> sorted[kTileSlices];
    std::vector<int32_t> slot_at[kTileSlices];
    auto close_tile = [&](int s) {
        std::vector<Entry> &e = cur[s];
        if (e.empty()) return;
        // by slot; the entries of a slot keep their column order (counting sort)
        {
            std::vector<int32_t> &at = slot_at[s];
            at.assign((size_t)kTileSlots + 1, 0);
            for (const Entry &x : e) at[(size_t)x.slot + 1]++;
            for (int q = 0; q < kTileSlots; ++q) at[(size_t)q + 1] += at[(size_t)q];
            sorted[s].resize(e.size());
            for (const Entry &x : e) sorted[s][(size_t)at[x.slot]++] = x;
            e.swap(sorted[s]);
        }
        int4 h = make_int4((int)base[s], 0, 0, (int)sslot[s].size());
        const size_t off = tiloc[s].size();
        if (!unit) tval[s].resize(off + kChunk, 0.0);
        tiloc[s].resize(off + kChunk, 0);
        tflags[s].resize((off + kChunk) / 8, 0);
        for (size_t k = 0; k < e.size(); ++k) {
            if (!unit) tval[s][off + k] = e[k].val;
            tiloc[s][off + k] = e[k].iloc;
            if (k + 1 == e.size() || e[k + 1].slot != e[k].slot) {
                tflags[s][(off + k) / 8] |= (uint8_t)(1u << (k % 8));
                sslot[s].push_back(e[k].slot);
                h.y += 1;
            }
        }
        while (sslot[s].size() % 8) sslot[s].push_back(0);
        for (const Entry &x : e) h.z = std::max<int>(h.z, x.iloc + 1);   // columns the tile spans
        hdrs[s].push_back(h);
        e.clear();
    };

    // the kernels gather from a copy of the tile's columns in LDS: a tile spans at most kTileWindow of them
    const int64_t span = kTileWindow;
    // The slices are independent of each other (own features, own tiles): one host thread per slice walks the matrix
    // and keeps the entries of its slice.
    int64_t slice_nnz[kTileSlices] = {0};
    bool slice_failed[kTileSlices] = {false};
    // the code of every entry's feature (slice and slot; kNoCode: not in the tiles), looked up once, so that the slice
    // threads stream through 16-bit codes instead of each looking every feature up again
    static_assert(kTileSlices * kTileSlots < 0xffff, "entry codes are 16 bits");
    constexpr uint16_t kNoCode = 0xffff;
    std::vector<uint16_t> ecode;
    try {
        ecode.resize((size_t)t_rowptr[A.cols]);
    } catch (const std::exception &) { set_error("out of host memory building the hot-row tiles"); return TRON_ENOMEM; }
    parallel_ranges(A.cols, [&](int64_t i0, int64_t i1) {
        for (int64_t k = t_rowptr[i0]; k < t_rowptr[i1]; ++k) {
            const int32_t code = slot_code[t_col[k]];
            ecode[k] = code >= 0 ? (uint16_t)code : kNoCode;
        }
    });
    auto build_slice = [&](int s) {
        try {
            int64_t nnz = 0;
            for (int64_t i = 0; i < A.cols; ++i) {
                int cnt = 0;
                for (int64_t k = t_rowptr[i]; k < t_rowptr[i + 1]; ++k)
                    if (ecode[k] != kNoCode && ecode[k] / kTileSlots == s) ++cnt;
                if (!cnt) continue;
                if ((int)cur[s].size() + cnt > kChunk || (!cur[s].empty() && i - base[s] >= span)) close_tile(s);
                if (cur[s].empty()) base[s] = i;
                for (int64_t k = t_rowptr[i]; k < t_rowptr[i + 1]; ++k) {
                    const int code = ecode[k];
                    if (code == kNoCode || code / kTileSlots != s) continue;
                    ++nnz;
                    cur[s].push_back({(uint16_t)(code % kTileSlots), (uint16_t)(i - base[s]), unit ? 1.0 : t_val[k]});
                }
            }
            close_tile(s);
            slice_nnz[s] = nnz;
        } catch (const std::exception &) {
            slice_failed[s] = true;
        }
    };
    {
        std::vector<std::thread> workers;
        try {
            for (int s = 1; s < kTileSlices; ++s) workers.emplace_back(build_slice, s);
        } catch (const std::exception &) {
            // fewer threads than slices could be started: the rest run here
        }
        const int started = (int)workers.size();
        build_slice(0);
        for (int s = 1 + started; s < kTileSlices; ++s) build_slice(s);
        for (std::thread &t : workers) t.join();
    }
    for (int s = 0; s < kTileSlices; ++s) {
        if (slice_failed[s]) { set_error("out of host memory building the hot-row tiles"); return TRON_ENOMEM; }
        H.nnz += slice_nnz[s];
    }

    // concatenate the slices; segment offsets become global
    int64_t ntiles = 0, nseg = 0;
    for (int s = 0; s < kTileSlices; ++s) {
        H.tile0[s] = ntiles;
        H.ntiles[s] = (int64_t)hdrs[s].size();
        for (int4 &h : hdrs[s]) h.w += (int)nseg;
        ntiles += H.ntiles[s];
        nseg += (int64_t)sslot[s].size();
    }
    H.ntiles_total = ntiles;
    H.nseg_padded = nseg;
    for (int s = 0; s < kTileSlices; ++s)
        for (const int4 &h : hdrs[s]) H.span_total += h.z;
    if (ntiles == 0) return TRON_OK;
    if (nseg > 0x7ffffff0 || ntiles > 0x7ffffff0 / kChunk * 1024) { set_error("hot tiles too large"); return TRON_EINVAL; }
    if (!unit) TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.val), sizeof(double) * ntiles * kChunk));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.iloc), sizeof(uint16_t) * ntiles * kChunk));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.flags), ntiles * kBlock));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.hdr), sizeof(int4) * ntiles));
    TRON_HIP(hipMalloc(reinterpret_cast<void **>(&H.seg_slot), sizeof(uint16_t) * std::max<int64_t>(nseg, 8)));
    int64_t segpos = 0;
    for (int s = 0; s < kTileSlices; ++s) {
        const int64_t t0 = H.tile0[s];
        if (H.ntiles[s] == 0) continue;
        if (!unit) TRON_HIP(hipMemcpyAsync(H.val + t0 * kChunk, tval[s].data(), sizeof(double) * tval[s].size(), hipMemcpyHostToDevice, st));
        TRON_HIP(hipMemcpyAsync(H.iloc + t0 * kChunk, tiloc[s].data(), sizeof(uint16_t) * tiloc[s].size(), hipMemcpyHostToDevice, st));
        TRON_HIP(hipMemcpyAsync(H.flags + t0 * kBlock, tflags[s].data(), tflags[s].size(), hipMemcpyHostToDevice, st));
        TRON_HIP(hipMemcpyAsync(H.hdr + t0, hdrs[s].data(), sizeof(int4) * hdrs[s].size(), hipMemcpyHostToDevice, st));
        TRON_HIP(hipMemcpyAsync(H.seg_slot + segpos, sslot[s].data(), sizeof(uint16_t) * sslot[s].size(), hipMemcpyHostToDevice, st));
        segpos += (int64_t)sslot[s].size();
    }
    TRON_TRY(upload(&H.slot_of_row, slot_code.data(), slot_code.size(), st));
    int64_t maxt = 0;
    for (int s = 0; s < kTileSlices; ++s) maxt = std::max(maxt, H.ntiles[s]);
    // 0 = automatic: 3 workgroups per CU with values (the kernel is then bound by HBM), 5 without (as many as fit in LDS:
    // the kernel is bound by instruction issue and LDS latency)
    const int64_t want_blocks = g_tuning.csr_tile_blocks_per_slice > 0 ? g_tuning.csr_tile_blocks_per_slice : (A.unit ? 160 : 96);
    H.blocks_per_slice = (int)std::max<int64_t>(1, std::min<int64_t>(maxt, std::min<int64_t>(want_blocks, kMaxTileBlocks)));
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
    uint4 slots;        // slots of the segments 8*tid .. 8*tid+7 (16 bits each)
    unsigned flags;     // bit e: entry 8*tid + e is the last of its segment
    double w[2];        // the two columns of the tile that the thread copies into LDS
    int4 hdr;
};

struct TilePtrs {
    const double *val;
    const uint16_t *iloc;
    const uint8_t *flags;
    const int4 *hdr;
    const uint16_t *seg_slot;
    double *wg_acc;
};

// data of tile T whose header h is already in registers; columns clamped to the tile's last one
__device__ __forceinline__ TileRegs load_tile(const TilePtrs &tp, const double *__restrict__ x, int4 h, int64_t T)
{
    TileRegs r;
    r.hdr = h;
    {
        const int tid = threadIdx.x, lastc = h.z - 1;
        const double *xt = x + h.x;
        r.w[0] = xt[tid < lastc ? tid : lastc];
        r.w[1] = xt[tid + kBlock < lastc ? tid + kBlock : lastc];
    }
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int64_t k = T * kChunk + m * kQuarter + threadIdx.x * 2;
        r.v[m] = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(tp.val + k));
        r.il[m] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(tp.iloc + k));
    }
    r.flags = tp.flags[T * kBlock + threadIdx.x];
    // slot blocks are padded to a multiple of 8; threads beyond the tile's segments re-read its first block
    const int nseg = h.y;
    const int64_t d0 = (int64_t)h.w + ((8 * (int)threadIdx.x < nseg) ? 8 * (int)threadIdx.x : 0);
    r.slots = *reinterpret_cast<const uint4 *>(tp.seg_slot + d0);
    return r;
}

// Persistent workgroup (slice s, q): tiles q, q + B, ... of the slice; LDS accumulators for the slice's hot rows.
// Software pipeline: while tile t is reduced, the data of tiles t + B and t + 2B and the header of tile t + 3B are
// in flight (all indices clamped to the last tile, so every iteration issues the same loads).
// Slots inside a tile are distinct, so the accumulator updates of different segments never collide.
template <bool SQ>
__device__ __forceinline__ void tiles_body(double *prod, uint16_t *slots, double *acc, double (*window)[kTileWindow], const TileArgs &ta,
                                           const int s, const int q, const int B, const TilePtrs &tp, const double *__restrict__ x)
{
    const int tid = threadIdx.x;
    for (int k = tid; k < kTileSlots; k += kBlock) acc[k] = 0.0;
    const int64_t nt = ta.ntiles[s];
    if (q < nt) {
        const int64_t T0 = ta.tile0[s];
        const int64_t last = nt - 1;
        auto clampt = [&](int64_t t) { return T0 + (t < last ? t : last); };
        TileRegs cur = load_tile(tp, x, load_uniform(tp.hdr + clampt(q)), clampt(q));
        TileRegs nxt = load_tile(tp, x, load_uniform(tp.hdr + clampt(q + B)), clampt(q + B));
        int4 hdr2 = load_uniform(tp.hdr + clampt(q + 2 * (int64_t)B));
        window[0][tid] = cur.w[0];
        window[0][tid + kBlock] = cur.w[1];
        __syncthreads();
        int buf = 0;
        for (int64_t t = q; t < nt; t += B) {
            const int nseg = cur.hdr.y;
            // gathers from the copy of the tile's columns (at most kTileWindow of them) in LDS: see k_hot_tiles_unit
            const double *xt = window[buf];
            double xg[4][2];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                xg[m][0] = xt[cur.il[m] & 0xffffu];
                xg[m][1] = xt[cur.il[m] >> 16];
            }
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                double2 p;
                p.x = (SQ ? cur.v[m].x * cur.v[m].x : cur.v[m].x) * xg[m][0];
                p.y = (SQ ? cur.v[m].y * cur.v[m].y : cur.v[m].y) * xg[m][1];
                *reinterpret_cast<double2 *>(prod + prod_pos(m * kQuarter + tid * 2)) = p;
            }
            __builtin_amdgcn_sched_barrier(0);
            const TileRegs nn = load_tile(tp, x, hdr2, clampt(t + 2 * (int64_t)B));
            const int4 hdr3 = load_uniform(tp.hdr + clampt(t + 3 * (int64_t)B));
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            // every thread is past the accumulator updates of the tile before: its slots may be replaced; and past the
            // gathers of the tile before that one, which were the last to read the other window buffer
            if (8 * tid < nseg) *reinterpret_cast<uint4 *>(slots + 8 * tid) = cur.slots;
            window[buf ^ 1][tid] = nxt.w[0];
            window[buf ^ 1][tid + kBlock] = nxt.w[1];
            buf ^= 1;
            double p[8], cin;
            int idx0;
            chunk_runs(prod, cur.flags, p, cin, idx0);   // barrier inside: the slots and the next tile's columns are visible after it
            int i = idx0;
            bool first = true;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if ((cur.flags >> e) & 1u) {
                    acc[slots[i]] += first ? p[e] + cin : p[e];
                    first = false;
                    ++i;
                }
            }
            // no barrier here: the next tile's products do not touch acc or slots, and its wavefront totals are
            // written after its first barrier
            cur = nxt;
            nxt = nn;
            hdr2 = hdr3;
        }
    }
    __syncthreads();
    double *out = tp.wg_acc + ((int64_t)s * B + q) * kTileSlots;
    for (int k = tid; k < kTileSlots; k += kBlock) out[k] = acc[k];
}

// The tiles of a unit plan: an entry is a 16-bit column offset and nothing else; thread t loads the offsets of entries
// 8t .. 8t+7 with one 16-byte load.  A tile spans at most kTileWindow columns: the workgroup copies them from x into
// LDS with two coalesced loads per thread and gathers from the copy -- the gathers of a tile go to a few hundred
// consecutive doubles, and the vector memory pipeline, which handles about one lane of such a gather per clock, was
// what bound this kernel when they went to x itself.
struct TileRegsU {
    v4i il;             // eight 16-bit local column offsets
    uint4 slots;
    unsigned flags;
    double w[2];        // the two columns of the tile that the thread copies into LDS
    int4 hdr;
};

// *a += v with the LDS add instruction: one operation instead of a read, an add and a write, and nothing to wait for.
// Used where no two lanes address the same word between two barriers and a lane's own additions to one word are issued
// in program order (LDS operations of a wavefront complete in order), so the sum is built in a fixed order.
__device__ __forceinline__ void lds_add(double *a, double v)
{
    (void)__hip_atomic_fetch_add(a, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// the data of tile T, whose header is h; columns clamped to the tile's last one
__device__ __forceinline__ void load_tile_unit(TileRegsU &r, const TilePtrs &tp, const double *__restrict__ x, int4 h, int64_t T)
{
    const int tid = threadIdx.x;
    r.hdr = h;
    r.il = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(tp.iloc + T * kChunk + 8 * tid));
    r.flags = tp.flags[T * kBlock + tid];
    const int nseg = h.y;
    const int64_t d0 = (int64_t)h.w + ((8 * tid < nseg) ? 8 * tid : 0);
    r.slots = *reinterpret_cast<const uint4 *>(tp.seg_slot + d0);
    const int lastc = h.z - 1;
    const double *xt = x + h.x;
    r.w[0] = xt[tid < lastc ? tid : lastc];
    r.w[1] = xt[tid + kBlock < lastc ? tid + kBlock : lastc];
}

__device__ __forceinline__ void store_window(double *window, const TileRegsU &r)
{
    window[threadIdx.x] = r.w[0];
    window[threadIdx.x + kBlock] = r.w[1];
}

// One tile: cur is reduced (its columns are in window[BUF]) while the data of the next tile of the workgroup, whose
// header is ahead, are loaded into nxt; they are not waited for before the end of the step, where the columns go to
// the other window buffer.  ahead becomes the header of the tile after that.
template <int BUF>
__device__ __forceinline__ void tile_step_unit(double *prod, uint16_t *slots, double *acc, double (*window)[kTileWindow], TileRegsU &cur,
                                               TileRegsU &nxt, int4 &ahead, const TilePtrs &tp, const double *__restrict__ x,
                                               const int64_t Tn, const int64_t Tnn)
{
    const int tid = threadIdx.x;
    const int nseg = cur.hdr.y;
    __builtin_amdgcn_sched_barrier(0);
    load_tile_unit(nxt, tp, x, ahead, Tn);
    ahead = load_uniform(tp.hdr + Tnn);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    // every thread is past the accumulator updates and the totals of the tile before, and this tile's columns are
    // in window[BUF]
    double p[8], cin;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const unsigned two = (unsigned)cur.il[m];
        p[2 * m] = window[BUF][two & 0xffffu];
        p[2 * m + 1] = window[BUF][two >> 16];
    }
    if (8 * tid < nseg) *reinterpret_cast<uint4 *>(slots + 8 * tid) = cur.slots;
    int idx0;
    runs_from_regs(prod, cur.flags, p, cin, idx0);   // barrier inside: the slots are visible after it
    // What the threads before add to the thread's first segment goes in on its own, before the segment's own sum.
    int sl[8];
    int i = idx0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        sl[e] = slots[i];   // an entry that ends no segment reads a slot it does not use (then i < 2048: there are fewer segments than entries)
        i += (cur.flags >> e) & 1u;
    }
    if (cur.flags) lds_add(acc + sl[0], cin);   // sl[0] is the slot of the thread's first segment
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if ((cur.flags >> e) & 1u) lds_add(acc + sl[e], p[e]);
    // the other buffer was last read before the barrier inside runs_from_regs of the step before
    store_window(window[BUF ^ 1], nxt);
}

// Persistent workgroup (slice s, q): tiles q, q + B, ... of the slice, two steps per iteration so that the two sets of
// tile registers and the two window buffers swap roles without copies (indices clamped to the last tile, so every
// step issues the same loads).
__device__ __forceinline__ void tiles_unit_body(double *prod, uint16_t *slots, double *acc, double (*window)[kTileWindow],
                                                const TileArgs &ta, const int s, const int q, const int B, const TilePtrs &tp,
                                                const double *__restrict__ x)
{
    const int tid = threadIdx.x;
    for (int k = tid; k < kTileSlots; k += kBlock) acc[k] = 0.0;
    const int64_t nt = ta.ntiles[s];
    if (q < nt) {
        const int64_t T0 = ta.tile0[s];
        const int64_t last = nt - 1;
        auto clampt = [&](int64_t t) { return T0 + (t < last ? t : last); };
        TileRegsU r0, r1;
        load_tile_unit(r0, tp, x, load_uniform(tp.hdr + clampt(q)), clampt(q));
        int4 ahead = load_uniform(tp.hdr + clampt(q + B));
        store_window(window[0], r0);
        for (int64_t t = q; t < nt; t += 2 * (int64_t)B) {
            tile_step_unit<0>(prod, slots, acc, window, r0, r1, ahead, tp, x, clampt(t + B), clampt(t + 2 * (int64_t)B));
            if (t + B >= nt) break;
            tile_step_unit<1>(prod, slots, acc, window, r1, r0, ahead, tp, x, clampt(t + 2 * (int64_t)B), clampt(t + 3 * (int64_t)B));
        }
    }
    __syncthreads();
    double *out = tp.wg_acc + ((int64_t)s * B + q) * kTileSlots;
    for (int k = tid; k < kTileSlots; k += kBlock) out[k] = acc[k];
}

__global__ __launch_bounds__(kBlock) void k_hot_tiles_unit(TileArgs ta, int B, TilePtrs tp, const double *__restrict__ x)
{
    __shared__ __align__(16) double prod[kOutOffset];   // the wavefront totals only
    __shared__ __align__(16) uint16_t slots[kChunk];
    __shared__ double acc[kTileSlots];
    __shared__ double window[2][kTileWindow];
    static_assert(kTileWindow == 2 * kBlock, "two columns per thread");
    tiles_unit_body(prod, slots, acc, window, ta, blockIdx.x % kTileSlices, blockIdx.x / kTileSlices, B, tp, x);
}

template <bool SQ>
__global__ __launch_bounds__(kBlock) void k_hot_tiles(TileArgs ta, int B, TilePtrs tp, const double *__restrict__ x)
{
    __shared__ __align__(16) double prod[kProdDoubles];
    __shared__ __align__(16) uint16_t slots[kChunk];
    __shared__ double acc[kTileSlots];
    __shared__ double window[2][kTileWindow];
    tiles_body<SQ>(prod, slots, acc, window, ta, blockIdx.x % kTileSlices, blockIdx.x / kTileSlices, B, tp, x);
}

// sums[s*K + k] = sum over the B workgroups of slice s: sixteen partial sums (workgroup order inside each), added in
// order.  A workgroup covers 64 consecutive slots, one wavefront per part, so every read is one 512-byte row and a CU
// has sixteen rows in flight (with four the kernel waited for HBM most of the time).
constexpr int kReduceWaves = 16;
__global__ __launch_bounds__(kReduceWaves * kWave) void k_hot_reduce(int B, const double *__restrict__ wg_acc, double *__restrict__ sums)
{
    __shared__ double part[kReduceWaves][kWave];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int idx = blockIdx.x * kWave + lane;   // s*K + k
    const int s = idx / kTileSlots, k = idx % kTileSlots;
    const int per = (B + kReduceWaves - 1) / kReduceWaves;
    const int q0 = wv * per, q1 = (q0 + per < B) ? q0 + per : B;
    const double *p = wg_acc + (int64_t)s * B * kTileSlots + k;
    double a = 0.0;
    for (int q = q0; q < q1; ++q) a += p[(int64_t)q * kTileSlots];
    part[wv][lane] = a;
    __syncthreads();
    if (wv == 0) {
        double t = part[0][lane];
#pragma unroll
        for (int m = 1; m < kReduceWaves; ++m) t += part[m][lane];
        sums[idx] = t;
    }
}

static TileArgs tile_args(const HotTiles &H)
{
    TileArgs ta;
    for (int s = 0; s < kTileSlices; ++s) { ta.tile0[s] = H.tile0[s]; ta.ntiles[s] = H.ntiles[s]; }
    return ta;
}

static TilePtrs tile_ptrs(const HotTiles &H) { return TilePtrs{H.val, H.iloc, H.flags, H.hdr, H.seg_slot, H.wg_acc}; }

// tiles + the reduction of the workgroup accumulators (B = workgroups per slice)
static int launch_hot_tiles(tron_dataset *ds, const CsrPlan &A, const double *x, bool square)
{
    const HotTiles &H = A.hot;
    hipStream_t st = ds->stream;
    {
        ProfScope ps(ds, SLOT_SPMV_TILES, st);
        if (A.unit)   // squares, if any, are in the scaled vector
            hipLaunchKernelGGL(k_hot_tiles_unit, dim3(kTileSlices * H.blocks_per_slice), dim3(kBlock), 0, st, tile_args(H),
                               H.blocks_per_slice, tile_ptrs(H), x);
        else if (square)
            hipLaunchKernelGGL((k_hot_tiles<true>), dim3(kTileSlices * H.blocks_per_slice), dim3(kBlock), 0, st, tile_args(H),
                               H.blocks_per_slice, tile_ptrs(H), x);
        else
            hipLaunchKernelGGL((k_hot_tiles<false>), dim3(kTileSlices * H.blocks_per_slice), dim3(kBlock), 0, st, tile_args(H),
                               H.blocks_per_slice, tile_ptrs(H), x);
        TRON_HIP(hipGetLastError());
    }
    {
        ProfScope ps(ds, SLOT_SPMV_TILE_REDUCE, st);
        hipLaunchKernelGGL(k_hot_reduce, dim3(kTileSlices * kTileSlots / kWave), dim3(kReduceWaves * kWave), 0, st, H.blocks_per_slice,
                           H.wg_acc, H.sums);
        TRON_HIP(hipGetLastError());
    }
    return TRON_OK;
}

// ------------------------------------------------------------------ fix-up of split rows
// G lanes per split row: y[row] += factor * (carry[b0] + ... + carry[b0+cnt-1]).  G = 8 when no row spans more than
// 64 chunks (one workgroup then fixes 32 rows), else a whole wavefront per row.
template <int EPI, int G>
__global__ __launch_bounds__(kBlock) void k_csr_fixup(int nfix, int64_t rows, const int32_t *__restrict__ fix_row,
                                                      const int32_t *__restrict__ fix_part, const int32_t *__restrict__ fix_b0,
                                                      const int32_t *__restrict__ fix_cnt, const double *__restrict__ carry,
                                                      double *__restrict__ yout, const double *__restrict__ aux, double alpha)
{
    const int m = blockIdx.x * (kBlock / G) + threadIdx.x / G;
    const int sub = threadIdx.x & (G - 1);
    const bool live = m < nfix;   // the lane sums below need every lane of the wavefront
    const int b0 = live ? fix_b0[m] : 0, cnt = live ? fix_cnt[m] : 0;
    double s = 0.0;
    for (int k = sub; k < cnt; k += G) s += carry[b0 + k];
    s = group_sum(s, G);
    if (live && sub == 0) {
        const int64_t r = fix_row[m];
        double factor = 1.0;
        if (EPI == EPI_SCALE) factor = aux[r];
        if (EPI == EPI_AXPY) factor = alpha;
        double *dst = yout + (int64_t)fix_part[m] * rows + r;   // fix_part is 0 when unpartitioned
        *dst = fma(factor, s, *dst);
    }
}

template <int EPI>
static int launch_fixup(tron_dataset *ds, const CsrPlan &A, double *yout, const double *aux, double alpha)
{
    if (A.nfix <= 0) return TRON_OK;
    ProfScope ps(ds, SLOT_SPMV_FIXUP);
    if (A.fix_max_cnt <= 64) {
        const int per = kBlock / 8;
        hipLaunchKernelGGL((k_csr_fixup<EPI, 8>), dim3((A.nfix + per - 1) / per), dim3(kBlock), 0, ds->stream, A.nfix, A.rows, A.fix_row,
                           A.fix_part, A.fix_b0, A.fix_cnt, A.carry, yout, aux, alpha);
    } else {
        const int per = kBlock / kWave;
        hipLaunchKernelGGL((k_csr_fixup<EPI, kWave>), dim3((A.nfix + per - 1) / per), dim3(kBlock), 0, ds->stream, A.nfix, A.rows,
                           A.fix_row, A.fix_part, A.fix_b0, A.fix_cnt, A.carry, yout, aux, alpha);
    }
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

// ------------------------------------------------------------------ combine kernels (partitioned layout)
// The partial sums of a plan are stored one per segment (a segment = a row's entries in one partition), partition by
// partition, rows ascending inside a partition -- the kernels above write them as dense 512-byte stores.  A row's
// slots are found by rank: mask[r] says in which partitions row r has a segment; inside the 64 rows of a wavefront
// the slot of (r, x) is group_base[x][r / 64] + (number of lower rows of the group with bit x set).
struct PartialRef {
    const double *partial;
    const uint16_t *mask;
    const GroupBase *group_base;   // one record per group of 64 rows
    const double *row_scale;       // unit plan of X: the value of row i's entries (null otherwise)
    const double *head_sums;       // head partition kept as sorted slices: its sums, row r's at head_pos[r] (null otherwise)
    const int32_t *head_pos;
};

struct HotRef {
    const int32_t *slot_of_row;   // null: no hot rows
    const double *sums;
};

// Sum over the partitions of row r = 64 G + lane, in partition order.  Every lane of the wavefront calls it with
// the same G; `valid` is false for rows past the end.  All loads are issued before the first is used.
__device__ __forceinline__ double sum_parts(const PartialRef &P, int64_t G, int64_t r, bool valid, HotRef hot = HotRef{nullptr, nullptr})
{
    const unsigned m = valid ? P.mask[r] : 0u;
    const GroupBase gb = P.group_base[G];   // uniform: scalar loads
    double s = 0.0;
    if (valid && P.head_sums) s = P.head_sums[P.head_pos[r]];
    if (valid && hot.slot_of_row) {
        const int hs = hot.slot_of_row[r];
        if (hs >= 0) s = hot.sums[hs];
    }
    double v[kMaxParts];
#pragma unroll
    for (int x = 0; x < kMaxParts; ++x) {
        const bool bit = (m >> x) & 1u;
        const uint64_t b = __ballot(bit);
        const int rank = __builtin_amdgcn_mbcnt_hi((unsigned)(b >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)b, 0u));
        v[x] = bit ? P.partial[(int64_t)gb.first[x] + rank] : 0.0;
    }
#pragma unroll
    for (int x = 0; x < kMaxParts; ++x) s += v[x];
    if (P.row_scale && valid) s *= P.row_scale[r];
    return s;
}

// rows are dealt to wavefronts in groups of 64: group g0, g0 + (wavefronts in the grid), ...
#define TRON_FOR_ROW_GROUPS(rows, G, r, valid)                                                                     \
    for (int64_t G = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave, r = G * kWave + (threadIdx.x & (kWave - 1)); \
         G * kWave < (rows); G += (int64_t)gridDim.x * kWavesPerBlock, r += (int64_t)gridDim.x * kBlock)            \
        if (const bool valid = r < (rows); true)

// z = sum of partials; loss terms; partial slot 0 = sum loss
template <int LOSS>
__global__ __launch_bounds__(kBlock) void k_combine_loss(int64_t n, PartialRef P, const double *__restrict__ y,
                                                         double *__restrict__ zhat, double *__restrict__ D, double *__restrict__ red,
                                                         const double *__restrict__ post, Finish fin)
{
    __shared__ double lds[kWavesPerBlock];
    double acc = 0.0;
    TRON_FOR_ROW_GROUPS(n, G, i, valid) {
        const double z = sum_parts(P, G, i, valid);
        if (valid) {
            double a, zh, Di;
            loss_terms_dev<LOSS>(z, y[i], a, zh, Di);
            zhat[i] = post ? post[i] * zh : zh;
            D[i] = Di;
            acc += a;
        }
    }
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) red[blockIdx.x] = acc;
    finish_partials<1>(fin, red, 0, lds);
}

// out = scale .* sum of partials
__global__ __launch_bounds__(kBlock) void k_combine_scale(int64_t rows, PartialRef P, const double *__restrict__ scale,
                                                          double *__restrict__ out, const double *__restrict__ post)
{
    TRON_FOR_ROW_GROUPS(rows, G, i, valid) {
        const double s = sum_parts(P, G, i, valid);
        if (valid) {
            const double o = scale[i] * s;
            out[i] = post ? post[i] * o : o;
        }
    }
}

// out = add + alpha * sum of partials (add == null: add 1); partial slot 0 = out . (SELF ? out : add)
template <bool SELF>
__global__ __launch_bounds__(kBlock) void k_combine_axpy(int64_t rows, PartialRef P, const double *__restrict__ add, double alpha,
                                                         double *__restrict__ out, double *__restrict__ red, HotRef hot, Finish fin)
{
    __shared__ double lds[kWavesPerBlock];
    double acc = 0.0;
    TRON_FOR_ROW_GROUPS(rows, G, i, valid) {
        const double s = sum_parts(P, G, i, valid, hot);
        if (valid) {
            const double a = add ? add[i] : 1.0;
            const double o = fma(alpha, s, a);
            out[i] = o;
            acc += o * (SELF ? o : a);
        }
    }
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) red[blockIdx.x] = acc;
    finish_partials<1>(fin, red, 0, lds);
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
                        double alpha, bool square = false)
{
    {
        ProfScope ps(ds, slot);
        if (square)
            hipLaunchKernelGGL((k_csr_spmv<EPI, true>), dim3(A.nblocks), dim3(kBlock), 0, ds->stream, A.part_nnz[0], A.rowptr, A.col, A.val,
                               A.row_lo, x, yout, aux, alpha, A.carry);
        else
            hipLaunchKernelGGL((k_csr_spmv<EPI, false>), dim3(A.nblocks), dim3(kBlock), 0, ds->stream, A.part_nnz[0], A.rowptr, A.col, A.val,
                               A.row_lo, x, yout, aux, alpha, A.carry);
        TRON_HIP(hipGetLastError());
    }
    TRON_TRY(launch_fixup<EPI>(ds, A, yout, aux, alpha));
    return TRON_OK;
}

static PartArgs part_args(const CsrPlan &A)
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
    pa.slots = A.range_slots;
    return pa;
}

// The head partition as a one-partition launch: val, hot_ids and the partials are passed pre-offset, col16 only
// holds this partition; chunk and segment tables are indexed through the offsets in the arguments.
static PartArgs head_args(const CsrPlan &A)
{
    const int h = A.head;
    PartArgs ha;
    std::memset(&ha, 0, sizeof(ha));
    ha.P = 1;
    ha.nnz[0] = A.part_nnz[h];
    ha.seg0[0] = A.part_seg0[h];
    ha.chunk0[0] = A.part_chunk0[h];
    ha.nchunks[0] = A.part_nchunks[h];
    ha.nhot[0] = A.part_nhot[h];
    ha.slots = kHotSlots;
    return ha;
}

static PartialRef partial_ref(const tron_dataset *ds, const CsrPlan &A)
{
    return PartialRef{ds->row_partials, A.row_mask, A.group_base, A.row_scale, A.sell.on ? A.sell.sums : nullptr, A.sell.on ? A.sell.pos : nullptr};
}

static PartPtrs part_ptrs(const tron_dataset *ds, const CsrPlan &A)
{
    return PartPtrs{A.col, A.val, A.chunk_tab, A.flags, A.hot_x, ds->row_partials, A.carry};
}

static PartPtrs head_ptrs(const tron_dataset *ds, const CsrPlan &A)
{
    const int h = A.head;
    return PartPtrs{A.col16, A.val ? A.val + A.part_base[h] : nullptr, A.chunk_tab, A.flags, A.hot_x ? A.hot_x + (size_t)h * kHotSlots : nullptr,
                    ds->row_partials, A.carry};
}

// partial row sums of all partitions into ds->row_partials (with split rows fixed up)
static int launch_partials(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, bool square = false)
{
    const PartArgs pa = part_args(A);
    if (A.hot_ids) {
        ProfScope ps(ds, SLOT_SPMV_GATHER);
        const int nh = A.P * kHotSlots + A.head_slots;
        hipLaunchKernelGGL(k_gather_hot, dim3((nh + kBlock - 1) / kBlock), dim3(kBlock), 0, ds->stream, nh, A.hot_ids, x, A.hot_x);
        TRON_HIP(hipGetLastError());
    }
    if (A.head >= 0) {
        ProfScope ps(ds, SLOT_SPMV_HEAD);
        const int grid = std::max(1, std::min(A.part_nchunks[A.head], (int)g_tuning.csr_hot_blocks_per_part * kColParts));
        if (A.sell.on) {
            const SellHead &S = A.sell;
            hipLaunchKernelGGL(k_head_sell, dim3((S.nwaves + kSellBlock / kWave - 1) / (kSellBlock / kWave)), dim3(kSellBlock), 0, ds->stream, S.nwaves, S.wave_off, S.data,
                               A.hot_x + (size_t)A.head * kHotSlots, S.sums);
        } else if (A.unit)
            hipLaunchKernelGGL(k_csr_head_unit, dim3(grid), dim3(kBlock), kHotSlots * sizeof(double), ds->stream, head_args(A),
                               head_ptrs(ds, A));
        else
            hipLaunchKernelGGL((k_csr_spmv_part<true, true, false, false>), dim3(grid), dim3(kBlock), kHotSlots * sizeof(double), ds->stream,
                               head_args(A), A.rows, head_ptrs(ds, A), x);
        TRON_HIP(hipGetLastError());
    }
    {
        ProfScope ps(ds, slot);
        const int want = (int)(A.hot_ids ? g_tuning.csr_range_blocks_per_part : g_tuning.csr_blocks_per_part);
        // a single range (small matrices) gets the workgroups that eight ranges would share
        const int per_part = std::max(1, std::min(A.max_chunks, A.P == 1 ? want * kColParts : want));
        if (A.hot_ids && A.unit)
            hipLaunchKernelGGL((k_csr_spmv_part<true, false, false, true>), dim3(per_part * A.P), dim3(kBlock), A.range_slots * sizeof(double), ds->stream,
                               pa, A.rows, part_ptrs(ds, A), x);
        else if (A.hot_ids)
            hipLaunchKernelGGL((k_csr_spmv_part<true, false, false, false>), dim3(per_part * A.P), dim3(kBlock), A.range_slots * sizeof(double), ds->stream,
                               pa, A.rows, part_ptrs(ds, A), x);
        else if (A.unit)   // squares, if any, are in the scaled vector
            hipLaunchKernelGGL((k_csr_spmv_part<false, false, false, true>), dim3(per_part * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows,
                               part_ptrs(ds, A), x);
        else if (square)
            hipLaunchKernelGGL((k_csr_spmv_part<false, false, true, false>), dim3(per_part * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows,
                               part_ptrs(ds, A), x);
        else
            hipLaunchKernelGGL((k_csr_spmv_part<false, false, false, false>), dim3(per_part * A.P), dim3(kBlock), 0, ds->stream, pa, A.rows,
                               part_ptrs(ds, A), x);
        TRON_HIP(hipGetLastError());
    }
    TRON_TRY(launch_fixup<EPI_PLAIN>(ds, A, ds->row_partials, nullptr, 0.0));
    return TRON_OK;
}

int spmv_loss(tron_dataset *ds, const CsrPlan &A, int slot, int loss, const double *x, double *zwork, double *zhat, double *D,
              const double *post, int first)
{
    if (A.plain) {
        if (post) { set_error("internal: post-scaling on an unpartitioned plan"); return TRON_EINVAL; }
        TRON_TRY(launch_plain<EPI_PLAIN>(ds, A, slot, x, zwork, nullptr, 0.0));
        return loss_terms(ds, loss, zwork, zhat, D, first);
    }
    TRON_TRY(launch_partials(ds, A, slot, x));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    const int g = vec_grid(A.rows);
    const Finish fin = finish_for(ds, first, g);
    if (loss == TRON_LOSS_LR)
        hipLaunchKernelGGL(k_combine_loss<TRON_LOSS_LR>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, partial_ref(ds, A), ds->y, zhat, D, ds->partials, post, fin);
    else
        hipLaunchKernelGGL(k_combine_loss<TRON_LOSS_L2SVM>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, partial_ref(ds, A), ds->y, zhat, D, ds->partials, post, fin);
    TRON_HIP(hipGetLastError());
    return g;
}

int spmv_scale(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, const double *scale, double *out, const double *post)
{
    if (A.plain) {
        if (post) { set_error("internal: post-scaling on an unpartitioned plan"); return TRON_EINVAL; }
        return launch_plain<EPI_SCALE>(ds, A, slot, x, out, scale, 0.0);
    }
    TRON_TRY(launch_partials(ds, A, slot, x));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    hipLaunchKernelGGL(k_combine_scale, dim3(vec_grid(A.rows)), dim3(kBlock), 0, ds->stream, A.rows, partial_ref(ds, A), scale, out, post);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

// xs = x .* scale  (or x .* scale^2)
__global__ __launch_bounds__(kBlock) void k_prescale(int64_t m, const double *__restrict__ x, const double *__restrict__ scale,
                                                     int square, double *__restrict__ xs)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < m; i += (int64_t)gridDim.x * kBlock) {
        const double r = scale[i];
        xs[i] = x[i] * (square ? r * r : r);
    }
}

int spmv_axpy(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, const double *add, double alpha, bool dot_self,
              double *out, bool square, bool x_prescaled, int first)
{
    if (square && A.hot_ids) { set_error("internal: squared product on a layout with LDS tables"); return TRON_EINVAL; }
    if (A.unit && A.col_scale && !x_prescaled) {
        // the plan gathers from x .* col_scale (the entries themselves carry no values)
        ProfScope ps(ds, SLOT_SPMV_GATHER);
        hipLaunchKernelGGL(k_prescale, dim3(vec_grid(A.cols)), dim3(kBlock), 0, ds->stream, A.cols, x, A.col_scale, square ? 1 : 0, A.xs);
        TRON_HIP(hipGetLastError());
        x = A.xs;
    } else if (x_prescaled && !(A.unit && A.col_scale)) {
        set_error("internal: pre-scaled vector for a plan without column scale");
        return TRON_EINVAL;
    }
    if (A.plain) {
        TRON_TRY(launch_plain<EPI_AXPY>(ds, A, slot, x, out, add, alpha, square));
        if (!add) return 0;
        return dot_partials(ds, A.rows, out, dot_self ? out : add, nullptr, nullptr, nullptr, nullptr, first);
    }
    HotRef hot{nullptr, nullptr};
    if (A.hot.ntiles_total > 0) {
        TRON_TRY(launch_hot_tiles(ds, A, x, square));
        hot.slot_of_row = A.hot.slot_of_row;
        hot.sums = A.hot.sums;
    }
    TRON_TRY(launch_partials(ds, A, slot, x, square));
    ProfScope ps(ds, SLOT_SPMV_COMBINE);
    const int g = vec_grid(A.rows);
    const Finish fin = finish_for(ds, add ? first : -1, g);
    if (dot_self)
        hipLaunchKernelGGL(k_combine_axpy<true>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, partial_ref(ds, A), add, alpha, out, ds->partials, hot, fin);
    else
        hipLaunchKernelGGL(k_combine_axpy<false>, dim3(g), dim3(kBlock), 0, ds->stream, A.rows, partial_ref(ds, A), add, alpha, out, ds->partials, hot, fin);
    TRON_HIP(hipGetLastError());
    return g;
}

// ------------------------------------------------------------------ byte accounting (see PlanBytes)
PlanBytes plan_bytes(const CsrPlan &A)
{
    PlanBytes b{0, 0, 0, 0, 0, 0};
    const int64_t vbytes = A.unit ? 0 : 8;   // value stream per stored entry
    if (A.plain) {
        // plain CSR in chunks: columns and values once, row offsets, the gathered vector and the result once each
        b.ranges = A.part_nnz[0] * (4 + 8) + 8 * (A.rows + 1) + 4 * ((int64_t)A.nblocks + 1) + 8 * A.cols + 8 * A.rows;
        return b;
    }
    const int64_t per_chunk = kBlock /* flag bits */ + (int64_t)sizeof(int4) /* table entry */ + 8 /* carry */;
    int64_t nseg_head = 0;
    if (A.hot_ids) {
        const int64_t nh = (int64_t)A.P * kHotSlots + A.head_slots;
        b.gather = nh * (4 + 8 + 8);
    }
    if (A.sell.on) {
        b.head = A.sell.ngroups * kWave * 16 + 8 * ((int64_t)A.sell.nwaves + 1) + 8 * (int64_t)kSellSlots + 8 * A.sell.nrows_with_entries;
    } else if (A.head >= 0) {
        const int h = A.head;
        nseg_head = A.nseg_total - A.part_seg0[h];
        b.head = (int64_t)A.part_nchunks[h] * (kChunk * (2 + vbytes) + per_chunk) + 8 * (int64_t)kHotSlots + 8 * nseg_head;
    }
    int64_t range_chunks = 0;
    for (int x = 0; x < A.P; ++x) range_chunks += A.part_nchunks[x];
    const int64_t nseg_ranges = A.nseg_total - nseg_head;
    b.ranges = range_chunks * (kChunk * (4 + vbytes) + per_chunk) + 8 * nseg_ranges + 8 * A.cold_cols +
               (A.hot_ids ? 8 * (int64_t)A.P * A.range_slots : 0);
    if (A.hot.ntiles_total > 0) {
        const HotTiles &H = A.hot;
        const int64_t acc = 8 * (int64_t)kTileSlices * H.blocks_per_slice * kTileSlots;
        b.tiles = H.ntiles_total * (kChunk * (2 + vbytes) + kBlock + (int64_t)sizeof(int4)) + 2 * H.nseg_padded + 8 * H.span_total + acc;
        b.tile_reduce = acc + 8 * (int64_t)kTileSlices * kTileSlots;
    }
    // combine: every partial sum once, the row mask, the group table, the result; plus what the plan's extras need per row
    b.combine = 8 * A.nseg_total + 2 * A.rows + (int64_t)sizeof(GroupBase) * A.ngroups + 8 * A.rows;
    if (A.sell.on) b.combine += (8 + 4) * A.rows;                        // sorted sums through the position array
    if (A.hot.ntiles_total > 0) b.combine += 4 * A.rows + 8 * (int64_t)A.hot.nhot;   // slot of each row, sums of the hot rows
    if (A.row_scale) b.combine += 8 * A.rows;
    return b;
}

}  // namespace tron
