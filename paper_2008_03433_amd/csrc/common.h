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

// ---------------------------------------------------------------- process-wide tuning knobs (tron_tuning_set)
struct Tuning {
    int64_t csr_parts = 0;   // column partitions of the CSR layouts: 0 = automatic, 1 = never, 8 = always
    int64_t csr_hot = 1;     // LDS table of frequent columns for the partitioned forward layout (0 = off)
    int64_t csr_range_blocks_per_part = 96;   // persistent workgroups per column range when LDS tables are used
    int64_t csr_range_slots = 4096;   // LDS table entries per column range (the head partition always has kHotSlots)
    int64_t csr_head = 1;    // head partition for the matrix' most frequent columns (needs csr_hot; 0 = off)
    int64_t csr_hot_blocks_per_part = 96;  // persistent workgroups per partition when the LDS table is used
    int64_t csr_blocks_per_part = 128;     // persistent workgroups per column range without LDS tables
    int64_t csr_tiles = 1;   // hot-row tiles for the transposed orientation of partitioned matrices (0 = off)
    int64_t csr_tile_blocks_per_slice = 0;   // persistent workgroups per slice of hot rows (0 = automatic: 96, or 160 for unit plans)
    int64_t csr_sell_blocks = 1024;   // workgroups of the sorted-slice head kernel
    int64_t csr_sell = 1;    // unit plans: the head partition as sorted slices of 64 rows, one row per lane (0 = as chunks)
    int64_t csr_segmented = -1;  // unpartitioned layouts as segments + flag bits instead of plain CSR: 0 never, 1 always, -1 when a
                             //   chunk of the plain layout would leave one thread a long row (see csr_plan_build)
    int64_t csr_unit = 1;    // partitioned layouts: drop the value stream when every row of X holds one repeated value (0 = off)
    int64_t dense_compact = -1;         // dense L2-SVM: Hessian-vector products on a compacted copy of the active rows:
                                        //   0 never, 1 whenever rows are inactive, -1 automatic (see dense_compact_wanted)
    int64_t cg_speculate = -1;  // enqueue CG iteration k + 1 before the host has read iteration k's scalars: 0 never, 1 always,
                                // -1 when a Hessian-vector product is cheap (a wasted one costs less than the waits saved)
    int64_t fuse_reductions = -1;  // second reduction stage inside the producing kernel (last workgroup): 0 never, 1 always,
                                   //   -1 automatic (launches of few workgroups, where the extra launch costs more than it does)
    int64_t dense_device_driver = -1;   // tron_solve on dense d <= 32 without preconditioner driven from the device:
                                        //   0 never, 1 always, -1 automatic (the L2-SVM on matrices up to 1 GB)
    int64_t batch_grid = 0;  // workgroups of the multi-problem pass: 0 = as many as are resident at once
    int64_t batch_mfma = -1; // multi-problem pass on the matrix units: 1 = yes, 0 = no, -1 = the library decides
    int64_t batch_lean = 1;         // matrix-unit pass: rounds without function / gradient requests run a kernel compiled without those steps
    int64_t batch_mfma_rows = 0;    // rows of X a wavefront of that pass keeps in LDS at a time: 32 or 64; 0 = by LDS footprint
};
extern Tuning g_tuning;

// ---------------------------------------------------------------- launch geometry
constexpr int kBlock = 256;          // threads per workgroup everywhere (4 wavefronts of 64)
constexpr int kWave = 64;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxGrid = 2048;       // 256 CUs x 8 resident workgroups: grid-stride kernels use at most this
constexpr int kChunk = 2048;         // nonzeros per workgroup in the CSR kernels (256 threads x 8)
constexpr int kScalars = 16;         // scalar slots shared by the reductions

// ---------------------------------------------------------------- profiling slots
enum Slot {
    SLOT_SPMV_FWD = 0,     // X times a vector: the chunk kernel (unpartitioned) or the kernel over the column ranges
    SLOT_SPMV_BWD,         // the same for the transposed copy
    SLOT_SPMV_HEAD,        // head partition of X (most frequent columns)
    SLOT_SPMV_TILES,       // hot-row tiles of the transposed product
    SLOT_SPMV_TILE_REDUCE, // sum of the tiles' workgroup accumulators
    SLOT_SPMV_GATHER,      // vector entries of the LDS-resident columns
    SLOT_SPMV_FIXUP,       // rows split across workgroups
    SLOT_SPMV_COMBINE,     // sum of the partitions' partial row sums + epilogue
    SLOT_LOSS_TERMS,       // zhat, D, sum loss from z
    SLOT_DENSE_FUN_GRAD,   // fused dense z / loss / D / X^T zhat
    SLOT_DENSE_HV,         // fused dense X^T (D (X v))
    SLOT_DENSE_FINALIZE,   // column sums of per-workgroup partials
    SLOT_DENSE_COMPACT,    // compacted copy of the active rows
    SLOT_DOT,              // dot products / norms (first stage)
    SLOT_REDUCE_FINAL,     // second reduction stage -> scalars
    SLOT_CG_VEC,           // CG vector updates
    SLOT_BATCH_PASS,       // multi-problem pass over X
    SLOT_BATCH_ADVANCE,    // multi-problem partial sums + trust-region / CG step
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
// One orientation of the sparse matrix (rows x cols) laid out for the SpMV kernels.
//
// Work is split by nonzeros: a workgroup streams chunks of kChunk consecutive nonzeros and owns the
// rows that *start* inside a chunk; a row that continues into later chunks receives the remainder
// through `carry` and the fix-up list.
//
// P == 1 (small matrices): plain CSR, one workgroup per chunk, epilogue applied directly -- or, when long and short rows
// share chunks, the segment layout of the partitioned case with a single range.
//
// P == 8 (the gathered vector would not stay resident in one L2): the column space is cut into 8
// contiguous ranges with equal nonzero counts and the nonzeros are stored range-major: partition x
// holds, row by row, the entries whose column lies in range x.  Workgroup b works on partition b % 8,
// so -- with workgroups dealt round-robin to the 8 XCDs -- each XCD's L2 only ever gathers from its own
// slice of the vector.  Inside a partition only the non-empty rows ("segments") are described: per
// chunk a table entry and one flag bit per entry (last entry of its segment).  Every segment owns one
// partial sum, stored in segment order; row_mask and group_base let the combine kernels find the
// partial sums of a row and add them in a fixed order before applying the epilogue.
constexpr int kColParts = 8;            // column ranges, one per XCD
constexpr int kMaxParts = kColParts + 1;   // + the head partition (see CsrPlan::head)
constexpr int kHotSlots = 4096;   // LDS table entries per workgroup (32 KiB)
// The head partition kept as sorted slices has one table for a workgroup of 16 wavefronts, one workgroup per CU:
// 16384 entries (128 KiB).  Its place in hot_ids / hot_x is behind the P range tables, which stay kHotSlots apart.
constexpr int kSellSlots = 16384;
constexpr int kSellBlock = 1024;

// Hot-row tiles of the transposed product  out[j] += sum_i val * x[i]  (j = row of the plan, i = column).
// The rows with the most entries (up to kTileSlices * kTileSlots of them) are taken out of the CSR layout and
// stored as tiles: a tile holds the entries of one slice of those rows for a short range of consecutive
// columns (at most 512), sorted by (row slot, column).  The workgroup copies those columns of x into LDS and
// gathers from the copy (no L2 request per entry, and none of the vector memory pipeline's one-lane-per-clock
// gathers), and the per-row sums of a tile are added to LDS accumulators that a persistent workgroup keeps for its
// slice; workgroup accumulators are summed in a fixed order.  The header of a tile is {first column, segments,
// columns spanned, offset of its segment slots}.
constexpr int kTileSlices = 8;      // slices of hot rows, one per XCD
constexpr int kTileSlots = 2048;    // hot rows per slice = LDS accumulators per workgroup (16 KiB)
constexpr int kTileMinCount = 32;   // rows with fewer entries stay in the CSR layout
constexpr int kTileWindow = 512;    // columns a tile may span (the kernels copy them into LDS, two per thread)

struct HotTiles {
    int64_t nnz = 0;                     // entries held in tiles
    int nhot = 0;                        // hot rows; row with rank r (by entry count) is slot r / 8 of slice r % 8
    int64_t ntiles_total = 0;
    int64_t tile0[kTileSlices] = {0};    // first tile of slice s
    int64_t ntiles[kTileSlices] = {0};
    int blocks_per_slice = 0;            // persistent workgroups per slice
    int64_t nseg_padded = 0;             // entries of seg_slot (every tile's block padded to a multiple of 8)
    int64_t span_total = 0;              // sum over the tiles of the columns they span (what the kernels copy into LDS)
    double *val = nullptr;               // device, ntiles_total * kChunk (zero padded); null for a unit plan
    uint16_t *iloc = nullptr;            // device, ntiles_total * kChunk: column minus the tile's first column
    uint8_t *flags = nullptr;            // device, ntiles_total * 256: bit e of byte t = entry 8t + e of the tile is the last of its segment
    int4 *hdr = nullptr;                 // device, per tile: {first column, segments, unused, index into seg_slot}
    uint16_t *seg_slot = nullptr;        // device: slot of every segment, tile by tile (a tile's block starts at a multiple of 8)
    int32_t *slot_of_row = nullptr;      // device, rows: slice * kTileSlots + slot, or -1
    double *wg_acc = nullptr;            // device, kTileSlices * blocks_per_slice * kTileSlots workgroup accumulators
    double *sums = nullptr;              // device, kTileSlices * kTileSlots: per hot row, sum over its tiles
    void release();
};

// per group of 64 consecutive rows: the first segment of each partition whose row lies in the group or after it
struct alignas(64) GroupBase {
    int32_t first[16];   // kMaxParts used
};

// Head partition of a unit plan as sorted slices (sliced ELLPACK): the rows are sorted by their number of head entries
// inside windows of kSellWindow consecutive rows and cut into slices of 64; a slice stores, for each of its rows, the
// 16-bit LDS slots of the row's entries padded to the slice's longest row (a multiple of 8), in groups of 8 entries
// per row: a group is 64 x 16 bytes, lane after lane.  A header group precedes the groups of a slice: lane l's 16 bytes
// hold where the sum of lane l's row goes (int32, -1: no row) and the number of groups that follow (int32).  One lane
// then sums one row -- no segment bookkeeping at all.  The sums are stored in sorted order, sums[pos[row]] -- the 64 sums
// of a slice are one 512-byte store; scattered 8-byte stores, one per row, cost a third of the kernel -- and the combine
// kernels read them through pos (a row's position stays inside its window).  Rows without head entries are never
// written and stay 0.
// The slices are dealt to a fixed number of wavefronts (longest first, each to the wavefront with the least work so
// far) and stored wavefront by wavefront, so that a wavefront reads one contiguous stream of groups.
constexpr int kSellWindow = 8192;
constexpr int kSellAhead = 8;     // groups a wavefront keeps in flight; every wavefront's stream is a multiple of it long
struct SellHead {
    bool on = false;
    int nwaves = 0;               // wavefronts the slices were dealt to (= 4 x workgroups of the kernel)
    int nslices = 0;
    int64_t ngroups = 0;          // groups of 64 x 16 bytes in data (headers, slots and padding)
    int64_t nrows_with_entries = 0;
    int64_t *wave_off = nullptr;     // device, nwaves + 1: first group of each wavefront's stream in data
    uint16_t *data = nullptr;     // device: groups (headers and slots; kSellSlots = the padding slot, whose table entry is 0)
    double *sums = nullptr;       // device, rows: in sorted order
    int32_t *pos = nullptr;       // device, rows: where the sum of a row is
    void release();
};

struct CsrPlan {
    int64_t rows = 0, cols = 0, nnz = 0;
    SellHead sell;                       // optional (head partition of a unit plan)
    HotTiles hot;                        // optional (transposed orientation of large matrices)
    int P = 1;                           // number of column ranges (1 = unpartitioned)
    bool plain = true;                   // P == 1 stored as plain CSR (row offsets, one workgroup per chunk, epilogue applied directly);
                                         //   false: the segment layout below (always for P > 1; for P == 1 when rows of very
                                         //   different lengths share chunks, which the plain kernel handles badly)
    int head = -1;                       // P, when partition P holds the entries of the matrix' most frequent columns
                                         //   (whole rows, every entry served from one LDS table, 16-bit slots in col16); else -1
    int32_t *col = nullptr;              // device, (padded) nnz of the ranges; with an LDS table, hot columns are stored as ~slot
    uint16_t *col16 = nullptr;           // device, (padded) nnz of the head partition: LDS slot of each entry
    double *val = nullptr;               // device, (padded) nnz; null for a unit plan
    // Unit plan (partitioned layouts of a matrix X = diag(r) B with B binary, i.e. every instance's entries share one
    // value r_i): the entries carry no values.  The plan of X multiplies row sum i by row_scale[i]; the plan of X^T
    // gathers from the vector x .* col_scale (formed by the caller or by spmv_axpy itself into xs).
    bool unit = false;
    const double *row_scale = nullptr;   // device, rows (not owned) or null
    const double *col_scale = nullptr;   // device, cols (not owned) or null
    double *xs = nullptr;                // device, cols: work space for x .* col_scale
    int nblocks = 0;                     // total number of chunks
    double *carry = nullptr;             // device, nblocks: sum of the part of a row entering chunk c from before
    int nfix = 0;                        // number of (partition, split row) pairs
    int fix_max_cnt = 0;                 // largest fix_cnt
    int32_t *fix_row = nullptr;          // device, nfix: the split row (P > 1: its segment's slot in the partial sums)
    int32_t *fix_part = nullptr;         // device, nfix: 0 (kept for the address arithmetic shared by both layouts)
    int32_t *fix_b0 = nullptr;           // device, nfix: first chunk id holding a continuation of it
    int32_t *fix_cnt = nullptr;          // device, nfix: number of consecutive chunks that do
    // ---- P == 1
    int64_t *rowptr = nullptr;           // device, rows+1
    int32_t *row_lo = nullptr;           // device, nblocks+1: first row starting at or after chunk c
    // ---- P > 1
    int64_t part_base[kMaxParts] = {0};  // position of partition x in col/val (multiple of kChunk)
    int64_t part_nnz[kMaxParts] = {0};
    int64_t part_seg0[kMaxParts] = {0};  // first segment of partition x (segments are numbered partition by partition)
    int part_chunk0[kMaxParts] = {0};    // first chunk id of partition x (= part_base / kChunk)
    int part_nchunks[kMaxParts] = {0};
    int part_nhot[kMaxParts] = {0};      // LDS-resident columns of partition x
    int max_chunks = 0;                  // max over the column ranges
    int range_slots = 0;                 // LDS table entries used by the column ranges (<= kHotSlots)
    int head_slots = 0;                  // LDS table entries of the head partition (kHotSlots, or kSellSlots as sorted slices)
    int32_t *hot_ids = nullptr;          // device, P*kHotSlots + head_slots column ids of the LDS tables (null: no LDS table)
    double *hot_x = nullptr;             // device, as many: the gather vector at those columns, refreshed every call
    int64_t nseg_total = 0;              // segments (= partial sums) of the plan
    int64_t cold_cols = 0;               // columns with entries that no LDS table serves (P > 1): what the gathers must fetch
    int64_t ngroups = 0;                 // ceil(rows / 64)
    GroupBase *group_base = nullptr;     // device, ngroups records
    int4 *chunk_tab = nullptr;           // device, per chunk: {first owned segment (partition-relative), number of owned
                                         //   segments, offset where the first owned segment starts, unused}
    uint8_t *flags = nullptr;            // device, nblocks * 256: bit e of byte t of a chunk = its entry 8t + e is the last
                                         //   entry of a row inside the chunk
    uint16_t *row_mask = nullptr;        // device, rows: bit x set iff the row has entries in partition x
    void release();
};

}  // namespace tron

// ---------------------------------------------------------------- the handle
struct tron_batch;
struct tron_dataset {
    int64_t n = 0, d = 0;
    bool dense = false;
    hipStream_t stream = nullptr;
    int device = 0;

    // dense
    double *X = nullptr;
    // sparse: forward (n x d) and explicit transposed (d x n) copies
    tron::CsrPlan fwd, bwd;

    double *y = nullptr;         // n (sparse layouts)
    int8_t *y8 = nullptr;        // n (dense layout: labels as +1 / -1 bytes)
    double *z = nullptr;         // n   (sparse: margins X w; also a0 / a1 work space for Hv)
    double *zhat = nullptr;      // n   (sparse only; dense folds it into the fused pass)
    double *Dbuf[2] = {nullptr, nullptr};  // n each: D at the accepted w and at the trial point
    double active_frac[2] = {1.0, 1.0};    // dense: fraction of rows with D != 0 in each buffer (from the last fun/grad pass)
    bool D_is_mask[2] = {false, false};    // dense L2-SVM: the buffer holds one active-set byte per row instead
    int Dcur = 0;
    bool have_D = false;

    // reductions
    double *row_partials = nullptr;  // sparse, partitioned: P x max(n, d) partial row sums
    double *partials = nullptr;  // device scratch for first-stage partial sums
    int64_t partials_len = 0;
    double *scal_host = nullptr; // kScalars pinned host scalars, mapped into the device's address space
    double *scal_dev = nullptr;  // the device address of scal_host (kernels write the scalars there)
    double *scal_copy = nullptr; // the same scalars in device memory, for kernels that continue from them without the host
    unsigned *ticket = nullptr;  // counter of finished workgroups for reductions completed inside the producing kernel (zero between kernels)
    bool finish_done = false;    // the last producing kernel did: the next reduce_final call is a no-op
    int dense_grid = 0;          // workgroups of the dense kernels
    int vec_grid_n = 0, vec_grid_d = 0;  // workgroups of elementwise kernels over n / d

    double *unit_scale = nullptr;  // sparse, unit plans: r (n), the value shared by the entries of instance i

    // dense L2-SVM: compacted copy of the active rows of D buffer `hat_slot` (-1: none), see dense_compact_build
    double *Xhat = nullptr;          // hat_cap rows x d
    int64_t hat_cap = 0, hat_rows = 0;
    uint64_t *hat_bits = nullptr;    // hat_cap / 64 + 1 words: the all-active set of the compacted copy
    int64_t *tile_off = nullptr;     // ceil(n / 64) + 1: active rows before each 64-row tile
    int64_t *scan_blocks = nullptr;  // partial sums of the scan over the tiles
    int hat_slot = -1;
    int64_t active_count[2] = {0, 0};   // rows with D != 0 in each buffer

    tron_batch *self_batch = nullptr;   // dense: one problem over all rows, for solves driven from the device

    // solver vectors (d each), allocated on first tron_solve
    double *sv[9] = {nullptr};
    hipEvent_t cg_event[2] = {nullptr, nullptr};   // end of a CG iteration's kernels, by iteration parity
    double *cg_partials = nullptr;   // kCgRegions x kMaxGrid: per-workgroup sums that the next CG kernel adds up itself

    tron::Profiler prof;
};

namespace tron {

// Where the kernel that produces first-stage partial sums puts the finished sums when it adds them itself (the workgroup
// that finishes last does it, see finish_partials): scalar slots first, first + 1, ... of both copies.  ticket == null:
// a separate k_reduce_final launch adds them.
struct Finish {
    unsigned *ticket;
    double *scal, *scal_copy;
    int first;
};
// The Finish for a producing kernel of `grid` workgroups whose sums go to scalars first_scalar...: with a ticket when
// the launch is small enough for that to pay (then the reduce_final call that follows does nothing), without otherwise or
// when first_scalar < 0.
Finish finish_for(tron_dataset *ds, int first_scalar, int grid);

// RAII bracket used by the launch helpers
struct ProfScope {
    tron_dataset *ds; int idx;
    hipStream_t st;
    ProfScope(tron_dataset *d, int slot, hipStream_t s = nullptr)
        : ds(d), idx(d->prof.on ? d->prof.begin(slot, s ? s : d->stream) : -1), st(s ? s : d->stream) {}
    ~ProfScope() { if (idx >= 0) ds->prof.end(idx, st); }
};

// ---- kernels_vec.hip
// out_scal[s] = sum of partials[s*stride .. s*stride+count) for s < nslots (second stage)
int reduce_final(tron_dataset *ds, int nslots, int count, int stride, int first_scalar);
// partial sums of a.b (and optionally c.e, f.h) into partial slots 0..k-1; returns #partials per slot
// `first` (here and below): scalar slot the finished sums go to when the kernel completes the reduction itself (see Finish)
int dot_partials(tron_dataset *ds, int64_t m, const double *a0, const double *b0, const double *a1, const double *b1,
                 const double *a2, const double *b2, int first = -1);
int loss_terms(tron_dataset *ds, int loss, const double *z, double *zhat, double *D, int first = -1);  // partial slot 0 = sum loss
int read_scalars(tron_dataset *ds, int count);  // stream sync; then scal_host[0..count) holds what the kernels wrote
// CG vector kernels (see solver.hip); M = diagonal preconditioner or null
// The scalars a CG run keeps on the device between its kernels, by iteration parity (iteration it reads r.r from
// kScalRR + it % 2 and its reduction leaves the new r.r in kScalRR + (it + 1) % 2; whether iteration it stepped to the
// trust-region boundary is in kScalFlag + it % 2).  Two slots each, so that the kernels of iteration it + 1 can be
// enqueued before the host has read what iteration it left.
constexpr int kScalRR = 6, kScalFlag = 8;
// The step and direction kernels leave per-workgroup partial sums in regions of cg_partials, kMaxGrid doubles each.  With
// at most kCgDirectGrid workgroups the consumer adds them up itself (every workgroup, in the order of the second-stage
// kernel, so all get the same bits), which saves the two launches that would do nothing else; above that every workgroup
// re-reading every partial sum costs more than those launches, and the second-stage kernel runs in between.
enum { CGP_RR = 0, CGP_PP, CGP_SP, CGP_SS, kCgRegions };
constexpr int kCgDirectGrid = 512;
// rr0 >= 0: also starts a CG run (scalar kScalRR = rr0, both flags cleared)
int cg_init(tron_dataset *ds, const double *g, const double *M, double *s, double *r, double *p, int first = -1, double rr0 = -1.0);  // M: slot0 = g.(g/M); returns #partials
// What the CG step kernel needs to form the step length itself from the device copy of the scalars (slot 0 = p.Hp,
// slots 1..3 = p.p, s.p, s.s unless it == 0, r.r as above): alpha = rr / p.Hp, or the step to the trust-region boundary
// if |s + alpha p| >= delta.  The kernel leaves the step taken in scalar 4 and the boundary flag in its slot.
// An iteration that was enqueued ahead although the run had ended -- the iteration before it went to the boundary, or
// left sqrt(r.r) <= tol -- changes nothing: both kernels test for that themselves, with the host's own comparison.
struct CgStepCtl {
    double tol, delta;   // tol = xi times the length of the gradient the run started from
    int it;              // iteration number, from 0 (then s = 0 and p.p = r.r)
};
// n_dir: workgroups of the direction kernel before (its partial sums of p.p, s.p, s.s; unused when it == 0), 0 = take the
// sums from scalars 1..3.  n_php: partial sums of p.Hp at the start of ds->partials, 0 = take p.Hp from scalar 0.
// Returns its own number of workgroups: the partial sums of r.r | r.(r/M) in region CGP_RR.
int cg_step(tron_dataset *ds, const CgStepCtl &ctl, int n_dir, int n_php, const double *p, const double *Hp, const double *M, double *s, double *r);
int vec_workgroups(int64_t m);   // workgroups of the vector kernels (and of the sparse combine kernels) over m elements
// n_step: workgroups of the step kernel before: adds up the new r.r and leaves it in its scalar slot (host and device copy);
// 0 = the slot holds it already.  beta = (new r.r) / (old r.r); partial sums of p.p, s.p, s.s (M-weighted) in their regions.
// Returns its number of workgroups.
int cg_dir(tron_dataset *ds, const CgStepCtl &ctl, int n_step, const double *r, const double *s, const double *M, double *p);
// the second stage as a launch of its own, for `count` partial sums in each of nregions regions of cg_partials from `region` on
int reduce_cg_regions(tron_dataset *ds, int region, int nregions, int count, int first_scalar);
int trial_point(tron_dataset *ds, const double *w, const double *s, const double *g, const double *r, const double *M,
                double *wnew, int first = -1);  // wnew = w+s; slots: g.s, s.r, s.s | s.Ms
int probe_read(const double *src, int64_t count, int reps, hipStream_t st, double *ms, double *checksum);
int probe_copy(double *dst, const double *src, int64_t count, int reps, hipStream_t st, double *ms);

// ---- kernels_csr.hip
// parts: 1 = plain CSR, 0 = choose from the size of the gathered vector
// unit: build a unit plan (see CsrPlan::unit; partitioned layouts only; h_val is not read)
int csr_plan_build(CsrPlan &P, int64_t rows, int64_t cols, const int64_t *h_rowptr, const int32_t *h_col,
                   const double *h_val, int parts, bool hot, bool unit, hipStream_t st);
// Hot-row tiles for plan A (rows x cols) from the *other* orientation's CSR (cols x rows: t_rowptr over A's columns,
// t_col = A's row ids).  slot_code[row] = slice * kTileSlots + slot for hot rows, -1 otherwise.
int hot_tiles_build(CsrPlan &A, const int64_t *t_rowptr, const int32_t *t_col, const double *t_val,
                    const std::vector<int32_t> &slot_code, int nhot, hipStream_t st);
// Products with one orientation; all enqueue on ds->stream.
//   spmv_loss:  z = A x, then per-instance loss terms: zhat, D; partial slot 0 of ds->partials = sum loss
//   spmv_scale: out = scale .* (A x)
//   spmv_axpy:  out = add + alpha (A x); partial slot 0 = out . (dot_self ? out : add).  add == null: add 1.
//               square: the entries of A are squared (transposed orientation only)
//   post (spmv_loss: applied to zhat; spmv_scale: to out), when not null: the stored vector is multiplied by it
//   elementwise -- the column scale of the unit plan that will gather from it (then passed with x_prescaled = true)
// Each returns the number of first-stage partials in slot 0 (0 if none), or a negative error.
int spmv_loss(tron_dataset *ds, const CsrPlan &A, int slot, int loss, const double *x, double *zwork, double *zhat, double *D,
              const double *post = nullptr, int first = -1);
int spmv_scale(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, const double *scale, double *out,
               const double *post = nullptr);
int spmv_axpy(tron_dataset *ds, const CsrPlan &A, int slot, const double *x, const double *add, double alpha,
              bool dot_self, double *out, bool square = false, bool x_prescaled = false, int first = -1);

// Bytes one launch of each kernel of a product with plan A has to move in the format A stores (what the byte counters
// of the memory system would read for a launch without any wasted traffic): the streams it reads once, the vector
// elements it must fetch at least once, and what it writes.  Zero for parts the plan does not have.
struct PlanBytes {
    int64_t gather;        // k_gather_hot: ids, the gathered elements, the table copy
    int64_t head;          // head partition (sorted slices or chunks)
    int64_t ranges;        // the column ranges (or the single chunk kernel of an unpartitioned plan)
    int64_t tiles;         // hot-row tiles incl. the workgroup accumulators
    int64_t tile_reduce;
    int64_t combine;       // partial sums in, row vector(s) in, result out
};
PlanBytes plan_bytes(const CsrPlan &A);

// ---- kernels_dense.hip
bool dense_supported(int64_t d);
int dense_grid_for(int64_t n, int64_t d);
int64_t dense_partials_needed(int64_t n, int64_t d);
// fused pass: z = X w, loss terms, D -> Dout, partial sums of X^T zhat and of the loss;
// then g = w + C (column sums) (if g != null), scalars[0] = sum loss, [1] = w.w, [2] = g.g, [3] = rows with D != 0
// (the caller reads the four scalars and records scalars[3] / n in active_frac[Dslot])
int dense_fun_grad(tron_dataset *ds, int loss, double C, const double *w, int Dslot, double *g);
int dense_labels_from_device(tron_dataset *ds, int64_t row0, int64_t m, const double *y_dev);
int dense_validate_device(tron_dataset *ds, int64_t m, const double *X_dev, const double *y_dev, int *what);
// Hv = v + C X^T (D (X v)); scalars[0] = v.Hv
int dense_hv(tron_dataset *ds, double C, int Dslot, const double *v, double *Hv);

// out = 1 + C diag(X^T D X)
int dense_hess_diag(tron_dataset *ds, double C, int Dslot, double *out);
// X_hat = the rows of X that are active in Dbuf[Dslot] (the compacted copy of Section 5 of the paper), built on the device;
// dense_hv then runs over it.  Needs the active set as bit words (L2-SVM, d <= 32) and active_count[Dslot].  Enqueue only
// (allocates, and therefore synchronises, when the copy has to grow).
int dense_compact_build(tron_dataset *ds, int Dslot);
// whether the knob asks for the copy, given how many Hessian-vector products the last inner solve took
bool dense_compact_wanted(const tron_dataset *ds, int Dslot, int recent_cg_iters);
void dense_compact_release(tron_dataset *ds);

// ---- batch.hip
int dense_device_solve(tron_dataset *ds, const tron_params &P, double *w_dev, tron_result *res);
void dense_device_release(tron_dataset *ds);

// ---- solver.hip
int fun_enqueue(tron_dataset *ds, int loss, const double *w, int Dslot);                        // scalars[0]=sum of loss terms, [1]=w.w, no sync
int fun_eval(tron_dataset *ds, int loss, double C, const double *w, int Dslot, double *f_out);  // syncs
int grad_enqueue(tron_dataset *ds, double C, const double *w, double *g, int scalar);           // scalars[scalar]=g.g, no sync
// out = 1 + C sum_i D_i x_ij^2 with D = Dbuf[Dslot] (the diagonal of the Hessian; C scaled by the caller for a blend). Enqueue only.
int hess_diag_enqueue(tron_dataset *ds, double C, int Dslot, double *out);
int grad_eval(tron_dataset *ds, double C, const double *w, double *g, double *gnorm_out);        // syncs
int hv_enqueue(tron_dataset *ds, double C, const double *v, double *Hv, int *vhv_partials = nullptr);   // scalars[0]=v.Hv, no sync

}  // namespace tron
