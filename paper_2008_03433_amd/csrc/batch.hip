// Several problems of Section 3 of the paper over one resident dense matrix: the cross-validation setting of
// Section 2.1 (three folds, nested cross-validation inside each), where the problems differ only in the instances
// they train on and in C.  The problems advance in lock-step rounds.  A round is
//   1. one pass over X (k_batch_pass on the vector units, up to eight problems; k_batch_pass_mfma on the fp64 matrix
//      units, up to sixteen) that serves every problem's pending request -- X^T (D (X v)) for a problem inside its CG
//      iteration, or z = X w / loss / D / X^T zhat for one at a trial point (Table 1) -- so that an element of X read
//      from HBM is used by all of them;
//   2. one small kernel (k_batch_advance) that adds up the pass's per-workgroup partial sums and then runs, for every
//      problem, the step of Algorithm 1 / of the truncated CG iteration that was waiting for the product, and posts
//      the problem's next request.
// The trust-region logic runs on the device: the vectors have d <= 32 entries, one lane each.  The host only reads,
// every few rounds, which problems are still running.
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "dense_tile.h"

namespace tron {
namespace {

constexpr int kBatchMax = TRON_BATCH_MAX;
constexpr int kVecPad = TRON_BATCH_MAX_D;   // doubles per stored vector
static_assert(kVecPad <= kWave, "one lane per vector entry");

enum { MODE_IDLE = 0, MODE_HV = 1, MODE_FG = 2, MODE_DIAG = 3 };   // MODE_DIAG: column sums of D_i x_ij^2 (the Hessian diagonal)
enum { PH_DONE = 0, PH_ONESHOT, PH_REF, PH_START, PH_CG, PH_TRIAL, PH_DIAG0, PH_DIAG };
enum { BEGIN_SOLVE = 0, BEGIN_FG, BEGIN_HV };

// request of the next pass: written by the begin / advance kernels, read by the pass
struct BatchCtl {
    int32_t mode[kBatchMax];    // MODE_*
    int32_t dslot[kBatchMax];   // which of the problem's two D buffers the pass reads (MODE_HV) or writes (MODE_FG)
    double vec[kBatchMax][kVecPad];   // v (MODE_HV) or w (MODE_FG), zero past d
};

struct ProbScalars {
    int32_t phase, status, converged, outer, cg_total, n_fun, n_grad, n_hv, cg_it, onb, dcur, trace_len;
    double C, f, gnorm, gnorm0, delta, rr, pred, snorm, out_scal;
    double gscaled;   // what the inner solver measures its residual against: |g|, or sqrt(g.M^-1 g) with a preconditioner
};

// solver state of one problem (device memory)
struct ProbState {
    ProbScalars sc;
    double w[kVecPad], wnew[kVecPad], g[kVecPad], s[kVecPad], r[kVecPad], p[kVecPad], out[kVecPad];
    double M[kVecPad];   // diagonal preconditioner (1 - a) I + a diag(H) of the current iterate (used when blend > 0)
};

struct SolveParams {
    int loss, max_outer, max_cg, trace_cap;
    double eps, xi;
    double blend;   // 0: plain CG; a in (0, 1]: CG preconditioned by M = (1 - a) I + a diag(H), rebuilt at every accepted iterate
};

struct BatchC { double v[kBatchMax]; };

typedef const uint64_t __attribute__((address_space(4))) *ConstWords;

// ------------------------------------------------------------------ the pass over X
// Work layout as in the single-problem kernels: a wave tile is 64 consecutive rows, a wavefront walks a contiguous
// range of tiles.  Per tile and problem one 64-bit word says which rows concern the problem: its members
// (function/gradient pass, logistic Hessian) or its active set I (L2-SVM Hessian: D_ii = 2 on I).  Rows that concern no
// problem are not read.  The words of the next tile are fetched (scalar loads) while the current one is processed.
// New active-set words are collected in LDS and stored 64 tiles at a time.
//   member: [k][tile]     Dbits: [k][slot][tile]     Dval (logistic D): [k][slot][row]
//   partials: [k][column 0..d-1, then the loss sum][workgroup]
// Dbits_in and Dbits_out are the same array: a problem's plane is either read (MODE_HV) or written (MODE_FG) by a pass.
template <int E, int L, int U, bool VEC, int KT, int LOSS>
__global__ __launch_bounds__(kBlock, 2) void k_batch_pass(int64_t n, int64_t d, const double *__restrict__ X,
                                                       const int8_t *__restrict__ y,
                                                       const BatchCtl *__restrict__ ctl, const uint64_t *__restrict__ member,
                                                       const uint64_t *__restrict__ Dbits_in, uint64_t *Dbits_out,
                                                       double *Dval, int64_t ntiles, double *__restrict__ partials, int /* K: unused here */)
{
    using T = Tile<E, L, U, VEC>;
    static_assert(T::RT == kWave, "one 64-bit word per tile");
    __shared__ double lvec[KT][E * L];
    __shared__ double lds[kWavesPerBlock * E * L];
    __shared__ double lds_red[kWavesPerBlock];
    // function/gradient pass only, kept out of the registers: per wavefront and problem the loss sum of every lane's rows
    // and the new active-set words of up to 64 tiles
    __shared__ double lloss[kWavesPerBlock][KT][kWave];
    __shared__ uint64_t lheld[kWavesPerBlock][KT][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int q = lane % L;
    int mode[KT], dslot[KT];
    bool any = false, any_fg = false;
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        mode[k] = ctl->mode[k];
        dslot[k] = ctl->dslot[k];
        any |= mode[k] != MODE_IDLE;
        any_fg |= mode[k] == MODE_FG;
    }
    if (!any) return;
    constexpr bool svm = LOSS == TRON_LOSS_L2SVM;
    // L2-SVM Hessian: D_ii = 2 on the active set.  The factor is put into v (exact: a power of two), the product
    // then only selects rows.
    for (int i = threadIdx.x; i < KT * E * L; i += kBlock) {
        const int k = i / (E * L), c = i % (E * L);
        const double scale = (svm && ctl->mode[k] == MODE_HV) ? 2.0 : 1.0;
        lvec[k][c] = (c < d) ? scale * ctl->vec[k][c] : 0.0;
    }
    __syncthreads();
    // this lane's row in step u is tile row u * RW + rl: its bit in a 64-bit word, as a 32-bit mask of the word's half
    const int rl = lane / L;
    uint32_t rowbit[U];
#pragma unroll
    for (int u = 0; u < U; ++u) rowbit[u] = 1u << ((u * T::RW + rl) & 31);
    // plane of the words that say which rows concern problem k.  The words are the same for all lanes: read through
    // the constant address space they arrive in scalar registers.  (No plane read here is written by this pass.)
    ConstWords words[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        if ((mode[k] == MODE_HV || mode[k] == MODE_DIAG) && svm) words[k] = (ConstWords)(Dbits_in + ((int64_t)k * 2 + dslot[k]) * ntiles);
        else words[k] = (ConstWords)(member + (int64_t)k * ntiles);
    }
    double acc[KT][E];
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        lloss[wv][k][lane] = 0.0;
        lheld[wv][k][lane] = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[k][e] = 0.0;
    }
    const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t wave_id = (int64_t)blockIdx.x * kWavesPerBlock + wv;
    const int64_t per_wave = (ntiles + nwaves - 1) / nwaves;
    const int64_t first = wave_id * per_wave;
    const int64_t last = (first + per_wave < ntiles) ? first + per_wave : ntiles;
    uint64_t wnext[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) wnext[k] = (mode[k] != MODE_IDLE && first < last) ? words[k][first] : 0;
    int it = 0;
    for (int64_t tile = first; tile < last; ++tile, ++it) {
        const int slotl = it & (kWave - 1);
        const int64_t row0 = tile * kWave;
        uint64_t wk[KT], rows = 0;
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            wk[k] = wnext[k];
            rows |= wk[k];
            wnext[k] = (mode[k] != MODE_IDLE && tile + 1 < last) ? words[k][tile + 1] : 0;
        }
        if (rows != 0) {
            double x[U][E];
            T::load(X, n, d, row0, lane, x, rows);
            const double yrow = (any_fg && row0 + lane < n) ? (double)y[row0 + lane] : 1.0;
            // logistic Hessian: D of the tile's rows for every problem, lane i taking row i, fetched together with x
            double Drow[KT];
            if constexpr (!svm) {
#pragma unroll
                for (int k = 0; k < KT; ++k) {
                    Drow[k] = 0.0;
                    if ((mode[k] == MODE_HV || mode[k] == MODE_DIAG) && wk[k] != 0 && row0 + lane < n)
                        Drow[k] = Dval[((int64_t)k * 2 + dslot[k]) * n + row0 + lane];   // zero outside the problem's rows
                }
            }
            // the vectors are read from LDS again for every tile: hoisted out of the loop they would take KT * E
            // registers per lane (the empty statement hides the loop invariance from the compiler)
            int qoff = q * E;
            asm volatile("" : "+v"(qoff));
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                if (mode[k] == MODE_IDLE || wk[k] == 0) continue;   // uniform
                double vk[E], t[U], c[U];
                if (mode[k] == MODE_DIAG) {
                    // sum_i D_i x_ij^2: the row coefficient is D itself, the entries are squared
                    if (svm) {
                        const uint32_t lo = (uint32_t)wk[k], hi = (uint32_t)(wk[k] >> 32);
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            uint32_t half;
                            if (T::RW == kWave) half = (lane < 32) ? lo : hi;
                            else half = (u * T::RW < 32) ? lo : hi;
                            c[u] = (half & rowbit[u]) ? 2.0 : 0.0;
                        }
                    } else {
                        T::from_row_owner(Drow[k], lane, c);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
#pragma unroll
                        for (int e = 0; e < E; ++e) acc[k][e] = fma(c[u] * x[u][e], x[u][e], acc[k][e]);
                    }
                    continue;
                }
#pragma unroll
                for (int e = 0; e < E; ++e) vk[e] = lvec[k][qoff + e];
                T::row_dots(x, vk, t);
                if (mode[k] == MODE_HV) {
                    // a1 = D (X v), formed by every lane of a row for itself (all of them hold the row's x.v)
                    if (svm) {
                        const uint32_t lo = (uint32_t)wk[k], hi = (uint32_t)(wk[k] >> 32);
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            uint32_t half;
                            if (T::RW == kWave) half = (lane < 32) ? lo : hi;
                            else half = (u * T::RW < 32) ? lo : hi;
                            c[u] = (half & rowbit[u]) ? t[u] : 0.0;
                        }
                    } else {
                        T::from_row_owner(Drow[k], lane, c);
#pragma unroll
                        for (int u = 0; u < U; ++u) c[u] *= t[u];
                    }
                } else {
                    // the per-row terms of Table 1 run once per row, lane i owning tile row i
                    const double z = T::to_row_owner(t, lane);
                    const bool mine = (wk[k] >> lane) & 1u;
                    double alpha, zhat, Di;
                    loss_terms_dev<LOSS>(z, yrow, alpha, zhat, Di);
                    if (!mine) { alpha = 0.0; zhat = 0.0; Di = 0.0; }
                    lloss[wv][k][lane] += alpha;
                    if (svm) {
                        const uint64_t nb = __ballot(Di != 0.0);
                        if (lane == 0) lheld[wv][k][slotl] = nb;
                    } else if (mine) {
                        Dval[((int64_t)k * 2 + dslot[k]) * n + row0 + lane] = Di;
                    }
                    T::from_row_owner(zhat, lane, c);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[k][e] = fma(c[u], x[u][e], acc[k][e]);
                }
            }
        }
        if (svm && any_fg && (slotl == kWave - 1 || tile + 1 == last)) {
            // lane i takes the word of tile (tile - slotl + i): consecutive 8-byte words per problem
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                if (mode[k] == MODE_FG && lane <= slotl)
                    Dbits_out[((int64_t)k * 2 + dslot[k]) * ntiles + (tile - slotl) + lane] = lheld[wv][k][lane];
                lheld[wv][k][lane] = 0;
            }
        }
    }
    const int64_t cols = d + 1;
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        if (mode[k] == MODE_IDLE) continue;   // uniform over the workgroup
        double *pk = partials + (int64_t)k * cols * gridDim.x;
        T::flush(acc[k], d, lane, wv, lds, pk);
        const double ls = block_sum(lloss[wv][k][lane], lds_red);   // its barriers also order the reuse of lds
        if (threadIdx.x == 0) pk[d * (int64_t)gridDim.x + blockIdx.x] = ls;
    }
}

// ------------------------------------------------------------------ the pass over X on the matrix units
// With several problems the pass is two skinny matrix products per tile of 64 rows: Z = X V (64 x d by d x K) and
// G += X^T C (d x 64 by 64 x K), C = the row coefficients formed from Z.  This kernel runs them as fp64 matrix
// instructions (16 x 16 x 4: A 16 x 4, B 4 x 16, result 16 x 16; lane l holds A[l % 16][l / 16], B[l / 16][l % 16] and, in
// its result register v, the element [4 v + l / 16][l % 16]) with the problems as the 16 result columns:
//   * a wavefront copies its tile of X into LDS exactly as it lies in memory (16-byte pieces, the loads of the next tile
//     in flight during the work on the current one; rows that concern no problem are not read);
//   * Z: per 16 rows and 4 columns of X one instruction, A read from LDS, B = V kept in registers;
//   * lane (g = l / 16, p = l % 16) then holds Z of problem p at rows 4 v + g of every 16-row group, and C is formed where
//     Z lies.  Hessian rounds: the L2-SVM selects by the bit of the active-set word (factor 2 folded into V), the
//     logistic loss multiplies by D, which each lane loads for its own elements (four consecutive rows of a problem
//     per instruction and group of lanes; the four instructions of a 16-row step use up whole lines).  Function/gradient rounds of the
//     L2-SVM: the lane evaluates the loss terms of its own sixteen (row, problem) elements per tile (the same
//     per-element function as k_batch_pass; labels and membership come as bits of two 64-bit words per tile), keeps one
//     loss sum -- its problem's -- and its rows' bits of the new active-set word, which the four lanes of a problem put
//     together once per tile.  The logistic terms (an exponential, a logarithm and a division each) cost more than
//     everything else in the pass, so they are evaluated once per row and problem that asks -- not for the sixteen
//     result columns: Z goes through an LDS exchange area to a row-per-lane layout, where the new D is stored as
//     64 consecutive rows of a problem, and zhat comes back the same way;
//   * G: the result rows are the columns of X (two instructions for d > 16); the four rows 4 v + g, g = 0..3, that the
//     lanes hold in register v are the summation index, so C is used where it lies.  A = X[row][column] read from LDS
//     along a row: conflict-free.  Problems asking for the Hessian diagonal use the same instructions with A squared and
//     C = D.
// Results go to the same partials array, in the same layout, as k_batch_pass writes: the steps after the pass do not
// know which kernel ran.  Sums are formed in a fixed order (the instruction's, then tiles in order, wavefronts 0..3).
typedef double mfma4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wavefront complete in the order issued; this keeps the compiler from reordering them
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// the 64-bit value of lane `src` (per-lane index)
__device__ __forceinline__ uint64_t lane_value(uint64_t v, int src)
{
    const int lo = __builtin_amdgcn_ds_bpermute(src * 4, (int)(uint32_t)v);
    const int hi = __builtin_amdgcn_ds_bpermute(src * 4, (int)(uint32_t)(v >> 32));
    return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}

// doubles of LDS per wavefront: a unit of RT rows of X (rows padded to at most dmax + 2 doubles, 16 doubles of slack) and,
// where logistic function / gradient requests are served (kex = K, otherwise 0), the exchange area: kex rows of RT + 1
// doubles for Z and zhat by problem and row
__host__ __device__ constexpr int mfma_wave_doubles(int dmax, int kex, int rt) { return rt * (dmax + 2) + 16 + ((kex * (rt + 1) + 1) & ~1); }

// RT = rows of X a wavefront keeps in LDS at a time: a whole 64-row tile, or half of one (smaller LDS footprint and
// fewer registers for the loads in flight, so more wavefronts per SIMD to cover the dependent chains of matrix
// instructions; the row-per-lane steps then serve 64 / RT problems side by side).
// FG = false: a pass in which no problem asks for function and gradient (the host knows the modes of the round).  The
// per-element loss terms, the labels, the loss sums and the new active-set words are compiled out: fewer registers, so
// more wavefronts per SIMD.
template <bool VEC, int DMAX, int KT, int LOSS, int RT, bool FG>
__global__ __launch_bounds__(kBlock, FG ? 2 : 3) void k_batch_pass_mfma(int64_t n, int64_t d, const double *__restrict__ X,
                                                            const int8_t *__restrict__ y,
                                                            const BatchCtl *__restrict__ ctl, const uint64_t *__restrict__ member,
                                                            const uint64_t *__restrict__ Dbits_in, uint64_t *Dbits_out,
                                                            double *Dval, int64_t ntiles, double *__restrict__ partials, int K)
{
    static_assert(KT <= 16 && KT <= kBatchMax, "one result column per problem");
    static_assert(RT == 32 || RT == 64, "a tile or half a tile");
    constexpr bool svm = LOSS == TRON_LOSS_L2SVM;
    static_assert(DMAX % 4 == 0 && DMAX <= kVecPad, "d <= DMAX, in steps of the instruction's four columns");
    constexpr int PW = VEC ? 2 : 1;                 // doubles per piece
    constexpr int NH = kWave / RT;                  // units per tile
    constexpr int NS = RT / 16;                     // groups of 16 rows per unit
    constexpr int NP = RT * DMAX / PW / kWave;      // pieces per lane and unit at most (a unit is RT d doubles)
    constexpr int PP = kWave / RT;                  // problems side by side in the row-per-lane layout
    static_assert(RT * DMAX / PW % kWave == 0 && KT % PP == 0, "whole pieces per lane; whole groups of problems");
    constexpr int kExRow = RT + 1;                  // doubles per problem in the exchange area (padded against bank conflicts)
    constexpr bool kHasEx = FG && !svm;             // logistic function / gradient requests go through the exchange area
    extern __shared__ double dyn[];
    __shared__ double lds_red[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int D = (int)d;
    int mode[KT], dslot[KT];
    bool any = false, any_fg = false, any_hv = false, any_diag = false, any_mul = false, any_exd = false;
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        mode[k] = ctl->mode[k];
        dslot[k] = ctl->dslot[k];
        any |= mode[k] != MODE_IDLE;
        any_fg |= mode[k] == MODE_FG;
        any_hv |= mode[k] == MODE_HV;
        any_diag |= mode[k] == MODE_DIAG;
        any_mul |= (FG && mode[k] == MODE_FG) || mode[k] == MODE_HV;
        any_exd |= !svm && (mode[k] == MODE_HV || mode[k] == MODE_DIAG);
    }
    any_fg = FG && any_fg;
    if (!any) return;
    // The unit in LDS: row r at r S, S = the first length >= d whose rows start in different banks for 16 consecutive rows
    // (16-byte pieces: S = 2 mod 4; 8-byte pieces: S odd).  Every lane copies NP pieces per unit; those past the unit
    // (d < DMAX) are fetched from the first bytes of X and land in the slack behind it.
    constexpr int xs_len = RT * (DMAX + 2) + 16;
    const int S = VEC ? D + ((6 - D % 4) % 4) : (D | 1);
    const int kex = kHasEx ? K : 0;
    double *Xs = dyn + (size_t)wv * mfma_wave_doubles(DMAX, kex, RT);
    double *Ex = Xs + xs_len;                                    // [problem][row of the unit]: Z, then zhat
    for (int i = lane; i < mfma_wave_doubles(DMAX, kex, RT); i += kWave) Xs[i] = 0.0;
    // this lane in the matrix layouts: g = summation index / row block, p = problem (result column) or row / column of X
    const int p = lane & 15, g = lane >> 4;
    const bool pk = p < K;   // K <= KT
    const int modeM = pk ? ctl->mode[pk ? p : 0] : MODE_IDLE;
    const int dslotM = pk ? ctl->dslot[pk ? p : 0] : 0;
    const bool exM = !svm && (modeM == MODE_HV || modeM == MODE_DIAG);   // this lane's problem reads its D
    const int rowl = lane & (RT - 1), sub = lane / RT;   // row-per-lane layout: row of the unit, problem of a group of PP
    // logistic D of this lane's problem in the slot it reads; lanes without such a problem stay at the start of the array
    const double *const DvalM = (!svm && pk) ? Dval + ((int64_t)p * 2 + dslotM) * n : Dval;
    double Vop[DMAX / 4];
#pragma unroll
    for (int kk = 0; kk < DMAX / 4; ++kk) {
        const int f = 4 * kk + g;
        const bool use = f < D && (modeM == MODE_HV || (FG && modeM == MODE_FG));
        const double scale = (svm && modeM == MODE_HV) ? 2.0 : 1.0;
        Vop[kk] = use ? scale * ctl->vec[pk ? p : 0][f] : 0.0;
    }
    // lane k < KT fetches the word of problem k: its active set (L2-SVM Hessian / diagonal) or its members
    const uint64_t *plane = nullptr;
    if (lane < KT) {
        const int m = ctl->mode[lane < KT ? lane : 0];
        if ((m == MODE_HV || m == MODE_DIAG) && svm) plane = Dbits_in + ((int64_t)lane * 2 + ctl->dslot[lane < KT ? lane : 0]) * ntiles;
        else if (m != MODE_IDLE) plane = member + (int64_t)lane * ntiles;
    }
    const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t wave_id = (int64_t)blockIdx.x * kWavesPerBlock + wv;
    const int64_t per_wave = (ntiles + nwaves - 1) / nwaves;
    const int64_t first = wave_id * per_wave;
    const int64_t last = (first + per_wave < ntiles) ? first + per_wave : ntiles;
    const uint64_t inv_d = (0x100000000ull + (uint64_t)D - 1) / (uint64_t)D;   // row of element e < 2048: (e inv_d) >> 32 (2^32 itself for d = 1)
    // per piece of this lane, fixed for the whole pass: its row in the unit (RT = past the unit) and where it goes in LDS
    uint32_t prow[NP], plds[NP];
#pragma unroll
    for (int it = 0; it < NP; ++it) {
        const uint32_t e = (uint32_t)(it * kWave + lane) * PW;
        const uint32_t row = (uint32_t)(((uint64_t)e * inv_d) >> 32);
        prow[it] = row < (uint32_t)RT ? row : (uint32_t)RT;
        plds[it] = row < (uint32_t)RT ? row * (uint32_t)S + (e - row * (uint32_t)D) : (uint32_t)(xs_len - 2);
    }

    double xr[NP][PW];
    double lossM = 0.0;   // L2-SVM: loss terms of this lane's rows of its problem
    double lossK[KT];     // logistic: loss terms of this lane's row, by problem
#pragma unroll
    for (int k = 0; k < KT; ++k) lossK[k] = 0.0;
    uint64_t nbM = 0;     // this lane's rows' bits of its problem's new active-set word for the current tile
    mfma4 G1 = {0.0, 0.0, 0.0, 0.0}, G2 = {0.0, 0.0, 0.0, 0.0};

    // the rows of unit h of a tile that concern some problem
    auto unit_rows = [&](uint64_t rows, int h) -> uint64_t { return RT == kWave ? rows : ((rows >> (RT * h)) & 0xffffffffull); };
    // Loads of a unit into xr, then xr into LDS.  No load sits behind a branch on a per-lane condition (the compiler would
    // wait for every load in flight where such paths join): a piece of a row that concerns no problem, or past the end, is
    // fetched from the first bytes of X instead -- one cached line for all of them -- and copied like the others; its row
    // coefficient is zero in every problem and X is finite, so what lies there does not matter.
    auto fetch = [&](int64_t tile, int h, uint64_t urows) {
        const int64_t row0 = tile * kWave + RT * h;
        const double *base = X + row0 * d;
        const bool full = urows == (RT == kWave ? ~0ull : 0xffffffffull) && row0 + RT <= n;   // the same for every lane: no per-row questions
#pragma unroll
        for (int it = 0; it < NP; ++it) {
            const uint32_t e = (uint32_t)(it * kWave + lane) * PW;
            const uint32_t row = prow[it];
            bool take = row < (uint32_t)RT;
            if (!full) take = take && ((urows >> (row & (RT - 1))) & 1u) && row0 + row < n;
            const double *src = take ? base + e : X;
            if constexpr (VEC) {
                const double2 t = *reinterpret_cast<const double2 *>(src);
                xr[it][0] = t.x;
                xr[it][1] = t.y;
            } else {
                xr[it][0] = *src;
            }
        }
    };
    auto to_lds = [&]() {
#pragma unroll
        for (int it = 0; it < NP; ++it) {
            if constexpr (VEC) *reinterpret_cast<double2 *>(Xs + plds[it]) = make_double2(xr[it][0], xr[it][1]);
            else Xs[plds[it]] = xr[it][0];
        }
    };
    const uint64_t *plane_c = plane ? plane : member;   // a valid address for the lanes that fetch no word
    // raw loads (clamped addresses); what they are worth is decided where they are used, so that nothing waits for them early
    auto word_raw = [&](int64_t tile) { return plane_c[tile < last ? tile : last - 1]; };
    auto word_ok = [&](int64_t tile) { return plane != nullptr && tile < last; };
    auto label_raw = [&](int64_t tile, int h) {
        const int64_t i = tile * kWave + RT * h + rowl;
        return (int)y[i < n ? i : n - 1];   // rows past n belong to no problem: their label is never used
    };
    // a value that is the same within each group of RT lanes: x[sub] of PP values that are the same for every lane
    auto by_sub_i = [&](const int *x) { return (PP == 1 || sub == 0) ? x[0] : x[PP - 1]; };
    auto by_sub_u = [&](const uint64_t *x) { return (PP == 1 || sub == 0) ? x[0] : x[PP - 1]; };
    static_assert(PP <= 2, "by_sub picks between two");

    // words of the current tile (w0), the next (w1) and the one after (loaded in the loop); their scalar copies
    uint64_t w0 = 0, w1 = 0;
    if (first < last) {   // the same for the whole wavefront
        w0 = word_ok(first) ? word_raw(first) : 0ull;
        w1 = word_ok(first + 1) ? word_raw(first + 1) : 0ull;
    }
    uint64_t wk[KT], rows_cur = 0;
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        wk[k] = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(w0 >> 32), k) << 32) | (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)w0, k);
        rows_cur |= wk[k];
    }
    int ycur = 1;   // the labels travel with the unit: asked for with its loads, first touched after they have all arrived
    if (first < last && unit_rows(rows_cur, 0) != 0) {
        if (any_fg) ycur = label_raw(first, 0);
        fetch(first, 0, unit_rows(rows_cur, 0));
    }
    for (int64_t tile = first; tile < last; ++tile) {
        const uint64_t w2 = word_raw(tile + 2);
        uint64_t wkn[KT], rows_next = 0;
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            wkn[k] = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(w1 >> 32), k) << 32) | (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)w1, k);
            rows_next |= wkn[k];
        }
        // the word of this lane's problem
        uint64_t wordM = 0;
        if (svm || any_fg) wordM = lane_value(w0, p);
#pragma unroll 1
        for (int h = 0; h < NH; ++h) {
            const uint64_t urows = unit_rows(rows_cur, h);
            if (urows != 0) to_lds();
            // the loads of the unit after this one
            int ynext = 1;
            {
                const bool same_tile = h + 1 < NH;
                const int64_t nt = same_tile ? tile : tile + 1;
                const int nh = same_tile ? h + 1 : 0;
                const uint64_t nrows = unit_rows(same_tile ? rows_cur : rows_next, nh);
                if (nt < last && nrows != 0) {
                    if (any_fg) ynext = label_raw(nt, nh);
                    fetch(nt, nh, nrows);
                }
            }
            if (urows != 0) {
                wave_lds_fence();
                // Z = X V for rows 16 s .. 16 s + 15 of the unit
                auto z_of = [&](int s) {
                    mfma4 z = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                    for (int kk = 0; kk < DMAX / 4; ++kk) {   // columns past d: V is zero there and what A reads is finite
                        const double a = Xs[(16 * s + p) * S + 4 * kk + g];
                        z = __builtin_amdgcn_mfma_f64_16x16x4f64(a, Vop[kk], z, 0, 0, 0);
                    }
                    return z;
                };
                if (kHasEx && any_fg) {
                    // logistic function / gradient requests: Z to the row-per-lane layout, the terms once per row and
                    // problem that asks (D stored from there), zhat back
#pragma unroll 1
                    for (int s = 0; s < NS; ++s) {
                        const mfma4 z = z_of(s);
                        if (modeM == MODE_FG) {
#pragma unroll
                            for (int v = 0; v < 4; ++v) Ex[p * kExRow + 16 * s + 4 * v + g] = z[v];
                        }
                    }
                    wave_lds_fence();
                    const double yrow = (double)ycur;
#pragma unroll
                    for (int k = 0; k < KT; k += PP) {
                        bool some = false;
                        int mk[PP], dk[PP];
                        uint64_t wq[PP];
#pragma unroll
                        for (int j = 0; j < PP; ++j) {
                            mk[j] = mode[k + j];
                            dk[j] = dslot[k + j];
                            wq[j] = wk[k + j];
                            some |= mk[j] == MODE_FG;
                        }
                        if (!some) continue;   // uniform
                        const int kk = k + sub;
                        const bool act = by_sub_i(mk) == MODE_FG && kk < K;
                        const double z = Ex[(kk < K ? kk : 0) * kExRow + rowl];
                        const bool mine = act && ((by_sub_u(wq) >> (RT * h + rowl)) & 1u);
                        double alpha, zhat, Di;
                        loss_terms_dev<LOSS>(z, yrow, alpha, zhat, Di);
                        if (!mine) { alpha = 0.0; zhat = 0.0; Di = 0.0; }
#pragma unroll
                        for (int j = 0; j < PP; ++j) lossK[k + j] += (sub == j) ? alpha : 0.0;
                        if (mine) Dval[((int64_t)kk * 2 + by_sub_i(dk)) * n + tile * kWave + RT * h + rowl] = Di;
                        if (act) Ex[kk * kExRow + rowl] = zhat;
                    }
                    wave_lds_fence();
                }
                // labels of the unit's rows as a word (the same in every lane)
                const uint64_t yword = (svm && any_fg) ? __ballot(ycur > 0) : 0ull;
                // G += X^T C, 16 rows at a time
#pragma unroll 1
                for (int s = 0; s < NS; ++s) {
                    // logistic D of the lane's four elements, asked for before the products that form Z (zero outside the
                    // problem's rows: never written there); no load sits behind a per-lane branch
                    double ev[4] = {0.0, 0.0, 0.0, 0.0};
                    bool evok[4] = {false, false, false, false};
                    if (any_exd) {   // uniform
                        const int64_t r0 = tile * kWave + RT * h + 16 * s + g;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            evok[v] = exM && r0 + 4 * v < n;
                            ev[v] = *(evok[v] ? DvalM + r0 + 4 * v : Dval);
                        }
                    }
                    mfma4 z = {0.0, 0.0, 0.0, 0.0};
                    if (any_hv || (svm && any_fg)) z = z_of(s);
                    // every LDS read of the 16 rows first (none behind a per-lane condition), then the selects and the products.
                    // Columns of X past d give result rows that nobody reads: A is used as it lies in LDS.
                    double a1v[4], a2v[4], ex[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int r = 16 * s + 4 * v + g;
                        ex[v] = kHasEx ? Ex[(pk ? p : 0) * kExRow + r] : 0.0;   // zhat of a logistic function / gradient request
                        a1v[v] = Xs[r * S + p];
                        a2v[v] = (DMAX > 16) ? Xs[r * S + 16 + p] : 0.0;
                    }
                    const uint32_t bits = (uint32_t)(wordM >> (RT * h + 16 * s + g));   // bit 4 v: row 16 s + 4 v + g of the unit
                    const uint32_t ybits = (uint32_t)(yword >> (16 * s + g));            // the same rows' labels
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const double e = evok[v] ? ev[v] : 0.0;
                        const bool bit = (bits >> (4 * v)) & 1u;
                        double cfg = 0.0;   // zhat of a function / gradient request
                        if (kHasEx) cfg = (modeM == MODE_FG) ? ex[v] : 0.0;
                        if (svm && any_fg) {   // uniform
                            const double yv = ((ybits >> (4 * v)) & 1u) ? 1.0 : -1.0;
                            double alpha, zhat, Di;
                            loss_terms_dev<LOSS>(z[v], yv, alpha, zhat, Di);
                            const bool mine = modeM == MODE_FG && bit;   // a row of this lane's problem (rows past n have no bit)
                            lossM += mine ? alpha : 0.0;
                            cfg = mine ? zhat : 0.0;
                            const int rt = RT * h + 16 * s + 4 * v + g;   // the row in its tile
                            nbM |= (uint64_t)(mine && Di != 0.0) << rt;
                        }
                        double c;
                        if (svm) c = (modeM == MODE_HV) ? (bit ? z[v] : 0.0) : cfg;
                        else c = (modeM == MODE_HV) ? e * z[v] : cfg;
                        if (any_mul) {
                            G1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1v[v], c, G1, 0, 0, 0);
                            if (DMAX > 16) G2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a2v[v], c, G2, 0, 0, 0);
                        }
                        if (any_diag) {
                            double cd;
                            if (svm) cd = (modeM == MODE_DIAG && bit) ? 2.0 : 0.0;
                            else cd = (modeM == MODE_DIAG) ? e : 0.0;
                            G1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1v[v] * a1v[v], cd, G1, 0, 0, 0);
                            if (DMAX > 16) G2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a2v[v] * a2v[v], cd, G2, 0, 0, 0);
                        }
                    }
                }
                wave_lds_fence();   // the next unit is written over this one
            }
            asm volatile("" : "+v"(ynext));   // nothing of the next unit's loads is touched before this point
            ycur = ynext;
        }
        if (svm && any_fg) {
            // the four lanes of a problem hold disjoint rows' bits of its new word; a tile without rows still gets its zero
            uint64_t word = nbM | lane_value(nbM, lane ^ 16);
            word |= lane_value(word, lane ^ 32);
            if (g == 0 && modeM == MODE_FG) Dbits_out[((int64_t)p * 2 + dslotM) * ntiles + tile] = word;
            nbM = 0;
        }
        w0 = w1;
        w1 = word_ok(tile + 2) ? w2 : 0ull;
        rows_cur = rows_next;
#pragma unroll
        for (int k = 0; k < KT; ++k) wk[k] = wkn[k];
    }
    // wavefronts 0..3 added in order; result register v of lane (g, p) is column 4 v + g (G1) / 16 + 4 v + g (G2) of problem p
    __syncthreads();
    double *Gs = dyn;   // [wavefront][column 0..31][problem 0..15]
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        Gs[((wv * 32) + 4 * v + g) * 16 + p] = G1[v];
        Gs[((wv * 32) + 16 + 4 * v + g) * 16 + p] = G2[v];
    }
    __syncthreads();
    const int64_t cols = d + 1;
    for (int i = threadIdx.x; i < KT * D; i += kBlock) {
        const int k = i / D, col = i % D;
        if (ctl->mode[k] == MODE_IDLE) continue;
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) t += Gs[((w * 32) + col) * 16 + k];
        partials[((int64_t)k * cols + col) * gridDim.x + blockIdx.x] = t;
    }
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        if (mode[k] == MODE_IDLE) continue;   // uniform over the workgroup
        const double ls = FG ? block_sum(svm ? (p == k ? lossM : 0.0) : lossK[k], lds_red) : 0.0;
        if (threadIdx.x == 0) partials[((int64_t)k * cols + d) * gridDim.x + blockIdx.x] = ls;
    }
}

// ------------------------------------------------------------------ membership words
// planes[k][tile] bit i = bit k of member[tile*64 + i] (member == null: every row belongs to every problem); rows past n
// give zero bits.  bad[0] is set when a word has a bit at or above K.
__global__ __launch_bounds__(kBlock) void k_member_planes(int64_t n, int K, const uint32_t *__restrict__ member,
                                                          int64_t ntiles, uint64_t *__restrict__ planes, int *bad)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
    for (int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; tile < ntiles; tile += nwaves) {
        const int64_t row = tile * kWave + lane;
        const uint32_t m = (row < n) ? (member ? member[row] : ((K < 32) ? (1u << K) - 1u : ~0u)) : 0u;
        if (K < 32 && (m >> K) != 0u) bad[0] = 1;
        for (int k = 0; k < K; ++k) {
            const uint64_t b = __ballot((m >> k) & 1u);
            if (lane == 0) planes[(int64_t)k * ntiles + tile] = b;
        }
    }
}

// ------------------------------------------------------------------ per-problem steps on the device
// Every lane of the wavefront executes every statement (the sums run over all 64 lanes); lanes at or past d hold zeros
// and their memory accesses are masked by `in`.
__device__ __forceinline__ double dot64(double a, double b) { return wave_sum(a * b); }

struct Request {
    int mode, slot;
    double vec;   // this lane's entry of the vector
};

// Start of the truncated CG iteration at the current iterate: s = 0, r = -g, p = r (preconditioned: p = r / M, and the
// residual is measured by r.M^-1 r); the first product is H p.  m: this lane's entry of M, 1 without a preconditioner.
__device__ __forceinline__ Request cg_begin(ProbState &S, ProbScalars &sc, int j, bool in, double g, double m)
{
    const double p0 = -g / m;
    if (in) {
        S.s[j] = 0.0;
        S.r[j] = -g;
        S.p[j] = p0;
    }
    sc.rr = sc.gscaled * sc.gscaled;
    sc.cg_it = 0;
    sc.onb = 0;
    sc.phase = PH_CG;
    return Request{MODE_HV, sc.dcur, p0};
}

// End of the inner iteration: trial point w + s and the model's reduction pred = -q(s) = -1/2 (g.s - s.r);
// the next pass evaluates f and the gradient there, D going to the problem's other buffer.
__device__ __forceinline__ Request cg_end(ProbState &S, ProbScalars &sc, int j, bool in, double s, double r, double m)
{
    const double w = in ? S.w[j] : 0.0, g = in ? S.g[j] : 0.0;
    const double wnew = w + s;
    const double gs = dot64(g, s), sr = dot64(s, r);
    sc.snorm = sqrt(dot64(m * s, s));   // the length the radius rules use: the M-norm of the iteration
    sc.pred = -0.5 * (gs - sr);
    if (in) S.wnew[j] = wnew;
    sc.phase = PH_TRIAL;
    return Request{MODE_FG, 1 - sc.dcur, wnew};
}

__device__ __forceinline__ void finish(ProbScalars &sc, int status)
{
    sc.status = status;
    sc.converged = (status == TRON_OK) ? 1 : 0;
    sc.phase = PH_DONE;
}

constexpr int kAdvanceBlock = 1024;

// One workgroup per problem.  All sixteen wavefronts add up the pass's partial sums (fixed order); the first one then runs
// the step that was waiting for them.  The rules are those of the single-problem driver (Algorithm 1 with
// Steihaug's truncated CG), lane j holding entry j of every vector.
__global__ __launch_bounds__(kAdvanceBlock) void k_batch_advance(int64_t d, int grid, const double *__restrict__ partials,
                                                          BatchCtl *ctl, ProbState *st, SolveParams P,
                                                          tron_trace_rec *trace)
{
    const int k = blockIdx.x;
    const int mode = ctl->mode[k];
    if (mode == MODE_IDLE) return;
    __shared__ double cs[kVecPad + 1];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    for (int c = wv; c <= d; c += kAdvanceBlock / kWave) {
        const double *p = partials + ((int64_t)k * (d + 1) + c) * grid;
        double s = 0.0;
        for (int b = lane; b < grid; b += kWave) s += p[b];
        s = wave_sum(s);
        if (lane == 0) cs[c] = s;
    }
    __syncthreads();
    if (wv != 0) return;

    ProbState &S = st[k];
    ProbScalars sc = S.sc;   // every lane works on a copy; lane 0 writes it back
    const bool in = lane < d;
    const int j = in ? lane : 0;
    const double C = sc.C;
    const double u = in ? ctl->vec[k][j] : 0.0;     // entry j of the vector the pass used
    const double o = in ? fma(C, cs[j], u) : 0.0;   // entry j of  v + C X^T(D(Xv))  or of  w + C X^T zhat
    Request next{MODE_IDLE, sc.dcur, 0.0};
    const double eta0 = 1e-4, eta1 = 0.25, eta2 = 0.75, sig2 = 0.5, sig3 = 4.0;
    const bool precond = P.blend > 0.0;
    // this lane's entry of the preconditioner; 1 without one (and past d), which leaves every product below unchanged
    double m = (precond && in && sc.phase != PH_ONESHOT) ? S.M[j] : 1.0;

    if (mode == MODE_DIAG) {
        // cs[j] = sum_i D_i x_ij^2 at the current iterate: M = (1 - a) + a (1 + C cs) = 1 + a C cs, then the inner solve starts
        m = in ? fma(P.blend * C, cs[j], 1.0) : 1.0;
        if (in) S.M[j] = m;
        const double g = in ? S.g[j] : 0.0;
        sc.gscaled = sqrt(dot64(g, g / m));
        if (sc.phase == PH_DIAG0) sc.delta = sc.gscaled;   // Delta_0 = sqrt(g.M^-1 g)
        next = cg_begin(S, sc, j, in, g, m);
    } else if (mode == MODE_HV) {
        const double pHp = dot64(u, o);
        if (sc.phase == PH_ONESHOT) {
            if (in) S.out[j] = o;
            sc.out_scal = pHp;
            sc.phase = PH_DONE;
        } else {   // PH_CG: u is the direction p
            double s = in ? S.s[j] : 0.0, r = in ? S.r[j] : 0.0;
            sc.cg_it += 1;
            sc.n_hv += 1;
            sc.cg_total += 1;
            const double alpha = sc.rr / pHp;
            const double pp = dot64(m * u, u), sp = dot64(m * s, u), ss = dot64(m * s, s);
            bool end = false;
            if (sqrt(ss + alpha * (2.0 * sp + alpha * pp)) >= sc.delta) {
                // to the boundary along p
                const double gap = sc.delta * sc.delta - ss;
                const double rad = sqrt(sp * sp + pp * gap);
                const double tau = (sp >= 0.0) ? gap / (sp + rad) : (rad - sp) / pp;
                s = fma(tau, u, s);
                r = fma(-tau, o, r);
                sc.onb = 1;
                end = true;
            } else {
                s = fma(alpha, u, s);
                r = fma(-alpha, o, r);
                const double zr = r / m;
                const double rr_new = dot64(r, zr);
                const double beta = rr_new / sc.rr;
                sc.rr = rr_new;
                if (sqrt(rr_new) <= P.xi * sc.gscaled || sc.cg_it >= P.max_cg) {
                    end = true;
                } else {
                    const double p = fma(beta, u, zr);
                    if (in) S.p[j] = p;
                    next = Request{MODE_HV, sc.dcur, p};
                }
            }
            if (in) {
                S.s[j] = s;
                S.r[j] = r;
            }
            if (end) next = cg_end(S, sc, j, in, s, r, m);
        }
    } else {   // MODE_FG: u is the point, o the gradient there
        const double f = 0.5 * dot64(u, u) + C * cs[d];
        const double gn = sqrt(dot64(o, o));
        if (sc.phase == PH_ONESHOT) {
            if (in) S.out[j] = o;
            sc.out_scal = f;
            sc.phase = PH_DONE;
        } else if (sc.phase == PH_REF) {
            // the gradient at w = 0 is the reference of the stopping test; now the starting point itself
            sc.gnorm0 = gn;
            sc.n_fun += 1;
            sc.n_grad += 1;
            sc.phase = PH_START;
            next = Request{MODE_FG, sc.dcur, in ? S.w[j] : 0.0};
        } else if (sc.phase == PH_START) {
            sc.f = f;
            sc.gnorm = gn;
            if (in) S.g[j] = o;
            sc.n_fun += 1;
            sc.n_grad += 1;
            if (sc.gnorm0 == 0.0) sc.gnorm0 = gn;
            sc.delta = gn;
            sc.gscaled = gn;
            if (gn <= P.eps * sc.gnorm0) finish(sc, TRON_OK);
            else if (precond) {   // the Hessian diagonal at this iterate first
                sc.phase = PH_DIAG0;
                next = Request{MODE_DIAG, sc.dcur, 0.0};
            } else next = cg_begin(S, sc, j, in, o, 1.0);
        } else {   // PH_TRIAL
            sc.n_fun += 1;
            const double ared = sc.f - f;
            const bool noise = fabs(ared) <= 1e-12 * fabs(sc.f) && sc.pred <= 1e-12 * fabs(sc.f);
            const double sigma = noise ? 1.0 : ared / sc.pred;
            const double gnorm_before = sc.gnorm;
            if (sigma < eta1) sc.delta = sig2 * fmin(sc.snorm, sc.delta);
            else if (sigma < eta2) { /* unchanged */ }
            else sc.delta = fmin(sig3 * sc.delta, fmax(sc.delta, sig3 * sc.snorm));
            const bool accepted = sigma > eta0;
            double g = in ? S.g[j] : 0.0;
            if (accepted) {
                if (in) {
                    S.w[j] = u;
                    S.g[j] = o;
                }
                g = o;
                sc.dcur = 1 - sc.dcur;   // the Hessian now uses D at the accepted point
                sc.f = f;
                sc.gnorm = gn;
                sc.gscaled = gn;
                sc.n_grad += 1;
            }
            sc.outer += 1;
            if (trace && sc.trace_len < P.trace_cap) {
                if (lane == 0) {
                    tron_trace_rec &t = trace[(int64_t)k * P.trace_cap + sc.trace_len];
                    t.iter = sc.outer; t.cg_iters = sc.cg_it; t.accepted = accepted ? 1 : 0; t.on_boundary = sc.onb;
                    t.f = sc.f; t.gnorm = sc.gnorm; t.delta = sc.delta; t.ared = ared; t.pred = sc.pred; t.snorm = sc.snorm;
                }
                sc.trace_len += 1;
            }
            if (accepted && sc.gnorm <= P.eps * sc.gnorm0) finish(sc, TRON_OK);
            else if (sc.pred <= 0.0 || (noise && sc.gnorm >= gnorm_before)) finish(sc, TRON_EMAXITER);
            else if (sc.outer >= P.max_outer) finish(sc, TRON_EMAXITER);
            else if (precond && accepted) {   // the iterate moved: its Hessian diagonal, then the inner solve
                sc.phase = PH_DIAG;
                next = Request{MODE_DIAG, sc.dcur, 0.0};
            } else next = cg_begin(S, sc, j, in, g, m);   // after a rejected step M and sqrt(g.M^-1 g) still hold
        }
    }
    if (lane < kVecPad) ctl->vec[k][lane] = in ? next.vec : 0.0;
    if (lane == 0) {
        ctl->mode[k] = next.mode;
        ctl->dslot[k] = next.slot;
        S.sc = sc;
    }
}

// First request of every problem.  what = BEGIN_SOLVE: state reset, w0 = IN[k]; when w0 is not zero the gradient at zero
// is evaluated first (it is the reference of the stopping test).  BEGIN_FG / BEGIN_HV: a single product with IN[k],
// using the problem's current D buffer.
__global__ __launch_bounds__(kWave) void k_batch_begin(int what, int64_t d, const double *__restrict__ IN, BatchC Cs,
                                                       BatchCtl *ctl, ProbState *st)
{
    const int k = blockIdx.x, lane = threadIdx.x;
    ProbState &S = st[k];
    const bool in = lane < d;
    const double x = in ? IN[(int64_t)k * d + lane] : 0.0;
    ProbScalars sc = S.sc;
    sc.C = Cs.v[k];
    Request next{MODE_IDLE, 0, 0.0};
    if (what == BEGIN_SOLVE) {
        sc.status = TRON_EMAXITER;
        sc.converged = sc.outer = sc.cg_total = sc.n_fun = sc.n_grad = sc.n_hv = sc.cg_it = sc.onb = sc.trace_len = 0;
        sc.dcur = 0;
        sc.f = sc.gnorm = sc.gnorm0 = sc.delta = sc.rr = sc.pred = sc.snorm = sc.out_scal = sc.gscaled = 0.0;
        if (in) S.w[lane] = x;
        const bool nonzero = __ballot(x != 0.0) != 0;
        sc.phase = nonzero ? PH_REF : PH_START;
        next = Request{MODE_FG, 0, nonzero ? 0.0 : x};
    } else {
        sc.phase = PH_ONESHOT;
        next = Request{what == BEGIN_FG ? MODE_FG : MODE_HV, sc.dcur, x};
    }
    if (lane < kVecPad) ctl->vec[k][lane] = in ? next.vec : 0.0;
    if (lane == 0) {
        ctl->mode[k] = next.mode;
        ctl->dslot[k] = next.slot;
        S.sc = sc;
    }
}

// OUT[k*d + j] = entry j of problem k's iterate (which = 0) or of its last single product (which = 1)
__global__ __launch_bounds__(kWave) void k_batch_store(int which, int64_t d, const ProbState *__restrict__ st,
                                                       double *__restrict__ OUT)
{
    const int k = blockIdx.x, lane = threadIdx.x;
    if (lane < d) OUT[(int64_t)k * d + lane] = which ? st[k].out[lane] : st[k].w[lane];
}

// ------------------------------------------------------------------ kernel choice
using PassFn = void (*)(int64_t, int64_t, const double *, const int8_t *, const BatchCtl *, const uint64_t *,
                        const uint64_t *, uint64_t *, double *, int64_t, double *, int);

struct PassPair { PassFn fn[2]; };   // by loss

template <int E, int L, int KT>
PassPair pass_for(bool vec)
{
    constexpr int U = pick_U(E, L);
    if constexpr (E % 2 == 0) {
        if (vec) return {{k_batch_pass<E, L, U, true, KT, TRON_LOSS_LR>, k_batch_pass<E, L, U, true, KT, TRON_LOSS_L2SVM>}};
    }
    return {{k_batch_pass<E, L, U, false, KT, TRON_LOSS_LR>, k_batch_pass<E, L, U, false, KT, TRON_LOSS_L2SVM>}};
}

template <int KT>
PassPair pass_for_shape(const Shape &s, bool vec)
{
    switch (s.L * 16 + s.E) {
    case 16 + 1: return pass_for<1, 1, KT>(vec);
    case 16 + 2: return pass_for<2, 1, KT>(vec);
    case 16 + 3: return pass_for<3, 1, KT>(vec);
    case 16 + 4: return pass_for<4, 1, KT>(vec);
    case 16 + 5: return pass_for<5, 1, KT>(vec);
    case 16 + 6: return pass_for<6, 1, KT>(vec);
    case 16 + 7: return pass_for<7, 1, KT>(vec);
    case 16 + 8: return pass_for<8, 1, KT>(vec);
    case 32 + 5: return pass_for<5, 2, KT>(vec);
    case 32 + 6: return pass_for<6, 2, KT>(vec);
    case 32 + 7: return pass_for<7, 2, KT>(vec);
    case 32 + 8: return pass_for<8, 2, KT>(vec);
    case 64 + 5: return pass_for<5, 4, KT>(vec);
    case 64 + 6: return pass_for<6, 4, KT>(vec);
    case 64 + 7: return pass_for<7, 4, KT>(vec);
    case 64 + 8: return pass_for<8, 4, KT>(vec);
    default: return {{nullptr, nullptr}};
    }
}

template <int DMAX, int KT, int RT, bool FG>
PassPair mfma_pass_pair(bool vec)
{
    if (vec) return {{k_batch_pass_mfma<true, DMAX, KT, TRON_LOSS_LR, RT, FG>, k_batch_pass_mfma<true, DMAX, KT, TRON_LOSS_L2SVM, RT, FG>}};
    return {{k_batch_pass_mfma<false, DMAX, KT, TRON_LOSS_LR, RT, FG>, k_batch_pass_mfma<false, DMAX, KT, TRON_LOSS_L2SVM, RT, FG>}};
}

template <int KT, int RT, bool FG>
PassPair mfma_pass_for(int64_t d)
{
    const bool vec = d % 2 == 0;
    if (d <= 16) return mfma_pass_pair<16, KT, RT, FG>(vec);
    if (d <= 24) return mfma_pass_pair<24, KT, RT, FG>(vec);
    return mfma_pass_pair<32, KT, RT, FG>(vec);
}

template <bool FG>
PassPair mfma_pass_select(int KT, int rt, int64_t d)
{
    if (rt == 64) return (KT == 8) ? mfma_pass_for<8, 64, FG>(d) : mfma_pass_for<16, 64, FG>(d);
    return (KT == 8) ? mfma_pass_for<8, 32, FG>(d) : mfma_pass_for<16, 32, FG>(d);
}

}  // namespace
}  // namespace tron

// ------------------------------------------------------------------ the handle
struct tron_batch {
    tron_dataset *ds = nullptr;
    int K = 0, KT = 0;
    int64_t ntiles = 0;
    uint64_t *member = nullptr;   // K planes of ntiles words
    uint64_t *Dbits = nullptr;    // K x 2 planes (L2-SVM active sets)
    double *Dval = nullptr;       // K x 2 x n (logistic D), allocated at the first logistic call
    tron::BatchCtl *ctl = nullptr;
    tron::ProbState *st = nullptr;
    tron::ProbState *st_host = nullptr;   // pinned
    int32_t *mode_host = nullptr;         // pinned, kBatchMax
    tron_trace_rec *trace = nullptr;      // device, K * trace_cap
    int trace_cap = 0;
    double *partials = nullptr;           // K x (d+1) x grid
    tron::PassPair pass{{nullptr, nullptr}};
    size_t pass_lds[2] = {0, 0};          // dynamic LDS of the pass kernel per loss (the matrix-unit pass; 0 otherwise)
    // the matrix-unit pass for rounds in which no problem asks for function and gradient (null: none), with its own
    // dynamic LDS and number of resident workgroups per loss; grid_used = the workgroups of the pass launched last
    tron::PassPair pass_nofg{{nullptr, nullptr}};
    size_t pass_nofg_lds[2] = {0, 0};
    int grid_nofg[2] = {0, 0};
    int grid_pass[2] = {0, 0};            // workgroups of pass.fn per loss
    bool on_matrix_units[2] = {false, false};   // per loss: pass.fn is the matrix-unit kernel
    int grid_used = 0;
    int D_loss = -1;                      // loss whose D the buffers hold (-1: none)
};

namespace tron {
namespace {

// no_fg: the caller knows that no problem is in MODE_FG in this round
int launch_pass(tron_batch *b, int loss, bool no_fg = false)
{
    tron_dataset *ds = b->ds;
    ProfScope ps(ds, SLOT_BATCH_PASS);
    const int li = loss == TRON_LOSS_L2SVM ? 1 : 0;
    const bool lean = no_fg && b->pass_nofg.fn[li] != nullptr;
    const PassFn fn = lean ? b->pass_nofg.fn[li] : b->pass.fn[li];
    const size_t lds = lean ? b->pass_nofg_lds[li] : b->pass_lds[li];
    b->grid_used = lean ? b->grid_nofg[li] : b->grid_pass[li];
    int64_t n = ds->n, d = ds->d, ntiles = b->ntiles;
    const double *X = ds->X;
    const int8_t *y = ds->y8;
    const BatchCtl *ctl = b->ctl;
    const uint64_t *member = b->member, *Din = b->Dbits;
    uint64_t *Dout = b->Dbits;
    double *Dval = b->Dval, *partials = b->partials;
    int K = b->K;
    void *args[] = {&n, &d, &X, &y, &ctl, &member, &Din, &Dout, &Dval, &ntiles, &partials, &K};
    TRON_HIP(hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3(b->grid_used), dim3(kBlock), args, lds, ds->stream));
    return TRON_OK;
}

int launch_advance(tron_batch *b, const SolveParams &P)
{
    tron_dataset *ds = b->ds;
    ProfScope ps(ds, SLOT_BATCH_ADVANCE);
    hipLaunchKernelGGL(k_batch_advance, dim3(b->K), dim3(kAdvanceBlock), 0, ds->stream, ds->d, b->grid_used, b->partials, b->ctl, b->st, P,
                       P.trace_cap > 0 ? b->trace : nullptr);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

int launch_begin(tron_batch *b, int what, const double *IN, const double *C_host)
{
    BatchC Cs;
    for (int k = 0; k < kBatchMax; ++k) Cs.v[k] = (k < b->K) ? C_host[k] : 1.0;
    ProfScope ps(b->ds, SLOT_BATCH_ADVANCE);
    hipLaunchKernelGGL(k_batch_begin, dim3(b->K), dim3(kWave), 0, b->ds->stream, what, b->ds->d, IN, Cs, b->ctl, b->st);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

int ensure_D(tron_batch *b, int loss)
{
    if (loss == TRON_LOSS_LR && !b->Dval) {
        // zero once: a pass only ever writes D of a problem's own rows, the others stay zero
        const size_t bytes = sizeof(double) * 2 * (size_t)b->K * (size_t)b->ds->n;
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&b->Dval), bytes));
        TRON_HIP(hipMemsetAsync(b->Dval, 0, bytes, b->ds->stream));
    }
    return TRON_OK;
}

bool bad_C(const tron_batch *b, const double *C_host)
{
    for (int k = 0; k < b->K; ++k)
        if (!(C_host[k] > 0.0) || !std::isfinite(C_host[k])) return true;
    return false;
}

// one single product for every problem: begin, pass, advance, results to OUT (K*d) and scal_host (K)
int one_shot(tron_batch *b, int what, int loss, const double *C_host, const double *IN, double *OUT, double *scal_host)
{
    tron_dataset *ds = b->ds;
    SolveParams P{};
    P.loss = loss;
    TRON_TRY(launch_begin(b, what, IN, C_host));
    TRON_TRY(launch_pass(b, loss, what == BEGIN_HV));
    TRON_TRY(launch_advance(b, P));
    if (OUT) {
        hipLaunchKernelGGL(k_batch_store, dim3(b->K), dim3(kWave), 0, ds->stream, 1, ds->d, b->st, OUT);
        TRON_HIP(hipGetLastError());
    }
    TRON_HIP(hipMemcpyAsync(b->st_host, b->st, sizeof(ProbState) * b->K, hipMemcpyDeviceToHost, ds->stream));
    TRON_HIP(hipStreamSynchronize(ds->stream));
    if (scal_host)
        for (int k = 0; k < b->K; ++k) scal_host[k] = b->st_host[k].sc.out_scal;
    return TRON_OK;
}

}  // namespace
}  // namespace tron

using namespace tron;

extern "C" void tron_batch_destroy(tron_batch *b)
{
    if (!b) return;
    if (b->ds) hipStreamSynchronize(b->ds->stream);
    hipFree(b->member); hipFree(b->Dbits); hipFree(b->Dval); hipFree(b->ctl); hipFree(b->st); hipFree(b->trace); hipFree(b->partials);
    if (b->st_host) hipHostFree(b->st_host);
    if (b->mode_host) hipHostFree(b->mode_host);
    delete b;
}

// member == null: every row belongs to every problem
static int batch_create_impl(tron_dataset *ds, int K, const uint32_t *member, int mem, tron_batch **out)
{
    *out = nullptr;
    if (!ds->dense || ds->d > kVecPad) {
        set_error("tron_batch_create: needs a dense dataset with d <= %d", kVecPad);
        return TRON_EINVAL;
    }
    const int64_t n = ds->n, d = ds->d;
    if (member && mem == TRON_MEM_HOST && K < 32)
        for (int64_t i = 0; i < n; ++i)
            if ((member[i] >> K) != 0u) { set_error("tron_batch_create: member[%lld] has a bit at or above K", (long long)i); return TRON_EINVAL; }
    Shape s;
    if (!pick_shape(d, s) || s.L > 4) { set_error("tron_batch_create: internal: no tile shape for d = %lld", (long long)d); return TRON_EINVAL; }
    tron_batch *b = new (std::nothrow) tron_batch();
    if (!b) { set_error("out of host memory"); return TRON_ENOMEM; }
    b->ds = ds;
    b->K = K;
    b->KT = (K <= 4) ? 4 : 8;
    b->ntiles = (n + kWave - 1) / kWave;
    const bool vec = (s.E % 2 == 0) && (d % 2 == 0);
    // up to 8 problems: the pass on the vector units (4 or 8 problem slots), unless the matrix units take it (below)
    b->pass = (b->KT == 4) ? pass_for_shape<4>(s, vec) : pass_for_shape<8>(s, vec);
    auto fail = [&](int rc) { tron_batch_destroy(b); return rc; };
#define TRON_B(expr) do { hipError_t e__ = (expr); if (e__ != hipSuccess) return fail(hip_fail(e__, #expr, __FILE__, __LINE__)); } while (0)
    if (!b->pass.fn[0]) { set_error("tron_batch_create: internal: no kernel for E=%d L=%d", s.E, s.L); return fail(TRON_EINVAL); }
    // The pass as matrix instructions (8 or 16 problem columns; the tile of X of every wavefront in LDS, and where logistic
    // function / gradient requests are served the exchange area), chosen per loss: above eight problems always; otherwise
    // where it is the faster one (measured at 20M x 24: the L2-SVM from eight problems on, the logistic loss -- whose
    // vector kernel evaluates every problem's terms in every lane and spills -- from five).
    const int mfma_from[2] = {5, 8};   // logistic, L2-SVM
    const int dmax = d <= 16 ? 16 : (d <= 24 ? 24 : 32);
    const size_t floor_lds = sizeof(double) * kWavesPerBlock * 32 * 16;   // the final sums of the four wavefronts
    const int KTm = (K <= 8) ? 8 : 16;
    for (int l = 0; l < 2; ++l) {
        b->on_matrix_units[l] = K > 8 || g_tuning.batch_mfma > 0 || (g_tuning.batch_mfma < 0 && K >= mfma_from[l]);
        if (!b->on_matrix_units[l]) continue;
        // half tiles (measured: as fast or faster than whole tiles for both losses, 3 to 12% at 12 problems)
        const int rt = g_tuning.batch_mfma_rows != 0 ? (int)g_tuning.batch_mfma_rows : 32;
        b->pass.fn[l] = mfma_pass_select<true>(KTm, rt, d).fn[l];
        b->pass_lds[l] = sizeof(double) * kWavesPerBlock * (size_t)mfma_wave_doubles(dmax, l == 0 ? K : 0, rt);
        if (b->pass_lds[l] < floor_lds) b->pass_lds[l] = floor_lds;
        TRON_B(hipFuncSetAttribute(reinterpret_cast<const void *>(b->pass.fn[l]), hipFuncAttributeMaxDynamicSharedMemorySize, (int)b->pass_lds[l]));
        if (g_tuning.batch_lean != 0) {
            // rounds without function / gradient requests: three or four wavefronts per SIMD; whole tiles for the L2-SVM,
            // half tiles for the logistic loss (measured: 3% either way)
            const int rt_lean = g_tuning.batch_mfma_rows != 0 ? (int)g_tuning.batch_mfma_rows : (l == 1 ? 64 : 32);
            b->pass_nofg.fn[l] = mfma_pass_select<false>(KTm, rt_lean, d).fn[l];
            b->pass_nofg_lds[l] = sizeof(double) * kWavesPerBlock * (size_t)mfma_wave_doubles(dmax, 0, rt_lean);
            if (b->pass_nofg_lds[l] < floor_lds) b->pass_nofg_lds[l] = floor_lds;
            TRON_B(hipFuncSetAttribute(reinterpret_cast<const void *>(b->pass_nofg.fn[l]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)b->pass_nofg_lds[l]));
        }
    }
    // resident workgroups of a pass: all of them hold their accumulators for the whole pass
    int cus = 0;
    TRON_B(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ds->device));
    const int64_t by_tiles = (b->ntiles + kWavesPerBlock - 1) / kWavesPerBlock;
    auto resident = [&](PassFn fn, size_t lds, int *out) -> int {
        int pc = 0;
        const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&pc, reinterpret_cast<const void *>(fn), kBlock, lds);
        if (e != hipSuccess) return hip_fail(e, "hipOccupancyMaxActiveBlocksPerMultiprocessor", __FILE__, __LINE__);
        int64_t gl = (int64_t)cus * (pc < 1 ? 1 : pc);
        if (g_tuning.batch_grid > 0) gl = g_tuning.batch_grid;
        if (gl > by_tiles) gl = by_tiles;
        if (gl < 1) gl = 1;
        *out = (int)gl;
        return TRON_OK;
    };
    int64_t grid_max = 1;
    for (int l = 0; l < 2; ++l) {
        int rc = resident(b->pass.fn[l], b->pass_lds[l], &b->grid_pass[l]);
        if (rc == TRON_OK && b->pass_nofg.fn[l]) rc = resident(b->pass_nofg.fn[l], b->pass_nofg_lds[l], &b->grid_nofg[l]);
        if (rc != TRON_OK) return fail(rc);
        if (b->grid_pass[l] > grid_max) grid_max = b->grid_pass[l];
        if (b->grid_nofg[l] > grid_max) grid_max = b->grid_nofg[l];
    }
    if (!b->on_matrix_units[0] && !b->on_matrix_units[1]) {
        // the two vector kernels share one grid (the larger residency), as they always have
        b->grid_pass[0] = b->grid_pass[1] = (int)grid_max;
    }
    b->grid_used = b->grid_pass[1];
    TRON_B(hipMalloc(reinterpret_cast<void **>(&b->member), sizeof(uint64_t) * (size_t)K * (size_t)b->ntiles));
    TRON_B(hipMalloc(reinterpret_cast<void **>(&b->Dbits), sizeof(uint64_t) * 2 * (size_t)K * (size_t)b->ntiles));
    TRON_B(hipMalloc(reinterpret_cast<void **>(&b->ctl), sizeof(BatchCtl)));
    TRON_B(hipMalloc(reinterpret_cast<void **>(&b->st), sizeof(ProbState) * kBatchMax));
    TRON_B(hipMalloc(reinterpret_cast<void **>(&b->partials), sizeof(double) * (size_t)K * (size_t)(d + 1) * (size_t)grid_max));
    TRON_B(hipHostMalloc(reinterpret_cast<void **>(&b->st_host), sizeof(ProbState) * kBatchMax, hipHostMallocDefault));
    TRON_B(hipHostMalloc(reinterpret_cast<void **>(&b->mode_host), sizeof(int32_t) * (kBatchMax + 1), hipHostMallocDefault));
    TRON_B(hipMemsetAsync(b->ctl, 0, sizeof(BatchCtl), ds->stream));
    TRON_B(hipMemsetAsync(b->st, 0, sizeof(ProbState) * kBatchMax, ds->stream));
    TRON_B(hipMemsetAsync(b->Dbits, 0, sizeof(uint64_t) * 2 * (size_t)K * (size_t)b->ntiles, ds->stream));
    // membership words; a device-side check of the unused bits for device input
    uint32_t *staged = nullptr;
    int *bad = nullptr;
    TRON_B(hipMalloc(reinterpret_cast<void **>(&bad), sizeof(int)));
    hipError_t e = hipMemsetAsync(bad, 0, sizeof(int), ds->stream);
    const uint32_t *src = member;
    if (e == hipSuccess && member && mem == TRON_MEM_HOST) {
        e = hipMalloc(reinterpret_cast<void **>(&staged), sizeof(uint32_t) * (size_t)n);
        if (e == hipSuccess) e = hipMemcpyAsync(staged, member, sizeof(uint32_t) * (size_t)n, hipMemcpyHostToDevice, ds->stream);
        src = staged;
    }
    int bad_host = 0;
    if (e == hipSuccess) {
        int64_t g = (b->ntiles + kWavesPerBlock - 1) / kWavesPerBlock;
        if (g > kMaxGrid) g = kMaxGrid;
        hipLaunchKernelGGL(k_member_planes, dim3((int)g), dim3(kBlock), 0, ds->stream, n, K, src, b->ntiles, b->member, bad);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&bad_host, bad, sizeof(int), hipMemcpyDeviceToHost, ds->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ds->stream);
    hipFree(staged);
    hipFree(bad);
    if (e != hipSuccess) return fail(hip_fail(e, "membership words", __FILE__, __LINE__));
    if (bad_host) { set_error("tron_batch_create: a member word has a bit at or above K"); return fail(TRON_EINVAL); }
#undef TRON_B
    *out = b;
    return TRON_OK;
}

extern "C" int tron_batch_create(tron_dataset *ds, int K, const uint32_t *member, int mem, tron_batch **out)
{
    if (out) *out = nullptr;
    if (!ds || !out || !member || K < 1 || K > kBatchMax || (mem != TRON_MEM_HOST && mem != TRON_MEM_DEVICE)) {
        set_error("tron_batch_create: bad argument (need a handle, 1 <= K <= %d, member, mem in {0,1}, out)", kBatchMax);
        return TRON_EINVAL;
    }
    return batch_create_impl(ds, K, member, mem, out);
}

extern "C" int tron_batch_fun_grad(tron_batch *b, int loss, const double *C_host, const double *W_dev, double *f_host,
                                   double *G_dev)
{
    if (!b || !C_host || !W_dev || !f_host || (loss != TRON_LOSS_LR && loss != TRON_LOSS_L2SVM) || bad_C(b, C_host)) {
        set_error("tron_batch_fun_grad: bad argument (null batch/C/W/f, unknown loss, or some C <= 0)");
        return TRON_EINVAL;
    }
    TRON_TRY(ensure_D(b, loss));
    TRON_TRY(one_shot(b, BEGIN_FG, loss, C_host, W_dev, G_dev, f_host));
    b->D_loss = loss;
    return TRON_OK;
}

extern "C" int tron_batch_hv(tron_batch *b, const double *C_host, const double *V_dev, double *HV_dev, double *vHv_host)
{
    if (!b || !C_host || !V_dev || !HV_dev || V_dev == HV_dev || bad_C(b, C_host)) {
        set_error("tron_batch_hv: bad argument (null batch/C/V/HV, V aliases HV, or some C <= 0)");
        return TRON_EINVAL;
    }
    if (b->D_loss < 0) { set_error("tron_batch_hv: no cached D; call tron_batch_fun_grad first"); return TRON_ESTATE; }
    return one_shot(b, BEGIN_HV, b->D_loss, C_host, V_dev, HV_dev, vHv_host);
}

extern "C" int tron_batch_solve(tron_batch *b, const tron_params *params, const double *C_host, double *W_dev,
                                tron_result *res, int *status_host)
{
    if (!b || !params || !C_host || !W_dev || !res) { set_error("tron_batch_solve: null argument"); return TRON_EINVAL; }
    const tron_params &Q = *params;
    if ((Q.loss != TRON_LOSS_LR && Q.loss != TRON_LOSS_L2SVM) || bad_C(b, C_host) || !(Q.eps > 0.0) || Q.max_outer < 1 ||
        Q.max_cg < 1 || !(Q.cg_xi > 0.0) || !(Q.cg_xi < 1.0) || !(Q.precond_blend >= 0.0) || !(Q.precond_blend <= 1.0)) {
        set_error("tron_batch_solve: bad parameter (loss, every C > 0, eps > 0, max_outer >= 1, max_cg >= 1, 0 < cg_xi < 1, "
                  "0 <= precond_blend <= 1)");
        return TRON_EINVAL;
    }
    int cap = 0;
    for (int k = 0; k < b->K; ++k) {
        if (res[k].trace_cap < 0 || (res[k].trace_cap > 0 && !res[k].trace)) { set_error("tron_batch_solve: bad trace of problem %d", k); return TRON_EINVAL; }
        if (res[k].trace_cap > cap) cap = res[k].trace_cap;
    }
    tron_dataset *ds = b->ds;
    TRON_TRY(ensure_D(b, Q.loss));
    if (cap > b->trace_cap) {
        hipFree(b->trace);
        b->trace = nullptr;
        b->trace_cap = 0;
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&b->trace), sizeof(tron_trace_rec) * (size_t)b->K * (size_t)cap));
        b->trace_cap = cap;
    }
    SolveParams P{Q.loss, Q.max_outer, Q.max_cg, cap, Q.eps, Q.cg_xi, Q.precond_blend};
    b->D_loss = -1;
    TRON_TRY(launch_begin(b, BEGIN_SOLVE, W_dev, C_host));
    // A problem needs at most 3 + max_outer (max_cg + 2) rounds (one more per iterate with a preconditioner).  The host looks at the modes every `poll` rounds; a
    // pass that finds every problem idle returns at once.
    const int64_t round_cap = 3 + (int64_t)Q.max_outer * ((int64_t)Q.max_cg + 2);
    const double pass_bytes = (double)ds->n * (double)ds->d * 8.0;
    const int poll = pass_bytes < 4e8 ? 4 : 1;
    bool live = true;
    bool no_fg = false;   // known only right after the host has looked: the first round of a group of `poll`
    for (int64_t round = 0; live && round < round_cap + poll; round += poll) {
        for (int i = 0; i < poll; ++i) {
            TRON_TRY(launch_pass(b, Q.loss, i == 0 && no_fg));
            TRON_TRY(launch_advance(b, P));
        }
        TRON_HIP(hipMemcpyAsync(b->mode_host, b->ctl->mode, sizeof(int32_t) * kBatchMax, hipMemcpyDeviceToHost, ds->stream));
        TRON_HIP(hipStreamSynchronize(ds->stream));
        live = false;
        no_fg = true;
        for (int k = 0; k < b->K; ++k) {
            live |= b->mode_host[k] != MODE_IDLE;
            no_fg = no_fg && b->mode_host[k] != MODE_FG;
        }
    }
    if (live) { set_error("tron_batch_solve: internal: problems still running after the round limit"); return TRON_ESTATE; }
    hipLaunchKernelGGL(k_batch_store, dim3(b->K), dim3(kWave), 0, ds->stream, 0, ds->d, b->st, W_dev);
    TRON_HIP(hipGetLastError());
    TRON_HIP(hipMemcpyAsync(b->st_host, b->st, sizeof(ProbState) * b->K, hipMemcpyDeviceToHost, ds->stream));
    TRON_HIP(hipStreamSynchronize(ds->stream));
    int overall = TRON_OK;
    for (int k = 0; k < b->K; ++k) {
        const ProbScalars &sc = b->st_host[k].sc;
        tron_result &r = res[k];
        r.f = sc.f; r.gnorm = sc.gnorm; r.gnorm0 = sc.gnorm0;
        r.outer_iters = sc.outer; r.cg_iters_total = sc.cg_total; r.n_fun = sc.n_fun; r.n_grad = sc.n_grad; r.n_hv = sc.n_hv;
        r.converged = sc.converged;
        r.trace_len = sc.trace_len < r.trace_cap ? sc.trace_len : r.trace_cap;
        if (r.trace_len > 0)
            TRON_HIP(hipMemcpy(r.trace, b->trace + (size_t)k * cap, sizeof(tron_trace_rec) * r.trace_len, hipMemcpyDeviceToHost));
        if (status_host) status_host[k] = sc.status;
        if (sc.status != TRON_OK) overall = TRON_EMAXITER;
    }
    b->D_loss = Q.loss;
    return overall;
}

// ------------------------------------------------------------------ one problem, driven from the device
// tron_solve for a dense matrix with d <= 32 as a batch of one problem over all rows: the trust-region and CG steps run
// on the device between the passes, so no scalar is waited for by the host inside an iteration.  For matrices of a few
// GB and less that wait is most of a host-driven solve.
namespace tron {

int dense_device_solve(tron_dataset *ds, const tron_params &P, double *w_dev, tron_result *res)
{
    if (!ds->self_batch) TRON_TRY(batch_create_impl(ds, 1, nullptr, TRON_MEM_DEVICE, &ds->self_batch));
    tron_batch *b = ds->self_batch;
    const double C = P.C;
    int status = TRON_OK;
    TRON_TRY(tron_batch_solve(b, &P, &C, w_dev, res, &status));
    // D at the final iterate goes where the single-problem calls expect it (same layouts: one bit per row in 64-bit
    // words for the L2-SVM, fp64 per row for the logistic loss)
    const int slot = b->st_host[0].sc.dcur;
    if (P.loss == TRON_LOSS_L2SVM)
        TRON_HIP(hipMemcpyAsync(ds->Dbuf[0], b->Dbits + (size_t)slot * (size_t)b->ntiles, sizeof(uint64_t) * (size_t)b->ntiles,
                                hipMemcpyDeviceToDevice, ds->stream));
    else
        TRON_HIP(hipMemcpyAsync(ds->Dbuf[0], b->Dval + (size_t)slot * (size_t)ds->n, sizeof(double) * (size_t)ds->n,
                                hipMemcpyDeviceToDevice, ds->stream));
    TRON_HIP(hipStreamSynchronize(ds->stream));
    ds->Dcur = 0;
    ds->have_D = true;
    ds->D_is_mask[0] = (P.loss == TRON_LOSS_L2SVM);
    ds->active_frac[0] = 1.0;   // not counted here: the Hessian pass then reads every row, which is always right
    return status;
}

void dense_device_release(tron_dataset *ds)
{
    tron_batch_destroy(ds->self_batch);
    ds->self_batch = nullptr;
}

}  // namespace tron
