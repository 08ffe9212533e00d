// Dense row-major kernels: one pass over X computes both products of Table 1 of the paper,
//   Hessian-vector:  X^T ( D (X v) )        (written there as 2C X_I^T (X_I v) for the L2-SVM; the
//                                            active set enters through D_ii in {0, 2})
//   function/gradient:  z = X w, the per-instance loss, zhat and D, and X^T zhat
// so each element of X is read from HBM exactly once per call.
//
// Layout of the work inside a wavefront (64 lanes): a row is covered by L consecutive lanes, each
// holding E consecutive columns (E*L >= d); one "step" therefore covers 64/L rows and a wave tile of
// U steps covers RT = U*64/L consecutive rows.  For d = 24: E = 6, L = 4, U = 4 -- 64 rows = 12 KiB per
// tile, each lane issuing three 16-byte loads per step, twelve per tile, all in flight together.
//   1. partial dot products x.v per lane, butterfly over the L lanes of the row;
//   2. the RT row results are moved so that lane i owns row i of the tile: the per-row scalar work
//      (sigmoid / log1p for the logistic loss, D scaling) runs once per row, and D, y are read/written
//      as one coalesced 8-byte-per-lane access;
//   3. the per-row coefficient is broadcast back to the row's lanes and accumulated into E private
//      column accumulators, which are reduced over the wavefront / workgroup once, at the end.
// Workgroup partial column sums go to `partials[col * grid + block]`; a second kernel adds them in a
// fixed order (no atomics) and applies  out = add + C * sum  together with the dot products the
// trust-region driver needs.
#include <cmath>

#include "dense_tile.h"

namespace tron {

namespace {

// ------------------------------------------------------------------ Hessian-vector pass
// MASK: D is the active set of the L2-SVM (D_ii = 2 on it, else 0) instead of an fp64 value per row: one bit per row,
// a 64-bit word per wave tile, when a tile has 64 rows (d <= 32); one byte per row otherwise.
// DIAG: column sums of D_i x_ij^2 instead (the diagonal of X^T D X; v is not read).
// SKIP (with the bit words only): rows outside the active set are not read.  Chosen by the host when a noticeable
// part of the rows is inactive; with (almost) every row active the plain loop is about 1% faster.
template <int E, int L, int U, bool VEC, bool MASK, bool DIAG, bool SKIP>
__global__ __launch_bounds__(kBlock) void k_dense_hv(int64_t n, int64_t d, const double *__restrict__ X,
                                                     const void *__restrict__ Dv, const double *__restrict__ v,
                                                     double *__restrict__ partials)
{
    const double *D = static_cast<const double *>(Dv);
    const uint8_t *Dm = static_cast<const uint8_t *>(Dv);
    using T = Tile<E, L, U, VEC>;
    __shared__ double lds[kWavesPerBlock * E * L];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int q = lane % L;
    double vreg[E], acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        vreg[e] = (!DIAG && q * E + e < d) ? v[q * E + e] : 0.0;
        acc[e] = 0.0;
    }
    const int64_t ntiles = (n + T::RT - 1) / T::RT;
    const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
    // With the active set as one 64-bit word per tile (bit i = row row0 + i is active; rows past n are never set)
    // the rows outside it are not read: the pass moves 8 |I| d bytes, the saving the paper gets from a compacted
    // copy X_I (Section 5) without the copy.  The word of the next tile is fetched one iteration ahead.
    constexpr bool kBits = MASK && T::RT == kWave;
    const uint64_t *Dbits = static_cast<const uint64_t *>(Dv);
    const int64_t tile0 = (int64_t)blockIdx.x * kWavesPerBlock + wv;
    uint64_t bits_next = (kBits && SKIP && tile0 < ntiles) ? Dbits[tile0] : 0;
    for (int64_t tile = tile0; tile < ntiles; tile += nwaves) {
        const int64_t row0 = tile * T::RT;
        double x[U][E], t[U], c[U];
        uint64_t bits = 0;
        if (kBits && SKIP) {
            bits = bits_next;
            bits_next = (tile + nwaves < ntiles) ? Dbits[tile + nwaves] : 0;
            if (bits == 0) continue;   // no active row in the tile
        }
        T::load(X, n, d, row0, lane, x, (kBits && SKIP) ? bits : ~0ull);
        if (kBits && !SKIP) bits = Dbits[tile];
        double Drow = 0.0;
        if (kBits) {
            Drow = ((bits >> lane) & 1u) ? 2.0 : 0.0;
        } else if (lane < T::RT && row0 + lane < n) {
            Drow = MASK ? (Dm[row0 + lane] ? 2.0 : 0.0) : D[row0 + lane];
        }
        if (DIAG) {
            T::from_row_owner(Drow, lane, c);
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = fma(c[u] * x[u][e], x[u][e], acc[e]);
            }
        } else {
            T::row_dots(x, vreg, t);
            const double a1 = Drow * T::to_row_owner(t, lane);   // a1 = D (X v)
            T::from_row_owner(a1, lane, c);
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = fma(c[u], x[u][e], acc[e]);
            }
        }
    }
    T::flush(acc, d, lane, wv, lds, partials);
}

// ------------------------------------------------------------------ function / gradient pass
template <int E, int L, int U, bool VEC, int LOSS>
__global__ __launch_bounds__(kBlock) void k_dense_fun_grad(int64_t n, int64_t d, const double *__restrict__ X,
                                                           const int8_t *__restrict__ y, const double *__restrict__ w,
                                                           void *__restrict__ Dv, double *__restrict__ partials,
                                                           double *__restrict__ loss_partials, double *__restrict__ active_partials)
{
    double *Dout = static_cast<double *>(Dv);       // logistic loss: fp64 D
    uint8_t *Dmask = static_cast<uint8_t *>(Dv);    // L2-SVM: active-set mask
    using T = Tile<E, L, U, VEC>;
    __shared__ double lds[kWavesPerBlock * E * L];
    __shared__ double lds_red[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int q = lane % L;
    double wreg[E], acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        wreg[e] = (q * E + e < d) ? w[q * E + e] : 0.0;
        acc[e] = 0.0;
    }
    double loss_acc = 0.0, active_acc = 0.0;   // sum of the losses; number of rows with D != 0
    // D of a tile is stored only after the loads of the next tile have been issued: the memory counter retires in
    // order, so a store issued before them would have to complete before their data could be used.
    // Active set of the L2-SVM when a tile has 64 rows: one 64-bit word per tile.  A wavefront then walks a
    // contiguous range of tiles, lane i keeps the word of its i-th, 64+i-th, ... tile, and every 64 tiles the words
    // go out as one 512-byte store: small stores between the reads cost far more than their bytes.
    constexpr bool kBits = (LOSS == TRON_LOSS_L2SVM) && (T::RT == kWave);
    uint64_t *Dbits = static_cast<uint64_t *>(Dv);
    uint64_t held_bits = 0;
    int64_t held_tile = -1;
    const int64_t ntiles = (n + T::RT - 1) / T::RT;
    const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t wave_id = (int64_t)blockIdx.x * kWavesPerBlock + wv;
    const int64_t per_wave = (ntiles + nwaves - 1) / nwaves;
    // kBits: tiles [first, last) one after the other; otherwise tiles wave_id, wave_id + nwaves, ...
    const int64_t first = kBits ? wave_id * per_wave : wave_id;
    const int64_t last = kBits ? ((first + per_wave < ntiles) ? first + per_wave : ntiles) : ntiles;
    const int64_t step = kBits ? 1 : nwaves;
    int it = 0;
    for (int64_t tile = first; tile < last; tile += step, ++it) {
        const int64_t row0 = tile * T::RT;
        double x[U][E], t[U], c[U];
        T::load(X, n, d, row0, lane, x);
        const bool mine = lane < T::RT && row0 + lane < n;
        const double yrow = mine ? (double)y[row0 + lane] : 1.0;
        T::row_dots(x, wreg, t);
        const double z = T::to_row_owner(t, lane);            // z = X w
        double alpha, zhat, Di;
        loss_terms_dev<LOSS>(z, yrow, alpha, zhat, Di);
        if (mine) {
            loss_acc += alpha;
            active_acc += (Di != 0.0) ? 1.0 : 0.0;
        } else {
            Di = 0.0;
            zhat = 0.0;
        }
        if (kBits) {
            const uint64_t bits = __ballot(Di != 0.0);
            if (lane == (it & (kWave - 1))) { held_bits = bits; held_tile = tile; }
            if ((it & (kWave - 1)) == kWave - 1) {
                Dbits[held_tile] = held_bits;   // every lane holds one: 64 consecutive words
                held_tile = -1;
            }
        } else if (mine) {
            if (LOSS == TRON_LOSS_L2SVM) Dmask[row0 + lane] = (Di != 0.0) ? 1 : 0;
            else Dout[row0 + lane] = Di;
        }
        T::from_row_owner(zhat, lane, c);
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] = fma(c[u], x[u][e], acc[e]);
        }
    }
    if (kBits && held_tile >= 0) Dbits[held_tile] = held_bits;
    T::flush(acc, d, lane, wv, lds, partials);
    loss_acc = block_sum(loss_acc, lds_red);
    if (threadIdx.x == 0) loss_partials[blockIdx.x] = loss_acc;
    active_acc = block_sum(active_acc, lds_red);
    if (threadIdx.x == 0) active_partials[blockIdx.x] = active_acc;
}

// ------------------------------------------------------------------ second stage
// One wavefront per column: out[c] = add[c] + C * sum_b partials[c*grid + b]; colprod[c] = out[c]*dotw[c]
// (dotw = v for the Hessian-vector product, out itself for the gradient norm).
__global__ __launch_bounds__(kBlock) void k_dense_columns(int64_t d, int grid, const double *__restrict__ partials,
                                                          const double *__restrict__ add, double C, double *__restrict__ out,
                                                          const double *__restrict__ dotw, double *__restrict__ colprod)
{
    const int c = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (c >= d) return;
    const int lane = threadIdx.x & (kWave - 1);
    const double *p = partials + (int64_t)c * grid;
    double s = 0.0;
    for (int b = lane; b < grid; b += kWave) s += p[b];
    s = wave_sum(s);
    if (lane == 0) {
        const double o = fma(C, s, add ? add[c] : 1.0);
        if (out) out[c] = o;
        colprod[c] = o * (dotw ? dotw[c] : o);
    }
}

// scal[0] = sum loss partials (or v.Hv when nloss == 0: then scal[0] = sum colprod), scal[1] = w.w, scal[2] = sum colprod,
// scal[3] = sum of the active-row counts
__global__ __launch_bounds__(kBlock) void k_dense_scalars(int64_t d, int nloss, const double *__restrict__ loss_partials,
                                                          const double *__restrict__ active_partials,
                                                          const double *__restrict__ w, const double *__restrict__ colprod,
                                                          double *__restrict__ scal, double *__restrict__ scal_copy)
{
    __shared__ double lds[kWavesPerBlock];
    double a = 0.0, b = 0.0, c = 0.0, e = 0.0;
    for (int i = threadIdx.x; i < nloss; i += kBlock) {
        a += loss_partials[i];
        e += active_partials[i];
    }
    for (int64_t j = threadIdx.x; j < d; j += kBlock) {
        if (w) b += w[j] * w[j];
        c += colprod[j];
    }
    a = block_sum(a, lds);
    b = block_sum(b, lds);
    c = block_sum(c, lds);
    e = block_sum(e, lds);
    if (threadIdx.x == 0) {
        if (nloss > 0) {
            scal[0] = a;
            scal[1] = b;
            scal[2] = c;
            scal[3] = e;
        } else {
            scal[0] = c;
            scal_copy[0] = c;   // p.Hp: the CG step kernel continues from it
        }
    }
}

// Both second-stage kernels in one launch, for d <= kFinishMaxD: a single workgroup of 16 wavefronts; wavefront w adds the
// per-workgroup partial sums of columns w, w + 16, ... (sixteen loads per lane in flight at a time, added in index
// order), then the workgroup adds the column products and the other scalars.  Same outputs as k_dense_columns followed
// by k_dense_scalars; the launch and the wait between the two are saved, which is a third of a Hessian-vector call on a
// matrix of a million rows.
constexpr int kFinishMaxD = 64;
constexpr int kFinishWaves = 16;
__global__ __launch_bounds__(kFinishWaves * kWave) void k_dense_finish(int64_t d, int grid, const double *__restrict__ partials,
                                                                       const double *__restrict__ add, double C, double *__restrict__ out,
                                                                       const double *__restrict__ dotw, int nloss,
                                                                       const double *__restrict__ loss_partials,
                                                                       const double *__restrict__ active_partials,
                                                                       const double *__restrict__ w, double *__restrict__ scal,
                                                                       double *__restrict__ scal_copy)
{
    __shared__ double colprod[kFinishMaxD];
    __shared__ double red[4][kFinishWaves];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    for (int c = wv; c < d; c += kFinishWaves) {
        const double *p = partials + (int64_t)c * grid;
        double s = 0.0;
        for (int b0 = 0; b0 < grid; b0 += 16 * kWave) {
            double t[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int b = b0 + k * kWave + lane;
                t[k] = (b < grid) ? p[b] : 0.0;
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) s += t[k];
        }
        s = wave_sum(s);
        if (lane == 0) {
            const double o = fma(C, s, add ? add[c] : 1.0);
            if (out) out[c] = o;
            colprod[c] = o * (dotw ? dotw[c] : o);
        }
    }
    double a = 0.0, e = 0.0, ww = 0.0;
    for (int i = threadIdx.x; i < nloss; i += kFinishWaves * kWave) {
        a += loss_partials[i];
        e += active_partials[i];
    }
    if (w && threadIdx.x < d) ww = w[threadIdx.x] * w[threadIdx.x];
    __syncthreads();
    double cp = (threadIdx.x < d) ? colprod[threadIdx.x] : 0.0;   // d <= 64: all in wavefront 0
    a = wave_sum(a); e = wave_sum(e); ww = wave_sum(ww); cp = wave_sum(cp);
    if (lane == 0) { red[0][wv] = a; red[1][wv] = e; red[2][wv] = ww; red[3][wv] = cp; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double ta = 0.0, te = 0.0, tw = 0.0, tc = 0.0;
#pragma unroll
        for (int k = 0; k < kFinishWaves; ++k) { ta += red[0][k]; te += red[1][k]; tw += red[2][k]; tc += red[3][k]; }
        if (nloss > 0) {
            scal[0] = ta;
            scal[1] = tw;
            scal[2] = tc;
            scal[3] = te;
        } else {
            scal[0] = tc;
            scal_copy[0] = tc;   // p.Hp: the CG step kernel continues from it
        }
    }
}

// ------------------------------------------------------------------ dispatch
constexpr double kSkipBelow = 0.95;   // active fraction under which the Hessian-vector pass skips the inactive rows

// What a Hessian-vector pass runs over: the matrix itself with D of one buffer, or the compacted copy of its active rows
// (then every row is active: the bit words are all ones).
struct HvInput {
    const double *X;
    int64_t n;
    const void *D;
    bool mask, skip;
    int grid;
};

HvInput hv_input(const tron_dataset *ds, int Dslot)
{
    if (ds->hat_slot == Dslot && ds->Xhat)
        return HvInput{ds->Xhat, ds->hat_rows, ds->hat_bits, true, false, dense_grid_for(ds->hat_rows, ds->d)};
    const bool mask = ds->D_is_mask[Dslot];
    return HvInput{ds->X, ds->n, ds->Dbuf[Dslot], mask, mask && ds->active_frac[Dslot] < kSkipBelow, ds->dense_grid};
}

template <int E, int L>
int launch_hv(tron_dataset *ds, const HvInput &in, const double *v, double *partials)
{
    constexpr int U = pick_U(E, L);
    const bool vec = (E % 2 == 0) && (ds->d % 2 == 0);
    const int grid = in.grid;
    const void *D = in.D;
    const bool mask = in.mask, skip = in.skip;
#define TRON_HV(V, M, G, S) \
    hipLaunchKernelGGL((k_dense_hv<E, L, U, V, M, G, S>), dim3(grid), dim3(kBlock), 0, ds->stream, in.n, ds->d, in.X, D, v, partials)
#define TRON_HV_V(M, G, S) do { if (vec) TRON_HV((E % 2 == 0), M, G, S); else TRON_HV(false, M, G, S); } while (0)
    if (v) {
        if (!mask) TRON_HV_V(false, false, false);
        else if (skip) TRON_HV_V(true, false, true);
        else TRON_HV_V(true, false, false);
    } else {   // no vector: the diagonal sums
        if (!mask) TRON_HV_V(false, true, false);
        else if (skip) TRON_HV_V(true, true, true);
        else TRON_HV_V(true, true, false);
    }
#undef TRON_HV_V
#undef TRON_HV
    return TRON_OK;
}

template <int E, int L>
int launch_fg(tron_dataset *ds, int loss, const double *w, void *Dout, double *loss_partials, double *active_partials)
{
    constexpr int U = pick_U(E, L);
    const bool vec = (E % 2 == 0) && (ds->d % 2 == 0);
    const int grid = ds->dense_grid;
#define TRON_FG(V, LS) \
    hipLaunchKernelGGL((k_dense_fun_grad<E, L, U, V, LS>), dim3(grid), dim3(kBlock), 0, ds->stream, ds->n, ds->d, ds->X, ds->y8, w, Dout, ds->partials, loss_partials, active_partials)
    if (loss == TRON_LOSS_LR) {
        if (vec) TRON_FG((E % 2 == 0), TRON_LOSS_LR); else TRON_FG(false, TRON_LOSS_LR);
    } else {
        if (vec) TRON_FG((E % 2 == 0), TRON_LOSS_L2SVM); else TRON_FG(false, TRON_LOSS_L2SVM);
    }
#undef TRON_FG
    return TRON_OK;
}

// E in 1..8 for L = 1, E in 5..8 for L >= 2 (smaller d picks a smaller L)
#define TRON_DISPATCH_E(L_, FN, ...)                         \
    switch (s.E) {                                           \
    case 5: return FN<5, L_>(__VA_ARGS__);                   \
    case 6: return FN<6, L_>(__VA_ARGS__);                   \
    case 7: return FN<7, L_>(__VA_ARGS__);                   \
    case 8: return FN<8, L_>(__VA_ARGS__);                   \
    default: break;                                          \
    }

#define TRON_DISPATCH(FN, ...)                                                   \
    Shape s;                                                                     \
    if (!pick_shape(ds->d, s)) { set_error("dense d = %lld not supported (max 512)", (long long)ds->d); return TRON_EINVAL; } \
    switch (s.L) {                                                               \
    case 1:                                                                      \
        switch (s.E) {                                                           \
        case 1: return FN<1, 1>(__VA_ARGS__);                                    \
        case 2: return FN<2, 1>(__VA_ARGS__);                                    \
        case 3: return FN<3, 1>(__VA_ARGS__);                                    \
        case 4: return FN<4, 1>(__VA_ARGS__);                                    \
        default: break;                                                          \
        }                                                                        \
        TRON_DISPATCH_E(1, FN, __VA_ARGS__) break;                               \
    case 2: TRON_DISPATCH_E(2, FN, __VA_ARGS__) break;                           \
    case 4: TRON_DISPATCH_E(4, FN, __VA_ARGS__) break;                           \
    case 8: TRON_DISPATCH_E(8, FN, __VA_ARGS__) break;                           \
    case 16: TRON_DISPATCH_E(16, FN, __VA_ARGS__) break;                         \
    case 32: TRON_DISPATCH_E(32, FN, __VA_ARGS__) break;                         \
    case 64: TRON_DISPATCH_E(64, FN, __VA_ARGS__) break;                         \
    default: break;                                                              \
    }                                                                            \
    set_error("internal: no dense kernel for E=%d L=%d", s.E, s.L);              \
    return TRON_EINVAL;

int dispatch_hv(tron_dataset *ds, const HvInput &in, const double *v, double *partials) { TRON_DISPATCH(launch_hv, ds, in, v, partials) }
int dispatch_fg(tron_dataset *ds, int loss, const double *w, void *Dout, double *lp, double *ap) { TRON_DISPATCH(launch_fg, ds, loss, w, Dout, lp, ap) }

}  // namespace

__global__ __launch_bounds__(kBlock) void k_labels_to_int8(int64_t m, const double *__restrict__ y, int8_t *__restrict__ y8)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < m; i += (int64_t)gridDim.x * kBlock)
        y8[i] = (y[i] > 0.0) ? 1 : -1;
}

// Input check for rows handed over in device memory: flag[0] = 1 when a label is not exactly +1 or -1, flag[1] = 1 when
// an entry of X is not finite (every offending thread stores the same value).
__global__ __launch_bounds__(kBlock) void k_dense_validate(int64_t m, int64_t count, const double *__restrict__ X,
                                                           const double *__restrict__ y, double *__restrict__ flag)
{
    const int64_t t0 = (int64_t)blockIdx.x * kBlock + threadIdx.x, stride = (int64_t)gridDim.x * kBlock;
    bool bad_y = false, bad_x = false;
    for (int64_t i = t0; i < m; i += stride) bad_y |= !(y[i] == 1.0 || y[i] == -1.0);
    for (int64_t k = t0; k < count; k += stride) bad_x |= !isfinite(X[k]);
    if (bad_y) flag[0] = 1.0;
    if (bad_x) flag[1] = 1.0;
}

// what: 0 = fine, 1 = a label is not +1 / -1, 2 = a matrix entry is not finite.  Synchronises the stream.
int dense_validate_device(tron_dataset *ds, int64_t m, const double *X_dev, const double *y_dev, int *what)
{
    double *flag_host = ds->scal_host + kScalars - 2;   // the last two scalar slots: written by no other kernel
    flag_host[0] = 0.0;
    flag_host[1] = 0.0;
    int64_t g = (m * ds->d + kBlock * 8 - 1) / (kBlock * 8);
    if (g < 1) g = 1;
    if (g > kMaxGrid) g = kMaxGrid;
    hipLaunchKernelGGL(k_dense_validate, dim3((int)g), dim3(kBlock), 0, ds->stream, m, m * ds->d, X_dev, y_dev, ds->scal_dev + kScalars - 2);
    TRON_HIP(hipGetLastError());
    TRON_HIP(hipStreamSynchronize(ds->stream));
    *what = flag_host[0] != 0.0 ? 1 : (flag_host[1] != 0.0 ? 2 : 0);
    return TRON_OK;
}

int dense_labels_from_device(tron_dataset *ds, int64_t row0, int64_t m, const double *y_dev)
{
    int64_t g = (m + kBlock - 1) / kBlock;
    if (g > kMaxGrid) g = kMaxGrid;
    hipLaunchKernelGGL(k_labels_to_int8, dim3((int)g), dim3(kBlock), 0, ds->stream, m, y_dev, ds->y8 + row0);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

// ------------------------------------------------------------------ compacted copy of the active rows
// Section 5 of the paper keeps X_hat = X_{I,:} in device memory so that its matrix-vector products touch active rows
// only.  Here the copy is optional (the Hessian-vector pass over X skips inactive rows by itself): it pays when many
// products follow at one iterate with a small active set, because a pass over contiguous rows streams faster than one
// that picks 192-byte rows out of X.  Built on the device from the bit words the function/gradient pass left:
//   1. active rows before every 64-row tile: popcounts, scanned in three steps (per workgroup, over the workgroups, back);
//   2. every wavefront copies the active rows of its tiles to their places in X_hat (reads of inactive rows are not issued);
//   3. the active set of the copy is all ones.
constexpr int kScanPer = 4;                                   // tiles per thread in the scan
constexpr int kScanTile = kBlock * kScanPer;                  // tiles per workgroup

__global__ __launch_bounds__(kBlock) void k_active_block_sums(int64_t ntiles, const uint64_t *__restrict__ bits, int64_t *__restrict__ block_sums)
{
    __shared__ double lds[kWavesPerBlock];
    const int64_t t0 = (int64_t)blockIdx.x * kScanTile + threadIdx.x * kScanPer;
    int c = 0;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k)
        if (t0 + k < ntiles) c += __popcll(bits[t0 + k]);
    const double s = block_sum((double)c, lds);   // exact: at most 2^18 per workgroup
    if (threadIdx.x == 0) block_sums[blockIdx.x] = (int64_t)s;
}

// exclusive scan of the workgroup sums, in place, by one workgroup (thread t owns a contiguous run of them)
__global__ __launch_bounds__(kBlock) void k_active_scan_blocks(int nblocks, int64_t *__restrict__ block_sums)
{
    __shared__ int64_t run[kBlock];
    const int per = (nblocks + kBlock - 1) / kBlock;
    const int b0 = threadIdx.x * per, b1 = (b0 + per < nblocks) ? b0 + per : nblocks;
    int64_t s = 0;
    for (int b = b0; b < b1; ++b) s += block_sums[b];
    run[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t acc = 0;
        for (int t = 0; t < kBlock; ++t) { const int64_t v = run[t]; run[t] = acc; acc += v; }
    }
    __syncthreads();
    int64_t acc = run[threadIdx.x];
    for (int b = b0; b < b1; ++b) { const int64_t v = block_sums[b]; block_sums[b] = acc; acc += v; }
}

__global__ __launch_bounds__(kBlock) void k_active_tile_offsets(int64_t ntiles, const uint64_t *__restrict__ bits,
                                                                const int64_t *__restrict__ block_sums, int64_t *__restrict__ tile_off)
{
    __shared__ int wave_tot[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int64_t t0 = (int64_t)blockIdx.x * kScanTile + threadIdx.x * kScanPer;
    int c[kScanPer], mine = 0;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k) {
        c[k] = (t0 + k < ntiles) ? __popcll(bits[t0 + k]) : 0;
        mine += c[k];
    }
    const int incl = wave_scan_add(mine);
    if (lane == kWave - 1) wave_tot[wv] = incl;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wv; ++w) before += wave_tot[w];
    int64_t off = block_sums[blockIdx.x] + before + incl - mine;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k) {
        if (t0 + k < ntiles) tile_off[t0 + k] = off;
        off += c[k];
    }
}

// VEC: d is even, rows are moved in 16-byte pieces
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_compact_rows(int64_t n, int d, uint64_t inv_d, const double *__restrict__ X,
                                                         const uint64_t *__restrict__ bits, const int64_t *__restrict__ tile_off,
                                                         double *__restrict__ Xhat)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t ntiles = (n + kWave - 1) / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
    constexpr int W = VEC ? 2 : 1;
    for (int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; tile < ntiles; tile += nwaves) {
        const uint64_t b = bits[tile];   // rows past n are never set
        if (b == 0) continue;
        const double *src = X + tile * kWave * d;
        double *dst = Xhat + tile_off[tile] * d;
        const int total = kWave * d;
        for (int e = lane * W; e < total; e += kWave * W) {
            const int row = (int)(((uint64_t)e * inv_d) >> 32);   // e / d, exact for e < 64 * 32 (inv_d = ceil(2^32 / d))
            if ((b >> row) & 1u) {
                const int rank = __popcll(b & ((1ull << row) - 1ull));
                const int col = e - row * d;
                if (VEC) *reinterpret_cast<double2 *>(dst + rank * d + col) = *reinterpret_cast<const double2 *>(src + e);
                else dst[rank * d + col] = src[e];
            }
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_all_active_bits(int64_t rows, uint64_t *__restrict__ bits)
{
    const int64_t words = (rows + kWave - 1) / kWave;
    for (int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x; t < words; t += (int64_t)gridDim.x * kBlock) {
        const int64_t left = rows - t * kWave;
        bits[t] = (left >= kWave) ? ~0ull : ((1ull << left) - 1ull);
    }
}

bool dense_compact_wanted(const tron_dataset *ds, int Dslot, int recent_cg_iters)
{
    if (!ds->dense || ds->d > 32 || !ds->D_is_mask[Dslot] || g_tuning.dense_compact == 0) return false;
    if (ds->active_count[Dslot] <= 0 || ds->active_frac[Dslot] >= kSkipBelow) return false;
    if (g_tuning.dense_compact > 0) return true;
    // Building the copy costs about as much as 2.5 products over it and a product over it saves about a quarter of the
    // row-skipping one: worth it from about ten products per iterate on, with no more than 60% of the rows active.
    return ds->active_frac[Dslot] <= 0.6 && recent_cg_iters >= 10;
}

int dense_compact_build(tron_dataset *ds, int Dslot)
{
    if (!ds->dense || ds->d > 32 || !ds->D_is_mask[Dslot]) { set_error("internal: no bit-word active set to compact"); return TRON_EINVAL; }
    const int64_t rows = ds->active_count[Dslot];
    const int64_t ntiles = (ds->n + kWave - 1) / kWave;
    const int nblocks = (int)((ntiles + kScanTile - 1) / kScanTile);
    ds->hat_slot = -1;
    if (!ds->tile_off) {
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->tile_off), sizeof(int64_t) * (size_t)(ntiles + 1)));
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->scan_blocks), sizeof(int64_t) * (size_t)(nblocks + 1)));
    }
    if (rows > ds->hat_cap) {
        // grow with some room, so that a slowly growing active set does not reallocate at every iterate
        TRON_HIP(hipStreamSynchronize(ds->stream));
        hipFree(ds->Xhat); hipFree(ds->hat_bits);
        ds->Xhat = nullptr; ds->hat_bits = nullptr; ds->hat_cap = 0;
        int64_t cap = rows + rows / 8 + 1024;
        if (cap > ds->n) cap = ds->n;
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->Xhat), sizeof(double) * (size_t)cap * (size_t)ds->d));
        TRON_HIP(hipMalloc(reinterpret_cast<void **>(&ds->hat_bits), sizeof(uint64_t) * (size_t)(cap / kWave + 1)));
        ds->hat_cap = cap;
    }
    ProfScope ps(ds, SLOT_DENSE_COMPACT);
    const uint64_t *bits = static_cast<const uint64_t *>(static_cast<const void *>(ds->Dbuf[Dslot]));
    hipLaunchKernelGGL(k_active_block_sums, dim3(nblocks), dim3(kBlock), 0, ds->stream, ntiles, bits, ds->scan_blocks);
    hipLaunchKernelGGL(k_active_scan_blocks, dim3(1), dim3(kBlock), 0, ds->stream, nblocks, ds->scan_blocks);
    hipLaunchKernelGGL(k_active_tile_offsets, dim3(nblocks), dim3(kBlock), 0, ds->stream, ntiles, bits, ds->scan_blocks, ds->tile_off);
    int64_t g = (ntiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (g > kMaxGrid) g = kMaxGrid;
    const uint64_t inv_d = ((1ull << 32) + (uint64_t)ds->d - 1) / (uint64_t)ds->d;
    if (ds->d % 2 == 0)
        hipLaunchKernelGGL(k_compact_rows<true>, dim3((int)g), dim3(kBlock), 0, ds->stream, ds->n, (int)ds->d, inv_d, ds->X, bits, ds->tile_off, ds->Xhat);
    else
        hipLaunchKernelGGL(k_compact_rows<false>, dim3((int)g), dim3(kBlock), 0, ds->stream, ds->n, (int)ds->d, inv_d, ds->X, bits, ds->tile_off, ds->Xhat);
    const int64_t words = (rows + kWave - 1) / kWave;
    int64_t gb = (words + kBlock - 1) / kBlock;
    if (gb < 1) gb = 1;
    if (gb > kMaxGrid) gb = kMaxGrid;
    hipLaunchKernelGGL(k_all_active_bits, dim3((int)gb), dim3(kBlock), 0, ds->stream, rows, ds->hat_bits);
    TRON_HIP(hipGetLastError());
    ds->hat_rows = rows;
    ds->hat_slot = Dslot;
    return TRON_OK;
}

void dense_compact_release(tron_dataset *ds)
{
    hipFree(ds->Xhat); hipFree(ds->hat_bits); hipFree(ds->tile_off); hipFree(ds->scan_blocks);
    ds->Xhat = nullptr; ds->hat_bits = nullptr; ds->tile_off = nullptr; ds->scan_blocks = nullptr;
    ds->hat_cap = ds->hat_rows = 0;
    ds->hat_slot = -1;
}

bool dense_supported(int64_t d)
{
    Shape s;
    return d >= 1 && pick_shape(d, s);
}

int dense_grid_for(int64_t n, int64_t d)
{
    Shape s;
    if (!pick_shape(d, s)) return 1;
    const int U = pick_U(s.E, s.L);
    const int64_t RT = (int64_t)U * (kWave / s.L);
    const int64_t tiles = (n + RT - 1) / RT;
    int64_t g = (tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (g < 1) g = 1;
    if (g > kMaxGrid) g = kMaxGrid;
    return (int)g;
}

// column partials (d * grid) followed by loss partials (grid), column products (d) and active-row counts (grid)
int64_t dense_partials_needed(int64_t n, int64_t d)
{
    const int64_t g = dense_grid_for(n, d);
    return d * g + g + d + g;
}

int dense_hv(tron_dataset *ds, double C, int Dslot, const double *v, double *Hv)
{
    const HvInput in = hv_input(ds, Dslot);
    const int grid = in.grid;
    double *colprod = ds->partials + ds->d * ds->dense_grid + ds->dense_grid;
    {
        ProfScope ps(ds, SLOT_DENSE_HV);
        TRON_TRY(dispatch_hv(ds, in, v, ds->partials));
        TRON_HIP(hipGetLastError());
    }
    ProfScope ps(ds, SLOT_DENSE_FINALIZE);
    if (ds->d <= kFinishMaxD) {
        hipLaunchKernelGGL(k_dense_finish, dim3(1), dim3(kFinishWaves * kWave), 0, ds->stream, ds->d, grid, ds->partials, v, C, Hv, v, 0,
                           (const double *)nullptr, (const double *)nullptr, (const double *)nullptr, ds->scal_dev, ds->scal_copy);
    } else {
        const int cg = (int)((ds->d + kWavesPerBlock - 1) / kWavesPerBlock);
        hipLaunchKernelGGL(k_dense_columns, dim3(cg), dim3(kBlock), 0, ds->stream, ds->d, grid, ds->partials, v, C, Hv, v, colprod);
        hipLaunchKernelGGL(k_dense_scalars, dim3(1), dim3(kBlock), 0, ds->stream, ds->d, 0, (const double *)nullptr,
                           (const double *)nullptr, (const double *)nullptr, colprod, ds->scal_dev, ds->scal_copy);
    }
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

// out = 1 + C diag(X^T D X): the same pass as dense_hv with squared entries
int dense_hess_diag(tron_dataset *ds, double C, int Dslot, double *out)
{
    const HvInput in = hv_input(ds, Dslot);
    const int grid = in.grid;
    double *colprod = ds->partials + ds->d * ds->dense_grid + ds->dense_grid;
    {
        ProfScope ps(ds, SLOT_DENSE_HV);
        TRON_TRY(dispatch_hv(ds, in, nullptr, ds->partials));
        TRON_HIP(hipGetLastError());
    }
    ProfScope ps(ds, SLOT_DENSE_FINALIZE);
    const int cg = (int)((ds->d + kWavesPerBlock - 1) / kWavesPerBlock);
    hipLaunchKernelGGL(k_dense_columns, dim3(cg), dim3(kBlock), 0, ds->stream, ds->d, grid, ds->partials, (const double *)nullptr, C,
                       out, (const double *)nullptr, colprod);
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

int dense_fun_grad(tron_dataset *ds, int loss, double C, const double *w, int Dslot, double *g)
{
    void *Dout = ds->Dbuf[Dslot];
    if (ds->hat_slot == Dslot) ds->hat_slot = -1;   // the compacted copy belonged to the D that is overwritten now
    ds->D_is_mask[Dslot] = (loss == TRON_LOSS_L2SVM);
    const int grid = ds->dense_grid;
    double *loss_partials = ds->partials + ds->d * grid;
    double *colprod = loss_partials + grid;
    double *active_partials = colprod + ds->d;
    {
        ProfScope ps(ds, SLOT_DENSE_FUN_GRAD);
        TRON_TRY(dispatch_fg(ds, loss, w, Dout, loss_partials, active_partials));
        TRON_HIP(hipGetLastError());
    }
    ProfScope ps(ds, SLOT_DENSE_FINALIZE);
    if (ds->d <= kFinishMaxD) {
        hipLaunchKernelGGL(k_dense_finish, dim3(1), dim3(kFinishWaves * kWave), 0, ds->stream, ds->d, grid, ds->partials, w, C, g,
                           (const double *)nullptr, grid, loss_partials, active_partials, w, ds->scal_dev, ds->scal_copy);
    } else {
        const int cg = (int)((ds->d + kWavesPerBlock - 1) / kWavesPerBlock);
        hipLaunchKernelGGL(k_dense_columns, dim3(cg), dim3(kBlock), 0, ds->stream, ds->d, grid, ds->partials, w, C, g,
                           (const double *)nullptr, colprod);
        hipLaunchKernelGGL(k_dense_scalars, dim3(1), dim3(kBlock), 0, ds->stream, ds->d, grid, loss_partials, active_partials, w, colprod,
                           ds->scal_dev, ds->scal_copy);
    }
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}

}  // namespace tron

// ------------------------------------------------------------------ Hessian-vector product without any allocation
// The work space of the dense Hessian-vector product -- per-workgroup column sums (d * grid), the d column products
// and the curvature scalar -- in a file-scope device array instead of the handle's allocation.  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the process ends.
namespace {
constexpr int64_t kStaticScratchDoubles = TRON_HV_STATIC_MAX_DOUBLES;
__device__ __align__(256) double scratch[kStaticScratchDoubles];
constexpr int kStaticMaxDevices = 64;
double *g_scratch_ptr[kStaticMaxDevices] = {nullptr};   // device address of `scratch` on each GPU, looked up once
}  // namespace

extern "C" int tron_hv_static(tron_dataset *ds, double C, const double *v_dev, double *Hv_dev, double *vHv_dev)
{
    using namespace tron;
    if (!ds || !v_dev || !Hv_dev || v_dev == Hv_dev || !(C > 0.0) || !std::isfinite(C)) {
        set_error("tron_hv_static: bad argument (null handle/v/Hv, v aliases Hv, or C <= 0)");
        return TRON_EINVAL;
    }
    if (!ds->dense) { set_error("tron_hv_static: dense handles only"); return TRON_EINVAL; }
    if (!ds->have_D) { set_error("tron_hv_static: no cached D; call tron_fun_grad first"); return TRON_ESTATE; }
    const int Dslot = ds->Dcur;
    const HvInput in = hv_input(ds, Dslot);
    const int grid = in.grid;
    const int64_t need = ds->d * grid + ds->d + 1;
    if (need > kStaticScratchDoubles) {
        set_error("tron_hv_static: n = %lld, d = %lld needs %lld doubles of work space (d * %d workgroups + d + 1); the static "
                  "work space holds %lld: use tron_hv", (long long)ds->n, (long long)ds->d, (long long)need, grid,
                  (long long)kStaticScratchDoubles);
        return TRON_EINVAL;
    }
    int dev = -1;
    TRON_HIP(hipGetDevice(&dev));
    if (dev != ds->device || dev < 0 || dev >= kStaticMaxDevices) {
        set_error("tron_hv_static: current device %d is not the handle's device %d (or beyond %d devices)", dev, ds->device,
                  kStaticMaxDevices);
        return TRON_EINVAL;
    }
    if (!g_scratch_ptr[dev]) {
        // in host code the array's name is only a stand-in: its address on this GPU comes from the runtime
        double *p = nullptr;
        TRON_HIP(hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)));
        if (!p) { set_error("tron_hv_static: the static work space has no device address"); return TRON_EDEVICE; }
        g_scratch_ptr[dev] = p;
    }
    double *partials = g_scratch_ptr[dev];
    double *colprod = partials + ds->d * grid;
    double *scalar = colprod + ds->d;
    // Nothing has to start at zero: every workgroup of the pass writes all d of its column sums, the second stage
    // writes all d column products, the third the scalar.
    TRON_TRY(dispatch_hv(ds, in, v_dev, partials));
    if (ds->d <= kFinishMaxD) {
        hipLaunchKernelGGL(k_dense_finish, dim3(1), dim3(kFinishWaves * kWave), 0, ds->stream, ds->d, grid, partials, v_dev, C, Hv_dev, v_dev, 0,
                           (const double *)nullptr, (const double *)nullptr, (const double *)nullptr, vHv_dev ? vHv_dev : scalar, scalar);
    } else {
        const int cg = (int)((ds->d + kWavesPerBlock - 1) / kWavesPerBlock);
        hipLaunchKernelGGL(k_dense_columns, dim3(cg), dim3(kBlock), 0, ds->stream, ds->d, grid, partials, v_dev, C, Hv_dev, v_dev, colprod);
        hipLaunchKernelGGL(k_dense_scalars, dim3(1), dim3(kBlock), 0, ds->stream, ds->d, 0, (const double *)nullptr,
                           (const double *)nullptr, (const double *)nullptr, colprod, vHv_dev ? vHv_dev : scalar, scalar);
    }
    TRON_HIP(hipGetLastError());
    return TRON_OK;
}
