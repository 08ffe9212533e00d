/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Stand-alone driver that runs every routine of tron_oracle.c once on a small CSR problem with empty rows,
 * empty columns, a single-entry row and a full row, and on its dense twin.  The test suite builds it with
 * -fsanitize=address,undefined and expects exit status 0: an out-of-bounds index, a read of uninitialised
 * heap memory that reaches a branch, a leak or undefined arithmetic in the oracle ends the run with a report.
 * It checks memory safety only; what the routines compute is pinned elsewhere.
 */
#include "tron_oracle.c"

#include <stdio.h>

static uint64_t state = 0x9e3779b97f4a7c15ull;
static double unif(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0;
}

int main(void)
{
    enum { N = 37, D = 11 };
    int64_t rowptr[N + 1];
    int32_t col[N * D];
    double val[N * D], Xd[N * D], y[N];
    int64_t nnz = 0;
    memset(Xd, 0, sizeof(Xd));
    rowptr[0] = 0;
    for (int i = 0; i < N; ++i) {
        y[i] = unif() < 0.5 ? 1.0 : -1.0;
        for (int j = 0; j < D; ++j) {
            int keep;
            if (i % 7 == 0) keep = 0;                 /* empty rows, including the first */
            else if (i == N - 1) keep = 0;            /* ... and the last */
            else if (i == 5) keep = 1;                /* a full row (except the empty columns) */
            else if (i == 6) keep = (j == D - 2);     /* a single entry */
            else keep = unif() < 0.35;
            if (j == 0 || j == 4 || j == D - 1) keep = 0;   /* empty columns, including the first and the last */
            if (keep) {
                const double v = 2.0 * unif() - 1.0;
                col[nnz] = j; val[nnz] = v; Xd[i * D + j] = v; ++nnz;
            }
        }
        rowptr[i + 1] = nnz;
    }
    const orc_data csr = { N, D, rowptr, col, val, NULL, y };
    const orc_data dense = { N, D, NULL, NULL, NULL, Xd, y };
    const orc_data *both[2] = { &csr, &dense };
    double w[D], v[D], g[D], Hv[D], hd[D], s[D], r[D], M[D], z[N], zhat[N], Dg[N];
    double checksum = 0.0;
    for (int k = 0; k < 2; ++k) {
        for (int loss = 0; loss < 2; ++loss) {
            const orc_data *A = both[k];
            double f;
            int nhv, onb, tl;
            orc_result res;
            orc_trace_rec trace[4];   /* shorter than the solves: the cap must hold */
            for (int j = 0; j < D; ++j) { w[j] = unif() - 0.5; v[j] = unif() - 0.5; }
            if (orc_fun(A, loss, 1.5, w, &f, z, zhat, Dg)) return 2;
            if (orc_fun(A, loss, 1.5, w, &f, NULL, NULL, NULL)) return 2;
            if (orc_grad(A, 1.5, w, zhat, g)) return 2;
            if (orc_hv(A, 1.5, Dg, v, Hv)) return 2;
            if (orc_hess_diag(A, 1.5, Dg, hd)) return 2;
            for (int j = 0; j < D; ++j) M[j] = 0.99 + 0.01 * hd[j];
            if (orc_cg(A, 1.5, Dg, g, 1e30, 0.1, 50, s, r, &nhv, &onb)) return 2;
            if (orc_cg(A, 1.5, Dg, g, 1e-3, 0.1, 50, s, r, &nhv, &onb) || !onb) return 3;
            if (orc_cg(A, 1.5, Dg, g, 1e30, 0.0, 1, s, r, &nhv, &onb)) return 2;
            if (orc_pcg(A, 1.5, Dg, g, M, 1e30, 0.1, 50, s, r, &nhv, &onb)) return 2;
            if (orc_pcg(A, 1.5, Dg, g, M, 1e-3, 0.1, 50, s, r, &nhv, &onb) || !onb) return 3;
            for (int j = 0; j < D; ++j) w[j] = 0.0;
            if (orc_tron(A, loss, 1.5, 1e-9, 100, 50, 0.1, w, &res, trace, 4, &tl) < 0 || tl > 4) return 4;
            checksum += res.f;
            for (int j = 0; j < D; ++j) w[j] = 4.0 * (unif() - 0.5);   /* warm start: the extra gradient at 0 */
            if (orc_tron(A, loss, 40.0, 1e-6, 100, 50, 0.1, w, &res, NULL, 0, NULL) < 0) return 4;
            if (orc_tron_pcg(A, loss, 1.5, 1e-9, 100, 50, 0.1, 0.01, w, &res, trace, 4, &tl) < 0 || tl > 4) return 4;
            if (orc_tron(A, loss, 1.5, 1e-9, 1, 1, 0.1, w, &res, trace, 1, &tl) < 0) return 4;
            checksum += res.f;
        }
    }
    /* n = 1, d = 1 and a matrix without entries */
    {
        const int64_t rp1[2] = { 0, 0 };
        const double y1[1] = { -1.0 };
        const orc_data empty = { 1, 1, rp1, col, val, NULL, y1 };
        double w1[1] = { 0.0 };
        orc_result res;
        if (orc_tron(&empty, ORC_LOSS_LR, 1.0, 1e-6, 10, 10, 0.1, w1, &res, NULL, 0, NULL) < 0) return 5;
        if (orc_tron(&empty, ORC_LOSS_L2SVM, 1.0, 1e-6, 10, 10, 0.1, w1, &res, NULL, 0, NULL) < 0) return 5;
        checksum += res.f;
    }
    printf("oracle sanitize run ok %.17g\n", checksum);
    return 0;
}
