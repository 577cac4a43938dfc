/*
 * CPU oracle for fused sparse contraction trees -- TEST INFRASTRUCTURE ONLY.
 *
 * Nothing in the product path may call this file; it exists so that tests, the
 * smoke check and the benchmark's CPU-baseline leg can compare the GPU library
 * against the plain definition.  It shares no code with the GPU library.
 *
 * What is computed is the paper's definition of a tensor network (Sec. 2.1,
 * "Tensor contractions" and "Tensor networks", and the direct nested loop of
 * Fig. 2b): for every assignment of the external indices, the sum over all
 * values of the contraction indices of the product of the tensor elements, a
 * sparse tensor being zero outside its nonzero set.  For one sparse operand and
 * dense factors this is a loop over the coordinate list (COO) of the sparse
 * tensor with dense accumulation into the output; no CSF, no fusion, no tiling.
 *
 * Summation order: nonzeros are first grouped by output row with a stable
 * counting sort, rows are then processed independently (OpenMP over rows), so
 * every output element sums its terms in COO input order whatever the thread
 * count.  fp64 throughout; compile without -ffast-math.
 *
 * All pointers are host pointers.  Dense matrices are row-major.
 * Return value: 0 on success, -1 on bad arguments / out-of-range coordinate,
 * -2 on allocation failure.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Stable grouping of nonzeros by output row: start[r]..start[r+1] index into
 * order[], which lists nonzero positions of row r in input order. */
static int bucket_rows(int64_t nnz, const int32_t *row, int64_t nrows,
                       int64_t **start_out, int64_t **order_out)
{
    int64_t *start = (int64_t *)calloc((size_t)nrows + 2, sizeof(int64_t));
    int64_t *order = (int64_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(int64_t));
    if (!start || !order) { free(start); free(order); return -2; }
    for (int64_t n = 0; n < nnz; ++n) {
        if (row[n] < 0 || row[n] >= nrows) { free(start); free(order); return -1; }
        start[row[n] + 2]++;
    }
    for (int64_t r = 0; r < nrows; ++r) start[r + 2] += start[r + 1];
    /* start[r+1] is now the write cursor of row r */
    for (int64_t n = 0; n < nnz; ++n) order[start[row[n] + 1]++] = n;
    *start_out = start;   /* after the fill, start[r] .. start[r+1] bound row r */
    *order_out = order;
    return 0;
}

static int check_range(int64_t nnz, const int32_t *c, int64_t n)
{
    for (int64_t e = 0; e < nnz; ++e)
        if (c[e] < 0 || c[e] >= n) return -1;
    return 0;
}

/*
 * Order-3 TTMc (Sec. 5.3): for output mode `mode`, with (a,b) the two other
 * modes in increasing order,
 *     Y[c_mode, ra, rb] += X(c0,c1,c2) * Fa[c_a, ra] * Fb[c_b, rb]
 * for every nonzero.  Y is dims[mode] x Ra x Rb, zeroed here.
 */
int oracle_ttmc3(int64_t nnz, const int32_t *c0, const int32_t *c1, const int32_t *c2,
                 const double *vals, const int64_t dims[3], int mode,
                 int Ra, int Rb, const double *Fa, const double *Fb, double *Y)
{
    if (mode < 0 || mode > 2 || Ra <= 0 || Rb <= 0 || nnz < 0) return -1;
    const int32_t *c[3] = { c0, c1, c2 };
    int a = (mode == 0) ? 1 : 0, b = (mode == 2) ? 1 : 2;
    if (check_range(nnz, c[a], dims[a]) || check_range(nnz, c[b], dims[b])) return -1;
    int64_t *start, *order;
    int rc = bucket_rows(nnz, c[mode], dims[mode], &start, &order);
    if (rc) return rc;
    const int64_t rowlen = (int64_t)Ra * Rb;
    memset(Y, 0, (size_t)(dims[mode] * rowlen) * sizeof(double));
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t r = 0; r < dims[mode]; ++r) {
        double *y = Y + r * rowlen;
        for (int64_t p = start[r]; p < start[r + 1]; ++p) {
            int64_t n = order[p];
            const double *fa = Fa + (int64_t)c[a][n] * Ra;
            const double *fb = Fb + (int64_t)c[b][n] * Rb;
            double v = vals[n];
            for (int ra = 0; ra < Ra; ++ra)
                for (int rb = 0; rb < Rb; ++rb)
                    y[(int64_t)ra * Rb + rb] += v * fa[ra] * fb[rb];
        }
    }
    free(start); free(order);
    return 0;
}

/*
 * Order-4 TTMc, output mode 0 (the order-4 generalisation of Sec. 5.3):
 *     Y[i, r1, r2, r3] += X(i,j,k,l) * U1[j,r1] * U2[k,r2] * U3[l,r3].
 */
int oracle_ttmc4(int64_t nnz, const int32_t *c0, const int32_t *c1, const int32_t *c2,
                 const int32_t *c3, const double *vals, const int64_t dims[4],
                 int R1, int R2, int R3, const double *U1, const double *U2, const double *U3,
                 double *Y)
{
    if (R1 <= 0 || R2 <= 0 || R3 <= 0 || nnz < 0) return -1;
    if (check_range(nnz, c1, dims[1]) || check_range(nnz, c2, dims[2]) ||
        check_range(nnz, c3, dims[3])) return -1;
    int64_t *start, *order;
    int rc = bucket_rows(nnz, c0, dims[0], &start, &order);
    if (rc) return rc;
    const int64_t rowlen = (int64_t)R1 * R2 * R3;
    memset(Y, 0, (size_t)(dims[0] * rowlen) * sizeof(double));
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < dims[0]; ++r) {
        double *y = Y + r * rowlen;
        for (int64_t p = start[r]; p < start[r + 1]; ++p) {
            int64_t n = order[p];
            const double *u1 = U1 + (int64_t)c1[n] * R1;
            const double *u2 = U2 + (int64_t)c2[n] * R2;
            const double *u3 = U3 + (int64_t)c3[n] * R3;
            double v = vals[n];
            for (int r1 = 0; r1 < R1; ++r1)
                for (int r2 = 0; r2 < R2; ++r2)
                    for (int r3 = 0; r3 < R3; ++r3)
                        y[((int64_t)r1 * R2 + r2) * R3 + r3] += v * u1[r1] * u2[r2] * u3[r3];
        }
    }
    free(start); free(order);
    return 0;
}

/*
 * Order-3 MTTKRP (Sec. 5.2): for output mode `mode`, with (a,b) the other modes,
 *     M[c_mode, r] += X(c0,c1,c2) * Fa[c_a, r] * Fb[c_b, r].
 * r is a batch index: it appears in both factors and in the output.
 */
int oracle_mttkrp3(int64_t nnz, const int32_t *c0, const int32_t *c1, const int32_t *c2,
                   const double *vals, const int64_t dims[3], int mode, int R,
                   const double *Fa, const double *Fb, double *M)
{
    if (mode < 0 || mode > 2 || R <= 0 || nnz < 0) return -1;
    const int32_t *c[3] = { c0, c1, c2 };
    int a = (mode == 0) ? 1 : 0, b = (mode == 2) ? 1 : 2;
    if (check_range(nnz, c[a], dims[a]) || check_range(nnz, c[b], dims[b])) return -1;
    int64_t *start, *order;
    int rc = bucket_rows(nnz, c[mode], dims[mode], &start, &order);
    if (rc) return rc;
    memset(M, 0, (size_t)(dims[mode] * R) * sizeof(double));
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t r = 0; r < dims[mode]; ++r) {
        double *m = M + r * R;
        for (int64_t p = start[r]; p < start[r + 1]; ++p) {
            int64_t n = order[p];
            const double *fa = Fa + (int64_t)c[a][n] * R;
            const double *fb = Fb + (int64_t)c[b][n] * R;
            double v = vals[n];
            for (int q = 0; q < R; ++q) m[q] += v * fa[q] * fb[q];
        }
    }
    free(start); free(order);
    return 0;
}

/*
 * Three-tensor network of Sec. 1:  Z[i,m] = sum_{j,k,l} U(i,j,k) V[j,l] W(k,l,m),
 * evaluated through the binary tree (U.V).W (Sec. 2.1, "Contraction tree"):
 * per output row i a dense T_i[k,l] = sum_j U(i,j,k) V[j,l] is formed from U's
 * COO entries of that row, then every COO entry of W adds T_i[k,l]*W(k,l,m) to
 * Z[i,m].  The direct six-index loop is the same sum in another order; the test
 * suite checks the two against each other on small tensors.
 */
int oracle_sptn3(int64_t nnzU, const int32_t *ui, const int32_t *uj, const int32_t *uk,
                 const double *uv, int64_t Ni, int64_t Nj, int64_t Nk, int64_t L,
                 const double *V, int64_t nnzW, const int32_t *wk, const int32_t *wl,
                 const int32_t *wm, const double *wv, int64_t Mm, double *Z)
{
    if (nnzU < 0 || nnzW < 0 || L <= 0 || Mm <= 0) return -1;
    if (check_range(nnzU, uj, Nj) || check_range(nnzU, uk, Nk)) return -1;
    if (check_range(nnzW, wk, Nk) || check_range(nnzW, wl, L) || check_range(nnzW, wm, Mm)) return -1;
    int64_t *start, *order;
    int rc = bucket_rows(nnzU, ui, Ni, &start, &order);
    if (rc) return rc;
    memset(Z, 0, (size_t)(Ni * Mm) * sizeof(double));
    int fail = 0;
#pragma omp parallel
    {
        double *T = (double *)malloc((size_t)(Nk * L) * sizeof(double));
        if (!T) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t i = 0; i < Ni; ++i) {
                if (start[i] == start[i + 1]) continue;       /* empty slice: Z row stays 0 */
                memset(T, 0, (size_t)(Nk * L) * sizeof(double));
                for (int64_t p = start[i]; p < start[i + 1]; ++p) {
                    int64_t n = order[p];
                    double u = uv[n];
                    const double *vrow = V + (int64_t)uj[n] * L;
                    double *trow = T + (int64_t)uk[n] * L;
                    for (int64_t l = 0; l < L; ++l) trow[l] += u * vrow[l];
                }
                double *z = Z + i * Mm;
                for (int64_t e = 0; e < nnzW; ++e)
                    z[wm[e]] += T[(int64_t)wk[e] * L + wl[e]] * wv[e];
            }
        }
        free(T);
    }
    free(start); free(order);
    return fail ? -2 : 0;
}
