/* Host sanitizer check of the CPU oracle (test infrastructure): oracle.c is compiled together with
 * this driver under -fsanitize=address,undefined and every routine is run on small seeded inputs,
 * ragged sizes, an empty tensor and an out-of-range coordinate.  Results are compared with a
 * plain nested loop over the densified tensor so that the run also means something; the point is
 * that the sanitizers stay silent. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_ttmc3(int64_t, const int32_t *, const int32_t *, const int32_t *, const double *, const int64_t[3], int,
                 int, int, const double *, const double *, double *);
int oracle_ttmc4(int64_t, const int32_t *, const int32_t *, const int32_t *, const int32_t *, const double *,
                 const int64_t[4], int, int, int, const double *, const double *, const double *, double *);
int oracle_mttkrp3(int64_t, const int32_t *, const int32_t *, const int32_t *, const double *, const int64_t[3], int,
                   int, const double *, const double *, double *);
int oracle_sptn3(int64_t, const int32_t *, const int32_t *, const int32_t *, const double *, int64_t, int64_t, int64_t,
                 int64_t, const double *, int64_t, const int32_t *, const int32_t *, const int32_t *, const double *,
                 int64_t, double *);

static uint64_t state = 88172645463325252ull;
static double rnd(void) {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static int32_t rint_below(int64_t n) { return (int32_t)((rnd() * 0.5 + 0.5) * (double)n) % (int32_t)n; }
static double *dense(int64_t n) { double *p = malloc((size_t)(n ? n : 1) * sizeof(double)); for (int64_t i = 0; i < n; ++i) p[i] = rnd(); return p; }
static int fails = 0;
static void expect(int ok, const char *what) { if (!ok) { printf("FAIL: %s\n", what); ++fails; } }

int main(void) {
    const int64_t d3[3] = {5, 7, 3}, d4[4] = {4, 3, 5, 2};
    for (int round = 0; round < 3; ++round) {
        const int64_t nnz = round == 0 ? 0 : (round == 1 ? 1 : 41);
        int32_t *c[4];
        for (int m = 0; m < 4; ++m) { c[m] = malloc((size_t)(nnz ? nnz : 1) * sizeof(int32_t)); }
        double *v = dense(nnz);
        for (int64_t e = 0; e < nnz; ++e) for (int m = 0; m < 3; ++m) c[m][e] = rint_below(d3[m]);
        /* order-3 TTMc and MTTKRP, every output mode, ragged ranks */
        for (int mode = 0; mode < 3; ++mode) {
            const int a = mode == 0 ? 1 : 0, b = mode == 2 ? 1 : 2, Ra = 3, Rb = 2, R = 4;
            double *Fa = dense(d3[a] * Ra), *Fb = dense(d3[b] * Rb), *Y = dense(d3[mode] * Ra * Rb);
            expect(oracle_ttmc3(nnz, c[0], c[1], c[2], v, d3, mode, Ra, Rb, Fa, Fb, Y) == 0, "ttmc3 status");
            double *ref = calloc((size_t)(d3[mode] * Ra * Rb), sizeof(double));
            for (int64_t e = 0; e < nnz; ++e)
                for (int ra = 0; ra < Ra; ++ra) for (int rb = 0; rb < Rb; ++rb)
                    ref[(c[mode][e] * Ra + ra) * Rb + rb] += v[e] * Fa[c[a][e] * Ra + ra] * Fb[c[b][e] * Rb + rb];
            for (int64_t i = 0; i < d3[mode] * Ra * Rb; ++i) expect(fabs(ref[i] - Y[i]) < 1e-12, "ttmc3 value");
            free(ref); free(Fa); free(Fb); free(Y);
            double *Ga = dense(d3[a] * R), *Gb = dense(d3[b] * R), *M = dense(d3[mode] * R);
            expect(oracle_mttkrp3(nnz, c[0], c[1], c[2], v, d3, mode, R, Ga, Gb, M) == 0, "mttkrp3 status");
            ref = calloc((size_t)(d3[mode] * R), sizeof(double));
            for (int64_t e = 0; e < nnz; ++e)
                for (int r = 0; r < R; ++r) ref[c[mode][e] * R + r] += v[e] * Ga[c[a][e] * R + r] * Gb[c[b][e] * R + r];
            for (int64_t i = 0; i < d3[mode] * R; ++i) expect(fabs(ref[i] - M[i]) < 1e-12, "mttkrp3 value");
            free(ref); free(Ga); free(Gb); free(M);
        }
        /* order-4 TTMc */
        for (int64_t e = 0; e < nnz; ++e) for (int m = 0; m < 4; ++m) c[m][e] = rint_below(d4[m]);
        {
            const int R1 = 2, R2 = 3, R3 = 2;
            double *U1 = dense(d4[1] * R1), *U2 = dense(d4[2] * R2), *U3 = dense(d4[3] * R3), *Y = dense(d4[0] * R1 * R2 * R3);
            expect(oracle_ttmc4(nnz, c[0], c[1], c[2], c[3], v, d4, R1, R2, R3, U1, U2, U3, Y) == 0, "ttmc4 status");
            double *ref = calloc((size_t)(d4[0] * R1 * R2 * R3), sizeof(double));
            for (int64_t e = 0; e < nnz; ++e)
                for (int r1 = 0; r1 < R1; ++r1) for (int r2 = 0; r2 < R2; ++r2) for (int r3 = 0; r3 < R3; ++r3)
                    ref[((c[0][e] * R1 + r1) * R2 + r2) * R3 + r3] +=
                        v[e] * U1[c[1][e] * R1 + r1] * U2[c[2][e] * R2 + r2] * U3[c[3][e] * R3 + r3];
            for (int64_t i = 0; i < d4[0] * R1 * R2 * R3; ++i) expect(fabs(ref[i] - Y[i]) < 1e-12, "ttmc4 value");
            free(ref); free(U1); free(U2); free(U3); free(Y);
        }
        /* three-tensor network Z[i,m] = U[i,j,k] V[j,l] W[k,l,m] */
        {
            const int64_t Ni = 4, Nj = 5, Nk = 3, L = 6, Mm = 2, nw = nnz ? 17 : 0;
            int32_t *w[3];
            for (int m = 0; m < 3; ++m) w[m] = malloc((size_t)(nw ? nw : 1) * sizeof(int32_t));
            double *wv = dense(nw), *V = dense(Nj * L), *Z = dense(Ni * Mm);
            for (int64_t e = 0; e < nnz; ++e) { c[0][e] = rint_below(Ni); c[1][e] = rint_below(Nj); c[2][e] = rint_below(Nk); }
            for (int64_t e = 0; e < nw; ++e) { w[0][e] = rint_below(Nk); w[1][e] = rint_below(L); w[2][e] = rint_below(Mm); }
            expect(oracle_sptn3(nnz, c[0], c[1], c[2], v, Ni, Nj, Nk, L, V, nw, w[0], w[1], w[2], wv, Mm, Z) == 0, "sptn3 status");
            double *ref = calloc((size_t)(Ni * Mm), sizeof(double));
            for (int64_t e = 0; e < nnz; ++e)
                for (int64_t f = 0; f < nw; ++f)
                    if (w[0][f] == c[2][e]) ref[c[0][e] * Mm + w[2][f]] += v[e] * V[c[1][e] * L + w[1][f]] * wv[f];
            for (int64_t i = 0; i < Ni * Mm; ++i) expect(fabs(ref[i] - Z[i]) < 1e-12, "sptn3 value");
            /* a coordinate beyond its extent is refused, nothing is read or written out of bounds */
            if (nnz) { c[1][0] = (int32_t)Nj; expect(oracle_sptn3(nnz, c[0], c[1], c[2], v, Ni, Nj, Nk, L, V, nw, w[0], w[1], w[2], wv, Mm, Z) != 0, "sptn3 range"); }
            free(ref); free(wv); free(V); free(Z);
            for (int m = 0; m < 3; ++m) free(w[m]);
        }
        if (nnz) {
            double Y[5 * 4];
            double F[7 * 2], G[3 * 2];
            memset(F, 0, sizeof F); memset(G, 0, sizeof G);
            for (int64_t e = 0; e < nnz; ++e) for (int m = 0; m < 3; ++m) c[m][e] = rint_below(d3[m]);
            c[2][nnz - 1] = -1;
            expect(oracle_ttmc3(nnz, c[0], c[1], c[2], v, d3, 0, 2, 2, F, G, Y) != 0, "ttmc3 range");
            expect(oracle_mttkrp3(nnz, c[0], c[1], c[2], v, d3, 0, 2, F, G, Y) != 0, "mttkrp3 range");
        }
        for (int m = 0; m < 4; ++m) free(c[m]);
        free(v);
    }
    printf("%s\n", fails ? "san_oracle: FAILED" : "san_oracle: ok");
    return fails ? 1 : 0;
}
