/*
 * fp64 CPU oracle for the gradient of the truncated path-signature transform
 * with respect to the path.
 *
 * TEST INFRASTRUCTURE ONLY (see sig_oracle.c): the product never calls it.
 *
 * What it computes.  The signature layer of the paper sits between trainable
 * layers (Section 4.2, Eq. 11), so training needs d(loss)/d(path) from
 * d(loss)/d(output).  The paper obtains it by automatic differentiation of
 * Eqs. 2-5; this file is that derivative written out by hand, the plain way:
 *
 *   forward  : every prefix signature P_k = P_{k-1} (x) E_k, E_k = exp(dX_k), is
 *              computed with the functions of sig_oracle.c and KEPT (no
 *              reconstruction of earlier prefixes from later ones);
 *   reverse  : k = K-1 .. 0, with A = d(loss)/d(P_k):
 *      product  C_n = sum_{i+j=n} S_i (x) E_j   (Eq. 4)  gives
 *                 d/dS_i[I] += sum_J A_{i+j}[I,J] E_j[J]
 *                 d/dE_j[J] += sum_I A_{i+j}[I,J] S_i[I]
 *      exponential E_n[I,a] = E_{n-1}[I] dX[a] / n  (Eq. 2), n = N .. 1, gives
 *                 d/dE_{n-1}[I] += sum_a d/dE_n[I,a] dX[a] / n
 *                 d/ddX[a]      += sum_I d/dE_n[I,a] E_{n-1}[I] / n
 *      increments dX_k = X_{k+1} - X_k give d/dX_{k+1} += d/ddX_k, d/dX_k -= d/ddX_k.
 *   In stream mode row k of the output is P_k, so its upstream gradient is
 *   added to A when the sweep reaches k.  Level 0 is the constant 1: it has no
 *   upstream gradient and its own gradient is dropped.
 *
 * Pins (tests/test_grad_oracle_pins.py): central finite differences of the
 * forward oracle, the closed form for depth 1, the closed form of a single
 * segment written with explicit indices, translation invariance, linearity in
 * the upstream gradient, homogeneity under scaling of the path, stream mode
 * against final mode on truncated paths, batch independence.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

int64_t oracle_sig_size(int d, int N);
void oracle_exp(const double *v, int d, int N, double *E);
void oracle_mul(const double *a, const double *b, int d, int N, double *c);

static int64_t lvl_start(int d, int n)
{
    int64_t s = 0, p = 1;
    for (int m = 0; m < n; ++m) { s += p; p *= d; }
    return s;
}

static int64_t int_pow(int d, int n)
{
    int64_t p = 1;
    for (int m = 0; m < n; ++m) p *= d;
    return p;
}

/*
 * Reverse of C = S (x) E (Eq. 4): given A = d(loss)/dC (1 + D numbers, slot 0 unused),
 * ADD d(loss)/dS into gS and d(loss)/dE into gE (both 1 + D numbers).
 */
static void mul_backward(const double *S, const double *E, const double *A, int d, int N,
                         double *gS, double *gE)
{
    for (int n = 1; n <= N; ++n) {
        const double *An = A + lvl_start(d, n);
        for (int i = 0; i <= n; ++i) {
            int j = n - i;
            const double *Si = S + lvl_start(d, i);
            const double *Ej = E + lvl_start(d, j);
            double *gSi = gS + lvl_start(d, i);
            double *gEj = gE + lvl_start(d, j);
            int64_t ni = int_pow(d, i), nj = int_pow(d, j);
            for (int64_t I = 0; I < ni; ++I)
                for (int64_t J = 0; J < nj; ++J) {
                    double a = An[I * nj + J];
                    gSi[I] += a * Ej[J];
                    gEj[J] += a * Si[I];
                }
        }
    }
}

/*
 * Reverse of Eq. 2: given gE = d(loss)/dE (modified in place: lower levels
 * receive what flows down from higher ones), ADD d(loss)/dv into gv (d numbers).
 */
static void exp_backward(const double *v, const double *E, double *gE, int d, int N, double *gv)
{
    for (int n = N; n >= 1; --n) {
        const double *prev = E + lvl_start(d, n - 1);
        double *gprev = gE + lvl_start(d, n - 1);
        const double *gcur = gE + lvl_start(d, n);
        int64_t np = int_pow(d, n - 1);
        for (int64_t I = 0; I < np; ++I)
            for (int a = 0; a < d; ++a) {
                double g = gcur[I * d + a];
                gprev[I] += g * v[a] / (double)n;
                gv[a] += g * prev[I] / (double)n;
            }
    }
}

/*
 *   path      : [B][L][d]
 *   grad_out  : stream == 0: [B][D];  stream != 0: [B][L-1][D]  (same layout as the forward output)
 *   grad_path : [B][L][d], overwritten
 * returns 0, -1 on bad arguments, -2 if a work buffer cannot be allocated.
 */
int oracle_signature_backward(const double *path, int64_t B, int64_t L, int d, int N, int stream,
                              const double *grad_out, double *grad_path)
{
    int64_t D = oracle_sig_size(d, N);
    if (!path || !grad_out || !grad_path || B < 0 || L < 2 || D < 0) return -1;
    int64_t K = L - 1;
    size_t row = (size_t)(1 + D);
    int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double *P = (double *)malloc(sizeof(double) * row * (size_t)K);   /* prefix signatures */
        double *E = (double *)malloc(sizeof(double) * row * (size_t)K);   /* exponentials */
        double *A = (double *)calloc(row, sizeof(double));
        double *gS = (double *)malloc(sizeof(double) * row);
        double *gE = (double *)malloc(sizeof(double) * row);
        double *dx = (double *)malloc(sizeof(double) * (size_t)d * (size_t)K);
        double *gdx = (double *)malloc(sizeof(double) * (size_t)d);
        if (!P || !E || !A || !gS || !gE || !dx || !gdx) {
#pragma omp atomic write
            failed = 1;
        } else {
            const double *X = path + b * L * d;
            double *G = grad_path + b * L * d;
            for (int64_t i = 0; i < L * d; ++i) G[i] = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                for (int j = 0; j < d; ++j) dx[k * d + j] = X[(k + 1) * d + j] - X[k * d + j];
                oracle_exp(dx + k * d, d, N, E + (size_t)k * row);
                if (k == 0) memcpy(P, E, sizeof(double) * row);
                else oracle_mul(P + (size_t)(k - 1) * row, E + (size_t)k * row, d, N, P + (size_t)k * row);
            }
            if (!stream) memcpy(A + 1, grad_out + b * D, sizeof(double) * (size_t)D);
            for (int64_t k = K - 1; k >= 0; --k) {
                if (stream) {
                    const double *g = grad_out + (b * K + k) * D;
                    for (int64_t w = 0; w < D; ++w) A[1 + w] += g[w];
                }
                memset(gS, 0, sizeof(double) * row);
                memset(gE, 0, sizeof(double) * row);
                if (k == 0) memcpy(gE, A, sizeof(double) * row);
                else mul_backward(P + (size_t)(k - 1) * row, E + (size_t)k * row, A, d, N, gS, gE);
                for (int j = 0; j < d; ++j) gdx[j] = 0.0;
                exp_backward(dx + k * d, E + (size_t)k * row, gE, d, N, gdx);
                for (int j = 0; j < d; ++j) {
                    G[(k + 1) * d + j] += gdx[j];
                    G[k * d + j] -= gdx[j];
                }
                memcpy(A, gS, sizeof(double) * row);
                A[0] = 0.0;
            }
        }
        free(P); free(E); free(A); free(gS); free(gE); free(dx); free(gdx);
    }
    return failed ? -2 : 0;
}
