/*
 * fp64 CPU oracle for the truncated path-signature transform.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is judged against.  It shares no code with the HIP path and the
 * product never calls it: only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load it.
 *
 * What it computes (paper, Section 3.1 "Traditional Approach"):
 *   - increments  dX_k = X_{k+1} - X_k of a piecewise-linear path (text above Eq. 2);
 *   - the restricted tensor exponential of one increment        (Eq. 2);
 *   - the recursion  Sig_1 = exp(dX_1), Sig_k = Sig_{k-1} (x) exp(dX_k)   (Eq. 3, batched in Eq. 5);
 *   - the truncated tensor-algebra product                        (Eq. 4);
 *   - the output row [S_1, ..., S_N] at a prefix, level 0 dropped (Eq. 10).
 * The method is exact, so the oracle is the definition written out: the
 * exponential of every increment is materialised, every product is the full
 * double sum of Eq. 4 into a fresh buffer, and time is walked strictly left to
 * right.  No Horner form, no in-place update, no blocking over time.
 *
 * Readings of the paper taken here:
 *   - Eq. 4 sums over i + j = n with i and j running from 0 and a_0 = b_0 = 1
 *     (the printed tuples start at index 1; without the 0 terms level 1 of a
 *     product would vanish, contradicting level 1 of Eq. 1);
 *   - a path of L points has L - 1 increments, so Eq. 3 has L - 1 factors and
 *     stream mode has L - 1 prefixes (the printed range k = 2..L counts points);
 *   - earlier time is the left tensor factor (Eq. 1 integrates dX_{t1} (x) dX_{t2}
 *     with t1 < t2; Eq. 3 keeps Sig_{k-1} on the left) and a level is flattened
 *     row-major, first letter slowest.  The paper does not state a flattening.
 *
 * A tensor-algebra element is stored with its level 0 in slot 0, then level 1
 * (d numbers), level 2 (d*d numbers) ... level N; size 1 + D.
 *
 * Pins (tests/test_oracle_pins.py): closed form of a single segment, level 1 =
 * total increment, collinear paths, d = 1, a hand-worked two-segment example,
 * shuffle identities up to total length 3, Levy area by the shoelace sum,
 * Chen concatenation, time reversal, scaling, brute-force iterated sums with
 * explicit indices, stream-versus-truncated-path consistency.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* D = d + d^2 + ... + d^N, or -1 if it does not fit in int64 (Eq. 10 row length). */
int64_t oracle_sig_size(int d, int N)
{
    if (d < 1 || N < 1) return -1;
    int64_t total = 0, p = 1;
    for (int n = 1; n <= N; ++n) {
        if (p > INT64_MAX / d) return -1;
        p *= d;
        if (total > INT64_MAX - p) return -1;
        total += p;
    }
    return total;
}

/* start of level n inside a (1 + D)-element buffer: 1 + d + ... + d^{n-1}; level 0 is slot 0 */
static int64_t level_start(int d, int n)
{
    int64_t s = 0, p = 1;
    for (int m = 0; m < n; ++m) { s += p; p *= d; }
    return s;
}

static int64_t ipow(int d, int n)
{
    int64_t p = 1;
    for (int m = 0; m < n; ++m) p *= d;
    return p;
}

/*
 * Eq. 2: E = (1, v, v(x)v / 2!, ..., v^{(x)N} / N!).
 * Level n is built from level n-1 by one more tensor factor on the right and
 * a division by n:  E_n[I*d + j] = E_{n-1}[I] * v[j] / n.
 */
void oracle_exp(const double *v, int d, int N, double *E)
{
    E[0] = 1.0;
    for (int n = 1; n <= N; ++n) {
        const double *prev = E + level_start(d, n - 1);
        double *cur = E + level_start(d, n);
        int64_t np = ipow(d, n - 1);
        for (int64_t I = 0; I < np; ++I)
            for (int j = 0; j < d; ++j)
                cur[I * d + j] = prev[I] * v[j] / (double)n;
    }
}

/*
 * Eq. 4 for general elements (level 0 of each factor is whatever slot 0 holds):
 *   c_n = sum_{i=0..n} a_i (x) b_{n-i},   (a_i (x) b_j)[I * d^j + J] = a_i[I] * b_j[J].
 * c must not alias a or b.
 */
void oracle_mul(const double *a, const double *b, int d, int N, double *c)
{
    for (int n = 0; n <= N; ++n) {
        double *cn = c + level_start(d, n);
        int64_t sz = ipow(d, n);
        for (int64_t w = 0; w < sz; ++w) cn[w] = 0.0;
        for (int i = 0; i <= n; ++i) {
            int j = n - i;
            const double *ai = a + level_start(d, i);
            const double *bj = b + level_start(d, j);
            int64_t ni = ipow(d, i), nj = ipow(d, j);
            for (int64_t I = 0; I < ni; ++I)
                for (int64_t J = 0; J < nj; ++J)
                    cn[I * nj + J] += ai[I] * bj[J];
        }
    }
}

/*
 * Eq. 3 / Eq. 5 / Eq. 10.
 *   path : [B][L][d] doubles (the fp32 inputs widened exactly by the caller)
 *   out  : stream == 0: [B][D];  stream != 0: [B][L-1][D]   (level 0 omitted)
 * returns 0, or -1 on bad arguments / size overflow, -2 if a work buffer cannot be allocated.
 */
int oracle_signature(const double *path, int64_t B, int64_t L, int d, int N,
                     int stream, double *out)
{
    int64_t D = oracle_sig_size(d, N);
    if (!path || !out || B < 0 || L < 2 || D < 0) return -1;
    int64_t K = L - 1;
    int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double *S = (double *)malloc(sizeof(double) * (size_t)(1 + D));
        double *E = (double *)malloc(sizeof(double) * (size_t)(1 + D));
        double *C = (double *)malloc(sizeof(double) * (size_t)(1 + D));
        double *dx = (double *)malloc(sizeof(double) * (size_t)d);
        if (!S || !E || !C || !dx) {
#pragma omp atomic write
            failed = 1;
        } else {
            const double *X = path + b * L * d;
            for (int64_t k = 0; k < K; ++k) {
                for (int j = 0; j < d; ++j) dx[j] = X[(k + 1) * d + j] - X[k * d + j];
                oracle_exp(dx, d, N, E);
                if (k == 0) {
                    memcpy(S, E, sizeof(double) * (size_t)(1 + D));
                } else {
                    oracle_mul(S, E, d, N, C);
                    double *t = S; S = C; C = t;
                }
                if (stream)
                    memcpy(out + (b * K + k) * D, S + 1, sizeof(double) * (size_t)D);
            }
            if (!stream) memcpy(out + b * D, S + 1, sizeof(double) * (size_t)D);
        }
        free(S); free(E); free(C); free(dx);
    }
    return failed ? -2 : 0;
}

/* number of OpenMP threads oracle_signature will use (for the benchmark's "cores" field) */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
