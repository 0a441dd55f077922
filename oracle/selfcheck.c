/*
 * Stand-alone driver of the oracle for sanitizer runs (test infrastructure only): built by
 * tests/test_oracle_sanitized.py together with sig_oracle.c and sig_grad_oracle.c under
 * -fsanitize=address,undefined and run as a process.  It walks a few shapes, final and stream mode,
 * forward and gradient, and checks two facts that need no second implementation: level 1 of a
 * signature is the total increment (Eq. 1), and the gradients over the points of a path sum to
 * zero (the signature does not change when the whole path is shifted).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t oracle_sig_size(int d, int N);
int oracle_signature(const double *path, int64_t B, int64_t L, int d, int N, int stream, double *out);
int oracle_signature_backward(const double *path, int64_t B, int64_t L, int d, int N, int stream,
                              const double *grad_out, double *grad_path);

static double next_uniform(uint64_t *state)
{
    *state = *state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(*state >> 11) / 9007199254740992.0 - 0.5;
}

static int run(int64_t B, int64_t L, int d, int N, int stream)
{
    const int64_t D = oracle_sig_size(d, N), K = L - 1, rows = stream ? K : 1;
    double *x = malloc(sizeof(double) * (size_t)(B * L * d));
    double *out = malloc(sizeof(double) * (size_t)(B * rows * D));
    double *g = malloc(sizeof(double) * (size_t)(B * rows * D));
    double *gx = malloc(sizeof(double) * (size_t)(B * L * d));
    if (!x || !out || !g || !gx) return 1;
    uint64_t s = 12345u + (uint64_t)(B * 131 + L * 17 + d * 7 + N);
    for (int64_t i = 0; i < B * L * d; ++i) x[i] = next_uniform(&s);
    for (int64_t i = 0; i < B * rows * D; ++i) g[i] = next_uniform(&s);
    int bad = oracle_signature(x, B, L, d, N, stream, out) != 0;
    bad |= oracle_signature_backward(x, B, L, d, N, stream, g, gx) != 0;
    for (int64_t b = 0; b < B && !bad; ++b) {
        const double *last = out + (b * rows + (rows - 1)) * D;
        for (int j = 0; j < d; ++j) {
            double total = x[(b * L + K) * d + j] - x[b * L * d + j];
            if (fabs(last[j] - total) > 1e-12) bad = 1;
            double sum = 0.0;
            for (int64_t k = 0; k < L; ++k) sum += gx[(b * L + k) * d + j];
            if (fabs(sum) > 1e-10) bad = 1;
        }
    }
    free(x); free(out); free(g); free(gx);
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= run(3, 2, 1, 1, 0);
    bad |= run(2, 7, 3, 4, 0);
    bad |= run(2, 7, 3, 4, 1);
    bad |= run(5, 16, 2, 3, 1);
    bad |= run(1, 30, 5, 4, 0);
    bad |= run(4, 3, 10, 2, 1);
    printf(bad ? "selfcheck FAILED\n" : "selfcheck ok\n");
    return bad;
}
