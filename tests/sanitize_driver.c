/* Exercises every entry point of the CPU oracle (oracle/slim_oracle.c) on small random layers, built with
 * AddressSanitizer and UndefinedBehaviorSanitizer: exact-size heap buffers, ragged shapes, row subsets.
 * Exit code 0 = every internal check passed and the sanitizers stayed silent.  Test infrastructure. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int slim_oracle_mask(const float *W, int64_t n, int64_t k, uint8_t *mask);
int slim_oracle_scale(const float *W, int64_t n, int64_t k, float *scale);
int slim_oracle_quantize(const float *W, const uint8_t *mask, const float *scale, int64_t n, int64_t k, int8_t *codes);
int slim_oracle_pack(const int8_t *codes, const uint8_t *mask, int64_t n, int64_t k, uint8_t *qvals, uint8_t *meta);
int slim_oracle_unpack(const uint8_t *qvals, const uint8_t *meta, int64_t n, int64_t k, int8_t *codes, uint8_t *mask);
int slim_oracle_dequant(const uint8_t *qvals, const uint8_t *meta, const float *scale, int64_t n, int64_t k, double *Wd);
int slim_oracle_xr(const double *X, const double *R, int64_t m, int64_t k, int64_t r, double *T);
int slim_oracle_forward(const uint8_t *qvals, const uint8_t *meta, const float *scale, const double *L, const double *R,
                        const double *X, int64_t n, int64_t k, int64_t r, int64_t m, const int64_t *rows, int64_t nrows,
                        double *Y, double *T_out);

static uint64_t rng = 88172645463325252ull;
static double uni(void) { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return (double)(rng >> 11) / 9007199254740992.0; }
static double gauss(void) { double a = 0; for (int i = 0; i < 12; ++i) a += uni(); return a - 6.0; }

static int one_case(int64_t n, int64_t k, int64_t r, int64_t m)
{
    float *W = malloc(sizeof(float) * n * k);
    uint8_t *mask = malloc(n * k), *mask2 = malloc(n * k), *qv = malloc(n * k / 4), *me = malloc(n * k / 8);
    int8_t *codes = malloc(n * k), *codes2 = malloc(n * k);
    float *scale = malloc(sizeof(float) * n);
    double *Wd = malloc(sizeof(double) * n * k), *X = malloc(sizeof(double) * m * k);
    double *L = r ? malloc(sizeof(double) * n * r) : NULL, *R = r ? malloc(sizeof(double) * r * k) : NULL;
    double *T = r ? malloc(sizeof(double) * m * r) : NULL, *T2 = r ? malloc(sizeof(double) * m * r) : NULL;
    double *Y = malloc(sizeof(double) * m * n);
    for (int64_t i = 0; i < n * k; ++i) W[i] = (float)(0.02 * gauss());
    if (n > 1) memset(W + k, 0, sizeof(float) * k);                     /* an all-zero row */
    for (int64_t i = 0; i < m * k; ++i) X[i] = gauss();
    for (int64_t i = 0; i < n * r; ++i) L[i] = 0.01 * gauss();
    for (int64_t i = 0; i < r * k; ++i) R[i] = 0.01 * gauss();
    int bad = 0;
    bad |= slim_oracle_mask(W, n, k, mask);
    bad |= slim_oracle_scale(W, n, k, scale);
    bad |= slim_oracle_quantize(W, mask, scale, n, k, codes);
    bad |= slim_oracle_pack(codes, mask, n, k, qv, me);
    bad |= slim_oracle_unpack(qv, me, n, k, codes2, mask2);
    bad |= memcmp(codes, codes2, n * k) != 0 || memcmp(mask, mask2, n * k) != 0;
    bad |= slim_oracle_dequant(qv, me, scale, n, k, Wd);
    if (r) bad |= slim_oracle_xr(X, R, m, k, r, T);
    bad |= slim_oracle_forward(qv, me, scale, L, R, X, n, k, r, m, NULL, n, Y, T2);
    if (r) bad |= memcmp(T, T2, sizeof(double) * m * r) != 0;
    /* the forward is the dequantized dense product plus the low-rank term */
    for (int64_t i = 0; i < m && !bad; ++i)
        for (int64_t o = 0; o < n; ++o) {
            double a = 0, b = 0;
            for (int64_t c = 0; c < k; ++c) a += X[i * k + c] * Wd[o * k + c];
            for (int64_t j = 0; j < r; ++j) b += T[i * r + j] * L[o * r + j];
            if (fabs(Y[i * n + o] - (a + b)) > 1e-12 * (fabs(a) + fabs(b) + 1e-30)) bad = 1;
        }
    /* a row subset (last row, first row, a repeat) gives the same numbers */
    int64_t rows[3] = {n - 1, 0, n - 1};
    double *Ys = malloc(sizeof(double) * m * 3);
    bad |= slim_oracle_forward(qv, me, scale, L, R, X, n, k, r, m, rows, 3, Ys, NULL);
    for (int64_t i = 0; i < m; ++i)
        for (int t = 0; t < 3; ++t) bad |= Ys[i * 3 + t] != Y[i * n + rows[t]];
    /* argument errors are reported, not acted on */
    bad |= slim_oracle_mask(W, n, 6, mask) == 0;                      /* not whole groups of four */
    rows[1] = n;
    bad |= slim_oracle_forward(qv, me, scale, L, R, X, n, k, r, m, rows, 3, Ys, NULL) == 0;
    free(W); free(mask); free(mask2); free(qv); free(me); free(codes); free(codes2); free(scale); free(Wd); free(X);
    free(L); free(R); free(T); free(T2); free(Y); free(Ys);
    if (bad) fprintf(stderr, "case n=%lld k=%lld r=%lld m=%lld failed\n", (long long)n, (long long)k, (long long)r, (long long)m);
    return bad;
}

int main(void)
{
    int bad = 0;
    const int64_t cases[][4] = {{1, 8, 0, 1}, {3, 8, 1, 2}, {17, 136, 5, 3}, {64, 256, 0, 4}, {33, 1024, 51, 16}, {130, 72, 7, 5}};
    for (unsigned i = 0; i < sizeof cases / sizeof cases[0]; ++i) bad |= one_case(cases[i][0], cases[i][1], cases[i][2], cases[i][3]);
    printf(bad ? "FAILED\n" : "sanitized oracle ok\n");
    return bad ? 1 : 0;
}
