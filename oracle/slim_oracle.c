/*
 * CPU oracle for one SLiM-compressed linear layer (arXiv 2410.09615).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 statement of
 * what the layer computes.  It is used by the tests, by the smoke check and by
 * the CPU-baseline leg of the benchmark; the product library never calls it
 * and shares no code, header, table or helper with it.
 *
 * Orientation (PyTorch nn.Linear): W is [n][k] = d_out x d_in, row-major.
 * The paper writes Y = X W^C + (X L) R with W^C of shape d_in x d_out
 * (Sec. 3.2, "W ~= W^C + L R"); here the same product is written
 *     Y = X . dequant(Wq (.) M_2:4)^T + (X . R^T) . L^T
 * with L [n][r] and R [r][k] (L here = paper's R^T, R here = paper's L^T).
 *
 * Steps, each a direct transcription of its definition:
 *   mask      keep the 2 largest |w| of every 4 consecutive inputs
 *             (magnitude pruning to the 2:4 pattern; Sec. 4 lists it as the
 *             "Magnitude" baseline, Sec. 1 describes the 2:4 pattern).
 *   scale     AbsMax per output row (Sec. 2, "AbsMax"): s = max|w| / 7,
 *             one IEEE binary32 division.  An all-zero row gets s = 1.
 *   quantize  symmetric uniform quantization (Sec. 2 "Symmetric Quantization",
 *             Sec. 3.1 Eq. 2): code = round(w / s), binary32 quotient,
 *             round-half-to-even, clamped to the int4 range [-8, 7].
 *   pack      canonical byte layout (this build's own; the paper gives none):
 *             qvals[o][g]  = (c(i0) & 15) | ((c(i1) & 15) << 4)
 *             meta[o][g/2] = m4(even g) | (m4(odd g) << 4), m4 = i0 | (i1 << 2)
 *             where i0 < i1 are the kept in-group positions of group g.
 *   forward   fp64, no intermediate rounding:
 *             Y[m][o] = sum_k X[m][k] Wd[o][k]
 *                     + sum_j (sum_k X[m][k] R[j][k]) L[o][j]
 *
 * Build with IEEE semantics (no -ffast-math, no contraction): the build script
 * passes -O2 -fno-fast-math -ffp-contract=off.
 *
 * Every function is pinned by tests/test_oracle_*.py against brute force,
 * invariants, a hand-derived example and library special cases.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int slim_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- step 1: 2:4 magnitude mask ---------------------------------------- */

/* The two kept positions of one group of 4: order the positions by
 * (|w| descending, index ascending) and take the first two; return them as
 * i0 < i1.  -0.0 and +0.0 have the same magnitude. */
static void keep_two_of_four(const float *w, int *i0, int *i1)
{
    int first = 0;
    for (int i = 1; i < 4; ++i)
        if (fabsf(w[i]) > fabsf(w[first])) first = i;
    int second = -1;
    for (int i = 0; i < 4; ++i) {
        if (i == first) continue;
        if (second < 0 || fabsf(w[i]) > fabsf(w[second])) second = i;
    }
    if (first < second) { *i0 = first;  *i1 = second; }
    else                { *i0 = second; *i1 = first;  }
}

/* mask[o][k] = 1 where W[o][k] is kept.  k must be a multiple of 4. */
int slim_oracle_mask(const float *W, int64_t n, int64_t k, uint8_t *mask)
{
    if (!W || !mask || n <= 0 || k <= 0 || k % 4) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n; ++o) {
        const float *row = W + o * k;
        uint8_t *mrow = mask + o * k;
        memset(mrow, 0, (size_t)k);
        for (int64_t g = 0; g < k / 4; ++g) {
            int i0, i1;
            keep_two_of_four(row + 4 * g, &i0, &i1);
            mrow[4 * g + i0] = 1;
            mrow[4 * g + i1] = 1;
        }
    }
    return 0;
}

/* ---- step 2: per-row AbsMax scale -------------------------------------- */

int slim_oracle_scale(const float *W, int64_t n, int64_t k, float *scale)
{
    if (!W || !scale || n <= 0 || k <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n; ++o) {
        float a = 0.0f;
        for (int64_t j = 0; j < k; ++j) {
            float v = fabsf(W[o * k + j]);
            if (v > a) a = v;
        }
        scale[o] = (a == 0.0f) ? 1.0f : a / 7.0f;   /* one binary32 division */
    }
    return 0;
}

/* ---- step 3: symmetric int4 quantization of the kept entries ----------- */

/* codes[o][k] = clamp(rint(W[o][k] / scale[o]), -8, 7) where mask is set,
 * 0 elsewhere. */
int slim_oracle_quantize(const float *W, const uint8_t *mask, const float *scale,
                         int64_t n, int64_t k, int8_t *codes)
{
    if (!W || !mask || !scale || !codes || n <= 0 || k <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n; ++o) {
        const float s = scale[o];
        for (int64_t j = 0; j < k; ++j) {
            int8_t c = 0;
            if (mask[o * k + j]) {
                float q = W[o * k + j] / s;            /* binary32 quotient */
                float r = rintf(q);                    /* half to even      */
                if (r < -8.0f) r = -8.0f;
                if (r > 7.0f) r = 7.0f;
                c = (int8_t)r;
            }
            codes[o * k + j] = c;
        }
    }
    return 0;
}

/* ---- step 4: canonical packing ----------------------------------------- */

/* Needs exactly two mask bits per group of 4 and k % 8 == 0. */
int slim_oracle_pack(const int8_t *codes, const uint8_t *mask, int64_t n, int64_t k,
                     uint8_t *qvals, uint8_t *meta)
{
    if (!codes || !mask || !qvals || !meta || n <= 0 || k <= 0 || k % 8) return -1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t o = 0; o < n; ++o) {
        memset(meta + o * (k / 8), 0, (size_t)(k / 8));
        for (int64_t g = 0; g < k / 4; ++g) {
            int pos[4], cnt = 0;
            for (int i = 0; i < 4; ++i)
                if (mask[o * k + 4 * g + i]) pos[cnt++] = i;
            if (cnt != 2) { bad = 1; continue; }
            int i0 = pos[0], i1 = pos[1];
            unsigned c0 = (unsigned)codes[o * k + 4 * g + i0] & 0xFu;
            unsigned c1 = (unsigned)codes[o * k + 4 * g + i1] & 0xFu;
            qvals[o * (k / 4) + g] = (uint8_t)(c0 | (c1 << 4));
            unsigned m4 = (unsigned)i0 | ((unsigned)i1 << 2);
            meta[o * (k / 8) + g / 2] |= (uint8_t)(m4 << (4 * (g & 1)));
        }
    }
    return bad ? -2 : 0;
}

/* ---- step 5: unpack and dequantize ------------------------------------- */

static int sign_extend_nibble(unsigned v) { return (int)(v & 7u) - (int)(v & 8u); }

int slim_oracle_unpack(const uint8_t *qvals, const uint8_t *meta, int64_t n, int64_t k,
                       int8_t *codes, uint8_t *mask)
{
    if (!qvals || !meta || !codes || !mask || n <= 0 || k <= 0 || k % 8) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n; ++o) {
        memset(codes + o * k, 0, (size_t)k);
        memset(mask + o * k, 0, (size_t)k);
        for (int64_t g = 0; g < k / 4; ++g) {
            unsigned q = qvals[o * (k / 4) + g];
            unsigned m4 = (meta[o * (k / 8) + g / 2] >> (4 * (g & 1))) & 0xFu;
            int i0 = (int)(m4 & 3u), i1 = (int)(m4 >> 2);
            codes[o * k + 4 * g + i0] = (int8_t)sign_extend_nibble(q & 0xFu);
            mask[o * k + 4 * g + i0] = 1;
            /* a malformed nibble with i1 == i0 would overwrite: last wins */
            codes[o * k + 4 * g + i1] = (int8_t)sign_extend_nibble(q >> 4);
            mask[o * k + 4 * g + i1] = 1;
        }
    }
    return 0;
}

/* One dequantized row: wd[k] = code * scale in fp64, 0 at dropped positions. */
static void dequant_row(const uint8_t *qrow, const uint8_t *mrow, float s, int64_t k,
                        double *wd)
{
    for (int64_t j = 0; j < k; ++j) wd[j] = 0.0;
    for (int64_t g = 0; g < k / 4; ++g) {
        unsigned q = qrow[g];
        unsigned m4 = (mrow[g / 2] >> (4 * (g & 1))) & 0xFu;
        int i0 = (int)(m4 & 3u), i1 = (int)(m4 >> 2);
        wd[4 * g + i0] = (double)sign_extend_nibble(q & 0xFu) * (double)s;
        wd[4 * g + i1] = (double)sign_extend_nibble(q >> 4) * (double)s;
    }
}

/* Wd[n][k] fp64: the dense dequantized weight matrix. */
int slim_oracle_dequant(const uint8_t *qvals, const uint8_t *meta, const float *scale,
                        int64_t n, int64_t k, double *Wd)
{
    if (!qvals || !meta || !scale || !Wd || n <= 0 || k <= 0 || k % 8) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n; ++o)
        dequant_row(qvals + o * (k / 4), meta + o * (k / 8), scale[o], k, Wd + o * k);
    return 0;
}

/* ---- step 6: forward in fp64 -------------------------------------------- */

/* T[m][j] = sum_k X[m][k] R[j][k]   (adapter stage 1, no rounding). */
int slim_oracle_xr(const double *X, const double *R, int64_t m, int64_t k, int64_t r,
                   double *T)
{
    if (!X || !R || !T || m <= 0 || k <= 0 || r <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < r; ++j)
        for (int64_t i = 0; i < m; ++i) {
            double acc = 0.0;
            for (int64_t c = 0; c < k; ++c) acc += X[i * k + c] * R[j * k + c];
            T[i * r + j] = acc;
        }
    return 0;
}

/*
 * Y[i][t] for the output rows rows[0..nrows) (rows == NULL: all n rows, t = o).
 *   Y[i][t] = sum_k X[i][k] Wd[o][k] + sum_j T[i][j] L[o][j],  o = rows[t]
 * X [m][k], L [n][r], R [r][k] are fp64 copies of the fp16 inputs (exact).
 * r may be 0 (no adapters; L and R may then be NULL).  Y is [m][nrows].
 * T_out (may be NULL): receives T = X R^T [m][r] as it was used, for error budgets in tests.
 */
int slim_oracle_forward(const uint8_t *qvals, const uint8_t *meta, const float *scale,
                        const double *L, const double *R, const double *X,
                        int64_t n, int64_t k, int64_t r, int64_t m,
                        const int64_t *rows, int64_t nrows, double *Y, double *T_out)
{
    if (!qvals || !meta || !scale || !X || !Y) return -1;
    if (n <= 0 || k <= 0 || k % 8 || m <= 0 || r < 0) return -1;
    if (r > 0 && (!L || !R)) return -1;
    if (!rows) nrows = n;
    if (nrows <= 0) return -1;
    for (int64_t t = 0; rows && t < nrows; ++t)
        if (rows[t] < 0 || rows[t] >= n) return -1;

    double *T = NULL;
    if (r > 0) {
        T = (double *)malloc(sizeof(double) * (size_t)m * (size_t)r);
        if (!T) return -3;
        slim_oracle_xr(X, R, m, k, r, T);
        if (T_out) memcpy(T_out, T, sizeof(double) * (size_t)m * (size_t)r);
    }
    int fail = 0;
#pragma omp parallel
    {
        double *wd = (double *)malloc(sizeof(double) * (size_t)k);
        if (!wd) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(static)
            for (int64_t t = 0; t < nrows; ++t) {
                int64_t o = rows ? rows[t] : t;
                dequant_row(qvals + o * (k / 4), meta + o * (k / 8), scale[o], k, wd);
                for (int64_t i = 0; i < m; ++i) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < k; ++c) acc += X[i * k + c] * wd[c];
                    double lr = 0.0;
                    for (int64_t j = 0; j < r; ++j) lr += T[i * r + j] * L[o * r + j];
                    Y[i * nrows + t] = acc + lr;
                }
            }
        }
        free(wd);
    }
    free(T);
    return fail ? -3 : 0;
}
