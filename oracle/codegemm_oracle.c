/*
 * CPU fp64 oracle for the codebook-quantized linear layer  y = x W^T.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call this file:
 * it exists so that the HIP kernels can be compared against a slow, plain,
 * independently written implementation of the definitions in the paper.
 * It shares no code, header, table or helper with the HIP path.
 *
 * What it computes, written out from the definitions (no Psumbook here):
 *
 *   W[n][v*j + k] = s[n][(v*j + k) / g] * sum_{c<m} C[c][ code[c][n][j] ][k]
 *       a weight vector of length v is the sum of m centroid vectors, each
 *       picked by its code (Section 2.2, additive multi-codebook paragraph);
 *       vectors are consecutive runs of v elements along K (Section 3,
 *       x^j_k = x_{v*j+k}); every run of g consecutive weights of a row (g/v
 *       vectors, g >= v) is de-normalised by its own scale (Section 2.2,
 *       Step 1); g = -1 means one scale per output row, s[n].
 *   y[b][n] = sum_{kk<K} x[b][kk] * W[n][kk]                     (y = x W^T)
 *   T[b][n] = sum_{kk<K} | x[b][kk] * W[n][kk] |                 (sum of |terms|)
 *
 * and, separately, the Psumbook of Section 3, Eq. 2:
 *
 *   P[b][c][j][i] = sum_{k<v} C[c][i][k] * x[b][v*j + k]
 *
 * Inputs are IEEE binary16 bit patterns; each is converted exactly to double.
 * Every sum is accumulated in double in index order.  Layouts (row-major):
 *   x[B][K] u16, codes[m][N][K/v] u8, codebooks[m][256][v] u16,
 *   scales[N] u16 (g = -1) or scales[N][K/g] u16 (g > 0, g a multiple of v dividing K),
 *   W[N][K] f64, y[B][N] f64, T[B][N] f64, P[B][m][K/v][256] f64.
 *
 * Pins (tests/test_oracle_*.py): exact rational brute force on tiny shapes,
 * the gather identity against a separate numpy Psumbook path, zero / one-hot /
 * +-1 codebooks (the last against an integer sign-matrix product), scale
 * linearity, row permutation, constant codes; for g > 0: g = K against g = -1,
 * per-group scale linearity, exact rational brute force with groups, one group
 * switched off against the same layer with that K range removed.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_CENTROIDS 256

/* IEEE 754 binary16 -> double, exact. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double mag;
    if (expo == 0) {
        mag = ldexp((double)frac, -24);               /* zero and subnormals */
    } else if (expo == 31) {
        mag = frac ? NAN : INFINITY;
    } else {
        mag = ldexp((double)(frac | 0x400), expo - 25);
    }
    return sign ? -mag : mag;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads the following calls use (n >= 1); only how the rows are shared out changes, no sum does. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static int bad_shape(int N, int K, int v, int m)
{
    return N < 1 || K < 1 || v < 1 || m < 1 || (K % v) != 0;
}

static int bad_group(int K, int v, int g)
{
    return !(g == -1 || (g >= v && (g % v) == 0 && (K % g) == 0));
}

/* One dequantized row of W, in double. */
static void dequantize_row(int n, int N, int K, int v, int m, int g,
                           const uint8_t *codes, const double *cb, const uint16_t *scales, double *w)
{
    const int J = K / v;
    for (int j = 0; j < J; ++j) {
        /* g is a multiple of v, so the v weights of vector j share the group (v * j) / g */
        const double scale = (g == -1) ? half_bits_to_double(scales[n])
                                       : half_bits_to_double(scales[(size_t)n * (K / g) + (v * j) / g]);
        for (int k = 0; k < v; ++k) {
            const int kk = v * j + k;
            double sum = 0.0;
            for (int c = 0; c < m; ++c) {
                int code = codes[((size_t)c * N + n) * J + j];
                sum += cb[((size_t)c * ORACLE_CENTROIDS + code) * v + k];
            }
            w[kk] = scale * sum;
        }
    }
}

static double *codebooks_to_double(int m, int v, const uint16_t *codebooks)
{
    size_t n = (size_t)m * ORACLE_CENTROIDS * v;
    double *cb = (double *)malloc(n * sizeof(double));
    if (cb)
        for (size_t i = 0; i < n; ++i) cb[i] = half_bits_to_double(codebooks[i]);
    return cb;
}

/* W[N][K] = dequantized weight matrix. */
int oracle_dequantize(int N, int K, int v, int m, int g, const uint8_t *codes,
                      const uint16_t *codebooks, const uint16_t *scales, double *W)
{
    if (bad_shape(N, K, v, m) || bad_group(K, v, g)) return -1;
    double *cb = codebooks_to_double(m, v, codebooks);
    if (!cb) return -2;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        dequantize_row(n, N, K, v, m, g, codes, cb, scales, W + (size_t)n * K);
    free(cb);
    return 0;
}

/* y = x W^T and T = sum of |terms|, dequantizing one row of W at a time. */
int oracle_gemm(int B, int N, int K, int v, int m, int g, const uint16_t *x, const uint8_t *codes,
                const uint16_t *codebooks, const uint16_t *scales, double *y, double *T)
{
    if (B < 1 || bad_shape(N, K, v, m) || bad_group(K, v, g)) return -1;
    double *cb = codebooks_to_double(m, v, codebooks);
    double *xd = (double *)malloc((size_t)B * K * sizeof(double));
    if (!cb || !xd) { free(cb); free(xd); return -2; }
    for (size_t i = 0; i < (size_t)B * K; ++i) xd[i] = half_bits_to_double(x[i]);
    int failed = 0;
#pragma omp parallel
    {
        double *w = (double *)malloc((size_t)K * sizeof(double));
        if (!w) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (int n = 0; n < N; ++n) {
                dequantize_row(n, N, K, v, m, g, codes, cb, scales, w);
                for (int b = 0; b < B; ++b) {
                    const double *xb = xd + (size_t)b * K;
                    double sum = 0.0, sum_abs = 0.0;
                    for (int kk = 0; kk < K; ++kk) {
                        double term = xb[kk] * w[kk];
                        sum += term;
                        sum_abs += fabs(term);
                    }
                    y[(size_t)b * N + n] = sum;
                    if (T) T[(size_t)b * N + n] = sum_abs;
                }
            }
        }
        free(w);
    }
    free(cb);
    free(xd);
    return failed ? -2 : 0;
}

/* Section 3, Eq. 2: P[b][c][j][i] = sum_k C[c][i][k] * x[b][v*j+k]. */
int oracle_psumbook(int B, int K, int v, int m, const uint16_t *x,
                    const uint16_t *codebooks, double *P)
{
    if (B < 1 || bad_shape(1, K, v, m)) return -1;
    const int J = K / v;
    double *cb = codebooks_to_double(m, v, codebooks);
    if (!cb) return -2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < J; ++j) {
            for (int c = 0; c < m; ++c) {
                for (int i = 0; i < ORACLE_CENTROIDS; ++i) {
                    double sum = 0.0;
                    for (int k = 0; k < v; ++k)
                        sum += cb[((size_t)c * ORACLE_CENTROIDS + i) * v + k] *
                               half_bits_to_double(x[(size_t)b * K + (size_t)v * j + k]);
                    P[(((size_t)b * m + c) * J + j) * ORACLE_CENTROIDS + i] = sum;
                }
            }
        }
    }
    free(cb);
    return 0;
}
