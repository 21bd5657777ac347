/*
 * Runs the CPU oracle (oracle/codegemm_oracle.c, included as source) under
 * AddressSanitizer and UndefinedBehaviorSanitizer: every buffer is allocated at
 * exactly the size the oracle's header documents, so a read or write one element
 * past any of them is reported; shapes are ragged on purpose.  Also checks two
 * properties that need no second implementation: a zero codebook gives y == 0
 * exactly, and with x = e_k (one-hot) y[n] equals column k of the dequantized W.
 * Built and run by tests/test_oracle_sanitizers.py; exit code 0 = clean.
 */
#include "../../oracle/codegemm_oracle.c"

#include <stdio.h>

static uint32_t rng_state = 12345u;
static uint32_t next_u32(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}

/* a finite fp16 bit pattern of modest magnitude: exponent 8..17 */
static uint16_t random_half(void)
{
    uint32_t r = next_u32();
    return (uint16_t)(((r & 1u) << 15) | ((8u + (r >> 1) % 10u) << 10) | ((r >> 8) & 0x3ffu));
}

static int run_case(int B, int N, int K, int v, int m, int g)
{
    const int J = K / v;
    const int G = (g == -1) ? 1 : K / g;
    uint16_t *x = malloc(sizeof(uint16_t) * (size_t)B * K);
    uint8_t *codes = malloc((size_t)m * N * J);
    uint16_t *cb = malloc(sizeof(uint16_t) * (size_t)m * ORACLE_CENTROIDS * v);
    uint16_t *scales = malloc(sizeof(uint16_t) * (size_t)N * G);
    double *y = malloc(sizeof(double) * (size_t)B * N);
    double *T = malloc(sizeof(double) * (size_t)B * N);
    double *W = malloc(sizeof(double) * (size_t)N * K);
    double *P = malloc(sizeof(double) * (size_t)B * m * J * ORACLE_CENTROIDS);
    int bad = 0;
    if (!x || !codes || !cb || !scales || !y || !T || !W || !P) return 1;
    for (size_t i = 0; i < (size_t)B * K; ++i) x[i] = random_half();
    for (size_t i = 0; i < (size_t)m * N * J; ++i) codes[i] = (uint8_t)next_u32();
    for (size_t i = 0; i < (size_t)m * ORACLE_CENTROIDS * v; ++i) cb[i] = random_half();
    for (size_t i = 0; i < (size_t)N * G; ++i) scales[i] = random_half();

    bad |= oracle_gemm(B, N, K, v, m, g, x, codes, cb, scales, y, T);
    bad |= oracle_dequantize(N, K, v, m, g, codes, cb, scales, W);
    bad |= oracle_psumbook(B, K, v, m, x, cb, P);
    for (size_t i = 0; i < (size_t)B * N; ++i)
        if (!(T[i] >= fabs(y[i]) * (1.0 - 1e-12))) bad |= 2;      /* sum of |terms| bounds |sum| */

    /* one-hot x in batch row 0: y[0][n] must be exactly W[n][k] */
    {
        const int k = (int)(next_u32() % (uint32_t)K);
        memset(x, 0, sizeof(uint16_t) * (size_t)K);
        x[k] = 0x3c00;                                            /* 1.0 */
        bad |= oracle_gemm(B, N, K, v, m, g, x, codes, cb, scales, y, T);
        for (int n = 0; n < N; ++n)
            if (y[n] != W[(size_t)n * K + k]) bad |= 4;
    }
    /* zero codebooks: y == 0 exactly */
    memset(cb, 0, sizeof(uint16_t) * (size_t)m * ORACLE_CENTROIDS * v);
    bad |= oracle_gemm(B, N, K, v, m, g, x, codes, cb, scales, y, T);
    for (size_t i = 0; i < (size_t)B * N; ++i)
        if (y[i] != 0.0 || T[i] != 0.0) bad |= 8;

    free(x); free(codes); free(cb); free(scales); free(y); free(T); free(W); free(P);
    if (bad) fprintf(stderr, "case B=%d N=%d K=%d v=%d m=%d g=%d: flags %d\n", B, N, K, v, m, g, bad);
    return bad;
}

int main(void)
{
    static const int cases[][6] = {
        /* B, N, K, v, m, g */
        {1, 1, 4, 4, 1, -1},   {1, 7, 8, 8, 1, -1},    {2, 33, 24, 8, 2, -1},  {3, 5, 20, 4, 3, -1},
        {1, 129, 264, 8, 4, -1}, {2, 17, 48, 16, 3, -1}, {1, 9, 64, 8, 2, 8},    {2, 11, 96, 4, 1, 32},
        {1, 3, 128, 16, 4, 64}, {5, 2, 40, 8, 1, 40},   {1, 64, 1032, 8, 2, -1},
    };
    int bad = 0;
    for (size_t i = 0; i < sizeof(cases) / sizeof(cases[0]); ++i)
        bad |= run_case(cases[i][0], cases[i][1], cases[i][2], cases[i][3], cases[i][4], cases[i][5]);
    /* arguments the oracle must refuse rather than touch memory for */
    if (oracle_gemm(1, 4, 10, 4, 1, -1, NULL, NULL, NULL, NULL, NULL, NULL) == 0) bad |= 16;      /* K % v != 0 */
    if (oracle_dequantize(4, 16, 4, 1, 6, NULL, NULL, NULL, NULL) == 0) bad |= 16;                /* g % v != 0 */
    if (bad) return 1;
    printf("oracle clean under sanitizers: %zu cases\n", sizeof(cases) / sizeof(cases[0]));
    return 0;
}
