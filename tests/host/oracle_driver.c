/* Exercise of the C oracle for a sanitizer build (address + undefined behaviour): every entry point on exactly
 * sized heap buffers (so that any access past an operand is caught), shapes from empty to a few ragged blocks,
 * every `ways`, one thread and several.  The block-wise routines must reproduce the definitions exactly on
 * the small-integer operands used here.  Exit code 0 = every expectation held. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_linear_rows(const float*, const float*, const float*, int64_t, int64_t, int64_t, int64_t, int64_t, double*, int);
int oracle_linear(const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, int);
int oracle_magnitude(const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, int);
int oracle_entries(const float*, const float*, const float*, int64_t, const int64_t*, const int64_t*, int64_t, double*, double*, int);
int oracle_jigsaw(int, const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, int);
int oracle_backward(const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, double*, int, int);
int oracle_jigsaw_backward(int, const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, double*, int);
int oracle_linear_xtw(const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, int, int);
int oracle_jigsaw_xtw(int, const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, int);
int oracle_linear_xw(const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, int, int);
int oracle_jigsaw_xw(int, const float*, const float*, const float*, int64_t, int64_t, int64_t, double*, int);
int oracle_gelu(const double*, int64_t, double*);
int oracle_mlp(const float*, const float*, const float*, const float*, const float*, int64_t, int64_t, int64_t, int,
               double*, double*, double*, double*, double*, int);
int oracle_layernorm(const float*, const float*, const float*, int64_t, int64_t, int64_t, double, double*, double*, int);
int oracle_round_bf16(const float*, int64_t, float*);

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

static uint64_t state = 88172645463325252ULL;
static int small_int(void)      /* -3 .. 3 */
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (int)(state % 7) - 3;
}
static float* ints(int64_t n)
{
    float* a = (float*)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
    for (int64_t i = 0; i < n; ++i) a[i] = (float)small_int();
    return a;
}
static double* out64(int64_t n) { return (double*)malloc((size_t)(n > 0 ? n : 1) * sizeof(double)); }
static int same(const double* a, const double* b, int64_t n) { return n == 0 || memcmp(a, b, (size_t)n * sizeof(double)) == 0; }

static void layer(int64_t M, int64_t K, int64_t N, int threads)
{
    float *X = ints(M * K), *W = ints(N * K), *Wt = ints(K * N), *b = ints(N), *G = ints(M * N);
    double *Y = out64(M * N), *Z = out64(M * N), *S = out64(M * N), *dX = out64(M * K), *dW = out64(N * K);
    double *eX = out64(M * K), *eW = out64(N * K);
    EXPECT(oracle_linear(X, W, b, M, K, N, Y, threads) == 0);
    EXPECT(oracle_magnitude(X, W, b, M, K, N, S, threads) == 0);
    for (int64_t i = 0; i < M * N; ++i) EXPECT(fabs(Y[i]) <= S[i]);
    if (M > 1) {
        EXPECT(oracle_linear_rows(X, W, b, M, K, N, 1, M, Z, threads) == 0);
        EXPECT(same(Z, Y + N, (M - 1) * N));
    }
    EXPECT(oracle_backward(X, W, G, M, K, N, dX, dW, 0, threads) == 0);
    for (int ways = 1; ways <= 4; ways *= 2) {
        const int ok = !(ways >= 2 && ((K | N) & 1)) && !(ways == 4 && (M & 1));
        EXPECT((oracle_jigsaw(ways, X, W, b, M, K, N, Z, threads) == 0) == ok);
        if (ok) EXPECT(same(Z, Y, M * N));
        EXPECT((oracle_jigsaw_backward(ways, X, W, G, M, K, N, eX, eW, threads) == 0) == ok);
        if (ok) EXPECT(same(eX, dX, M * K) && same(eW, dW, N * K));
    }
    /* the other two permutations on the same buffers: X^T W reads X as [M tokens x K channels], W := G [M x N] */
    double* T = out64(K * N);
    double* U = out64(K * N);
    EXPECT(oracle_linear_xtw(X, G, NULL, M, K, N, T, 0, threads) == 0);
    for (int ways = 1; ways <= 4; ways *= 2) {
        const int ok = !(ways >= 2 && ((K | N) & 1)) && !(ways == 4 && (M & 1));
        EXPECT((oracle_jigsaw_xtw(ways, X, G, NULL, M, K, N, U, threads) == 0) == ok);
        if (ok) EXPECT(same(U, T, K * N));
    }
    EXPECT(oracle_linear_xw(X, Wt, b, M, K, N, Y, 0, threads) == 0);
    for (int ways = 1; ways <= 4; ways *= 2) {
        const int ok = !(ways >= 2 && ((K | N) & 1)) && !(ways == 4 && (M & 1));
        EXPECT((oracle_jigsaw_xw(ways, X, Wt, b, M, K, N, Z, threads) == 0) == ok);
        if (ok) EXPECT(same(Z, Y, M * N));
    }
    free(X); free(W); free(Wt); free(b); free(G); free(Y); free(Z); free(S); free(dX); free(dW); free(eX); free(eW);
    free(T); free(U);
}

int main(void)
{
    const int64_t shapes[][3] = {{0, 0, 0}, {1, 1, 1}, {2, 2, 2}, {3, 5, 7}, {4, 6, 2}, {6, 2, 4}, {10, 14, 6}, {1, 8, 8},
                                 {33, 18, 20}};
    for (size_t s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s)
        for (int threads = 1; threads <= 5; threads += 4) layer(shapes[s][0], shapes[s][1], shapes[s][2], threads);

    /* sampled entries */
    {
        const int64_t K = 9, n = 5;
        float *Xr = ints(4 * K), *Wr = ints(3 * K), *bj = ints(n);
        const int64_t ix[5] = {0, 3, 3, 1, 2}, jw[5] = {2, 0, 2, 1, 1};
        double val[5], mag[5];
        EXPECT(oracle_entries(Xr, Wr, bj, K, ix, jw, n, val, mag, 3) == 0);
        for (int e = 0; e < 5; ++e) {
            double acc = bj[e];
            for (int64_t k = 0; k < K; ++k) acc += (double)Xr[ix[e] * K + k] * (double)Wr[jw[e] * K + k];
            EXPECT(acc == val[e] && fabs(val[e]) <= mag[e]);
        }
        free(Xr); free(Wr); free(bj);
    }
    /* point-wise pieces, the MLP and the layer norm on exactly sized buffers */
    {
        const int64_t M = 5, C = 6, Hd = 4;
        float *X = ints(M * C), *W1 = ints(Hd * C), *b1 = ints(Hd), *W2 = ints(C * Hd), *b2 = ints(C);
        double *H = out64(M * Hd), *Y = out64(M * C), *S1 = out64(M * Hd), *SY = out64(M * C), *PY = out64(M * C);
        for (int residual = 0; residual <= 1; ++residual)
            EXPECT(oracle_mlp(X, W1, b1, W2, b2, M, C, Hd, residual, H, Y, S1, SY, PY, 2) == 0);
        EXPECT(oracle_mlp(X, W1, NULL, W2, NULL, M, C, Hd, 1, H, Y, S1, SY, PY, 1) == 0);
        double in[4] = {-40.0, 0.0, 1.0, 40.0}, out[4];
        EXPECT(oracle_gelu(in, 4, out) == 0 && out[0] == 0.0 && out[1] == 0.0 && out[3] == 40.0);
        double *L = out64(M * C), *Sl = out64(M * C);
        float *gamma = ints(C), *beta = ints(C);
        for (int64_t groups = 1; groups <= 3; ++groups)
            EXPECT(oracle_layernorm(X, gamma, beta, M, C, groups, 1e-5, L, Sl, 2) == 0);
        EXPECT(oracle_layernorm(X, NULL, NULL, M, C, 1, 0.0, L, NULL, 1) == 0);
        EXPECT(oracle_layernorm(X, gamma, beta, M, C, 4, 1e-5, L, Sl, 1) != 0);      /* 6 channels do not split in 4 */
        float r[6] = {1.0f, 1.00390625f, -0.1f, 3.4e38f, 0.0f, -2.5f}, q[6];
        EXPECT(oracle_round_bf16(r, 6, q) == 0 && q[0] == 1.0f && q[1] == 1.0f && q[5] == -2.5f && isinf(q[3]));
        free(X); free(W1); free(b1); free(W2); free(b2); free(H); free(Y); free(S1); free(SY); free(PY);
        free(L); free(Sl); free(gamma); free(beta);
    }
    /* refused arguments come back as codes */
    {
        double y;
        float x = 1.f;
        EXPECT(oracle_linear(NULL, &x, NULL, 1, 1, 1, &y, 1) != 0);
        EXPECT(oracle_jigsaw(3, &x, &x, NULL, 1, 1, 1, &y, 1) != 0);
        EXPECT(oracle_linear_xw(&x, NULL, NULL, 1, 1, 1, &y, 0, 1) != 0);
    }
    printf("oracle driver: %d failures\n", failures);
    return failures ? 1 : 0;
}
