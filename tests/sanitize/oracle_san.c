/*
 * Driver for a build of the CPU oracle (oracle/cube3d_oracle.c) under AddressSanitizer and
 * UndefinedBehaviorSanitizer: every exported function on small, ragged and empty shapes, with
 * the operands in heap blocks of exactly the sizes the interface states, so that a read or
 * write one element outside them is reported.  Results are checked against values known in
 * closed form (integer data, all sums exact).  Exit status 0 = clean.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_matmul_nn(const double *X, const double *W, double *Y, int64_t M, int64_t K, int64_t N, int threads);
int oracle_matmul_nt(const double *dY, const double *W, double *dX, int64_t M, int64_t K, int64_t N, int threads);
int oracle_matmul_tn(const double *X, const double *dY, double *dW, int64_t M, int64_t K, int64_t N, int threads);
int oracle_matmul_nn_at(const double *X, const double *W, double *out, int64_t M, int64_t K, int64_t N,
                        const int64_t *rows, const int64_t *cols, int64_t n);
int oracle_matmul_nt_at(const double *dY, const double *W, double *out, int64_t M, int64_t K, int64_t N,
                        const int64_t *rows, const int64_t *cols, int64_t n);
int oracle_matmul_tn_at(const double *X, const double *dY, double *out, int64_t M, int64_t K, int64_t N,
                        const int64_t *rows, const int64_t *cols, int64_t n);
int oracle_max_threads(void);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

/* exactly n doubles (one byte for an empty operand, so that any element access is out of bounds) */
static double *block(int64_t n) { return (double *)malloc(n > 0 ? (size_t)n * sizeof(double) : 1); }

/* X[r,t] = r + 1, W[t,c] = c - 2, dY[r,c] = r - c:
 *   Y[r,c] = K (r+1)(c-2);  dX[r,t] = sum_c (r-c)(c-2);  dW[t,c] = sum_r (r+1)(r-c) */
static void one_shape(int64_t M, int64_t K, int64_t N, int threads)
{
    double *X = block(M * K), *W = block(K * N), *G = block(M * N);
    double *Y = block(M * N), *dX = block(M * K), *dW = block(K * N);
    for (int64_t r = 0; r < M; ++r) for (int64_t t = 0; t < K; ++t) X[r * K + t] = (double)(r + 1);
    for (int64_t t = 0; t < K; ++t) for (int64_t c = 0; c < N; ++c) W[t * N + c] = (double)(c - 2);
    for (int64_t r = 0; r < M; ++r) for (int64_t c = 0; c < N; ++c) G[r * N + c] = (double)(r - c);
    CHECK(oracle_matmul_nn(X, W, Y, M, K, N, threads) == 0);
    CHECK(oracle_matmul_nt(G, W, dX, M, K, N, threads) == 0);
    CHECK(oracle_matmul_tn(X, G, dW, M, K, N, threads) == 0);
    for (int64_t r = 0; r < M; ++r)
        for (int64_t c = 0; c < N; ++c) CHECK(Y[r * N + c] == (double)(K * (r + 1) * (c - 2)));
    for (int64_t r = 0; r < M; ++r) {
        double s = 0;
        for (int64_t c = 0; c < N; ++c) s += (double)((r - c) * (c - 2));
        for (int64_t t = 0; t < K; ++t) CHECK(dX[r * K + t] == s);
    }
    for (int64_t c = 0; c < N; ++c) {
        double s = 0;
        for (int64_t r = 0; r < M; ++r) s += (double)((r + 1) * (r - c));
        for (int64_t t = 0; t < K; ++t) CHECK(dW[t * N + c] == s);
    }
    if (M > 0 && K > 0 && N > 0) {
        /* the samplers at the four corners */
        int64_t rows[4] = {0, 0, M - 1, M - 1}, cols[4] = {0, N - 1, 0, N - 1}, kc[4] = {0, K - 1, 0, K - 1};
        int64_t kr[4] = {0, 0, K - 1, K - 1};
        double out[4];
        CHECK(oracle_matmul_nn_at(X, W, out, M, K, N, rows, cols, 4) == 0);
        for (int s = 0; s < 4; ++s) CHECK(out[s] == Y[rows[s] * N + cols[s]]);
        CHECK(oracle_matmul_nt_at(G, W, out, M, K, N, rows, kc, 4) == 0);
        for (int s = 0; s < 4; ++s) CHECK(out[s] == dX[rows[s] * K + kc[s]]);
        CHECK(oracle_matmul_tn_at(X, G, out, M, K, N, kr, cols, 4) == 0);
        for (int s = 0; s < 4; ++s) CHECK(out[s] == dW[kr[s] * N + cols[s]]);
        /* positions outside the output are refused, nothing is read */
        int64_t bad_r[1] = {M}, bad_c[1] = {0}, neg[1] = {-1};
        CHECK(oracle_matmul_nn_at(X, W, out, M, K, N, bad_r, bad_c, 1) == -1);
        CHECK(oracle_matmul_nt_at(G, W, out, M, K, N, bad_c, neg, 1) == -1);
        CHECK(oracle_matmul_tn_at(X, G, out, M, K, N, neg, bad_c, 1) == -1);
    }
    free(X); free(W); free(G); free(Y); free(dX); free(dW);
}

int main(void)
{
    const int64_t shapes[][3] = {{1, 1, 1}, {8, 8, 8}, {5, 3, 7}, {7, 1, 2}, {1, 9, 1}, {33, 17, 65}, {0, 4, 4}, {4, 0, 4},
                                 {4, 4, 0}, {0, 0, 0}, {64, 48, 32}};
    CHECK(oracle_max_threads() >= 1);
    for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s)
        for (int threads = 0; threads <= 5; threads += (threads ? 2 : 1))
            one_shape(shapes[s][0], shapes[s][1], shapes[s][2], threads);
    CHECK(oracle_matmul_nn(NULL, NULL, NULL, -1, 1, 1, 1) == -1);
    CHECK(oracle_matmul_nt(NULL, NULL, NULL, 1, -1, 1, 1) == -1);
    CHECK(oracle_matmul_tn(NULL, NULL, NULL, 1, 1, -1, 1) == -1);
    if (failures) { fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
    printf("oracle under sanitizers: ok\n");
    return 0;
}
