/*
 * CPU oracle for the 3-D parallel linear layer: the plain matrix products.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or
 * call this file; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.  It shares no code with the HIP kernels.
 *
 * The 3-D scheme of the paper (Section 2.3, and Section 3.1.1 for the
 * load-balanced storage) is a block decomposition of the ordinary product: the
 * l-sum of the per-processor products A_il B_lj is C_ij, hence C = AB.  So the
 * oracle is the definition written out, once per product of the first
 * differentiation formula of Section 3.1.2:
 *
 *     C = AB,   dA = dC B^T,   dB = A^T dC.
 *
 * In the notation used in this repository (X = A, W = B, Y = C; X is [M,K],
 * W is [K,N], Y is [M,N]; all row-major):
 *
 *     Y [r,c] = sum_t X[r,t]  * W[t,c]
 *     dX[r,t] = sum_c dY[r,c] * W[t,c]
 *     dW[t,c] = sum_r X[r,t]  * dY[r,c]
 *
 * Every output element is accumulated in fp64 with the contraction index
 * ascending.  The loops are ordered so that the innermost one walks memory
 * contiguously; that changes which element is worked on when, never the order
 * of the additions that form one element.  No blocking, no BLAS.
 *
 * `threads` > 1 splits the outermost loop over OpenMP threads (each output
 * element is still produced by one thread, in the same order).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int clamp_threads(int threads)
{
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    return threads;
#else
    (void)threads;
    return 1;
#endif
}

/* Y = X W  (Section 3.1.2, first formula, C = AB). */
int oracle_matmul_nn(const double *X, const double *W, double *Y,
                     int64_t M, int64_t K, int64_t N, int threads)
{
    if (M < 0 || K < 0 || N < 0) return -1;
    threads = clamp_threads(threads);
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        double *y = Y + r * N;
        for (int64_t c = 0; c < N; ++c) y[c] = 0.0;
        for (int64_t t = 0; t < K; ++t) {
            const double x = X[r * K + t];
            const double *w = W + t * N;
            for (int64_t c = 0; c < N; ++c) y[c] += x * w[c];
        }
    }
    return 0;
}

/* dX = dY W^T  (Section 3.1.2, first formula, dA = dC B^T). */
int oracle_matmul_nt(const double *dY, const double *W, double *dX,
                     int64_t M, int64_t K, int64_t N, int threads)
{
    if (M < 0 || K < 0 || N < 0) return -1;
    threads = clamp_threads(threads);
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        const double *g = dY + r * N;
        for (int64_t t = 0; t < K; ++t) {
            const double *w = W + t * N;
            double acc = 0.0;
            for (int64_t c = 0; c < N; ++c) acc += g[c] * w[c];
            dX[r * K + t] = acc;
        }
    }
    return 0;
}

/* dW = X^T dY  (Section 3.1.2, first formula, dB = A^T dC). */
int oracle_matmul_tn(const double *X, const double *dY, double *dW,
                     int64_t M, int64_t K, int64_t N, int threads)
{
    if (M < 0 || K < 0 || N < 0) return -1;
    threads = clamp_threads(threads);
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t t = 0; t < K; ++t) {
        double *d = dW + t * N;
        for (int64_t c = 0; c < N; ++c) d[c] = 0.0;
        for (int64_t r = 0; r < M; ++r) {
            const double x = X[r * K + t];
            const double *g = dY + r * N;
            for (int64_t c = 0; c < N; ++c) d[c] += x * g[c];
        }
    }
    return 0;
}

/*
 * The same three definitions evaluated only at `n` listed output positions
 * (rows[s], cols[s]); used where the full output is too large to form on the
 * host.  Each sampled element is the full contraction, t ascending, in fp64.
 */
int oracle_matmul_nn_at(const double *X, const double *W, double *out,
                        int64_t M, int64_t K, int64_t N,
                        const int64_t *rows, const int64_t *cols, int64_t n)
{
    for (int64_t s = 0; s < n; ++s) {
        const int64_t r = rows[s], c = cols[s];
        if (r < 0 || r >= M || c < 0 || c >= N) return -1;
        double acc = 0.0;
        for (int64_t t = 0; t < K; ++t) acc += X[r * K + t] * W[t * N + c];
        out[s] = acc;
    }
    return 0;
}

int oracle_matmul_nt_at(const double *dY, const double *W, double *out,
                        int64_t M, int64_t K, int64_t N,
                        const int64_t *rows, const int64_t *cols, int64_t n)
{
    for (int64_t s = 0; s < n; ++s) {
        const int64_t r = rows[s], t = cols[s];
        if (r < 0 || r >= M || t < 0 || t >= K) return -1;
        double acc = 0.0;
        for (int64_t c = 0; c < N; ++c) acc += dY[r * N + c] * W[t * N + c];
        out[s] = acc;
    }
    return 0;
}

int oracle_matmul_tn_at(const double *X, const double *dY, double *out,
                        int64_t M, int64_t K, int64_t N,
                        const int64_t *rows, const int64_t *cols, int64_t n)
{
    for (int64_t s = 0; s < n; ++s) {
        const int64_t t = rows[s], c = cols[s];
        if (t < 0 || t >= K || c < 0 || c >= N) return -1;
        double acc = 0.0;
        for (int64_t r = 0; r < M; ++r) acc += X[r * K + t] * dY[r * N + c];
        out[s] = acc;
    }
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
