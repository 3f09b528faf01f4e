/*
 * CPU oracle for the Ternary-SVD forward map  y = U (diag(S) (V x)).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the GPU library, and nothing in the product path may call it.
 *
 * What it computes (paper, section "Truncated SVD in Network Compression":
 * the identity y = W x ~= U(diag(S)(V x)); section "Ternary SVD": U and V are
 * restricted to entries in {-1, 0, +1}; supplement Table S1: V(.) and U(.)
 * cost only additions, diag(S)(.) costs K multiplications):
 *
 *     for every token b:   t[k]    = sum_{n<N} V[k][n] * X[n][b]      k < K
 *                          z[k]    = S[k] * t[k]
 *                          Y[m][b] = sum_{k<K} U[m][k] * z[k]         m < M
 *
 * Shapes follow the paper: W is [M,N], U is [M,K], V is [K,N], S is [K],
 * x is [N,1], y is [M,1]; a batch is B independent columns.  All arithmetic
 * is IEEE double, loops run in natural index order, nothing is tiled, fused
 * or reordered.  Ternary entries are used as the integers -1, 0, +1.
 *
 * Pinned (tests/test_oracle_pins.py) by: the explicit dense product
 * (U diag(S) V) x, an independent brute-force triple sum on tiny shapes, a
 * hand-computed 2x2 example, special cases that reduce to library matmuls,
 * the 1-D Winograd F(2,3) instance of the paper's unfolded convolution
 * matrix, linearity / sign-flip / permutation invariants and the U = U+ - U-
 * bit-plane identity of the section "Connection with BNN".
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Returns 0 on success, 1 on a bad argument, 2 if U or V holds a value
 * outside {-1,0,+1}, 3 if scratch memory could not be obtained.
 *
 * U: int8 [M][K] row-major, V: int8 [K][N] row-major, S: float [K],
 * X: double [N][B] row-major (token index contiguous), Y: double [M][B]. */
int tsvd_oracle_forward(const int8_t *U, const float *S, const int8_t *V,
                        const double *X, double *Y,
                        int64_t M, int64_t K, int64_t N, int64_t B)
{
    if (!U || !S || !V || !X || !Y || M <= 0 || K <= 0 || N <= 0 || B <= 0)
        return 1;
    for (int64_t i = 0; i < M * K; ++i)
        if (U[i] < -1 || U[i] > 1) return 2;
    for (int64_t i = 0; i < K * N; ++i)
        if (V[i] < -1 || V[i] > 1) return 2;

    int failed = 0;
    /* Tokens are independent columns: the only parallelism used is over b. */
#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)K * sizeof(double));
        if (!z) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            if (!z) continue;
            for (int64_t k = 0; k < K; ++k) {
                double t = 0.0;
                for (int64_t n = 0; n < N; ++n)
                    t += (double)V[k * N + n] * X[n * B + b];
                z[k] = (double)S[k] * t;
            }
            for (int64_t m = 0; m < M; ++m) {
                double y = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    y += (double)U[m * K + k] * z[k];
                Y[m * B + b] = y;
            }
        }
        free(z);
    }
    return failed ? 3 : 0;
}

/* Single-token variant parallelised over output rows instead of tokens, so a
 * B = 1 call can use more than one core.  Same arithmetic, same order within
 * each sum.  z must hold K doubles of caller-owned scratch. */
int tsvd_oracle_forward_vec(const int8_t *U, const float *S, const int8_t *V,
                            const double *x, double *y, double *z,
                            int64_t M, int64_t K, int64_t N)
{
    if (!U || !S || !V || !x || !y || !z || M <= 0 || K <= 0 || N <= 0)
        return 1;
    for (int64_t i = 0; i < M * K; ++i)
        if (U[i] < -1 || U[i] > 1) return 2;
    for (int64_t i = 0; i < K * N; ++i)
        if (V[i] < -1 || V[i] > 1) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k) {
        double t = 0.0;
        for (int64_t n = 0; n < N; ++n)
            t += (double)V[k * N + n] * x[n];
        z[k] = (double)S[k] * t;
    }
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += (double)U[m * K + k] * z[k];
        y[m] = acc;
    }
    return 0;
}

/* Number of threads the parallel regions above use. */
int tsvd_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
