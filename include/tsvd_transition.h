/*
 * C ABI of the direct transition W -> (U, S, V) on the GPU: the steps of the paper's section
 * "Direct Transition Algorithm to TSVD form", each as its own call, and the loop that chains them.
 *
 * All matrices are DEVICE pointers, row-major; W and the residual are fp64 (the algorithm runs
 * once per layer, offline: it is latency-bound at the paper's matrix sizes, not throughput-bound),
 * ternary factors are int8 in {-1, 0, +1}.  Calls enqueue on `stream` (hipStream_t as void*,
 * NULL = default stream) and return without synchronising unless stated otherwise.  Status
 * codes are those of tsvd.h.  Caller keeps ownership of every buffer.
 */
#ifndef TSVD_TRANSITION_H
#define TSVD_TRANSITION_H

#include <stddef.h>
#include <stdint.h>

#include "tsvd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Algorithm 1, T(x, theta), for `count` vectors at once: t[v] is the sparsest ternary vector
 * whose angle to x[v] is at most theta, i.e. sign(x) on the q largest magnitudes for the smallest
 * q with (sum of the q largest |x_i|) / (sqrt(q) |x|) >= cos(theta)  (Eq. (tran_struct)); entries
 * tied with the q-th largest magnitude are kept.  The decision is taken in fp64.
 *   x_dev      : [count][ldx] fp64, n <= 8192 entries used per row.
 *   t_dev      : [count][ldt] int8, n entries written per row.
 *   status_dev : [count] int32: 0 = found, 1 = no ternary vector within theta (or x = 0): the row
 *                of t is then all zero.  The paper's algorithm raises an error in that case.
 * Returns TSVD_EINVAL for null pointers, n < 1, n > 8192, count < 1 or strides < n. */
tsvd_status tsvd_ternarize(const double* x_dev, int64_t n, int64_t count, int64_t ldx, double theta, int8_t* t_dev,
                           int64_t ldt, int32_t* status_dev, void* stream);

/* Eq. (3): S* = [(U^T U) o (V V^T)]^+ diag(U^T W V^T), the least-squares scales for fixed ternary
 * U [M][K] (row stride ldu >= K) and V [K][N] (row stride N) and W [M][N] fp64.  The K x K system is
 * solved by conjugate gradients with diagonal scaling in fp64, started from zero (for a singular
 * system this converges to the minimum-norm solution, which is what the pseudo-inverse gives).
 *   S_dev     : [K] fp64, written.
 *   workspace : device, at least tsvd_fit_scales_workspace(K) bytes, 256-byte aligned.
 *   iters_dev : optional int32[1]: iterations the solver took (negative: not converged).
 * K <= 2048. */
size_t tsvd_fit_scales_workspace(int64_t K);
tsvd_status tsvd_fit_scales(const int8_t* U_dev, int64_t ldu, const int8_t* V_dev, const double* W_dev, int64_t M, int64_t K,
                            int64_t N, double* S_dev, void* workspace, size_t workspace_bytes, int32_t* iters_dev, void* stream);

/* Last step of an iteration of Algorithm 2: R = W - U diag(S) V (fp64), and |R|_F^2 into
 * norm2_dev[0] (fp64; pass NULL to skip it). */
tsvd_status tsvd_residual(const double* W_dev, const int8_t* U_dev, int64_t ldu, const double* S_dev, const int8_t* V_dev,
                          int64_t M, int64_t K, int64_t N, double* R_dev, double* norm2_dev, void* stream);

/* First step of an iteration of Algorithm 2 for q = 1: the leading singular triple of R [M][N]
 * (the paper calls a full SVD and keeps the leading vectors; only those are needed), by
 * Golub-Kahan-Lanczos bidiagonalisation with full reorthogonalisation in fp64: tens of steps where
 * a power iteration needs thousands on the close singular values of a random matrix.  The small
 * bidiagonal problem is solved on the host, so the call SYNCHRONISES with the stream.  Stops when
 * the residual |R^T u - sigma v| of the pair is below 1e-12 sigma, restarting from the current
 * estimate every 128 steps, or after max_steps steps in total.
 *   u_dev [M], v_dev [N] : unit vectors; sigma_dev [1]; steps_dev optional int32[1].
 *   workspace : device, at least tsvd_leading_singular_pair_workspace(M, N) bytes, 256-byte aligned.
 * The sign of the pair (u, v) is arbitrary, as it is for any SVD routine.  M, N <= 8192. */
size_t tsvd_leading_singular_pair_workspace(int64_t M, int64_t N);
tsvd_status tsvd_leading_singular_pair(const double* R_dev, int64_t M, int64_t N, int32_t max_steps, double* u_dev,
                                       double* v_dev, double* sigma_dev, int32_t* steps_dev, void* workspace,
                                       size_t workspace_bytes, void* stream);

/* Algorithm 2 with q = 1, chaining the calls above: until |W - U diag(S) V|_F / |W|_F <= tol or
 * the rank reaches max_rank.  SYNCHRONISES with the stream once per iteration (the exit test
 * reads one number back).
 *   W_dev : [M][N] fp64.   U_dev : [M][max_rank] int8, V_dev : [max_rank][N] int8, S_dev :
 *   [max_rank] fp64: the first *rank_out columns / rows / entries are the result (U has row stride
 *   max_rank).   errors_host : optional host array [max_rank]: relative error after each iteration.
 * Inside the loop Eq. (3) is solved by conjugate gradients started from the previous scales (the new ones at 0).
 * For a non-singular Gram matrix that is the solution of Eq. (3); if two components coincide (a singular Gram
 * matrix) it is A least-squares optimum with the same residual, not necessarily the minimum-norm one that the
 * pseudo-inverse of Eq. (3) selects (tsvd_fit_scales, started from zero, gives that one).
 * Returns TSVD_EVALUE if some leading vector has no ternary vector within theta (the paper's
 * algorithm raises an error there); the components found so far are kept in *rank_out.
 * max_rank <= 2048, M, N <= 8192.  Allocates and frees its own device scratch. */
tsvd_status tsvd_transition(const double* W_dev, int64_t M, int64_t N, double theta, double tol, int64_t max_rank,
                            int8_t* U_dev, double* S_dev, int8_t* V_dev, int64_t* rank_out, double* errors_host,
                            void* stream);

/* Algorithm 2 with q components per iteration (the paper's q; its experiments use an adaptive q): every iteration
 * takes the q leading singular triples of the residual -- the leading triple of R, then of R minus that triple, and
 * so on (deflation in a working copy of R) --, ternarizes the 2 q vectors, appends the q components, refits all
 * scales (Eq. 3) and recomputes the residual.  The last iteration takes only what still fits below max_rank.
 * errors_host[k] is the relative error after the iteration that added component k.  If a vector of an iteration
 * has no ternary neighbour within theta the whole iteration is dropped (TSVD_EVALUE, *rank_out = rank before it).
 * 1 <= q <= min(M, N, max_rank); everything else as for tsvd_transition, which is this call with q = 1. */
tsvd_status tsvd_transition_q(const double* W_dev, int64_t M, int64_t N, double theta, double tol, int64_t max_rank, int64_t q,
                              int8_t* U_dev, double* S_dev, int8_t* V_dev, int64_t* rank_out, double* errors_host, void* stream);

#ifdef __cplusplus
}
#endif
#endif
