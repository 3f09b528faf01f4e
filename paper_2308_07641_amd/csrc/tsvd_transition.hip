// Direct transition W -> (U, S, V) on the GPU (paper, section "Direct Transition Algorithm to
// TSVD form": Algorithm 1, Eq. (3), Algorithm 2).  The algorithm runs once per layer and every
// step is small at the paper's matrix sizes ([512, 256] in its random-matrix study), so the steps
// are bound by launch and memory latency, not by arithmetic: each is one launch, the two
// iterative ones (power iteration, conjugate gradients) are single-workgroup kernels that keep
// their vectors in LDS and never return to the host inside the iteration.  Everything is fp64:
// the decisions of Algorithm 1 compare sums against cos(theta) and must not depend on fp32 noise.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>
#include <vector>

#include "../../include/tsvd_transition.h"

#define TERN_MAX_N 8192
#define FIT_MAX_K 2048

namespace {

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// Sum over the 256 threads of a workgroup, in a fixed order (tree in LDS); result in every thread.
__device__ __forceinline__ double block_sum256(double v, double* red) {
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const double r = red[0];
    __syncthreads();
    return r;
}

// ---- Algorithm 1: one workgroup per vector ---------------------------------------------------
// LDS: magnitudes [npow2] fp64, sorted largest first by a bitonic network (padding sorts last),
// then prefix sums in the order of the sorted list: thread t adds its chunk of npow2 / 256
// consecutive entries, thread 0 turns the 256 chunk sums into offsets, every thread walks its
// chunk again and reports the smallest q whose cosine reaches cos(theta).
__global__ void __launch_bounds__(256)
tsvd_ternarize_kernel(const double* __restrict__ x, long long ldx, int n, int npow2, double cos_theta,
                      int8_t* __restrict__ t, long long ldt, int* __restrict__ status) {
    extern __shared__ __align__(16) unsigned char smem[];
    double* keys = reinterpret_cast<double*>(smem);            // [npow2]
    double* red = keys + npow2;                                 // [256]
    double* offs = red + 256;                                   // [256]
    __shared__ int qmin;
    const int tid = threadIdx.x;
    const double* xr = x + (size_t)blockIdx.x * ldx;
    int8_t* tr = t + (size_t)blockIdx.x * ldt;
    if (tid == 0) qmin = 0x7FFFFFFF;
    double ss = 0.0;
    for (int i = tid; i < npow2; i += 256) {
        const double v = i < n ? xr[i] : 0.0;
        keys[i] = i < n ? fabs(v) : -1.0;
        ss += v * v;
    }
    const double length = sqrt(block_sum256(ss, red));
    for (int k = 2; k <= npow2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < npow2; i += 256) {
                const int l = i ^ j;
                if (l > i) {
                    const double a = keys[i], b = keys[l];
                    const bool largest_first = (i & k) == 0;
                    if (largest_first ? a < b : a > b) {
                        keys[i] = b;
                        keys[l] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    const int chunk = npow2 >= 256 ? npow2 / 256 : 1;
    const int first = tid * chunk;
    double mine = 0.0;
    if (first < npow2)
        for (int e = 0; e < chunk; ++e) mine += fmax(keys[first + e], 0.0);
    red[tid] = mine;
    __syncthreads();
    if (tid == 0) {
        double run = 0.0;
        for (int c = 0; c < 256; ++c) {
            offs[c] = run;
            run += red[c];
        }
    }
    __syncthreads();
    if (first < npow2 && length > 0.0) {
        double run = offs[tid];
        for (int e = 0; e < chunk; ++e) {
            const double key = keys[first + e];
            if (key < 0.0) break;                               // padding
            run += key;
            const int q = first + e + 1;
            if (run / (sqrt((double)q) * length) >= cos_theta) {
                atomicMin(&qmin, q);
                break;
            }
        }
    }
    __syncthreads();
    const int q = qmin;
    const bool found = q != 0x7FFFFFFF;
    const double threshold = found ? keys[q - 1] : 0.0;
    for (int i = tid; i < n; i += 256) {
        const double v = xr[i];
        tr[i] = (found && fabs(v) >= threshold) ? (v >= 0.0 ? 1 : -1) : 0;
    }
    if (tid == 0) status[blockIdx.x] = found ? 0 : 1;
}

// ---- Eq. (3), left side: G[k][l] = (sum_m U[m][k] U[m][l]) (sum_n V[k][n] V[l][n]) ------------------
// One thread per (k, l), l fastest (U[m][l] is then read along rows; V[l][n] is strided but V is
// small and cached).  Integer sums, exact.
// only_row >= 0: just row and column `only_row` (the component appended last; grid.y = 1).
__global__ void __launch_bounds__(256)
tsvd_gram_kernel(const int8_t* __restrict__ U, long long ldu, const int8_t* __restrict__ V, int M, int K, int N,
                 double* __restrict__ G, long long ldg, int only_row) {
    const int l = blockIdx.x * 256 + threadIdx.x, k = only_row >= 0 ? only_row : (int)blockIdx.y;
    if (l >= K) return;
    int uu = 0, vv = 0;
    for (int m = 0; m < M; ++m) uu += (int)U[(size_t)m * ldu + k] * (int)U[(size_t)m * ldu + l];
    const int8_t* vk = V + (size_t)k * N;
    const int8_t* vl = V + (size_t)l * N;
    for (int n = 0; n < N; ++n) vv += (int)vk[n] * (int)vl[n];
    G[(size_t)k * ldg + l] = (double)uu * (double)vv;
    if (only_row >= 0) G[(size_t)l * ldg + k] = (double)uu * (double)vv;
}

// ---- Eq. (3), right side: d[k] = sum_m sum_n U[m][k] W[m][n] V[k][n]; one workgroup per k ----------
__global__ void __launch_bounds__(256)
tsvd_rhs_kernel(const int8_t* __restrict__ U, long long ldu, const int8_t* __restrict__ V, const double* __restrict__ W, int M,
                int N, double* __restrict__ d, int k_first) {
    __shared__ double red[256];
    const int k = k_first + blockIdx.x;
    const int8_t* vk = V + (size_t)k * N;
    double acc = 0.0;
    for (int m = 0; m < M; ++m) {
        const int um = U[(size_t)m * ldu + k];
        if (um == 0) continue;                                  // (uniform over the workgroup)
        const double* wr = W + (size_t)m * N;
        double row = 0.0;
        for (int n = threadIdx.x; n < N; n += 256) row += (double)vk[n] * wr[n];
        acc += um > 0 ? row : -row;
    }
    const double total = block_sum256(acc, red);
    if (threadIdx.x == 0) d[k] = total;
}

// ---- Eq. (3), the solve: conjugate gradients with diagonal scaling, one workgroup -------------
// G s = d for the symmetric positive semi-definite G of the normal equations, started from s = 0,
// so for a singular G the iterates stay in its range and converge to the minimum-norm solution
// (the pseudo-inverse solution).  Vectors live in LDS; G (K^2 fp64) is re-read from L2 each
// iteration.  Stops at |r| <= 1e-13 |d| or after 20 K iterations.
__global__ void __launch_bounds__(1024)
// warm: start from the values found in s instead of zero (any least-squares solution gives the
// same residual; the loop of Algorithm 2 starts from the previous scales).
tsvd_pcg_kernel(const double* __restrict__ G, long long ldg, const double* __restrict__ d, int K, double* __restrict__ s, int warm,
                int* __restrict__ iters) {
    extern __shared__ __align__(16) unsigned char smem[];
    double* xs = reinterpret_cast<double*>(smem);   // [K] solution
    double* r = xs + K;                             // residual
    double* p = r + K;                              // direction
    double* q = p + K;                              // G p
    double* dg = q + K;                             // 1 / diagonal (1 where the diagonal is 0)
    double* red = dg + K;                           // [1024]
    const int tid = threadIdx.x;
    auto dot = [&](auto f) {                        // sum_k f(k), fixed order, result in every thread
        double v = 0.0;
        for (int k = tid; k < K; k += 1024) v += f(k);
        red[tid] = v;
        __syncthreads();
        for (int st = 512; st > 0; st >>= 1) {
            if (tid < st) red[tid] += red[tid + st];
            __syncthreads();
        }
        const double out = red[0];
        __syncthreads();
        return out;
    };
    const int wave = tid >> 6, lane = tid & 63;
    auto matvec = [&](const double* in, double* out) {          // out = G in: one wavefront per row, lanes along the row
        for (int k = wave; k < K; k += 16) {
            const double* row = G + (size_t)k * ldg;
            double v = 0.0;
            for (int l = lane; l < K; l += 64) v += row[l] * in[l];
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            if (lane == 0) out[k] = v;
        }
        __syncthreads();
    };
    for (int k = tid; k < K; k += 1024) {
        const double g = G[(size_t)k * ldg + k];
        dg[k] = g > 0.0 ? 1.0 / g : 1.0;
        xs[k] = warm ? s[k] : 0.0;
    }
    __syncthreads();
    if (warm) matvec(xs, q);
    for (int k = tid; k < K; k += 1024) {
        r[k] = d[k] - (warm ? q[k] : 0.0);
        p[k] = r[k] * dg[k];
    }
    __syncthreads();
    const double dd = dot([&](int k) { return d[k] * d[k]; });
    double rz = dot([&](int k) { return r[k] * r[k] * dg[k]; });
    int it = 0;
    bool converged = !(dd > 0.0);
    const int max_it = 20 * K + 20;
    if (dd > 0.0 && dot([&](int k) { return r[k] * r[k]; }) <= 1e-26 * dd) converged = true;    // (a warm start may already fit)
    while (!converged && it < max_it) {
        matvec(p, q);
        const double pq = dot([&](int k) { return p[k] * q[k]; });
        if (!(pq > 0.0)) break;                                 // direction in the null space: done
        const double alpha = rz / pq;
        for (int k = tid; k < K; k += 1024) {
            xs[k] += alpha * p[k];
            r[k] -= alpha * q[k];
        }
        __syncthreads();
        const double rr = dot([&](int k) { return r[k] * r[k]; });
        ++it;
        if (rr <= 1e-26 * dd) {
            converged = true;
            break;
        }
        const double rz_new = dot([&](int k) { return r[k] * r[k] * dg[k]; });
        const double beta = rz_new / rz;
        rz = rz_new;
        for (int k = tid; k < K; k += 1024) p[k] = r[k] * dg[k] + beta * p[k];
        __syncthreads();
    }
    for (int k = tid; k < K; k += 1024) s[k] = xs[k];
    if (tid == 0 && iters) iters[0] = converged ? it : -it;
}

// ---- residual: R = W - U diag(S) V and partial sums of |R|_F^2 ----------------------------------
// One workgroup per row m; the scaled row of U (S_k U[m][k], non-zero entries only) is gathered in
// LDS once, then every thread owns columns n, n + 256, ...
__global__ void __launch_bounds__(256)
tsvd_residual_kernel(const double* __restrict__ W, const int8_t* __restrict__ U, long long ldu, const double* __restrict__ S,
                     const int8_t* __restrict__ V, int K, int N, double* __restrict__ R, double* __restrict__ partial) {
    extern __shared__ __align__(16) unsigned char smem[];
    double* us = reinterpret_cast<double*>(smem);               // [K]
    __shared__ double red[256];
    const int m = blockIdx.x;
    for (int k = threadIdx.x; k < K; k += 256) us[k] = (double)U[(size_t)m * ldu + k] * S[k];
    __syncthreads();
    double ss = 0.0;
    for (int n = threadIdx.x; n < N; n += 256) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k) acc += us[k] * (double)V[(size_t)k * N + n];
        const double rv = W[(size_t)m * N + n] - acc;
        R[(size_t)m * N + n] = rv;
        ss += rv * rv;
    }
    const double total = block_sum256(ss, red);
    if (threadIdx.x == 0 && partial) partial[m] = total;
}

// Sum of `count` partial values in a fixed order (one workgroup).
__global__ void __launch_bounds__(256)
tsvd_sum_kernel(const double* __restrict__ partial, int count, double* __restrict__ out) {
    __shared__ double red[256];
    double v = 0.0;
    for (int i = threadIdx.x; i < count; i += 256) v += partial[i];
    const double total = block_sum256(v, red);
    if (threadIdx.x == 0) out[0] = total;
}

// ---- leading singular pair by Golub-Kahan-Lanczos bidiagonalisation ------------------------------------
// R V_k = U_k B_k with B_k upper bidiagonal (alpha on the diagonal, beta above it):
//   u_i = R v_i - beta_{i-1} u_{i-1},  alpha_i = |u_i|;   w = R^T u_i - alpha_i v_i,  beta_i = |w|,  v_{i+1} = w / beta_i,
// every new vector orthogonalised against all earlier ones (classical Gram-Schmidt, twice).  The
// leading singular triple of the small B_k (found on the host) gives that of R; for the close
// singular values of a random matrix this needs tens of steps where the power iteration needs
// thousands.  A step is four launches: the two matrix-vector products run on all compute units
// (tsvd_gkl_rv_kernel: a wavefront per row; tsvd_gkl_rtu_kernel: 64 columns x a slice of the rows per
// workgroup, partial sums), each followed by one workgroup that orthogonalises and normalises the new
// vector with it in LDS (tsvd_gkl_finish_kernel).  (One workgroup doing everything took 100 us per step on
// a [512, 256] matrix, 95 % of the transition's time.)  The bases ub [kmax][M], vb [kmax + 1][N] live in
// global memory (L2).
#define GKL_MAX_STEPS 128
#define GKL_ROW_SLICES 16

// uw[m] = sum_n R[m][n] v[n] - beta_prev * u_prev[m]: one wavefront per row (grid ceil(M / 4), block 256).
__global__ void __launch_bounds__(256)
tsvd_gkl_rv_kernel(const double* __restrict__ R, int M, int N, const double* __restrict__ v, const double* __restrict__ u_prev,
                   const double* __restrict__ beta_prev, double* __restrict__ uw) {
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (m >= M) return;
    const double* row = R + (size_t)m * N;
    double a0 = 0.0, a1 = 0.0;
    int n = lane;
    for (; n + 64 < N; n += 128) {
        a0 += row[n] * v[n];
        a1 += row[n + 64] * v[n + 64];
    }
    if (n < N) a0 += row[n] * v[n];
    double a = a0 + a1;
    for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
    if (lane == 0) uw[m] = a - (u_prev ? beta_prev[0] * u_prev[m] : 0.0);
}

// part[slice][n] = sum over the rows of the slice of R[m][n] u[m]: grid (ceil(N / 64), GKL_ROW_SLICES), block 256 =
// 64 columns x 4 row phases.
__global__ void __launch_bounds__(256)
tsvd_gkl_rtu_kernel(const double* __restrict__ R, int M, int N, const double* __restrict__ u, double* __restrict__ part) {
    __shared__ double red[4][64];
    const int col = blockIdx.x * 64 + (threadIdx.x & 63), phase = threadIdx.x >> 6;
    const int m0 = (int)(((long long)M * blockIdx.y) / GKL_ROW_SLICES), m1 = (int)(((long long)M * (blockIdx.y + 1)) / GKL_ROW_SLICES);
    double a0 = 0.0, a1 = 0.0;
    if (col < N) {
        int m = m0 + phase;
        for (; m + 4 < m1; m += 8) {
            a0 += R[(size_t)m * N + col] * u[m];
            a1 += R[(size_t)(m + 4) * N + col] * u[m + 4];
        }
        if (m < m1) a0 += R[(size_t)m * N + col] * u[m];
    }
    red[phase][threadIdx.x & 63] = a0 + a1;
    __syncthreads();
    if (phase == 0 && col < N) part[(size_t)blockIdx.y * N + col] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// One workgroup: x = (raw vector, or the sum of `slices` partial vectors minus scale[0] * sub) orthogonalised twice
// against basis[0 .. count), normalised, written to basis[count]; its norm to norm_out[0].  init: x is the fixed start
// vector instead (count = 0).
__global__ void __launch_bounds__(1024)
tsvd_gkl_finish_kernel(const double* __restrict__ raw, int slices, const double* __restrict__ sub, const double* __restrict__ scale,
                       int len, double* __restrict__ basis, int count, double* __restrict__ norm_out, int init) {
    extern __shared__ __align__(16) unsigned char smem[];
    double* x = reinterpret_cast<double*>(smem);    // [len]
    double* part = x + len;                         // [4][len] partial sums of the projections
    double* coef = part + 4 * (size_t)len;          // [GKL_MAX_STEPS + 1]
    double* red = coef + GKL_MAX_STEPS + 1;         // [1024]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (init) {                  // a fixed start vector with no special symmetry
        for (int n = tid; n < len; n += 1024) x[n] = 1.0 + 0.5 * sin(1.0 + 0.7 * (double)n);
    } else {
        const double sc = sub ? scale[0] : 0.0;
        for (int e = tid; e < len; e += 1024) {
            double a = raw[e];
            for (int q = 1; q < slices; ++q) a += raw[(size_t)q * len + e];
            x[e] = a - (sub ? sc * sub[e] : 0.0);
        }
    }
    __syncthreads();
    for (int pass = 0; pass < 2 && count > 0; ++pass) {
        // four basis vectors per wavefront at a time: their loads overlap
        for (int j0 = wave * 4; j0 < count; j0 += 64) {
            double a[4] = {0.0, 0.0, 0.0, 0.0};
            // (sixteen loads in flight per lane: the loop waits for L2, not for arithmetic; 4.07 -> 3.59 ms per iteration
            // of Algorithm 2 on a [512, 256] matrix; 32 in flight: 3.77)
            for (int e0 = lane; e0 < len; e0 += 256) {
                double b[4][4];
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int t = 0; t < 4; ++t) b[c][t] = basis[(size_t)min(j0 + t, count - 1) * len + min(e0 + 64 * c, len - 1)];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const double xe = e0 + 64 * c < len ? x[e0 + 64 * c] : 0.0;
#pragma unroll
                    for (int t = 0; t < 4; ++t) a[t] += b[c][t] * xe;
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                for (int o = 32; o > 0; o >>= 1) a[t] += __shfl_xor(a[t], o, 64);
                if (lane == 0 && j0 + t < count) coef[j0 + t] = a[t];
            }
        }
        __syncthreads();
        // x[e] -= sum_j coef[j] basis_j[e]: for short vectors the basis range is split over groups of threads
        const int groups = len <= 256 ? 4 : len <= 512 ? 2 : 1, per = 1024 / groups;
        const int grp = tid / per, t = tid - grp * per;
        const int j0 = (count * grp) / groups, j1 = (count * (grp + 1)) / groups;
        for (int e = t; e < len; e += per) {
            double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
            int j = j0;
            for (; j + 3 < j1; j += 4) {
                a0 += coef[j] * basis[(size_t)j * len + e];
                a1 += coef[j + 1] * basis[(size_t)(j + 1) * len + e];
                a2 += coef[j + 2] * basis[(size_t)(j + 2) * len + e];
                a3 += coef[j + 3] * basis[(size_t)(j + 3) * len + e];
            }
            for (; j < j1; ++j) a0 += coef[j] * basis[(size_t)j * len + e];
            part[(size_t)grp * len + e] = (a0 + a1) + (a2 + a3);
        }
        __syncthreads();
        for (int e = tid; e < len; e += 1024) {
            double a = x[e];
            for (int gq = 0; gq < groups; ++gq) a -= part[(size_t)gq * len + e];
            x[e] = a;
        }
        __syncthreads();
    }
    double ss = 0.0;
    for (int e = tid; e < len; e += 1024) ss += x[e] * x[e];
    red[tid] = ss;
    __syncthreads();
    for (int st = 512; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    const double nrm = sqrt(red[0]);
    for (int e = tid; e < len; e += 1024) basis[(size_t)count * len + e] = nrm > 0.0 ? x[e] / nrm : 0.0;
    if (tid == 0 && norm_out) norm_out[0] = nrm;
}

// x = sum_j c_j basis_j (j < count), normalised; one workgroup per output vector (blockIdx.x: 0 = u, 1 = v).
__global__ void __launch_bounds__(256)
tsvd_combine_kernel(const double* __restrict__ ub, const double* __restrict__ vb, const double* __restrict__ zc,
                    const double* __restrict__ yc, int count, int M, int N, double* __restrict__ u_out, double* __restrict__ v_out) {
    __shared__ double red[256];
    const bool left = blockIdx.x == 0;
    const double* basis = left ? ub : vb;
    const double* c = left ? zc : yc;
    double* out = left ? u_out : v_out;
    const int len = left ? M : N;
    double ss = 0.0;
    for (int e = threadIdx.x; e < len; e += 256) {
        double a = 0.0;
        for (int j = 0; j < count; ++j) a += c[j] * basis[(size_t)j * len + e];
        out[e] = a;
        ss += a * a;
    }
    const double nrm = sqrt(block_sum256(ss, red));
    for (int e = threadIdx.x; e < len; e += 256) out[e] = nrm > 0.0 ? out[e] / nrm : 0.0;
}

// Largest eigenpair of the symmetric tridiagonal matrix (diagonal d, off-diagonal e) of order k, on
// the host: bisection on the Sturm count, then inverse iteration with a pivoted tridiagonal solve.
double tridiagonal_top_eigenpair(const std::vector<double>& d, const std::vector<double>& e, int k, std::vector<double>& x) {
    double lo = 0.0, hi = 0.0;
    for (int i = 0; i < k; ++i) {
        const double r = (i > 0 ? std::fabs(e[i - 1]) : 0.0) + (i + 1 < k ? std::fabs(e[i]) : 0.0);
        hi = std::max(hi, d[i] + r);
        lo = std::min(lo, d[i] - r);
    }
    auto count_below = [&](double xq) {          // number of eigenvalues < xq
        int c = 0;
        double q = 1.0;
        for (int i = 0; i < k; ++i) {
            q = d[i] - xq - (i > 0 ? e[i - 1] * e[i - 1] / q : 0.0);
            if (q == 0.0) q = 1e-300;
            if (q < 0.0) ++c;
        }
        return c;
    };
    double a = lo, b = hi;
    for (int it = 0; it < 200 && b - a > 4e-16 * std::max(std::fabs(a), std::fabs(b)); ++it) {
        const double mid = 0.5 * (a + b);
        if (count_below(mid) >= k) b = mid; else a = mid;      // the largest eigenvalue lies in (a, b]
    }
    const double lam = 0.5 * (a + b);
    // inverse iteration: (T - lam I) x = rhs by Gaussian elimination with partial pivoting (band of width 2)
    x.assign(k, 0.0);
    std::vector<double> rhs(k);
    for (int i = 0; i < k; ++i) rhs[i] = 1.0 + 0.3 * std::sin(1.0 + (double)i);
    const double shift = lam + 1e-13 * std::max(std::fabs(lam), 1e-300);
    for (int round = 0; round < 4; ++round) {
        std::vector<double> dl(k, 0.0), dm(k), du(k, 0.0), du2(k, 0.0), bb = rhs;
        for (int i = 0; i < k; ++i) {
            dm[i] = d[i] - shift;
            if (i + 1 < k) { du[i] = e[i]; dl[i] = e[i]; }
        }
        for (int i = 0; i + 1 < k; ++i) {
            if (std::fabs(dm[i]) >= std::fabs(dl[i])) {
                if (dm[i] == 0.0) dm[i] = 1e-300;
                const double f = dl[i] / dm[i];
                dm[i + 1] -= f * du[i];
                bb[i + 1] -= f * bb[i];
                dl[i] = 0.0;
            } else {                                            // swap rows i and i + 1
                const double f = dm[i] / dl[i];
                dm[i] = dl[i];
                const double t1 = dm[i + 1];
                dm[i + 1] = du[i] - f * t1;
                du[i] = t1;
                if (i + 2 < k) {
                    du2[i] = du[i + 1];
                    du[i + 1] = -f * du2[i];
                }
                std::swap(bb[i], bb[i + 1]);
                bb[i + 1] -= f * bb[i];
            }
        }
        if (dm[k - 1] == 0.0) dm[k - 1] = 1e-300;
        x[k - 1] = bb[k - 1] / dm[k - 1];
        if (k > 1) x[k - 2] = (bb[k - 2] - du[k - 2] * x[k - 1]) / dm[k - 2];
        for (int i = k - 3; i >= 0; --i) x[i] = (bb[i] - du[i] * x[i + 1] - du2[i] * x[i + 2]) / dm[i];
        double nrm = 0.0;
        for (int i = 0; i < k; ++i) nrm += x[i] * x[i];
        nrm = std::sqrt(nrm);
        for (int i = 0; i < k; ++i) x[i] /= nrm;
        rhs = x;
    }
    return lam;
}

int pow2_at_least(int64_t v) {
    int r = 1;
    while (r < v) r *= 2;
    return r;
}

}  // namespace

// R[m][n] -= sigma u[m] v[n]: removes a converged singular triple, so that the next call for the leading pair
// returns the following one (Algorithm 2 with q > 1 takes the top q vectors of the same residual).
__global__ void __launch_bounds__(256)
tsvd_deflate_kernel(double* __restrict__ R, int M, int N, const double* __restrict__ u, const double* __restrict__ v,
                    const double* __restrict__ sigma) {
    const int m = blockIdx.y;
    const double f = sigma[0] * u[m];
    for (int n = blockIdx.x * 256 + threadIdx.x; n < N; n += gridDim.x * 256) R[(size_t)m * N + n] -= f * v[n];
}

extern "C" tsvd_status tsvd_ternarize(const double* x_dev, int64_t n, int64_t count, int64_t ldx, double theta, int8_t* t_dev,
                                      int64_t ldt, int32_t* status_dev, void* stream) {
    if (!x_dev || !t_dev || !status_dev || n < 1 || n > TERN_MAX_N || count < 1 || count > (1 << 30) || ldx < n || ldt < n)
        return TSVD_EINVAL;
    const int npow2 = pow2_at_least(n);
    const size_t lds = (size_t)npow2 * 8 + 2 * 256 * 8;
    hipLaunchKernelGGL(tsvd_ternarize_kernel, dim3((unsigned)count), dim3(256), lds, static_cast<hipStream_t>(stream), x_dev,
                       (long long)ldx, (int)n, npow2, std::cos(theta), t_dev, (long long)ldt, status_dev);
    return hipGetLastError() == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
}

extern "C" size_t tsvd_fit_scales_workspace(int64_t K) {
    if (K < 1 || K > FIT_MAX_K) return 0;
    return round256((size_t)K * (size_t)K * 8) + round256((size_t)K * 8);      // G, d
}

extern "C" tsvd_status tsvd_fit_scales(const int8_t* U_dev, int64_t ldu, const int8_t* V_dev, const double* W_dev, int64_t M,
                                       int64_t K, int64_t N, double* S_dev, void* workspace, size_t workspace_bytes,
                                       int32_t* iters_dev, void* stream) {
    if (!U_dev || !V_dev || !W_dev || !S_dev || !workspace || M < 1 || N < 1 || K < 1 || K > FIT_MAX_K || ldu < K ||
        M > (1 << 30) || N > (1 << 30))
        return TSVD_EINVAL;
    if (workspace_bytes < tsvd_fit_scales_workspace(K) || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return TSVD_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    double* G = static_cast<double*>(workspace);
    double* d = reinterpret_cast<double*>(static_cast<uint8_t*>(workspace) + round256((size_t)K * (size_t)K * 8));
    hipLaunchKernelGGL(tsvd_gram_kernel, dim3((unsigned)((K + 255) / 256), (unsigned)K), dim3(256), 0, s, U_dev, (long long)ldu,
                       V_dev, (int)M, (int)K, (int)N, G, (long long)K, -1);
    hipLaunchKernelGGL(tsvd_rhs_kernel, dim3((unsigned)K), dim3(256), 0, s, U_dev, (long long)ldu, V_dev, W_dev, (int)M, (int)N, d, 0);
    const size_t lds = (size_t)5 * K * 8 + 1024 * 8;
    hipLaunchKernelGGL(tsvd_pcg_kernel, dim3(1), dim3(1024), lds, s, G, (long long)K, d, (int)K, S_dev, 0, iters_dev);
    return hipGetLastError() == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
}

extern "C" tsvd_status tsvd_residual(const double* W_dev, const int8_t* U_dev, int64_t ldu, const double* S_dev,
                                     const int8_t* V_dev, int64_t M, int64_t K, int64_t N, double* R_dev, double* norm2_dev,
                                     void* stream) {
    if (!W_dev || !U_dev || !S_dev || !V_dev || !R_dev || M < 1 || N < 1 || K < 1 || K > FIT_MAX_K || ldu < K || M > (1 << 30) ||
        N > (1 << 30))
        return TSVD_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    double* partial = nullptr;
    if (norm2_dev) {
        // (the partial sums use the output matrix's own stream order: a scratch array per call)
        if (hipMallocAsync(reinterpret_cast<void**>(&partial), (size_t)M * 8, s) != hipSuccess) return TSVD_EDEVICE;
    }
    hipLaunchKernelGGL(tsvd_residual_kernel, dim3((unsigned)M), dim3(256), (size_t)K * 8, s, W_dev, U_dev, (long long)ldu, S_dev,
                       V_dev, (int)K, (int)N, R_dev, partial);
    if (norm2_dev) {
        hipLaunchKernelGGL(tsvd_sum_kernel, dim3(1), dim3(256), 0, s, partial, (int)M, norm2_dev);
        (void)hipFreeAsync(partial, s);
    }
    return hipGetLastError() == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
}

extern "C" size_t tsvd_leading_singular_pair_workspace(int64_t M, int64_t N) {
    if (M < 1 || N < 1 || M > TERN_MAX_N || N > TERN_MAX_N) return 0;
    return round256((size_t)GKL_MAX_STEPS * M * 8) + round256((size_t)(GKL_MAX_STEPS + 1) * N * 8) + 4 * round256(GKL_MAX_STEPS * 8) +
           round256((size_t)M * 8) + round256((size_t)GKL_ROW_SLICES * N * 8);      // raw R v, partial R^T u
}

extern "C" tsvd_status tsvd_leading_singular_pair(const double* R_dev, int64_t M, int64_t N, int32_t max_steps, double* u_dev,
                                                  double* v_dev, double* sigma_dev, int32_t* steps_dev, void* workspace,
                                                  size_t workspace_bytes, void* stream) {
    if (!R_dev || !u_dev || !v_dev || !sigma_dev || !workspace || M < 1 || N < 1 || M > TERN_MAX_N || N > TERN_MAX_N ||
        max_steps < 1)
        return TSVD_EINVAL;
    if (workspace_bytes < tsvd_leading_singular_pair_workspace(M, N) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return TSVD_EINVAL;
    auto finish_lds = [](int64_t len) { return ((size_t)5 * (size_t)len + GKL_MAX_STEPS + 1 + 1024) * 8; };
    if (finish_lds(std::max(M, N)) > 150 * 1024) return TSVD_EUNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* w8 = static_cast<uint8_t*>(workspace);
    double* ub = reinterpret_cast<double*>(w8);
    double* vb = reinterpret_cast<double*>(w8 + round256((size_t)GKL_MAX_STEPS * M * 8));
    double* alpha = reinterpret_cast<double*>(reinterpret_cast<uint8_t*>(vb) + round256((size_t)(GKL_MAX_STEPS + 1) * N * 8));
    double* beta = alpha + round256(GKL_MAX_STEPS * 8) / 8;
    double* zc = beta + round256(GKL_MAX_STEPS * 8) / 8;
    double* yc = zc + round256(GKL_MAX_STEPS * 8) / 8;
    double* uw = yc + round256(GKL_MAX_STEPS * 8) / 8;                          // R v_i before orthogonalisation
    double* wpart = uw + round256((size_t)M * 8) / 8;                           // [GKL_ROW_SLICES][N] partial R^T u_i
    const int kmax = (int)std::min<int64_t>(GKL_MAX_STEPS, std::min(M, N));   // the Krylov space cannot outgrow the matrix
    std::vector<double> ha(GKL_MAX_STEPS), hb(GKL_MAX_STEPS), d, e, y, z;
    int total = 0, fresh = 1;
    double theta = 0.0;
    for (;;) {
        int k = 0;
        bool done = false;
        while (!done) {
            const int k1 = std::min(kmax, k == 0 ? std::min(32, kmax) : k + 16);
            if (k == 0 && fresh)       // a restart finds its start vector in vb[0]
                hipLaunchKernelGGL(tsvd_gkl_finish_kernel, dim3(1), dim3(1024), finish_lds(N), s, static_cast<const double*>(nullptr), 0,
                                   static_cast<const double*>(nullptr), static_cast<const double*>(nullptr), (int)N, vb, 0,
                                   static_cast<double*>(nullptr), 1);
            for (int i = k; i < k1; ++i) {
                const double* vi = vb + (size_t)i * N;
                hipLaunchKernelGGL(tsvd_gkl_rv_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, s, R_dev, (int)M, (int)N, vi,
                                   i > 0 ? ub + (size_t)(i - 1) * M : static_cast<const double*>(nullptr), i > 0 ? beta + (i - 1) : beta, uw);
                hipLaunchKernelGGL(tsvd_gkl_finish_kernel, dim3(1), dim3(1024), finish_lds(M), s, uw, 1, static_cast<const double*>(nullptr),
                                   static_cast<const double*>(nullptr), (int)M, ub, i, alpha + i, 0);
                hipLaunchKernelGGL(tsvd_gkl_rtu_kernel, dim3((unsigned)((N + 63) / 64), GKL_ROW_SLICES), dim3(256), 0, s, R_dev, (int)M, (int)N,
                                   ub + (size_t)i * M, wpart);
                hipLaunchKernelGGL(tsvd_gkl_finish_kernel, dim3(1), dim3(1024), finish_lds(N), s, wpart, GKL_ROW_SLICES, vi, alpha + i, (int)N,
                                   vb, i + 1, beta + i, 0);
            }
            if (hipMemcpyAsync(ha.data(), alpha, (size_t)k1 * 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
                hipMemcpyAsync(hb.data(), beta, (size_t)k1 * 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess)
                return TSVD_EDEVICE;
            total += k1 - k;
            k = k1;
            // leading singular triple of the k x k upper bidiagonal B through T = B^T B
            d.assign(k, 0.0);
            e.assign(k > 1 ? k - 1 : 0, 0.0);
            for (int i = 0; i < k; ++i) {
                d[i] = ha[i] * ha[i] + (i > 0 ? hb[i - 1] * hb[i - 1] : 0.0);
                if (i + 1 < k) e[i] = ha[i] * hb[i];
            }
            const double lam = tridiagonal_top_eigenpair(d, e, k, y);
            theta = std::sqrt(std::max(lam, 0.0));
            z.assign(k, 0.0);
            for (int i = 0; i < k; ++i) z[i] = theta > 0.0 ? (ha[i] * y[i] + (i + 1 < k ? hb[i] * y[i + 1] : 0.0)) / theta : 0.0;
            const double resid = hb[k - 1] * std::fabs(z[k - 1]);        // |R^T u - theta v| of the Ritz pair
            done = resid <= 1e-12 * theta || k >= kmax || total >= max_steps || !(theta > 0.0);
            if (done) {
                if (hipMemcpyAsync(zc, z.data(), (size_t)k * 8, hipMemcpyHostToDevice, s) != hipSuccess ||
                    hipMemcpyAsync(yc, y.data(), (size_t)k * 8, hipMemcpyHostToDevice, s) != hipSuccess)
                    return TSVD_EDEVICE;
                hipLaunchKernelGGL(tsvd_combine_kernel, dim3(2), dim3(256), 0, s, ub, vb, zc, yc, k, (int)M, (int)N, u_dev, v_dev);
                if (hipStreamSynchronize(s) != hipSuccess) return TSVD_EDEVICE;    // (z, y are host vectors reused below)
                if (resid <= 1e-12 * theta || total >= max_steps || !(theta > 0.0) || kmax < GKL_MAX_STEPS) {
                    if (hipMemcpy(sigma_dev, &theta, 8, hipMemcpyHostToDevice) != hipSuccess) return TSVD_EDEVICE;
                    if (steps_dev && hipMemcpy(steps_dev, &total, 4, hipMemcpyHostToDevice) != hipSuccess) return TSVD_EDEVICE;
                    return hipGetLastError() == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
                }
            }
        }
        // not converged within the basis: restart from the current estimate of v
        if (hipMemcpyAsync(vb, v_dev, (size_t)N * 8, hipMemcpyDeviceToDevice, s) != hipSuccess) return TSVD_EDEVICE;
        fresh = 0;
    }
}

hipError_t tsvd_transition_init() {
    hipError_t e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_ternarize_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TERN_MAX_N * 8 + 2 * 256 * 8)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_pcg_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 5 * FIT_MAX_K * 8 + 1024 * 8)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_residual_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 FIT_MAX_K * 8)) != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gkl_finish_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
}

extern "C" tsvd_status tsvd_transition(const double* W_dev, int64_t M, int64_t N, double theta, double tol, int64_t max_rank,
                                       int8_t* U_dev, double* S_dev, int8_t* V_dev, int64_t* rank_out, double* errors_host,
                                       void* stream) {
    return tsvd_transition_q(W_dev, M, N, theta, tol, max_rank, 1, U_dev, S_dev, V_dev, rank_out, errors_host, stream);
}

extern "C" tsvd_status tsvd_transition_q(const double* W_dev, int64_t M, int64_t N, double theta, double tol, int64_t max_rank,
                                         int64_t q, int8_t* U_dev, double* S_dev, int8_t* V_dev, int64_t* rank_out,
                                         double* errors_host, void* stream) {
    if (!W_dev || !U_dev || !S_dev || !V_dev || !rank_out || M < 1 || N < 1 || M > TERN_MAX_N || N > TERN_MAX_N || max_rank < 1 ||
        max_rank > FIT_MAX_K || !(tol >= 0.0) || q < 1 || q > max_rank || q > std::min(M, N))
        return TSVD_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    *rank_out = 0;
    // scratch: R [M][N], u [M], v [N], t_u [M] int8, sigma, |R|^2, status[2], fit workspace
    const size_t bytes_R = round256((size_t)M * N * 8), bytes_u = round256((size_t)M * 8), bytes_v = round256((size_t)N * 8);
    const size_t bytes_tu = round256((size_t)M), bytes_misc = 256, bytes_fit = tsvd_fit_scales_workspace(max_rank);
    const size_t bytes_svd = tsvd_leading_singular_pair_workspace(M, N);
    const size_t bytes_defl = q > 1 ? bytes_R : 0;             // working copy of the residual for the second .. q-th triple
    uint8_t* base = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&base), bytes_R + bytes_u + bytes_v + bytes_tu + bytes_misc + bytes_fit + bytes_svd + bytes_defl) !=
        hipSuccess) {
        (void)hipGetLastError();
        return TSVD_EDEVICE;
    }
    double* R = reinterpret_cast<double*>(base);
    double* u = reinterpret_cast<double*>(base + bytes_R);
    double* v = reinterpret_cast<double*>(base + bytes_R + bytes_u);
    int8_t* tu = reinterpret_cast<int8_t*>(base + bytes_R + bytes_u + bytes_v);
    double* misc = reinterpret_cast<double*>(base + bytes_R + bytes_u + bytes_v + bytes_tu);   // [0] sigma, [1] |R|^2
    int32_t* flags = reinterpret_cast<int32_t*>(misc + 4);                                     // ternarize status x 2
    uint8_t* fit_ws = base + bytes_R + bytes_u + bytes_v + bytes_tu + bytes_misc;
    double* G = reinterpret_cast<double*>(fit_ws);                              // [max_rank][max_rank], grown row by row
    double* dvec = reinterpret_cast<double*>(fit_ws + round256((size_t)max_rank * (size_t)max_rank * 8));
    void* svd_ws = fit_ws + bytes_fit;
    double* Rwork = q > 1 ? reinterpret_cast<double*>(fit_ws + bytes_fit + bytes_svd) : nullptr;

    tsvd_status st = TSVD_OK;
    auto ok = [&](hipError_t e) {
        if (e != hipSuccess && st == TSVD_OK) st = TSVD_EDEVICE;
        return e == hipSuccess;
    };
    // |W|^2 and R = W: the residual of one all-zero component
    double wnorm2 = 0.0;
    ok(hipMemsetAsync(S_dev, 0, (size_t)max_rank * 8, s));
    ok(hipMemsetAsync(U_dev, 0, (size_t)M * max_rank, s));
    ok(hipMemsetAsync(V_dev, 0, (size_t)N, s));
    if (st == TSVD_OK) st = tsvd_residual(W_dev, U_dev, max_rank, S_dev, V_dev, M, 1, N, R, misc + 1, s);
    ok(hipMemcpyAsync(&wnorm2, misc + 1, 8, hipMemcpyDeviceToHost, s));
    ok(hipStreamSynchronize(s));
    int64_t K = 0;
    while (st == TSVD_OK && K < max_rank && wnorm2 > 0.0) {
        // the top q singular triples of the residual, one after the other: the leading triple of R, then of R with
        // that triple removed, ... (the last iteration takes what still fits below max_rank)
        const int64_t take = std::min<int64_t>(q, max_rank - K);
        if (take > 1 && !ok(hipMemcpyAsync(Rwork, R, (size_t)M * N * 8, hipMemcpyDeviceToDevice, s))) break;
        const int64_t K0 = K;
        for (int64_t j = 0; j < take && st == TSVD_OK; ++j) {
            const double* src = take > 1 ? Rwork : R;
            st = tsvd_leading_singular_pair(src, M, N, 4 * GKL_MAX_STEPS, u, v, misc, nullptr, svd_ws, bytes_svd, s);
            if (st != TSVD_OK) break;
            if (j + 1 < take) {
                hipLaunchKernelGGL(tsvd_deflate_kernel, dim3((unsigned)std::min<int64_t>(16, (N + 255) / 256), (unsigned)M), dim3(256), 0, s,
                                   Rwork, (int)M, (int)N, u, v, misc);
                if (!ok(hipGetLastError())) break;
            }
            // column K of U (row stride max_rank) is written through a contiguous temporary
            st = tsvd_ternarize(u, M, 1, M, theta, tu, M, flags, s);
            if (st != TSVD_OK) break;
            st = tsvd_ternarize(v, N, 1, N, theta, V_dev + (size_t)K * N, N, flags + 1, s);
            if (st != TSVD_OK) break;
            int32_t fl[2] = {0, 0};
            if (!ok(hipMemcpy2DAsync(U_dev + K, (size_t)max_rank, tu, 1, 1, (size_t)M, hipMemcpyDeviceToDevice, s))) break;
            if (!ok(hipMemcpyAsync(fl, flags, 8, hipMemcpyDeviceToHost, s)) || !ok(hipStreamSynchronize(s))) break;
            if (fl[0] != 0 || fl[1] != 0) {
                st = TSVD_EVALUE;                                   // no ternary vector within theta
                break;
            }
            ++K;
        }
        if (st != TSVD_OK) {
            K = K0;            // (the components of an unfinished iteration are dropped: *rank_out stays at the last complete one)
            break;
        }
        // Eq. (3) with what changed only: the new rows / columns of the Gram matrix and entries of the right
        // side; the solve starts from the previous scales (the new ones at 0, set when S was cleared)
        for (int64_t r = K0; r < K; ++r) {
            hipLaunchKernelGGL(tsvd_gram_kernel, dim3((unsigned)((K + 255) / 256), 1), dim3(256), 0, s, U_dev, (long long)max_rank, V_dev,
                               (int)M, (int)K, (int)N, G, (long long)max_rank, (int)r);
            hipLaunchKernelGGL(tsvd_rhs_kernel, dim3(1), dim3(256), 0, s, U_dev, (long long)max_rank, V_dev, W_dev, (int)M, (int)N, dvec,
                               (int)r);
        }
        hipLaunchKernelGGL(tsvd_pcg_kernel, dim3(1), dim3(1024), (size_t)5 * K * 8 + 1024 * 8, s, G, (long long)max_rank, dvec, (int)K,
                           S_dev, 1, static_cast<int*>(nullptr));
        if (!ok(hipGetLastError())) break;
        st = tsvd_residual(W_dev, U_dev, max_rank, S_dev, V_dev, M, K, N, R, misc + 1, s);
        if (st != TSVD_OK) break;
        double rnorm2 = 0.0;
        if (!ok(hipMemcpyAsync(&rnorm2, misc + 1, 8, hipMemcpyDeviceToHost, s)) || !ok(hipStreamSynchronize(s))) break;
        const double err = std::sqrt(rnorm2 / wnorm2);
        if (errors_host)
            for (int64_t r = K0; r < K; ++r) errors_host[r] = err;      // (one error per iteration, repeated for its components)
        *rank_out = K;
        if (err <= tol) break;
    }
    (void)hipStreamSynchronize(s);
    (void)hipFree(base);
    return st;
}
