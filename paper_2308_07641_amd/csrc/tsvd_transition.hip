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
__global__ void __launch_bounds__(256)
tsvd_gram_kernel(const int8_t* __restrict__ U, long long ldu, const int8_t* __restrict__ V, int M, int K, int N,
                 double* __restrict__ G) {
    const int l = blockIdx.x * 256 + threadIdx.x, k = blockIdx.y;
    if (l >= K) return;
    int uu = 0, vv = 0;
    for (int m = 0; m < M; ++m) uu += (int)U[(size_t)m * ldu + k] * (int)U[(size_t)m * ldu + l];
    const int8_t* vk = V + (size_t)k * N;
    const int8_t* vl = V + (size_t)l * N;
    for (int n = 0; n < N; ++n) vv += (int)vk[n] * (int)vl[n];
    G[(size_t)k * K + l] = (double)uu * (double)vv;
}

// ---- Eq. (3), right side: d[k] = sum_m sum_n U[m][k] W[m][n] V[k][n]; one workgroup per k ----------
__global__ void __launch_bounds__(256)
tsvd_rhs_kernel(const int8_t* __restrict__ U, long long ldu, const int8_t* __restrict__ V, const double* __restrict__ W, int M,
                int N, double* __restrict__ d) {
    __shared__ double red[256];
    const int k = blockIdx.x;
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
tsvd_pcg_kernel(const double* __restrict__ G, const double* __restrict__ d, int K, double* __restrict__ s, int* __restrict__ iters) {
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
    for (int k = tid; k < K; k += 1024) {
        const double g = G[(size_t)k * K + k];
        dg[k] = g > 0.0 ? 1.0 / g : 1.0;
        xs[k] = 0.0;
        r[k] = d[k];
        p[k] = r[k] * dg[k];
    }
    __syncthreads();
    const double dd = dot([&](int k) { return d[k] * d[k]; });
    double rz = dot([&](int k) { return r[k] * r[k] * dg[k]; });
    int it = 0;
    bool converged = !(dd > 0.0);
    const int max_it = 20 * K + 20;
    const int wave = tid >> 6, lane = tid & 63;
    while (!converged && it < max_it) {
        // q = G p: one wavefront per row, lanes along the row
        for (int k = wave; k < K; k += 16) {
            const double* row = G + (size_t)k * K;
            double v = 0.0;
            for (int l = lane; l < K; l += 64) v += row[l] * p[l];
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            if (lane == 0) q[k] = v;
        }
        __syncthreads();
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

// ---- leading singular pair by power iteration on R^T R, one workgroup -------------------------
// v <- R^T (R v) / |.| until the direction stops moving.  u and v live in LDS; R is re-read
// from L2 (row by row with one wavefront per row for R v, column-wise with coalesced rows for
// R^T y).
__global__ void __launch_bounds__(1024)
tsvd_power_kernel(const double* __restrict__ R, int M, int N, int max_iters, double* __restrict__ u_out, double* __restrict__ v_out,
                  double* __restrict__ sigma_out, int* __restrict__ iters_out) {
    extern __shared__ __align__(16) unsigned char smem[];
    double* v = reinterpret_cast<double*>(smem);    // [N]
    double* y = v + N;                              // [M]  R v
    double* z = y + M;                              // [N]  R^T y, then the next v
    double* part = z + N;                           // [4][N] partial column sums
    double* red = part + 4 * (size_t)N;             // [1024]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    auto dot = [&](auto f, int len) {
        double a = 0.0;
        for (int k = tid; k < len; k += 1024) a += f(k);
        red[tid] = a;
        __syncthreads();
        for (int st = 512; st > 0; st >>= 1) {
            if (tid < st) red[tid] += red[tid + st];
            __syncthreads();
        }
        const double out = red[0];
        __syncthreads();
        return out;
    };
    // a fixed start vector with no special symmetry
    for (int n = tid; n < N; n += 1024) v[n] = 1.0 + 0.5 * sin(1.0 + 0.7 * (double)n);
    __syncthreads();
    {
        const double nv = sqrt(dot([&](int k) { return v[k] * v[k]; }, N));
        for (int n = tid; n < N; n += 1024) v[n] /= nv;
        __syncthreads();
    }
    int it = 0;
    double sigma = 0.0;
    for (; it < max_iters; ++it) {
        for (int m = wave; m < M; m += 16) {                    // y = R v
            const double* row = R + (size_t)m * N;
            double a = 0.0;
            for (int n = lane; n < N; n += 64) a += row[n] * v[n];
            for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
            if (lane == 0) y[m] = a;
        }
        __syncthreads();
        {                                                       // z = R^T y: four row groups per column
            const int grp = tid >> 8, t = tid & 255;
            const int m0 = (int)(((long long)M * grp) / 4), m1 = (int)(((long long)M * (grp + 1)) / 4);
            for (int n = t; n < N; n += 256) {
                double a = 0.0;
                for (int m = m0; m < m1; ++m) a += R[(size_t)m * N + n] * y[m];
                part[(size_t)grp * N + n] = a;
            }
        }
        __syncthreads();
        for (int n = tid; n < N; n += 1024) z[n] = (part[n] + part[N + n]) + (part[2 * (size_t)N + n] + part[3 * (size_t)N + n]);
        __syncthreads();
        const double nz = sqrt(dot([&](int k) { return z[k] * z[k]; }, N));
        if (!(nz > 0.0)) break;                                 // R v = 0: R is zero (or v is in its null space)
        const double move = dot([&](int k) { const double dlt = z[k] / nz - v[k]; return dlt * dlt; }, N);
        for (int n = tid; n < N; n += 1024) v[n] = z[n] / nz;
        __syncthreads();
        if (move < 1e-24) {
            ++it;
            break;
        }
    }
    // u = R v / sigma with the final v
    for (int m = wave; m < M; m += 16) {
        const double* row = R + (size_t)m * N;
        double a = 0.0;
        for (int n = lane; n < N; n += 64) a += row[n] * v[n];
        for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
        if (lane == 0) y[m] = a;
    }
    __syncthreads();
    sigma = sqrt(dot([&](int k) { return y[k] * y[k]; }, M));
    for (int m = tid; m < M; m += 1024) u_out[m] = sigma > 0.0 ? y[m] / sigma : 0.0;
    for (int n = tid; n < N; n += 1024) v_out[n] = v[n];
    if (tid == 0) {
        sigma_out[0] = sigma;
        if (iters_out) iters_out[0] = it;
    }
}

int pow2_at_least(int64_t v) {
    int r = 1;
    while (r < v) r *= 2;
    return r;
}

}  // namespace

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
                       V_dev, (int)M, (int)K, (int)N, G);
    hipLaunchKernelGGL(tsvd_rhs_kernel, dim3((unsigned)K), dim3(256), 0, s, U_dev, (long long)ldu, V_dev, W_dev, (int)M, (int)N, d);
    const size_t lds = (size_t)5 * K * 8 + 1024 * 8;
    hipLaunchKernelGGL(tsvd_pcg_kernel, dim3(1), dim3(1024), lds, s, G, d, (int)K, S_dev, iters_dev);
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

extern "C" tsvd_status tsvd_leading_singular_pair(const double* R_dev, int64_t M, int64_t N, int32_t max_iters, double* u_dev,
                                                  double* v_dev, double* sigma_dev, int32_t* iters_dev, void* stream) {
    if (!R_dev || !u_dev || !v_dev || !sigma_dev || M < 1 || N < 1 || M > TERN_MAX_N || N > TERN_MAX_N || max_iters < 1)
        return TSVD_EINVAL;
    const size_t lds = ((size_t)6 * N + (size_t)M) * 8 + 1024 * 8;
    if (lds > 150 * 1024) return TSVD_EUNSUPPORTED;
    hipLaunchKernelGGL(tsvd_power_kernel, dim3(1), dim3(1024), lds, static_cast<hipStream_t>(stream), R_dev, (int)M, (int)N,
                       (int)max_iters, u_dev, v_dev, sigma_dev, iters_dev);
    return hipGetLastError() == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
}

hipError_t tsvd_transition_init() {
    hipError_t e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_ternarize_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TERN_MAX_N * 8 + 2 * 256 * 8)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_pcg_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 5 * FIT_MAX_K * 8 + 1024 * 8)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_residual_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 FIT_MAX_K * 8)) != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_power_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
}

extern "C" tsvd_status tsvd_transition(const double* W_dev, int64_t M, int64_t N, double theta, double tol, int64_t max_rank,
                                       int8_t* U_dev, double* S_dev, int8_t* V_dev, int64_t* rank_out, double* errors_host,
                                       void* stream) {
    if (!W_dev || !U_dev || !S_dev || !V_dev || !rank_out || M < 1 || N < 1 || M > TERN_MAX_N || N > TERN_MAX_N || max_rank < 1 ||
        max_rank > FIT_MAX_K || !(tol >= 0.0))
        return TSVD_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    *rank_out = 0;
    // scratch: R [M][N], u [M], v [N], t_u [M] int8, sigma, |R|^2, status[2], fit workspace
    const size_t bytes_R = round256((size_t)M * N * 8), bytes_u = round256((size_t)M * 8), bytes_v = round256((size_t)N * 8);
    const size_t bytes_tu = round256((size_t)M), bytes_misc = 256, bytes_fit = tsvd_fit_scales_workspace(max_rank);
    uint8_t* base = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&base), bytes_R + bytes_u + bytes_v + bytes_tu + bytes_misc + bytes_fit) != hipSuccess) {
        (void)hipGetLastError();
        return TSVD_EDEVICE;
    }
    double* R = reinterpret_cast<double*>(base);
    double* u = reinterpret_cast<double*>(base + bytes_R);
    double* v = reinterpret_cast<double*>(base + bytes_R + bytes_u);
    int8_t* tu = reinterpret_cast<int8_t*>(base + bytes_R + bytes_u + bytes_v);
    double* misc = reinterpret_cast<double*>(base + bytes_R + bytes_u + bytes_v + bytes_tu);   // [0] sigma, [1] |R|^2
    int32_t* flags = reinterpret_cast<int32_t*>(misc + 4);                                     // ternarize status x 2
    void* fit_ws = base + bytes_R + bytes_u + bytes_v + bytes_tu + bytes_misc;

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
        st = tsvd_leading_singular_pair(R, M, N, 4000, u, v, misc, nullptr, s);
        if (st != TSVD_OK) break;
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
        st = tsvd_fit_scales(U_dev, max_rank, V_dev, W_dev, M, K, N, S_dev, fit_ws, bytes_fit, nullptr, s);
        if (st != TSVD_OK) break;
        st = tsvd_residual(W_dev, U_dev, max_rank, S_dev, V_dev, M, K, N, R, misc + 1, s);
        if (st != TSVD_OK) break;
        double rnorm2 = 0.0;
        if (!ok(hipMemcpyAsync(&rnorm2, misc + 1, 8, hipMemcpyDeviceToHost, s)) || !ok(hipStreamSynchronize(s))) break;
        const double err = std::sqrt(rnorm2 / wnorm2);
        if (errors_host) errors_host[K - 1] = err;
        *rank_out = K;
        if (err <= tol) break;
    }
    (void)hipStreamSynchronize(s);
    (void)hipFree(base);
    return st;
}
