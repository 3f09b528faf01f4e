// Skinny path (one or two tokens per pass; the B = 1 weight-streaming case): one launch per
// stage of y = U (diag(S) (V x)) (paper, section "Truncated SVD in Network Compression";
// supplement Table S1: V(.) and U(.) are additions only, diag(S)(.) is K multiplications).
//
// The kernel is bound by HBM: every 2-bit code is read exactly once, 16 bytes per lane, 1 KiB
// per wavefront load.  To keep the vector ALU out of the way the codes are not expanded to
// 16- or 32-bit numbers.  Three ALU operations turn a 32-bit word (16 codes) into two
// registers of fp4 (E2M1) numbers 0 / +2 / -2, the A operand of
// v_mfma_scale_f32_16x16x128_f8f6f4.  The activations are converted once per workgroup to
// 31-bit fixed point relative to the token's largest magnitude and cut into eight balanced
// base-16 digits in [-8, 7]; each digit plane, stored as fp8 (E4M3, exact for these integers),
// is one of the MFMA's 16 output columns.  Every product is +-2 * digit and every sum is an
// integer below 2^24, so the matrix core performs exact integer additions and subtractions in
// its fp32 accumulators; the planes are recombined in fp64 (Horner in base 16) and scaled
// back.  Nothing but the fixed-point conversion of the activations (2^-31 of the token's
// largest magnitude) and the final rounding to fp32 is inexact.
//
// Stage V digitises x in the kernel, multiplies by S and writes z already digitised (with a
// power-of-two scale from the bound |z_k| <= max_k(|S_k| nnz(V[k,:])) * max|x|) so that stage U
// only copies digit planes into LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsvd_epilogue.h"
#include "tsvd_kernels.h"

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define NPRE 8   // tiles per wavefront whose loads are issued before the activations are staged

namespace {

__device__ __forceinline__ f32x4 mfma_step(uint32_t w0, uint32_t w1, const u32x4& b0, const u32x4& b1, f32x4 acc) {
    const i32x8 a = {(int)((w0 << 2) & 0xCCCCCCCCu), (int)(w0 & 0xCCCCCCCCu),
                     (int)((w1 << 2) & 0xCCCCCCCCu), (int)(w1 & 0xCCCCCCCCu), 0, 0, 0, 0};
    const i32x8 b = {(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
    // cbsz = 4: A is fp4 (E2M1); blgp = 0: B is fp8 (E4M3); both block scales 2^0
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 4, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
}

// xrow: LDS address of this lane's digit-plane row at (tile start + 32 * lane group).
__device__ __forceinline__ void tile_steps(const u32x4& w, const unsigned char* xrow, f32x4& acc0, f32x4& acc1) {
    const u32x4* xb = reinterpret_cast<const u32x4*>(xrow);
    acc0 = mfma_step(w.x, w.y, xb[0], xb[1], acc0);      // columns   0..127 of the tile
    acc1 = mfma_step(w.z, w.w, xb[8], xb[9], acc1);      // columns 128..255
}

// Eight balanced base-16 digits of a 31-bit fixed-point number as fp8 (E4M3) bytes,
// least significant digit in byte 0 of lo.
__device__ __forceinline__ void fixed_digits(int q, uint32_t& lo, uint32_t& hi) {
    const uint32_t t = (uint32_t)q + 0x88888888u;        // nibble p of t = digit p + 8
    float d[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) d[p] = (float)((int)((t >> (4 * p)) & 15u) - 8);
    int a = __builtin_amdgcn_cvt_pk_fp8_f32(d[0], d[1], 0, false);
    a = __builtin_amdgcn_cvt_pk_fp8_f32(d[2], d[3], a, true);
    int b = __builtin_amdgcn_cvt_pk_fp8_f32(d[4], d[5], 0, false);
    b = __builtin_amdgcn_cvt_pk_fp8_f32(d[6], d[7], b, true);
    lo = (uint32_t)a;
    hi = (uint32_t)b;
}

__device__ __forceinline__ int to_fixed(float v, int ex) {
    // |v| < 2^ex  ->  |q| <= 2^30
    return (int)rintf(ldexpf(v, 30 - ex));
}

// exponent ex with m < 2^ex (m >= 0 finite); 0 for m == 0
__device__ __forceinline__ int bound_exponent(float m) {
    int ex = 0;
    if (m > 0.f && m < 3.0e38f) (void)frexpf(m, &ex);
    return ex;
}

__device__ __forceinline__ float load_act(const void* in, int is_bf16, size_t off) {
    if (is_bf16) return __uint_as_float(((uint32_t) reinterpret_cast<const uint16_t*>(in)[off]) << 16);
    return reinterpret_cast<const float*>(in)[off];
}

}  // namespace

// Workgroup = sw strips x kw contraction splits, one wavefront each (sw * kw * 64 threads).
// Dynamic LDS: [8 * tokens planes][slab_k + 16] bytes, then [sw][kw][16][16] fp32, then 64 floats.
__global__ void __launch_bounds__(1024)
tsvd_skinny_kernel(tsvd_skinny_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;
    const int sidx = wave / p.kw;        // strip within the workgroup
    const int q = wave - sidx * p.kw;    // contraction split
    const int cols = p.tokens * 8;
    const int slab_k = p.slab_tiles * 256;
    const int xstride = slab_k + 16;     // bytes per digit-plane row; +16 spreads the rows over banks
    unsigned char* xs = smem;
    float* red = reinterpret_cast<float*>(smem + (((size_t)cols * xstride + 255) & ~(size_t)255));
    float* wmax = red + (size_t)p.sw * p.kw * 256;       // per-wave maxima, then per-token results

    const int strip = blockIdx.x * p.sw + sidx;
    const bool active = strip < p.strips;
    const int i = lane & 15, g = lane >> 4;
    const int col = i < cols ? i : cols - 1;             // surplus MFMA columns re-read the last plane
    const unsigned char* xlane = xs + (size_t)col * xstride + 32 * g;
    const u32x4* wp = reinterpret_cast<const u32x4*>(p.tiles) + ((size_t)(active ? strip : 0) * p.nkt) * 64 + lane;

    // ---- issue the first weight loads before anything else: they overlap the staging below
    const int first_end = min(p.slab_tiles, p.nkt);
    u32x4 pre[NPRE];
#pragma unroll
    for (int n = 0; n < NPRE; ++n) {
        const int T = q + n * p.kw;
        pre[n] = (active && T < first_end) ? __builtin_nontemporal_load(wp + (size_t)T * 64) : u32x4{0u, 0u, 0u, 0u};
    }

    // ---- per-token exponents of the fixed-point conversions
    int ex_in[2] = {0, 0}, ex_out[2] = {0, 0};
    if (p.mode == TSVD_SKINNY_STAGE_V) {
        float m0 = 0.f, m1 = 0.f;
        for (int idx = threadIdx.x; idx < p.kvalid * p.tokens; idx += blockDim.x) {
            const int k = idx / p.tokens, tok = idx - k * p.tokens;
            const float v = fabsf(load_act(p.in, p.in_is_bf16, (size_t)k * p.ld_in + tok));
            if (tok == 0) m0 = fmaxf(m0, v); else m1 = fmaxf(m1, v);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            m0 = fmaxf(m0, __shfl_xor(m0, o));
            m1 = fmaxf(m1, __shfl_xor(m1, o));
        }
        if (lane == 0) { wmax[2 * wave] = m0; wmax[2 * wave + 1] = m1; }
        __syncthreads();
        m0 = 0.f; m1 = 0.f;
        for (int w = 0; w < nwaves; ++w) { m0 = fmaxf(m0, wmax[2 * w]); m1 = fmaxf(m1, wmax[2 * w + 1]); }
        ex_in[0] = bound_exponent(m0);
        ex_in[1] = bound_exponent(m1);
        // |z| <= bound_V * max|x|; one more bit of room for the rounding of the bound itself
        ex_out[0] = bound_exponent(p.bound_V * m0) + 1;
        ex_out[1] = bound_exponent(p.bound_V * m1) + 1;
        if (blockIdx.x == 0 && threadIdx.x < p.tokens) p.meta_out[threadIdx.x] = threadIdx.x == 0 ? ex_out[0] : ex_out[1];
    } else {
        ex_in[0] = p.meta_in[0];
        ex_in[1] = p.tokens > 1 ? p.meta_in[1] : 0;
    }

    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};

    for (int t0 = 0; t0 < p.nkt; t0 += p.slab_tiles) {
        const int t1 = min(t0 + p.slab_tiles, p.nkt);
        const int kbeg = t0 * 256, kcnt = (t1 - t0) * 256;
        if (t0 > 0) __syncthreads();
        // ---- stage the digit planes of this slab
        if (p.mode == TSVD_SKINNY_STAGE_V) {
            for (int idx = threadIdx.x; idx < kcnt * p.tokens; idx += blockDim.x) {
                const int kk = idx / p.tokens, tok = idx - kk * p.tokens;
                const int k = kbeg + kk;
                uint32_t lo = 0, hi = 0;
                if (k < p.kvalid) {
                    const float v = load_act(p.in, p.in_is_bf16, (size_t)k * p.ld_in + tok);
                    fixed_digits(to_fixed(v, tok == 0 ? ex_in[0] : ex_in[1]), lo, hi);
                }
                unsigned char* dst = xs + (size_t)(tok * 8) * xstride + kk;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    dst[(size_t)d * xstride] = (unsigned char)(lo >> (8 * d));
                    dst[(size_t)(d + 4) * xstride] = (unsigned char)(hi >> (8 * d));
                }
            }
        } else {
            // digit planes were written by stage V: [cols][ld_in] bytes, 16-byte chunks
            const int chunks = kcnt / 16;
            for (int idx = threadIdx.x; idx < chunks * cols; idx += blockDim.x) {
                const int c = idx / chunks, ch = idx - c * chunks;
                const u32x4 v = *reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(p.in) + (size_t)c * p.ld_in + kbeg + ch * 16);
                *reinterpret_cast<u32x4*>(xs + (size_t)c * xstride + ch * 16) = v;
            }
        }
        __syncthreads();
        if (active) {
            int T = t0 + q;
            if (t0 == 0) {
#pragma unroll
                for (int n = 0; n < NPRE; ++n) {
                    const int Tn = q + n * p.kw;
                    if (Tn < t1) tile_steps(pre[n], xlane + Tn * 256, acc0, acc1);
                }
                T = q + NPRE * p.kw;
            }
            const int step = p.kw;
            for (; T + 3 * step < t1; T += 4 * step) {
                const u32x4 w0 = __builtin_nontemporal_load(wp + (size_t)T * 64);
                const u32x4 w1 = __builtin_nontemporal_load(wp + (size_t)(T + step) * 64);
                const u32x4 w2 = __builtin_nontemporal_load(wp + (size_t)(T + 2 * step) * 64);
                const u32x4 w3 = __builtin_nontemporal_load(wp + (size_t)(T + 3 * step) * 64);
                tile_steps(w0, xlane + (T - t0) * 256, acc0, acc1);
                tile_steps(w1, xlane + (T + step - t0) * 256, acc0, acc1);
                tile_steps(w2, xlane + (T + 2 * step - t0) * 256, acc0, acc1);
                tile_steps(w3, xlane + (T + 3 * step - t0) * 256, acc0, acc1);
            }
            for (; T < t1; T += step) {
                const u32x4 w0 = __builtin_nontemporal_load(wp + (size_t)T * 64);
                tile_steps(w0, xlane + (T - t0) * 256, acc0, acc1);
            }
        }
    }

    // ---- reduce the kw partial tiles, recombine the digit planes, scale, store.
    // D layout of the 16x16 MFMA: lane holds column i, rows 4 g + v.
    float* mine = red + ((size_t)(sidx * p.kw + q) * 256);
#pragma unroll
    for (int v = 0; v < 4; ++v) mine[(4 * g + v) * 16 + i] = acc0[v] + acc1[v];     // integers < 2^24: exact
    __syncthreads();
    for (int idx = threadIdx.x; idx < p.sw * 16 * p.tokens; idx += blockDim.x) {
        const int s = idx / (16 * p.tokens);
        const int rem = idx - s * 16 * p.tokens;
        const int r = rem / p.tokens, tok = rem - r * p.tokens;
        const int row = (blockIdx.x * p.sw + s) * 16 + r;
        if (row >= p.rows_out) continue;
        double acc = 0.0;
        for (int pc = 7; pc >= 0; --pc) {
            float part = 0.f;
            for (int qq = 0; qq < p.kw; ++qq) part += red[(size_t)(s * p.kw + qq) * 256 + r * 16 + tok * 8 + pc];
            acc = acc * 16.0 + (double)part;
        }
        // acc = 2 * sum_k A[row][k] * fixed(in[k]);  undo the factor 2 and the fixed-point scale
        const double val = ldexp(acc, (tok == 0 ? ex_in[0] : ex_in[1]) - 31);
        if (p.mode == TSVD_SKINNY_STAGE_V) {
            const float z = (float)((double)p.rowscale[row] * val);
            uint32_t lo, hi;
            fixed_digits(to_fixed(z, tok == 0 ? ex_out[0] : ex_out[1]), lo, hi);
            unsigned char* dst = static_cast<unsigned char*>(p.out) + (size_t)(tok * 8) * p.ld_out + row;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                dst[(size_t)d * p.ld_out] = (unsigned char)(lo >> (8 * d));
                dst[(size_t)(d + 4) * p.ld_out] = (unsigned char)(hi >> (8 * d));
            }
        } else {
            tsvd_store_y(p.out, p.out_token_major ? (size_t)tok * p.ld_out + row : (size_t)row * p.ld_out + tok,
                         (float)(p.bias ? val + (double)p.bias[row] : val), p.out_bf16);
        }
    }
}

hipError_t tsvd_skinny_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_skinny_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, TSVD_SKINNY_MAX_LDS);
}

size_t tsvd_skinny_lds_bytes(int tokens, int slab_tiles, int sw, int kw) {
    const size_t xbytes = (((size_t)8 * tokens * (slab_tiles * 256 + 16)) + 255) & ~(size_t)255;
    return xbytes + (size_t)sw * kw * 256 * sizeof(float) + 64 * sizeof(float);
}

hipError_t tsvd_launch_skinny(const tsvd_skinny_args& a, hipStream_t stream) {
    const size_t lds = tsvd_skinny_lds_bytes(a.tokens, a.slab_tiles, a.sw, a.kw);
    if (lds > TSVD_SKINNY_MAX_LDS || a.tokens < 1 || a.tokens > 2 || a.sw * a.kw > 16 || a.sw < 1 || a.kw < 1 ||
        a.slab_tiles < 1)
        return hipErrorInvalidValue;
    const int grid = (a.strips + a.sw - 1) / a.sw;
    hipLaunchKernelGGL(tsvd_skinny_kernel, dim3(grid), dim3(a.sw * a.kw * 64), lds, stream, a);
    return hipGetLastError();
}
