// Skinny path: out[rows][tokens] = post * rowscale[row] * (A [rows][kdim] . in [kdim][tokens])
// for at most 16 "columns" (tokens x bf16 parts), A a packed ternary matrix.
//
// Used for both stages of y = U (diag(S) (V x)) (paper, section "Truncated SVD in Network
// Compression"; cost per token in supplement Table S1: additions only in V(.) and U(.), K
// multiplications in diag(S)(.)) when the token count is small, in particular the B = 1
// weight-streaming case.  The kernel is bound by HBM: each 2-bit code is read once.
//
// Each wavefront owns a strip of 16 rows and walks tiles along the contraction index.  A
// tile is one coalesced 1 KiB load (16 bytes per lane).  A code pair becomes two 16-bit
// floats with one shift and one mask (+-2 or 0, identical bit patterns in bf16 and fp16) and
// eight v_mfma_f32_16x16x32_bf16 per tile accumulate in fp32; the MFMA's 16 output columns
// carry the tokens, and for fp32 activations their exact hi/mid/lo bf16 parts, so nothing
// is rounded before the fp32 accumulation.  Activations are staged once per workgroup in
// LDS, one row per column, contraction index contiguous.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsvd_kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define TSVD_DEC(w, j) ((((uint32_t)(w)) << (14 - 2 * (j))) & 0xC000C000u)

namespace {

__device__ __forceinline__ f32x4 mfma_step(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                           const u32x4& b, f32x4 acc) {
    u32x4 a = {a0, a1, a2, a3};
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

// One 32-bit word of codes = two k-steps of 32.
__device__ __forceinline__ void word_steps(uint32_t w, const u32x4& b0, const u32x4& b1,
                                           f32x4& acc0, f32x4& acc1) {
    acc0 = mfma_step(TSVD_DEC(w, 0), TSVD_DEC(w, 1), TSVD_DEC(w, 2), TSVD_DEC(w, 3), b0, acc0);
    acc1 = mfma_step(TSVD_DEC(w, 4), TSVD_DEC(w, 5), TSVD_DEC(w, 6), w & 0xC000C000u, b1, acc1);
}

// xrow: LDS pointer of this lane's column row at contraction offset (tile start + 8 g).
__device__ __forceinline__ void tile_steps(const u32x4& w, const uint16_t* xrow, f32x4& acc0, f32x4& acc1) {
    const u32x4* xb = reinterpret_cast<const u32x4*>(xrow);   // 16 bytes = 8 values; step q at +32 q values
    word_steps(w.x, xb[0], xb[4], acc0, acc1);
    word_steps(w.y, xb[8], xb[12], acc0, acc1);
    word_steps(w.z, xb[16], xb[20], acc0, acc1);
    word_steps(w.w, xb[24], xb[28], acc0, acc1);
}

__device__ __forceinline__ uint16_t bf16_trunc(float v) { return (uint16_t)(__float_as_uint(v) >> 16); }
__device__ __forceinline__ float bf16_widen(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t bf16_rne(float v) {
    uint32_t u = __float_as_uint(v);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

}  // namespace

// Workgroup = sw strips x kw contraction splits, one wavefront each (sw * kw * 64 threads).
// Dynamic LDS: [cols][slab_k + 8] bf16  followed by  [sw][kw][16 rows][16 cols] fp32.
__global__ void __launch_bounds__(1024)
tsvd_skinny_kernel(tsvd_skinny_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int sidx = wave / p.kw;        // strip within the workgroup
    const int q = wave - sidx * p.kw;    // contraction split
    const int cols = p.tokens * p.pieces;
    const int slab_k = p.slab_tiles * 256;
    const int xstride = slab_k + 8;      // in 16-bit units; +16 B keeps 16 rows on distinct banks
    uint16_t* xs = reinterpret_cast<uint16_t*>(smem);
    float* red = reinterpret_cast<float*>(smem + (((size_t)cols * xstride * 2 + 255) & ~(size_t)255));

    const int strip = blockIdx.x * p.sw + sidx;
    const bool active = strip < p.strips;
    const int i = lane & 15, g = lane >> 4;
    const int col = i < cols ? i : cols - 1;             // surplus MFMA columns re-read the last one
    const uint16_t* xlane = xs + (size_t)col * xstride + 8 * g;
    const u32x4* wp = reinterpret_cast<const u32x4*>(p.tiles) + ((size_t)(active ? strip : 0) * p.nkt) * 64 + lane;

    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};

    for (int t0 = 0; t0 < p.nkt; t0 += p.slab_tiles) {
        const int t1 = min(t0 + p.slab_tiles, p.nkt);
        const int kbeg = t0 * 256, kcnt = (t1 - t0) * 256;
        if (t0 > 0) __syncthreads();
        // ---- stage the activations of this slab: split into exact bf16 parts, zero-fill k >= kvalid
        for (int idx = threadIdx.x; idx < kcnt * p.tokens; idx += blockDim.x) {
            const int kk = idx / p.tokens, tok = idx - kk * p.tokens;
            const int k = kbeg + kk;
            uint16_t h0 = 0, h1 = 0, h2 = 0;
            if (k < p.kvalid) {
                const size_t off = (size_t)k * p.ld_in + tok;
                if (p.in_is_bf16) {
                    h0 = reinterpret_cast<const uint16_t*>(p.in)[off];
                } else {
                    const float v = reinterpret_cast<const float*>(p.in)[off];
                    if (p.pieces == 1) {
                        h0 = bf16_rne(v);
                    } else {
                        h0 = bf16_trunc(v);
                        const float r1 = v - bf16_widen(h0);          // exact
                        if (p.pieces == 2) {
                            h1 = bf16_rne(r1);
                        } else {
                            h1 = bf16_trunc(r1);
                            h2 = bf16_trunc(r1 - bf16_widen(h1));     // <= 8 significant bits: exact
                        }
                    }
                }
            }
            uint16_t* dst = xs + (size_t)(tok * p.pieces) * xstride + kk;
            dst[0] = h0;
            if (p.pieces > 1) dst[xstride] = h1;
            if (p.pieces > 2) dst[2 * xstride] = h2;
        }
        __syncthreads();
        if (active) {
            // ---- stream this wavefront's tiles, four loads in flight
            int T = t0 + q;
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

    // ---- reduce the kw partial tiles, add the parts of each token, scale, store
    // D layout of the 16x16 MFMA: lane holds column i, rows 4 g + v.
    float* mine = red + ((size_t)(sidx * p.kw + q) * 256);
    for (int v = 0; v < 4; ++v) mine[(4 * g + v) * 16 + i] = acc0[v] + acc1[v];
    __syncthreads();
    for (int idx = threadIdx.x; idx < p.sw * 16 * p.tokens; idx += blockDim.x) {
        const int s = idx / (16 * p.tokens);
        const int rem = idx - s * 16 * p.tokens;
        const int r = rem / p.tokens, tok = rem - r * p.tokens;
        const int row = (blockIdx.x * p.sw + s) * 16 + r;
        if (row >= p.rows_valid) continue;
        float sum = 0.f;
        for (int pc = p.pieces - 1; pc >= 0; --pc) {      // smallest parts first
            float part = 0.f;
            for (int qq = 0; qq < p.kw; ++qq) part += red[(size_t)(s * p.kw + qq) * 256 + r * 16 + tok * p.pieces + pc];
            sum += part;
        }
        float f = p.post;
        if (p.rowscale) f *= p.rowscale[row];
        p.out[(size_t)row * p.ld_out + tok] = sum * f;
    }
}

hipError_t tsvd_skinny_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_skinny_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, TSVD_SKINNY_MAX_LDS);
}

hipError_t tsvd_launch_skinny(const tsvd_skinny_args& a, hipStream_t stream) {
    const int cols = a.tokens * a.pieces;
    const size_t xbytes = (((size_t)cols * (a.slab_tiles * 256 + 8) * 2) + 255) & ~(size_t)255;
    const size_t lds = xbytes + (size_t)a.sw * a.kw * 256 * sizeof(float);
    if (lds > TSVD_SKINNY_MAX_LDS || cols < 1 || cols > 16 || a.sw * a.kw > 16 || a.sw < 1 || a.kw < 1)
        return hipErrorInvalidValue;
    const int grid = (a.strips + a.sw - 1) / a.sw;
    hipLaunchKernelGGL(tsvd_skinny_kernel, dim3(grid), dim3(a.sw * a.kw * 64), lds, stream, a);
    return hipGetLastError();
}
