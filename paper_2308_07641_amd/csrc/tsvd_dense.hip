// Stage U of a single token on the denser code of U (five ternary elements per byte, 1.6 bits per element
// instead of 2): the measurement behind the question the paper's discussion raises (it calls 2 bits per
// ternary element overly redundant).  Same arithmetic as tsvd_gemv_kernel<true>: the digit planes of z, the
// codes as fp4 operands of v_mfma_scale_f32_16x16x128_f8f6f4, exact integer sums, fp64 recombination.
// What differs is the decoding: a byte is looked up in a 256-entry table in LDS that returns its five 2-bit
// codes, the 64 ten-bit fields of a lane are concatenated into the 20 words of five tiles (five 16-row
// strips of one tile column), and from there on the three operations per word of the 2-bit path apply.
// One workgroup = one group of five strips (80 rows); wavefront w takes the tile columns w, w + 16, ...
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsvd_epilogue.h"
#include "tsvd_kernels.h"

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {
__device__ __forceinline__ f32x4 mfma_fp4_fp8(uint32_t w0, uint32_t w1, const u32x4& b0, const u32x4& b1, f32x4 acc) {
    const i32x8 a = {(int)((w0 << 2) & 0xCCCCCCCCu), (int)(w0 & 0xCCCCCCCCu),
                     (int)((w1 << 2) & 0xCCCCCCCCu), (int)(w1 & 0xCCCCCCCCu), 0, 0, 0, 0};
    const i32x8 b = {(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 4, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
}
__device__ __forceinline__ double pow2d(int e) { return __hiloint2double((1023 + e) << 20, 0); }
}  // namespace

// Dynamic LDS: digit planes [8][Kp + 16], table [256] u16, partial sums [16 wavefronts][80 rows][8] fp32.
__global__ void __launch_bounds__(1024)
tsvd_gemv_dense_kernel(tsvd_gemv_dense_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int pstride = p.Kp + 16;
    unsigned char* planes = smem;
    uint16_t* lut = reinterpret_cast<uint16_t*>(smem + (((size_t)8 * pstride + 255) & ~(size_t)255));
    float* red = reinterpret_cast<float*>(lut + 256);                 // [16][80][8]
    const int ex_in = p.meta[0];
    // digit planes of z: plane c copied by threads 128 c .. 128 c + 127, 16 bytes at a time
    {
        const int c = threadIdx.x >> 7, t = threadIdx.x & 127;
        const u32x4* src = reinterpret_cast<const u32x4*>(p.planes_in + (size_t)c * p.Kp);
        for (int ch = t; ch * 16 < p.Kp; ch += 128) *reinterpret_cast<u32x4*>(planes + (size_t)c * pstride + ch * 16) = src[ch];
    }
    if (threadIdx.x < 256) {
        // byte -> five 2-bit codes (trit 0 / 1 / 2 = element 0 / +1 / -1 = code 00 / 01 / 11); bytes above 242 never occur
        unsigned v = threadIdx.x, f = 0;
#pragma unroll
        for (int d = 0; d < 5; ++d) {
            const unsigned trit = v % 3u;
            v /= 3u;
            f |= (trit == 0u ? 0u : trit == 1u ? 1u : 3u) << (2 * d);
        }
        lut[threadIdx.x] = (uint16_t)f;
    }
    __syncthreads();

    const unsigned char* xlane = planes + (size_t)(i & 7) * pstride + 32 * g;
    f32x4 acc[5][2];
#pragma unroll
    for (int t = 0; t < 5; ++t) acc[t][0] = acc[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    const u32x4* gt = reinterpret_cast<const u32x4*>(p.dense) + ((size_t)blockIdx.x * p.nkt) * 256 + lane;
    for (int T = wave; T < p.nkt; T += 16) {
        u32x4 c[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] = __builtin_nontemporal_load(gt + (size_t)T * 256 + k * 64);
        // 64 bytes -> 64 ten-bit fields -> 20 words of 16 codes (tile t: words 4 t .. 4 t + 3)
        uint32_t W[20];
        unsigned long long bits = 0;
        int fill = 0, x = 0;
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            const uint32_t word = c[j >> 4][(j >> 2) & 3];
            const uint32_t byte = (word >> (8 * (j & 3))) & 0xFFu;
            bits |= (unsigned long long)lut[byte] << fill;
            fill += 10;
            if (fill >= 32) {
                W[x++] = (uint32_t)bits;
                bits >>= 32;
                fill -= 32;
            }
        }
        const u32x4* xb = reinterpret_cast<const u32x4*>(xlane + T * 256);
#pragma unroll
        for (int t = 0; t < 5; ++t) {
            acc[t][0] = mfma_fp4_fp8(W[4 * t], W[4 * t + 1], xb[0], xb[1], acc[t][0]);
            acc[t][1] = mfma_fp4_fp8(W[4 * t + 2], W[4 * t + 3], xb[8], xb[9], acc[t][1]);
        }
    }
    // result block of strip t: lane holds plane i (only 0..7 matter), rows 4 g + v
    if (i < 8) {
#pragma unroll
        for (int t = 0; t < 5; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[((size_t)wave * 80 + 16 * t + 4 * g + v) * 8 + i] = acc[t][0][v] + acc[t][1][v];
    }
    __syncthreads();
    if (threadIdx.x < 80) {
        const int row = blockIdx.x * 80 + threadIdx.x;
        if (row < p.M) {
            float s[8];
#pragma unroll
            for (int pc = 0; pc < 8; ++pc) {
                float part = 0.f;
                for (int w = 0; w < 16; ++w) part += red[((size_t)w * 80 + threadIdx.x) * 8 + pc];   // integers < 2^24: exact
                s[pc] = part;
            }
            double a = (double)s[7];
#pragma unroll
            for (int pc = 6; pc >= 0; --pc) a = a * 16.0 + (double)s[pc];
            const double val = a * pow2d(ex_in - 31);
            tsvd_store_y(p.y, (size_t)row * p.ldy, (float)(p.bias ? val + (double)p.bias[row] : val), p.out_bf16);
        }
    }
}

size_t tsvd_gemv_dense_lds(long long Kp) {
    return ((8 * (size_t)(Kp + 16) + 255) & ~(size_t)255) + 512 + (size_t)16 * 80 * 8 * sizeof(float);
}
hipError_t tsvd_gemv_dense_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemv_dense_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               TSVD_SKINNY_MAX_LDS);
}
hipError_t tsvd_launch_gemv_dense(const tsvd_gemv_dense_args& a, hipStream_t stream) {
    if (!a.dense || !a.planes_in || !a.meta || a.groups < 1 || a.nkt < 1 || a.Kp != a.nkt * 256 || a.groups * 80 < a.M ||
        tsvd_gemv_dense_lds(a.Kp) > TSVD_SKINNY_MAX_LDS)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(tsvd_gemv_dense_kernel, dim3(a.groups), dim3(1024), tsvd_gemv_dense_lds(a.Kp), stream, a);
    return hipGetLastError();
}
