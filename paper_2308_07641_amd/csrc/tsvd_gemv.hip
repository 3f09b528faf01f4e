// Fast single-token path (B = 1): the two stages of y = U (diag(S) (V x)) (paper, section
// "Truncated SVD in Network Compression"; supplement Table S1: V(.) and U(.) are additions only,
// diag(S)(.) is K multiplications), one launch each, 16 wavefronts per workgroup and about one
// workgroup per compute unit.
//
// Arithmetic.  The 2-bit codes are never widened to 16 or 32 bits: three ALU operations turn a
// 32-bit word (16 codes) into two registers of fp4 (E2M1) numbers 0 / +2 / -2, the A operand of
// v_mfma_scale_f32_16x16x128_f8f6f4.  The activation vector is converted to sign-magnitude
// 30-bit fixed point relative to its largest magnitude and cut into eight base-16 digits; digit
// plane p (sign * digit, exact in fp8 E4M3) is column p of the MFMA's B operand.  Every product
// is +-2 * digit and every sum an integer below 2^24, so the matrix core performs exact integer
// additions and subtractions in its fp32 accumulators; the eight planes are recombined in fp64
// (Horner, base 16) and scaled back.  Only the fixed-point conversion (2^-31 of the largest
// magnitude) and the final rounding to fp32 are inexact.
//
// Schedule.  At B = 1 a call lasts a few microseconds and every instruction of the prologue is
// executed by all 16 wavefronts of a compute unit, so the code is kept short and every serial
// round trip to memory counts.  Vector-memory results return to a wavefront in issue order:
// each wavefront issues its loads at entry in the order it needs them, first the small,
// latency-critical activations (x, or the digit planes of z written by stage V), and once those
// have arrived its first weight tiles; the rest are streamed with a fixed number in flight (NPRE
// below: requesting everything at once made every load slower).  The activations are staged in LDS while the
// weights are in flight.  Stage V multiplies by S and writes z already digitised (power-of-two
// scale from the bound |z_k| <= max_k(|S_k| nnz(V[k,:])) * max|x|), so stage U only copies planes.
// (Measured on MI355X: a device-wide barrier inside one launch costs 4 us or more with
// agent-scope atomics and fences, more than the boundary between two launches, so the stages
// are separate launches.)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "tsvd_epilogue.h"
#include "tsvd_kernels.h"

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Weight tiles per wavefront in flight.  16 wavefronts x 256 compute units x 2 KiB = 8.4 MB is
// about the bandwidth-delay product of the memory system; with 8 in flight (all 33.5 MB of the
// decode workload requested in the first microsecond) every load, the activations included, came
// back later: 17.0 us per token against 13.9 us.
#ifndef NPRE
#define NPRE 2
#endif
#define XR_MAX 4     // x: groups of 4 consecutive elements per thread  (N <= 16384)
#define ZR_MAX 8     // z planes: 16-byte chunks per thread             (K <= 16384)

// Optional phase timestamps (100 MHz wall clock) of thread 0 of every workgroup, for tuning.
#define TICK(n) do { if (p.clocks && threadIdx.x == 0 && blockIdx.x < TSVD_GEMV_MAX_GRID) p.clocks[blockIdx.x * 16 + (n)] = wall_clock64(); } while (0)

namespace {

__device__ __forceinline__ f32x4 mfma_step(uint32_t w0, uint32_t w1, const u32x4& b0, const u32x4& b1, f32x4 acc) {
    const i32x8 a = {(int)((w0 << 2) & 0xCCCCCCCCu), (int)(w0 & 0xCCCCCCCCu),
                     (int)((w1 << 2) & 0xCCCCCCCCu), (int)(w1 & 0xCCCCCCCCu), 0, 0, 0, 0};
    const i32x8 b = {(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
    // cbsz = 4: A is fp4 (E2M1); blgp = 0: B is fp8 (E4M3); both block scales 2^0
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 4, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
}

__device__ __forceinline__ void tile_steps(const u32x4& w, const unsigned char* xrow, f32x4& acc0, f32x4& acc1) {
    const u32x4* xb = reinterpret_cast<const u32x4*>(xrow);
    acc0 = mfma_step(w.x, w.y, xb[0], xb[1], acc0);      // columns   0..127 of the tile
    acc1 = mfma_step(w.z, w.w, xb[8], xb[9], acc1);      // columns 128..255
}

// fp8 (E4M3) codes of four integers 0..15 held one per byte.
__device__ __forceinline__ uint32_t fp8_of_nibbles(uint32_t v) {
    // 0..7 by table (0x00 0x38 0x40 0x44 | 0x48 0x4A 0x4C 0x4E), 8..15 are 0x48 + n
    const uint32_t small = __builtin_amdgcn_perm(0x4E4C4A48u, 0x44403800u, v & 0x07070707u);
    const uint32_t big = v + 0x48484848u;
    const uint32_t mask = ((v >> 3) & 0x01010101u) * 0xFFu;
    return (big & mask) | (small & ~mask);
}

// Digit planes of one activation: sign-magnitude fixed point, |v| < 2^ex -> magnitude <= 2^30.
// even: digits 0,2,4,6 (one per byte), odd: digits 1,3,5,7, as fp8 codes with the sign applied.
__device__ __forceinline__ uint32_t fixed_magnitude(float v, int ex) { return (uint32_t)rintf(ldexpf(fabsf(v), 30 - ex)); }
__device__ __forceinline__ void codes_of_fixed(uint32_t mag, bool negative, uint32_t& even, uint32_t& odd) {
    const uint32_t sign = negative ? 0x80808080u : 0u;
    even = fp8_of_nibbles(mag & 0x0F0F0F0Fu) | sign;
    odd = fp8_of_nibbles((mag >> 4) & 0x0F0F0F0Fu) | sign;
}
__device__ __forceinline__ void digit_codes(float v, int ex, uint32_t& even, uint32_t& odd) {
    codes_of_fixed(fixed_magnitude(v, ex), v < 0.f, even, odd);
}
// Four consecutive activations' codes (even[e], odd[e]) -> one 32-bit word per digit plane in LDS.
__device__ __forceinline__ void store_plane_words(unsigned char* planes, int pstride, int k, const uint32_t (&ev)[4], const uint32_t (&od)[4]) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t we = ((ev[0] >> (8 * d)) & 0xFFu) | (((ev[1] >> (8 * d)) & 0xFFu) << 8) |
                            (((ev[2] >> (8 * d)) & 0xFFu) << 16) | (((ev[3] >> (8 * d)) & 0xFFu) << 24);
        const uint32_t wo = ((od[0] >> (8 * d)) & 0xFFu) | (((od[1] >> (8 * d)) & 0xFFu) << 8) |
                            (((od[2] >> (8 * d)) & 0xFFu) << 16) | (((od[3] >> (8 * d)) & 0xFFu) << 24);
        *reinterpret_cast<uint32_t*>(planes + (size_t)(2 * d) * pstride + k) = we;
        *reinterpret_cast<uint32_t*>(planes + (size_t)(2 * d + 1) * pstride + k) = wo;
    }
}

// 4 x 4 byte transposition: out[d] byte e = in[e] byte d (eight byte permutes).
__device__ __forceinline__ void transpose_bytes(const uint32_t (&in)[4], uint32_t (&out)[4]) {
    const uint32_t t0 = __builtin_amdgcn_perm(in[1], in[0], 0x05010400u);    // in0.b0 in1.b0 in0.b1 in1.b1
    const uint32_t t1 = __builtin_amdgcn_perm(in[1], in[0], 0x07030602u);    // in0.b2 in1.b2 in0.b3 in1.b3
    const uint32_t t2 = __builtin_amdgcn_perm(in[3], in[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(in[3], in[2], 0x07030602u);
    out[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    out[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

// Digit planes of four consecutive activations given as sign-magnitude fixed point (bit 31 sign, magnitude
// <= 2^30): eight 32-bit words, one per plane, written at column k of the planes in LDS.  The digits are
// transposed first (nibbles of the four magnitudes -> one word of four digits per plane), so that the
// fp8 conversion and the sign run once per plane word.  Same codes as digit_codes element by element.
__device__ __forceinline__ void store_planes_of_fixed(unsigned char* planes, int pstride, int k, const uint32_t (&w)[4]) {
    uint32_t even[4], odd[4], te[4], to[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        even[e] = w[e] & 0x0F0F0F0Fu;              // digits 0, 2, 4, 6
        odd[e] = (w[e] >> 4) & 0x070F0F0Fu;        // digits 1, 3, 5, 7 (bit 31 is the sign; the top digit is below 8)
    }
    transpose_bytes(even, te);
    transpose_bytes(odd, to);
    // sign bytes: 0x80 in byte e for a negative element e
    const uint32_t sign = ((w[0] >> 24) & 0x80u) | ((w[1] >> 16) & 0x8000u) | ((w[2] >> 8) & 0x800000u) | (w[3] & 0x80000000u);
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        *reinterpret_cast<uint32_t*>(planes + (size_t)(2 * d) * pstride + k) = fp8_of_nibbles(te[d]) | sign;
        *reinterpret_cast<uint32_t*>(planes + (size_t)(2 * d + 1) * pstride + k) = fp8_of_nibbles(to[d]) | sign;
    }
}
__device__ __forceinline__ uint32_t fixed_word(float v, int ex) { return fixed_magnitude(v, ex) | (v < 0.f ? 0x80000000u : 0u); }

// exponent ex with m < 2^ex (m >= 0 finite); 0 for m == 0
__device__ __forceinline__ int bound_exponent(float m) {
    int ex = 0;
    if (m > 0.f && m < 3.0e38f) (void)frexpf(m, &ex);
    return ex;
}

__device__ __forceinline__ double pow2(int e) {      // 2^e for -1022 <= e <= 1023
    return __hiloint2double((1023 + e) << 20, 0);
}

// Maximum over the 64 lanes, returned in every lane (inputs >= 0).
__device__ __forceinline__ float wave_max(float v) {
    int x = __float_as_int(v);                                          // order-preserving for v >= 0
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, true));   // row_half_mirror
    x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, true));   // row_mirror
    const int r = max(max(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
                      max(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
    return __int_as_float(r);
}

// Horner recombination (base 16) of the eight digit-plane sums of one output row.
__device__ __forceinline__ double combine_planes(const float* sums) {
    const f32x4 lo = *reinterpret_cast<const f32x4*>(sums), hi = *reinterpret_cast<const f32x4*>(sums + 4);
    double acc = (double)hi.w;
    acc = acc * 16.0 + (double)hi.z;
    acc = acc * 16.0 + (double)hi.y;
    acc = acc * 16.0 + (double)hi.x;
    acc = acc * 16.0 + (double)lo.w;
    acc = acc * 16.0 + (double)lo.z;
    acc = acc * 16.0 + (double)lo.y;
    acc = acc * 16.0 + (double)lo.x;
    return acc;
}

}  // namespace

// Dynamic LDS: digit planes [8][kdim + 16] bytes, reduction tiles [16 wavefronts][16][16] fp32,
// plane sums [256 rows][8] fp32, 64 words of scratch.  blockDim.x = 1024; wavefront w works on strip w >> kw_log2 of the
// workgroup with contraction split w & (kw - 1).  ROUNDS = activation load rounds per thread
// (stage V: 4096 elements of x per round; stage U: 2048 columns of the planes per round).
// All loads are unconditional (out-of-range indices are clamped to valid memory and the values
// discarded): a load under a branch would make the compiler wait for every outstanding load.
template <bool STAGE_U, int ROUNDS>
__global__ void __launch_bounds__(1024)
tsvd_gemv_kernel(tsvd_gemv_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int kdim = STAGE_U ? p.Kp : p.Np;               // contraction length (padded)
    const int pstride = kdim + 16;
    unsigned char* planes = smem;
    float* red = reinterpret_cast<float*>(smem + (((size_t)8 * pstride + 255) & ~(size_t)255));
    float* sums = red + 16 * 256;
    float* scratch = sums + 256 * 8;
    const unsigned char* xlane = planes + (size_t)(i & 7) * pstride + 32 * g;   // MFMA columns 8..15 repeat 0..7
    const int kw = 1 << p.kw_log2;
    const int sidx = wave >> p.kw_log2, q = wave & (kw - 1);
    const int strip = blockIdx.x * p.sw + sidx;
    const bool active = sidx < p.sw && strip < p.strips;
    const u32x4* wp = reinterpret_cast<const u32x4*>(p.tiles) + ((size_t)(active ? strip : 0) * p.nkt) * 64 + lane;
    TICK(0);

    // ---- every load of this wavefront, in the order of need: activations first, then weights
    float xv[ROUNDS][4];
    u32x4 zv[ROUNDS];
    int ex_in = 0, ex_z = 0;
    // the scale (stage V) or bias (stage U) of the row this thread finishes, requested first: a load issued in the
    // epilogue would cost a full round trip to memory at the very end of the launch
    const int row_own = min((int)blockIdx.x * p.sw * 16 + (int)(threadIdx.x & 255), p.rows_out - 1);
    float tail_own = 0.f;
    if constexpr (STAGE_U) { if (p.bias) tail_own = p.bias[row_own]; }
    else tail_own = p.S[row_own];
    if constexpr (STAGE_U) {
        ex_in = p.meta[0];
        // plane c is copied by threads c * 128 .. c * 128 + 127, 16 bytes each per round
        const int c = threadIdx.x >> 7, t = threadIdx.x & 127;
        const u32x4* src = reinterpret_cast<const u32x4*>(p.planes_in + (size_t)c * p.Kp);
        const int last = p.Kp / 16 - 1;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) zv[r] = src[min(t + 128 * r, last)];
    } else {
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int k = 4 * (threadIdx.x + 1024 * r);
            if (p.x_vec) {                                     // contiguous, aligned, N % 4 == 0
                const int kc = min(k, p.N - 4);
                if (p.x_is_bf16) {
                    const u32x2 v = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(p.x) + kc);
                    xv[r][0] = __uint_as_float(v.x << 16); xv[r][1] = __uint_as_float(v.x & 0xFFFF0000u);
                    xv[r][2] = __uint_as_float(v.y << 16); xv[r][3] = __uint_as_float(v.y & 0xFFFF0000u);
                } else {
                    const f32x4 v = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p.x) + kc);
                    xv[r][0] = v.x; xv[r][1] = v.y; xv[r][2] = v.z; xv[r][3] = v.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const size_t off = (size_t)min(k + e, p.N - 1) * p.ldx;
                    xv[r][e] = p.x_is_bf16 ? __uint_as_float(((uint32_t) static_cast<const uint16_t*>(p.x)[off]) << 16)
                                           : static_cast<const float*>(p.x)[off];
                }
            }
        }
    }
    // The activations are a few KB that every workgroup needs before it can use a single tile.  Requesting all
    // NPRE tiles right behind them queued them behind 256 compute units' weight traffic (14.2 us per call on the
    // decode workload), waiting for them before any tile request 13.75 us; ONE tile request with them and the
    // others once they are in is another 0.25 us better (15.15 against 15.40 us on a slower box).
    u32x4 pre[NPRE];
    if (p.early_tiles) {
        pre[0] = __builtin_nontemporal_load(wp + (size_t)min(q, p.nkt - 1) * 64);
        asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
#pragma unroll
        for (int n = 1; n < NPRE; ++n) pre[n] = __builtin_nontemporal_load(wp + (size_t)min(q + n * kw, p.nkt - 1) * 64);
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int n = 0; n < NPRE; ++n) pre[n] = __builtin_nontemporal_load(wp + (size_t)min(q + n * kw, p.nkt - 1) * 64);
    }
    TICK(1);

    // ---- stage the digit planes in LDS
    if constexpr (STAGE_U) {
        const int c = threadIdx.x >> 7, t = threadIdx.x & 127;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int ch = t + 128 * r;
            if (ch * 16 < p.Kp) *reinterpret_cast<u32x4*>(planes + (size_t)c * pstride + ch * 16) = zv[r];
        }
    } else {
        float m = 0.f;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int k = 4 * (threadIdx.x + 1024 * r);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                xv[r][e] = k + e < p.N ? xv[r][e] : 0.f;          // clamped loads beyond N
                m = fmaxf(m, fabsf(xv[r][e]));
            }
        }
        m = wave_max(m);
        if (lane == 0) scratch[wave] = m;
        __syncthreads();
        m = scratch[lane & 15];
        m = wave_max(m);
        ex_in = bound_exponent(m);
        ex_z = bound_exponent(p.bound_V * m) + 1;   // one more bit for the rounding of the bound itself
        if (blockIdx.x == 0 && threadIdx.x == 0) p.meta[0] = ex_z;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int k = 4 * (threadIdx.x + 1024 * r);
            if (k < p.Np) {
                // four consecutive activations -> one 32-bit word per plane
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = fixed_word(xv[r][e], ex_in);
                store_planes_of_fixed(planes, pstride, k, w);
            }
        }
    }
    __syncthreads();
    TICK(2);

    // ---- stream this wavefront's tiles T = q, q + kw, ...
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    if (active) {
        // NPRE tiles stay in flight: each one is replaced by the tile NPRE places further on as soon
        // as it has been copied out of its registers (unconditional, clamped loads; results return
        // in issue order, so the wait before tile n is for all but the NPRE - 1 younger loads).
        for (int T0 = q; T0 < p.nkt; T0 += NPRE * kw) {
#pragma unroll
            for (int n = 0; n < NPRE; ++n) {
                const int T = T0 + n * kw;
                const u32x4 w0 = pre[n];
                pre[n] = __builtin_nontemporal_load(wp + (size_t)min(T + NPRE * kw, p.nkt - 1) * 64);
                if (T < p.nkt) tile_steps(w0, xlane + T * 256, acc0, acc1);
            }
        }
    }
    // D layout of the 16x16 MFMA: lane holds column i, rows 4 g + v.  Only columns 0..7 matter.
    if (i < 8) {
        float* mine = red + (size_t)wave * 256;
#pragma unroll
        for (int v = 0; v < 4; ++v) mine[(4 * g + v) * 16 + i] = acc0[v] + acc1[v];
    }
    __syncthreads();
    TICK(3);

    // ---- add the kw partial tiles (all threads), then recombine the planes, scale, store
    for (int idx = threadIdx.x; idx < p.sw * 128; idx += blockDim.x) {
        const int rl = idx >> 3, pc = idx & 7;                      // row within the workgroup, plane
        const float* src = red + (size_t)((rl >> 4) * kw) * 256 + (rl & 15) * 16 + pc;
        float part = 0.f;
        for (int qq = 0; qq < kw; ++qq) part += src[qq * 256];      // integers < 2^24: exact
        sums[idx] = part;
    }
    __syncthreads();
    for (int rl = threadIdx.x; rl < p.sw * 16; rl += blockDim.x) {
        const int row = blockIdx.x * p.sw * 16 + rl;
        if (row >= p.rows_out) continue;
        // acc = 2 * sum_k A[row][k] * fixed(in[k]): undo the factor 2 and the fixed-point scale
        const double val = combine_planes(sums + rl * 8) * pow2(ex_in - 31);
        if constexpr (STAGE_U) {
            tsvd_store_y(p.y, (size_t)row * p.ldy, (float)(p.bias ? val + (double)tail_own : val), p.out_bf16);
        } else {
            const float z = (float)((double)tail_own * val);
            uint32_t ev, od;
            digit_codes(z, ex_z, ev, od);
            unsigned char* dst = p.planes_out + row;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                dst[(size_t)(2 * d) * p.Kp] = (unsigned char)(ev >> (8 * d));
                dst[(size_t)(2 * d + 1) * p.Kp] = (unsigned char)(od >> (8 * d));
            }
        }
    }
    TICK(4);
}

// ---- both stages in one launch of one workgroup (small matrices) ---------------------------------
// For a matrix of a few dozen tiles a call is nothing but latency: two launches, each with its own
// round trips for x / z and the weights.  Here one workgroup issues ALL its loads at entry (x, then
// the tiles of V and of U: at most four per wavefront and stage, held in registers), runs stage V
// with wavefront w on strips w, w + 16, ..., digitises z straight into LDS, and runs stage U
// from there: one launch, z never leaves the compute unit, and the U tiles arrive while stage V
// computes.  Same arithmetic as tsvd_gemv_kernel (exact integer sums, fp64 recombination).
#define FUSED_MAX_ITEMS 4      // tiles per wavefront and stage
__global__ void __launch_bounds__(1024)
tsvd_gemv_fused_kernel(tsvd_gemv_fused_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int xstride = p.Np + 16, zstride = p.Kp + 16;
    unsigned char* xplanes = smem;                                              // [8][Np + 16]
    unsigned char* zplanes = smem + (((size_t)8 * xstride + 255) & ~(size_t)255);   // [8][Kp + 16]
    float* wred = reinterpret_cast<float*>(zplanes + (((size_t)8 * zstride + 255) & ~(size_t)255));   // [16][16][8]
    float* scratch = wred + 16 * 128;

    // ---- every load, in the order of need
    float xv[4];
    {
        const int k = 4 * threadIdx.x;
        if (p.x_vec) {
            const int kc = min(k, p.N - 4);
            if (p.x_is_bf16) {
                const u32x2 v = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(p.x) + kc);
                xv[0] = __uint_as_float(v.x << 16); xv[1] = __uint_as_float(v.x & 0xFFFF0000u);
                xv[2] = __uint_as_float(v.y << 16); xv[3] = __uint_as_float(v.y & 0xFFFF0000u);
            } else {
                const f32x4 v = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p.x) + kc);
                xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const size_t off = (size_t)min(k + e, p.N - 1) * p.ldx;
                xv[e] = p.x_is_bf16 ? __uint_as_float(((uint32_t) static_cast<const uint16_t*>(p.x)[off]) << 16)
                                    : static_cast<const float*>(p.x)[off];
            }
        }
    }
    // item j of a stage: strip wave + 16 (j / nkt), tile j % nkt (clamped loads; unused items are never consumed)
    const int rounds_v = (p.strips_v + 15) / 16, rounds_u = (p.strips_u + 15) / 16;
    u32x4 pv[FUSED_MAX_ITEMS], pu[FUSED_MAX_ITEMS];
#pragma unroll
    for (int j = 0; j < FUSED_MAX_ITEMS; ++j) {
        const int strip = min(wave + 16 * (j / p.nkt_v), p.strips_v - 1), T = j % p.nkt_v;
        pv[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.tiles_v) + ((size_t)strip * p.nkt_v + T) * 64 + lane);
    }
#pragma unroll
    for (int j = 0; j < FUSED_MAX_ITEMS; ++j) {
        const int strip = min(wave + 16 * (j / p.nkt_u), p.strips_u - 1), T = j % p.nkt_u;
        pu[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.tiles_u) + ((size_t)strip * p.nkt_u + T) * 64 + lane);
    }

    // ---- x -> digit planes in LDS
    float m = 0.f;
    {
        const int k = 4 * threadIdx.x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xv[e] = k + e < p.N ? xv[e] : 0.f;
            m = fmaxf(m, fabsf(xv[e]));
        }
    }
    m = wave_max(m);
    if (lane == 0) scratch[wave] = m;
    __syncthreads();
    m = wave_max(scratch[lane & 15]);
    const int ex_x = bound_exponent(m);
    const int ex_z = bound_exponent(p.bound_V * m) + 1;
    {
        const int k = 4 * threadIdx.x;
        if (k < p.Np) {
            uint32_t ev[4], od[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) digit_codes(xv[e], ex_x, ev[e], od[e]);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t we = ((ev[0] >> (8 * d)) & 0xFFu) | (((ev[1] >> (8 * d)) & 0xFFu) << 8) |
                                    (((ev[2] >> (8 * d)) & 0xFFu) << 16) | (((ev[3] >> (8 * d)) & 0xFFu) << 24);
                const uint32_t wo = ((od[0] >> (8 * d)) & 0xFFu) | (((od[1] >> (8 * d)) & 0xFFu) << 8) |
                                    (((od[2] >> (8 * d)) & 0xFFu) << 16) | (((od[3] >> (8 * d)) & 0xFFu) << 24);
                *reinterpret_cast<uint32_t*>(xplanes + (size_t)(2 * d) * xstride + k) = we;
                *reinterpret_cast<uint32_t*>(xplanes + (size_t)(2 * d + 1) * xstride + k) = wo;
            }
        }
    }
    __syncthreads();

    // One round of a stage: wavefront w multiplies strip w + 16 r with the planes, the 256 rows of
    // the round are finished by threads 0..255 (row t of the round) from the plane sums in LDS.
    auto round_sums = [&](const u32x4 (&tiles)[FUSED_MAX_ITEMS], int r, int nkt, const unsigned char* planes, int pstride) {
        const unsigned char* xlane = planes + (size_t)(i & 7) * pstride + 32 * g;
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < FUSED_MAX_ITEMS; ++j)
            if (j / nkt == r) tile_steps(tiles[j], xlane + (j % nkt) * 256, acc0, acc1);
        if (i < 8) {
#pragma unroll
            for (int v = 0; v < 4; ++v) wred[wave * 128 + (4 * g + v) * 8 + i] = acc0[v] + acc1[v];
        }
    };
    // ---- stage V: z = S * (V x), digitised into LDS
    for (int r = 0; r < rounds_v; ++r) {
        round_sums(pv, r, p.nkt_v, xplanes, xstride);
        __syncthreads();
        if (threadIdx.x < 256) {
            const int row = 256 * r + threadIdx.x;
            if (row < p.Kp) {
                const double val = combine_planes(wred + threadIdx.x * 8) * pow2(ex_x - 31);
                const float z = (float)((double)p.S[row] * val);
                uint32_t ev, od;
                digit_codes(z, ex_z, ev, od);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    zplanes[(size_t)(2 * d) * zstride + row] = (unsigned char)(ev >> (8 * d));
                    zplanes[(size_t)(2 * d + 1) * zstride + row] = (unsigned char)(od >> (8 * d));
                }
            }
        }
        __syncthreads();
    }
    // ---- stage U: y = U z
    for (int r = 0; r < rounds_u; ++r) {
        round_sums(pu, r, p.nkt_u, zplanes, zstride);
        __syncthreads();
        if (threadIdx.x < 256) {
            const int row = 256 * r + threadIdx.x;
            if (row < p.M) {
                const double val = combine_planes(wred + threadIdx.x * 8) * pow2(ex_z - 31);
                tsvd_store_y(p.y, (size_t)row * p.ldy, (float)(p.bias ? val + (double)p.bias[row] : val), p.out_bf16);
            }
        }
        __syncthreads();
    }
}


// ---- both stages of a single token in ONE launch of about one workgroup per compute unit -----------
// Two launches cost two launch boundaries and two serial prologues (activations in, planes staged)
// in a call that streams its weights in a few microseconds.  Here every workgroup
//   1. requests x, then the tiles of its own slice of V AND all tiles of its rows of U (they stay in
//      registers: at most ONEPASS_NU per wavefront), so the U stream is in flight from the start;
//   2. digitises x, multiplies its slice of V, scales by S and publishes its rows of z;
//   3. collects the whole z from the other workgroups, digitises it into LDS;
//   4. multiplies its rows of U (tiles already there) and stores y.
// Hand-over of z between workgroups (they run on different XCDs, each with its own L2): element k
// of z travels as ONE 64-bit word {tag : 32 | sign-magnitude fixed point : 32} written and read with
// device-scope atomic stores / loads (they bypass the non-coherent caches), so a reader that sees the
// call's tag has the value, with no fence and no separate flag.  The tag is the value of a counter in
// device memory that every workgroup reads at entry and increments when it is done: a call never sees
// a tag left by an earlier one (the words of a call carry tags from [c, c + grid), the next call's
// start at c + grid), and a captured launch replays correctly because the host passes no per-call state.
// The buffer and the counter belong to the handle (zeroed at tsvd_pack); calls of one handle must
// not overlap on the device (the dispatcher keeps them on one stream).
// No workgroup ever depends on another one for progress: a reader polls at most spin_limit times for
// a slice and then computes that slice itself from V and x (same arithmetic, so same bits), straight
// into its LDS planes.  Workgroups that are not resident yet (a busy GPU) therefore cost time, never
// a hang, and a launch of any size drains.
#define ONEPASS_XR 2      // x: rounds of 4096 elements        (Np <= 8192)
#define ONEPASS_ZR 2      // z: rounds of 4096 elements        (Kp <= 8192)
template <int NV, int NU>
__global__ void __launch_bounds__(1024)
tsvd_gemv_onepass_kernel(tsvd_gemv_onepass_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int xstride = p.Np + 16, zstride = p.Kp + 16;
    unsigned char* xplanes = smem;                                                       // [8][Np + 16]
    unsigned char* zplanes = smem + (((size_t)8 * xstride + 255) & ~(size_t)255);        // [8][Kp + 16]
    float* red = reinterpret_cast<float*>(zplanes + (((size_t)8 * zstride + 255) & ~(size_t)255));   // [16][256]
    float* sums = red + 16 * 256;                                                        // [256][8]
    float* scratch = sums + 256 * 8;                                                     // [16]
    unsigned* missing = reinterpret_cast<unsigned*>(scratch + 16);                       // [8]: bit per slice
    const int kw_v = 1 << p.kwl_v, kw_u = 1 << p.kwl_u;
    const int sidx_v = wave >> p.kwl_v, q_v = wave & (kw_v - 1);
    const int sidx_u = wave >> p.kwl_u, q_u = wave & (kw_u - 1);
    const int strip_u = blockIdx.x * p.sw_u + sidx_u;
    const bool active_u = sidx_u < p.sw_u && strip_u < p.strips_u;
    const u32x4* tv = reinterpret_cast<const u32x4*>(p.tiles_v) + lane;
    const u32x4* tu = reinterpret_cast<const u32x4*>(p.tiles_u) + ((size_t)(active_u ? strip_u : 0) * p.nkt_u) * 64 + lane;
    TICK(0);
    const long long wave_t0 = p.clocks ? wall_clock64() : 0;

    // ---- loads, in the order of need: the call's tag and x, then (once x is here) the weight tiles
    const unsigned tag = __hip_atomic_load(p.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float xv[ONEPASS_XR][4];
#pragma unroll
    for (int r = 0; r < ONEPASS_XR; ++r) {
        const int k = 4 * (threadIdx.x + 1024 * r);
        if (p.x_vec) {
            const int kc = min(k, p.N - 4);
            if (p.x_is_bf16) {
                const u32x2 v = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(p.x) + kc);
                xv[r][0] = __uint_as_float(v.x << 16); xv[r][1] = __uint_as_float(v.x & 0xFFFF0000u);
                xv[r][2] = __uint_as_float(v.y << 16); xv[r][3] = __uint_as_float(v.y & 0xFFFF0000u);
            } else {
                const f32x4 v = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p.x) + kc);
                xv[r][0] = v.x; xv[r][1] = v.y; xv[r][2] = v.z; xv[r][3] = v.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const size_t off = (size_t)min(k + e, p.N - 1) * p.ldx;
                xv[r][e] = p.x_is_bf16 ? __uint_as_float(((uint32_t) static_cast<const uint16_t*>(p.x)[off]) << 16)
                                       : static_cast<const float*>(p.x)[off];
            }
        }
    }
    // scale of the row of z and bias of the row of y that this thread finishes (vector-memory results return in
    // issue order: a load issued after the weight tiles would hold its consumer back until all of them are in)
    const float s_own = p.S[min((int)blockIdx.x * p.sw_v * 16 + (int)(threadIdx.x & 255), p.Kp - 1)];
    const float bias_own = p.bias ? p.bias[min((int)blockIdx.x * p.sw_u * 16 + (int)(threadIdx.x & 255), p.M - 1)] : 0.f;
    // tiles of slice j of V for this wavefront (clamped, unconditional loads)
    u32x4 pv[NV];
    auto load_v = [&](int j) {
        const int strip = min(j * p.sw_v + sidx_v, p.strips_v - 1);
#pragma unroll
        for (int n = 0; n < NV; ++n)
            pv[n] = __builtin_nontemporal_load(tv + ((size_t)strip * p.nkt_v + min(q_v + n * kw_v, p.nkt_v - 1)) * 64);
    };
    // The tiles of U are requested in batches, so that the memory system always has work but the latency-critical
    // answers (the tiles of V, the polls for z) never queue behind all of U: a quarter with the tiles of V, a
    // quarter once x is digitised, a quarter once z is published, the rest around the polls.
    constexpr int NU1 = (NU + 3) / 4, NU2 = NU / 2, NU3 = NU2 + NU / 4;
    u32x4 pu[NU];
    auto load_u = [&](int from, int to) {
#pragma unroll
        for (int n = 0; n < NU; ++n)
            if (n >= from && n < to) pu[n] = __builtin_nontemporal_load(tu + (size_t)min(q_u + n * kw_u, p.nkt_u - 1) * 64);
    };
    load_v(blockIdx.x);
    load_u(0, NU1);
    TICK(1);

    // ---- x -> digit planes in LDS
    float m = 0.f;
#pragma unroll
    for (int r = 0; r < ONEPASS_XR; ++r) {
        const int k = 4 * (threadIdx.x + 1024 * r);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xv[r][e] = k + e < p.N ? xv[r][e] : 0.f;
            m = fmaxf(m, fabsf(xv[r][e]));
        }
    }
    m = wave_max(m);
    if (lane == 0) scratch[wave] = m;
    if (threadIdx.x < 8) missing[threadIdx.x] = 0u;
    if (p.clocks && lane == 0) reinterpret_cast<long long*>(sums)[wave] = wave_t0;
    __syncthreads();
    TICK(9);
    if (p.clocks && threadIdx.x == 0) {
        long long mx = 0;
        for (int w2 = 0; w2 < 16; ++w2) mx = max(mx, reinterpret_cast<long long*>(sums)[w2]);
        p.clocks[blockIdx.x * 16 + 8] = mx;
    }
    m = wave_max(scratch[lane & 15]);
    const int ex_x = bound_exponent(m);
    const int ex_z = bound_exponent(p.bound_V * m) + 1;   // one more bit for the rounding of the bound itself
#pragma unroll
    for (int r = 0; r < ONEPASS_XR; ++r) {
        const int k = 4 * (threadIdx.x + 1024 * r);
        if (k < p.Np) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = fixed_word(xv[r][e], ex_x);
            store_planes_of_fixed(xplanes, xstride, k, w);
        }
    }
    TICK(10);
    __syncthreads();
    load_u(NU1, NU2);
    TICK(2);

    // ---- slice j of z = S * (V x) from the tiles in pv: published (own slice) or written into zplanes (help)
    const unsigned char* xlane = xplanes + (size_t)(i & 7) * xstride + 32 * g;
    auto v_slice = [&](int j, bool publish) {
        float s_row = s_own;
        if (!publish) s_row = p.S[min(j * p.sw_v * 16 + (int)(threadIdx.x & 255), p.Kp - 1)];
        const bool active = sidx_v < p.sw_v && j * p.sw_v + sidx_v < p.strips_v;
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const int T = q_v + n * kw_v;
            if (active && T < p.nkt_v) tile_steps(pv[n], xlane + T * 256, acc0, acc1);
        }
        if (i < 8) {
            float* mine = red + (size_t)wave * 256;
#pragma unroll
            for (int v = 0; v < 4; ++v) mine[(4 * g + v) * 16 + i] = acc0[v] + acc1[v];
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < p.sw_v * 128; idx += 1024) {
            const int rl = idx >> 3, pc = idx & 7;
            const float* src = red + (size_t)((rl >> 4) * kw_v) * 256 + (rl & 15) * 16 + pc;
            float part = 0.f;
            for (int qq = 0; qq < kw_v; ++qq) part += src[qq * 256];      // integers < 2^24: exact
            sums[idx] = part;
        }
        __syncthreads();
        for (int rl = threadIdx.x; rl < p.sw_v * 16; rl += 1024) {
            const int row = j * p.sw_v * 16 + rl;
            if (row >= p.Kp) continue;
            const double val = combine_planes(sums + rl * 8) * pow2(ex_x - 31);
            const float z = (float)((double)s_row * val);
            const uint32_t mag = fixed_magnitude(z, ex_z);
            if (publish) {
                const unsigned long long word = ((unsigned long long)tag << 32) | mag | (z < 0.f ? 0x80000000u : 0u);
                __hip_atomic_store(p.zbuf + row, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                uint32_t ev, od;
                codes_of_fixed(mag, z < 0.f, ev, od);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    zplanes[(size_t)(2 * d) * zstride + row] = (unsigned char)(ev >> (8 * d));
                    zplanes[(size_t)(2 * d + 1) * zstride + row] = (unsigned char)(od >> (8 * d));
                }
            }
        }
        __syncthreads();
    };
    v_slice(blockIdx.x, true);
    TICK(3);

    // ---- collect z: thread t owns elements 4 (t + 1024 r) .. + 3
    unsigned long long zw[ONEPASS_ZR][4] = {};
    bool have = p.spin_limit >= 0;
    auto poll = [&]() {
#pragma unroll
        for (int r = 0; r < ONEPASS_ZR; ++r) {
            const int k = min(4 * (threadIdx.x + 1024 * r), p.Kp - 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) zw[r][e] = __hip_atomic_load(p.zbuf + k + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    // One more batch of U, then the first poll.  While a poll fails (a slice of another workgroup is not there yet),
    // every retry is preceded by ONE more tile request per wavefront: the memory system stays busy, and the retry
    // queues behind 4 MB instead of behind the rest of U.  The loop is uniform over the wavefront.
    load_u(NU2, NU3);
    int issued = NU3;
    if (p.spin_limit >= 0) {
        for (int spin = 0;; ++spin) {
            poll();
            have = true;
#pragma unroll
            for (int r = 0; r < ONEPASS_ZR; ++r)
#pragma unroll
                for (int e = 0; e < 4; ++e) have = have && (unsigned)(zw[r][e] >> 32) == tag;
            if (__builtin_amdgcn_ballot_w64(!have) == 0ull || spin >= p.spin_limit) break;
#pragma unroll
            for (int n = 0; n < NU; ++n)
                if (n >= NU3 && n == issued) pu[n] = __builtin_nontemporal_load(tu + (size_t)min(q_u + n * kw_u, p.nkt_u - 1) * 64);
            ++issued;
            __builtin_amdgcn_s_sleep(1);
        }
    }
#pragma unroll
    for (int n = 0; n < NU; ++n)
        if (n >= NU3 && n >= issued) pu[n] = __builtin_nontemporal_load(tu + (size_t)min(q_u + n * kw_u, p.nkt_u - 1) * 64);
    const int slice_rows = p.sw_v * 16;
#pragma unroll
    for (int r = 0; r < ONEPASS_ZR; ++r) {
        const int k = 4 * (threadIdx.x + 1024 * r);
        if (k < p.Kp) {
            uint32_t w[4];
            bool all = p.spin_limit >= 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                w[e] = (uint32_t)zw[r][e];
                all = all && (unsigned)(zw[r][e] >> 32) == tag;
            }
            if (all) {
                store_planes_of_fixed(zplanes, zstride, k, w);
            } else {
                // (a slice holds a multiple of 16 rows, so the four elements lie in one slice)
                const int j = k / slice_rows;
                atomicOr(&missing[j >> 5], 1u << (j & 31));
            }
        }
    }
    __syncthreads();
    TICK(4);
    // ---- slices that did not arrive in time: compute them here (uniform over the workgroup)
    for (int wd = 0; wd < 8; ++wd) {
        unsigned bits = missing[wd];
        while (bits) {
            const int j = 32 * wd + __builtin_ctz(bits);
            bits &= bits - 1;
            load_v(j);
            v_slice(j, false);
        }
    }
    TICK(5);

    // ---- y = U z for this workgroup's rows, tiles from registers
    const unsigned char* zlane = zplanes + (size_t)(i & 7) * zstride + 32 * g;
    {
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int n = 0; n < NU; ++n) {
            const int T = q_u + n * kw_u;
            if (active_u && T < p.nkt_u) tile_steps(pu[n], zlane + T * 256, acc0, acc1);
        }
        if (i < 8) {
            float* mine = red + (size_t)wave * 256;
#pragma unroll
            for (int v = 0; v < 4; ++v) mine[(4 * g + v) * 16 + i] = acc0[v] + acc1[v];
        }
    }
    __syncthreads();
    TICK(6);
    for (int idx = threadIdx.x; idx < p.sw_u * 128; idx += 1024) {
        const int rl = idx >> 3, pc = idx & 7;
        const float* src = red + (size_t)((rl >> 4) * kw_u) * 256 + (rl & 15) * 16 + pc;
        float part = 0.f;
        for (int qq = 0; qq < kw_u; ++qq) part += src[qq * 256];
        sums[idx] = part;
    }
    __syncthreads();
    for (int rl = threadIdx.x; rl < p.sw_u * 16; rl += 1024) {
        const int row = blockIdx.x * p.sw_u * 16 + rl;
        if (row >= p.M) continue;
        const double val = combine_planes(sums + rl * 8) * pow2(ex_z - 31);
        tsvd_store_y(p.y, (size_t)row * p.ldy, (float)(p.bias ? val + (double)bias_own : val), p.out_bf16);
    }
    // this workgroup is done with the call's tag (no result wanted: fire and forget)
    if (threadIdx.x == 0) (void)__hip_atomic_fetch_add(p.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    TICK(7);
}

namespace {
size_t onepass_lds_bytes(long long Np, long long Kp) {
    return ((8 * (size_t)(Np + 16) + 255) & ~(size_t)255) + ((8 * (size_t)(Kp + 16) + 255) & ~(size_t)255) +
           (16 * 256 + 256 * 8 + 16 + 8) * sizeof(float);
}
// tiles per wavefront of a stage for a workgroup shape
int onepass_tiles(int nkt, int kwl) { return (nkt + (1 << kwl) - 1) >> kwl; }
}  // namespace

// Shape of the one-launch call: grid, strips per workgroup and contraction splits of both stages.
// Returns false when the problem does not fit (tiles per wavefront beyond the register budget, LDS).
bool tsvd_gemv_onepass_shape(long long M, long long Mp, long long Kp, long long Np, int cus, tsvd_gemv_onepass_args* a) {
    (void)Mp;
    if (Np > 4096 * ONEPASS_XR || Kp > 4096 * ONEPASS_ZR || onepass_lds_bytes(Np, Kp) > TSVD_SKINNY_MAX_LDS) return false;
    const int strips_v = (int)(Kp / 16), strips_u = (int)((M + 15) / 16);
    const int nkt_v = (int)(Np / 256), nkt_u = (int)(Kp / 256);
    const int G = std::min(std::min(cus, 256), std::max(strips_v, strips_u));
    const int sw_v = (strips_v + G - 1) / G, sw_u = (strips_u + G - 1) / G;
    if (sw_v > 16 || sw_u > 16) return false;
    auto splits = [](int sw, int nkt) {
        int kl = 0;
        while ((sw << (kl + 1)) <= 16 && (2 << kl) <= nkt) ++kl;
        return kl;
    };
    const int kwl_v = splits(sw_v, nkt_v), kwl_u = splits(sw_u, nkt_u);
    const int nv = onepass_tiles(nkt_v, kwl_v), nu = onepass_tiles(nkt_u, kwl_u);
    if (nv > 4 || nu > 16 || (nv > 2 && nu > 8)) return false;       // register budget of 1024-thread workgroups
    if (a) {
        a->strips_v = strips_v; a->nkt_v = nkt_v; a->sw_v = sw_v; a->kwl_v = kwl_v;
        a->strips_u = strips_u; a->nkt_u = nkt_u; a->sw_u = sw_u; a->kwl_u = kwl_u;
        a->grid = G;
    }
    return true;
}

hipError_t tsvd_launch_gemv_onepass(const tsvd_gemv_onepass_args& a, hipStream_t stream) {
    if (a.grid < 1 || a.grid > 256 || a.sw_v < 1 || a.sw_u < 1 || (a.sw_v << a.kwl_v) > 16 || (a.sw_u << a.kwl_u) > 16 ||
        a.grid * a.sw_v < a.strips_v || a.grid * a.sw_u < a.strips_u || a.Np > 4096 * ONEPASS_XR || a.Kp > 4096 * ONEPASS_ZR ||
        a.Np != a.nkt_v * 256 || a.Kp != a.nkt_u * 256 || a.Kp != a.strips_v * 16 || !a.zbuf || !a.counter)
        return hipErrorInvalidValue;
    const int nv = onepass_tiles(a.nkt_v, a.kwl_v), nu = onepass_tiles(a.nkt_u, a.kwl_u);
    if (nv > 4 || nu > 16 || (nv > 2 && nu > 8)) return hipErrorInvalidValue;
    const size_t lds = onepass_lds_bytes(a.Np, a.Kp);
    const dim3 grid(a.grid), block(1024);
#define ONEPASS_LAUNCH(NV_, NU_) hipLaunchKernelGGL((tsvd_gemv_onepass_kernel<NV_, NU_>), grid, block, lds, stream, a)
    if (nv <= 2) {
        if (nu <= 4) ONEPASS_LAUNCH(2, 4);
        else if (nu <= 8) ONEPASS_LAUNCH(2, 8);
        else ONEPASS_LAUNCH(2, 16);
    } else {
        if (nu <= 4) ONEPASS_LAUNCH(4, 4);
        else if (nu <= 8) ONEPASS_LAUNCH(4, 8);
        else return hipErrorInvalidValue;
    }
#undef ONEPASS_LAUNCH
    return hipGetLastError();
}

size_t gemv_fused_lds_bytes(long long Np, long long Kp) {
    return ((8 * (size_t)(Np + 16) + 255) & ~(size_t)255) + ((8 * (size_t)(Kp + 16) + 255) & ~(size_t)255) + (16 * 128 + 64) * sizeof(float);
}

namespace {
template <bool STAGE_U, int ROUNDS>
hipError_t init_one() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemv_kernel<STAGE_U, ROUNDS>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, TSVD_SKINNY_MAX_LDS);
}
size_t gemv_lds_bytes(long long kdim) {
    return ((8 * (size_t)(kdim + 16) + 255) & ~(size_t)255) + (16 * 256 + 256 * 8 + 64) * sizeof(float);
}
}  // namespace

bool tsvd_gemv_fused_fits(long long Mp, long long Kp, long long Np) {
    // at most FUSED_MAX_ITEMS tiles per wavefront and stage; x in one load round
    const long long rounds_v = (Kp / 16 + 15) / 16, rounds_u = (Mp / 16 + 15) / 16;
    return Np <= 4096 && rounds_v * (Np / 256) <= FUSED_MAX_ITEMS && rounds_u * (Kp / 256) <= FUSED_MAX_ITEMS &&
           gemv_fused_lds_bytes(Np, Kp) <= TSVD_SKINNY_MAX_LDS;
}

hipError_t tsvd_launch_gemv_fused(const tsvd_gemv_fused_args& a, hipStream_t stream) {
    if (a.strips_v < 1 || a.strips_u < 1 || a.nkt_v < 1 || a.nkt_u < 1 || a.Np > 4096 ||
        ((a.strips_v + 15) / 16) * a.nkt_v > FUSED_MAX_ITEMS || ((a.strips_u + 15) / 16) * a.nkt_u > FUSED_MAX_ITEMS)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(tsvd_gemv_fused_kernel, dim3(1), dim3(1024), gemv_fused_lds_bytes(a.Np, a.Kp), stream, a);
    return hipGetLastError();
}

hipError_t tsvd_gemv_init() {
    hipError_t e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemv_fused_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_SKINNY_MAX_LDS)) != hipSuccess) return e;
#define ONEPASS_ATTR(NV_, NU_) \
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemv_onepass_kernel<NV_, NU_>), \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, TSVD_SKINNY_MAX_LDS)) != hipSuccess) return e;
    ONEPASS_ATTR(2, 4) ONEPASS_ATTR(2, 8) ONEPASS_ATTR(2, 16) ONEPASS_ATTR(4, 4) ONEPASS_ATTR(4, 8)
#undef ONEPASS_ATTR
    if ((e = init_one<false, 1>()) != hipSuccess) return e;
    if ((e = init_one<false, 2>()) != hipSuccess) return e;
    if ((e = init_one<false, 4>()) != hipSuccess) return e;
    if ((e = init_one<true, 1>()) != hipSuccess) return e;
    if ((e = init_one<true, 2>()) != hipSuccess) return e;
    if ((e = init_one<true, 4>()) != hipSuccess) return e;
    return init_one<true, 8>();
}

// Limits of the one-batch loads and of LDS.
bool tsvd_gemv_fits(long long Np, long long Kp) {
    return Np <= 4096LL * XR_MAX && Kp <= 2048LL * ZR_MAX && gemv_lds_bytes(Np > Kp ? Np : Kp) <= TSVD_SKINNY_MAX_LDS;
}

hipError_t tsvd_launch_gemv(const tsvd_gemv_args& a, bool stage_u, hipStream_t stream) {
    if (!tsvd_gemv_fits(a.Np, a.Kp) || a.sw < 1 || a.kw_log2 < 0 || (a.sw << a.kw_log2) > 16 || a.strips < 1)
        return hipErrorInvalidValue;
    const dim3 grid((a.strips + a.sw - 1) / a.sw), block(1024);
    if (stage_u) {
        const size_t lds = gemv_lds_bytes(a.Kp);
        if (a.Kp <= 2048) hipLaunchKernelGGL((tsvd_gemv_kernel<true, 1>), grid, block, lds, stream, a);
        else if (a.Kp <= 4096) hipLaunchKernelGGL((tsvd_gemv_kernel<true, 2>), grid, block, lds, stream, a);
        else if (a.Kp <= 8192) hipLaunchKernelGGL((tsvd_gemv_kernel<true, 4>), grid, block, lds, stream, a);
        else hipLaunchKernelGGL((tsvd_gemv_kernel<true, 8>), grid, block, lds, stream, a);
    } else {
        const size_t lds = gemv_lds_bytes(a.Np);
        if (a.Np <= 4096) hipLaunchKernelGGL((tsvd_gemv_kernel<false, 1>), grid, block, lds, stream, a);
        else if (a.Np <= 8192) hipLaunchKernelGGL((tsvd_gemv_kernel<false, 2>), grid, block, lds, stream, a);
        else hipLaunchKernelGGL((tsvd_gemv_kernel<false, 4>), grid, block, lds, stream, a);
    }
    return hipGetLastError();
}
