// Few-token path (2 <= B <= 16, bf16 activations): the two stages of Y = U (diag(S) (V X))
// (paper, section "Truncated SVD in Network Compression"; supplement Table S1: V(.) and U(.) are
// additions only, diag(S)(.) is K multiplications per token), one launch each.
//
// With a handful of tokens a call is bound, as for B = 1, by streaming the packed weights once
// from HBM, but all tokens fit the 16 columns of one MFMA block.  So the data movement is that of
// the single-token kernels (16 wavefronts per workgroup, about one workgroup per compute unit,
// every wavefront streaming the 1-KiB tiles of its own 16-row strip with two tiles in flight,
// contraction split over wavefronts and reduced through LDS) and the arithmetic is that of the
// batched kernels: codes expanded in registers to the 16-bit floats 0 / +2 / -2 (a shift and a
// mask per pair), bf16 MFMA for stage V, fp16 MFMA for stage U on z rounded to fp16 after a
// per-token power-of-two scaling (11 significant bits), fp32 accumulation.
//
// Activations [k][16 tokens] (32 bytes per row) pass through LDS in slabs of 2048 contraction
// indices, double-buffered: slab s + 1 is fetched into registers while slab s is consumed, one
// barrier per slab.  Inside a slab the rows are stored stage by stage in the order
// of the code words (64 rows per word, see tsvd_layout.h) and read in MFMA operand order with
// ds_read_b64_tr_b16.  Stage V finds the per-token maxima of |x| (for the scaling) from the
// slabs as they pass through its registers, so there is no separate reduction launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "tsvd_epilogue.h"
#include "tsvd_kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define MID_DEC(w, j) ((((uint32_t)(w)) << (14 - 2 * (j))) & 0xC000C000u)
#define MID_SLAB_TILES 8                                  // 256-wide tiles per slab
#define MID_STAGE_BYTES 2048                              // 64 rows x 16 tokens x 2 bytes
#define MID_SLAB_BYTES (MID_SLAB_TILES * 4 * MID_STAGE_BYTES)   // 64 KiB
#define MID_LDS_BYTES (2 * MID_SLAB_BYTES + 256 + 16384 + 512)   // slabs, token factors, maxima scratch
#ifndef MID_LOOKAHEAD
#define MID_LOOKAHEAD 2                                   // weight tiles per wavefront in flight
#endif

namespace {

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_max_u16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ u32x2 lds_tr(const unsigned char* lds_byte_ptr) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(lds_byte_ptr));
    return __builtin_bit_cast(u32x2, r);
}
template <bool STAGE2>
__device__ __forceinline__ f32x4 mfma16(const u32x4& w, const u32x2& xlo, const u32x2& xhi, f32x4 acc) {
    u32x4 x = {xlo.x, xlo.y, xhi.x, xhi.y};
    if constexpr (STAGE2)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), acc, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), acc, 0, 0, 0);
}
// Exponent e of the power-of-two scale of a token whose largest |x| is m: bound_V * m * 2^e <= 2^14
// (the rule of the batched kernels).
__device__ __forceinline__ int scale_exponent(float m, float bound_V) {
    const float bound = bound_V * m;
    int ex = 0;
    if (bound > 0.f && bound < 3.0e38f) (void)frexpf(bound, &ex);
    return max(-110, min(110, 14 - ex));
}

template <int V> using ic = std::integral_constant<int, V>;
// f(ic<0>{}), f(ic<1>{}), ...: a loop whose index is a compile-time constant in the body
template <class F, int... U>
__device__ __forceinline__ void unrolled(F& f, std::integer_sequence<int, U...>) {
    (f(ic<U>{}), ...);
}

}  // namespace

// blockDim.x = 1024.  Wavefront w works on strip (w >> kw_log2) of the workgroup's sw strips with
// contraction split q = w & (kw - 1): tiles q, q + kw, q + 2 kw, ... of the strip; kw <= 8 divides
// the 8 tiles of a slab.  Wavefronts beyond sw << kw_log2 and strips beyond the matrix repeat valid
// work whose results are dropped, so every wavefront takes part in every barrier and every
// load is unconditional (clamped).
// VEC: activation rows are 16-byte aligned (16-byte buffer loads whose range check returns zero
// beyond the buffer); otherwise the slab is gathered element by element.  Either way a slab goes
// global -> registers (requested one slab ahead) -> LDS, with loads the compiler can see, so that
// its wait counts for the weight tiles stay exact.
// LDS position r' of a 64-row stage holds row r' ^ 2 ((r' >> 4 ^ r' >> 5) & 1): a transposed read
// touches rows {0, 4, 1, 5} + const of four lane groups, and with 32-byte rows the swap keeps
// the two lane groups served in one cycle on different banks.
// LTS: log2 of the tiles per wavefront and slab, 3 - log2(kw).  Everything in the main loop is
// unconditional and at a fixed place of the unrolled body (slabs beyond the contraction length
// are fetched as zeros by the range check, tiles beyond it are clamped re-reads that meet those
// zeros), so the compiler's wait counts are exact and no wait drains the tiles still in flight.
// RES: the contraction is at most two slabs long, so all activations are fetched at once and stay
// in LDS: no slab hand-over in the loop, and stage V reduces the token maxima while the first
// weight tiles are still on their way (measured on the 16384 x 4096 x 8192 shape, stage V with one
// tile per wavefront and slab: each hand-over waited a full L2 round trip, 6 us for two tiles).
template <bool STAGE2, bool VEC, int LTS, bool RES>
__global__ void __launch_bounds__(1024)
tsvd_mid_kernel(tsvd_mid_args p) {
    constexpr int KWL = 3 - LTS, n_ts = 1 << LTS, kw = 1 << KWL;
    extern __shared__ __align__(16) unsigned char smem[];
    float* cs_lds = reinterpret_cast<float*>(smem + 2 * MID_SLAB_BYTES);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    auto tick = [&](int n) {      // phase timestamps (100 MHz wall clock) of thread 0, for tuning
        if (p.clocks && tid == 0 && blockIdx.x < TSVD_GEMV_MAX_GRID) p.clocks[blockIdx.x * 16 + (STAGE2 ? 8 : 0) + n] = wall_clock64();
    };
    tick(0);
    const int sidx = wave >> KWL, q = wave & (kw - 1);
    const int strip = min(blockIdx.x * p.sw + sidx, p.strips - 1);
    const u32x4* wp = reinterpret_cast<const u32x4*>(p.tiles) + (size_t)strip * p.nkt * 64 + lane;
    const int nslab = (p.nkt + MID_SLAB_TILES - 1) / MID_SLAB_TILES;
    // operands of the epilogue, requested first: thread t finishes outputs t, t + 1024, ... (row
    // (t >> 4) + 64 n of the workgroup, token t & 15)
    float fin[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        if constexpr (STAGE2) fin[n] = n == 0 ? p.colmax[tid & 15] : 0.f;
        else fin[n] = p.S[min((int)blockIdx.x * p.sw * 16 + (tid >> 4) + 64 * n, p.strips * 16 - 1)];
    }

    // ---- slab fetch: thread t owns the 16-byte chunks t, t + 1024, t + 2048, t + 3072 of a slab
    // (chunk c: stage c >> 7, position (c >> 1) & 63, half c & 1)
    const int dd = (tid >> 7) & 3, rp = (tid >> 1) & 63, half = tid & 1;
    const int r = rp ^ ((((rp >> 4) ^ (rp >> 5)) & 1) << 1);
    const int kk = 256 * (tid >> 9) + 128 * (dd >> 1) + 32 * (dd & 1) + 64 * (r >> 5) + (r & 31);
    const int x_voff = kk * (int)p.ld * 2 + half * 16;
    const __amdgpu_buffer_rsrc_t act_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.act), 0, p.act_bytes, 0x00020000);
    u32x4 xreg[4], xreg2[4];
    auto fetch_slab = [&](int s, u32x4 (&xr)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (VEC) {
                xr[j] = __builtin_amdgcn_raw_buffer_load_b128(act_rsrc, x_voff, (s * 2048 + 512 * j) * (int)p.ld * 2, 0);
            } else {
                // unconditional loads (a load under a divergent condition makes the compiler wait for
                // it, and for the weight tiles in flight, right there), and none at all for token
                // positions that no thread needs: the bound is wave-uniform, so the skip is a scalar
                // branch.  The masks are applied only when the values are packed.
                const int k = s * 2048 + 512 * j + kk;
                const int tb = __builtin_amdgcn_readfirstlane(min(p.bvalid, 8));
                uint32_t e[8];
                if (p.pairs) {
                    // rows start on 4-byte boundaries: two tokens per range-checked 4-byte load (zero
                    // beyond the last row; with two tokens, one load per chunk instead of eight)
#pragma unroll
                    for (int t = 0; t < 8; t += 2) {
                        uint32_t v = 0u;
                        if (t < tb) v = __builtin_amdgcn_raw_buffer_load_b32(act_rsrc, k * (int)p.ld * 2 + (8 * half + t) * 2, 0, 0);
                        e[t] = v & 0xFFFFu;
                        e[t + 1] = v >> 16;
                    }
                } else {
                    const uint16_t* row = p.act + (size_t)min(k, p.kvalid - 1) * p.ld;
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        e[t] = 0u;
                        if (t < tb) e[t] = row[min(8 * half + t, p.bvalid - 1)];
                    }
                }
                const bool krow = k < p.kvalid;
#pragma unroll
                for (int t = 0; t < 8; ++t) e[t] = krow && 8 * half + t < p.bvalid ? e[t] : 0u;
                xr[j] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            }
        }
    };
    // the fetched slab goes to LDS; stage V also keeps running maxima of |x| over this thread's
    // chunks (tokens 8 half .. 8 half + 7, packed pairs)
    u32x4 cmax = {0u, 0u, 0u, 0u};
    auto commit_slab = [&](int s, const u32x4 (&xr)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            *reinterpret_cast<u32x4*>(smem + (s & 1) * MID_SLAB_BYTES + j * 16384 + tid * 16) = xr[j];
            if constexpr (!STAGE2)
                cmax = u32x4{pk_max_u16(cmax.x, xr[j].x & 0x7FFF7FFFu), pk_max_u16(cmax.y, xr[j].y & 0x7FFF7FFFu),
                             pk_max_u16(cmax.z, xr[j].z & 0x7FFF7FFFu), pk_max_u16(cmax.w, xr[j].w & 0x7FFF7FFFu)};
        }
    };
    // stage V: token maxima over all threads -> per-token factors in LDS (three barriers)
    u32x4* cm = reinterpret_cast<u32x4*>(smem + 2 * MID_SLAB_BYTES + 256);          // [1024]
    uint32_t* cm2 = reinterpret_cast<uint32_t*>(smem + 2 * MID_SLAB_BYTES + 256 + 16384);   // [128]
    auto reduce_maxima = [&]() {
        cm[tid] = cmax;
        __syncthreads();
        // threads of parity h hold tokens 8 h + 2 w (low half of word w) and 8 h + 2 w + 1 (high half)
        if (tid < 128) {
            const int h = tid & 1, w = (tid >> 1) & 3, part = tid >> 3;
            const uint32_t* cw = reinterpret_cast<const uint32_t*>(cm);
            uint32_t best = 0;
            for (int n = 0; n < 32; ++n) best = pk_max_u16(best, cw[(2 * (part * 32 + n) + h) * 4 + w]);
            cm2[tid] = best;
        }
        __syncthreads();
        if (tid < 16) {
            const int h = tid >> 3, w = (tid & 7) >> 1;
            uint32_t best = 0;
            for (int part = 0; part < 16; ++part) best = pk_max_u16(best, cm2[(part << 3) | (w << 1) | h]);
            const float mx = __uint_as_float(((tid & 1) ? (best >> 16) : (best & 0xFFFFu)) << 16);
            cs_lds[tid] = ldexpf(1.0f, scale_exponent(mx, p.bound_V) - 1);   // 1/2 undoes the +-2 of the codes
            if (blockIdx.x == 0) p.colmax[tid] = mx;
        }
        __syncthreads();
    };

    // ---- operand reads: lane (i, g) of a transposed read supplies the address of row
    // 32 (g & 1) + 16 (g >> 1) + {0, 4, 1, 5}[i >> 2] (first four operand elements; + 2 for the last
    // four; + 8 for the odd codes), bytes 8 (i & 3) .. of it
    const int rsel = i >> 2;
    const int tr_row = 32 * (g & 1) + 16 * (g >> 1) + (rsel >> 1) + 4 * (rsel & 1);
    const int sw2 = (g & 1) ^ (g >> 1);                   // bit 4 ^ bit 5 of tr_row
    const int rd_lo = (tr_row + 2 * sw2) * 32 + (i & 3) * 8;
    const int rd_hi = (tr_row + 2 * (1 - sw2)) * 32 + (i & 3) * 8;
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    auto tile = [&](const u32x4& w, const unsigned char* tb) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t ww = d == 0 ? w.x : d == 1 ? w.y : d == 2 ? w.z : w.w;
            const unsigned char* sb = tb + d * MID_STAGE_BYTES;
            const u32x2 lo0 = lds_tr(sb + rd_lo), hi0 = lds_tr(sb + rd_hi);
            const u32x2 lo1 = lds_tr(sb + rd_lo + 256), hi1 = lds_tr(sb + rd_hi + 256);
            // register m of the operand = codes hh + 2 m (low half) and hh + 2 m + 8 (high half)
            const u32x4 av0 = {MID_DEC(ww, 0), MID_DEC(ww, 2), MID_DEC(ww, 4), MID_DEC(ww, 6)};
            const u32x4 av1 = {MID_DEC(ww, 1), MID_DEC(ww, 3), MID_DEC(ww, 5), ww & 0xC000C000u};
            acc0 = mfma16<STAGE2>(av0, lo0, hi0, acc0);
            acc1 = mfma16<STAGE2>(av1, lo1, hi1, acc1);
        }
    };
    // Tile m of this wavefront is tile T = q + m kw of the strip and lies in slab m >> LTS.  Four
    // register sets rotate: tile m is consumed from set m % 4 while tiles m + 1 .. m + LA are in
    // flight (the loop is unrolled so that the sets are fixed registers: a rotation by copying
    // would have to wait for the tiles still in flight).  The first tile of slab s moves the slab
    // (fetched one slab earlier) from registers into LDS and requests slab s + 1.
    constexpr int LA = MID_LOOKAHEAD, ROUND = n_ts > 4 ? n_ts : 4;
    static_assert(LA >= 1 && LA <= 3, "lookahead");
    u32x4 wbuf[4];
    const int steps_valid = nslab << LTS;
    const int steps = (steps_valid + ROUND - 1) / ROUND * ROUND;
    fetch_slab(0, xreg);
    if constexpr (RES) fetch_slab(1, xreg2);
    __builtin_amdgcn_sched_barrier(0);        // activations first: the same request order as inside the loop
#pragma unroll
    for (int n = 0; n < LA; ++n) wbuf[n] = __builtin_nontemporal_load(wp + (size_t)min(q + n * kw, p.nkt - 1) * 64);
    tick(1);
    if constexpr (RES) {
        commit_slab(0, xreg);
        commit_slab(1, xreg2);
        __syncthreads();
        if constexpr (!STAGE2) reduce_maxima();
    }
    for (int m0 = 0; m0 < steps; m0 += ROUND) {
        auto step = [&](auto uc) {
            constexpr int u = decltype(uc)::value;
            const int m = m0 + u, s = m >> LTS, T = q + (m << KWL);
            if constexpr (!RES && (u & (n_ts - 1)) == 0) {
                commit_slab(s, xreg);
                __syncthreads();                   // slab s complete; nobody reads slab s - 1 any more
                fetch_slab(s + 1, xreg);
                if (s == 0) tick(6);
                if (s == nslab - 1) tick(7);
            }
            __builtin_amdgcn_sched_barrier(0);
            wbuf[(u + LA) % 4] = __builtin_nontemporal_load(wp + (size_t)min(T + LA * kw, p.nkt - 1) * 64);
            const unsigned char* tb = smem + (s & 1) * MID_SLAB_BYTES + (T & (MID_SLAB_TILES - 1)) * (4 * MID_STAGE_BYTES);
            if constexpr (RES) {
                if (m < steps_valid) tile(wbuf[u % 4], tb);     // (no third slab to meet the padding steps)
            } else {
                tile(wbuf[u % 4], tb);
            }
        };
        unrolled(step, std::make_integer_sequence<int, ROUND>{});
    }
    tick(2);
    __syncthreads();
    tick(3);

    // ---- reduce the contraction splits through LDS (the slabs are dead), finish, store
    float* red = reinterpret_cast<float*>(smem);                      // [16 wavefronts][16 rows][16 tokens]
    // result block of the MFMA: lane (i, g) holds token i, weight rows 4 g + v
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave * 256 + (4 * g + v) * 16 + i] = acc0[v] + acc1[v];
    if constexpr (!STAGE2 && !RES) reduce_maxima();      // (its first barrier also publishes red)
    else __syncthreads();
    tick(4);
    const int tok = tid & 15;
    const float ftok = STAGE2 ? ldexpf(1.0f, -scale_exponent(fin[0], p.bound_V) - 1) : cs_lds[tok];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int rl = (tid >> 4) + 64 * n;                    // row within the workgroup
        if (rl < p.sw * 16) {
            const float* src = red + (size_t)((rl >> 4) * kw) * 256 + (rl & 15) * 16 + tok;
            float sum = 0.f;
#pragma unroll
            for (int c = 0; c < kw; ++c) sum += src[c * 256];
            const int row = blockIdx.x * p.sw * 16 + rl;
            if constexpr (STAGE2) {
                if (row < p.rows_valid && tok < p.bvalid)
                    tsvd_store_y(p.out, p.out_token_major ? (size_t)tok * p.ld_out + row : (size_t)row * p.ld_out + tok,
                                 p.bias ? sum * ftok + p.bias[row] : sum * ftok, p.out_bf16);
            } else {
                if (row < p.strips * 16)   // S is zero beyond K: padded rows of z are written as zeros
                    static_cast<_Float16*>(p.out)[(size_t)row * 16 + tok] = (_Float16)((sum * fin[n]) * ftok);
            }
        }
    }
    tick(5);
}

namespace {
template <bool STAGE2, bool VEC, int LTS>
hipError_t init_one() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_mid_kernel<STAGE2, VEC, LTS, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, MID_LDS_BYTES);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_mid_kernel<STAGE2, VEC, LTS, true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, MID_LDS_BYTES);
}
template <bool STAGE2, bool VEC>
hipError_t init_all() {
    hipError_t e;
    if ((e = init_one<STAGE2, VEC, 0>()) != hipSuccess) return e;
    if ((e = init_one<STAGE2, VEC, 1>()) != hipSuccess) return e;
    if ((e = init_one<STAGE2, VEC, 2>()) != hipSuccess) return e;
    return init_one<STAGE2, VEC, 3>();
}
template <bool STAGE2, bool VEC>
void launch(const tsvd_mid_args& a, dim3 grid, hipStream_t stream) {
    const dim3 block(1024);
    const bool res = a.nkt <= 2 * MID_SLAB_TILES && a.resident_ok;
#define MID_LAUNCH(LTS)                                                                                              \
    do {                                                                                                             \
        if (res) hipLaunchKernelGGL((tsvd_mid_kernel<STAGE2, VEC, LTS, true>), grid, block, MID_LDS_BYTES, stream, a);  \
        else hipLaunchKernelGGL((tsvd_mid_kernel<STAGE2, VEC, LTS, false>), grid, block, MID_LDS_BYTES, stream, a);     \
    } while (0)
    switch (3 - a.kw_log2) {
        case 0: MID_LAUNCH(0); break;
        case 1: MID_LAUNCH(1); break;
        case 2: MID_LAUNCH(2); break;
        default: MID_LAUNCH(3); break;
    }
#undef MID_LAUNCH
}
}  // namespace

hipError_t tsvd_mid_init() {
    hipError_t e;
    if ((e = init_all<false, true>()) != hipSuccess) return e;
    if ((e = init_all<false, false>()) != hipSuccess) return e;
    return init_all<true, true>();
}

hipError_t tsvd_launch_mid(const tsvd_mid_args& a, bool stage_u, bool vec, hipStream_t stream) {
    if (a.sw < 1 || a.kw_log2 < 0 || a.kw_log2 > 3 || (a.sw << a.kw_log2) > 16 || a.strips < 1 || a.nkt < 1 ||
        a.bvalid < 1 || a.bvalid > 16 || (stage_u && !vec))
        return hipErrorInvalidValue;
    const dim3 grid((a.strips + a.sw - 1) / a.sw);
    if (stage_u) launch<true, true>(a, grid, stream);
    else if (vec) launch<false, true>(a, grid, stream);
    else launch<false, false>(a, grid, stream);
    return hipGetLastError();
}
