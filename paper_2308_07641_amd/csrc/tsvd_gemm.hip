// Batched path (B >= 17, bf16 activations; the few-token kernels take most calls below 65 tokens): both stages of Y = U (diag(S) (V X)) as
// ternary-weight x 16-bit-activation contractions on the matrix cores.
//
// Paper: section "Truncated SVD in Network Compression" (the three-step identity) and
// supplement Table S1 (V(.) and U(.) are additions, diag(S)(.) is K multiplications per
// token).  With hundreds of tokens per weight the work is a dense contraction, so the 2-bit
// codes are expanded exactly to +-2 / 0 16-bit floats in registers (one shift and one mask per
// pair) and fed to v_mfma_f32_16x16x32; products are exact and accumulation is fp32.
//
//   kernel 0  column maxima of |X| (partial, per row slice)       -> workspace
//   kernel 1  Z = fp16( scale_b * S_k * (V X)[k][b] )            (bf16 MFMA, S fused in the epilogue)
//   kernel 2  Y = (U Z)[m][b] / scale_b                           (fp16 MFMA)
//
// scale_b is a power of two chosen from the bound |z[k][b]| <= max_k(|S_k| nnz(V[k,:])) *
// max_n |x[n][b]| so that fp16 cannot overflow; fp16 keeps 11 significant bits of z where bf16
// would keep 8 (the 8-bit rounding alone costs about 1.7e-3 of max|y| at these shapes).
//
// Weights never pass through LDS: each wavefront loads the code words of its own rows straight
// from L2 (they are 8x smaller than the activations).  One 32-bit code word per lane covers the
// 64 contraction indices k0 + {0..31} and k0 + 64 + {0..31} (the tile order is that of the fp4
// MFMA operand used by the skinny path), so an LDS stage holds exactly those 64 activation rows
// [64][BT tokens], row-major with a 32-byte XOR swizzle, read in MFMA operand order with
// ds_read_b64_tr_b16.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <algorithm>
#include <type_traits>
#include <cmath>

#include "tsvd_gemm_common.h"

#ifndef TSVD_SCHED
#define TSVD_SCHED 1
#endif
#ifndef TSVD_STEP_FENCE
#define TSVD_STEP_FENCE 1
#endif
// workgroup shape of the large-tile kernels: WM x WN wavefronts of TM x TN MFMA blocks (256 x 256 tile)
#ifndef TSVD_BIG
#define TSVD_BIG 2, 4, 8, 4
#endif

namespace {

// ---- kernel 0: partial column maxima of |x| ----------------------------------------------
// grid (ceil(B/128), PARTS); block 256 = 64 column pairs x 4 row lanes.  part[p][b] = max over
// the rows of slice p of |x[n][b]| as an fp32 value.
__global__ void __launch_bounds__(256)
tsvd_colmax_kernel(const uint16_t* __restrict__ x, long long ldx, int N, int B, int Bp, float* __restrict__ part) {
    __shared__ uint32_t red[4][128];
    const int cp = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int c0 = blockIdx.x * 128 + 2 * cp;
    const int rows_per = (N + gridDim.y - 1) / gridDim.y;
    const int r0 = blockIdx.y * rows_per, r1 = min(N, r0 + rows_per);
    uint32_t m0 = 0, m1 = 0;       // magnitudes as bf16 bit patterns (order-preserving)
    for (int r = r0 + rl; r < r1; r += 4) {
        const uint16_t* row = x + (size_t)r * ldx;
        if (c0 < B) m0 = max(m0, (uint32_t)(row[c0] & 0x7FFFu));
        if (c0 + 1 < B) m1 = max(m1, (uint32_t)(row[c0 + 1] & 0x7FFFu));
    }
    red[rl][2 * cp] = m0;
    red[rl][2 * cp + 1] = m1;
    __syncthreads();
    if (threadIdx.x < 128) {
        const int c = blockIdx.x * 128 + threadIdx.x;
        uint32_t m = max(max(red[0][threadIdx.x], red[1][threadIdx.x]), max(red[2][threadIdx.x], red[3][threadIdx.x]));
        if (c < Bp) part[(size_t)blockIdx.y * Bp + c] = __uint_as_float(m << 16);
    }
}

// Per-half maximum of two words holding two 16-bit magnitudes each.
__device__ __forceinline__ uint32_t max_halves(uint32_t a, uint32_t b) {
    const uint32_t lo = max(a & 0xFFFFu, b & 0xFFFFu), hi = max(a >> 16, b >> 16);
    return lo | (hi << 16);
}

// Same result for 16-byte-aligned rows: each thread owns 8 adjacent columns and reads 16 bytes per
// row.  grid (ceil(B/128), PARTS); block 256 = 16 column groups x 16 row lanes.  Columns >= B of
// the group that straddles B are read element by element.
__global__ void __launch_bounds__(256)
tsvd_colmax_vec_kernel(const uint16_t* __restrict__ x, long long ldx, int N, int B, int Bp, float* __restrict__ part) {
    __shared__ u32x4 red[16][16];
    const int cg = threadIdx.x & 15, rl = threadIdx.x >> 4;
    const int c0 = blockIdx.x * 128 + 8 * cg;
    const int rows_per = (N + gridDim.y - 1) / gridDim.y;
    const int r0 = blockIdx.y * rows_per, r1 = min(N, r0 + rows_per);
    u32x4 m = {0u, 0u, 0u, 0u};          // packed 16-bit magnitudes (order-preserving bit patterns)
    if (c0 + 8 <= B) {
        // four independent 16-byte loads in flight; rows past the slice are clamped (max is idempotent)
        for (int r = r0 + rl; r < r1; r += 64) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const u32x4*>(x + (size_t)min(r + 16 * u, r1 - 1) * ldx + c0);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v[u] &= 0x7FFF7FFFu;
                m = u32x4{max_halves(m.x, v[u].x), max_halves(m.y, v[u].y), max_halves(m.z, v[u].z), max_halves(m.w, v[u].w)};
            }
        }
    } else if (c0 < B) {                  // the group that straddles B: element by element
        for (int r = r0 + rl; r < r1; r += 16) {
            uint32_t e[8];
            for (int t = 0; t < 8; ++t) e[t] = c0 + t < B ? (uint32_t)(x[(size_t)r * ldx + c0 + t] & 0x7FFFu) : 0u;
            const u32x4 v = {e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            m = u32x4{max_halves(m.x, v.x), max_halves(m.y, v.y), max_halves(m.z, v.z), max_halves(m.w, v.w)};
        }
    }
    red[rl][cg] = m;
    __syncthreads();
    if (threadIdx.x < 64) {              // thread t finishes column pair t of the block's 128 columns
        const int grp = threadIdx.x >> 2, w = threadIdx.x & 3;
        uint32_t best = 0;
        for (int l = 0; l < 16; ++l) {
            const u32x4 q = red[l][grp];
            best = max_halves(best, w == 0 ? q.x : w == 1 ? q.y : w == 2 ? q.z : q.w);
        }
        const int c = blockIdx.x * 128 + 2 * threadIdx.x;
        if (c < Bp) part[(size_t)blockIdx.y * Bp + c] = __uint_as_float(best << 16);
        if (c + 1 < Bp) part[(size_t)blockIdx.y * Bp + c + 1] = __uint_as_float(best & 0xFFFF0000u);
    }
}

// XOR swizzle of the activation tiles in LDS: row r stores its logical 32-byte block j at block
// j ^ swizzle(r).  One transposed read (ds_read_b64_tr_b16) touches rows
// 32 (g & 1) + 16 (g >> 1) + {0, 4, 1, 5} (+ a constant) for lane groups g = 0..3, 32 bytes of each.
// The 64-bank LDS serves half a wavefront (two lane groups, eight such segments = 256 bytes) per
// cycle, so those eight rows need eight different bank groups: row bits 0 and 2 tell the four
// rows of a lane group apart and bit 4 ^ bit 5 tells apart the lane groups of either half
// (and of the even/odd pairing).  With 128-byte rows (4 blocks) bit 0 already selects the bank
// half, so two swizzle bits suffice; 64-byte rows (2 blocks) cannot avoid two-way conflicts.
template <int NBLK>
__device__ __forceinline__ constexpr int swizzle(int r) {
    const int q = ((r >> 4) ^ (r >> 5)) & 1;
    return NBLK >= 8 ? (((r >> 2) & 1) | ((r & 1) << 1) | (q << 2)) : NBLK == 4 ? (((r >> 2) & 1) | (q << 1)) : ((r >> 2) & 1);
}

// ---- kernels 1 and 2 ------------------------------------------------------------------------

// One MFMA block: decoded weights as the row operand, activations as the column operand, so a lane
// (i, g) of the result holds token i of the weight rows 4 g .. 4 g + 3.  (Both operands have the same
// register layout, so swapping them gives the transposed result, four adjacent tokens of one weight
// row per lane and one vector store per block: measured in the ring kernel on a 3072 x 1536 factor at
// 512 tokens, the stores of a workgroup then issue in 0.6 instead of 1.3 us but the call stays at
// 17.1 us, so the plain layout was kept.)
template <bool STAGE2>
__device__ __forceinline__ f32x4 mfma16(const u32x4& w, const u32x2& xlo, const u32x2& xhi, f32x4 acc) {
    u32x4 x = {xlo.x, xlo.y, xhi.x, xhi.y};
    if constexpr (STAGE2)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), acc, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), acc, 0, 0, 0);
}

__device__ __forceinline__ u32x2 lds_tr(const unsigned char* lds_byte_ptr) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(lds_byte_ptr));
    return __builtin_bit_cast(u32x2, r);
}

// Workgroup tile (WM*TM*16 rows) x (WN*TN*16 tokens); WM x WN wavefronts, each TM x TN MFMA blocks.
// FAST: activation rows are 16-byte aligned, so tiles are fetched with buffer loads whose
// range check returns zero beyond the last row (no per-element guards, no address arithmetic
// in the loop: a per-thread offset plus a scalar offset per stage).
template <int WM, int WN, int TM, int TN, bool STAGE2, bool FAST, int EX = 0>
__global__ void __launch_bounds__(64 * WM * WN)
tsvd_gemm_kernel(gemm_args p) {
    constexpr int THREADS = 64 * WM * WN;
    constexpr int BT = WN * TN * 16;                 // tokens per workgroup tile
    constexpr int ROWB = BT * 2;                     // bytes per LDS row
    constexpr int NBLK = BT / 16;                    // 32-byte blocks per LDS row
    constexpr int CPR = BT / 8;                      // 16-byte chunks per LDS row
    constexpr int CHUNKS = KT * CPR;                 // chunks per stage
    constexpr int CPT = CHUNKS / THREADS;            // chunks per thread
    constexpr int STAGE_BYTES = KT * ROWB;
    static_assert(CHUNKS % THREADS == 0 && THREADS % CPR == 0, "tile/threads mismatch");
    static_assert(BT <= THREADS, "one thread per token of the tile");
    extern __shared__ __align__(16) unsigned char smem[];   // 2 stages x KT x ROWB, then BT column factors
    float* cs_lds = reinterpret_cast<float*>(smem + 2 * STAGE_BYTES);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave - wm * WN;
    const int i = lane & 15, g = lane >> 4;
    const int b0 = blockIdx.x * BT;
    const int strip0 = (blockIdx.y * WM + wm) * TM;  // first 16-row strip of this wavefront
    const int nstages = 2 * p.npairs - (p.last_steps <= 2 ? 1 : 0);   // (a stage is one code word: two sub-steps)

    // Stage st covers code word d = st & 3 of tile T = st >> 2: contraction indices
    // k0 + 64 (r >> 5) + (r & 31), r = 0..63, with k0 = 256 T + 128 (d >> 1) + 32 (d & 1).
    // LDS row r, 32-byte block j is stored at block j ^ f(r),
    //   f(r) = ((r & 1) << 1) | ((r >> 2) & 1) | (((r >> 4) & 3) << 2).
    // For MFMA step hh (code parity) lane group g needs rows 32 (g & 1) + 16 (g >> 1) + 8 hh + o with
    // o = {0,4,1,5} (first four operand elements) and o + 2 (last four): 16 rows with 16 distinct f.
    const int rsel = i >> 2;
    const int tr_row = 32 * (g & 1) + 16 * (g >> 1) + (rsel >> 1) + 4 * (rsel & 1);
    const int f_lane = swizzle<NBLK>(tr_row);
    int lds_rd[TN];                                   // byte offset of this lane's transposed reads
#pragma unroll
    for (int b = 0; b < TN; ++b) lds_rd[b] = tr_row * ROWB + (((wn * TN + b) ^ f_lane) * 32) + (i & 3) * 8;

    // activation chunk c of this thread: LDS row r_c, 16-byte chunk ch (same for all c)
    const int ch = threadIdx.x % CPR, r_first = threadIdx.x / CPR;
    int lds_wr[CPT], x_voff[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int r = r_first + c * (THREADS / CPR);
        const int f = swizzle<NBLK>(r);
        lds_wr[c] = r * ROWB + (((ch >> 1) ^ f) * 32) + (ch & 1) * 16;
        x_voff[c] = (64 * (r >> 5) + (r & 31)) * (int)p.ld * 2 + (b0 + ch * 8) * 2;
    }
    const __amdgpu_buffer_rsrc_t act_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.act), 0, p.act_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.tiles), 0, p.tile_bytes, 0x00020000);

    f32x4 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto stage_k0 = [](int stage) { return 256 * (stage >> 2) + 128 * ((stage >> 1) & 1) + 32 * (stage & 1); };

    // ---- activation tile: global -> registers -> LDS
    u32x4 xreg[CPT];
    auto load_x = [&](int stage) {
        const int k0 = stage_k0(stage);
        if constexpr (FAST) {
            const int soff = k0 * (int)p.ld * 2;
#pragma unroll
            for (int c = 0; c < CPT; ++c) xreg[c] = buf_load128(act_rsrc, x_voff[c], soff);
        } else {
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const int r = r_first + c * (THREADS / CPR);
                const int k = k0 + 64 * (r >> 5) + (r & 31), col = b0 + ch * 8;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (k < p.kvalid) {
                    const uint16_t* src = p.act + (size_t)k * p.ld + col;
                    uint32_t e[8];
#pragma unroll
                    for (int t = 0; t < 8; ++t) e[t] = (col + t < p.bvalid) ? (uint32_t)src[t] : 0u;
                    v = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
                }
                xreg[c] = v;
            }
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int c = 0; c < CPT; ++c) *reinterpret_cast<u32x4*>(smem + buf * STAGE_BYTES + lds_wr[c]) = xreg[c];
    };
    // ---- weights: one code word per strip and stage, straight from global/L2
    const int w_voff = lane * 16;
    auto load_w = [&](int stage, uint32_t (&w)[TM]) {
        const int soff = (strip0 * p.nkt + (stage >> 2)) * 1024 + (stage & 3) * 4;
#pragma unroll
        for (int a = 0; a < TM; ++a) w[a] = buf_load32(w_rsrc, w_voff, soff + a * p.nkt * 1024);
    };
    auto compute = [&](int buf, const uint32_t (&w)[TM]) {
        const unsigned char* base = smem + buf * STAGE_BYTES;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            u32x2 blo[TN], bhi[TN];
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                blo[b] = lds_tr(base + lds_rd[b] + hh * 8 * ROWB);
                bhi[b] = lds_tr(base + lds_rd[b] + hh * 8 * ROWB + 2 * ROWB);
            }
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const uint32_t ww = w[a];
                // register m of the operand = codes hh + 2 m (low half) and hh + 2 m + 8 (high half)
                u32x4 av;
                if (hh == 0) av = u32x4{TSVD_DEC(ww, 0), TSVD_DEC(ww, 2), TSVD_DEC(ww, 4), TSVD_DEC(ww, 6)};
                else         av = u32x4{TSVD_DEC(ww, 1), TSVD_DEC(ww, 3), TSVD_DEC(ww, 5), ww & 0xC000C000u};
#pragma unroll
                for (int b = 0; b < TN; ++b) acc[a][b] = mfma16<STAGE2>(av, blo[b], bhi[b], acc[a][b]);
            }
        }
    };

    uint32_t w0[TM], w1[TM];
    load_x(0);
    load_w(0, w0);
    if (threadIdx.x < BT)
        publish_column_factor<STAGE2>(p, b0 + threadIdx.x, load_column_max<STAGE2>(p, b0 + threadIdx.x), cs_lds, threadIdx.x);
    store_x(0);
    __syncthreads();

    // Two stages per iteration so that the LDS buffer and the weight registers alternate at
    // compile time.  The prefetch of the stage after the last one re-reads the last stage
    // (unconditional loads keep the wait counts exact); its results are never used.
    const int last = nstages - 1;
    for (int s = 0; s < nstages; s += 2) {
        load_x(min(s + 1, last));
        load_w(min(s + 1, last), w1);
        compute(0, w0);
        store_x(1);
        __syncthreads();
        load_x(min(s + 2, last));
        load_w(min(s + 2, last), w0);
        if (s + 1 < nstages) compute(1, w1);
        store_x(0);
        __syncthreads();
    }

    gemm_epilogue<TM, TN, STAGE2, EX>(p, acc, strip0, b0, wn * TN * 16, cs_lds, i, g);
}

// ---- pipelined variant (activation rows 16-byte aligned) -----------------------------------
// Same tiling and arithmetic as tsvd_gemm_kernel, different data movement: activation tiles go
// from global memory straight into LDS (buffer_load ... lds, 16 bytes per lane, no registers, the
// range check writes zeros beyond the last row), two stages ahead of the MFMAs, through a ring of
// four LDS buffers.  One barrier per stage.  Each wavefront fills SPW 1-KiB slots per stage; a
// slot is written in lane order, so the XOR swizzle is applied on the global side (which chunk
// of the row a lane fetches).
template <int WM, int WN, int TM, int TN, bool STAGE2, int EX = 0>
__global__ void __launch_bounds__(64 * WM * WN, 2)     // two wavefronts per SIMD: at most 256 VGPRs
tsvd_gemm_pipe_kernel(gemm_args p) {
    constexpr int NW = WM * WN;
    constexpr int BT = WN * TN * 16;                 // tokens per workgroup tile
    constexpr int ROWB = BT * 2;                     // bytes per LDS row
    constexpr int NBLK = BT / 16;                    // 32-byte blocks per LDS row
    constexpr int CPR = BT / 8;                      // 16-byte chunks per LDS row
    constexpr int STAGE_BYTES = KT * ROWB;
    constexpr int SLOTS = STAGE_BYTES / 1024;        // 1-KiB slots per stage
    constexpr int SPW = SLOTS / NW;                  // slots per wavefront
    constexpr int RPS = 64 / CPR;                    // rows per slot
    static_assert(SLOTS % NW == 0 && 64 % CPR == 0, "tile/wavefront mismatch");
    static_assert(BT <= 64 * NW, "one thread per token of the tile");
    extern __shared__ __align__(16) unsigned char smem[];   // 4 stages x KT x ROWB, then BT column factors
    float* cs_lds = reinterpret_cast<float*>(smem + 4 * STAGE_BYTES);

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave - wm * WN;
    const int i = lane & 15, g = lane >> 4;
    const int b0 = blockIdx.x * BT;
    const int strip0 = (blockIdx.y * WM + wm) * TM;
    const int nstages = 2 * p.npairs;
    auto tick = [&](int n) {
        const unsigned wg = blockIdx.y * gridDim.x + blockIdx.x;
        if (p.clocks && threadIdx.x == 0 && wg < TSVD_GEMV_MAX_GRID) p.clocks[wg * 16 + (STAGE2 ? 8 : 0) + n] = wall_clock64();
    };
    tick(0);

    // (row and swizzle conventions: see tsvd_gemm_kernel)
    const int rsel = i >> 2;
    const int tr_row = 32 * (g & 1) + 16 * (g >> 1) + (rsel >> 1) + 4 * (rsel & 1);
    const int f_lane = swizzle<NBLK>(tr_row);
    int lds_rd[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) lds_rd[b] = tr_row * ROWB + (((wn * TN + b) ^ f_lane) * 32) + (i & 3) * 8;

    // slot j = c * NW + wave of a stage holds LDS rows j * RPS .. ; lane l writes physical chunk l % CPR
    // of row j * RPS + l / CPR, which must hold logical chunk ((pc >> 1) ^ f(row)) * 2 + (pc & 1).
    int x_voff[SPW];
#pragma unroll
    for (int c = 0; c < SPW; ++c) {
        const int r = (c * NW + wave) * RPS + lane / CPR, pc = lane % CPR;
        const int f = swizzle<NBLK>(r);
        const int lc = (((pc >> 1) ^ f) << 1) | (pc & 1);
        x_voff[c] = (64 * (r >> 5) + (r & 31)) * (int)p.ld * 2 + (b0 + lc * 8) * 2;
    }
    const i32x4 act_rsrc = raw_rsrc(p.act, p.act_bytes);
    const __amdgpu_buffer_rsrc_t w_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.tiles), 0, p.tile_bytes, 0x00020000);
    typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_byte_ptr)smem + wave * 1024;

    f32x4 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto issue_x = [&](int stage, int buf) {
        const int soff = (256 * (stage >> 2) + 128 * ((stage >> 1) & 1) + 32 * (stage & 1)) * (int)p.ld * 2;
#pragma unroll
        for (int c = 0; c < SPW; ++c)
            buf_load128_to_lds(act_rsrc, lds0 + buf * STAGE_BYTES + c * NW * 1024, x_voff[c], soff);
    };
    // weights: the two code words of a pair of stages per strip, straight from global/L2
    const int w_voff = lane * 16;
    auto load_w = [&](int pair, u32x2 (&w)[TM]) {
        const int soff = (strip0 * p.nkt + (pair >> 1)) * 1024 + (pair & 1) * 8;
#pragma unroll
        for (int a = 0; a < TM; ++a) w[a] = __builtin_amdgcn_raw_buffer_load_b64(w_rsrc, w_voff, soff + a * p.nkt * 1024, 0);
    };
    // A pair of stages = four MFMA steps (stage, code parity).  The activation operands of step
    // n + 1 are read from LDS while the MFMAs of step n run (two register sets); scheduling fences
    // keep the compiler from hoisting later steps and overflowing the register file.
    auto load_frags = [&](int buf, int hh, u32x2 (&lo)[TN], u32x2 (&hi)[TN]) {
        const unsigned char* base = smem + buf * STAGE_BYTES + hh * 8 * ROWB;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            lo[b] = lds_tr(base + lds_rd[b]);
            hi[b] = lds_tr(base + lds_rd[b] + 2 * ROWB);
        }
    };
    auto mfma_step = [&](const u32x2 (&w)[TM], int word, int hh, const u32x2 (&lo)[TN], const u32x2 (&hi)[TN]) {
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const uint32_t ww = word == 0 ? w[a].x : w[a].y;
            u32x4 av;
            if (hh == 0) av = u32x4{TSVD_DEC(ww, 0), TSVD_DEC(ww, 2), TSVD_DEC(ww, 4), TSVD_DEC(ww, 6)};
            else         av = u32x4{TSVD_DEC(ww, 1), TSVD_DEC(ww, 3), TSVD_DEC(ww, 5), ww & 0xC000C000u};
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] = mfma16<STAGE2>(av, lo[b], hi[b], acc[a][b]);
        }
    };
    // Issue order inside one step: the LDS reads of the next step first, the decode of the first
    // strip, then one MFMA followed by two decode operations of the next strip, and so on: the
    // decode hides in the shadow of the MFMAs instead of alternating with them in blocks.
    // (The 8-wavefront shape has no registers to spare for the second set of decoded operands.)
#define TSVD_INTERLEAVE(DS_READS)                                                        \
    do {                                                                                 \
        if constexpr (TSVD_SCHED && NW <= 4) {                                           \
            if constexpr ((DS_READS) > 0) __builtin_amdgcn_sched_group_barrier(0x100, (DS_READS), 0); \
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);                           \
            _Pragma("unroll") for (int n_ = 0; n_ < TM * TN; ++n_) {                     \
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       \
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);                       \
            }                                                                            \
        }                                                                                \
    } while (0)
    auto compute_pair = [&](int buf0, const u32x2 (&w)[TM]) {
        u32x2 f0lo[TN], f0hi[TN], f1lo[TN], f1hi[TN];
        load_frags(buf0, 0, f0lo, f0hi);
        load_frags(buf0, 1, f1lo, f1hi);
        mfma_step(w, 0, 0, f0lo, f0hi);
        TSVD_INTERLEAVE(4 * TN);
        if (TSVD_STEP_FENCE) __builtin_amdgcn_sched_barrier(0);
        load_frags(buf0 + 1, 0, f0lo, f0hi);
        mfma_step(w, 0, 1, f1lo, f1hi);
        TSVD_INTERLEAVE(2 * TN);
        if (TSVD_STEP_FENCE) __builtin_amdgcn_sched_barrier(0);
        load_frags(buf0 + 1, 1, f1lo, f1hi);
        mfma_step(w, 1, 0, f0lo, f0hi);
        TSVD_INTERLEAVE(2 * TN);
        if (TSVD_STEP_FENCE) __builtin_amdgcn_sched_barrier(0);
        mfma_step(w, 1, 1, f1lo, f1hi);
        TSVD_INTERLEAVE(0);
        __builtin_amdgcn_sched_barrier(0);
    };

    // A pair of stages (128 contraction indices, two LDS buffers) per barrier.  While pair P is
    // multiplied, the activations of pair P + 1 stream into the other two buffers and its code
    // words into registers.  Loads past the last pair re-read it (never used).
    // The compiler does not see the LDS-bound loads, so its own wait for a code word (counted in
    // the loads it knows) would also drain the activation loads issued after it.  Using the words
    // right after the explicit wait makes the compiler place its wait there, where it costs nothing.
    auto touch = [&](const u32x2 (&w)[TM]) {
#pragma unroll
        for (int a = 0; a < TM; ++a) asm volatile("" :: "v"(w[a].x), "v"(w[a].y));
    };
    const int npairs = nstages / 2, lastp = npairs - 1;
    u32x2 wa[TM], wb[TM];
    float cmax = 0.f;
    if (threadIdx.x < BT) cmax = load_column_max<STAGE2>(p, b0 + threadIdx.x);
    load_w(0, wa);
    issue_x(0, 0);
    issue_x(1, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    touch(wa);
    if (threadIdx.x < BT) publish_column_factor<STAGE2>(p, b0 + threadIdx.x, cmax, cs_lds, threadIdx.x);
    __syncthreads();
    tick(2);

    for (int P = 0; P < npairs; P += 2) {           // one 256-wide tile of codes per iteration
        int nx = min(P + 1, lastp);
        load_w(nx, wb);
        issue_x(2 * nx, 2);
        issue_x(2 * nx + 1, 3);
        compute_pair(0, wa);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // pair P + 1 has landed (this wavefront's part)
        touch(wb);
        __syncthreads();

        nx = min(P + 2, lastp);
        load_w(nx, wa);
        issue_x(2 * nx, 0);
        issue_x(2 * nx + 1, 1);
        if (P + 1 <= lastp) compute_pair(2, wb);      // (an odd number of 128-index steps: the contraction ends inside this tile of codes)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        touch(wa);
        __syncthreads();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no LDS write may still be in flight at exit
    tick(3);

    gemm_epilogue<TM, TN, STAGE2, EX>(p, acc, strip0, b0, wn * TN * 16, cs_lds, i, g);
    tick(5);
}

// ---- ring variant for small problems -----------------------------------------------------------
// A launch with about one workgroup per compute unit cannot lean on other workgroups to hide its
// waits, and the 256-row tiles above would leave most compute units idle.  This variant uses small
// tiles and EVERY load of its main loop is a buffer_load ... lds issued from inline assembly: a ring
// of NPB slots, each holding one pair of stages (128 contraction indices) of activations AND the
// code words of the workgroup's rows for that pair; pair P + NPB - 1 is requested before pair P is
// multiplied, and the only waits are the explicit s_waitcnt vmcnt(n) below (vector-memory results
// return in issue order: the loads of the NPB - 2 younger pairs may still be in flight).  Code
// words take 4 bytes per lane per load (word j of strip s of the pair lands at
// s * 512 + j * 256 + 4 lane).  Measured on MI355X: small tiles are bound by what one compute unit
// can move (64 bytes per clock into LDS, 128 bytes per clock out of it), not by memory latency, so
// a ring of 3 that lets two or three workgroups share a compute unit beats rings of 4 to 6 with one.
//
// FUSEMAX (stage 1 only): the workgroup streams all N rows of its token columns through LDS anyway,
// so it also computes their largest magnitudes there; no column-maximum kernel runs before it.
__device__ __forceinline__ void buf_load32_to_lds(i32x4 rsrc, uint32_t lds_addr, int voff, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_pk_max_u16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// KG > 1 splits the contraction over KG groups of WM x WN wavefronts: a ring slot then holds KG
// pairs, group kg multiplies pair KG * P + kg, and the groups' accumulators are added through LDS
// at the end.  Same tile and same bytes moved, KG times the wavefronts to hide waits with.
template <int WM, int WN, int TM, int TN, bool STAGE2, int NPB, bool FUSEMAX, int KG, int EX = 0>
__global__ void __launch_bounds__(64 * WM * WN * KG)
tsvd_gemm_ring_kernel(gemm_args p) {
    constexpr int NWG = WM * WN, NW = NWG * KG, THREADS = 64 * NW;
    constexpr int BT = WN * TN * 16;                 // tokens per workgroup tile
    constexpr int ROWB = BT * 2;                     // bytes per LDS row
    constexpr int NBLK = BT / 16;                    // 32-byte blocks per LDS row
    constexpr int CPR = BT / 8;                      // 16-byte chunks per LDS row
    constexpr int STAGE_BYTES = KT * ROWB;
    constexpr int SLOTS = STAGE_BYTES / 1024;        // 1-KiB pieces per stage
    constexpr int SPW = SLOTS / NW;                  // pieces per wavefront and stage
    constexpr int RPS = 64 / CPR;                    // rows per piece
    constexpr int WSTRIPS = WM * TM;                 // 16-row strips of the workgroup tile
    constexpr int W_BYTES = WSTRIPS * 512;           // code words of one pair
    constexpr int WOPS = (WSTRIPS * 2 + NW - 1) / NW; // code-word loads per wavefront and pair (a load past the last strip repeats it)
    constexpr int SUB_BYTES = 2 * STAGE_BYTES + W_BYTES;   // one pair
    constexpr int SLOT_BYTES = KG * SUB_BYTES;       // one ring slot: KG pairs
    constexpr int OPS = KG * (2 * SPW + WOPS);       // loads per wavefront and slot
    constexpr int CPT = KT * CPR / THREADS;          // FUSEMAX: chunks per thread and stage
    static_assert(SLOTS % NW == 0 && 64 % CPR == 0 && NW % 2 == 0, "tile/wavefront mismatch");
    static_assert(NPB >= 2 && (NPB - 2) * OPS <= 63, "ring too deep for the load counter");
    static_assert(BT <= THREADS && (KT * CPR) % THREADS == 0 && THREADS % CPR == 0, "one thread per token of the tile");
    static_assert(!(FUSEMAX && STAGE2), "column maxima belong to stage 1");
    static_assert(THREADS * 16 <= NPB * SLOT_BYTES && (KG - 1) * NWG * 64 * TM * TN * 16 <= NPB * SLOT_BYTES, "the reductions reuse the ring");
    static_assert(KG == 1 || KG == 2, "pairs per tile of codes");
    extern __shared__ __align__(16) unsigned char smem[];   // NPB slots, then BT column factors
    float* cs_lds = reinterpret_cast<float*>(smem + NPB * SLOT_BYTES);

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kg = wave / NWG, w2 = wave - kg * NWG;
    const int wm = w2 / WN, wn = w2 - wm * WN;
    const int i = lane & 15, g = lane >> 4;
    const int b0 = blockIdx.x * BT;
    const int strip0 = (blockIdx.y * WM + wm) * TM;
    const int nslots = (p.npairs + KG - 1) / KG, lasts = nslots - 1;   // ring slots to go through
    // sub-steps of this wavefront group's pair in the last slot: all four, the partly filled last pair's, or none
    const int tail_steps = KG * lasts + kg < p.npairs - 1 ? 4 : KG * lasts + kg == p.npairs - 1 ? p.last_steps : 0;
    auto tick = [&](int n) {
        const unsigned wg = blockIdx.y * gridDim.x + blockIdx.x;
        if (p.clocks && threadIdx.x == 0 && wg < TSVD_GEMV_MAX_GRID) p.clocks[wg * 16 + (STAGE2 ? 8 : 0) + n] = wall_clock64();
    };
    tick(0);

    // (row and swizzle conventions: see tsvd_gemm_kernel)
    const int rsel = i >> 2;
    const int tr_row = 32 * (g & 1) + 16 * (g >> 1) + (rsel >> 1) + 4 * (rsel & 1);
    const int f_lane = swizzle<NBLK>(tr_row);
    int lds_rd[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) lds_rd[b] = tr_row * ROWB + (((wn * TN + b) ^ f_lane) * 32) + (i & 3) * 8;

    int x_voff[SPW];
#pragma unroll
    for (int c = 0; c < SPW; ++c) {
        const int r = (c * NW + wave) * RPS + lane / CPR, pc = lane % CPR;
        const int f = swizzle<NBLK>(r);
        const int lc = (((pc >> 1) ^ f) << 1) | (pc & 1);
        x_voff[c] = (64 * (r >> 5) + (r & 31)) * (int)p.ld * 2 + (b0 + lc * 8) * 2;
    }
    const i32x4 act_rsrc = raw_rsrc(p.act, p.act_bytes);
    const i32x4 w_rsrc = raw_rsrc(p.tiles, p.tile_bytes);
    typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_byte_ptr)smem;
    const uint32_t lds_x = lds_base + wave * 1024;
    // code-word load q of this wavefront: strip min(q * (NW / 2) + (wave >> 1), WSTRIPS - 1), word wave & 1
    const uint32_t lds_w = lds_base + 2 * STAGE_BYTES + (wave & 1) * 256;
    const int w_voff = lane * 16 + (wave & 1) * 4;
    const int w_soff0 = blockIdx.y * WSTRIPS * p.nkt * 1024;

    f32x4 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // The loads of a ring slot (all wavefronts load for all KG pairs), in four parts (part < 0: all
    // of them): a wavefront's load occupies the address unit for many cycles, so inside the loop
    // they are spread over the four MFMA steps of the pair being multiplied.
    auto issue = [&](int sl, int slot, int part) {
        if (sl > lasts) return;                      // nothing left to fetch (uniform)
#pragma unroll
        for (int s = 0; s < KG; ++s) {
            const int pair = KG * sl + s;
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const int stage = 2 * pair + st;
                const int soff = (256 * (stage >> 2) + 128 * ((stage >> 1) & 1) + 32 * (stage & 1)) * (int)p.ld * 2;
#pragma unroll
                for (int c = 0; c < SPW; ++c)
                    if (part < 0 || (((s * 2 + st) * SPW + c) & 3) == part)
                        buf_load128_to_lds(act_rsrc, lds_x + slot * SLOT_BYTES + s * SUB_BYTES + st * STAGE_BYTES + c * NW * 1024,
                                           x_voff[c], soff);
            }
            const int soff_w = w_soff0 + (pair >> 1) * 1024 + (pair & 1) * 8;
#pragma unroll
            for (int q = 0; q < WOPS; ++q)
                if (part < 0 || ((KG * 2 * SPW + s * WOPS + q) & 3) == part) {
                    const int strip = min(q * (NW / 2) + (wave >> 1), WSTRIPS - 1);
                    buf_load32_to_lds(w_rsrc, lds_w + slot * SLOT_BYTES + s * SUB_BYTES + strip * 512, w_voff,
                                      soff_w + strip * p.nkt * 1024);
                }
        }
    };
    auto load_frags = [&](const unsigned char* stage_base, int hh, u32x2 (&lo)[TN], u32x2 (&hi)[TN]) {
        const unsigned char* base = stage_base + hh * 8 * ROWB;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            lo[b] = lds_tr(base + lds_rd[b]);
            hi[b] = lds_tr(base + lds_rd[b] + 2 * ROWB);
        }
    };
    auto mfma_step = [&](const u32x2 (&w)[TM], int word, int hh, const u32x2 (&lo)[TN], const u32x2 (&hi)[TN]) {
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const uint32_t ww = word == 0 ? w[a].x : w[a].y;
            u32x4 av;
            if (hh == 0) av = u32x4{TSVD_DEC(ww, 0), TSVD_DEC(ww, 2), TSVD_DEC(ww, 4), TSVD_DEC(ww, 6)};
            else         av = u32x4{TSVD_DEC(ww, 1), TSVD_DEC(ww, 3), TSVD_DEC(ww, 5), ww & 0xC000C000u};
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] = mfma16<STAGE2>(av, lo[b], hi[b], acc[a][b]);
        }
    };
    // this wavefront's pair of ring slot `slot`, while the loads of slot index next_sl go out
    auto compute_pair = [&](int slot, int next_sl, int next_slot, int steps) {
        const unsigned char* base = smem + slot * SLOT_BYTES + kg * SUB_BYTES;
        if (steps < 4) {            // (uniform over the wavefront; only ever in the last slot, where nothing is left to request)
            u32x2 wl2[TM];
            const uint32_t* wq = reinterpret_cast<const uint32_t*>(base + 2 * STAGE_BYTES) + wm * TM * 128 + lane;
#pragma unroll
            for (int a = 0; a < TM; ++a) wl2[a] = u32x2{wq[a * 128], wq[a * 128 + 64]};
            u32x2 flo[TN], fhi[TN];
            if (steps > 0) { load_frags(base, 0, flo, fhi); mfma_step(wl2, 0, 0, flo, fhi); }
            if (steps > 1) { load_frags(base, 1, flo, fhi); mfma_step(wl2, 0, 1, flo, fhi); }
            if (steps > 2) { load_frags(base + STAGE_BYTES, 0, flo, fhi); mfma_step(wl2, 1, 0, flo, fhi); }
            __builtin_amdgcn_sched_barrier(0);
            return;
        }
        u32x2 w[TM];
        const uint32_t* wl = reinterpret_cast<const uint32_t*>(base + 2 * STAGE_BYTES) + wm * TM * 128 + lane;
#pragma unroll
        for (int a = 0; a < TM; ++a) w[a] = u32x2{wl[a * 128], wl[a * 128 + 64]};
        u32x2 f0lo[TN], f0hi[TN], f1lo[TN], f1hi[TN];
        load_frags(base, 0, f0lo, f0hi);
        load_frags(base, 1, f1lo, f1hi);
        issue(next_sl, next_slot, 0);
        mfma_step(w, 0, 0, f0lo, f0hi);
        __builtin_amdgcn_sched_barrier(0);
        load_frags(base + STAGE_BYTES, 0, f0lo, f0hi);
        issue(next_sl, next_slot, 1);
        mfma_step(w, 0, 1, f1lo, f1hi);
        __builtin_amdgcn_sched_barrier(0);
        load_frags(base + STAGE_BYTES, 1, f1lo, f1hi);
        issue(next_sl, next_slot, 2);
        mfma_step(w, 1, 0, f0lo, f0hi);
        __builtin_amdgcn_sched_barrier(0);
        issue(next_sl, next_slot, 3);
        mfma_step(w, 1, 1, f1lo, f1hi);
        __builtin_amdgcn_sched_barrier(0);
    };

    // FUSEMAX: thread t scans logical chunk t % CPR (8 tokens) of rows t / CPR + c * (THREADS / CPR)
    u32x4 cm = {0u, 0u, 0u, 0u};                      // packed 16-bit magnitudes (order-preserving bit patterns)
    int lds_sc[FUSEMAX ? CPT : 1];
    if constexpr (FUSEMAX) {
        const int ch = threadIdx.x % CPR;
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const int r = threadIdx.x / CPR + c * (THREADS / CPR);
            const int f = swizzle<NBLK>(r);
            lds_sc[c] = r * ROWB + (((ch >> 1) ^ f) * 32) + (ch & 1) * 16;
        }
    }
    auto scan_slot = [&](int slot) {
        if constexpr (FUSEMAX) {
#pragma unroll
            for (int s = 0; s < KG; ++s)
#pragma unroll
                for (int st = 0; st < 2; ++st)
#pragma unroll
                    for (int c = 0; c < CPT; ++c) {
                        u32x4 v = *reinterpret_cast<const u32x4*>(smem + slot * SLOT_BYTES + s * SUB_BYTES + st * STAGE_BYTES + lds_sc[c]);
                        v &= 0x7FFF7FFFu;
                        cm = u32x4{pk_max_u16(cm.x, v.x), pk_max_u16(cm.y, v.y), pk_max_u16(cm.z, v.z), pk_max_u16(cm.w, v.w)};
                    }
        }
    };

    float cmax = 0.f;
    if constexpr (!FUSEMAX)
        if (threadIdx.x < BT) cmax = load_column_max<STAGE2>(p, b0 + threadIdx.x);
#pragma unroll
    for (int j = 0; j < NPB - 1; ++j) issue(j, j, -1);
    tick(1);
    if (NPB - 2 <= lasts) wait_vmcnt<(NPB - 2) * OPS>();   // slot 0 has landed (this wavefront's part)
    else wait_vmcnt<0>();
    if constexpr (!FUSEMAX)
        if (threadIdx.x < BT) publish_column_factor<STAGE2>(p, b0 + threadIdx.x, cmax, cs_lds, threadIdx.x);
    __syncthreads();
    tick(2);

    for (int P = 0; P < nslots; P += NPB) {
#pragma unroll
        for (int j = 0; j < NPB; ++j) {
            if (P + j >= nslots) break;
            compute_pair(j, P + j + NPB - 1, (j + NPB - 1) % NPB, P + j == lasts ? tail_steps : 4);   // loads go into the slot multiplied last time
            scan_slot(j);
            // slot P + j + 1 has landed: all but the loads of the NPB - 2 younger slots are back.  Near
            // the end fewer slots are requested, so everything outstanding is awaited.
            if (P + j + NPB - 1 <= lasts) wait_vmcnt<(NPB - 2) * OPS>();
            else wait_vmcnt<0>();
            __syncthreads();
        }
    }
    wait_vmcnt<0>();                                  // no LDS write may still be in flight
    tick(3);

    if constexpr (FUSEMAX) {
        __syncthreads();                              // every wavefront's loads have landed: the ring is free
        u32x4* red = reinterpret_cast<u32x4*>(smem);  // [THREADS / CPR][CPR]
        red[threadIdx.x] = cm;
        __syncthreads();
        if (threadIdx.x < BT) {
            const uint16_t* r16 = reinterpret_cast<const uint16_t*>(smem) + threadIdx.x;   // chunk t / 8, element t % 8
            uint32_t best = 0;
#pragma unroll 4
            for (int l = 0; l < THREADS / CPR; ++l) best = max(best, (uint32_t)r16[l * CPR * 8]);
            publish_column_factor<false>(p, b0 + threadIdx.x, __uint_as_float(best << 16), cs_lds, threadIdx.x);
        }
        __syncthreads();
    }
    if constexpr (KG > 1) {
        // group 1 hands its accumulators to group 0 through the (now free) ring: [wavefront][block][lane]
        __syncthreads();
        f32x4* xch = reinterpret_cast<f32x4*>(smem) + (size_t)w2 * (TM * TN * 64) + lane;
        if (kg == 1) {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) xch[(a * TN + b) * 64] = acc[a][b];
        }
        __syncthreads();
        if (kg != 0) return;
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] += xch[(a * TN + b) * 64];
    }
    tick(4);

    gemm_epilogue<TM, TN, STAGE2, EX>(p, acc, strip0, b0, wn * TN * 16, cs_lds, i, g);
    tick(5);
}

// ---- token-panel kernel: both stages in one launch, z never leaves the compute unit ----------
// For many tokens and a small factorisation (K <= 1024, code words of U and V a few MB: the MLP of
// a convolutional network) a workgroup of 8 wavefronts owns 64 tokens from x to y:
//   phase 1  the activation panel X[N][64 tokens] is fetched whole into LDS (N <= 1024), then
//            Z[K][64] = fp16(scale * S * (V X)) replaces it (128 KB), with the column maxima of X
//            computed on the way;
//   phase 2  Y[M][64] = (U Z) / scale, in passes of 1024 rows; Z is read from LDS in MFMA operand
//            order, the code words of U go straight to registers, so this phase has no barrier at
//            all: the wavefronts drift apart and one's stores of Y overlap the others' MFMAs.
// No intermediate in HBM, no column-maximum launch, no launch boundary, and one round of
// workgroups (ceil(B / 64) of them) instead of separate rounds per stage.  Arithmetic, operand
// order and rounding are those of the two-launch path.
#define TSVD_PANEL_MAX_KP 1024
#ifndef TSVD_PANEL_SCHED
#define TSVD_PANEL_SCHED 0
#endif
#ifndef TSVD_PANEL_BALANCE
#define TSVD_PANEL_BALANCE 1
#endif
#define TSVD_PANEL_MAX_NP 1024
#define TSVD_PANEL_LDS(NW) (TSVD_PANEL_MAX_KP * 128 + 64 * (NW) * 16 + 2 * 64 * 4 + 64 * (NW) * 4)
#define TSVD_PANEL_LDS_EX(NW) (TSVD_PANEL_LDS(NW) + TSVD_PANEL_BIAS_ROWS * 4)

// NW = 8 wavefronts of 128 rows each (two per SIMD, up to 256 registers) or 16 of 64 rows (four per SIMD).
template <int NW, int EX = 0>
__global__ void __launch_bounds__(64 * NW, NW / 4)
tsvd_panel_kernel(panel_args p) {
    constexpr int TM = 64 / NW, TN = 4, BT = 64, THREADS = 64 * NW;
    constexpr int ROWB = BT * 2, NBLK = BT / 16, CPR = BT / 8, STAGE_BYTES = KT * ROWB, RPS = 64 / CPR;
    static_assert(NW == 8 || NW == 16, "1024 rows of Z per pass");
    static_assert(STAGE_BYTES == 8 * 1024 && KT * CPR == 512, "eight 1-KiB pieces and 512 scan chunks per stage");
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* zl = smem;                                   // X, then Z: stages of [64 rows][64 tokens] 16-bit, swizzled
    unsigned char* ring = smem + TSVD_PANEL_MAX_KP * ROWB;      // reductions and per-token factors
    float* cs1 = reinterpret_cast<float*>(ring + THREADS * 16); // per-token factor of phase 1 (scale / 2) ...
    float* cs2 = cs1 + BT;                                      // ... and of phase 2 (1 / (2 scale))

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int b0 = blockIdx.x * BT;
    auto tick = [&](int n) {
        if (p.clocks && threadIdx.x == 0 && blockIdx.x < TSVD_GEMV_MAX_GRID) p.clocks[blockIdx.x * 16 + n] = wall_clock64();
    };
    tick(0);
    const float* bias_lds = nullptr;           // (visible to all after the barriers of phase 1)
    if constexpr (EX != 0) {
        if (p.bias && p.M <= TSVD_PANEL_BIAS_ROWS) {
            float* dst = reinterpret_cast<float*>(smem + TSVD_PANEL_LDS(NW));
            for (int r = threadIdx.x; r < p.M; r += THREADS) dst[r] = p.bias[r];
            bias_lds = dst;
        }
    }

    // (row and swizzle conventions: see tsvd_gemm_kernel; this tile is one wavefront wide)
    const int rsel = i >> 2;
    const int tr_row = 32 * (g & 1) + 16 * (g >> 1) + (rsel >> 1) + 4 * (rsel & 1);
    const int f_lane = swizzle<NBLK>(tr_row);
    int lds_rd[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) lds_rd[b] = tr_row * ROWB + ((b ^ f_lane) * 32) + (i & 3) * 8;

    f32x4 acc[TM][TN];
    auto clear_acc = [&]() {
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto load_frags = [&](const unsigned char* stage_base, int hh, u32x2 (&lo)[TN], u32x2 (&hi)[TN]) {
        const unsigned char* base = stage_base + hh * 8 * ROWB;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            lo[b] = lds_tr(base + lds_rd[b]);
            hi[b] = lds_tr(base + lds_rd[b] + 2 * ROWB);
        }
    };
#define TSVD_PANEL_INTERLEAVE(DS_READS)                                                  \
    do {                                                                                 \
        if constexpr (TSVD_PANEL_SCHED && STAGE2) {                                      \
            if constexpr ((DS_READS) > 0) __builtin_amdgcn_sched_group_barrier(0x100, (DS_READS), 0); \
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);                           \
            _Pragma("unroll") for (int n_ = 0; n_ < TM * TN; ++n_) {                     \
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       \
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);                       \
            }                                                                            \
        }                                                                                \
    } while (0)
    // the four MFMA steps of a pair of stages whose activations sit at s0 and s1 in LDS
    auto compute_pair = [&](auto stage2, const unsigned char* s0, const unsigned char* s1, const u32x2 (&w)[TM]) {
        constexpr bool STAGE2 = decltype(stage2)::value;
        auto mfma_step = [&](int word, int hh, const u32x2 (&lo)[TN], const u32x2 (&hi)[TN]) {
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const uint32_t ww = word == 0 ? w[a].x : w[a].y;
                u32x4 av;
                if (hh == 0) av = u32x4{TSVD_DEC(ww, 0), TSVD_DEC(ww, 2), TSVD_DEC(ww, 4), TSVD_DEC(ww, 6)};
                else         av = u32x4{TSVD_DEC(ww, 1), TSVD_DEC(ww, 3), TSVD_DEC(ww, 5), ww & 0xC000C000u};
#pragma unroll
                for (int b = 0; b < TN; ++b) acc[a][b] = mfma16<STAGE2>(av, lo[b], hi[b], acc[a][b]);
            }
        };
        if constexpr (NW == 16) {
            // four wavefronts per SIMD hide the LDS latency of one another: one operand set, half the registers
            u32x2 lo[TN], hi[TN];
            load_frags(s0, 0, lo, hi);
            mfma_step(0, 0, lo, hi);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(s0, 1, lo, hi);
            mfma_step(0, 1, lo, hi);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(s1, 0, lo, hi);
            mfma_step(1, 0, lo, hi);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(s1, 1, lo, hi);
            mfma_step(1, 1, lo, hi);
            __builtin_amdgcn_sched_barrier(0);
            return;
        }
        u32x2 f0lo[TN], f0hi[TN], f1lo[TN], f1hi[TN];
        load_frags(s0, 0, f0lo, f0hi);
        load_frags(s0, 1, f1lo, f1hi);
        mfma_step(0, 0, f0lo, f0hi);
        TSVD_PANEL_INTERLEAVE(4 * TN);
        __builtin_amdgcn_sched_barrier(0);
        load_frags(s1, 0, f0lo, f0hi);
        mfma_step(0, 1, f1lo, f1hi);
        TSVD_PANEL_INTERLEAVE(2 * TN);
        __builtin_amdgcn_sched_barrier(0);
        load_frags(s1, 1, f1lo, f1hi);
        mfma_step(1, 0, f0lo, f0hi);
        TSVD_PANEL_INTERLEAVE(2 * TN);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(1, 1, f1lo, f1hi);
        TSVD_PANEL_INTERLEAVE(0);
        __builtin_amdgcn_sched_barrier(0);
    };
    const int w_voff = lane * 16;

    // ================= phase 1: Z = fp16(scale * S * (V X)) into LDS =================
    {
        const int strip0 = wave * TM;                 // this wavefront's rows of Z: 128 wave .. 128 wave + 127
        // piece wave % 8 of the stages wave / 8, wave / 8 + NW / 8, ...: LDS rows piece * RPS + lane / CPR,
        // physical chunk lane % CPR
        const int piece = wave & 7;
        const int r = piece * RPS + lane / CPR, pc = lane % CPR;
        const int lc = (((pc >> 1) ^ swizzle<NBLK>(r)) << 1) | (pc & 1);
        const int x_voff = (64 * (r >> 5) + (r & 31)) * (int)p.ldx * 2 + (b0 + lc * 8) * 2;
        const i32x4 act_rsrc = raw_rsrc(p.x, p.x_bytes);
        const __amdgpu_buffer_rsrc_t w_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.tiles_v), 0, p.tile_v_bytes, 0x00020000);
        typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
        const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_byte_ptr)zl + piece * 1024;
        auto issue_x = [&](int stage, int buf) {
            const int soff = (256 * (stage >> 2) + 128 * ((stage >> 1) & 1) + 32 * (stage & 1)) * (int)p.ldx * 2;
            buf_load128_to_lds(act_rsrc, lds0 + buf * STAGE_BYTES, x_voff, soff);
        };
        auto load_w = [&](int pair, u32x2 (&w)[TM]) {
            const int soff = (strip0 * p.nkt_v + (pair >> 1)) * 1024 + (pair & 1) * 8;
#pragma unroll
            for (int a = 0; a < TM; ++a) w[a] = __builtin_amdgcn_raw_buffer_load_b64(w_rsrc, w_voff, soff + a * p.nkt_v * 1024, 0);
        };
        // The whole activation panel [Np][64 tokens] (at most 128 KB) is fetched into the area that
        // will hold Z afterwards: one wait, one barrier, and the wavefronts run their contraction
        // loops without meeting again until all of them are done with X.
        clear_acc();
        const int npairs = p.npairs_v, lastp = npairs - 1, nst = 2 * npairs;
        u32x2 wa[TM], wb[TM];
        load_w(0, wa);
        for (int st = wave >> 3; st < nst; st += NW / 8) issue_x(st, st);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        tick(1);

        // column maxima -> per-token factors.  Thread t scans logical chunk c % CPR (8 tokens) of LDS row
        // c / CPR, c = t % 512, of the stages t / 512, t / 512 + THREADS / 512, ...; then two levels of
        // reduction (every wavefront reduces 8 of the THREADS / 8 partial rows).
        {
            u32x4 cm = {0u, 0u, 0u, 0u};              // packed 16-bit magnitudes (order-preserving bit patterns)
            const int c = threadIdx.x & 511, sr_ = c / CPR, sch = c % CPR;
            const int lds_sc = sr_ * ROWB + (((sch >> 1) ^ swizzle<NBLK>(sr_)) * 32) + (sch & 1) * 16;
            for (int st = threadIdx.x >> 9; st < nst; st += THREADS / 512) {
                u32x4 v = *reinterpret_cast<const u32x4*>(zl + st * STAGE_BYTES + lds_sc);
                v &= 0x7FFF7FFFu;
                cm = u32x4{pk_max_u16(cm.x, v.x), pk_max_u16(cm.y, v.y), pk_max_u16(cm.z, v.z), pk_max_u16(cm.w, v.w)};
            }
            reinterpret_cast<u32x4*>(ring)[threadIdx.x] = cm;      // [THREADS / 8 partial rows][64 tokens] of 16-bit magnitudes
            __syncthreads();
            const uint16_t* r16 = reinterpret_cast<const uint16_t*>(ring) + wave * 8 * BT + lane;   // rows 8 wave .., token `lane`
            uint32_t part = 0;
#pragma unroll
            for (int l = 0; l < 8; ++l) part = max(part, (uint32_t)r16[l * BT]);
            uint32_t* partials = reinterpret_cast<uint32_t*>(ring + THREADS * 16 + 2 * BT * 4);    // [wavefront][token]
            partials[threadIdx.x] = part;
            __syncthreads();
            if (threadIdx.x < BT) {
                uint32_t best = 0;
#pragma unroll
                for (int l = 0; l < NW; ++l) best = max(best, partials[l * BT + threadIdx.x]);
                const int e = scale_exponent(__uint_as_float(best << 16), p.bound_V);
                cs1[threadIdx.x] = ldexpf(1.0f, e - 1);
                cs2[threadIdx.x] = ldexpf(1.0f, -e - 1);
            }
        }

        for (int P = 0; P < npairs; P += 2) {
            load_w(min(P + 1, lastp), wb);
            compute_pair(std::false_type{}, zl + (2 * P) * STAGE_BYTES, zl + (2 * P + 1) * STAGE_BYTES, wa);
            load_w(min(P + 2, lastp), wa);
            if (P + 1 <= lastp) compute_pair(std::false_type{}, zl + (2 * P + 2) * STAGE_BYTES, zl + (2 * P + 3) * STAGE_BYTES, wb);
        }
        // S of this wavefront's rows
        f32x4 sv[TM];
#pragma unroll
        for (int a = 0; a < TM; ++a) sv[a] = *reinterpret_cast<const f32x4*>(p.S + min((strip0 + a) * 16 + 4 * g, p.Kp - 4));
        __syncthreads();                              // every wavefront is done with X: its area becomes Z (factors are published)
        tick(2);

        // z of this wavefront's rows -> LDS in the stage/row order phase 2 reads: row k sits in stage
        // 4 (k >> 8) + 2 ((k >> 7) & 1) + ((k >> 5) & 1), LDS row 32 ((k >> 6) & 1) + (k & 31).  With
        // k = 16 s + 4 g + v, s = strip0 + a: stage 2 (strip0 >> 3) + ((a >> 1) & 1), row
        // 32 ((s >> 2) & 1) + 16 (a & 1) + 4 g + v, swizzle (g & 1) | (((s ^ (s >> 2)) & 1) << 1), where
        // (s >> 2) & 1 is (a >> 2) & 1 for 8 strips per wavefront and (strip0 >> 2) & 1 for 4:
        // everything but a few per-lane or per-wavefront terms is a compile-time offset.
        const int hi_rt = TM == 8 ? 0 : (strip0 >> 2) & 1;
        float c1[TN];
        int blk[TN];
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            c1[b] = cs1[b * 16 + i];
            blk[b] = (b ^ (g & 1) ^ (hi_rt << 1)) * 32;
        }
        unsigned char* lane_base = zl + (2 * (strip0 >> 3)) * STAGE_BYTES + (32 * hi_rt + 4 * g) * ROWB + i * 2;
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            if ((strip0 + a) * 16 < p.Kp) {                     // (uniform) rows of the padded rank only
                const int hi_ct = TM == 8 ? (a >> 2) & 1 : 0;
                unsigned char* pa = lane_base + ((a >> 1) & 1) * STAGE_BYTES + (32 * hi_ct + 16 * (a & 1)) * ROWB;
                const int fa = ((a ^ (TM == 8 ? a >> 2 : 0)) & 1) << 1;
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        *reinterpret_cast<_Float16*>(pa + v * ROWB + blk[b ^ fa]) = (_Float16)((acc[a][b][v] * sv[a][v]) * c1[b]);
            }
        }
        __syncthreads();
        tick(3);
    }

    // ================= phase 2: Y = (U Z) / scale, 1024 rows per pass, no barriers =================
    {
        const __amdgpu_buffer_rsrc_t w_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.tiles_u), 0, p.tile_u_bytes, 0x00020000);
        float c2[TN];
#pragma unroll
        for (int b = 0; b < TN; ++b) c2[b] = cs2[b * 16 + i];
        const int npairs = p.npairs_u, lastp = npairs - 1;
        // Units of TM strips (64 or 128 rows).  A SIMD always issues from its oldest ready wavefront,
        // so with equal shares the wavefronts of a SIMD (w, w + 4, w + 8, w + 12) finish one after
        // the other and the last runs alone (phase timestamps: 41, 47, 54, 60 us).  The units of a
        // SIMD are therefore split 3 : 2 : 2 : 1 by age (1 : 1 with two wavefronts per SIMD): unit
        // j of SIMD s is rows (4 j + s) * 16 TM .., and age group a takes units [lo, hi).
        const int simd = wave & 3, age = wave >> 2;
        const int per_simd = (p.Mp / (16 * TM) - simd + 3) / 4;
        int lo, hi;
        if (NW == 16 && TSVD_PANEL_BALANCE) {
            const int c1 = (3 * per_simd + 4) / 8, c2 = (5 * per_simd + 4) / 8, c3 = (7 * per_simd + 4) / 8;
            lo = age == 0 ? 0 : age == 1 ? c1 : age == 2 ? c2 : c3;
            hi = age == 0 ? c1 : age == 1 ? c2 : age == 2 ? c3 : per_simd;
        } else {
            lo = age * per_simd / (NW / 4);
            hi = (age + 1) * per_simd / (NW / 4);
        }
        for (int j = lo; j < hi; ++j) {
            const int strip0 = (4 * j + simd) * TM;
            auto load_w = [&](int pair, u32x2 (&w)[TM]) {
                const int soff = (strip0 * p.nkt_u + (pair >> 1)) * 1024 + (pair & 1) * 8;
#pragma unroll
                for (int a = 0; a < TM; ++a) w[a] = __builtin_amdgcn_raw_buffer_load_b64(w_rsrc, w_voff, soff + a * p.nkt_u * 1024, 0);
            };
            clear_acc();
            u32x2 wa[TM], wb[TM];
            load_w(0, wa);
            for (int P = 0; P < npairs; P += 2) {
                load_w(min(P + 1, lastp), wb);
                compute_pair(std::true_type{}, zl + (2 * P) * STAGE_BYTES, zl + (2 * P + 1) * STAGE_BYTES, wa);
                load_w(min(P + 2, lastp), wa);
                if (P + 1 <= lastp) compute_pair(std::true_type{}, zl + (2 * P + 2) * STAGE_BYTES, zl + (2 * P + 3) * STAGE_BYTES, wb);
            }
            float br[TM][4];
            if constexpr (EX != 0) {
                // one uniform choice of the source, then all reads back to back (rows clamped)
                auto fill = [&](auto src) {
#pragma unroll
                    for (int a = 0; a < TM; ++a)
#pragma unroll
                        for (int v = 0; v < 4; ++v) br[a][v] = src(min((strip0 + a) * 16 + 4 * g + v, p.M - 1));
                };
                if (bias_lds) fill([&](int row) { return bias_lds[row]; });
                else if (p.bias) fill([&](int row) { return p.bias[row]; });
                else fill([](int) { return 0.f; });
            }
            if constexpr (EX == 3) {
                const bool vec_ok = !(p.ldy & 3) && !(reinterpret_cast<uintptr_t>(p.y) & 15);
#pragma unroll
                for (int a = 0; a < TM; ++a) {
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        const int col = b0 + b * 16 + i;
                        if (col < p.B)
                            tsvd_store_token_major4(p.y, p.ldy, col, (strip0 + a) * 16 + 4 * g, p.M, acc[a][b][0] * c2[b] + br[a][0],
                                                    acc[a][b][1] * c2[b] + br[a][1], acc[a][b][2] * c2[b] + br[a][2],
                                                    acc[a][b][3] * c2[b] + br[a][3], p.out_bf16, vec_ok);
                    }
                }
            } else if constexpr (EX == 2) {
                const bool aligned4 = !(p.ldy & 1) && !(reinterpret_cast<uintptr_t>(p.y) & 3);
#pragma unroll
                for (int a = 0; a < TM; ++a) {
#pragma unroll
                    for (int vp = 0; vp < 4; vp += 2) {
#pragma unroll
                        for (int b = 0; b < TN; ++b)
                            tsvd_store_row_pair_bf16(p.y, p.ldy, (strip0 + a) * 16 + 4 * g + vp, p.M, b0 + b * 16, i, p.B,
                                                     acc[a][b][vp] * c2[b] + br[a][vp], acc[a][b][vp + 1] * c2[b] + br[a][vp + 1], aligned4);
                    }
                }
            } else if constexpr (EX == 1) {
#pragma unroll
                for (int a = 0; a < TM; ++a) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = (strip0 + a) * 16 + 4 * g + v;
                        if (row < p.M) {
#pragma unroll
                            for (int b = 0; b < TN; ++b) {
                                const int col = b0 + b * 16 + i;
                                if (col < p.B) static_cast<float*>(p.y)[(size_t)row * p.ldy + col] = acc[a][b][v] * c2[b] + br[a][v];
                            }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int a = 0; a < TM; ++a) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = (strip0 + a) * 16 + 4 * g + v;
                        if (row < p.M) {
                            float* dst = static_cast<float*>(p.y) + (size_t)row * p.ldy;
#pragma unroll
                            for (int b = 0; b < TN; ++b) {
                                const int col = b0 + b * 16 + i;
                                if (col < p.B) dst[col] = acc[a][b][v] * c2[b];
                            }
                        }
                    }
                }
            }
        }
    }
    tick(4);
    if (p.clocks && lane == 0 && blockIdx.x < TSVD_GEMV_MAX_GRID)
        p.clocks[blockIdx.x * 16 + 8 + wave / (NW / 8)] = wall_clock64();   // end of (one of) the wavefronts of each eighth
}

template <int WM, int WN, int TM, int TN, bool STAGE2>
hipError_t launch_gemm(const gemm_args& a, bool fast, long long rows, int Bp, hipStream_t stream) {
    constexpr int BT = WN * TN * 16, MT = WM * TM * 16;
    constexpr size_t lds = 2 * KT * BT * 2, cs = BT * 4;      // two stages; the column factors
    // (token tiles that lie wholly beyond the last token are not launched: nothing reads what they would write)
    (void)rows;   // (padded rows, a multiple of MT: the row tiles that hold rows to compute lie inside them)
    const dim3 grid((a.bvalid + BT - 1) / BT, (unsigned)((a.rows_need + MT - 1) / MT)), block(64 * WM * WN);
    if constexpr (STAGE2) {
        const int ex = out_variant(a.bias, a.out_bf16, a.out_token_major);    // the epilogues with bias / bf16 output
        if (ex == 2) {
            if (fast) hipLaunchKernelGGL((tsvd_gemm_pipe_kernel<WM, WN, TM, TN, true, 2>), grid, block, 2 * lds + cs, stream, a);
            else hipLaunchKernelGGL((tsvd_gemm_kernel<WM, WN, TM, TN, true, false, 2>), grid, block, lds + cs, stream, a);
            return hipGetLastError();
        }
        if (ex == 1) {
            if (fast) hipLaunchKernelGGL((tsvd_gemm_pipe_kernel<WM, WN, TM, TN, true, 1>), grid, block, 2 * lds + cs, stream, a);
            else hipLaunchKernelGGL((tsvd_gemm_kernel<WM, WN, TM, TN, true, false, 1>), grid, block, lds + cs, stream, a);
            return hipGetLastError();
        }
        if (ex == 3) {
            if (fast) hipLaunchKernelGGL((tsvd_gemm_pipe_kernel<WM, WN, TM, TN, true, 3>), grid, block, 2 * lds + cs, stream, a);
            else hipLaunchKernelGGL((tsvd_gemm_kernel<WM, WN, TM, TN, true, false, 3>), grid, block, lds + cs, stream, a);
            return hipGetLastError();
        }
    }
    if (fast) hipLaunchKernelGGL((tsvd_gemm_pipe_kernel<WM, WN, TM, TN, STAGE2>), grid, block, 2 * lds + cs, stream, a);
    else hipLaunchKernelGGL((tsvd_gemm_kernel<WM, WN, TM, TN, STAGE2, false>), grid, block, lds + cs, stream, a);
    return hipGetLastError();
}

template <int WM, int WN, int TM, int TN, bool STAGE2>
hipError_t init_gemm() {
    constexpr int BT = WN * TN * 16;
    constexpr int lds = 2 * KT * BT * 2, cs = BT * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_pipe_kernel<WM, WN, TM, TN, STAGE2>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 2 * lds + cs);
    if (e != hipSuccess) return e;
    if constexpr (STAGE2) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_pipe_kernel<WM, WN, TM, TN, true, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * lds + cs);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_pipe_kernel<WM, WN, TM, TN, true, 2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * lds + cs);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_pipe_kernel<WM, WN, TM, TN, true, 3>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * lds + cs);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_kernel<WM, WN, TM, TN, true, false, 3>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds + cs);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_kernel<WM, WN, TM, TN, true, false, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds + cs);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_kernel<WM, WN, TM, TN, true, false, 2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds + cs);
        if (e != hipSuccess) return e;
    }
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_kernel<WM, WN, TM, TN, STAGE2, false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds + cs);
}

template <int WM, int WN, int TM, int TN, int NPB, int KG>
constexpr int ring_lds_bytes() {
    return NPB * KG * (2 * KT * (WN * TN * 16) * 2 + WM * TM * 512) + WN * TN * 16 * 4;
}
template <int WM, int WN, int TM, int TN, bool STAGE2, int NPB, bool FUSEMAX, int KG>
hipError_t launch_ring(const gemm_args& a, long long rows, int Bp, hipStream_t stream) {
    constexpr int BT = WN * TN * 16, MT = WM * TM * 16;
    constexpr size_t lds = ring_lds_bytes<WM, WN, TM, TN, NPB, KG>();
    if (rows % MT) return hipErrorInvalidValue;      // (96-row tiles: the rule asks for them only when they divide the rows)
    const dim3 grid((a.bvalid + BT - 1) / BT, (unsigned)((a.rows_need + MT - 1) / MT)), block(64 * WM * WN * KG);
    if constexpr (STAGE2) {
        const int ex = out_variant(a.bias, a.out_bf16, a.out_token_major);
        if (ex == 2) hipLaunchKernelGGL((tsvd_gemm_ring_kernel<WM, WN, TM, TN, true, NPB, false, KG, 2>), grid, block, lds, stream, a);
        if (ex == 1) hipLaunchKernelGGL((tsvd_gemm_ring_kernel<WM, WN, TM, TN, true, NPB, false, KG, 1>), grid, block, lds, stream, a);
        if (ex == 3) hipLaunchKernelGGL((tsvd_gemm_ring_kernel<WM, WN, TM, TN, true, NPB, false, KG, 3>), grid, block, lds, stream, a);
        if (ex != 0) return hipGetLastError();
    }
    hipLaunchKernelGGL((tsvd_gemm_ring_kernel<WM, WN, TM, TN, STAGE2, NPB, FUSEMAX, KG>), grid, block, lds, stream, a);
    return hipGetLastError();
}
template <int WM, int WN, int TM, int TN, int NPB, int KG>
hipError_t init_ring() {
    constexpr int lds = ring_lds_bytes<WM, WN, TM, TN, NPB, KG>();
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_ring_kernel<WM, WN, TM, TN, true, NPB, false, KG>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_ring_kernel<WM, WN, TM, TN, true, NPB, false, KG, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_ring_kernel<WM, WN, TM, TN, true, NPB, false, KG, 2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_ring_kernel<WM, WN, TM, TN, true, NPB, false, KG, 3>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_ring_kernel<WM, WN, TM, TN, false, NPB, false, KG>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_ring_kernel<WM, WN, TM, TN, false, NPB, true, KG>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

// Tile shapes (rows x tokens of a workgroup tile; wavefronts):
//   0: 256 x 256, 8 wavefronts (one workgroup per compute unit)
//   1: 256 x 128, 4 wavefronts (two workgroups per compute unit, independent barriers)
//   2: 128 x 128, 4 wavefronts
//   3:  64 x 128, 4 wavefronts
// Ring-kernel shapes for launches of few workgroups (ring of 3 or 2 slots, small enough in LDS and
// registers for two to three workgroups per compute unit):
//   14:  64 x 64, 4 wavefronts     15: 128 x 64, 4 wavefronts
//   16:  64 x 64, 8 wavefronts: the contraction split over two groups of four     17: 96 x 64, likewise
// (96 x 64 with rings of three and four slots, one workgroup per compute unit either way: 10.8 and 11.6 us
// against 10.5 us for stage U of a 3072 x 1536 factor at 512 tokens)
#define TSVD_RING_SHAPES(X) X(14, 2, 2, 2, 2, 3, 1) X(15, 2, 2, 4, 2, 3, 1) X(16, 2, 2, 2, 2, 2, 2) X(17, 2, 2, 3, 2, 2, 2)
constexpr bool is_ring(int cfg) { return cfg >= 10; }

template <bool STAGE2, bool FUSEMAX>
hipError_t launch_cfg(int cfg, const gemm_args& a, bool fast, long long rows, int Bp, hipStream_t stream) {
    switch (cfg) {
        case 0: return launch_gemm<2, 4, 8, 4, STAGE2>(a, fast, rows, Bp, stream);
        case 1: return launch_gemm<2, 2, 8, 4, STAGE2>(a, fast, rows, Bp, stream);
        case 2: return launch_gemm<2, 2, 4, 4, STAGE2>(a, fast, rows, Bp, stream);
        case 3: return launch_gemm<2, 2, 2, 4, STAGE2>(a, fast, rows, Bp, stream);
#define TSVD_RING_CASE(id, wm, wn, tm, tn, npb, kg) \
        case id: return launch_ring<wm, wn, tm, tn, STAGE2, npb, FUSEMAX, kg>(a, rows, Bp, stream);
        TSVD_RING_SHAPES(TSVD_RING_CASE)
#undef TSVD_RING_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Tile shape per stage.  Large problems: 256 x 256 (one workgroup per compute unit) or 256 x 128
// (two, with independent barriers), whichever needs less time in rounds of workgroups; the
// second is about 3 % more efficient per unit of work on MI355X.  Small problems (fewer
// workgroups than about 1.5 per compute unit even at 256 x 128): the ring kernel, 128 x 64 tiles
// if they still give every compute unit a workgroup, else 64 x 64 with the contraction split
// over two groups of wavefronts; it needs 16-byte-aligned rows.
int tsvd_gemm_tile_shape(long long rows, long long B, long long cus, bool aligned) {
    // token tiles of 256, 128 and 64 that hold at least one token (the others are not launched)
    const long long c256 = (B + 255) / 256, c128 = (B + 127) / 128, c64 = (B + 63) / 64;
    const long long t0 = (rows / 256) * c256, t1 = (rows / 256) * c128, t2 = (rows / 128) * c128;
    if (2 * t1 >= 3 * cus) {
        const double c0 = (double)((t0 + cus - 1) / cus) / 0.97, c1 = 0.5 * (double)((t1 + cus - 1) / cus);
        return c0 < c1 ? 0 : 1;
    }
    if (!aligned) return t2 >= cus ? 2 : 3;
    if ((rows / 128) * c64 >= cus) return 15;
    // 96 x 64 tiles when they give (nearly) every compute unit exactly one workgroup where 64 x 64
    // tiles would give half of them two
    const long long t96 = (rows / 96) * c64;
    if (rows % 96 == 0 && t96 <= cus && 4 * t96 > 3 * cus && (rows / 64) * c64 > cus) return 17;
    return 16;
}

// Token-major x in place: the token-panel launch on fp4 x fp6, and the fp4 x fp6 stage V that needs no column maxima
// (TSVD_TOKEN_MAJOR_COPY = 1: always copy first).
bool tsvd_gemm_reads_token_major(long long Mp, long long Kp, long long Np, long long B, long long cus) {
    if (tsvd_tune("TSVD_TOKEN_MAJOR_COPY", 0) != 0) return false;
    if (tsvd_stage_mask() == 7 && tsvd_gemm_use_panel(Mp, Kp, Np, B, cus, true)) return tsvd_gemm_panel_fp6();
    return tsvd_gemm_use_fp6_v(Mp, Kp, Np, B, cus, true) && tsvd_fp6_direct_possible(Kp, B, cus);
}

// The token-panel kernel serves 16-byte-aligned activations, K <= 1024, N <= 1024, code words of both factors
// small enough to stay in every L2 (each workgroup reads all of them), and a token count whose
// 64-token panels fill at least 60 % of the compute units of their last round.
bool tsvd_gemm_use_panel(long long Mp, long long Kp, long long Np, long long B, long long cus, bool aligned) {
    const int mode = tsvd_tune("TSVD_PANEL", -1);       // 0 never, 1 whenever the shape allows, default: by rule
    if (!aligned || Kp > TSVD_PANEL_MAX_KP || Np > TSVD_PANEL_MAX_NP || mode == 0) return false;
    if (mode == 1) return true;
    const long long n = (B + 63) / 64, rounds = (n + cus - 1) / cus;
    return (Mp + Np) * Kp / 4 <= (8ll << 20) && 10 * n >= 6 * rounds * cus;
}

hipError_t tsvd_gemm_init() {
    hipError_t e;
    if ((e = tsvd_fp6_init()) != hipSuccess) return e;
    if ((e = init_gemm<2, 4, 8, 4, false>()) != hipSuccess) return e;
    if ((e = init_gemm<2, 4, 8, 4, true>()) != hipSuccess) return e;
    if ((e = init_gemm<2, 2, 8, 4, false>()) != hipSuccess) return e;
    if ((e = init_gemm<2, 2, 8, 4, true>()) != hipSuccess) return e;
    if ((e = init_gemm<2, 2, 4, 4, false>()) != hipSuccess) return e;
    if ((e = init_gemm<2, 2, 4, 4, true>()) != hipSuccess) return e;
    if ((e = init_gemm<2, 2, 2, 4, false>()) != hipSuccess) return e;
    if ((e = init_gemm<2, 2, 2, 4, true>()) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<8>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS(8))) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<16>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS(16))) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<8, 1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS_EX(8))) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<16, 1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS_EX(16))) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<8, 2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS_EX(8))) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<16, 2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS_EX(16))) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<8, 3>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS_EX(8))) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_kernel<16, 3>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL_LDS_EX(16))) != hipSuccess) return e;
#define TSVD_RING_INIT(id, wm, wn, tm, tn, npb, kg) \
    if ((e = init_ring<wm, wn, tm, tn, npb, kg>()) != hipSuccess) return e;
    TSVD_RING_SHAPES(TSVD_RING_INIT)
#undef TSVD_RING_INIT
    return hipSuccess;
}

hipError_t tsvd_forward_gemm(const tsvd_gemm_problem& g, hipStream_t stream) {
    const tsvd_blob_header& hd = *g.hd;
    const int Bp = (int)tsvd_round_up(g.B, 256);
    float* colpart = static_cast<float*>(g.ws);
    const size_t part_bytes = (((size_t)(TSVD_COLMAX_PARTS + 1) * Bp * 4) + 255) & ~(size_t)255;
    _Float16* Z = reinterpret_cast<_Float16*>(static_cast<uint8_t*>(g.ws) + part_bytes);

    // buffer loads address with 32-bit byte offsets
    if ((!g.x_f32 && (size_t)(g.x_token_major ? g.B : hd.N) * g.ldx * 2 >= (1ull << 31)) || (size_t)hd.Kp * Bp * 2 >= (1ull << 31) ||
        (size_t)hd.Mp * hd.Kp / 4 >= (1ull << 31) || (size_t)hd.Kp * hd.Np / 4 >= (1ull << 31))
        return hipErrorNotSupported;         // (reported as TSVD_EUNSUPPORTED; the limits are documented in tsvd.h)
    gemm_args a1;
    a1.tiles = reinterpret_cast<const uint32_t*>(g.blob + hd.off_V);
    a1.nkt = (int)(hd.Np / 256);
    a1.act = static_cast<const uint16_t*>(g.x);
    a1.ld = g.ldx;
    a1.kvalid = (int)hd.N;
    a1.bvalid = (int)g.B;
    // (token-major x is read in place by the fp4 x fp6 kernels only, which need no alignment: the rules see it as aligned)
    const bool fast1 = g.x_token_major || ((g.ldx % 8 == 0) && ((reinterpret_cast<uintptr_t>(g.x) & 15u) == 0));
    a1.act_bytes = (unsigned)((size_t)(g.x_token_major ? g.B : hd.N) * g.ldx * 2);
    a1.tile_bytes = (unsigned)((size_t)hd.Kp * hd.Np / 4);
    a1.S = reinterpret_cast<const float*>(g.blob + hd.off_S);
    a1.colpart = colpart;
    a1.colmax = colpart + (size_t)TSVD_COLMAX_PARTS * Bp;
    a1.Bp = Bp;
    a1.bound_V = g.bound_V;
    a1.out = Z;
    a1.ld_out = Bp;
    a1.bias = nullptr;
    a1.out_bf16 = 0;
    a1.rows_valid = (int)hd.Kp;
    a1.clocks = g.clocks;
    a1.big_tiles = 0;
    a1.plane_blocks = 0;
    a1.code_blocks = 0;
    a1.two_sets = 0;
    // contraction lengths: stage V runs over N, stage U over K, both in steps of 128 indices; the last step of K is
    // filled from its first sub-steps (tsvd_rank_position), so stage U stops after those
    const int pairs_n = (int)((hd.N + 127) / 128), pairs_k = (int)((hd.K + 127) / 128);
    a1.npairs = pairs_n;
    a1.last_steps = 4;
    a1.rows_need = 128 * pairs_k;              // every rank position that stage U reads is written (zeros beyond K)

    gemm_args a2 = a1;
    a2.tiles = reinterpret_cast<const uint32_t*>(g.blob + hd.off_U);
    a2.nkt = (int)(hd.Kp / 256);
    a2.act = reinterpret_cast<const uint16_t*>(Z);
    a2.ld = Bp;
    a2.kvalid = (int)hd.Kp;
    a2.bvalid = (int)g.B;
    a2.act_bytes = (unsigned)((size_t)hd.Kp * Bp * 2);
    a2.tile_bytes = (unsigned)((size_t)hd.Mp * hd.Kp / 4);
    a2.S = nullptr;
    a2.out = g.y;
    a2.ld_out = g.ldy;
    a2.bias = g.bias;
    a2.out_bf16 = g.out_bf16;
    a2.out_token_major = g.y_token_major;
    a2.rows_valid = (int)hd.M;
    a2.rows_need = (int)hd.M;
    a2.npairs = pairs_k;
    a2.last_steps = hd.K % 128 == 0 ? 4 : (int)((hd.K % 128 + 31) / 32);

    if (g.x_f32) {
        // fp32 activations: six planes of x (three, and three more for what those leave), both stages on fp4 codes x fp6
        // planes with the second set of planes as further blocks of the contraction (same code words again), stage V
        // writing six planes of z from its fp32 accumulators.  Workspace: planes of x, then planes of z.
        const size_t xp_bytes = tsvd_gemm_fp6_bytes(256ll * pairs_n, Bp), zp_bytes = tsvd_gemm_fp6_bytes(256ll * pairs_k, Bp);
        if (xp_bytes >= (1ull << 31) || zp_bytes >= (1ull << 31)) return hipErrorNotSupported;
        unsigned char* xplanes = static_cast<unsigned char*>(g.ws);
        unsigned char* zplanes = xplanes + ((xp_bytes + 255) & ~(size_t)255);
        const int mask = tsvd_stage_mask();
        hipError_t e = hipSuccess;
        if (mask & 1)
            if ((e = tsvd_fp6_launch_planes_f32(static_cast<const float*>(g.x), g.ldx, (int)hd.N, (int)g.B, pairs_n, xplanes, stream)) != hipSuccess) return e;
        if (mask & 2) {
            gemm_args a4 = a1;
            a4.act = reinterpret_cast<const uint16_t*>(xplanes);
            a4.act_bytes = (unsigned)xp_bytes;
            a4.npairs = 2 * pairs_n;
            a4.code_blocks = pairs_n;
            a4.plane_blocks = 2 * pairs_n;
            a4.out = zplanes;
            a4.ld_out = 2 * pairs_k;
            a4.two_sets = pairs_k;
            a4.colmax = nullptr;
            if ((e = tsvd_fp6_launch_direct(a4, hd.Kp, g.cu_count, stream)) != hipSuccess) return e;
        }
        if (mask & 4) {
            gemm_args a3 = a2;
            a3.act = reinterpret_cast<const uint16_t*>(zplanes);
            a3.act_bytes = (unsigned)zp_bytes;
            a3.npairs = 2 * pairs_k;
            a3.code_blocks = pairs_k;
            a3.plane_blocks = 2 * pairs_k;
            a3.colmax = nullptr;
            e = tsvd_fp6_launch(true, a3, hd.Mp, Bp, out_variant(a3.bias, a3.out_bf16, a3.out_token_major), g.cu_count, stream);
        }
        return e;
    }
    if (tsvd_stage_mask() == 7 && tsvd_gemm_use_panel(hd.Mp, hd.Kp, hd.Np, g.B, g.cu_count, fast1)) {
        panel_args pa;
        pa.tiles_v = a1.tiles;
        pa.tiles_u = a2.tiles;
        pa.tile_v_bytes = a1.tile_bytes;
        pa.tile_u_bytes = a2.tile_bytes;
        pa.nkt_v = a1.nkt;
        pa.nkt_u = a2.nkt;
        pa.npairs_v = a1.npairs;
        pa.npairs_u = a2.npairs;
        pa.x = a1.act;
        pa.ldx = g.ldx;
        pa.x_bytes = a1.act_bytes;
        pa.N = (int)hd.N;
        pa.x_token_major = g.x_token_major;
        pa.S = a1.S;
        pa.bound_V = g.bound_V;
        pa.Kp = (int)hd.Kp;
        pa.Mp = (int)hd.Mp;
        pa.M = (int)hd.M;
        pa.B = (int)g.B;
        pa.y = g.y;
        pa.ldy = g.ldy;
        pa.bias = g.bias;
        pa.out_bf16 = g.out_bf16;
        pa.out_token_major = g.y_token_major;
        pa.clocks = g.clocks;
        const dim3 pgrid((unsigned)((g.B + 63) / 64));
        const int ex = out_variant(g.bias, g.out_bf16, g.y_token_major);
        if (tsvd_gemm_panel_fp6()) {                   // fp4 codes x fp6 planes (TSVD_PANEL_FP6 = 0: the 16-bit panel kernel)
            return tsvd_fp6_launch_panel(pa, ex, stream);
        } else if (g.x_token_major) {
            return hipErrorInvalidValue;               // (tsvd_gemm_reads_token_major said no)
        } else if (env_cfg("TSVD_PANEL_WAVES", 16) == 16) {   // tuning switch: 16 is about 5 % faster on MI355X
            if (ex == 3) hipLaunchKernelGGL((tsvd_panel_kernel<16, 3>), pgrid, dim3(1024), TSVD_PANEL_LDS_EX(16), stream, pa);
            else if (ex == 2) hipLaunchKernelGGL((tsvd_panel_kernel<16, 2>), pgrid, dim3(1024), TSVD_PANEL_LDS_EX(16), stream, pa);
            else if (ex == 1) hipLaunchKernelGGL((tsvd_panel_kernel<16, 1>), pgrid, dim3(1024), TSVD_PANEL_LDS_EX(16), stream, pa);
            else hipLaunchKernelGGL((tsvd_panel_kernel<16>), pgrid, dim3(1024), TSVD_PANEL_LDS(16), stream, pa);
        } else {
            if (ex == 3) hipLaunchKernelGGL((tsvd_panel_kernel<8, 3>), pgrid, dim3(512), TSVD_PANEL_LDS_EX(8), stream, pa);
            else if (ex == 2) hipLaunchKernelGGL((tsvd_panel_kernel<8, 2>), pgrid, dim3(512), TSVD_PANEL_LDS_EX(8), stream, pa);
            else if (ex == 1) hipLaunchKernelGGL((tsvd_panel_kernel<8, 1>), pgrid, dim3(512), TSVD_PANEL_LDS_EX(8), stream, pa);
            else hipLaunchKernelGGL((tsvd_panel_kernel<8>), pgrid, dim3(512), TSVD_PANEL_LDS(8), stream, pa);
        }
        return hipGetLastError();
    }
    int cfg1 = env_cfg("TSVD_GEMM_CFG_V", tsvd_gemm_tile_shape(hd.Kp, g.B, g.cu_count, fast1));
    int cfg2 = env_cfg("TSVD_GEMM_CFG_U", tsvd_gemm_tile_shape(hd.Mp, g.B, g.cu_count, true));
    if (is_ring(cfg1) && !fast1) cfg1 = 3;
    const bool fp6_v = tsvd_gemm_use_fp6_v(hd.Mp, hd.Kp, hd.Np, g.B, g.cu_count, fast1);   // stage V on planes of x
    // ... writing the planes of z itself where its tile allows: no fp16 z, no column maxima, no separate pass over z
    const bool direct = fp6_v && tsvd_fp6_direct_possible(hd.Kp, g.B, g.cu_count);
    const bool fuse = is_ring(cfg1) && env_cfg("TSVD_FUSEMAX", 1) != 0 && !fp6_v;
    if (g.x_token_major && !direct) return hipErrorInvalidValue;   // (tsvd_gemm_reads_token_major said no)

    // Profiling switch: TSVD_STAGE_MASK selects the kernels to launch (1 column maxima,
    // 2 stage V, 4 stage U; default all).  Skipped kernels leave the workspace as it is.
    const int mask = tsvd_stage_mask();
    hipError_t e = hipSuccess;
    if ((mask & 1) && !fuse && !direct) {
        if (fast1 && env_cfg("TSVD_COLMAX_SCALAR", 0) == 0)
            hipLaunchKernelGGL(tsvd_colmax_vec_kernel, dim3((unsigned)((g.B + 127) / 128), TSVD_COLMAX_PARTS), dim3(256),
                               0, stream, static_cast<const uint16_t*>(g.x), g.ldx, (int)hd.N, (int)g.B, Bp, colpart);
        else
            hipLaunchKernelGGL(tsvd_colmax_kernel, dim3((unsigned)((g.B + 127) / 128), TSVD_COLMAX_PARTS), dim3(256), 0,
                               stream, static_cast<const uint16_t*>(g.x), g.ldx, (int)hd.N, (int)g.B, Bp, colpart);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // stage V on fp4 x fp6 as well when its own contraction (N) is long: X -> planes (after Z's planes in the workspace)
    if ((mask & 2) && fp6_v) {
        unsigned char* xplanes = reinterpret_cast<unsigned char*>(Z) + (((size_t)hd.Kp * Bp * 2 + 255) & ~(size_t)255) +
                                 ((tsvd_gemm_fp6_bytes(hd.Kp, Bp) + 255) & ~(size_t)255);
        if ((e = tsvd_fp6_launch_planes(true, static_cast<const uint16_t*>(g.x), (long long)g.ldx, (int)hd.N, (int)g.B, (int)(hd.Np / 128),
                                        a1.npairs, g.B, xplanes, stream, g.x_token_major != 0)) != hipSuccess) return e;
        gemm_args a4 = a1;
        a4.act = reinterpret_cast<const uint16_t*>(xplanes);
        a4.act_bytes = (unsigned)tsvd_gemm_fp6_bytes(hd.Np, Bp);
        if (direct) {
            a4.out = reinterpret_cast<unsigned char*>(Z) + (((size_t)hd.Kp * Bp * 2 + 255) & ~(size_t)255);   // the planes of z
            a4.ld_out = hd.Kp / 128;                                                                       // blocks per token group
            a4.colmax = nullptr;
            e = tsvd_fp6_launch_direct(a4, hd.Kp, g.cu_count, stream);
        } else {
            e = tsvd_fp6_launch(false, a4, hd.Kp, Bp, 0, g.cu_count, stream);
        }
    } else if (mask & 2) e = fuse ? launch_cfg<false, true>(cfg1, a1, fast1, hd.Kp, Bp, stream)
                           : launch_cfg<false, false>(cfg1, a1, fast1, hd.Kp, Bp, stream);
    if (e != hipSuccess) return e;
    if ((mask & 4) && tsvd_gemm_use_fp6(hd.Mp, hd.Kp, hd.Np, g.B, g.cu_count, fast1)) {
        // Z (fp16) -> three fp6 planes in operand order, then stage U on fp4 x fp6
        unsigned char* planes = reinterpret_cast<unsigned char*>(Z) + (((size_t)hd.Kp * Bp * 2 + 255) & ~(size_t)255);
        if (!direct) {
            if ((e = tsvd_fp6_launch_planes(false, reinterpret_cast<const uint16_t*>(Z), (long long)Bp, (int)hd.Kp, Bp, (int)(hd.Kp / 128),
                                            a2.npairs, g.B, planes, stream)) != hipSuccess) return e;
        }
        gemm_args a3 = a2;
        if (direct) a3.colmax = nullptr;               // (no per-token factors: z came scaled and as planes)
        a3.act = reinterpret_cast<const uint16_t*>(planes);
        a3.act_bytes = (unsigned)tsvd_gemm_fp6_bytes(hd.Kp, Bp);
        return tsvd_fp6_launch(true, a3, hd.Mp, Bp, out_variant(a3.bias, a3.out_bf16, a3.out_token_major), g.cu_count, stream);
    }
    if (mask & 4) e = launch_cfg<true, false>(cfg2, a2, true, hd.Mp, Bp, stream);
    return e;
}
