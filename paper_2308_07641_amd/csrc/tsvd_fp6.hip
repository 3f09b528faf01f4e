// Batched kernels on fp4 codes x three fp6 (E2M3) planes of the activations (v_mfma_scale_f32_16x16x128_f8f6f4):
// the operand pass that makes the planes, the two-launch kernel for long contractions with many tiles, the
// token-panel kernel that does both stages in one launch, their launch rules and launchers.  tsvd_forward_gemm
// (tsvd_gemm.hip) decides which of them a call takes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <type_traits>

#include "tsvd_gemm_common.h"

namespace {

// ---- stage U on fp4 codes x three fp6 planes of Z (large shapes) -------------------------------
// v_mfma_scale_f32_16x16x128_f8f6f4 with an fp4 A operand and an fp6 (E2M3) B operand issues at the
// rate of v_mfma_f32_16x16x32_f16 and contracts four times as many indices; the codes become fp4
// with 6 operations per 16 rows x 128 indices (against 32 for the 16-bit form).  Z is given as three
// planes (a value, the residual of its rounding, the residual of that), each with its own
// power-of-two scale per lane and block of 32 indices, which is the block-scale operand of the
// instruction: byte `plane` of the scale register of the lane that holds the block.  Three planes
// resolve about 2^-13 of a block's largest magnitude.  A separate pass (tsvd_z_planes_kernel) turns
// the fp16 Z of stage V into planes in the operand order of this kernel, so the loads into LDS
// are plain copies and the operand reads plain 16- and 8-byte reads.
// Status: same accuracy as the 16-bit path and 10 - 25 % faster per call on long contractions with
// many tiles, where it is used for both stages (tsvd_gemm_use_fp6, tsvd_gemm_use_fp6_v; TSVD_FP6 and
// TSVD_FP6_V = 0 / 1 force it off / on).
// Measured on MI355X, 36864 x 18432 weights, 2048 tokens: this kernel 1.50 ms + 0.03 ms for the
// planes against 1.78 ms for the 16-bit stage U; its MFMAs alone would take 0.87 ms at 2.4 GHz.  The
// counters show the matrix pipes busy 80 % of the compute units' busy cycles, 16 cycles per MFMA,
// and a sustained clock of 1.82 GHz under this load (2.08 GHz under the 16-bit kernel): what is left
// to gain in software is the last fifth of the pipe's cycles, the rest of the gap to the nominal
// peak is the clock.  Timing probes with every load redirected to two cached blocks (1.50 ms) and
// with no operand read ahead (1.53 ms) moved little: neither the L2 nor LDS latency bounds it.
// Tried and dropped: a ring of three blocks with every load under explicit wait counts in a
// 256 x 128 tile of eight wavefronts (1.78 - 1.83 ms, a barrier for every 0.35 us of MFMAs per
// wavefront); a 512 x 128 tile with 256 indices per barrier (register spills, 2.0 ms); a raised wavefront
// priority (s_setprio 1 or 2) during the MFMA steps of a block (1.51 against 1.49 - 1.50 ms).
//
// Record of one (16-token tile, 128-index block): planes' first 16 bytes per lane [3][64][16], last
// 8 bytes per lane [3][64][8], scale words [64][4] = 4864 bytes; lane (i, g) holds, for token i of
// the tile, the indices that meet elements 0..31 of lane group g of the A operand built from the
// tile format (tsvd_step_column).  Records are stored [128-token group][block][tile in group].
#define FP6_REC_BYTES 4864
#ifndef FP6_LDS_DEPTH
#define FP6_LDS_DEPTH 2                            // operand reads ahead of the MFMAs, in steps of eight MFMAs
#endif
#define FP6_PAIR_BYTES (8 * FP6_REC_BYTES)      // one block of one 128-token group: 38 KiB exactly
typedef int i32x8 __attribute__((ext_vector_type(8)));

// One lane's 32 values -> three E2M3 planes (the value, the residual of its rounding, the residual of that), each
// with its own power-of-two scale.  put(plane, first 16 bytes, last 8 bytes) receives the lane's 24 bytes of each
// plane; the return value holds the three scale bytes.  KEEP: v is left holding what the three planes do not resolve
// (for a second set of planes); else it is used up.
template <bool KEEP = false, typename Put>
__device__ __forceinline__ uint32_t tsvd_planes_of_32(float (&v)[32], Put put) {
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    typedef float f32x32 __attribute__((ext_vector_type(32)));
    typedef unsigned u32x6 __attribute__((ext_vector_type(6)));
    uint32_t scales = 0;
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
        float m = 0.f;
#pragma unroll
        for (int e = 0; e < 32; ++e) m = fmaxf(m, fabsf(v[e]));
        // exponent ex with m 2^-ex <= 7.5, the largest E2M3 magnitude (m = f 2^x, 0.5 <= f < 1)
        int x = 0;
        const float f = frexpf(m, &x);
        int ex = m > 0.f ? (f <= 0.9375f ? x - 3 : x - 2) : 0;
        ex = max(-126, min(126, ex));
        scales |= (uint32_t)(127 + ex) << (8 * pl);
        const float unit = ldexpf(1.0f, ex);
        // v_cvt_scalef32_2xpk16_fp6_f32: element 2 j of the result is src0[j] / scale, element 2 j + 1 is
        // src1[j] / scale, rounded to nearest even on the E2M3 grid (saturating); the reverse conversion
        // returns the elements in the same order, times the scale (measured on gfx950)
        f32x16 s0, s1;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            s0[j] = v[2 * j];
            s1[j] = v[2 * j + 1];
        }
        // The conversions take several passes over their registers, and the register allocator lets the result of the
        // builtins share registers with operands that die at the instruction.  Measured on gfx950: a result tuple that
        // started in the scale's register left elements 2..31 converted with a wrong scale.  Hence the instructions are
        // written out with results that may not overlap any operand.
        u32x6 w;
        asm("v_cvt_scalef32_2xpk16_fp6_f32 %0, %1, %2, %3" : "=&v"(w) : "v"(s0), "v"(s1), "v"(unit));
        if (pl < 2 || KEEP) {
            f32x32 back;
            asm("v_cvt_scalef32_pk32_f32_fp6 %0, %1, %2" : "=&v"(back) : "v"(w), "v"(unit));
#pragma unroll
            for (int e = 0; e < 32; ++e) v[e] -= back[e];         // exact: the next plane codes this residual
        }
        put(pl, u32x4{w[0], w[1], w[2], w[3]}, u32x2{w[4], w[5]});
    }
    return scales;
}
// ... written to the lane's places in the record at `rec`
template <bool KEEP = false>
__device__ __forceinline__ void tsvd_planes_of_32(float (&v)[32], unsigned char* rec, int lane) {
    const uint32_t scales = tsvd_planes_of_32<KEEP>(v, [&](int pl, u32x4 lo, u32x2 hi) {
        *reinterpret_cast<u32x4*>(rec + pl * 1024 + lane * 16) = lo;
        *reinterpret_cast<u32x2*>(rec + 3072 + pl * 512 + lane * 8) = hi;
    });
    *reinterpret_cast<uint32_t*>(rec + 4608 + lane * 4) = scales;
}
// Six planes for fp32 values: a record of three, and a second record for what those leave (2^-14.7 of a block's largest
// magnitude times 2^-14.7 again: below the last bit of an fp32 value of that magnitude).
__device__ __forceinline__ void tsvd_planes_of_32_twice(float (&v)[32], unsigned char* rec, unsigned char* rec2, int lane) {
    tsvd_planes_of_32<true>(v, rec, lane);
    tsvd_planes_of_32<false>(v, rec2, lane);
}

// The 32 values of one operand lane from bf16 activations stored one row per token (token-major, row pitch ld
// elements): indices k0 + 32 (e >> 4) + (e & 15), two runs of 16 consecutive elements.  vec: rows and base are 16-byte
// aligned (four 16-byte loads), else 32 two-byte loads.  The buffer's range check gives zero beyond the last token's
// row; indices beyond kvalid and tokens beyond the batch are zeroed here.
__device__ __forceinline__ void tsvd_gather_token_major(__amdgpu_buffer_rsrc_t x_rsrc, int ld2, int tok, int k0, int kvalid, bool tok_ok,
                                                        bool vec, float (&v)[32]) {
    const int voff = tok * ld2;
    if (vec) {
        u32x4 q[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) q[h] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, voff, (k0 + 32 * (h >> 1) + 8 * (h & 1)) * 2, 0);
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const uint32_t w = q[2 * (e >> 4) + ((e >> 3) & 1)][(e & 7) >> 1];
            v[e] = __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
        }
    } else {
#pragma unroll
        for (int e = 0; e < 32; ++e)
            v[e] = __uint_as_float((uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(x_rsrc, voff, (k0 + 32 * (e >> 4) + (e & 15)) * 2, 0) << 16);
    }
#pragma unroll
    for (int e = 0; e < 32; ++e)
        if (!tok_ok || k0 + 32 * (e >> 4) + (e & 15) >= kvalid) v[e] = 0.f;
}

// The operand pass for fp32 activations x [rows_valid][ld] (feature-major, any row pitch): two records per (16-token
// tile, 128-index block), the second `set_offset` blocks behind the first in a layout of `nblocks` blocks per token
// group.  A lane gathers its 32 values itself (rows beyond the matrix and tokens beyond the batch read as zero).
__global__ void __launch_bounds__(512)
tsvd_x_planes_f32_kernel(const float* __restrict__ x, long long ld, int rows_valid, int cols_valid, int nblocks, int set_offset,
                         unsigned char* __restrict__ planes) {
    const int tt = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
    const int tok = blockIdx.x * 128 + tt * 16 + i, k0 = blockIdx.y * 128 + 64 * (g & 1) + 16 * (g >> 1);
    float v[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const int k = k0 + 32 * (e >> 4) + (e & 15);
        const float q = x[(size_t)min(k, rows_valid - 1) * ld + min(tok, cols_valid - 1)];
        v[e] = k < rows_valid && tok < cols_valid ? q : 0.f;
    }
    unsigned char* rec = planes + ((size_t)(blockIdx.x * nblocks + blockIdx.y) * 8 + tt) * FP6_REC_BYTES;
    tsvd_planes_of_32_twice(v, rec, rec + (size_t)set_offset * 8 * FP6_REC_BYTES, lane);
}

// The operand pass for token-major bf16 activations x [cols_valid tokens][ld]: no transposition through LDS, a lane's
// values are contiguous in memory.  Same grid and records as tsvd_z_planes_kernel.
__global__ void __launch_bounds__(512)
tsvd_x_planes_token_major_kernel(const uint16_t* __restrict__ x, long long ld, unsigned x_bytes, int rows_valid, int cols_valid, int nblocks,
                                 int vec, unsigned char* __restrict__ planes) {
    const int tt = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(x), 0, x_bytes, 0x00020000);
    const int tok = blockIdx.x * 128 + tt * 16 + i;
    float v[32];
    tsvd_gather_token_major(x_rsrc, (int)ld * 2, tok, blockIdx.y * 128 + 64 * (g & 1) + 16 * (g >> 1), rows_valid, tok < cols_valid, vec != 0, v);
    tsvd_planes_of_32(v, planes + ((size_t)(blockIdx.x * nblocks + blockIdx.y) * 8 + tt) * FP6_REC_BYTES, lane);
}

// grid (Bp / 128, Kp / 128), block 512 = 8 tiles x 64 lanes.  The [128 indices][128 tokens] block of Z
// is read row by row (256 contiguous bytes each) into LDS, from where every thread picks the 32
// values of its lane of the operand (row pitch 129 words: the picks of a wavefront, 16 tokens x 4
// different rows, fall on different banks).
template <bool BF16>
__global__ void __launch_bounds__(512)
tsvd_z_planes_kernel(const uint16_t* __restrict__ Z, long long ld, int rows_valid, int cols_valid, int nblocks,
                     unsigned char* __restrict__ planes) {
    __shared__ uint32_t zt[128 * 65];                 // [index][token pair], pitch 65 words
    const int tt = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
    {
        // (ld is even and the matrix 4-byte aligned; rows and columns beyond the matrix read as zero:
        // clamped addresses, masked afterwards)
        const uint32_t* src = reinterpret_cast<const uint32_t*>(Z);
        uint32_t r[16];
#pragma unroll
        for (int n = 0; n < 16; ++n) {                // 128 rows x 64 words = 8192 words, 16 per thread
            const int idx = n * 512 + threadIdx.x, row = blockIdx.y * 128 + (idx >> 6), col = blockIdx.x * 128 + 2 * (idx & 63);
            uint32_t v = src[((size_t)min(row, rows_valid - 1) * ld + min(col, cols_valid - 1)) / 2];
            if (col + 1 >= cols_valid) v &= 0xFFFFu;
            r[n] = row < rows_valid && col < cols_valid ? v : 0u;
        }
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            const int idx = n * 512 + threadIdx.x;
            zt[(idx >> 6) * 65 + (idx & 63)] = r[n];
        }
    }
    __syncthreads();
    const int tok = tt * 16 + i;                      // token within the block's 128
    const int k0 = 64 * (g & 1) + 16 * (g >> 1);
    float v[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const uint32_t w = zt[(k0 + 32 * (e >> 4) + (e & 15)) * 65 + (tok >> 1)];
        const uint16_t h = (tok & 1) ? (uint16_t)(w >> 16) : (uint16_t)(w & 0xFFFFu);
        v[e] = BF16 ? __uint_as_float((uint32_t)h << 16) : (float)__builtin_bit_cast(_Float16, h);
    }
    tsvd_planes_of_32(v, planes + ((size_t)(blockIdx.x * nblocks + blockIdx.y) * 8 + tt) * FP6_REC_BYTES, lane);
}

template <int PL>
__device__ __forceinline__ f32x4 mfma_fp6(const u32x4& a, const u32x4& lo, const u32x2& hi, uint32_t scale, f32x4 acc) {
    const i32x8 av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
    const i32x8 bv = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
    // cbsz = 4: A is fp4 (E2M1); blgp = 2: B is fp6 (E2M3); A scale 2^0; B scale = byte PL of `scale`
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc, 4, 2, 0, 0x7F7F7F7F, PL, (int)scale);
}

// WM x WN = 2 x 2 wavefronts (256 rows x 128 tokens per workgroup) or 4 x 1 (512 x 64) of TM x 4 = 8 x 4 blocks
// each, two workgroups per compute unit, or 4 x 1 of 4 x 4 blocks (256 x 64), three, or of 2 x 4 blocks (128 x 64), four; two LDS buffers of one 128-index block each; code words straight from global memory to
// registers, one block ahead.
// NPL: planes multiplied, 3 or (switch TSVD_FP6_PLANES=2, never by default) the first two: two thirds of the MFMAs
// for activations exact to 2^-9.8 instead of 2^-14.7 of a block's largest magnitude.
// The work of one workgroup: the tile of WM TM 16 rows from strip tile_strip0 on, tokens b0 .. b0 + 16 TN WN
// (TN = 4 token blocks per wavefront everywhere but in the last, partly filled round of tsvd_gemm_fp6_tail_kernel).
template <bool STAGE2, int EX, int WM, int WN, int TM, int NPL, bool DIRECT, int TN = 4>
__device__ __forceinline__ void fp6_tile(const gemm_args& p, const int b0, const int tile_strip0, unsigned char* smem) {
    static_assert(WM * WN == 4, "four wavefronts");
    static_assert(!DIRECT || (!STAGE2 && TM == 8 && NPL == 3 && EX == 0), "planes straight from stage V: a wavefront owns whole 128-index blocks");
    constexpr int BT = WN * TN * 16;
    constexpr int BLK_BYTES = BT / 16 * FP6_REC_BYTES;      // one 128-index block of this workgroup's tokens
    constexpr int PIECES = (BLK_BYTES + 1023) / 1024;       // 38 or 19 pieces of 1 KiB (narrow tiles: the last one partly filled)
    constexpr bool PARTIAL = BLK_BYTES % 1024 != 0;
    float* cs_lds = reinterpret_cast<float*>(smem + 2 * BLK_BYTES);   // (LDS: 2 x BLK_BYTES, then BT column factors)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave - wm * WN;
    const int i = lane & 15, g = lane >> 4;
    const int strip0 = tile_strip0 + wm * TM;
    const int nblocks = p.plane_blocks ? p.plane_blocks : p.nkt * 2;   // blocks per token group in the planes' layout
    const int nrun = p.npairs, lastb = nrun - 1;      // blocks that hold anything

    const i32x4 act_rsrc = raw_rsrc(p.act, p.act_bytes);
    const __amdgpu_buffer_rsrc_t w_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.tiles), 0, p.tile_bytes, 0x00020000);
    typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_byte_ptr)smem;

    f32x4 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // one block of this workgroup's tokens = PIECES pieces of 1 KiB; wavefront w copies pieces
    // w, w + 4, ... (a wavefront whose last piece would lie beyond the block copies the last one again)
    auto issue = [&](int blk, int buf) {
        const int rec0 = ((b0 >> 7) * nblocks + blk) * FP6_PAIR_BYTES + ((b0 & 127) >> 4) * FP6_REC_BYTES;
#pragma unroll
        for (int c = 0; c < (PIECES + 3) / 4; ++c) {
            const int piece = min(c * 4 + wave, PIECES - 1);
            if (!PARTIAL || piece * 1024 + lane * 16 < BLK_BYTES)      // (lanes beyond the block would write into the other buffer)
                buf_load128_to_lds(act_rsrc, lds_base + buf * BLK_BYTES + piece * 1024, lane * 16, rec0 + piece * 1024);
        }
    };
    // DIRECT: row r = 4 gg + vv of result block a is loaded from row 64 (gg & 1) + 16 (gg >> 1) + 32 (a >> 2) + 4 (a & 3) + vv
    // of the wavefront's 128 rows (any row order is free on the A side), so that result lane (g, token) ends up holding the
    // 32 rank positions of lane (g, token) of stage U's B operand, in element order 4 a + v (see tsvd_panel_fp6_kernel)
    const int rr = lane & 15, gg = rr >> 2, vv = rr & 3;
    const int w_voff = DIRECT ? (4 * (gg & 1) + (gg >> 1)) * p.nkt * 1024 + (g * 16 + vv) * 16 : lane * 16;
    auto load_w = [&](int blk, u32x2 (&w)[TM]) {
        // (fp32 activations come as two sets of planes, the second set's blocks behind the first's: the same code words again)
        if (p.code_blocks && blk >= p.code_blocks) blk -= p.code_blocks;
        const int soff = (strip0 * p.nkt + (blk >> 1)) * 1024 + (blk & 1) * 8;
#pragma unroll
        for (int a = 0; a < TM; ++a)
            w[a] = __builtin_amdgcn_raw_buffer_load_b64(w_rsrc, w_voff, soff + (DIRECT ? 2 * (a >> 2) * p.nkt * 1024 + 4 * (a & 3) * 16 : a * p.nkt * 1024), 0);
    };
    auto compute = [&](int buf, const u32x2 (&w)[TM]) {
        u32x4 av[TM];
#pragma unroll
        for (int a = 0; a < TM; ++a)
            av[a] = u32x4{(w[a].x << 2) & 0xCCCCCCCCu, w[a].x & 0xCCCCCCCCu, (w[a].y << 2) & 0xCCCCCCCCu, w[a].y & 0xCCCCCCCCu};
        // NPL x 4 steps (token tile b = s / NPL, plane s % NPL) of TM MFMAs each; the operands of step s + DEPTH
        // are read from LDS before the MFMAs of step s are issued (the scheduler is held to this order:
        // left to itself it reads every operand right before its use and the wavefront waits for LDS
        // ten times per block)
        constexpr int DEPTH = FP6_LDS_DEPTH, NSET = DEPTH + 1;
        u32x4 lo[NSET];
        u32x2 hi[NSET];
        uint32_t sc[2];
        auto read_step = [&](int st) {
            const unsigned char* rec = smem + buf * BLK_BYTES + (wn * TN + st / NPL) * FP6_REC_BYTES;
            const int pl = st % NPL;
            lo[st % NSET] = *reinterpret_cast<const u32x4*>(rec + pl * 1024 + lane * 16);
            hi[st % NSET] = *reinterpret_cast<const u32x2*>(rec + 3072 + pl * 512 + lane * 8);
            if (pl == 0) sc[(st / NPL) & 1] = *reinterpret_cast<const uint32_t*>(rec + 4608 + lane * 4);
        };
#pragma unroll
        for (int st = 0; st < DEPTH; ++st) read_step(st);
#pragma unroll
        for (int st = 0; st < NPL * TN; ++st) {
            if (st + DEPTH < NPL * TN) read_step(st + DEPTH);
            __builtin_amdgcn_sched_barrier(0);
            const int b = st / NPL, q = st % NSET;
            // the eight row blocks of one plane: consecutive MFMAs never wait for each other's result
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                switch (st % NPL) {
                    case 0: acc[a][b] = mfma_fp6<0>(av[a], lo[q], hi[q], sc[b & 1], acc[a][b]); break;
                    case 1: acc[a][b] = mfma_fp6<1>(av[a], lo[q], hi[q], sc[b & 1], acc[a][b]); break;
                    default: acc[a][b] = mfma_fp6<2>(av[a], lo[q], hi[q], sc[b & 1], acc[a][b]); break;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto touch = [&](const u32x2 (&w)[TM]) {
#pragma unroll
        for (int a = 0; a < TM; ++a) asm volatile("" :: "v"(w[a].x), "v"(w[a].y));
    };

    u32x2 wa[TM], wb[TM];
    float cmax = 0.f;
    // (no per-token factors when z comes as planes straight from stage V, DIRECT there, colmax == null here:
    // the block scales carry the range, and S / 4 has undone the +-2 of both stages' codes)
    const bool factors = !DIRECT && p.colmax != nullptr;
    if (threadIdx.x < BT && factors) cmax = load_column_max<STAGE2>(p, b0 + threadIdx.x);
    load_w(0, wa);
    issue(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    touch(wa);
    if (threadIdx.x < BT) {
        if (factors) publish_column_factor<STAGE2>(p, b0 + threadIdx.x, cmax, cs_lds, threadIdx.x);
        else cs_lds[threadIdx.x] = 1.0f;
    }
    __syncthreads();
    for (int P = 0; P < nrun; P += 2) {
        int nx = min(P + 1, lastb);
        load_w(nx, wb);
        issue(nx, 1);
        compute(0, wa);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // block P + 1 has landed (this wavefront's part)
        touch(wb);
        __syncthreads();
        nx = min(P + 2, lastb);
        load_w(nx, wa);
        issue(nx, 0);
        if (P + 1 <= lastb) compute(1, wb);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        touch(wa);
        __syncthreads();
    }
    if constexpr (DIRECT) {
        // z = S (V x) / 4 -> three planes per lane and token tile, written as the records stage U reads
        // ([128-token group][128-index block][16-token tile], the layout of tsvd_z_planes_kernel)
        const int kb = strip0 >> 3;
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const f32x4 sv = *reinterpret_cast<const f32x4*>(p.S + 128 * kb + 64 * (g & 1) + 16 * (g >> 1) + 32 * (a >> 2) + 4 * (a & 3));
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] *= 0.25f * sv;
        }
        const int tok = b0 + wn * TN * 16;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            float v[32];
#pragma unroll
            for (int e = 0; e < 32; ++e) v[e] = acc[e >> 2][b][e & 3];
            unsigned char* rec = static_cast<unsigned char*>(p.out) +
                                 ((size_t)(((tok + 16 * b) >> 7) * (int)p.ld_out + kb) * 8 + (((tok + 16 * b) & 127) >> 4)) * FP6_REC_BYTES;   // (ld_out: blocks per token group)
            if (!p.two_sets) tsvd_planes_of_32(v, rec, lane);
            else if (kb < p.two_sets) tsvd_planes_of_32_twice(v, rec, rec + (size_t)p.two_sets * 8 * FP6_REC_BYTES, lane);   // (fp32 path: six planes)
        }
    } else {
        gemm_epilogue<TM, TN, STAGE2, EX>(p, acc, strip0, b0, wn * TN * 16, cs_lds, i, g);
    }
}

template <bool STAGE2, int EX, int WM = 2, int WN = 2, int TM = 8, int NPL = 3, bool DIRECT = false>
__global__ void __launch_bounds__(256, 2)
tsvd_gemm_fp6_kernel(gemm_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    fp6_tile<STAGE2, EX, WM, WN, TM, NPL, DIRECT>(p, blockIdx.x * WN * 64, blockIdx.y * WM * TM, smem);
}

// A stage in 512 x 64 tiles with a tail of narrower ones.  All tiles of a launch cost the same and two workgroups share a
// compute unit, so T tiles take ceil(T / (2 CUs)) rounds: stage U of a 36864 x 18432 factor at 2048 tokens is 4.5 rounds of work in
// the time of 5, its stage V 2.25 in the time of 3.  Here the rows of tiles that fill whole rounds (the first big_tiles) are
// 512 x 64; the rest is cut along the tokens into 512 x 16 TNT tiles (TNT = 2 or 1), two or four times as many workgroups that
// fill the last round.  (Cut along the rows instead, 256 x 64, a tail tile took 0.85 of a whole one: it streams the same planes
// for half the MFMAs.)  One-dimensional grid: big_tiles x ceil(B / 64) workgroups, then the tail's, token tile fastest.
template <bool STAGE2, int EX, bool DIRECT, int TNT>
__global__ void __launch_bounds__(256, 2)
tsvd_gemm_fp6_tail_kernel(gemm_args p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int cols = (p.bvalid + 63) / 64, nbig = p.big_tiles * cols, id = blockIdx.x;
    if (id < nbig) {
        fp6_tile<STAGE2, EX, 4, 1, 8, 3, DIRECT, 4>(p, (id % cols) * 64, (id / cols) * 32, smem);
    } else {
        const int tcols = (p.bvalid + 16 * TNT - 1) / (16 * TNT), t = id - nbig;
        fp6_tile<STAGE2, EX, 4, 1, 8, 3, DIRECT, TNT>(p, (t % tcols) * 16 * TNT, (p.big_tiles + t / tcols) * 32, smem);
    }
}

// ---- token-panel kernel on fp4 codes x fp6 planes ---------------------------------------------
// The same ownership as tsvd_panel_kernel (a workgroup takes 64 tokens from x to y, z never leaves the compute
// unit), with the arithmetic of tsvd_gemm_fp6_kernel: both stages multiply fp4 codes by three E2M3 planes on
// v_mfma_scale_f32_16x16x128_f8f6f4, 48 matrix-pipe cycles per 16 x 16 x 128 block against 64 for the 16-bit
// form, and 6 decoding operations per 8 bytes of code words against 32.
//   phase 0  x[N][64 tokens] -> plane records in LDS (a lane gathers the 32 values of its operand lane from
//            global memory; rows beyond N and tokens beyond B read as zero);
//   phase 1  wavefront w multiplies rank block w (128 rank positions x 64 tokens) and keeps it in registers.
//            Row r = 4 g + v of its j-th 16 x 16 result block is loaded from V's row 64 (g & 1) + 16 (g >> 1) +
//            32 (j >> 2) + 4 (j & 3) + v of the rank block (a per-lane address into the 1-KiB tiles), so that
//            result lane (g, token) ends up holding exactly the 32 rank positions, in element order 4 j + v,
//            of lane (g, token) of stage U's B operand: no exchange between lanes or wavefronts;
//   then     barrier (everyone is done with the planes of x), z = S * result -> planes straight from the
//            accumulators (fp32, not rounded to 16 bits first; no per-token factor: the block scales carry
//            the range) into the same LDS area, barrier;
//   phase 2  Y = U Z in units of 128 rows x 64 tokens, code words of U from global memory to registers two blocks
//            ahead, operands from the resident records two steps ahead: no barrier, no waiting for memory.
// Limits: N, K <= 1024 (eight records of 4864 bytes per 16 tokens fill the LDS of a compute unit).
// Measured on MI355X, M = 2048, N = 512, K = 1024, 12544 tokens (196 workgroups): 59 - 62 us per call against 63 - 67 us
// for tsvd_panel_kernel<16> on the same boxes, 2.6e-5 of max |y| against 1.8e-4 (z is not rounded to 16 bits).
// In-kernel clocks (us after the workgroup's start): planes of x 3.7, phase 1 multiplied 12.6, planes of z 15.8, the
// older wavefront of each SIMD done 45, the younger 54.  A stand-alone copy of the phase-2 loop reaches one MFMA per
// 19 cycles per SIMD with two wavefronts (16 is the pipe's limit; a single wavefront gets 24.5) and 21.5 with the
// stores of Y; the kernel itself 25 at the 2.0 GHz the chip sustains under it.  Tried and dropped: units of 128 rows x
// 32 tokens to start the stores earlier (+3 us: the code words are decoded twice as often), nontemporal stores (no
// change), the two wavefronts of a SIMD taking turns in priority (-0.5 us, inside the noise).
#define TSVD_PANEL6_MAX_BLOCKS 8
#ifndef TSVD_P6_UTN
#define TSVD_P6_UTN 4                   // token tiles per unit of phase 2
#endif
#define TSVD_PANEL6_LDS (TSVD_PANEL6_MAX_BLOCKS * 4 * FP6_REC_BYTES)          // 155648
#define TSVD_PANEL6_LDS_EX (TSVD_PANEL6_LDS + TSVD_PANEL_BIAS_ROWS * 4)        // 163840: all of it

template <int EX = 0>
__global__ void __launch_bounds__(512, 1)
tsvd_panel_fp6_kernel(panel_args p) {
    constexpr int TM = 8, TN = 4, NW = 8, BT = 64;
    extern __shared__ __align__(16) unsigned char smem[];     // records [block][token tile]: planes of x, then of z
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int b0 = blockIdx.x * BT;
    auto tick = [&](int n) {
        if (p.clocks && threadIdx.x == 0 && blockIdx.x < TSVD_GEMV_MAX_GRID) p.clocks[blockIdx.x * 16 + n] = wall_clock64();
    };
    tick(0);
    const float* bias_lds = nullptr;
    if constexpr (EX != 0) {
        if (p.bias && p.M <= TSVD_PANEL_BIAS_ROWS) {
            float* dst = reinterpret_cast<float*>(smem + TSVD_PANEL6_LDS);
            for (int r = threadIdx.x; r < p.M; r += 64 * NW) dst[r] = p.bias[r];
            bias_lds = dst;
        }
    }
    const int nvb = p.npairs_v, nub = p.npairs_u;             // 128-index blocks of N and of K that hold anything

    // One step = the eight MFMAs (row blocks) of one plane of one record.  The B operand of step t + 2 is read
    // from LDS before the MFMAs of step t are issued, across records and blocks, so that no step waits for LDS
    // (the scheduler is held to this order: left to itself it reads every operand right before its use).  The
    // operand set of a plane is slot `plane`; the scale words of consecutive records alternate between two.
    u32x4 lo[3];
    u32x2 hi[3];
    auto read_planes = [&](const unsigned char* rec, int pl) {
        lo[pl] = *reinterpret_cast<const u32x4*>(rec + pl * 1024 + lane * 16);
        hi[pl] = *reinterpret_cast<const u32x2*>(rec + 3072 + pl * 512 + lane * 8);
    };
    auto read_scales = [&](const unsigned char* rec) { return *reinterpret_cast<const uint32_t*>(rec + 4608 + lane * 4); };
    auto decode = [&](const u32x2 (&w)[TM], u32x4 (&av)[TM]) {
#pragma unroll
        for (int a = 0; a < TM; ++a)
            av[a] = u32x4{(w[a].x << 2) & 0xCCCCCCCCu, w[a].x & 0xCCCCCCCCu, (w[a].y << 2) & 0xCCCCCCCCu, w[a].y & 0xCCCCCCCCu};
    };

    // the MFMAs of one 128-index block for NT token tiles (NT x 3 planes x 8 row blocks): the tiles' records at cur, those
    // of the block that follows at nxt
    auto block_steps = [&](auto nt_c, const unsigned char* cur, const unsigned char* nxt, const u32x4 (&av)[TM], uint32_t (&sc)[2],
                           f32x4 (&acc)[TM][decltype(nt_c)::value]) {
        constexpr int NT = decltype(nt_c)::value;
        static_assert(NT % 2 == 0, "the scale words alternate between two registers");
#pragma unroll
        for (int st = 0; st < 3 * NT; ++st) {
            const int nt = st + 2, s2 = nt % (3 * NT);
            const unsigned char* rec = (nt < 3 * NT ? cur : nxt) + (s2 / 3) * FP6_REC_BYTES;
            read_planes(rec, s2 % 3);
            if (s2 % 3 == 0) sc[(s2 / 3) & 1] = read_scales(rec);
            __builtin_amdgcn_sched_barrier(0);
            const int b = st / 3;
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                switch (st % 3) {
                    case 0: acc[a][b] = mfma_fp6<0>(av[a], lo[0], hi[0], sc[b & 1], acc[a][b]); break;
                    case 1: acc[a][b] = mfma_fp6<1>(av[a], lo[1], hi[1], sc[b & 1], acc[a][b]); break;
                    default: acc[a][b] = mfma_fp6<2>(av[a], lo[2], hi[2], sc[b & 1], acc[a][b]); break;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ================= phase 0: planes of x =================
    {
        const __amdgpu_buffer_rsrc_t x_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), 0, p.x_bytes, 0x00020000);
        const int ld2 = (int)p.ldx * 2;
        const int njobs = nvb * TN;                           // job q: block q / 4 of N, token tile q % 4
        auto gather = [&](int q, uint32_t (&raw)[32]) {
            const int nb = q >> 2, b = q & 3;
            const int voff = (64 * (g & 1) + 16 * (g >> 1)) * ld2 + (b0 + 16 * b + i) * 2;
#pragma unroll
            for (int e = 0; e < 32; ++e)
                raw[e] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(x_rsrc, voff, (nb * 128 + 32 * (e >> 4) + (e & 15)) * ld2, 0);
        };
        if (p.x_token_major) {
            // x is [tokens][ldx]: a lane's two runs of 16 indices are contiguous, nothing to transpose
            const bool vec = !(p.ldx & 7) && !(reinterpret_cast<uintptr_t>(p.x) & 15);
            for (int q = wave; q < njobs; q += NW) {
                const int tok = b0 + 16 * (q & 3) + i;
                float v[32];
                tsvd_gather_token_major(x_rsrc, ld2, tok, (q >> 2) * 128 + 64 * (g & 1) + 16 * (g >> 1), p.N, tok < p.B, vec, v);
                tsvd_planes_of_32(v, smem + q * FP6_REC_BYTES, lane);
            }
        } else {
        // (two jobs in flight: the second one's trip to memory overlaps the first one's, not its conversion)
        uint32_t raw0[32], raw1[32];
        auto convert = [&](int q, const uint32_t (&raw)[32]) {
            const bool tok_ok = b0 + 16 * (q & 3) + i < p.B;
            float v[32];
#pragma unroll
            for (int e = 0; e < 32; ++e) v[e] = tok_ok ? __uint_as_float(raw[e] << 16) : 0.f;
            tsvd_planes_of_32(v, smem + q * FP6_REC_BYTES, lane);
        };
        if (wave < njobs) gather(wave, raw0);
        if (wave + NW < njobs) gather(wave + NW, raw1);
        for (int q = wave; q < njobs; q += 2 * NW) {
            convert(q, raw0);
            if (q + 2 * NW < njobs) gather(q + 2 * NW, raw0);
            if (q + NW < njobs) {
                convert(q + NW, raw1);
                if (q + 3 * NW < njobs) gather(q + 3 * NW, raw1);
            }
        }
        }
    }
    const __amdgpu_buffer_rsrc_t v_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.tiles_v), 0, p.tile_v_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t u_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.tiles_u), 0, p.tile_u_bytes, 0x00020000);

    // ================= phase 1: rank block `wave` of S V X =================
    // (Measured and dropped: one token tile after the other, the planes of a finished tile made while the other
    // wavefront of the SIMD multiplies: the code words are then decoded once per 24 MFMAs instead of once per 96,
    // and the stage took 15 instead of 12 us on N = 512, K = 1024.)
    {
        const bool has_block = wave < nub;
        f32x4 acc[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
        // lane (ga, r) of the A operand: row r = 4 gg + vv of result block j comes from row
        // 64 (gg & 1) + 16 (gg >> 1) + 32 (j >> 2) + 4 (j & 3) + vv of the rank block, i.e. strip
        // 8 wave + 4 (gg & 1) + (gg >> 1) + 2 (j >> 2), row 4 (j & 3) + vv of it
        const int r = lane & 15, gg = r >> 2, vv = r & 3;
        const int voff = ((8 * wave + 4 * (gg & 1) + (gg >> 1)) * p.nkt_v) * 1024 + (g * 16 + vv) * 16;
        auto load_wv = [&](int nb, u32x2 (&w)[TM]) {
#pragma unroll
            for (int j = 0; j < TM; ++j)
                w[j] = __builtin_amdgcn_raw_buffer_load_b64(
                    v_rsrc, voff, (2 * (j >> 2) * p.nkt_v + (nb >> 1)) * 1024 + 4 * (j & 3) * 16 + (nb & 1) * 8, 0);
        };
        u32x2 wa[TM];
        if (has_block) load_wv(0, wa);
        __syncthreads();                                  // the planes of x are complete
        tick(1);
        if (has_block) {
            const int lastb = nvb - 1;
            read_planes(smem, 0);
            read_planes(smem, 1);
            uint32_t sc[2];
            sc[0] = read_scales(smem);
            for (int nb = 0; nb < nvb; ++nb) {
                const unsigned char* cur = smem + nb * TN * FP6_REC_BYTES;
                const unsigned char* nxt = smem + min(nb + 1, lastb) * TN * FP6_REC_BYTES;
                u32x4 av[TM];
                decode(wa, av);
                load_wv(min(nb + 1, lastb), wa);          // (the wait for it falls at the next decode)
                block_steps(std::integral_constant<int, TN>{}, cur, nxt, av, sc, acc);
            }
            // z = S * (V x) / 4 (the codes of either stage multiply as +-2; powers of two, so nothing is rounded): S of this
            // lane's 32 rank positions, four consecutive ones per result block
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const f32x4 sv = *reinterpret_cast<const f32x4*>(p.S + 128 * wave + 64 * (g & 1) + 16 * (g >> 1) + 32 * (j >> 2) + 4 * (j & 3));
#pragma unroll
                for (int b = 0; b < TN; ++b) acc[j][b] *= 0.25f * sv;
            }
        }
        __syncthreads();                                  // every wavefront is done with the planes of x
        tick(2);
        if (has_block) {
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                float v[32];
#pragma unroll
                for (int e = 0; e < 32; ++e) v[e] = acc[e >> 2][b][e & 3];
                tsvd_planes_of_32(v, smem + (wave * TN + b) * FP6_REC_BYTES, lane);
            }
        }
        __syncthreads();
        tick(3);
    }

    // ================= phase 2: Y = U Z in units of 128 rows x 16 UTN tokens, no barriers =================
    // A wavefront's units follow each other as one sequence of blocks: the code words of block s + 2 of the sequence are
    // requested when block s is decoded, so those of the next unit's first two blocks are in registers before this
    // unit's stores are issued (stores and loads share one counter: a load requested after 64 stores is known to be
    // in only when they all are), and the B operands are read two steps ahead across unit boundaries as well.
    // (The stores cost the phase 8 of its 39 us: the same kernel without them takes 48 instead of 60 us per call, and
    // 56 with all of them going to one small cached region, so it is the store instructions, not HBM.)
    {
        constexpr int UTN = TSVD_P6_UTN, HALVES = TN / UTN;
        const int units = ((p.M + 127) / 128) * HALVES, lastb = nub - 1;
        const int w_voff = lane * 16;
        if (wave < units) {
            const int last_un = wave + (units - 1 - wave) / NW * NW;
            const int tile0 = (wave % HALVES) * UTN;          // (the same for all units of a wavefront: NW is a multiple of HALVES)
            int lu = wave, lb = 0;                            // the block of the sequence that the next request fetches
            auto load_next = [&](u32x2 (&w)[TM]) {
                const int soff = ((lu / HALVES) * TM * p.nkt_u + (lb >> 1)) * 1024 + (lb & 1) * 8;
#pragma unroll
                for (int a = 0; a < TM; ++a) w[a] = __builtin_amdgcn_raw_buffer_load_b64(u_rsrc, w_voff, soff + a * p.nkt_u * 1024, 0);
                if (lb < lastb) ++lb;
                else if (lu < last_un) { lu += NW; lb = 0; }  // (at the end: the last block again)
            };
            u32x2 w0[TM], w1[TM];
            load_next(w0);
            load_next(w1);
            const unsigned char* z0 = smem + tile0 * FP6_REC_BYTES;
            read_planes(z0, 0);
            read_planes(z0, 1);
            uint32_t sc[2];
            sc[0] = read_scales(z0);
            for (int unit = wave; unit < units; unit += NW) {
                const int strip0 = (unit / HALVES) * TM;
                f32x4 acc[TM][UTN];
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < UTN; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
                for (int blk = 0; blk < nub; blk += 2) {
                    u32x4 av[TM];
                    decode(w0, av);
                    load_next(w0);
                    block_steps(std::integral_constant<int, UTN>{}, z0 + blk * TN * FP6_REC_BYTES,
                                z0 + (blk == lastb ? 0 : blk + 1) * TN * FP6_REC_BYTES, av, sc, acc);
                    if (blk + 1 <= lastb) {
                        decode(w1, av);
                        load_next(w1);
                        block_steps(std::integral_constant<int, UTN>{}, z0 + (blk + 1) * TN * FP6_REC_BYTES,
                                    z0 + (blk + 1 == lastb ? 0 : blk + 2) * TN * FP6_REC_BYTES, av, sc, acc);
                    }
                }
                if (nub & 1) {                                // the sequence goes on in the other register set
#pragma unroll
                    for (int a = 0; a < TM; ++a) {
                        const u32x2 t = w0[a];
                        w0[a] = w1[a];
                        w1[a] = t;
                    }
                }
                // (wait for the next unit's code words here, before the stores)
#pragma unroll
                for (int a = 0; a < TM; ++a) asm volatile("" :: "v"(w0[a].x), "v"(w0[a].y), "v"(w1[a].x), "v"(w1[a].y));
                float br[TM][4];
                if constexpr (EX != 0) {
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
                int c0 = b0 + tile0 * 16;                     // first token of the unit
                asm volatile("" : "+s"(c0));                  // (addresses are formed here, not kept in registers over the MFMAs)
                if constexpr (EX == 3) {
                    const bool vec_ok = !(p.ldy & 3) && !(reinterpret_cast<uintptr_t>(p.y) & 15);
                    if (vec_ok && c0 + UTN * 16 <= p.B && strip0 * 16 + 128 <= p.M && p.ldy < (1ll << 22)) {
                        // every token and row of the unit exists: the lane's four rows of a token as one 16-byte (fp32) or
                        // 8-byte (bf16) store at a per-lane constant offset plus a scalar
                        const int esz = p.out_bf16 ? 2 : 4;
                        const size_t left = ((size_t)(p.B - c0) * p.ldy - strip0 * 16) * esz;
                        const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                            static_cast<unsigned char*>(p.y) + ((size_t)c0 * p.ldy + strip0 * 16) * esz, 0,
                            (int)(left < 0xFFFFFFFFull ? left : 0xFFFFFFFFull), 0x00020000);
                        const int y_voff = (i * (int)p.ldy + 4 * g) * esz;
#pragma unroll
                        for (int a = 0; a < TM; ++a)
#pragma unroll
                            for (int b = 0; b < UTN; ++b) {
                                const float v0 = acc[a][b][0] + br[a][0], v1 = acc[a][b][1] + br[a][1], v2 = acc[a][b][2] + br[a][2],
                                            v3 = acc[a][b][3] + br[a][3];
                                if (p.out_bf16)
                                    __builtin_amdgcn_raw_buffer_store_b64(u32x2{(uint32_t)tsvd_bf16_rne(v0) | ((uint32_t)tsvd_bf16_rne(v1) << 16),
                                                                                (uint32_t)tsvd_bf16_rne(v2) | ((uint32_t)tsvd_bf16_rne(v3) << 16)},
                                                                          y_rsrc, y_voff + a * 16 * 2, b * 16 * (int)p.ldy * 2, 0);
                                else
                                    __builtin_amdgcn_raw_buffer_store_b128(u32x4{__float_as_uint(v0), __float_as_uint(v1), __float_as_uint(v2), __float_as_uint(v3)},
                                                                           y_rsrc, y_voff + a * 16 * 4, b * 16 * (int)p.ldy * 4, 0);
                            }
                        continue;
                    }
#pragma unroll
                    for (int a = 0; a < TM; ++a) {
#pragma unroll
                        for (int b = 0; b < UTN; ++b) {
                            const int col = c0 + b * 16 + i;
                            if (col < p.B)
                                tsvd_store_token_major4(p.y, p.ldy, col, (strip0 + a) * 16 + 4 * g, p.M, acc[a][b][0] + br[a][0],
                                                        acc[a][b][1] + br[a][1], acc[a][b][2] + br[a][2], acc[a][b][3] + br[a][3],
                                                        p.out_bf16, vec_ok);
                        }
                    }
                } else if constexpr (EX == 2) {
                    const bool aligned4 = !(p.ldy & 1) && !(reinterpret_cast<uintptr_t>(p.y) & 3);
                    if (aligned4 && c0 + UTN * 16 <= p.B && p.ldy < (1ll << 21)) {
                        // all tokens of the unit exist: the row pairs of tsvd_store_row_pair_bf16 (neighbouring lanes swap one
                        // value, an even lane stores tokens (i, i + 1) of row r, the odd one next to it tokens (i - 1, i) of
                        // row r + 1) as stores at a per-lane constant offset plus a scalar; rows beyond M fall outside the
                        // buffer's range
                        typedef float f32x2_t __attribute__((ext_vector_type(2)));
                        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                        const size_t left = ((size_t)(p.M - strip0 * 16) * p.ldy - c0) * 2;
                        const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                            static_cast<uint16_t*>(p.y) + (size_t)strip0 * 16 * p.ldy + c0, 0, (int)(left < 0xFFFFFFFFull ? left : 0xFFFFFFFFull), 0x00020000);
                        const int odd = i & 1, ld2 = (int)p.ldy * 2, y_voff = (4 * g + odd) * ld2 + (i - odd) * 2;
#pragma unroll
                        for (int a = 0; a < TM; ++a)
#pragma unroll
                            for (int vp = 0; vp < 4; vp += 2)
#pragma unroll
                                for (int b = 0; b < UTN; ++b) {
                                    const float v0 = acc[a][b][vp] + br[a][vp], v1 = acc[a][b][vp + 1] + br[a][vp + 1];
                                    const float recv = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(odd ? v0 : v1), 0xB1, 0xF, 0xF, true));
                                    const f32x2_t two = odd ? f32x2_t{recv, v1} : f32x2_t{v0, recv};
                                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2_t)), y_rsrc,
                                                                          y_voff + b * 32, (a * 16 + vp) * ld2, 0);
                                }
                    } else {
#pragma unroll
                        for (int a = 0; a < TM; ++a) {
#pragma unroll
                            for (int vp = 0; vp < 4; vp += 2) {
#pragma unroll
                                for (int b = 0; b < UTN; ++b)
                                    tsvd_store_row_pair_bf16(p.y, p.ldy, (strip0 + a) * 16 + 4 * g + vp, p.M, c0 + b * 16, i, p.B,
                                                             acc[a][b][vp] + br[a][vp], acc[a][b][vp + 1] + br[a][vp + 1], aligned4);
                            }
                        }
                    }
                } else if (c0 + UTN * 16 <= p.B && p.ldy < (1ll << 21)) {
                    // All tokens of the unit exist: 32 UTN stores whose addresses are the lane's constant offset plus a
                    // scalar (no vector arithmetic per store); rows beyond M fall outside the buffer's range and are
                    // dropped by the range check (the range is exact where it matters, in the last unit).  (Two tokens per
                    // lane and 8-byte stores, as in the bf16 form below: 62 - 66 against 60.6 - 62 us on 12544 tokens x 2048 rows.)
                    const size_t left = ((size_t)(p.M - strip0 * 16) * p.ldy - c0) * 4;
                    const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                        static_cast<float*>(p.y) + (size_t)strip0 * 16 * p.ldy + c0, 0, (int)(left < 0xFFFFFFFFull ? left : 0xFFFFFFFFull), 0x00020000);
                    const int ld4 = (int)p.ldy * 4;
                    const int y_voff = 4 * g * ld4 + i * 4;
#pragma unroll
                    for (int a = 0; a < TM; ++a)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
#pragma unroll
                            for (int b = 0; b < UTN; ++b)
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(EX == 1 ? acc[a][b][v] + br[a][v] : acc[a][b][v]), y_rsrc,
                                                                      y_voff + b * 64, (a * 16 + v) * ld4, 0);
                } else {
#pragma unroll
                    for (int a = 0; a < TM; ++a) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int row = (strip0 + a) * 16 + 4 * g + v;
                            if (row < p.M) {
                                float* dst = static_cast<float*>(p.y) + (size_t)row * p.ldy;
#pragma unroll
                                for (int b = 0; b < UTN; ++b) {
                                    const int col = c0 + b * 16 + i;
                                    if (col < p.B) dst[col] = EX == 1 ? acc[a][b][v] + br[a][v] : acc[a][b][v];
                                }
                            }
                        }
                    }
                }
            }
        }
    }
    tick(4);
    if (p.clocks && lane == 0 && blockIdx.x < TSVD_GEMV_MAX_GRID) p.clocks[blockIdx.x * 16 + 8 + wave] = wall_clock64();
}

}  // namespace

// The token-panel launch on fp4 codes x fp6 planes (tsvd_panel_fp6_kernel) or on the 16-bit kernel (TSVD_PANEL_FP6 = 0).
bool tsvd_gemm_panel_fp6() { return tsvd_tune("TSVD_PANEL_FP6", 1) != 0; }

// Stage U through fp6 planes of Z (tsvd_gemm_fp6_kernel): TSVD_FP6 = 0 never, 1 whenever the sizes
// allow, default by rule.  The planes of Z need tsvd_gemm_fp6_bytes more workspace.
size_t tsvd_gemm_fp6_bytes(long long Kp, long long Bp) { return (size_t)(Bp / 128) * (size_t)(Kp / 128) * FP6_PAIR_BYTES; }
bool tsvd_gemm_use_fp6(long long Mp, long long Kp, long long Np, long long B, long long cus, bool aligned) {
    const int mode = tsvd_tune("TSVD_FP6", -1);
    const long long Bp = tsvd_round_up(B, 256);
    if (mode == 0 || tsvd_gemm_fp6_bytes(Kp, Bp) >= (1ull << 31)) return false;
    (void)Np; (void)aligned;
    if (mode == 1) return true;
    // measured on MI355X against the 16-bit stage U (whole call): 36864 x 9216 x 18432 at 2048 tokens
    // 2.29 -> 2.18 ms, 16384 x 4096 x 8192 at 512 tokens 191 -> 153 us, 8192 x 2048 x 4096 at 1024 tokens
    // 108 -> 93 us, 4096 x 1024 x 2048 at 2048 tokens 64 -> 58 us; 3072 x 768 x 1536 at 4096 tokens 66 -> 67 us
    // and at 512 tokens 17 -> 50 us; 4096 x 1024 x 2048 at 1024 tokens (128 tiles) 39 -> 47 us, 12288 x 3072 x 6144 at
    // 256 tokens (96 tiles) 78 -> 89 us: long contractions with a 256 x 128 tile for every compute unit.  With
    // fewer, 256 x 64 tiles (three workgroups per compute unit), same comparison: 16384 x 4096 x 8192 at 256 tokens
    // (256 tiles of 256 x 64) 113 -> 98 us, 12288 x 3072 x 6144 at 256 (192) 75 -> 64 us, 8192 x 2048 x 4096 at 512 (256)
    // 65 -> 57 us, 6144 x 1536 x 3072 at 512 (192) 45 -> 40 us, 4096 x 1024 x 2048 at 1024 (256) 39.0 -> 38.4 us;
    // 8192 x 2048 x 4096 at 256 (128) 45 -> 45 us, 4096 x 1024 x 2048 at 512 (128) 27 -> 29 us: those tiles where three
    // quarters of the compute units get one.  Below that, 128 x 64 tiles (four workgroups per compute unit): the last
    // two shapes 45 -> 39 us and 27 -> 26 us; 6144 x 1536 x 3072 at 256 tokens (192 tiles of 128 x 64) 28 -> 31 us:
    // every compute unit must get a 128 x 64 tile.  Contractions of 1024 - 1536 indices: no gain with any tile
    // (3072 x 768 x 1536 at 512 tokens 17 -> 22 us, at 1024 tokens 28 -> 28.5 us)
    return Kp >= 2048 && (Mp / 128) * ((B + 63) / 64) >= cus;
}

// The same for stage V (planes of x), only together with the fp6 stage U (the workspace holds both
// sets of planes then): TSVD_FP6_V = 0 never, 1 whenever possible, default by the rule of stage U
// applied to stage V's own sizes.  Needs x with an even row pitch at a 4-byte aligned address.
bool tsvd_gemm_use_fp6_v(long long Mp, long long Kp, long long Np, long long B, long long cus, bool aligned) {
    if (!aligned || !tsvd_gemm_use_fp6(Mp, Kp, Np, B, cus, aligned)) return false;
    const int mode = tsvd_tune("TSVD_FP6_V", -1);
    const long long Bp = tsvd_round_up(B, 256);
    if (mode == 0 || tsvd_gemm_fp6_bytes(Np, Bp) >= (1ull << 31)) return false;
    if (mode == 1) return true;
    // With a 256 x 128 tile for every compute unit (where stage V would run on the large-tile kernel): measured
    // 18432 x 9216 at 2048 tokens 480 -> 17 + 406 us.  With fewer tiles stage V would run on the ring kernel, which
    // has its column maxima fused in; planes, a separate column-maximum launch and 128 x 64 or 256 x 64 tiles beat
    // it for contractions of 4096 (whole call 97 -> 92 us on 16384 x 4096 x 8192 at 256 tokens, 73 -> 68 us on
    // 8192 x 4096 x 4096 at 512) but not of 3072 (64 -> 70 us on 12288 x 3072 x 6144 at 256) or 2048 (58 -> 58 us)
    return (Np >= 2048 && (Kp / 256) * ((B + 127) / 128) >= cus) || (Np >= 4096 && (Kp / 128) * ((B + 63) / 64) >= cus);
}

template <int WM, int WN>
hipError_t init_fp6_direct() {
    constexpr int lds = 2 * (WN * 4 * FP6_REC_BYTES) + 512;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_kernel<false, 0, WM, WN, 8, 3, true>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}
template <int WM, int WN, int TM, int NPL = 3>
hipError_t init_fp6() {
    constexpr int lds = 2 * (WN * 4 * FP6_REC_BYTES) + 512;
    hipError_t e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_kernel<true, 0, WM, WN, TM, NPL>), hipFuncAttributeMaxDynamicSharedMemorySize, lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_kernel<true, 1, WM, WN, TM, NPL>), hipFuncAttributeMaxDynamicSharedMemorySize, lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_kernel<true, 2, WM, WN, TM, NPL>), hipFuncAttributeMaxDynamicSharedMemorySize, lds)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_kernel<true, 3, WM, WN, TM, NPL>), hipFuncAttributeMaxDynamicSharedMemorySize, lds)) != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_kernel<false, 0, WM, WN, TM, NPL>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}
// rows_p: padded rows of the stage's weights; ex: output variant (stage U only)
template <int WM, int WN, int TM, int NPL = 3>
hipError_t launch_fp6(bool stage2, const gemm_args& a, long long rows_p, int Bp, int ex, hipStream_t stream) {
    constexpr int lds = 2 * (WN * 4 * FP6_REC_BYTES) + 512;
    if (rows_p % (WM * TM * 16)) return hipErrorInvalidValue;
    const dim3 grid((a.bvalid + WN * 64 - 1) / (WN * 64), (unsigned)((a.rows_need + WM * TM * 16 - 1) / (WM * TM * 16))), block(256);
    if (!stage2) hipLaunchKernelGGL((tsvd_gemm_fp6_kernel<false, 0, WM, WN, TM, NPL>), grid, block, lds, stream, a);
    else if (ex == 2) hipLaunchKernelGGL((tsvd_gemm_fp6_kernel<true, 2, WM, WN, TM, NPL>), grid, block, lds, stream, a);
    else if (ex == 1) hipLaunchKernelGGL((tsvd_gemm_fp6_kernel<true, 1, WM, WN, TM, NPL>), grid, block, lds, stream, a);
    else if (ex == 3) hipLaunchKernelGGL((tsvd_gemm_fp6_kernel<true, 3, WM, WN, TM, NPL>), grid, block, lds, stream, a);
    else hipLaunchKernelGGL((tsvd_gemm_fp6_kernel<true, 0, WM, WN, TM, NPL>), grid, block, lds, stream, a);
    return hipGetLastError();
}
// 512 x 64 tiles (4 x 1 wavefronts) when the rows allow: half the traffic of the planes, twice that of the codes;
// 256 x 64 (four row blocks per wavefront) when those would leave compute units without a tile, 128 x 64 (two)
// when even those would leave more than a quarter of them without
// The tile of a launch: 0: 256 x 128 (2 x 2 wavefronts), 1: 512 x 64, 2: 256 x 64, 3: 128 x 64 (4 x 1 wavefronts of 8, 4, 2 row blocks)
static int fp6_tile(long long rows_p, long long bvalid, long long cus) {
    const int tall = env_cfg("TSVD_FP6_TALL", -1);       // forces one of them, default by rule
    const long long c128 = (bvalid + 127) / 128, c64 = (bvalid + 63) / 64;   // token tiles that are launched
    const bool small = tall < 0 && (rows_p / 256) * c128 < cus;
    if (tall == 3 || (small && 4 * (rows_p / 256) * c64 < 3 * cus)) return 3;
    if (tall == 2 || small) return 2;
    if (rows_p % 512 == 0 && tall != 0) return 1;
    return 0;
}
// A stage in 512 x 64 tiles whose last round of workgroups would be at most half full: rows of tiles that fill whole rounds,
// then a tail cut along the tokens (tsvd_gemm_fp6_tail_kernel; TSVD_FP6_TAIL = 0: never).  Returns false when the plain launch is
// as good; else the rows of whole tiles, the rows of tail tiles and the token blocks per wavefront of the tail (2 or 1).
static bool fp6_tail_shape(const gemm_args& a, long long cus, int* big, int* rest, int* tnt) {
    if (env_cfg("TSVD_FP6_TAIL", 1) == 0) return false;
    const long long C = (a.bvalid + 63) / 64, slots = 2 * cus;
    if (C <= 0 || slots % C) return false;
    const long long rows_per_round = slots / C, R = (a.rows_need + 511) / 512;
    const long long b = R / rows_per_round * rows_per_round, r = R - b;
    if (b == 0 || r == 0 || 2 * r * C > slots) return false;
    *big = (int)b;
    *rest = (int)r;
    *tnt = 4 * r * C <= slots ? 1 : 2;
    return true;
}
template <bool STAGE2, int EX, bool DIRECT>
static hipError_t launch_fp6_tail(const gemm_args& a, int big, int rest, int tnt, hipStream_t stream) {
    constexpr int lds = 2 * (4 * FP6_REC_BYTES) + 512;
    gemm_args t = a;
    t.big_tiles = big;
    const long long C = (a.bvalid + 63) / 64, TC = (a.bvalid + 16 * tnt - 1) / (16 * tnt);
    const dim3 grid((unsigned)(big * C + rest * TC)), block(256);
    if (tnt == 1) hipLaunchKernelGGL((tsvd_gemm_fp6_tail_kernel<STAGE2, EX, DIRECT, 1>), grid, block, lds, stream, t);
    else hipLaunchKernelGGL((tsvd_gemm_fp6_tail_kernel<STAGE2, EX, DIRECT, 2>), grid, block, lds, stream, t);
    return hipGetLastError();
}
template <bool STAGE2, int EX, bool DIRECT>
static hipError_t init_fp6_tail() {
    constexpr int lds = 2 * (4 * FP6_REC_BYTES) + 512;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_tail_kernel<STAGE2, EX, DIRECT, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_gemm_fp6_tail_kernel<STAGE2, EX, DIRECT, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}
hipError_t tsvd_fp6_launch(bool stage2, const gemm_args& a, long long rows_p, int Bp, int ex, long long cus, hipStream_t stream) {
    if (env_cfg("TSVD_FP6_PLANES", 3) == 2) {            // accuracy / speed switch (512 x 64 and 256 x 64 tiles only)
        if (rows_p % 512 == 0 && (rows_p / 256) * ((a.bvalid + 127) / 128) >= cus) return launch_fp6<4, 1, 8, 2>(stage2, a, rows_p, Bp, ex, stream);
        return launch_fp6<4, 1, 4, 2>(stage2, a, rows_p, Bp, ex, stream);
    }
    switch (fp6_tile(rows_p, a.bvalid, cus)) {
        case 3: return launch_fp6<4, 1, 2>(stage2, a, rows_p, Bp, ex, stream);
        case 2: return launch_fp6<4, 1, 4>(stage2, a, rows_p, Bp, ex, stream);
        case 1: {
            int big, rest, tnt;
            if (stage2 && rows_p % 512 == 0 && fp6_tail_shape(a, cus, &big, &rest, &tnt)) {
                if (ex == 2) return launch_fp6_tail<true, 2, false>(a, big, rest, tnt, stream);
                if (ex == 1) return launch_fp6_tail<true, 1, false>(a, big, rest, tnt, stream);
                if (ex == 3) return launch_fp6_tail<true, 3, false>(a, big, rest, tnt, stream);
                return launch_fp6_tail<true, 0, false>(a, big, rest, tnt, stream);
            }
            return launch_fp6<4, 1, 8>(stage2, a, rows_p, Bp, ex, stream);
        }
        default: return launch_fp6<2, 2, 8>(stage2, a, rows_p, Bp, ex, stream);
    }
}
// Stage V writing the planes of z itself (tiles whose wavefronts own whole 128-index blocks: 256 x 128 and 512 x 64)
bool tsvd_fp6_direct_possible(long long rows_p, long long bvalid, long long cus) {
    return env_cfg("TSVD_FP6_DIRECT", 1) != 0 && env_cfg("TSVD_FP6_PLANES", 3) != 2 && fp6_tile(rows_p, bvalid, cus) <= 1;
}
hipError_t tsvd_fp6_launch_direct(const gemm_args& a, long long rows_p, long long cus, hipStream_t stream) {
    const bool tall = fp6_tile(rows_p, a.bvalid, cus) == 1;
    const int wn = tall ? 1 : 2, rows_tile = tall ? 512 : 256, lds = 2 * (wn * 4 * FP6_REC_BYTES) + 512;
    if (rows_p % rows_tile) return hipErrorInvalidValue;
    const dim3 grid((a.bvalid + wn * 64 - 1) / (wn * 64), (unsigned)((a.rows_need + rows_tile - 1) / rows_tile)), block(256);
    int big, rest, tnt;
    if (tall && fp6_tail_shape(a, cus, &big, &rest, &tnt)) return launch_fp6_tail<false, 0, true>(a, big, rest, tnt, stream);
    if (tall) hipLaunchKernelGGL((tsvd_gemm_fp6_kernel<false, 0, 4, 1, 8, 3, true>), grid, block, lds, stream, a);
    else hipLaunchKernelGGL((tsvd_gemm_fp6_kernel<false, 0, 2, 2, 8, 3, true>), grid, block, lds, stream, a);
    return hipGetLastError();
}

hipError_t tsvd_fp6_launch_planes(bool bf16, const uint16_t* src, long long ld, int rows_valid, int cols_valid, int nblocks_per_group,
                                  int blocks, long long B, unsigned char* planes, hipStream_t stream, bool token_major) {
    const dim3 grid((unsigned)((B + 127) / 128), (unsigned)blocks), block(512);
    if (token_major) {       // (bf16 x, one row per token)
        const int vec = !(ld & 7) && !(reinterpret_cast<uintptr_t>(src) & 15);
        hipLaunchKernelGGL(tsvd_x_planes_token_major_kernel, grid, block, 0, stream, src, ld, (unsigned)((size_t)cols_valid * ld * 2), rows_valid,
                           cols_valid, nblocks_per_group, vec, planes);
        return hipGetLastError();
    }
    if (bf16) hipLaunchKernelGGL(tsvd_z_planes_kernel<true>, grid, block, 0, stream, src, ld, rows_valid, cols_valid, nblocks_per_group, planes);
    else hipLaunchKernelGGL(tsvd_z_planes_kernel<false>, grid, block, 0, stream, src, ld, rows_valid, cols_valid, nblocks_per_group, planes);
    return hipGetLastError();
}

hipError_t tsvd_fp6_launch_planes_f32(const float* x, long long ld, int rows_valid, int cols_valid, int blocks, unsigned char* planes,
                                      hipStream_t stream) {
    hipLaunchKernelGGL(tsvd_x_planes_f32_kernel, dim3((unsigned)((cols_valid + 127) / 128), (unsigned)blocks), dim3(512), 0, stream, x, ld,
                       rows_valid, cols_valid, 2 * blocks, blocks, planes);
    return hipGetLastError();
}

hipError_t tsvd_fp6_launch_panel(const panel_args& pa, int ex, hipStream_t stream) {
    const dim3 grid((unsigned)((pa.B + 63) / 64)), block(512);
    if (ex == 3) hipLaunchKernelGGL((tsvd_panel_fp6_kernel<3>), grid, block, TSVD_PANEL6_LDS_EX, stream, pa);
    else if (ex == 2) hipLaunchKernelGGL((tsvd_panel_fp6_kernel<2>), grid, block, TSVD_PANEL6_LDS_EX, stream, pa);
    else if (ex == 1) hipLaunchKernelGGL((tsvd_panel_fp6_kernel<1>), grid, block, TSVD_PANEL6_LDS_EX, stream, pa);
    else hipLaunchKernelGGL((tsvd_panel_fp6_kernel<0>), grid, block, TSVD_PANEL6_LDS, stream, pa);
    return hipGetLastError();
}

hipError_t tsvd_fp6_init() {
    hipError_t e;
    if ((e = init_fp6<2, 2, 8>()) != hipSuccess) return e;
    if ((e = init_fp6<4, 1, 8>()) != hipSuccess) return e;
    if ((e = init_fp6<4, 1, 4>()) != hipSuccess) return e;
    if ((e = init_fp6<4, 1, 2>()) != hipSuccess) return e;
    if ((e = init_fp6<4, 1, 8, 2>()) != hipSuccess) return e;
    if ((e = init_fp6<4, 1, 4, 2>()) != hipSuccess) return e;
    if ((e = init_fp6_tail<true, 0, false>()) != hipSuccess) return e;
    if ((e = init_fp6_tail<true, 1, false>()) != hipSuccess) return e;
    if ((e = init_fp6_tail<true, 2, false>()) != hipSuccess) return e;
    if ((e = init_fp6_tail<true, 3, false>()) != hipSuccess) return e;
    if ((e = init_fp6_tail<false, 0, true>()) != hipSuccess) return e;
    if ((e = init_fp6_direct<2, 2>()) != hipSuccess) return e;
    if ((e = init_fp6_direct<4, 1>()) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_fp6_kernel<0>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL6_LDS)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_fp6_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL6_LDS_EX)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_fp6_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 TSVD_PANEL6_LDS_EX)) != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(tsvd_panel_fp6_kernel<3>), hipFuncAttributeMaxDynamicSharedMemorySize,
                               TSVD_PANEL6_LDS_EX);
}
