// What the batched kernels of tsvd_gemm.hip (16-bit operands) and tsvd_fp6.hip (fp4 codes x fp6 planes) share: the
// argument blocks of their launches, the per-token factors, the epilogues, the buffer-load helpers, and the host-side
// interface between the two files.  Everything device-side sits in an unnamed namespace: each file gets its own copy.
#ifndef TSVD_GEMM_COMMON_H
#define TSVD_GEMM_COMMON_H
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsvd_epilogue.h"
#include "tsvd_kernels.h"
#include "tsvd_layout.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define TSVD_DEC(w, j) ((((uint32_t)(w)) << (14 - 2 * (j))) & 0xC000C000u)
#define KT 64   // contraction depth of one LDS stage

struct gemm_args {
    const uint32_t* tiles;    // packed A: [strips][nkt][256 words]
    int nkt;                  // 256-wide tiles along the contraction index (the stride of a strip)
    int npairs;               // 128-index steps of the contraction that hold anything (<= 2 nkt): the loops end there
    int last_steps;           // 32-index sub-steps of the last of them that hold anything (1..4; see tsvd_rank_position)
    const uint16_t* act;      // activations [kdim][ld] 16-bit
    long long ld;
    int kvalid;               // activation rows that exist (stage 1: N); others read as zero
    int bvalid;               // activation columns that exist
    unsigned act_bytes;       // size of the activation buffer (buffer-load range check)
    unsigned tile_bytes;      // size of the packed tiles
    const float* S;           // stage 1: row scales
    const float* colpart;     // column maxima: partials [PARTS][Bp], then the final row [Bp]
    float* colmax;            // the final row (stage 1 writes it, stage 2 reads it)
    int Bp;
    float bound_V;
    void* out;                // stage 1: fp16 [Kp][Bp];  stage 2: fp32 (or bf16 with out_bf16) [M][ldy]
    long long ld_out;
    const float* bias;        // stage 2 (EX kernels): added per output row, or null
    int out_bf16;             // stage 2 (EX kernels): output type
    int out_token_major;      // stage 2 (EX = 3): out is [tokens][ld_out] (one row per token) instead of [M][ld_out]
    int rows_valid;           // stage 2: M
    int big_tiles;            // tsvd_gemm_fp6_tail_kernel: rows of 512 x 64 tiles before the narrower ones
    int plane_blocks;         // fp4 x fp6 kernels: 128-index blocks per token group in the planes at `act` (0: 2 nkt)
    int code_blocks;          // fp4 x fp6 kernels, fp32 activations: blocks of the contraction after which the code words repeat (0: never)
    int two_sets;             // fp4 x fp6 stage V writing planes: 0, or the number of valid blocks = distance of the second set of planes
    int rows_need;            // rows of the stage that have to be computed (stage 1: the rank positions stage 2 reads; stage 2: M)
    long long* clocks;        // tuning aid: phase timestamps per workgroup (stage 1: 0..7, stage 2: 8..15), or null
};

struct panel_args {
    const uint32_t* tiles_v;  // packed V [Kp/16][Np/256][256 words]
    const uint32_t* tiles_u;  // packed U [Mp/16][Kp/256][256 words]
    unsigned tile_v_bytes, tile_u_bytes;
    int nkt_v, nkt_u;         // Np / 256, Kp / 256
    int npairs_v, npairs_u;   // 128-index steps of either contraction that hold anything (ceil(N / 128), ceil(K / 128))
    const uint16_t* x;        // bf16 [N][ldx], or [B][ldx] with x_token_major (tsvd_panel_fp6_kernel only)
    long long ldx;
    unsigned x_bytes;
    int N, x_token_major;
    const float* S;
    float bound_V;
    int Kp, Mp, M, B;
    void* y;                  // fp32 (or bf16 with out_bf16) [M][ldy]
    long long ldy;
    const float* bias;        // EX kernels: added per output row, or null
    int out_bf16;             // EX kernels: output type
    int out_token_major;      // EX = 3: y is [tokens][ldy]
    long long* clocks;
};
// The variants with output options keep the bias of up to 2048 rows in LDS behind that (read at
// the end of every unit of phase 2: from global memory each read stalled the wavefront for an L2
// round trip, +8 us on 12544 tokens x 2048 rows).
#define TSVD_PANEL_BIAS_ROWS 2048

namespace {

// Exponent e of the power-of-two scale for a column whose largest |x| is m:
// bound_V * m * 2^e <= 2^14.
__device__ __forceinline__ int scale_exponent(float m, float bound_V) {
    const float bound = bound_V * m;
    int ex = 0;
    if (bound > 0.f && bound < 3.0e38f) (void)frexpf(bound, &ex);   // bound < 2^ex
    return max(-110, min(110, 14 - ex));
}

// Per-token factors of a workgroup tile, computed once per workgroup into LDS before the main
// loop (thread t owns token b0 + t): stage 1 multiplies by scale / 2, stage 2 by 1 / (2 scale); the
// 2 undoes the +-2 of the decoded weights.  Stage 1 reduces the partial maxima and (first row of
// workgroups only) publishes the final maximum for stage 2.
template <bool STAGE2>
__device__ __forceinline__ float load_column_max(const gemm_args& p, int col) {
    if constexpr (STAGE2) return p.colmax[col];
    float m = 0.f;
#pragma unroll
    for (int q = 0; q < TSVD_COLMAX_PARTS; ++q) m = fmaxf(m, p.colpart[(size_t)q * p.Bp + col]);
    return m;
}
template <bool STAGE2>
__device__ __forceinline__ void publish_column_factor(const gemm_args& p, int col, float m, float* cs_lds, int t) {
    const int e = scale_exponent(m, p.bound_V);
    cs_lds[t] = ldexpf(1.0f, STAGE2 ? -e - 1 : e - 1);
    if constexpr (!STAGE2)
        if (blockIdx.y == 0) p.colmax[col] = m;
}

// Result block layout: lane (i, g) holds token i, weight rows 4 g + v.
// EX: the variants with the bias and the choice of the output type (instantiated apart so that the
// plain fp32 epilogue of the tuned kernels stays as it is): 1 = fp32 with bias, 2 = bf16 (with or
// without bias), two rows per store, 3 = token-major output (either type, with or without bias).
template <int TM, int TN, bool STAGE2, int EX = 0>
__device__ __forceinline__ void gemm_epilogue(const gemm_args& p, f32x4 (&acc)[TM][TN], int strip0, int b0, int tok0,
                                              const float* cs_lds, int i, int g) {
    float cs[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) cs[b] = cs_lds[tok0 + b * 16 + i];
    const int col0 = b0 + tok0;
    float sr[TM][4];                  // stage 1: row scales S; stage 2 with options: the bias
    if constexpr (!STAGE2) {
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const f32x4 q = *reinterpret_cast<const f32x4*>(p.S + (strip0 + a) * 16 + 4 * g);
            sr[a][0] = q.x; sr[a][1] = q.y; sr[a][2] = q.z; sr[a][3] = q.w;
        }
    }
    if constexpr (STAGE2 && EX != 0) {
        // all bias loads first, unconditional (rows clamped), so that no store waits for its own load
        if (p.bias) {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 4; ++v) sr[a][v] = p.bias[min((strip0 + a) * 16 + 4 * g + v, p.rows_valid - 1)];
        } else {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 4; ++v) sr[a][v] = 0.f;
        }
    }
    if constexpr (STAGE2 && EX == 3) {        // token-major output (fp32 or bf16, with or without bias): four rows per store
        const bool vec_ok = !(p.ld_out & 3) && !(reinterpret_cast<uintptr_t>(p.out) & 15);
#pragma unroll
        for (int a = 0; a < TM; ++a) {
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const int col = col0 + b * 16 + i;
                if (col < p.bvalid)
                    tsvd_store_token_major4(p.out, p.ld_out, col, (strip0 + a) * 16 + 4 * g, p.rows_valid, acc[a][b][0] * cs[b] + sr[a][0],
                                            acc[a][b][1] * cs[b] + sr[a][1], acc[a][b][2] * cs[b] + sr[a][2], acc[a][b][3] * cs[b] + sr[a][3],
                                            p.out_bf16, vec_ok);
            }
        }
        return;
    }
    if constexpr (STAGE2 && EX == 2) {        // bf16 in pairs: rows two by two, tokens left to right
        const bool aligned4 = !(p.ld_out & 1) && !(reinterpret_cast<uintptr_t>(p.out) & 3);
#pragma unroll
        for (int a = 0; a < TM; ++a) {
#pragma unroll
            for (int vp = 0; vp < 4; vp += 2) {
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    tsvd_store_row_pair_bf16(p.out, p.ld_out, (strip0 + a) * 16 + 4 * g + vp, p.rows_valid, col0 + b * 16, i, p.bvalid,
                                             acc[a][b][vp] * cs[b] + sr[a][vp], acc[a][b][vp + 1] * cs[b] + sr[a][vp + 1], aligned4);
            }
        }
        return;
    }
    if constexpr (STAGE2 && EX == 1) {        // fp32 with bias, row by row
#pragma unroll
        for (int a = 0; a < TM; ++a) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = (strip0 + a) * 16 + 4 * g + v;
                if (row < p.rows_valid) {
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        const int col = col0 + b * 16 + i;
                        if (col < p.bvalid) static_cast<float*>(p.out)[(size_t)row * p.ld_out + col] = acc[a][b][v] * cs[b] + sr[a][v];
                    }
                }
            }
        }
        return;
    }
    if constexpr (STAGE2) {
        // All tokens of the wavefront's tile exist (every tile but the last of a ragged batch): stores at a per-lane
        // constant offset plus a scalar, no address arithmetic or masks per store; rows beyond M fall outside the
        // buffer's range and are dropped.
        if (col0 + TN * 16 <= p.bvalid && p.ld_out < (1ll << 21) && strip0 * 16 < p.rows_valid) {
            const size_t left = ((size_t)(p.rows_valid - strip0 * 16) * p.ld_out - col0) * 4;
            const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                static_cast<float*>(p.out) + (size_t)strip0 * 16 * p.ld_out + col0, 0, (int)(left < 0xFFFFFFFFull ? left : 0xFFFFFFFFull), 0x00020000);
            const int ld4 = (int)p.ld_out * 4, y_voff = 4 * g * ld4 + i * 4;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[a][b][v] * cs[b]), y_rsrc, y_voff + b * 64, (a * 16 + v) * ld4, 0);
            return;
        }
    }
#pragma unroll
    for (int a = 0; a < TM; ++a) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = (strip0 + a) * 16 + 4 * g + v;
            if constexpr (STAGE2) {
                if (row < p.rows_valid) {
                    float* dst = static_cast<float*>(p.out) + (size_t)row * p.ld_out;
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        const int col = col0 + b * 16 + i;
                        if (col < p.bvalid) dst[col] = acc[a][b][v] * cs[b];
                    }
                }
            } else {
                _Float16* dst = static_cast<_Float16*>(p.out) + (size_t)row * p.ld_out;   // zero S beyond K
#pragma unroll
                for (int b = 0; b < TN; ++b) dst[col0 + b * 16 + i] = (_Float16)((acc[a][b][v] * sr[a][v]) * cs[b]);
            }
        }
    }
}

__device__ __forceinline__ u32x4 buf_load128(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
}
__device__ __forceinline__ uint32_t buf_load32(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
}

// 16 bytes per lane from a buffer straight into LDS at lds_addr + 16 * lane (lds_addr wave-uniform).
// Written as inline assembly on purpose: when the compiler knows about an outstanding
// buffer_load ... lds it waits for ALL vector-memory operations (vmcnt(0)) before every later LDS
// read, which would serialise the prefetch with the MFMAs.  Hidden from it, the only waits are
// the explicit s_waitcnt vmcnt(n) before the barriers below.  M0 (the LDS destination) is a
// reserved register that the compiler re-initialises before each of its own uses.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void buf_load128_to_lds(i32x4 rsrc, uint32_t lds_addr, int voff, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ i32x4 raw_rsrc(const void* base, uint32_t bytes) {
    const uint64_t a = reinterpret_cast<uint64_t>(base);
    return i32x4{(int)(uint32_t)a, (int)(uint32_t)(a >> 32), (int)bytes, 0x00020000};
}

// Epilogue variant of a stage-U launch: 0 plain fp32, 1 fp32 with bias, 2 bf16, 3 token-major output.
int out_variant(const float* bias, int out_bf16, int token_major) {
    return token_major ? 3 : out_bf16 ? 2 : bias ? 1 : 0;
}

int env_cfg(const char* name, int fallback) { return tsvd_tune(name, fallback); }

}  // namespace

// ---- tsvd_fp6.hip, called from tsvd_forward_gemm -----------------------------------------------------------------
hipError_t tsvd_fp6_init();
// x (bf16) or z (fp16) [rows_valid][ld] (token_major: bf16 x [cols_valid][ld]) -> plane records [128-token group][nblocks_per_group][16-token tile]; `blocks`
// 128-index blocks of the source are converted
hipError_t tsvd_fp6_launch_planes(bool bf16, const uint16_t* src, long long ld, int rows_valid, int cols_valid, int nblocks_per_group,
                                  int blocks, long long B, unsigned char* planes, hipStream_t stream, bool token_major = false);
// one stage on fp4 codes x fp6 planes (a.act = the planes); rows_p: padded rows of the stage's weights; ex: output variant (stage U)
hipError_t tsvd_fp6_launch(bool stage2, const gemm_args& a, long long rows_p, int Bp, int ex, long long cus, hipStream_t stream);
// stage V writing the planes of z itself (a.out = those planes, a.ld_out = 128-index blocks per token group), where its tile allows
bool tsvd_fp6_direct_possible(long long rows_p, long long bvalid, long long cus);
hipError_t tsvd_fp6_launch_direct(const gemm_args& a, long long rows_p, long long cus, hipStream_t stream);
// fp32 x [rows_valid][ld] -> two sets of planes (six planes), `blocks` blocks each, layout of 2 * blocks blocks per token group
hipError_t tsvd_fp6_launch_planes_f32(const float* x, long long ld, int rows_valid, int cols_valid, int blocks, unsigned char* planes,
                                      hipStream_t stream);
// the token-panel launch on fp4 codes x fp6 planes
hipError_t tsvd_fp6_launch_panel(const panel_args& pa, int ex, hipStream_t stream);
#endif  // TSVD_GEMM_COMMON_H
