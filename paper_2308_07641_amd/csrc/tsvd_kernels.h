// Internal: kernel argument blocks and host launchers (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define TSVD_SKINNY_MAX_LDS (150 * 1024)
struct tsvd_blob_header;

// One stage of the skinny path: out = A . in for a packed ternary A and one or two tokens.
#define TSVD_SKINNY_STAGE_V 0   // in: raw activations; out: digit planes of z = S * (V x)
#define TSVD_SKINNY_STAGE_U 1   // in: digit planes of z;  out: y fp32
struct tsvd_skinny_args {
    const void* tiles;      // packed tiles of A: [strips_total][nkt][1 KiB]
    int strips;             // 16-row strips to compute
    int nkt;                // tiles per strip along the contraction index
    int mode;
    const void* in;         // stage V: activations [kvalid][tokens] (row stride ld_in elements)
                            // stage U: fp8 digit planes [8 * tokens][ld_in bytes]
    int in_is_bf16;         // stage V: 1 = bf16 bit patterns, 0 = fp32
    int kvalid;             // stage V: rows of `in` that exist; the rest is taken as zero
    long long ld_in;
    int tokens;             // 1 or 2
    const float* rowscale;  // stage V: S (zero-padded to the strips computed)
    float bound_V;          // stage V: |z| <= bound_V * max|x|
    const int* meta_in;     // stage U: per-token fixed-point exponent of z
    int* meta_out;          // stage V: writes that exponent
    void* out;              // stage V: digit planes [8 * tokens][ld_out bytes]; stage U: fp32 [rows_out][ld_out]
    long long ld_out;
    int rows_out;           // rows of the result that exist
    int slab_tiles;         // contraction tiles staged in LDS at a time
    int sw, kw;             // workgroup = sw strips x kw contraction splits (one wavefront each)
    const float* bias;      // stage U: added per output row, or null
    int out_bf16;           // stage U: out is bf16 [rows_out][ld_out] instead of fp32
    int out_token_major;    // stage U: out is [tokens][ld_out] instead of [rows_out][ld_out]
};

hipError_t tsvd_launch_skinny(const tsvd_skinny_args& a, hipStream_t stream);
hipError_t tsvd_skinny_init();
size_t tsvd_skinny_lds_bytes(int tokens, int slab_tiles, int sw, int kw);

// One stage of the single-token fast path (tsvd_gemv.hip).  Workgroup b owns strips
// [b sw, (b+1) sw) of the stage's matrix; wavefront w works on strip w >> kw_log2 with contraction
// split w & (kw - 1); sw << kw_log2 <= 16.
struct tsvd_gemv_args {
    const void* tiles; int strips, nkt;   // stage V: V, Kp/16 strips, Np/256 tiles; stage U: U, ceil(M/16), Kp/256
    int sw, kw_log2;
    int N, Np, Kp, rows_out;              // rows_out: Kp (stage V, padding rows give z = 0) or M (stage U)
    // stage V
    const void* x; int x_is_bf16; int x_vec; long long ldx;   // x_vec: contiguous and 16-byte aligned
    const float* S; float bound_V;
    unsigned char* planes_out;            // fp8 digit planes of z, [8][Kp]
    // stage U
    const unsigned char* planes_in;
    void* y; long long ldy;               // fp32 (or bf16 with out_bf16) [M][ldy]
    const float* bias; int out_bf16;      // bias per output row or null; output type
    int* meta;                            // fixed-point exponent of z (written by V, read by U)
    int early_tiles;                      // 1: the first tile request goes out with the activation loads (default), 0: after them
    long long* clocks;                    // optional tuning aid: [grid][16] phase timestamps, or null
};
// Both stages of a single token in ONE launch of ONE workgroup, for matrices of at most 64 tiles
// per stage (tsvd_gemv.hip): z never leaves LDS.
struct tsvd_gemv_fused_args {
    const void* tiles_v; int strips_v, nkt_v;     // V: Kp/16 strips, Np/256 tiles
    const void* tiles_u; int strips_u, nkt_u;     // U: ceil(M/16) strips, Kp/256 tiles
    int N, Np, Kp, M;
    const void* x; int x_is_bf16; int x_vec; long long ldx;
    const float* S; float bound_V;
    void* y; long long ldy; const float* bias; int out_bf16;
};
// Both stages of a single token in ONE launch of about one workgroup per compute unit (tsvd_gemv.hip):
// workgroup b computes slice b of z (sw_v strips of V) and rows [b sw_u 16, ...) of y; z crosses
// between workgroups as tagged 64-bit words in zbuf.
struct tsvd_gemv_onepass_args {
    const void* tiles_v; int strips_v, nkt_v, sw_v, kwl_v;   // V: Kp/16 strips, Np/256 tiles; workgroup = sw_v strips x 2^kwl_v splits
    const void* tiles_u; int strips_u, nkt_u, sw_u, kwl_u;   // U: ceil(M/16) strips, Kp/256 tiles
    int grid;                                                // workgroups (<= 256)
    int N, Np, Kp, M;
    const void* x; int x_is_bf16; int x_vec; long long ldx;
    const float* S; float bound_V;
    unsigned long long* zbuf;                                // [Kp] {tag : 32 | fixed-point z : 32}, handle-owned
    unsigned* counter;                                       // tag source, handle-owned
    int spin_limit;                                          // polls for a slice before computing it locally; < 0: never poll
    void* y; long long ldy; const float* bias; int out_bf16;
    long long* clocks;                                       // optional tuning aid: [grid][16] phase timestamps, or null
};
bool tsvd_gemv_onepass_shape(long long M, long long Mp, long long Kp, long long Np, int cus, tsvd_gemv_onepass_args* a);
hipError_t tsvd_launch_gemv_onepass(const tsvd_gemv_onepass_args& a, hipStream_t stream);
// Stage U of a single token on the denser code of U (tsvd_dense.hip): one workgroup per group of five strips.
struct tsvd_gemv_dense_args {
    const void* dense; int groups, nkt;                     // [groups][nkt][4 KiB]; Kp / 256 tile columns
    int Kp, M;
    const unsigned char* planes_in; const int* meta;        // digit planes of z [8][Kp] and their exponent (stage V's output)
    void* y; long long ldy; const float* bias; int out_bf16;
};
size_t tsvd_gemv_dense_lds(long long Kp);
hipError_t tsvd_gemv_dense_init();
hipError_t tsvd_launch_gemv_dense(const tsvd_gemv_dense_args& a, hipStream_t stream);
void tsvd_internal_dense_from_blob(const void* blob, void* out);   // tsvd_pack.cpp: recodes U's tiles of a host blob
bool tsvd_gemv_fused_fits(long long Mp, long long Kp, long long Np);
hipError_t tsvd_launch_gemv_fused(const tsvd_gemv_fused_args& a, hipStream_t stream);
hipError_t tsvd_gemv_init();
bool tsvd_gemv_fits(long long Np, long long Kp);
hipError_t tsvd_launch_gemv(const tsvd_gemv_args& a, bool stage_u, hipStream_t stream);
#define TSVD_GEMV_MAX_GRID 1024

// One stage of the few-token path (tsvd_mid.hip): 2 <= B <= 16 tokens of bf16 activations.
struct tsvd_mid_args {
    const void* tiles; int strips, nkt;   // stage V: V, Kp/16 strips, Np/256 tiles; stage U: U, ceil(M/16), Kp/256
    int sw, kw_log2;                      // workgroup = sw strips x (1 << kw_log2) contraction splits, kw <= 8
    const uint16_t* act;                  // stage V: x bf16 [N][ld]; stage U: z fp16 [Kp][16]
    long long ld;
    int kvalid, bvalid;                   // rows of act that exist (stage V: N), tokens (<= 16)
    unsigned act_bytes;                   // extent of act in bytes (reads beyond it give zero)
    int pairs;                            // gathered path: rows start on 4-byte boundaries (two tokens per load)
    const float* S; float bound_V;        // stage V: row scales (zero beyond K); |z| <= bound_V * max|x|
    float* colmax;                        // [16] per-token max |x| (stage V writes, stage U reads)
    void* out; long long ld_out;          // stage V: z fp16 [Kp][16]; stage U: y fp32 (or bf16) [M][ld_out]
    const float* bias; int out_bf16;      // stage U: bias per output row or null; output type
    int out_token_major;                  // stage U: out is [tokens][ld_out] instead of [M][ld_out]
    int rows_valid;                       // stage U: M
    long long* clocks;                    // optional tuning aid: [grid][16] phase timestamps (stage V 0..7, U 8..15), or null
    int resident_ok;                      // tuning switch: 0 forces the slab hand-over loop for short contractions too
};
hipError_t tsvd_mid_init();
hipError_t tsvd_launch_mid(const tsvd_mid_args& a, bool stage_u, bool vec, hipStream_t stream);

// Device blob of a handle and the host copy of its header (for kernels outside tsvd_api.hip that
// read code words themselves).
struct tsvd_handle;
const uint8_t* tsvd_internal_blob(const tsvd_handle* h, const struct tsvd_blob_header** hd);

hipError_t tsvd_transition_init();   // kernel attributes of tsvd_transition.hip

// ---- batched path ----------------------------------------------------------------------------
struct tsvd_gemm_problem {
    const uint8_t* blob;            // device blob
    const tsvd_blob_header* hd;     // host copy of its header
    float bound_V;                  // |z[k][b]| <= bound_V * max_n |x[n][b]|
    const void* x;                  // device bf16 [N][ldx], or [B][ldx] with x_token_major
    long long B, ldx;
    int x_token_major;              // only where tsvd_gemm_reads_token_major says so
    int x_f32;                      // x is fp32 [N][ldx] (six planes; the fp4 x fp6 kernels)
    void* y;                        // device fp32 (or bf16 with out_bf16) [M][ldy]
    long long ldy;
    const float* bias;              // device [M] added per output row, or null
    int out_bf16;
    int y_token_major;              // y is [B][ldy] (one row per token) instead of [M][ldy]
    void* ws;                       // device workspace (see gemm_workspace in tsvd_api.hip)
    int cu_count;                   // compute units of the device
    long long* clocks;              // optional tuning aid: [TSVD_GEMV_MAX_GRID][16] phase timestamps, or null
};
hipError_t tsvd_gemm_init();
hipError_t tsvd_forward_gemm(const tsvd_gemm_problem& g, hipStream_t stream);
// Tile shape of a batched stage (rows = padded output rows of the stage, Bp = padded tokens):
// 0..3 large-tile kernel (256x256, 256x128, 128x128, 64x128), 14..16 ring kernel.
int tsvd_gemm_tile_shape(long long rows, long long B, long long cus, bool aligned);
// True when a batched call runs as ONE token-panel launch (both stages, z kept in LDS).
bool tsvd_gemm_use_panel(long long Mp, long long Kp, long long Np, long long B, long long cus, bool aligned);
// ... and whether that launch multiplies fp4 codes by fp6 planes (tsvd_panel_fp6_kernel) or 16-bit operands.
bool tsvd_gemm_panel_fp6();
// True when a batched call reads token-major bf16 activations in place (the kernels on fp4 codes x fp6 planes gather
// their operand lanes themselves); other calls get a feature-major copy first.
bool tsvd_gemm_reads_token_major(long long Mp, long long Kp, long long Np, long long B, long long cus);
// Stage U through fp6 planes of Z: whether a call takes it, and the extra workspace it needs after Z.
bool tsvd_gemm_use_fp6(long long Mp, long long Kp, long long Np, long long B, long long cus, bool aligned);
size_t tsvd_gemm_fp6_bytes(long long Kp, long long Bp);
// Stage V through fp6 planes of x (only together with the above; its planes follow those of Z).
bool tsvd_gemm_use_fp6_v(long long Mp, long long Kp, long long Np, long long B, long long cus, bool aligned);
#define TSVD_COLMAX_PARTS 16
// Diagnostic switches (include/tsvd_tuning.h): value set by tsvd_tuning_set in this process, else the
// fallback.  The library never reads the environment.
int tsvd_tune(const char* name, int fallback);
int tsvd_stage_mask();   // stages the current call runs (7 = all; partial only inside tsvd_tuning_forward_stages)
