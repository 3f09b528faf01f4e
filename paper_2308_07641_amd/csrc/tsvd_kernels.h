// Internal: kernel argument blocks and host launchers (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define TSVD_SKINNY_MAX_LDS (150 * 1024)

// out[row][tok] = post * rowscale[row] * sum_k A[row][k] * in[k][tok]   (A entries are +-2, 0
// after decoding, so post carries the factor 1/2).
struct tsvd_skinny_args {
    const void* tiles;      // packed tiles of A: [strips_total][nkt][1 KiB]
    int strips;             // strips to compute = ceil(rows_valid / 16)
    int nkt;                // tiles per strip along the contraction index
    const void* in;         // activations [kvalid][tokens], row stride ld_in elements
    int in_is_bf16;         // 1: bf16 bit patterns, 0: fp32
    int kvalid;             // rows of `in` that exist; the rest is taken as zero
    long long ld_in;
    int tokens;             // tokens in this launch; tokens * pieces <= 16
    int pieces;             // bf16 parts per activation: 1 (bf16 input), 2 or 3 (fp32 input)
    const float* rowscale;  // nullable
    float post;
    float* out;             // [rows_valid][tokens], row stride ld_out
    long long ld_out;
    int rows_valid;
    int slab_tiles;         // contraction tiles staged in LDS at a time
    int sw, kw;             // workgroup = sw strips x kw contraction splits (one wavefront each)
};

hipError_t tsvd_launch_skinny(const tsvd_skinny_args& a, hipStream_t stream);

// Per-device one-time setup of kernel attributes (dynamic LDS limits).
hipError_t tsvd_skinny_init();

// ---- batched path ----------------------------------------------------------------------------
struct tsvd_blob_header;
struct tsvd_gemm_problem {
    const uint8_t* blob;            // device blob
    const tsvd_blob_header* hd;     // host copy of its header
    float bound_V;                  // |z[k][b]| <= bound_V * max_n |x[n][b]|
    const void* x;                  // device bf16 [N][ldx]
    long long B, ldx;
    float* y;                       // device fp32 [M][ldy]
    long long ldy;
    void* ws;                       // device workspace (see gemm_workspace in tsvd_api.hip)
};
hipError_t tsvd_gemm_init();
hipError_t tsvd_forward_gemm(const tsvd_gemm_problem& g, hipStream_t stream);
#define TSVD_COLMAX_PARTS 16
