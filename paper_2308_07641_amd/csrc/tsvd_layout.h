// Internal layout of the packed TSVD blob (host and device share this header; it is not
// part of the public ABI).
//
// Blob = [header 256 B][S: Kp floats][U tiles][V tiles][nnz(U tiles): u16][nnz(V tiles): u16]
// every section 256-byte aligned; Mp, Kp, Np are M, K, N rounded up to multiples of 256.
//
// A ternary matrix A [R][C] (U: R=Mp, C=Kp;  V: R=Kp, C=Np) is cut into tiles of 16 rows x
// 256 columns.  Tile (strip s, column block T) lives at tile index s * (C/256) + T and is
// 1 KiB: 64 lanes x 16 bytes in lane order, so one wavefront reads it with a single fully
// coalesced 16-byte-per-lane load.  Lane l = 16 g + i (i = l % 16, g = l / 16) owns row
// 16 s + i.  The order of the codes inside the lane's four 32-bit words w[0..3] is the A-operand
// order of v_mfma_scale_f32_16x16x128_f8f6f4 with A in fp4 (E2M1):
//   * words w[2h], w[2h+1] serve the MFMA step h (columns 128 h .. 128 h + 127 of the tile);
//   * (w << 2) & 0xCCCCCCCC and w & 0xCCCCCCCC are operand registers 2u and 2u+1 (u = word & 1):
//     code c = 2 n + p of the word becomes nibble n of register 2u + p, and a nibble holding
//     code << 2 is the fp4 number 0 (00), +2 (01) or -2 (11);
//   * operand element e = 8 (2u + p) + n of lane group g multiplies the B row
//         kk = 64 (g & 1) + 32 (e >> 4) + 16 (g >> 1) + (e & 15)
//     of the step (measured on gfx950: with an fp4 A operand the hardware pairs A elements 0..15
//     and 16..31 of lane group g with two different B lane groups).
// The same words feed v_mfma_f32_16x16x32_{bf16,f16} in the batched kernels: there
// (w << (14 - 2 c)) & 0xC000C000 turns codes c and c + 8 into the two 16-bit floats 0x0000,
// 0x4000 (+2), 0xC000 (-2) (same patterns in bf16 and fp16) and the activation rows are fetched
// in the matching order.  The factor 2 per stage is removed exactly by the epilogues.
//
// Position of the rank index.  The order of the rank index k (columns of U, entries of S, rows of V) is free
// (the sum over k does not depend on it), and the format uses that freedom in ONE place: when K is not a
// multiple of 128, the last, partly filled block of 128 rank positions stores its K % 128 valid indices in the
// positions that the first MFMA sub-steps of a 128-step touch.  A sub-step (u, p) of 32 contraction indices
// (word u of the pair, even / odd codes p) covers the positions kk = 64 a + 32 u + 16 b + 8 p + n (a, b in
// {0, 1}, n < 8), so logical offset j = 64 u + 32 p + 16 a + 8 b + n of that block lives at position kk: a
// permutation of four bits of the offset.  With r = K % 128 valid indices only the first ceil(r / 32)
// sub-steps of the last step hold anything but zeros, and the batched kernels skip the others.
// tsvd_rank_position / tsvd_rank_logical are the map and its inverse; every reader of U's columns, S and V's
// rows that starts from a logical rank index goes through them (the packer, the grouped-convolution kernel).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#define TSVD_MAGIC 0x5449423244565354ull /* "TSVD2BIT" little endian */
#define TSVD_FORMAT_VERSION 3u
#define TSVD_TILE_ROWS 16
#define TSVD_TILE_COLS 256
#define TSVD_TILE_BYTES 1024
#define TSVD_DIM_ALIGN 256

struct tsvd_blob_header {
    uint64_t magic;
    uint32_t version;
    uint32_t header_bytes;
    int64_t M, K, N;       // logical dimensions
    int64_t Mp, Kp, Np;    // padded to multiples of 256
    uint64_t off_S, off_U, off_V, off_nnzU, off_nnzV;   // byte offsets from the blob start
    uint64_t total_bytes;
    int64_t nnzU, nnzV;    // sums of the per-tile counts
    uint8_t reserved[256 - 8 - 4 - 4 - 6 * 8 - 6 * 8 - 2 * 8];
};
static_assert(sizeof(tsvd_blob_header) == 256, "header must be 256 bytes");

static inline int64_t tsvd_round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// Physical position of logical rank index k (0 <= k < Kp) for a matrix of rank K, and the inverse.
__host__ __device__ static inline int64_t tsvd_rank_position(int64_t k, int64_t K) {
    if ((K & 127) == 0 || (k >> 7) != (K >> 7)) return k;
    const int j = (int)(k & 127);
    const int kk = (((j >> 4) & 1) << 6) | (((j >> 6) & 1) << 5) | (((j >> 3) & 1) << 4) | (((j >> 5) & 1) << 3) | (j & 7);
    return (k & ~(int64_t)127) | kk;
}
__host__ __device__ static inline int64_t tsvd_rank_logical(int64_t pos, int64_t K) {
    if ((K & 127) == 0 || (pos >> 7) != (K >> 7)) return pos;
    const int kk = (int)(pos & 127);
    const int j = (((kk >> 5) & 1) << 6) | (((kk >> 3) & 1) << 5) | (((kk >> 6) & 1) << 4) | (((kk >> 4) & 1) << 3) | (kk & 7);
    return (pos & ~(int64_t)127) | j;
}

// Column kk (0..127) of an MFMA step  <->  (lane group g, operand element e).
static inline int tsvd_step_column(int g, int e) { return 64 * (g & 1) + 32 * (e >> 4) + 16 * (g >> 1) + (e & 15); }

// Bit position of element (row r, column c) inside its tile: returns the lane's 32-bit word
// index (0..255 within the tile) in *word and the bit offset of the 2-bit code.
__host__ __device__ static inline void tsvd_code_position(int r_in_tile, int c_in_tile, int* word, int* bit) {
    const int i = r_in_tile;                 // 0..15
    const int h = c_in_tile >> 7;            // MFMA step of 128 columns
    const int kk = c_in_tile & 127;
    const int g = ((kk >> 6) & 1) | (((kk >> 4) & 1) << 1);
    const int e = (((kk >> 5) & 1) << 4) | (kk & 15);
    const int v = e >> 3, n = e & 7;         // operand register, nibble
    const int lane = 16 * g + i;
    *word = lane * 4 + 2 * h + (v >> 1);
    *bit = 2 * (2 * n + (v & 1));
}
