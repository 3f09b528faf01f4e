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
// 16 s + i.  Its four 32-bit words d = 0..3 hold 16 codes each: the code at bit 2 j + 16 h
// (j = 0..7, h = 0..1) is the element of column
//      256 T + 32 (2 d + j / 4) + 8 g + 2 (j % 4) + h .
// This is the operand order of v_mfma_f32_16x16x32_{bf16,f16}: for k-step q = 2 d + j / 4
// lane l supplies row i and the 8 contraction indices 8 g + e, e = 2 (j % 4) + h, and
// (word << (14 - 2 j)) & 0xC000C000 turns codes j (low half) and j (high half) into the two
// 16-bit floats of register j % 4 of that step: 0x0000, 0x4000 (+2), 0xC000 (-2) in both
// bf16 and fp16.  The factor 2 per stage is removed exactly by the epilogues.
#pragma once
#include <stdint.h>
#include <stddef.h>

#define TSVD_MAGIC 0x5449423244565354ull /* "TSVD2BIT" little endian */
#define TSVD_FORMAT_VERSION 1u
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

// Bit position of element (row r, column c) inside its tile: returns the lane's 32-bit word
// index (0..255 within the tile) in *word and the bit offset of the 2-bit code.
static inline void tsvd_code_position(int r_in_tile, int c_in_tile, int* word, int* bit) {
    const int i = r_in_tile;            // 0..15
    const int q = c_in_tile >> 5;       // k-step 0..7
    const int g = (c_in_tile >> 3) & 3; // lane group
    const int e = c_in_tile & 7;        // element within the lane's 8
    const int lane = 16 * g + i;
    const int d = q >> 1;
    const int j = 4 * (q & 1) + (e >> 1);
    const int h = e & 1;
    *word = lane * 4 + d;
    *bit = 2 * j + 16 * h;
}
