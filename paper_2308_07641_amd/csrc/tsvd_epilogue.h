// Internal: the last step of stage U shared by every kernel family: optional bias (the paper's
// layer listing in the supplement shows its linear layers with bias=True: y = U(S*(Vx)) + b) and
// the choice of the output type (fp32, or bf16 rounded to nearest even from the fp32 result).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// fp32 -> bf16 bit pattern, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint16_t tsvd_bf16_rne(float v) {
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// y[idx] = v as fp32 or bf16 (out_bf16 is uniform over the launch).
__device__ __forceinline__ void tsvd_store_y(void* y, size_t idx, float v, int out_bf16) {
    if (out_bf16) static_cast<uint16_t*>(y)[idx] = tsvd_bf16_rne(v);
    else static_cast<float*>(y)[idx] = v;
}

// bf16 store of two rows of a 16 x 16 result block in the layout of the MFMA result: lane (i, g)
// holds token col16 + i (col16 a multiple of 16) of rows r and r + 1 (values v0, v1).
// Neighbouring lanes swap one value (DPP quad_perm [1,0,3,2]), so that an even lane holds tokens
// (i, i + 1) of row r and the odd lane next to it tokens (i - 1, i) of row r + 1; one packed
// conversion (nearest even) and one 4-byte store per lane then cover both rows with all 64 lanes
// active: half the store instructions of the fp32 form for half the bytes.  aligned4 (uniform):
// the row stride is even and y 4-byte aligned; otherwise the pair is written as two 2-byte stores.
// Must be called by all 16 lanes of a lane group together.
__device__ __forceinline__ void tsvd_store_row_pair_bf16(void* y, long long ld, int r, int rows_valid, int col16, int i,
                                                         int bvalid, float v0, float v1, bool aligned4) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const int odd = i & 1, c = col16 + i - odd;
    const float send = odd ? v0 : v1;
    const float recv = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(send), 0xB1, 0xF, 0xF, true));
    const f32x2_t two = odd ? f32x2_t{recv, v1} : f32x2_t{v0, recv};
    const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2_t));
    const int row = r + odd;
    if (row < rows_valid) {
        uint16_t* dst = static_cast<uint16_t*>(y) + (size_t)row * ld + c;
        if (c + 1 < bvalid) {
            if (aligned4) {
                *reinterpret_cast<uint32_t*>(dst) = pk;
            } else {
                dst[0] = (uint16_t)pk;
                dst[1] = (uint16_t)(pk >> 16);
            }
        } else if (c < bvalid) {
            *dst = (uint16_t)pk;
        }
    }
}

// Token-major output y[token][row]: the lane of a 16 x 16 result block that holds token `token` of rows
// row0 .. row0 + 3 (row0 a multiple of 4) writes them side by side: one 16-byte (fp32) or 8-byte (bf16)
// store when the four rows exist and vec_ok says that ld is a multiple of 4 elements and y is 16-byte
// aligned; element by element otherwise.
__device__ __forceinline__ void tsvd_store_token_major4(void* y, long long ld, int token, int row0, int rows_valid,
                                                        float v0, float v1, float v2, float v3, int out_bf16, bool vec_ok) {
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    const size_t at = (size_t)token * ld + row0;
    if (vec_ok && row0 + 3 < rows_valid) {
        if (out_bf16) {
            const u32x2_t pk = {(uint32_t)tsvd_bf16_rne(v0) | ((uint32_t)tsvd_bf16_rne(v1) << 16),
                                (uint32_t)tsvd_bf16_rne(v2) | ((uint32_t)tsvd_bf16_rne(v3) << 16)};
            *reinterpret_cast<u32x2_t*>(static_cast<uint16_t*>(y) + at) = pk;
        } else {
            *reinterpret_cast<f32x4_t*>(static_cast<float*>(y) + at) = f32x4_t{v0, v1, v2, v3};
        }
        return;
    }
    const float v[4] = {v0, v1, v2, v3};
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (row0 + e < rows_valid) tsvd_store_y(y, at + e, v[e], out_bf16);
}
