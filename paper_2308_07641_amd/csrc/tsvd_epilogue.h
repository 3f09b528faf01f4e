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
