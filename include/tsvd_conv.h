/*
 * C ABI of the convolution forms of the ternary SVD (paper, section "TSVD in Convolution Layer").
 *
 * The kernel [C_out, C_in, K1, K2] of a 2-d convolution is reshaped into one of four matrices
 * (Eq. (four_shape)) and that matrix is given as U diag(S) V, packed with tsvd_pack:
 *   form 0: [C_out,           C_in * K1 * K2]   V is a K1 x K2 convolution, U a 1 x 1 convolution
 *   form 1: [C_out * K1 * K2, C_in          ]   V 1 x 1, U K1 x K2
 *   form 2: [C_out * K1,      C_in * K2     ]   V 1 x K2, U K1 x 1
 *   form 3: [C_out * K2,      C_in * K1     ]   V K1 x 1, U 1 x K2
 * (index order inside a product dimension: row-major as written).  Each spatial dimension is
 * handled (kernel extent, stride, padding, dilation) by exactly one of the two factors; diag(S)
 * acts per rank channel in between.  The call gathers the taps of V's kernel into columns
 * (skipped when V is 1 x 1), runs the linear map of tsvd_forward_ex on them and sums the taps of
 * U's kernel (skipped when U is 1 x 1, where bias and output type are fused into the map).
 *
 * Grouped convolutions (groups > 1, form 0 only; the paper's converted network lists its depth-wise
 * 7 x 7 layers as form 0 with groups = channels and rank 5): every group g has its own factors, the
 * packed triple holds them side by side: U [C_out][K] (row co belongs to group co / (C_out / groups)
 * and uses only the ranks [g K / groups, (g + 1) K / groups) of its group; its other entries are not
 * read), S [K], V [K][(C_in / groups) K1 K2] (row k holds the K1 x K2 taps of rank k over the input
 * channels of group k / (K / groups)).  groups must divide C_in, C_out and K.  One direct kernel (no
 * scratch) handles them; limits: at most 8 output channels and 64 ranks per group,
 * (K / groups) * (C_in / groups) K1 K2 <= 4096, and an input window of one workgroup within 64 KB
 * of LDS; beyond them TSVD_EUNSUPPORTED.
 *
 * Activations are feature-major like everywhere in this library: x_dev is bf16
 * [C_in][images][H][W], y_dev is [C_out][images][Ho][Wo] fp32 or bf16, both contiguous, with
 * Ho = (H + 2 pad1 - dil1 (K1 - 1) - 1) / stride1 + 1 and Wo likewise.  Zero padding.
 */
#ifndef TSVD_CONV_H
#define TSVD_CONV_H

#include <stddef.h>
#include <stdint.h>

#include "tsvd.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t form;                 /* 0..3, see above */
    int32_t c_in, c_out, k1, k2;  /* channels and kernel extent */
    int32_t stride1, stride2, pad1, pad2, dil1, dil2;
    int32_t groups;               /* 0 or 1: ordinary convolution; > 1: grouped, see above */
} tsvd_conv_geometry;

/* Scratch needed by tsvd_conv2d_forward for `images` inputs of H x W (0 on invalid arguments or
 * when the packed matrix does not have the shape of the form). */
size_t tsvd_conv2d_workspace_bytes(const tsvd_handle* h, const tsvd_conv_geometry* g, int64_t images, int64_t H, int64_t W);

/* y = conv2d(x; kernel = U diag(S) V in form g->form) + bias.
 *   bias_dev : device fp32 [C_out] or NULL.   y_dtype : TSVD_F32 or TSVD_BF16.
 *   workspace : device, at least tsvd_conv2d_workspace_bytes(...) bytes, 256-byte aligned.
 * Enqueues on stream (hipStream_t as void*) without synchronising.  TSVD_EINVAL for null
 * pointers, non-positive sizes, an empty output or a packed matrix of the wrong shape;
 * TSVD_EUNSUPPORTED for groups > 1 with another form or beyond the limits above. */
tsvd_status tsvd_conv2d_forward(const tsvd_handle* h, const tsvd_conv_geometry* g, const void* x_dev, int64_t images, int64_t H,
                                int64_t W, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype, void* workspace,
                                size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
