/*
 * tsvd_tuning.h -- diagnostic interface of libtsvd.so for its test-suite and its benchmark.
 *
 * Not part of the product ABI (include/tsvd.h).  The library never reads the environment: every
 * kernel-selection rule has a compiled-in default, and the switches below override a rule only after
 * an explicit call in this process.  They exist so that small test instances can reach every kernel
 * family and tile shape, and so that the benchmark can time one stage of a call alone.  The table is
 * process-global and not thread-safe: set it while no other thread is inside the library.
 */
#ifndef TSVD_TUNING_H
#define TSVD_TUNING_H

#include "tsvd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Overrides one selection rule.  Names (values):
 *   TSVD_GEMV (0: single-token calls take the general slab kernel), TSVD_GEMV_FUSED (0: small single-token
 *   problems take two launches), TSVD_GEMV_ONEPASS (0: single-token calls take one launch per stage),
 *   TSVD_GEMV_SW / TSVD_GEMV_KWLOG2, TSVD_SKINNY_SW / TSVD_SKINNY_KW (workgroup shapes),
 *   TSVD_MID (0: few-token kernel off), TSVD_MID_MAX_B, TSVD_MID_SW, TSVD_MID_KWLOG2, TSVD_MID_RESIDENT,
 *   TSVD_GEMM_MIN_B, TSVD_GEMM_CFG_V / TSVD_GEMM_CFG_U (tile shape of a batched stage: 0..3 large tiles,
 *   14..17 ring kernel), TSVD_FUSEMAX, TSVD_COLMAX_SCALAR, TSVD_REALIGN, TSVD_PANEL, TSVD_PANEL_WAVES,
 *   TSVD_GEMM_MIN_B_F32 (fewest tokens of fp32 activations that take the batched kernels, default 17),
 *   TSVD_PANEL_FP6 (0: the token-panel launch on 16-bit operands instead of fp4 codes x fp6 planes),
 *   TSVD_FP6, TSVD_FP6_V, TSVD_FP6_TALL, TSVD_FP6_PLANES (2: two instead of three fp6 planes -- about five
 *   times the error, inside the tolerance without margin; never a default), TSVD_FP6_DIRECT (0: the fp4 x fp6
 *   stage V always writes fp16 z for a separate pass to turn into planes), TSVD_FP6_TAIL (0: no narrower tiles in the
 *   last round of a launch of 512 x 64 tiles), TSVD_TOKEN_MAJOR_COPY (1: token-major
 *   activations are always copied to feature-major rows first, also for the kernels that can read them in place),
 *   TSVD_GROUPED_PAIR,
 *   TSVD_CLOCKS (1 at tsvd_pack: record phase timestamps per workgroup), TSVD_SPIN_LIMIT (bound of the
 *   single-launch kernels' wait for another workgroup's slice of z, in polls), TSVD_DENSE_U (1 at tsvd_pack: keep a
 *   second copy of U in the five-elements-per-byte code and run stage U of single-token calls on it),
 *   TSVD_EARLY_TILES (0: the single-token kernels request their first weight tile only after the activations are in).
 * Returns 0, or 1 for an unknown name. */
int tsvd_tuning_set(const char* name, int value);

/* Back to the compiled-in rules. */
void tsvd_tuning_reset(void);

/* tsvd_forward_ex restricted to some kernels of the call: stage_mask is a bit set of 1 (column maxima /
 * operand planes of x), 2 (stage V), 4 (stage U); 7 is the whole call.  With a partial mask y (or z) is
 * NOT the result of the map: this is for timing one stage on the z an earlier full call left in the
 * workspace, which is why the public entry points cannot be given a mask. */
tsvd_status tsvd_tuning_forward_stages(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                                       int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                                       int64_t ldy, void* workspace, size_t workspace_bytes, void* stream, int stage_mask);

/* The tile shapes tsvd_forward picks for B tokens of 16-byte-aligned bf16 activations (stage V, stage U):
 * 0..3 / 14..17 as above, 32 / 33 for both when the call is one token-panel launch (16-bit operands / fp4 codes x fp6 planes), 40 for the
 * fp4 x fp6 kernels of the two-launch path,
 * -1 where the batched kernels are not used.  Returns 0 on success. */
int tsvd_tuning_tile_shapes(const tsvd_handle* h, long long B, int* shape_v, int* shape_u);

/* Copies the phase timestamps ([workgroups][16] 100 MHz ticks) of the last launch of a handle packed with
 * TSVD_CLOCKS = 1 to the host.  Returns 0 on success. */
int tsvd_tuning_read_clocks(const tsvd_handle* h, long long* out, int workgroups);

#ifdef __cplusplus
}
#endif
#endif /* TSVD_TUNING_H */
