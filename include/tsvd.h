/*
 * tsvd.h -- C ABI of the MI355X (gfx950) Ternary-SVD forward library.
 *
 * The operation (paper, section "Truncated SVD in Network Compression": a
 * linear layer y = W x with W [M,N] is evaluated as y ~= U (diag(S) (V x));
 * section "Ternary SVD": U [M,K] and V [K,N] hold only -1, 0, +1 and S [K] is
 * a real scale vector, so V(.) and U(.) need additions only and diag(S)(.)
 * needs K multiplications -- supplement Table S1).  The rank K is not assumed
 * small: K > min(M,N) is allowed.  There is no bias term (Eq. 1).
 *
 * All functions are plain C, never throw, and report failure through
 * tsvd_status; on failure outputs are left untouched.  "host" and "device"
 * below say where a pointer must live.  Nothing in the signatures is a torch
 * type: a stream is a hipStream_t passed as void*.
 */
#ifndef TSVD_H
#define TSVD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tsvd_handle tsvd_handle; /* opaque; owns or borrows the packed device blob */

typedef enum {
    TSVD_OK = 0,
    TSVD_EINVAL = 1,       /* null pointer, non-positive size, bad leading dimension, short buffer */
    TSVD_EVALUE = 2,       /* an entry of U or V is not -1, 0 or +1 (or a packed code is corrupt)  */
    TSVD_ENOMEM = 3,       /* host allocation failed                                               */
    TSVD_EDEVICE = 4,      /* a HIP call failed (no device, out of device memory, launch error)    */
    TSVD_EUNSUPPORTED = 5, /* valid request this build does not implement                          */
    TSVD_ETOOLARGE = 6     /* tsvd_forward_noalloc: the call needs more than TSVD_NOALLOC_MAX_WORKSPACE */
} tsvd_status;

typedef enum { TSVD_F32 = 0, TSVD_BF16 = 1 } tsvd_dtype;
/* Layout of the activations: feature-major x[n][b] (the paper's column vectors side by side) or
 * token-major x[b][n] (one row per token). */
typedef enum { TSVD_FEATURE_MAJOR = 0, TSVD_TOKEN_MAJOR = 1 } tsvd_layout;

/* ---- packing: the 2-bit ternary weight format ------------------------------------------
 *
 * The paper only says that a ternary element needs 2 bits (section "Connection with BNN").
 * This library's code is  bit0 = "non-zero", bit1 = "negative":  00 -> 0, 01 -> +1,
 * 11 -> -1; 10 is never produced and is rejected when read back.  That is the U = U+ - U-
 * bit-plane view of the same section (bit0 = U+ | U-, bit1 = U-).  Codes are stored in
 * 1 KiB tiles of 16 rows x 256 columns ordered for 128-byte-coalesced wavefront reads,
 * with one non-zero count per tile; dimensions are zero-padded to multiples of 256
 * (padding adds nothing to y and nothing to the counts).  The sum of the tile counts is
 * nnz(U) + nnz(V), the per-token addition count r K (M+N) of supplement Table S1.
 */

/* Size in bytes of the packed blob for given dimensions (0 if a dimension is <= 0). */
size_t tsvd_packed_bytes(int64_t M, int64_t K, int64_t N);

/* Pack on the host into host memory (no GPU needed).
 *   U: host int8 [M][K] row-major, V: host int8 [K][N] row-major, S: host float [K].
 *   blob: host buffer of at least tsvd_packed_bytes(M,K,N) bytes; fully overwritten.
 * Returns TSVD_EVALUE if U or V holds anything but -1, 0, +1. */
tsvd_status tsvd_pack_host(const int8_t* U, const float* S, const int8_t* V,
                           int64_t M, int64_t K, int64_t N, void* blob, size_t blob_bytes);

/* Exact inverse of tsvd_pack_host.  Any of U, S, V may be NULL (skipped); each of M, K, N
 * may be NULL.  With U, S and V all NULL only the dimensions are returned. */
tsvd_status tsvd_unpack_host(const void* blob, size_t blob_bytes, int8_t* U, float* S, int8_t* V,
                             int64_t* M, int64_t* K, int64_t* N);

/* Pack and upload.  U, S, V as for tsvd_pack_host (caller keeps ownership).
 *   dev_buf == NULL : the library hipMallocs the blob and tsvd_free releases it.
 *   dev_buf != NULL : caller-owned device memory (e.g. a torch uint8 tensor) of
 *                     dev_buf_bytes >= tsvd_packed_bytes(M,K,N), 256-byte aligned; it must
 *                     outlive the handle and is not freed by tsvd_free.
 * Uses the current HIP device; synchronous.  *out is written only on success. */
tsvd_status tsvd_pack(const int8_t* U, const float* S, const int8_t* V,
                      int64_t M, int64_t K, int64_t N,
                      void* dev_buf, size_t dev_buf_bytes, tsvd_handle** out);

/* Download and unpack (bit-exact inverse of tsvd_pack); host outputs, any may be NULL. */
tsvd_status tsvd_unpack(const tsvd_handle* h, int8_t* U, float* S, int8_t* V);

/* Dimensions and the sums of the per-tile non-zero counts; any output may be NULL. */
tsvd_status tsvd_info(const tsvd_handle* h, int64_t* M, int64_t* K, int64_t* N,
                      int64_t* nnzU, int64_t* nnzV);

/* ---- a denser code of U (measurement path) ----------------------------------------------
 *
 * The paper's discussion calls 2 bits per ternary element overly redundant.  These calls hold the densest
 * byte-aligned alternative: five elements per byte (3^5 = 243 <= 256), 1.6 bits per element, in groups of five
 * 16-row strips (4 KiB per group and 256 columns: lane-ordered like the 2-bit tiles, byte j of a lane =
 * sum_i trit(5 j + i) 3^i over the lane's 320 codes of the five strips, trit 0 / 1 / 2 for 0 / +1 / -1).  The
 * forward path uses it only when asked to (diagnostic switch TSVD_DENSE_U of tsvd_tuning.h at tsvd_pack:
 * stage U of single-token calls then reads this code): on MI355X it reads 20 % fewer bytes and is slower,
 * because decoding costs more than the bytes save.
 *   tsvd_dense_bytes(M, K)      : size of the code of U [M][K] (0 if a dimension is <= 0)
 *   tsvd_dense_pack_host        : U host int8 [M][K] row-major -> blob (host); TSVD_EVALUE for non-ternary entries
 *   tsvd_dense_unpack_host      : exact inverse; TSVD_EVALUE for a byte above 242 or a non-empty padding row
 */
size_t tsvd_dense_bytes(int64_t M, int64_t K);
tsvd_status tsvd_dense_pack_host(const int8_t* U, int64_t M, int64_t K, void* blob, size_t blob_bytes);
tsvd_status tsvd_dense_unpack_host(const void* blob, size_t blob_bytes, int8_t* U, int64_t M, int64_t K);

/* ---- forward ------------------------------------------------------------------------
 *
 * Y = U (diag(S) (V X)) for B tokens (columns), following the three steps of the paper's
 * identity: t = V x (additions), z = S * t (the K multiplications), y = U z (additions).
 *
 *   x_dev : device, [N][B] row-major with row stride ldx >= B elements of x_dtype.  Any stride and
 *           alignment is accepted; bf16 rows that start on 16-byte boundaries (ldx a multiple of 8, base
 *           16-byte aligned) are read in place, others are first copied to such rows inside the
 *           workspace when B > 16 (one extra pass over x).
 *   y_dev : device, [M][B] row-major with row stride ldy >= B elements of y_dtype (TSVD_F32, or
 *           TSVD_BF16: the fp32 result rounded to nearest even).
 *   workspace : device scratch for the intermediate z, at least
 *               tsvd_workspace_bytes(h, B, x_dtype) bytes, 256-byte aligned; contents
 *               are undefined afterwards.  NULL (with workspace_bytes 0) makes the library
 *               use scratch owned by the handle, grown with hipMalloc when needed; such
 *               calls on one handle must not overlap each other.
 *   stream : hipStream_t as void* (NULL = the default stream).  Work is enqueued and the
 *            call returns without synchronising.
 * x, y and workspace are owned by the caller and must not alias.  Inputs must be finite.
 *
 * Arithmetic (accumulation is fp32 or exact everywhere; the oracle-relative bounds are those the tests check):
 *   B = 1 (and TSVD_F32 activations with 2 <= B <= 16, which are handled one token at a time, each pass streaming
 *     the weights again): x is converted to sign-magnitude fixed point with 30 bits below the largest |x| (entries below
 *     2^-31 of it become 0), every sum of V(.) and U(.) is then an exact integer; z = S * (V x) is rounded to fp32
 *     and converted the same way relative to the bound max_k |S_k| nnz(V[k,:]) * max|x|.  Error: 1e-5 of max|y| at
 *     most (measured 1e-7 .. 8e-7).
 *   2 <= B (TSVD_BF16): x enters exactly, stage V accumulates exact products in fp32, z is multiplied by a
 *     per-token power of two that keeps it in range and rounded to fp16 (11 significant bits), stage U accumulates
 *     exact products in fp32.  Long contractions with many tiles, and calls with many tokens on a small
 *     factorisation (one launch for both stages), multiply fp4 codes by three fp6 (E2M3) planes of the
 *     activations with block scales, which resolve 2^-14.7 of the largest magnitude among 32 neighbours; where
 *     stage V makes the planes of z itself, z is never rounded to 16 bits.  Error: 2e-3 of max|y| at most
 *     (measured 2.0e-4 .. 2.4e-4 with fp16 z, 2e-5 .. 4e-5 without).
 *   17 <= B (TSVD_F32): fp4 codes times SIX fp6 planes of the activations of either stage (three, and three more for
 *     what those leave: below the last bit of an fp32 value of a block's largest magnitude), fp32 accumulation; z goes
 *     from the accumulators straight into its planes.  Error: 1e-5 of max|y| at most (measured 2e-7 .. 1.4e-6).
 * Limits of the batched kernels (32-bit buffer offsets): N * ldx, Kp * (B rounded up to 256), Mp * Kp / 8 and
 * Kp * Np / 8 must each be below 2^30; larger calls return TSVD_EUNSUPPORTED (split the tokens).  B <= 2^24.
 * A single-token call may also be enqueued on several streams at once with separate workspaces.
 */
size_t tsvd_workspace_bytes(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype);

tsvd_status tsvd_forward(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype,
                         int64_t B, int64_t ldx, void* y_dev, tsvd_dtype y_dtype, int64_t ldy,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ---- forward with the options of a linear layer -----------------------------------------
 *
 * Y = U (diag(S) (V X)) + bias: the same three steps, then the bias of the layer (the paper's
 * listing of a converted network in the supplement shows its ternary-SVD linear layers with
 * bias=True) added to every token, fused into the last kernel of the call.
 *
 *   x_layout : TSVD_FEATURE_MAJOR: x_dev is [N][B], ldx >= B (as tsvd_forward);
 *              TSVD_TOKEN_MAJOR:   x_dev is [B][N], ldx >= N.  Batched bf16 calls that run on fp4 codes x fp6
 *              planes (many tokens on a small factorisation; long contractions with many tiles) read it in place;
 *              other calls first rewrite it feature-major into the workspace (one extra pass over x).
 *   bias_dev : device fp32 [M], or NULL for none.
 *   y_dev    : [M][B] with row stride ldy >= B, TSVD_F32 or TSVD_BF16 (rounded to nearest even
 *              from the fp32 value after the bias).
 *   workspace: at least tsvd_workspace_bytes_ex(h, B, x_dtype, x_layout) bytes, 256-byte aligned,
 *              or NULL (with workspace_bytes 0) for scratch owned by the handle.
 * Everything else (ownership, stream, errors, arithmetic) is as for tsvd_forward, which is this
 * call with a feature-major x and no bias.
 */
size_t tsvd_workspace_bytes_ex(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype, tsvd_layout x_layout);

tsvd_status tsvd_forward_ex(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                            int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                            int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* ---- forward with a choice of both layouts -------------------------------------------------
 *
 * tsvd_forward_ex with the layout of y chosen as well:
 *   y_layout : TSVD_FEATURE_MAJOR: y_dev is [M][B], ldy >= B (as above);
 *              TSVD_TOKEN_MAJOR:   y_dev is [B][M], ldy >= M: one row per token, what a following
 *              token-major layer reads.  It is written in place by the last kernel of the call (each
 *              lane of a result block stores four consecutive rows of one token: 16-byte stores when
 *              ldy is a multiple of 4 and y_dev is 16-byte aligned), not by a transposition pass.
 * Everything else is as for tsvd_forward_ex, which is this call with a feature-major y.
 */
tsvd_status tsvd_forward_io(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                            int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                            tsvd_layout y_layout, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* ---- forward for callers that cannot allocate -------------------------------------------
 *
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc:
 * tsvd_forward_ex with the intermediate z (and the re-laid-out copy of x, where one is made) in a
 * fixed array of TSVD_NOALLOC_MAX_WORKSPACE bytes that the loaded library holds on every GPU it has
 * been used on, until the process ends.  The call allocates and frees nothing, on the host or on the
 * device, and takes no workspace argument; x, bias and y are the caller's as before.
 *   - Returns TSVD_ETOOLARGE (nothing enqueued, y untouched) when
 *     tsvd_workspace_bytes_ex(h, B, x_dtype, x_layout) exceeds TSVD_NOALLOC_MAX_WORKSPACE
 *     (16 MiB: any single-token or few-token call, and batched calls whose fp16 z [K][B rounded up to
 *     256] plus a copy of x fit, e.g. 512 tokens at K = 1536, N = 768 need 2.4 MB).
 *     An fp32 batch whose six planes of x and z do not fit is not rejected: it goes one token at a time, as fp32
 *     batches below 17 tokens do.
 *   - All calls on one GPU share that GPU's array, whatever the handle or stream: calls that
 *     overlap in time on one GPU race on z and give wrong results.  Order them on one stream (or with
 *     events).  The array keeps the previous call's contents; no kernel depends on them.
 *   - h must have been packed on the GPU the call runs on (tsvd_pack looks up that GPU's array).
 * Everything else is as for tsvd_forward_ex.
 */
#define TSVD_NOALLOC_MAX_WORKSPACE (16u << 20)
tsvd_status tsvd_forward_noalloc(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                                 int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                                 int64_t ldy, void* stream);

/* Releases the handle and whatever device memory it owns.  NULL is allowed. */
void tsvd_free(tsvd_handle* h);

/* Static description of a status code. */
const char* tsvd_strerror(tsvd_status s);

#ifdef __cplusplus
}
#endif
#endif /* TSVD_H */
