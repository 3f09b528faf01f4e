// Convolution forms of the ternary SVD (paper, section "TSVD in Convolution Layer", Eq.
// (four_shape)): V(.) and U(.) are small convolutions, diag(S) a channel-wise product.  The
// contraction itself is the linear map of tsvd_forward_ex on feature-major columns; this file adds
// the two data movements around it: gathering the taps of V's kernel into columns before the map
// (one row per (input channel, tap), one column per position V produces) and summing the taps of
// U's kernel after it.  Both are plain HBM-bound copies with coalesced accesses along the
// innermost image dimension.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "../../include/tsvd_conv.h"
#include "tsvd_epilogue.h"

namespace {

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// Which factor handles which spatial dimension, and the sizes that follow.
struct conv_plan {
    int kv1, kv2, ku1, ku2;        // kernel extents of V and U
    bool v_dim1, v_dim2;           // V handles dimension 1 (rows) / 2 (columns): kernel, stride, padding, dilation
    int Ho, Wo;                    // output size
    int Hv, Wv;                    // positions V produces per image (= what U reads)
    long long rows_v, rows_u;      // N and M of the packed matrix
    long long Bv, Bo;              // columns of the linear map, output positions (all images)
    long long ldx;                 // row stride of the gathered columns (multiple of 8)
};

bool make_plan(const tsvd_conv_geometry& g, int64_t images, int64_t H, int64_t W, conv_plan* p) {
    if (g.form < 0 || g.form > 3 || g.c_in < 1 || g.c_out < 1 || g.k1 < 1 || g.k2 < 1 || g.stride1 < 1 || g.stride2 < 1 ||
        g.pad1 < 0 || g.pad2 < 0 || g.dil1 < 1 || g.dil2 < 1 || images < 1 || H < 1 || W < 1)
        return false;
    const long long ho = ((long long)H + 2LL * g.pad1 - (long long)g.dil1 * (g.k1 - 1) - 1) / g.stride1 + 1;
    const long long wo = ((long long)W + 2LL * g.pad2 - (long long)g.dil2 * (g.k2 - 1) - 1) / g.stride2 + 1;
    if ((long long)H + 2LL * g.pad1 < (long long)g.dil1 * (g.k1 - 1) + 1 || (long long)W + 2LL * g.pad2 < (long long)g.dil2 * (g.k2 - 1) + 1)
        return false;
    p->v_dim1 = g.form == 0 || g.form == 3;
    p->v_dim2 = g.form == 0 || g.form == 2;
    p->kv1 = p->v_dim1 ? g.k1 : 1;
    p->kv2 = p->v_dim2 ? g.k2 : 1;
    p->ku1 = p->v_dim1 ? 1 : g.k1;
    p->ku2 = p->v_dim2 ? 1 : g.k2;
    p->Ho = (int)ho;
    p->Wo = (int)wo;
    p->Hv = p->v_dim1 ? (int)ho : (int)H;
    p->Wv = p->v_dim2 ? (int)wo : (int)W;
    p->rows_v = (long long)g.c_in * p->kv1 * p->kv2;
    p->rows_u = (long long)g.c_out * p->ku1 * p->ku2;
    p->Bv = images * (long long)p->Hv * p->Wv;
    p->Bo = images * ho * wo;
    p->ldx = (p->Bv + 7) / 8 * 8;
    // (grid.y carries the rows of the gather and the output channels of the tap sum)
    return p->Bv < (1LL << 24) && p->Bo < (1LL << 31) && images * H * W < (1LL << 31) && p->rows_v <= 65535 && g.c_out <= 65535;
}

// Columns for V: X[(ci, dy, dx)][(img, py, px)] = x[ci][img][iy][ix] (zero outside the image) with
// iy = py stride1 + dy dil1 - pad1 where V handles dimension 1, else iy = py (dy = 0); ix likewise.
// grid (ceil(ldx / 8 / 256), rows); a thread owns eight consecutive columns (the position is
// decomposed once and stepped along px) and writes them with one 16-byte store; consecutive
// threads walk along px, so the reads stay coalesced up to the stride.
__global__ void __launch_bounds__(256)
tsvd_unfold_kernel(const uint16_t* __restrict__ x, int images, int H, int W, int kv1, int kv2, int Hv, int Wv, int s1, int s2,
                   int p1, int p2, int d1, int d2, int v_dim1, int v_dim2, long long Bv, long long ldx, uint16_t* __restrict__ X) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const long long col0 = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
    if (col0 >= ldx) return;
    const int row = blockIdx.y;
    const int dx = row % kv2, dy = (row / kv2) % kv1, ci = row / (kv1 * kv2);
    int px = (int)(col0 % Wv), py = (int)((col0 / Wv) % Hv), img = (int)(col0 / ((long long)Wv * Hv));
    const uint16_t* xc = x + (size_t)ci * images * H * W;
    uint32_t e[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        uint32_t v = 0;
        if (col0 + t < Bv) {
            const int iy = v_dim1 ? py * s1 + dy * d1 - p1 : py, ix = v_dim2 ? px * s2 + dx * d2 - p2 : px;
            if (iy >= 0 && iy < H && ix >= 0 && ix < W) v = xc[((size_t)img * H + iy) * W + ix];
        }
        e[t] = v;
        if (++px == Wv) {
            px = 0;
            if (++py == Hv) {
                py = 0;
                ++img;
            }
        }
    }
    *reinterpret_cast<u32x4*>(X + (size_t)row * ldx + col0) =
        u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
}

// Taps of U: y[co][img][oy][ox] = bias[co] + sum_{du1, du2} T[(co, du1, du2)][img][ty][tx] with
// ty = oy stride1 + du1 dil1 - pad1 where U handles dimension 1, else ty = oy; tx likewise; taps
// outside the positions V produced contribute nothing (zero padding).
__global__ void __launch_bounds__(256)
tsvd_fold_kernel(const float* __restrict__ T, long long ldt, int images, int Hv, int Wv, int ku1, int ku2, int Ho, int Wo, int s1,
                 int s2, int p1, int p2, int d1, int d2, int u_dim1, int u_dim2, const float* __restrict__ bias, void* __restrict__ y,
                 long long Bo, int out_bf16) {
    const long long col = (long long)blockIdx.x * 256 + threadIdx.x;
    if (col >= Bo) return;
    const int co = blockIdx.y;
    const int ox = (int)(col % Wo), oy = (int)((col / Wo) % Ho), img = (int)(col / ((long long)Wo * Ho));
    float acc = bias ? bias[co] : 0.f;
    for (int a = 0; a < ku1; ++a) {
        const int ty = u_dim1 ? oy * s1 + a * d1 - p1 : oy;
        if (ty < 0 || ty >= Hv) continue;
        for (int b = 0; b < ku2; ++b) {
            const int tx = u_dim2 ? ox * s2 + b * d2 - p2 : ox;
            if (tx < 0 || tx >= Wv) continue;
            acc += T[(size_t)((co * ku1 + a) * ku2 + b) * ldt + ((size_t)img * Hv + ty) * Wv + tx];
        }
    }
    tsvd_store_y(y, (size_t)co * Bo + col, acc, out_bf16);
}

bool shapes_match(const tsvd_handle* h, const conv_plan& p) {
    int64_t M = 0, K = 0, N = 0, a = 0, b = 0;
    return tsvd_info(h, &M, &K, &N, &a, &b) == TSVD_OK && M == p.rows_u && N == p.rows_v;
}

}  // namespace

extern "C" size_t tsvd_conv2d_workspace_bytes(const tsvd_handle* h, const tsvd_conv_geometry* g, int64_t images, int64_t H,
                                              int64_t W) {
    conv_plan p;
    if (!h || !g || !make_plan(*g, images, H, W, &p) || !shapes_match(h, p)) return 0;
    const size_t cols = g->form == 1 ? 0 : round256((size_t)p.rows_v * p.ldx * 2);
    const size_t taps = g->form == 0 ? 0 : round256((size_t)p.rows_u * p.Bv * 4);
    return cols + taps + tsvd_workspace_bytes_ex(h, p.Bv, TSVD_BF16, TSVD_FEATURE_MAJOR);
}

extern "C" tsvd_status tsvd_conv2d_forward(const tsvd_handle* h, const tsvd_conv_geometry* g, const void* x_dev, int64_t images,
                                           int64_t H, int64_t W, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    conv_plan p;
    if (!h || !g || !x_dev || !y_dev || !workspace) return TSVD_EINVAL;
    if (y_dtype != TSVD_F32 && y_dtype != TSVD_BF16) return TSVD_EINVAL;
    if (!make_plan(*g, images, H, W, &p) || !shapes_match(h, p)) return TSVD_EINVAL;
    const size_t need = tsvd_conv2d_workspace_bytes(h, g, images, H, W);
    if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return TSVD_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const bool gather = g->form != 1, taps = g->form != 0;
    const void* X = x_dev;
    long long ldx = p.Bv;
    if (gather) {
        uint16_t* cols = reinterpret_cast<uint16_t*>(ws);
        ws += round256((size_t)p.rows_v * p.ldx * 2);
        hipLaunchKernelGGL(tsvd_unfold_kernel, dim3((unsigned)((p.ldx / 8 + 255) / 256), (unsigned)p.rows_v), dim3(256), 0, s,
                           static_cast<const uint16_t*>(x_dev), (int)images, (int)H, (int)W, p.kv1, p.kv2, p.Hv, p.Wv, g->stride1,
                           g->stride2, g->pad1, g->pad2, g->dil1, g->dil2, (int)p.v_dim1, (int)p.v_dim2, p.Bv, p.ldx, cols);
        if (hipGetLastError() != hipSuccess) return TSVD_EDEVICE;
        X = cols;
        ldx = p.ldx;
    }
    float* T = nullptr;
    if (taps) {
        T = reinterpret_cast<float*>(ws);
        ws += round256((size_t)p.rows_u * p.Bv * 4);
    }
    const size_t map_ws = tsvd_workspace_bytes_ex(h, p.Bv, TSVD_BF16, TSVD_FEATURE_MAJOR);
    // U is 1 x 1: the map writes the result itself, bias and output type fused
    tsvd_status st = taps ? tsvd_forward_ex(h, X, TSVD_BF16, TSVD_FEATURE_MAJOR, p.Bv, ldx, nullptr, T, TSVD_F32, p.Bv, ws, map_ws, s)
                          : tsvd_forward_ex(h, X, TSVD_BF16, TSVD_FEATURE_MAJOR, p.Bv, ldx, bias_dev, y_dev, y_dtype, p.Bv, ws, map_ws, s);
    if (st != TSVD_OK || !taps) return st;
    hipLaunchKernelGGL(tsvd_fold_kernel, dim3((unsigned)((p.Bo + 255) / 256), (unsigned)g->c_out), dim3(256), 0, s, T, p.Bv, (int)images,
                       p.Hv, p.Wv, p.ku1, p.ku2, p.Ho, p.Wo, g->stride1, g->stride2, g->pad1, g->pad2, g->dil1, g->dil2,
                       (int)!p.v_dim1, (int)!p.v_dim2, bias_dev, y_dev, p.Bo, (int)(y_dtype == TSVD_BF16));
    return hipGetLastError() == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
}
