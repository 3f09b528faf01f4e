// Convolution forms of the ternary SVD (paper, section "TSVD in Convolution Layer", Eq.
// (four_shape)): V(.) and U(.) are small convolutions, diag(S) a channel-wise product.  The
// contraction itself is the linear map of tsvd_forward_ex on feature-major columns; this file adds
// the two data movements around it: gathering the taps of V's kernel into columns before the map
// (one row per (input channel, tap), one column per position V produces) and summing the taps of
// U's kernel after it.  Both are plain HBM-bound copies with coalesced accesses along the
// innermost image dimension.
//
// Grouped convolutions (form 0 with groups; the paper's converted ConvNeXt lists its depth-wise
// 7 x 7 layers this way, rank 5 per channel) have per-group factors of a few hundred codes: a
// matrix-core map would multiply zeros almost everywhere.  tsvd_grouped_conv_kernel does the three
// steps directly: the window of the group's input channels is staged in LDS, V_g is turned into a
// list of its non-zero taps per rank, and every output position adds / subtracts the listed values
// (the additions of the method, zeros skipped), multiplies by S and combines the ranks with the
// signs of U: x is read once and y written once, z stays in registers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdlib>

#include "../../include/tsvd_conv.h"
#include "tsvd_epilogue.h"
#include "tsvd_kernels.h"
#include "tsvd_layout.h"

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
    bool fits;                     // within the index limits of the gather / map / tap-sum path
};

bool make_plan(const tsvd_conv_geometry& g, int64_t images, int64_t H, int64_t W, conv_plan* p) {
    if (g.groups < 0 || g.form < 0 || g.form > 3 || g.c_in < 1 || g.c_out < 1 || g.k1 < 1 || g.k2 < 1 || g.stride1 < 1 || g.stride2 < 1 ||
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
    p->fits = p->Bv < (1LL << 24) && p->Bo < (1LL << 31) && images * H * W < (1LL << 31) && p->rows_v <= 65535 && g.c_out <= 65535;
    return true;
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


// ---- grouped form 0 ------------------------------------------------------------------------------
#define GROUPED_MAX_MG 8            // output channels per group
#define GROUPED_MAX_KG 64           // ranks per group
#define GROUPED_MAX_ENTRIES 4096    // ranks per group x (taps per group rounded up to 4)
#define GROUPED_MAX_LDS (64 * 1024)

struct grouped_args {
    const uint32_t* U; int u_tps;        // code words of U, tiles per 16-row strip (Kp / 256)
    const uint32_t* V; int v_tps;        // code words of V, tiles per strip (Np / 256)
    const float* S;
    int K;                               // rank of the packed triple (positions of the rank index: tsvd_rank_position)
    const uint16_t* x; void* y; const float* bias; int out_bf16;
    int cg, mg, kg, ng;                  // per group: input channels, output channels, ranks, taps (cg k1 k2)
    int images, H, W, Ho, Wo, k1, k2, s1, s2, p1, p2, d1, d2;
    int rb, bpp;                         // output rows per workgroup, workgroups per plane
    int ipb;                             // images per workgroup (the tap lists are built once per workgroup)
    int rows_in, win;                    // staged window per input channel: rows, columns
};

// 2-bit code of element (r, c) of a packed matrix with tps tiles per strip.
__device__ __forceinline__ int code_at(const uint32_t* words, int tps, int r, int c) {
    int word, bit;
    tsvd_code_position(r & 15, c & 255, &word, &bit);
    return (int)(words[((size_t)(r >> 4) * tps + (c >> 8)) * 256 + word] >> bit) & 3;
}

// grid (bpp * ceil(images / ipb), groups), block 64..256.  Workgroup = group g, output rows
// [r0, r0 + rb) of ipb images, one after the other.  A thread owns ROWS vertically adjacent
// positions (ROWS = 4 needs stride1 = 1 and a compile-time row pitch P of the window: the four
// values of a tap are then one address plus constant offsets); consecutive lanes own consecutive
// columns, so every LDS read of a wavefront touches consecutive words (a thread owning four
// horizontally adjacent positions made lanes 16 words apart: four-way bank conflicts, 3 x slower).
// LDS: window [cg][rows_in][pitch] fp32, tap lists [kg][stride] as offsets into the window and signs
// +-1.0 (padded to a multiple of four with sign 0), their lengths, the signs of U [MG][kg] as
// +-1 / 0, S [kg], and for the prologue the codes of V_g.
// PAIR (stride1 = stride2 = 1, ROWS = 4): the window keeps the activations as they come, bf16, in
// two copies per row: words (x[2w], x[2w+1]) and words (x[2w+1], x[2w+2]); a thread owns 4 rows x 2
// adjacent columns and one 32-bit read gives it both values of a tap, whatever its column offset
// (even offsets in the first copy, odd ones in the second).  v_dot2c_f32_bf16 with the sign pairs
// (+-1, 0) and (0, +-1) adds each half to its position's fp32 sum: half the LDS bytes per tap, the
// same one instruction per position and tap.
template <int MG, int ROWS, int P, bool PAIR>
__global__ void __launch_bounds__(256)
tsvd_grouped_conv_kernel(grouped_args p) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    static_assert(!PAIR || (ROWS == 4 && P >= 64), "the paired form owns 4 rows and needs a compile-time pitch");
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int pitch = P ? P : p.win;
    const int tile_elems = p.cg * p.rows_in * pitch, stride = (p.ng + 3) & ~3;
    float* tile = reinterpret_cast<float*>(smem);
    int* offs = reinterpret_cast<int*>(tile + ((tile_elems + 3) & ~3));
    float* sgns = reinterpret_cast<float*>(offs + p.kg * stride);
    int* counts = reinterpret_cast<int*>(sgns + p.kg * stride);
    float* ucode = reinterpret_cast<float*>(counts + ((p.kg + 3) & ~3));
    float* sval = ucode + MG * p.kg;
    unsigned char* codes = reinterpret_cast<unsigned char*>(sval + p.kg);      // [kg][stride], prologue only
    const int g = blockIdx.y;
    const int rblk = blockIdx.x % p.bpp, iblk = blockIdx.x / p.bpp;
    const int r0 = rblk * p.rb, nrows = min(p.rb, p.Ho - r0);

    // ---- the codes of V_g, all loads in flight at once, then per rank (one wavefront each) the list of its non-zero taps
    for (int idx = threadIdx.x; idx < p.kg * p.ng; idx += blockDim.x) {
        const int k = idx / p.ng, j = idx - k * p.ng;
        codes[k * stride + j] = (unsigned char)code_at(p.V, p.v_tps, (int)tsvd_rank_position(g * p.kg + k, p.K), j);
    }
    for (int idx = threadIdx.x; idx < MG * p.kg; idx += blockDim.x) {
        const int m = idx / p.kg, k = idx % p.kg;
        const int code = m < p.mg ? code_at(p.U, p.u_tps, g * p.mg + m, (int)tsvd_rank_position(g * p.kg + k, p.K)) : 0;
        ucode[idx] = code == 1 ? 1.f : code == 3 ? -1.f : 0.f;
    }
    for (int k = threadIdx.x; k < p.kg; k += blockDim.x) sval[k] = p.S[tsvd_rank_position(g * p.kg + k, p.K)];
    __syncthreads();
    for (int k = wave; k < p.kg; k += nwaves) {
        int cnt = 0;
        for (int j0 = 0; j0 < p.ng; j0 += 64) {
            const int j = j0 + lane;
            const int code = j < p.ng ? codes[k * stride + j] : 0;
            const unsigned long long mask = __ballot(code & 1);
            if (code & 1) {
                const int dx = j % p.k2, dy = (j / p.k2) % p.k1, c = j / (p.k1 * p.k2);
                const int at = k * stride + cnt + __popcll(mask & ((1ull << lane) - 1));
                if constexpr (PAIR) {
                    const int dxd = dx * p.d2;
                    offs[at] = (c * p.rows_in + dy * p.d1) * P + (dxd & 1) * (P / 2) + (dxd >> 1);
                    sgns[at] = __uint_as_float(code == 3 ? 0xBF80u : 0x3F80u);        // bf16 -1 / +1 in the low half
                } else {
                    offs[at] = (c * p.rows_in + dy * p.d1) * pitch + dx * p.d2;
                    sgns[at] = code == 3 ? -1.f : 1.f;
                }
            }
            cnt += __popcll(mask);
        }
        const int padded = (cnt + 3) & ~3;                 // <= stride
        if (lane < padded - cnt) {
            offs[k * stride + cnt + lane] = 0;             // a tap of weight zero at the position itself
            sgns[k * stride + cnt + lane] = 0.f;
        }
        if (lane == 0) counts[k] = padded;
    }

    const int iy0 = r0 * p.s1 - p.p1;
    const int wcols = PAIR ? (p.Wo + 1) / 2 : p.Wo;         // units per row of units
    const int units = ((nrows + ROWS - 1) / ROWS) * wcols;  // a unit = ROWS rows x one column (PAIR: two columns)
    const size_t plane_in = (size_t)p.H * p.W, plane_out = (size_t)p.Ho * p.Wo;
    for (int img = iblk * p.ipb; img < min((iblk + 1) * p.ipb, p.images); ++img) {
        __syncthreads();            // lists complete / the previous image's window is no longer read
        // ---- window of the group's input channels, zero outside the image: 16 rows per wavefront in
        // flight at a time (unconditional loads from clamped addresses, so that none waits for another)
        const int nrow_tot = p.cg * p.rows_in;
        for (int row0 = wave * 16; row0 < nrow_tot; row0 += nwaves * 16) {
            for (int cc = lane; cc < p.win + (PAIR ? 1 : 0); cc += 64) {      // PAIR: one more column for a ragged last pair
                const int ix = cc - p.p2, ixc = min(max(ix, 0), p.W - 1);
                uint32_t raw[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = min(row0 + r, nrow_tot - 1), c = row / p.rows_in;
                    const int iyc = min(max(iy0 + row - c * p.rows_in, 0), p.H - 1);
                    raw[r] = p.x[((size_t)(g * p.cg + c) * p.images + img) * plane_in + (size_t)iyc * p.W + ixc];
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = row0 + r, c = row / p.rows_in, iy = iy0 + row - c * p.rows_in;
                    const uint32_t v = iy >= 0 && iy < p.H && ix == ixc ? raw[r] : 0u;
                    if constexpr (PAIR) {
                        uint16_t* row16 = reinterpret_cast<uint16_t*>(tile + row * P);
                        if (row < nrow_tot) {
                            row16[cc] = (uint16_t)v;                       // copy of even offsets
                            if (cc > 0) row16[P + cc - 1] = (uint16_t)v;   // copy of odd offsets, one element to the left
                        }
                    } else {
                        if (row < nrow_tot) tile[row * pitch + cc] = __uint_as_float(v << 16);
                    }
                }
            }
        }
        __syncthreads();
        // ---- per output position: t_k = sum of the listed taps, z_k = S_k t_k, y_m = sum_k U[m][k] z_k
        for (int u = threadIdx.x; u < units; u += blockDim.x) {
            constexpr int COLS = PAIR ? 2 : 1;
            const int q = u / wcols, oc = u - q * wcols, ox = oc * COLS, oy0 = q * ROWS;
            const float* base = tile + (oy0 * p.s1) * pitch + (PAIR ? oc : ox * p.s2);
            float acc[MG][ROWS][COLS];
#pragma unroll
            for (int m = 0; m < MG; ++m)
#pragma unroll
                for (int j = 0; j < ROWS; ++j)
#pragma unroll
                    for (int c = 0; c < COLS; ++c) acc[m][j][c] = 0.f;
            for (int k = 0; k < p.kg; ++k) {
                const int cnt = counts[k];
                const int* eo = offs + k * stride;
                const float* es = sgns + k * stride;
                float t[ROWS][COLS];
#pragma unroll
                for (int j = 0; j < ROWS; ++j)
#pragma unroll
                    for (int c = 0; c < COLS; ++c) t[j][c] = 0.f;
                auto tap = [&](int off, float sg) {
                    if constexpr (PAIR) {
                        const uint32_t slo = __float_as_uint(sg), shi = slo << 16;
#pragma unroll
                        for (int j = 0; j < ROWS; ++j) {
                            const bf16x2 v = __builtin_bit_cast(bf16x2, __float_as_uint(base[off + j * P]));
                            t[j][0] = __builtin_amdgcn_fdot2_f32_bf16(v, __builtin_bit_cast(bf16x2, slo), t[j][0], false);
                            t[j][COLS - 1] = __builtin_amdgcn_fdot2_f32_bf16(v, __builtin_bit_cast(bf16x2, shi), t[j][COLS - 1], false);
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < ROWS; ++j) t[j][0] += sg * base[off + j * P];   // ROWS > 1 only with P > 0 and stride1 = 1
                    }
                };
                for (int n = 0; n < cnt; n += 4) {
                    const int4 e4 = *reinterpret_cast<const int4*>(eo + n);
                    const f32x4 sg = *reinterpret_cast<const f32x4*>(es + n);
                    tap(e4.x, sg.x); tap(e4.y, sg.y); tap(e4.z, sg.z); tap(e4.w, sg.w);
                }
                const float sk = sval[k];
#pragma unroll
                for (int m = 0; m < MG; ++m) {
                    const float um = ucode[m * p.kg + k];
#pragma unroll
                    for (int j = 0; j < ROWS; ++j)
#pragma unroll
                        for (int c = 0; c < COLS; ++c) acc[m][j][c] += um * (sk * t[j][c]);
                }
            }
#pragma unroll
            for (int m = 0; m < MG; ++m) {
                if (m < p.mg) {
                    const int co = g * p.mg + m;
                    const float bv = p.bias ? p.bias[co] : 0.f;
                    const size_t at = ((size_t)co * p.images + img) * plane_out + (size_t)(r0 + oy0) * p.Wo + ox;
#pragma unroll
                    for (int j = 0; j < ROWS; ++j)
#pragma unroll
                        for (int c = 0; c < COLS; ++c)
                            if (oy0 + j < nrows && ox + c < p.Wo) tsvd_store_y(p.y, at + (size_t)j * p.Wo + c, acc[m][j][c] + bv, p.out_bf16);
                }
            }
        }
    }
}

// rows of the staged window for rb output rows (ROWS-row units may read past the last output row)
int grouped_rows_in(const tsvd_conv_geometry& g, int rb, int ROWS) {
    const int rows = (rb + ROWS - 1) / ROWS * ROWS;
    return (rows - 1) * g.stride1 + (g.k1 - 1) * g.dil1 + 1;
}

size_t grouped_lds_bytes(const grouped_args& a, int MG, int P) {
    const size_t tile = ((size_t)a.cg * a.rows_in * (P ? P : a.win) + 3) & ~(size_t)3, stride = ((size_t)a.ng + 3) & ~(size_t)3;
    return 4 * (tile + 2 * a.kg * stride + (((size_t)a.kg + 3) & ~(size_t)3) + (size_t)MG * a.kg + a.kg) + a.kg * stride;
}

// Fills the launch shape of the grouped kernel; false when the sizes exceed its limits.
bool plan_grouped(const tsvd_conv_geometry& g, const tsvd_blob_header& hd, int64_t images, int64_t H, int64_t W, grouped_args* a,
                  int* MG, int* ROWS, int* P, int* PAIR, int* threads) {
    const int G = g.groups;
    if (g.c_in % G || g.c_out % G || hd.K % G) return false;
    a->cg = g.c_in / G; a->mg = g.c_out / G; a->kg = (int)(hd.K / G); a->ng = a->cg * g.k1 * g.k2;
    if (hd.M != g.c_out || hd.N != a->ng) return false;
    if (a->mg > GROUPED_MAX_MG || a->kg > GROUPED_MAX_KG || (long long)a->kg * ((a->ng + 3) & ~3) > GROUPED_MAX_ENTRIES || G > 65535)
        return false;
    *MG = a->mg <= 1 ? 1 : a->mg <= 2 ? 2 : a->mg <= 4 ? 4 : 8;
    a->images = (int)images; a->H = (int)H; a->W = (int)W;
    a->k1 = g.k1; a->k2 = g.k2; a->s1 = g.stride1; a->s2 = g.stride2; a->p1 = g.pad1; a->p2 = g.pad2; a->d1 = g.dil1; a->d2 = g.dil2;
    a->Ho = (int)(((long long)H + 2LL * g.pad1 - (long long)g.dil1 * (g.k1 - 1) - 1) / g.stride1 + 1);
    a->Wo = (int)(((long long)W + 2LL * g.pad2 - (long long)g.dil2 * (g.k2 - 1) - 1) / g.stride2 + 1);
    a->win = (a->Wo - 1) * g.stride2 + (g.k2 - 1) * g.dil2 + 1;
    // four rows per thread where the window rows are one compile-time pitch apart
    *ROWS = g.stride1 == 1 && a->win <= 256 && a->Ho >= 4 && *MG <= 4 ? 4 : 1;
    // ... and two columns where the columns are one element apart (the pitch holds two bf16 copies of win + 1 elements)
    *PAIR = *ROWS == 4 && g.stride2 == 1 && a->win <= 255;
    const int need = a->win + (*PAIR ? 1 : 0);
    *P = *ROWS == 1 ? 0 : need <= 64 ? 64 : need <= 128 ? 128 : 256;
    const int cols = *PAIR ? (a->Wo + 1) / 2 : a->Wo;       // units per row of units
    // rows per workgroup: the split of the plane that wastes the fewest lanes (passes of 256
    // units), a workgroup's fixed cost (tap lists, window) counted as one pass
    long long best = -1;
    for (int rb = 1; rb <= a->Ho && rb <= 256; ++rb) {
        a->rb = rb;
        a->rows_in = grouped_rows_in(g, rb, *ROWS);
        if (grouped_lds_bytes(*a, *MG, *P) > GROUPED_MAX_LDS) break;
        const int bpp = (a->Ho + rb - 1) / rb, last = a->Ho - (bpp - 1) * rb;
        const long long ub = (long long)((rb + *ROWS - 1) / *ROWS) * cols, ul = (long long)((last + *ROWS - 1) / *ROWS) * cols;
        const long long cost = (long long)(bpp - 1) * ((ub + 255) / 256 + 1) + ((ul + 255) / 256 + 1);
        if (best < 0 || cost <= best) { best = cost; a->bpp = bpp; }
    }
    if (best < 0) return false;
    a->rb = (a->Ho + a->bpp - 1) / a->bpp;
    a->bpp = (a->Ho + a->rb - 1) / a->rb;
    a->rows_in = grouped_rows_in(g, a->rb, *ROWS);
    const long long per_block = (long long)((a->rb + *ROWS - 1) / *ROWS) * cols;
    // workgroup size: the one of 256 / 192 / 128 that pads the units least (64 for tiny blocks)
    *threads = 64;
    if (per_block > 64) {
        long long padded = -1;
        for (int t = 256; t >= 128; t -= 64) {
            const long long pt = (per_block + t - 1) / t * t;
            if (padded < 0 || pt < padded) { padded = pt; *threads = t; }
        }
    }
    // several images per workgroup only for tiny planes (measured: with 392 units per plane, two
    // images per workgroup cost 81 us against 75 us for one, four 113 us: more workgroups hide more latency)
    a->ipb = (int)std::max<long long>(1, std::min<long long>(images, 256 / per_block));
    const long long blocks = (long long)a->bpp * ((images + a->ipb - 1) / a->ipb);
    return blocks < (1LL << 31) && images * H * W < (1LL << 31) && images * (long long)a->Ho * a->Wo < (1LL << 31);
}

template <int MG>
void launch_grouped(const grouped_args& a, int ROWS, int P, int PAIR, int groups, int threads, hipStream_t s) {
    const dim3 grid((unsigned)(a.bpp * ((a.images + a.ipb - 1) / a.ipb)), (unsigned)groups), block(threads);
    const size_t lds = grouped_lds_bytes(a, MG, P);
    if constexpr (MG <= 4) {
        if (ROWS == 4 && PAIR) {
            if (P == 64) hipLaunchKernelGGL((tsvd_grouped_conv_kernel<MG, 4, 64, true>), grid, block, lds, s, a);
            else if (P == 128) hipLaunchKernelGGL((tsvd_grouped_conv_kernel<MG, 4, 128, true>), grid, block, lds, s, a);
            else hipLaunchKernelGGL((tsvd_grouped_conv_kernel<MG, 4, 256, true>), grid, block, lds, s, a);
            return;
        }
        if (ROWS == 4) {
            if (P == 64) hipLaunchKernelGGL((tsvd_grouped_conv_kernel<MG, 4, 64, false>), grid, block, lds, s, a);
            else if (P == 128) hipLaunchKernelGGL((tsvd_grouped_conv_kernel<MG, 4, 128, false>), grid, block, lds, s, a);
            else hipLaunchKernelGGL((tsvd_grouped_conv_kernel<MG, 4, 256, false>), grid, block, lds, s, a);
            return;
        }
    }
    hipLaunchKernelGGL((tsvd_grouped_conv_kernel<MG, 1, 0, false>), grid, block, lds, s, a);
}

bool shapes_match(const tsvd_handle* h, const conv_plan& p) {
    int64_t M = 0, K = 0, N = 0, a = 0, b = 0;
    return tsvd_info(h, &M, &K, &N, &a, &b) == TSVD_OK && M == p.rows_u && N == p.rows_v;
}

}  // namespace

extern "C" size_t tsvd_conv2d_workspace_bytes(const tsvd_handle* h, const tsvd_conv_geometry* g, int64_t images, int64_t H,
                                              int64_t W) {
    conv_plan p;
    if (!h || !g || !make_plan(*g, images, H, W, &p)) return 0;
    if (g->groups > 1) {
        const tsvd_blob_header* hd;
        grouped_args a;
        int MG, ROWS, P, PAIR, threads;
        (void)tsvd_internal_blob(h, &hd);
        return g->form == 0 && plan_grouped(*g, *hd, images, H, W, &a, &MG, &ROWS, &P, &PAIR, &threads) ? 256 : 0;   // no scratch is used
    }
    if (!p.fits || !shapes_match(h, p)) return 0;
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
    if (!make_plan(*g, images, H, W, &p)) return TSVD_EINVAL;
    if (g->groups > 1) {
        if (g->form != 0) return TSVD_EUNSUPPORTED;
        const tsvd_blob_header* hd;
        const uint8_t* blob = tsvd_internal_blob(h, &hd);
        grouped_args a;
        int MG, ROWS, P, PAIR, threads;
        if (g->c_in % g->groups || g->c_out % g->groups || hd->K % g->groups || hd->M != g->c_out ||
            hd->N != (int64_t)(g->c_in / g->groups) * g->k1 * g->k2)
            return TSVD_EINVAL;
        if (!plan_grouped(*g, *hd, images, H, W, &a, &MG, &ROWS, &P, &PAIR, &threads)) return TSVD_EUNSUPPORTED;
        if (tsvd_tune("TSVD_GROUPED_PAIR", 1) == 0) PAIR = 0;   // tuning switch: fp32 window
        a.U = reinterpret_cast<const uint32_t*>(blob + hd->off_U); a.u_tps = (int)(hd->Kp / TSVD_TILE_COLS);
        a.V = reinterpret_cast<const uint32_t*>(blob + hd->off_V); a.v_tps = (int)(hd->Np / TSVD_TILE_COLS);
        a.S = reinterpret_cast<const float*>(blob + hd->off_S);
        a.K = (int)hd->K;
        a.x = static_cast<const uint16_t*>(x_dev); a.y = y_dev; a.bias = bias_dev; a.out_bf16 = y_dtype == TSVD_BF16;
        hipStream_t gs = static_cast<hipStream_t>(stream);
        if (MG == 1) launch_grouped<1>(a, ROWS, P, PAIR, g->groups, threads, gs);
        else if (MG == 2) launch_grouped<2>(a, ROWS, P, PAIR, g->groups, threads, gs);
        else if (MG == 4) launch_grouped<4>(a, ROWS, P, PAIR, g->groups, threads, gs);
        else launch_grouped<8>(a, ROWS, P, PAIR, g->groups, threads, gs);
        return hipGetLastError() == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
    }
    if (!p.fits || !shapes_match(h, p)) return TSVD_EINVAL;
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
