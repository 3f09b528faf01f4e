// C ABI entry points that touch the device: upload, forward dispatch, release.
// (The host-only packer lives in tsvd_pack.cpp.)
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "../../include/tsvd.h"
#include "../../include/tsvd_tuning.h"
#include "tsvd_kernels.h"
#include "tsvd_layout.h"

struct tsvd_handle {
    int device;
    tsvd_blob_header hd;
    uint8_t* blob;          // device
    bool owns_blob;
    void* scratch;          // device, handle-owned workspace (grown on demand)
    size_t scratch_bytes;
    void* retired[16];      // earlier, smaller scratch buffers: enqueued work may still use them, so they live until tsvd_free
    int retired_count;
    float bound_V;          // max_k |S_k| * nnz(V[k,:]) : |z_k| <= bound_V * max|x| for every token
    int cu_count;           // compute units of the device
    long long* clocks;      // tuning aid (TSVD_CLOCKS=1 at pack time): phase timestamps of the B <= 2 kernel
    // One-launch single-token path: [counter: 256 B][z as tagged 64-bit words: Kp], device, zeroed at pack
    // (counter = 1); null when the shape does not fit that kernel.  The path belongs to the first stream
    // that uses it: calls on one stream never overlap, calls on other streams take the two-launch kernels.
    uint8_t* dense_u;       // device: U in the denser code (five elements per byte), only with TSVD_DENSE_U = 1 at pack time
    uint8_t* sync;
    std::atomic<int> sync_claimed;
    void* sync_stream;
};

// Workspace of tsvd_forward_noalloc: one array per GPU inside the loaded code object, so the entry point
// never allocates.  The name below is a host-side stand-in; the array's device address differs per GPU
// and is looked up once per device in device_init (noalloc_ptr), which is what host code passes on.
static __device__ __align__(256) unsigned char scratch[TSVD_NOALLOC_MAX_WORKSPACE];
static void* noalloc_ptr[64] = {};

namespace {

int env_int(const char* name, int fallback) { return tsvd_tune(name, fallback); }

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// Options of the last stage (tsvd_forward_ex).
struct out_opts {
    const float* bias;   // device [M] or null
    int out_bf16;
    int token_major;     // y is [B][ldy] instead of [M][ldy]
};

// Token-major activations [B][ldx] -> feature-major [N][ldt] (ldt a multiple of 8 elements, the
// padding columns zero), through 32 x 32 LDS tiles; T is the 16- or 32-bit storage type.
template <typename T>
__global__ void __launch_bounds__(256)
tsvd_transpose_kernel(const T* __restrict__ x, long long ldx, int B, int N, T* __restrict__ xt, long long ldt) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;          // 32 x 8 threads
    const int n0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int b = b0 + r, n = n0 + tx;
        tile[r][tx] = (b < B && n < N) ? x[(size_t)b * ldx + n] : T(0);
    }
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int n = n0 + r, b = b0 + tx;
        if (n < N && b < ldt) xt[(size_t)n * ldt + b] = tile[tx][r];
    }
}

// Feature-major activations with unaligned rows [N][ldx] -> [N][ldt] (ldt a multiple of 8 elements, the padding
// columns zero): one thread per element, consecutive threads along a row.
__global__ void __launch_bounds__(256)
tsvd_realign_kernel(const uint16_t* __restrict__ x, long long ldx, int B, uint16_t* __restrict__ xt, long long ldt) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    const size_t n = blockIdx.y;
    if (b < ldt) xt[n * ldt + b] = b < B ? x[n * ldx + b] : (uint16_t)0;
}

// One-time, per-device setup (the device is current): kernel attributes, address of the static workspace.
hipError_t device_init(int device) {
    static bool done[64] = {};
    if (device < 0 || device >= 64) return hipErrorInvalidDevice;
    if (done[device]) return hipSuccess;
    void* sp = nullptr;
    hipError_t e = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!sp || (reinterpret_cast<uintptr_t>(sp) & 255u)) return hipErrorInvalidSymbol;
    noalloc_ptr[device] = sp;
    e = tsvd_skinny_init();
    if (e != hipSuccess) return e;
    e = tsvd_gemm_init();
    if (e != hipSuccess) return e;
    e = tsvd_gemv_init();
    if (e != hipSuccess) return e;
    e = tsvd_mid_init();
    if (e != hipSuccess) return e;
    e = tsvd_gemv_dense_init();
    if (e != hipSuccess) return e;
    e = tsvd_transition_init();
    if (e != hipSuccess) return e;
    done[device] = true;
    return hipSuccess;
}

// ---- skinny path (few tokens): two launches per pair of tokens --------------------------------
void shape_skinny(tsvd_skinny_args& a) {
    // LDS: digit planes [8 * tokens][slab_k + 16] bytes + reduction tiles (<= 16 KiB) + 256 B
    const size_t budget = TSVD_SKINNY_MAX_LDS - 16 * 1024 - 1024;
    const int cols = 8 * a.tokens;
    const int slab = (int)std::min<size_t>((size_t)a.nkt, (budget / (size_t)cols - 16) / 256);
    a.slab_tiles = std::max(slab, 1);
    // One workgroup of up to 16 wavefronts per compute unit when the matrix is large enough:
    // sw strips x kw contraction splits, every wavefront streaming nkt / kw tiles.
    int sw = 1;
    while (sw < 16 && a.strips / (sw * 2) >= 256) sw *= 2;
    int kw = 1;
    while (sw * kw * 2 <= 16 && kw * 2 <= a.nkt) kw *= 2;
    a.sw = std::max(1, std::min(16, env_int("TSVD_SKINNY_SW", sw)));
    a.kw = std::max(1, std::min(std::min(16 / a.sw, a.nkt), env_int("TSVD_SKINNY_KW", kw)));
}

size_t skinny_workspace(const tsvd_handle* h) {
    return 256 + (size_t)16 * (size_t)h->hd.Kp;      // exponents, then 16 digit planes of Kp bytes
}

int pow2_ceil(int64_t v) {
    int r = 1;
    while (r < v) r *= 2;
    return r;
}
int pow2_floor(int64_t v) {
    int r = 1;
    while ((int64_t)r * 2 <= v) r *= 2;
    return r;
}

// One token through the tsvd_gemv kernels; returns false if the shape does not fit them.
bool try_gemv(const tsvd_handle* h, const void* x, tsvd_dtype x_dtype, int64_t ldx, void* y, int64_t ldy,
              const out_opts& oo, int* meta, unsigned char* planes, hipStream_t stream, tsvd_status* st) {
    const tsvd_blob_header& hd = h->hd;
    if (env_int("TSVD_GEMV", 1) == 0 || !tsvd_gemv_fits(hd.Np, hd.Kp)) return false;
    const int mask = tsvd_stage_mask();
    if (mask == 7 && !h->dense_u && env_int("TSVD_GEMV_FUSED", 1) != 0 && tsvd_gemv_fused_fits(hd.Mp, hd.Kp, hd.Np)) {
        // a small matrix: both stages in one launch of one workgroup
        tsvd_gemv_fused_args f;
        std::memset(&f, 0, sizeof f);
        f.tiles_v = h->blob + hd.off_V; f.strips_v = (int)(hd.Kp / 16); f.nkt_v = (int)(hd.Np / 256);
        f.tiles_u = h->blob + hd.off_U; f.strips_u = (int)((hd.M + 15) / 16); f.nkt_u = (int)(hd.Kp / 256);
        f.N = (int)hd.N; f.Np = (int)hd.Np; f.Kp = (int)hd.Kp; f.M = (int)hd.M;
        f.x = x; f.x_is_bf16 = x_dtype == TSVD_BF16; f.ldx = ldx;
        f.x_vec = ldx == 1 && hd.N % 4 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0;
        f.S = reinterpret_cast<const float*>(h->blob + hd.off_S);
        f.bound_V = h->bound_V;
        f.y = y; f.ldy = ldy; f.bias = oo.bias; f.out_bf16 = oo.out_bf16;
        *st = tsvd_launch_gemv_fused(f, stream) == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
        return true;
    }
    if (mask == 7 && h->sync && !h->dense_u && env_int("TSVD_GEMV_ONEPASS", 0) != 0) {
        // both stages in one launch (z handed over between workgroups through the handle's tagged buffer)
        tsvd_handle* hm = const_cast<tsvd_handle*>(h);
        int expected = 0;
        if (hm->sync_claimed.compare_exchange_strong(expected, 1)) hm->sync_stream = stream;
        tsvd_gemv_onepass_args f;
        std::memset(&f, 0, sizeof f);
        if (hm->sync_stream == (void*)stream && tsvd_gemv_onepass_shape(hd.M, hd.Mp, hd.Kp, hd.Np, h->cu_count, &f)) {
            f.tiles_v = h->blob + hd.off_V;
            f.tiles_u = h->blob + hd.off_U;
            f.N = (int)hd.N; f.Np = (int)hd.Np; f.Kp = (int)hd.Kp; f.M = (int)hd.M;
            f.x = x; f.x_is_bf16 = x_dtype == TSVD_BF16; f.ldx = ldx;
            f.x_vec = ldx == 1 && hd.N % 4 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0;
            f.S = reinterpret_cast<const float*>(h->blob + hd.off_S);
            f.bound_V = h->bound_V;
            f.counter = reinterpret_cast<unsigned*>(h->sync);
            f.zbuf = reinterpret_cast<unsigned long long*>(h->sync + 256);
            f.spin_limit = env_int("TSVD_SPIN_LIMIT", 256);
            f.y = y; f.ldy = ldy; f.bias = oo.bias; f.out_bf16 = oo.out_bf16;
            f.clocks = h->clocks;
            *st = tsvd_launch_gemv_onepass(f, stream) == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
            return true;
        }
    }
    // sw strips x kw splits = 16 wavefronts; about one workgroup per compute unit for large matrices
    auto shape = [&](tsvd_gemv_args& a) {
        int sw = 1;
        while (sw < 16 && a.strips / (sw * 2) >= 256) sw *= 2;
        int kl = 0;
        while ((sw << (kl + 1)) <= 16 && (2 << kl) <= a.nkt) ++kl;
        a.sw = std::max(1, std::min(16, env_int("TSVD_GEMV_SW", sw)));
        a.kw_log2 = std::max(0, env_int("TSVD_GEMV_KWLOG2", kl));
        while ((a.sw << a.kw_log2) > 16) --a.kw_log2;
    };
    tsvd_gemv_args a;
    std::memset(&a, 0, sizeof a);
    a.N = (int)hd.N; a.Np = (int)hd.Np; a.Kp = (int)hd.Kp;
    a.meta = meta;
    a.clocks = h->clocks;
    a.early_tiles = env_int("TSVD_EARLY_TILES", 1);
    if (mask & 2) {
        a.tiles = h->blob + hd.off_V;
        a.strips = (int)(hd.Kp / 16);
        a.nkt = (int)(hd.Np / 256);
        a.rows_out = (int)hd.Kp;
        a.x = x;
        a.x_is_bf16 = x_dtype == TSVD_BF16;
        a.ldx = ldx;
        a.x_vec = ldx == 1 && hd.N % 4 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0;
        a.S = reinterpret_cast<const float*>(h->blob + hd.off_S);
        a.bound_V = h->bound_V;
        a.planes_out = planes;
        shape(a);
        if (tsvd_launch_gemv(a, false, stream) != hipSuccess) {
            *st = TSVD_EDEVICE;
            return true;
        }
    }
    if ((mask & 4) && h->dense_u && tsvd_gemv_dense_lds(hd.Kp) <= TSVD_SKINNY_MAX_LDS) {
        tsvd_gemv_dense_args d;
        std::memset(&d, 0, sizeof d);
        d.dense = h->dense_u;
        d.groups = (int)((hd.Mp / 16 + 4) / 5);
        d.nkt = (int)(hd.Kp / 256);
        d.Kp = (int)hd.Kp; d.M = (int)hd.M;
        d.planes_in = planes; d.meta = meta;
        d.y = y; d.ldy = ldy; d.bias = oo.bias; d.out_bf16 = oo.out_bf16;
        *st = tsvd_launch_gemv_dense(d, stream) == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
        return true;
    }
    if (mask & 4) {
        a.tiles = h->blob + hd.off_U;
        a.strips = (int)((hd.M + 15) / 16);
        a.nkt = (int)(hd.Kp / 256);
        a.rows_out = (int)hd.M;
        a.planes_in = planes;
        a.y = y;
        a.ldy = ldy;
        a.bias = oo.bias;
        a.out_bf16 = oo.out_bf16;
        shape(a);
        if (tsvd_launch_gemv(a, true, stream) != hipSuccess) {
            *st = TSVD_EDEVICE;
            return true;
        }
    }
    *st = TSVD_OK;
    return true;
}

tsvd_status forward_skinny(const tsvd_handle* h, const void* x, tsvd_dtype x_dtype, int64_t B, int64_t ldx,
                           void* y, int64_t ldy, const out_opts& oo, void* ws, hipStream_t stream) {
    const size_t yelt = oo.out_bf16 ? 2 : 4;
    const tsvd_blob_header& hd = h->hd;
    int* meta = static_cast<int*>(ws);
    unsigned char* planes = static_cast<unsigned char*>(ws) + 256;
    const size_t xelt = x_dtype == TSVD_BF16 ? 2 : 4;
    const int mask = tsvd_stage_mask();
    if (tsvd_gemv_fits(hd.Np, hd.Kp) && env_int("TSVD_GEMV", 1) != 0) {
        // one token at a time through the fast kernels (each pass re-reads the weights)
        for (int64_t b0 = 0; b0 < B; ++b0) {
            tsvd_status gst = TSVD_OK;
            // one token's output: column b0 of y [M][ldy], or row b0 of y [B][ldy] (then consecutive in memory)
            uint8_t* yb = static_cast<uint8_t*>(y) + (oo.token_major ? (size_t)b0 * (size_t)ldy : (size_t)b0) * yelt;
            if (!try_gemv(h, static_cast<const uint8_t*>(x) + (size_t)b0 * xelt, x_dtype, ldx,
                          yb, oo.token_major ? 1 : ldy, oo, meta, planes, stream, &gst))
                return TSVD_EUNSUPPORTED;
            if (gst != TSVD_OK) return gst;
        }
        return TSVD_OK;
    }
    for (int64_t b0 = 0; b0 < B; b0 += 2) {
        const int tokens = (int)std::min<int64_t>(2, B - b0);
        tsvd_skinny_args v;
        std::memset(&v, 0, sizeof v);
        v.tiles = h->blob + hd.off_V;
        v.strips = (int)(hd.Kp / 16);           // padded rows give z = 0: every plane byte is written
        v.nkt = (int)(hd.Np / 256);
        v.mode = TSVD_SKINNY_STAGE_V;
        v.in = static_cast<const uint8_t*>(x) + (size_t)b0 * xelt;
        v.in_is_bf16 = x_dtype == TSVD_BF16;
        v.kvalid = (int)hd.N;
        v.ld_in = ldx;
        v.tokens = tokens;
        v.rowscale = reinterpret_cast<const float*>(h->blob + hd.off_S);
        v.bound_V = h->bound_V;
        v.meta_out = meta;
        v.out = planes;
        v.ld_out = hd.Kp;
        v.rows_out = (int)hd.Kp;
        shape_skinny(v);
        if ((mask & 2) && tsvd_launch_skinny(v, stream) != hipSuccess) return TSVD_EDEVICE;

        tsvd_skinny_args u;
        std::memset(&u, 0, sizeof u);
        u.tiles = h->blob + hd.off_U;
        u.strips = (int)((hd.M + 15) / 16);
        u.nkt = (int)(hd.Kp / 256);
        u.mode = TSVD_SKINNY_STAGE_U;
        u.in = planes;
        u.ld_in = hd.Kp;
        u.tokens = tokens;
        u.meta_in = meta;
        u.out = static_cast<uint8_t*>(y) + (oo.token_major ? (size_t)b0 * (size_t)ldy : (size_t)b0) * yelt;
        u.ld_out = ldy;
        u.out_token_major = oo.token_major;
        u.rows_out = (int)hd.M;
        u.bias = oo.bias;
        u.out_bf16 = oo.out_bf16;
        shape_skinny(u);
        if ((mask & 4) && tsvd_launch_skinny(u, stream) != hipSuccess) return TSVD_EDEVICE;
    }
    return TSVD_OK;
}

// ---- few-token path: groups of up to 16 tokens of bf16 activations, two launches per group ------
// Up to 16 tokens always; up to 64 tokens (2..4 groups, each streaming the weights again, mostly
// from the last-level cache) when the packed weights are large: there the batched kernels, with
// few and narrow token tiles, spend their time re-reading z through L2 (measured on MI355X,
// 16384 x 4096 x 8192: 38 us against 111 us at B = 32; 3072 x 768 x 1536: 24 us against 15 us).
bool use_mid(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype, int64_t ldx) {
    if (x_dtype != TSVD_BF16 || B < 2 || B > 64 || env_int("TSVD_MID", 1) == 0) return false;
    // (32-bit byte offsets into x in the kernel, which also addresses up to four slabs of 2048 rows
    // beyond the last one: the range check returns zeros there)
    if (((uint64_t)h->hd.Np + 8192) * (uint64_t)ldx * 2 >= (1ull << 31)) return false;
    if (B <= 16) return true;
    const int forced = env_int("TSVD_MID_MAX_B", 0);       // tuning switch: largest B served here
    if (forced > 0) return B <= forced;
    // Measured break-even against the batched kernels, which launch only the 64-token tiles that hold tokens.
    // Aligned rows: two groups of 16 pay off between about 4 and 60 MB of packed weights (10.5 MB: 21.5 against
    // 27 us; 42 MB: 39 against 49 us; 94 MB: 95 against 82 us; 255 MB: 194 against 142 us), three and four
    // groups never (24 MB at 48 tokens: 65 against 38 us; 42 MB: 61 against 50 us; 255 MB: 299 against 140 us).
    // Unaligned rows take a slower batched kernel: 2, 3, 4 groups pay off from about 1.7, 4.5 and 8 MB.
    const double code_bytes = (double)h->hd.Kp * (double)(h->hd.Mp + h->hd.Np) / 4.0;
    const int groups = (int)((B + 15) / 16);
    if (ldx % 8 == 0) return groups == 2 && code_bytes >= 4.2e6 && code_bytes < 60.0e6;
    static const double min_bytes[5] = {0.0, 0.0, 4.2e6, 11.2e6, 20.0e6};
    return code_bytes >= min_bytes[groups] * 0.4;
}

size_t mid_workspace(const tsvd_handle* h) {
    return 256 + (size_t)32 * (size_t)h->hd.Kp;      // per-token maxima, then z fp16 [Kp][16]
}

tsvd_status forward_mid(const tsvd_handle* h, const void* x, int64_t B, int64_t ldx, void* y, int64_t ldy,
                        const out_opts& oo, void* ws, hipStream_t stream) {
    const tsvd_blob_header& hd = h->hd;
    const int mask = tsvd_stage_mask();
    // about one workgroup of 16 wavefronts per compute unit: sw strips x kw contraction splits
    auto shape = [&](tsvd_mid_args& a) {
        int sw = 2;
        while (sw < 16 && a.strips / (sw * 2) >= h->cu_count) sw *= 2;
        int kl = 0;
        while (kl < 3 && (sw << (kl + 1)) <= 16 && (2 << kl) <= a.nkt) ++kl;
        a.sw = std::max(1, std::min(16, env_int("TSVD_MID_SW", sw)));
        a.kw_log2 = std::max(0, std::min(3, env_int("TSVD_MID_KWLOG2", kl)));
        while ((a.sw << a.kw_log2) > 16) --a.kw_log2;
    };
    for (int64_t b0 = 0; b0 < B; b0 += 16) {
    const int64_t nb = std::min<int64_t>(16, B - b0);
    tsvd_mid_args a;
    std::memset(&a, 0, sizeof a);
    a.bvalid = (int)nb;
    a.bound_V = h->bound_V;
    a.colmax = static_cast<float*>(ws);
    a.clocks = h->clocks;
    a.resident_ok = env_int("TSVD_MID_RESIDENT", 1) != 0;
    uint16_t* z = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(ws) + 256);
    if (mask & 2) {
        a.tiles = h->blob + hd.off_V;
        a.strips = (int)(hd.Kp / 16);
        a.nkt = (int)(hd.Np / 256);
        a.act = static_cast<const uint16_t*>(x) + b0;
        a.ld = ldx;
        a.kvalid = (int)hd.N;
        // extent of x, rounded up to the 4-byte granularity of the buffer range check (for odd B the
        // dword holding the last element would otherwise read as zero; it lies inside an aligned dword
        // whose first half is the caller's, so it cannot cross into an unmapped page)
        a.act_bytes = (unsigned)((((((size_t)hd.N - 1) * (size_t)ldx + (size_t)nb) * 2) + 3) & ~(size_t)3);
        a.S = reinterpret_cast<const float*>(h->blob + hd.off_S);
        a.out = z;
        a.ld_out = 16;
        a.rows_valid = (int)hd.Kp;
        shape(a);
        const bool vec = ldx % 8 == 0 && (reinterpret_cast<uintptr_t>(a.act) & 15u) == 0;
        a.pairs = ldx % 2 == 0 && (reinterpret_cast<uintptr_t>(a.act) & 3u) == 0;
        if (tsvd_launch_mid(a, false, vec, stream) != hipSuccess) return TSVD_EDEVICE;
    }
    if (mask & 4) {
        a.tiles = h->blob + hd.off_U;
        a.strips = (int)((hd.M + 15) / 16);
        a.nkt = (int)(hd.Kp / 256);
        a.act = z;
        a.ld = 16;
        a.kvalid = (int)hd.Kp;
        a.act_bytes = (unsigned)((size_t)hd.Kp * 32);
        a.S = nullptr;
        a.out = static_cast<uint8_t*>(y) + (oo.token_major ? (size_t)b0 * (size_t)ldy : (size_t)b0) * (oo.out_bf16 ? 2 : 4);
        a.ld_out = ldy;
        a.out_token_major = oo.token_major;
        a.rows_valid = (int)hd.M;
        a.bias = oo.bias;
        a.out_bf16 = oo.out_bf16;
        shape(a);
        if (tsvd_launch_mid(a, true, true, stream) != hipSuccess) return TSVD_EDEVICE;
    }
    }
    return TSVD_OK;
}

// (set for the duration of a tsvd_forward_noalloc call whose fp32 batch would not fit the fixed workspace as planes:
// such a call goes one token at a time, as every fp32 batch did before the six-plane path existed)
thread_local bool f32_one_token_at_a_time = false;

bool use_gemm(const tsvd_handle*, int64_t B, tsvd_dtype x_dtype) {
    if (x_dtype == TSVD_F32 && f32_one_token_at_a_time) return false;
    // (fp32 activations: fewer tokens are handled one at a time by the single-token kernels, each pass streaming the weights)
    const int min_b = x_dtype == TSVD_BF16 ? env_int("TSVD_GEMM_MIN_B", 17) : env_int("TSVD_GEMM_MIN_B_F32", 17);
    return B >= min_b;
}

size_t gemm_workspace(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype) {
    const int64_t Bp = tsvd_round_up(B, 256);
    if (x_dtype == TSVD_F32)      // two sets of planes of x, two of z (blocks that hold anything only)
        return round256(tsvd_gemm_fp6_bytes(256 * ((h->hd.N + 127) / 128), Bp)) + round256(tsvd_gemm_fp6_bytes(256 * ((h->hd.K + 127) / 128), Bp));
    // partial column maxima [PARTS][Bp] fp32, then Z as fp16 [Kp][Bp]
    size_t bytes = round256((size_t)(TSVD_COLMAX_PARTS + 1) * Bp * 4) + round256((size_t)h->hd.Kp * (size_t)Bp * 2);
    // (the rule is asked as for aligned rows: a caller with unaligned rows then reserves a little too much)
    if (tsvd_gemm_use_fp6(h->hd.Mp, h->hd.Kp, h->hd.Np, B, h->cu_count, true))      // planes of Z, and of X for stage V
        bytes += round256(tsvd_gemm_fp6_bytes(h->hd.Kp, Bp)) + round256(tsvd_gemm_fp6_bytes(h->hd.Np, Bp));
    return bytes;
}

}  // namespace

extern "C" tsvd_status tsvd_pack(const int8_t* U, const float* S, const int8_t* V, int64_t M, int64_t K,
                                 int64_t N, void* dev_buf, size_t dev_buf_bytes, tsvd_handle** out) {
    if (!U || !S || !V || !out) return TSVD_EINVAL;
    const size_t bytes = tsvd_packed_bytes(M, K, N);
    if (bytes == 0) return TSVD_EINVAL;
    if (dev_buf && (dev_buf_bytes < bytes || (reinterpret_cast<uintptr_t>(dev_buf) & 255u))) return TSVD_EINVAL;

    void* host = std::malloc(bytes);
    if (!host) return TSVD_ENOMEM;
    tsvd_status st = tsvd_pack_host(U, S, V, M, K, N, host, bytes);
    if (st != TSVD_OK) {
        std::free(host);
        return st;
    }
    tsvd_handle* h = new (std::nothrow) tsvd_handle();
    if (!h) {
        std::free(host);
        return TSVD_ENOMEM;
    }
    std::memcpy(&h->hd, host, sizeof h->hd);
    // bound on |z_k| / max|x|, used to scale the fp16 intermediate of the batched path
    double bound = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        int64_t nz = 0;
        const int8_t* row = V + k * N;
        for (int64_t n = 0; n < N; ++n) nz += row[n] != 0;
        bound = std::max(bound, std::fabs((double)S[k]) * (double)nz);
    }
    h->bound_V = (float)bound;
    h->scratch = nullptr;
    h->scratch_bytes = 0;
    h->retired_count = 0;
    h->clocks = nullptr;
    h->cu_count = 256;
    h->sync = nullptr;
    h->dense_u = nullptr;
    h->sync_claimed.store(0);
    h->sync_stream = nullptr;

    bool ok = hipGetDevice(&h->device) == hipSuccess && device_init(h->device) == hipSuccess;
    if (ok) {
        if (dev_buf) {
            h->blob = static_cast<uint8_t*>(dev_buf);
            h->owns_blob = false;
        } else {
            void* d = nullptr;
            ok = hipMalloc(&d, bytes) == hipSuccess;
            h->blob = static_cast<uint8_t*>(d);
            h->owns_blob = ok;
        }
    }
    if (ok) ok = hipMemcpy(h->blob, host, bytes, hipMemcpyHostToDevice) == hipSuccess;
    if (ok) {
        {
            int cus = 0;
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device) == hipSuccess && cus > 0)
                h->cu_count = cus;
            if (env_int("TSVD_GEMV_ONEPASS", 0) != 0 && tsvd_gemv_onepass_shape(h->hd.M, h->hd.Mp, h->hd.Kp, h->hd.Np, h->cu_count, nullptr)) {
                // hand-over buffer of the one-launch single-token path (small: 8 bytes per rank index)
                const size_t sb = 256 + (size_t)h->hd.Kp * 8;
                void* d = nullptr;
                const unsigned one = 1u;
                ok = hipMalloc(&d, sb) == hipSuccess;
                if (ok) {
                    h->sync = static_cast<uint8_t*>(d);
                    ok = hipMemset(d, 0, sb) == hipSuccess && hipMemcpy(d, &one, sizeof one, hipMemcpyHostToDevice) == hipSuccess;
                }
            }
            if (ok && env_int("TSVD_DENSE_U", 0) != 0) {
                // measurement switch: a second copy of U in the denser code, used by stage U of single-token calls
                const size_t db = tsvd_dense_bytes(M, K);
                void* hostd = std::malloc(db);
                void* d = nullptr;
                ok = hostd && hipMalloc(&d, db) == hipSuccess;
                if (ok) {
                    tsvd_internal_dense_from_blob(host, hostd);
                    h->dense_u = static_cast<uint8_t*>(d);
                    ok = hipMemcpy(d, hostd, db, hipMemcpyHostToDevice) == hipSuccess;
                }
                std::free(hostd);
            }
            if (ok && env_int("TSVD_CLOCKS", 0)) {
                void* c = nullptr;
                if (hipMalloc(&c, TSVD_GEMV_MAX_GRID * 16 * sizeof(long long)) == hipSuccess) {
                    (void)hipMemset(c, 0, TSVD_GEMV_MAX_GRID * 16 * sizeof(long long));
                    h->clocks = static_cast<long long*>(c);
                }
            }
        }
    }
    std::free(host);
    if (!ok) {
        if (h->owns_blob && h->blob) (void)hipFree(h->blob);
        if (h->sync) (void)hipFree(h->sync);
        if (h->dense_u) (void)hipFree(h->dense_u);
        delete h;
        (void)hipGetLastError();
        return TSVD_EDEVICE;
    }
    *out = h;
    return TSVD_OK;
}

extern "C" tsvd_status tsvd_unpack(const tsvd_handle* h, int8_t* U, float* S, int8_t* V) {
    if (!h) return TSVD_EINVAL;
    const size_t bytes = (size_t)h->hd.total_bytes;
    void* host = std::malloc(bytes);
    if (!host) return TSVD_ENOMEM;
    if (hipMemcpy(host, h->blob, bytes, hipMemcpyDeviceToHost) != hipSuccess) {
        std::free(host);
        return TSVD_EDEVICE;
    }
    tsvd_status st = tsvd_unpack_host(host, bytes, U, S, V, nullptr, nullptr, nullptr);
    std::free(host);
    return st;
}

extern "C" tsvd_status tsvd_info(const tsvd_handle* h, int64_t* M, int64_t* K, int64_t* N, int64_t* nnzU,
                                 int64_t* nnzV) {
    if (!h) return TSVD_EINVAL;
    if (M) *M = h->hd.M;
    if (K) *K = h->hd.K;
    if (N) *N = h->hd.N;
    if (nnzU) *nnzU = h->hd.nnzU;
    if (nnzV) *nnzV = h->hd.nnzV;
    return TSVD_OK;
}

namespace {
size_t base_workspace(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype) {
    // (the few-token path is chosen per call, by the row stride too: cover every candidate)
    const size_t few = round256(std::max(skinny_workspace(h), mid_workspace(h)));
    if (use_gemm(h, B, x_dtype)) return std::max(gemm_workspace(h, B, x_dtype), B <= 64 ? few : (size_t)0);
    return few;
}
// feature-major copy of token-major activations: [N][B rounded up to 8] elements
size_t transposed_bytes(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype) {
    return round256((size_t)h->hd.N * (size_t)tsvd_round_up(B, 8) * (x_dtype == TSVD_BF16 ? 2 : 4));
}
}  // namespace

extern "C" size_t tsvd_workspace_bytes_ex(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype, tsvd_layout x_layout) {
    if (!h || B <= 0 || (x_dtype != TSVD_F32 && x_dtype != TSVD_BF16)) return 0;
    if (x_layout != TSVD_FEATURE_MAJOR && x_layout != TSVD_TOKEN_MAJOR) return 0;
    // (feature-major rows that are not 16-byte aligned are copied too, when the call goes to the batched kernels:
    // the alignment is not known here, so the room is always there)
    const bool copy = x_layout == TSVD_TOKEN_MAJOR || use_gemm(h, B, x_dtype);
    return base_workspace(h, B, x_dtype) + (copy ? transposed_bytes(h, B, x_dtype) : 0);
}

extern "C" size_t tsvd_workspace_bytes(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype) {
    return tsvd_workspace_bytes_ex(h, B, x_dtype, TSVD_FEATURE_MAJOR);
}

extern "C" tsvd_status tsvd_forward_ex(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                                       int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                                       int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    return tsvd_forward_io(h, x_dev, x_dtype, x_layout, B, ldx, bias_dev, y_dev, y_dtype, TSVD_FEATURE_MAJOR, ldy, workspace,
                           workspace_bytes, stream);
}

extern "C" tsvd_status tsvd_forward_io(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                                       int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                                       tsvd_layout y_layout, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    if (!h || !x_dev || !y_dev || B <= 0) return TSVD_EINVAL;
    if (y_layout != TSVD_FEATURE_MAJOR && y_layout != TSVD_TOKEN_MAJOR) return TSVD_EINVAL;
    if (ldy < (y_layout == TSVD_TOKEN_MAJOR ? h->hd.M : B)) return TSVD_EINVAL;
    if (x_dtype != TSVD_F32 && x_dtype != TSVD_BF16) return TSVD_EINVAL;
    if (y_dtype != TSVD_F32 && y_dtype != TSVD_BF16) return TSVD_EINVAL;
    if (x_layout != TSVD_FEATURE_MAJOR && x_layout != TSVD_TOKEN_MAJOR) return TSVD_EINVAL;
    if (ldx < (x_layout == TSVD_TOKEN_MAJOR ? h->hd.N : B)) return TSVD_EINVAL;
    if (B > (int64_t(1) << 24)) return TSVD_EUNSUPPORTED;
    const size_t need = tsvd_workspace_bytes_ex(h, B, x_dtype, x_layout);
    void* ws = workspace;
    if (ws) {
        if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return TSVD_EINVAL;
    } else {
        if (workspace_bytes != 0) return TSVD_EINVAL;
        tsvd_handle* hm = const_cast<tsvd_handle*>(h);
        if (hm->scratch_bytes < need) {
            // Enqueued work may still use the old buffer.  It is not freed here (hipFree would wait for the whole
            // device): it is kept until tsvd_free, and the new one is at least twice as large, so at most 16
            // buffers ever retire and their sizes sum to less than the live one.  Only when that list is full
            // does the call fall back to draining the device.
            void* d = nullptr;
            const size_t grow = std::max(need, 2 * hm->scratch_bytes);
            if (hipMalloc(&d, grow) != hipSuccess) {
                (void)hipGetLastError();
                return TSVD_EDEVICE;
            }
            if (hm->scratch) {
                if (hm->retired_count < 16) {
                    hm->retired[hm->retired_count++] = hm->scratch;
                } else {
                    if (hipDeviceSynchronize() != hipSuccess) return TSVD_EDEVICE;
                    (void)hipFree(hm->scratch);
                }
            }
            hm->scratch = d;
            hm->scratch_bytes = grow;
        }
        ws = hm->scratch;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const out_opts oo = {bias_dev, y_dtype == TSVD_BF16, y_layout == TSVD_TOKEN_MAJOR};
    if (x_layout == TSVD_TOKEN_MAJOR && B == 1) {
        // a single token is one contiguous vector in either layout: feature-major with unit row pitch, no copy
        x_layout = TSVD_FEATURE_MAJOR;
        ldx = 1;
    }
    int x_in_place = 0;
    if (x_layout == TSVD_TOKEN_MAJOR && x_dtype == TSVD_BF16 && use_gemm(h, B, x_dtype) && !use_mid(h, B, x_dtype, tsvd_round_up(B, 8)) &&
        tsvd_gemm_reads_token_major(h->hd.Mp, h->hd.Kp, h->hd.Np, B, h->cu_count)) {
        x_in_place = 1;       // the kernels this call takes gather their operand lanes from [B][ldx] themselves
    } else if (x_layout == TSVD_TOKEN_MAJOR) {
        // one pass that rewrites x as [N][B rounded up to 8] at the front of the workspace; the rows
        // of the copy are 16-byte aligned, so every kernel family takes its fast loads
        const int64_t ldt = tsvd_round_up(B, 8);
        const dim3 grid((unsigned)((h->hd.N + 31) / 32), (unsigned)((ldt + 31) / 32));
        if (x_dtype == TSVD_BF16)
            hipLaunchKernelGGL(tsvd_transpose_kernel<uint16_t>, grid, dim3(256), 0, s, static_cast<const uint16_t*>(x_dev), ldx,
                               (int)B, (int)h->hd.N, static_cast<uint16_t*>(ws), ldt);
        else
            hipLaunchKernelGGL(tsvd_transpose_kernel<uint32_t>, grid, dim3(256), 0, s, static_cast<const uint32_t*>(x_dev), ldx,
                               (int)B, (int)h->hd.N, static_cast<uint32_t*>(ws), ldt);
        if (hipGetLastError() != hipSuccess) return TSVD_EDEVICE;
        x_dev = ws;
        ldx = ldt;
        ws = static_cast<uint8_t*>(ws) + transposed_bytes(h, B, x_dtype);
    } else if (x_dtype == TSVD_BF16 && use_gemm(h, B, x_dtype) && (ldx % 8 != 0 || (reinterpret_cast<uintptr_t>(x_dev) & 15u)) && env_int("TSVD_REALIGN", 1) != 0 &&
             h->hd.N <= 65535) {
        // more than 16 tokens in rows that are not 16-byte aligned: one pass that copies them to aligned rows costs
        // less than the element-wise gathers of the kernels that take such rows (stage V of a 4096 x 8192
        // factor at 300 tokens: 251 us gathered, 3 + 35 us copied); TSVD_REALIGN=0 keeps the gathers
        const int64_t ldt = tsvd_round_up(B, 8);
        hipLaunchKernelGGL(tsvd_realign_kernel, dim3((unsigned)((ldt + 255) / 256), (unsigned)h->hd.N), dim3(256), 0, s,
                           static_cast<const uint16_t*>(x_dev), (long long)ldx, (int)B, static_cast<uint16_t*>(ws), (long long)ldt);
        if (hipGetLastError() != hipSuccess) return TSVD_EDEVICE;
        x_dev = ws;
        ldx = ldt;
        ws = static_cast<uint8_t*>(ws) + transposed_bytes(h, B, x_dtype);
    }
    if (!x_in_place && use_mid(h, B, x_dtype, ldx)) return forward_mid(h, x_dev, B, ldx, y_dev, ldy, oo, ws, s);
    if (use_gemm(h, B, x_dtype)) {
        tsvd_gemm_problem g;
        g.blob = h->blob;
        g.hd = &h->hd;
        g.bound_V = h->bound_V;
        g.x = x_dev;
        g.B = B;
        g.ldx = ldx;
        g.x_token_major = x_in_place;
        g.x_f32 = x_dtype == TSVD_F32;
        g.y = y_dev;
        g.ldy = ldy;
        g.bias = oo.bias;
        g.out_bf16 = oo.out_bf16;
        g.y_token_major = oo.token_major;
        g.ws = ws;
        g.cu_count = h->cu_count;
        g.clocks = h->clocks;
        const hipError_t ge = tsvd_forward_gemm(g, s);
        return ge == hipSuccess ? TSVD_OK : ge == hipErrorNotSupported ? TSVD_EUNSUPPORTED : TSVD_EDEVICE;
    }
    return forward_skinny(h, x_dev, x_dtype, B, ldx, y_dev, ldy, oo, ws, s);
}

extern "C" tsvd_status tsvd_forward(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, int64_t B,
                                    int64_t ldx, void* y_dev, tsvd_dtype y_dtype, int64_t ldy, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    return tsvd_forward_ex(h, x_dev, x_dtype, TSVD_FEATURE_MAJOR, B, ldx, nullptr, y_dev, y_dtype, ldy, workspace,
                           workspace_bytes, stream);
}

extern "C" tsvd_status tsvd_forward_noalloc(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                                            int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                                            int64_t ldy, void* stream) {
    if (!h || B <= 0) return TSVD_EINVAL;
    if (x_dtype != TSVD_F32 && x_dtype != TSVD_BF16) return TSVD_EINVAL;
    if (x_layout != TSVD_FEATURE_MAJOR && x_layout != TSVD_TOKEN_MAJOR) return TSVD_EINVAL;
    if (h->device < 0 || h->device >= 64 || !noalloc_ptr[h->device]) return TSVD_EDEVICE;
    bool slow_f32 = false;
    if (tsvd_workspace_bytes_ex(h, B, x_dtype, x_layout) > (size_t)TSVD_NOALLOC_MAX_WORKSPACE) {
        // an fp32 batch whose planes do not fit can still go one token at a time (a small workspace)
        if (x_dtype != TSVD_F32) return TSVD_ETOOLARGE;
        f32_one_token_at_a_time = slow_f32 = true;
        if (tsvd_workspace_bytes_ex(h, B, x_dtype, x_layout) > (size_t)TSVD_NOALLOC_MAX_WORKSPACE) {
            f32_one_token_at_a_time = false;
            return TSVD_ETOOLARGE;
        }
    }
    // the workspace contents are undefined on entry for every kernel family (each writes z before it
    // reads it), so nothing has to be cleared between calls
    const tsvd_status st = tsvd_forward_ex(h, x_dev, x_dtype, x_layout, B, ldx, bias_dev, y_dev, y_dtype, ldy, noalloc_ptr[h->device],
                                           (size_t)TSVD_NOALLOC_MAX_WORKSPACE, stream);
    if (slow_f32) f32_one_token_at_a_time = false;
    return st;
}

// ---- diagnostic interface (include/tsvd_tuning.h) ------------------------------------------------
namespace {
const char* const tuning_names[] = {
    "TSVD_GEMV", "TSVD_GEMV_FUSED", "TSVD_GEMV_ONEPASS", "TSVD_GEMV_SW", "TSVD_GEMV_KWLOG2", "TSVD_SKINNY_SW", "TSVD_SKINNY_KW",
    "TSVD_MID", "TSVD_MID_MAX_B", "TSVD_MID_SW", "TSVD_MID_KWLOG2", "TSVD_MID_RESIDENT", "TSVD_GEMM_MIN_B", "TSVD_GEMM_MIN_B_F32",
    "TSVD_GEMM_CFG_V", "TSVD_GEMM_CFG_U", "TSVD_FUSEMAX", "TSVD_COLMAX_SCALAR", "TSVD_REALIGN", "TSVD_PANEL",
    "TSVD_PANEL_WAVES", "TSVD_PANEL_FP6", "TSVD_FP6", "TSVD_FP6_V", "TSVD_FP6_TALL", "TSVD_FP6_PLANES", "TSVD_FP6_DIRECT", "TSVD_FP6_TAIL", "TSVD_TOKEN_MAJOR_COPY", "TSVD_GROUPED_PAIR", "TSVD_CLOCKS",
    "TSVD_SPIN_LIMIT", "TSVD_DENSE_U", "TSVD_EARLY_TILES"};
constexpr int tuning_count = (int)(sizeof tuning_names / sizeof tuning_names[0]);
int tuning_value[tuning_count];
bool tuning_is_set[tuning_count];
int tuning_active = 0;                 // number of switches set: 0 in every process that never calls tsvd_tuning_set
thread_local int stage_mask_now = 7;
}  // namespace

int tsvd_tune(const char* name, int fallback) {
    if (tuning_active == 0) return fallback;
    for (int i = 0; i < tuning_count; ++i)
        if (tuning_is_set[i] && std::strcmp(name, tuning_names[i]) == 0) return tuning_value[i];
    return fallback;
}
int tsvd_stage_mask() { return stage_mask_now; }

extern "C" int tsvd_tuning_set(const char* name, int value) {
    if (!name) return 1;
    for (int i = 0; i < tuning_count; ++i)
        if (std::strcmp(name, tuning_names[i]) == 0) {
            if (!tuning_is_set[i]) ++tuning_active;
            tuning_is_set[i] = true;
            tuning_value[i] = value;
            return 0;
        }
    return 1;
}

extern "C" void tsvd_tuning_reset(void) {
    for (int i = 0; i < tuning_count; ++i) tuning_is_set[i] = false;
    tuning_active = 0;
}

extern "C" tsvd_status tsvd_tuning_forward_stages(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, tsvd_layout x_layout,
                                                  int64_t B, int64_t ldx, const float* bias_dev, void* y_dev, tsvd_dtype y_dtype,
                                                  int64_t ldy, void* workspace, size_t workspace_bytes, void* stream, int stage_mask) {
    if (stage_mask < 1 || stage_mask > 7) return TSVD_EINVAL;
    stage_mask_now = stage_mask;
    const tsvd_status st = tsvd_forward_ex(h, x_dev, x_dtype, x_layout, B, ldx, bias_dev, y_dev, y_dtype, ldy, workspace,
                                           workspace_bytes, stream);
    stage_mask_now = 7;
    return st;
}

extern "C" int tsvd_tuning_tile_shapes(const tsvd_handle* h, long long B, int* shape_v, int* shape_u) {
    if (!h || !shape_v || !shape_u || B < 1) return 1;
    *shape_v = *shape_u = -1;
    if (use_mid(h, B, TSVD_BF16, tsvd_round_up(B, 8))) return 0;
    if (use_gemm(h, B, TSVD_BF16)) {
        if (tsvd_gemm_use_panel(h->hd.Mp, h->hd.Kp, h->hd.Np, B, h->cu_count, true)) {
            *shape_v = *shape_u = tsvd_gemm_panel_fp6() ? 33 : 32;   // one token-panel launch (33: on fp4 codes x fp6 planes)
        } else {
            *shape_v = tsvd_gemm_tile_shape(h->hd.Kp, B, h->cu_count, true);
            *shape_u = tsvd_gemm_tile_shape(h->hd.Mp, B, h->cu_count, true);
            if (tsvd_gemm_use_fp6(h->hd.Mp, h->hd.Kp, h->hd.Np, B, h->cu_count, true)) *shape_u = 40;   // fp4 x fp6 planes
            if (tsvd_gemm_use_fp6_v(h->hd.Mp, h->hd.Kp, h->hd.Np, B, h->cu_count, true)) *shape_v = 40;
        }
    }
    return 0;
}

const uint8_t* tsvd_internal_blob(const tsvd_handle* h, const tsvd_blob_header** hd) {
    *hd = &h->hd;
    return h->blob;
}

extern "C" int tsvd_tuning_read_clocks(const tsvd_handle* h, long long* out, int workgroups) {
    if (!h || !h->clocks || !out || workgroups < 1 || workgroups > TSVD_GEMV_MAX_GRID) return 1;
    return hipMemcpy(out, h->clocks, (size_t)workgroups * 16 * sizeof(long long), hipMemcpyDeviceToHost) == hipSuccess ? 0 : 4;
}

extern "C" void tsvd_free(tsvd_handle* h) {
    if (!h) return;
    if (h->scratch) (void)hipFree(h->scratch);
    for (int r = 0; r < h->retired_count; ++r) (void)hipFree(h->retired[r]);
    if (h->clocks) (void)hipFree(h->clocks);
    if (h->sync) (void)hipFree(h->sync);
    if (h->dense_u) (void)hipFree(h->dense_u);
    if (h->owns_blob && h->blob) (void)hipFree(h->blob);
    delete h;
}
