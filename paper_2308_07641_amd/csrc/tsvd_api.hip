// C ABI entry points that touch the device: upload, forward dispatch, release.
// (The host-only packer lives in tsvd_pack.cpp.)
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "../../include/tsvd.h"
#include "tsvd_kernels.h"
#include "tsvd_layout.h"

struct tsvd_handle {
    int device;
    tsvd_blob_header hd;
    uint8_t* blob;          // device
    bool owns_blob;
    void* scratch;          // device, handle-owned workspace (grown on demand)
    size_t scratch_bytes;
    float bound_V;          // max_k |S_k| * nnz(V[k,:]) : |z_k| <= bound_V * max|x| for every token
};

namespace {

int env_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : fallback;
}

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// One-time, per-device kernel attribute setup.
hipError_t device_init(int device) {
    static bool done[64] = {};
    if (device < 0 || device >= 64) return hipErrorInvalidDevice;
    if (done[device]) return hipSuccess;
    hipError_t e = tsvd_skinny_init();
    if (e != hipSuccess) return e;
    e = tsvd_gemm_init();
    if (e != hipSuccess) return e;
    done[device] = true;
    return hipSuccess;
}

// ---- skinny path (few tokens): two launches per token chunk ---------------------------------
struct skinny_plan {
    int pieces_x, pieces_z, chunk;   // bf16 parts of x and of z, tokens per launch
};

skinny_plan plan_skinny(int64_t B, tsvd_dtype x_dtype) {
    skinny_plan p;
    p.pieces_x = x_dtype == TSVD_BF16 ? 1 : 3;
    // z is fp32.  Three parts are exact; two parts keep 16 significant bits (2^-17 relative),
    // far inside the bf16-activation tolerance, and let 8 tokens share one pass.
    if (x_dtype == TSVD_F32 || B * 3 <= 16) {
        p.pieces_z = 3;
        p.chunk = 5;
    } else {
        p.pieces_z = 2;
        p.chunk = 8;
    }
    return p;
}

void shape_skinny(tsvd_skinny_args& a, int cols) {
    // LDS budget: activations [cols][slab_k + 8] bf16 + reduction tiles (<= 16 KiB)
    const size_t budget = TSVD_SKINNY_MAX_LDS - 16 * 1024 - 512;
    int slab = (int)std::min<size_t>((size_t)a.nkt, (budget / ((size_t)cols * 2) - 8) / 256);
    a.slab_tiles = std::max(slab, 1);
    // Aim for >= 2 workgroups per compute unit when the matrix allows it, 8..16 wavefronts each.
    int sw = 1;
    while (sw < 4 && a.strips / (sw * 2) >= 512) sw *= 2;
    int kw = 1;
    while (sw * kw * 2 <= 16 && a.nkt / (kw * 2) >= 2) kw *= 2;
    a.sw = std::max(1, std::min(16, env_int("TSVD_SKINNY_SW", sw)));
    a.kw = std::max(1, std::min(16 / a.sw, env_int("TSVD_SKINNY_KW", kw)));
}

tsvd_status forward_skinny(const tsvd_handle* h, const void* x, tsvd_dtype x_dtype, int64_t B, int64_t ldx,
                           float* y, int64_t ldy, void* ws, hipStream_t stream) {
    const tsvd_blob_header& hd = h->hd;
    const skinny_plan pl = plan_skinny(B, x_dtype);
    float* z = static_cast<float*>(ws);   // [K][B] fp32
    const size_t xelt = x_dtype == TSVD_BF16 ? 2 : 4;
    for (int64_t b0 = 0; b0 < B; b0 += pl.chunk) {
        const int tokens = (int)std::min<int64_t>(pl.chunk, B - b0);
        tsvd_skinny_args v;
        std::memset(&v, 0, sizeof v);
        v.tiles = h->blob + hd.off_V;
        v.strips = (int)((hd.K + 15) / 16);
        v.nkt = (int)(hd.Np / 256);
        v.in = static_cast<const uint8_t*>(x) + (size_t)b0 * xelt;
        v.in_is_bf16 = x_dtype == TSVD_BF16;
        v.kvalid = (int)hd.N;
        v.ld_in = ldx;
        v.tokens = tokens;
        v.pieces = pl.pieces_x;
        v.rowscale = reinterpret_cast<const float*>(h->blob + hd.off_S);
        v.post = 0.5f;
        v.out = z + b0;
        v.ld_out = B;
        v.rows_valid = (int)hd.K;
        shape_skinny(v, v.tokens * v.pieces);
        if (tsvd_launch_skinny(v, stream) != hipSuccess) return TSVD_EDEVICE;

        tsvd_skinny_args u;
        std::memset(&u, 0, sizeof u);
        u.tiles = h->blob + hd.off_U;
        u.strips = (int)((hd.M + 15) / 16);
        u.nkt = (int)(hd.Kp / 256);
        u.in = z + b0;
        u.in_is_bf16 = 0;
        u.kvalid = (int)hd.K;
        u.ld_in = B;
        u.tokens = tokens;
        u.pieces = pl.pieces_z;
        u.rowscale = nullptr;
        u.post = 0.5f;
        u.out = y + b0;
        u.ld_out = ldy;
        u.rows_valid = (int)hd.M;
        shape_skinny(u, u.tokens * u.pieces);
        if (tsvd_launch_skinny(u, stream) != hipSuccess) return TSVD_EDEVICE;
    }
    return TSVD_OK;
}

bool use_gemm(const tsvd_handle*, int64_t B, tsvd_dtype x_dtype) {
    const int min_b = env_int("TSVD_GEMM_MIN_B", 64);
    return x_dtype == TSVD_BF16 && B >= min_b;
}

size_t gemm_workspace(const tsvd_handle* h, int64_t B) {
    // partial column maxima [PARTS][Bp] fp32, then Z as fp16 [Kp][Bp]
    const int64_t Bp = tsvd_round_up(B, 256);
    return round256((size_t)TSVD_COLMAX_PARTS * Bp * 4) + round256((size_t)h->hd.Kp * (size_t)Bp * 2);
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
    std::free(host);
    if (!ok) {
        if (h->owns_blob && h->blob) (void)hipFree(h->blob);
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

extern "C" size_t tsvd_workspace_bytes(const tsvd_handle* h, int64_t B, tsvd_dtype x_dtype) {
    if (!h || B <= 0 || (x_dtype != TSVD_F32 && x_dtype != TSVD_BF16)) return 0;
    if (use_gemm(h, B, x_dtype)) return gemm_workspace(h, B);
    return round256((size_t)h->hd.K * (size_t)B * sizeof(float));
}

extern "C" tsvd_status tsvd_forward(const tsvd_handle* h, const void* x_dev, tsvd_dtype x_dtype, int64_t B,
                                    int64_t ldx, void* y_dev, tsvd_dtype y_dtype, int64_t ldy, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    if (!h || !x_dev || !y_dev || B <= 0 || ldx < B || ldy < B) return TSVD_EINVAL;
    if (x_dtype != TSVD_F32 && x_dtype != TSVD_BF16) return TSVD_EINVAL;
    if (y_dtype != TSVD_F32) return y_dtype == TSVD_BF16 ? TSVD_EUNSUPPORTED : TSVD_EINVAL;
    if (B > (int64_t(1) << 24)) return TSVD_EUNSUPPORTED;
    const size_t need = tsvd_workspace_bytes(h, B, x_dtype);
    void* ws = workspace;
    if (ws) {
        if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return TSVD_EINVAL;
    } else {
        if (workspace_bytes != 0) return TSVD_EINVAL;
        tsvd_handle* hm = const_cast<tsvd_handle*>(h);
        if (hm->scratch_bytes < need) {
            // Stream-ordered work may still use the old buffer: drain before replacing it.
            if (hm->scratch) {
                if (hipDeviceSynchronize() != hipSuccess) return TSVD_EDEVICE;
                (void)hipFree(hm->scratch);
                hm->scratch = nullptr;
                hm->scratch_bytes = 0;
            }
            void* d = nullptr;
            if (hipMalloc(&d, need) != hipSuccess) {
                (void)hipGetLastError();
                return TSVD_EDEVICE;
            }
            hm->scratch = d;
            hm->scratch_bytes = need;
        }
        ws = hm->scratch;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (use_gemm(h, B, x_dtype)) {
        tsvd_gemm_problem g;
        g.blob = h->blob;
        g.hd = &h->hd;
        g.bound_V = h->bound_V;
        g.x = x_dev;
        g.B = B;
        g.ldx = ldx;
        g.y = static_cast<float*>(y_dev);
        g.ldy = ldy;
        g.ws = ws;
        return tsvd_forward_gemm(g, s) == hipSuccess ? TSVD_OK : TSVD_EDEVICE;
    }
    return forward_skinny(h, x_dev, x_dtype, B, ldx, static_cast<float*>(y_dev), ldy, ws, s);
}

extern "C" void tsvd_free(tsvd_handle* h) {
    if (!h) return;
    if (h->scratch) (void)hipFree(h->scratch);
    if (h->owns_blob && h->blob) (void)hipFree(h->blob);
    delete h;
}
