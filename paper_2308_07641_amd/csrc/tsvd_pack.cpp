// Host-side packer / unpacker of the 2-bit ternary tile format (see tsvd_layout.h).
// Pure host code: usable without a GPU.
#include "tsvd_layout.h"
#include "../../include/tsvd.h"

#include <algorithm>
#include <atomic>
#include <cstring>
#include <thread>
#include <vector>

namespace {

struct Sections {
    int64_t Mp, Kp, Np;
    uint64_t off_S, off_U, off_V, off_nnzU, off_nnzV, total;
    int64_t tilesU, tilesV;
};

bool sections(int64_t M, int64_t K, int64_t N, Sections* s) {
    if (M <= 0 || K <= 0 || N <= 0) return false;
    // keep every tile index and byte offset far inside 63 bits
    if (M > (int64_t(1) << 28) || K > (int64_t(1) << 28) || N > (int64_t(1) << 28)) return false;
    s->Mp = tsvd_round_up(M, TSVD_DIM_ALIGN);
    s->Kp = tsvd_round_up(K, TSVD_DIM_ALIGN);
    s->Np = tsvd_round_up(N, TSVD_DIM_ALIGN);
    s->tilesU = (s->Mp / TSVD_TILE_ROWS) * (s->Kp / TSVD_TILE_COLS);
    s->tilesV = (s->Kp / TSVD_TILE_ROWS) * (s->Np / TSVD_TILE_COLS);
    uint64_t off = sizeof(tsvd_blob_header);
    s->off_S = off;
    off += (uint64_t)tsvd_round_up(s->Kp * 4, 256);
    s->off_U = off;
    off += (uint64_t)s->tilesU * TSVD_TILE_BYTES;
    s->off_V = off;
    off += (uint64_t)s->tilesV * TSVD_TILE_BYTES;
    s->off_nnzU = off;
    off += (uint64_t)tsvd_round_up(s->tilesU * 2, 256);
    s->off_nnzV = off;
    off += (uint64_t)tsvd_round_up(s->tilesV * 2, 256);
    s->total = off;
    return true;
}

unsigned worker_count(int64_t work_items) {
    unsigned hw = std::thread::hardware_concurrency();
    if (hw == 0) hw = 1;
    hw = std::min(hw, 32u);
    if (work_items < 64) return 1;
    return (unsigned)std::min<int64_t>(hw, work_items / 32 + 1);
}

// Packs A [R][C] (row-major, valid part R x C, padded to Rp x Cp) into tiles.  rank_rows / rank_cols: the
// rank K when the rows / columns of A are the rank index (they are stored at tsvd_rank_position), else 0.
// Returns false if an entry is outside {-1,0,+1}.  nnz_total receives the sum of counts.
bool pack_matrix(const int8_t* A, int64_t R, int64_t C, int64_t Rp, int64_t Cp, int64_t rank_rows, int64_t rank_cols,
                 uint32_t* tiles, uint16_t* nnz, int64_t* nnz_total) {
    const int64_t strips = Rp / TSVD_TILE_ROWS, nkt = Cp / TSVD_TILE_COLS;
    std::atomic<bool> bad(false);
    std::atomic<int64_t> total(0);
    auto work = [&](int64_t s0, int64_t s1) {
        int64_t local_total = 0;
        for (int64_t s = s0; s < s1 && !bad.load(std::memory_order_relaxed); ++s) {
            for (int64_t T = 0; T < nkt; ++T) {
                uint32_t* tile = tiles + (s * nkt + T) * (TSVD_TILE_BYTES / 4);
                std::memset(tile, 0, TSVD_TILE_BYTES);
                int count = 0;
                for (int i = 0; i < TSVD_TILE_ROWS; ++i) {
                    const int64_t pr = s * TSVD_TILE_ROWS + i;                      // physical row -> logical row
                    const int64_t r = rank_rows ? tsvd_rank_logical(pr, rank_rows) : pr;
                    if (r >= R) continue;
                    const int64_t c0 = T * TSVD_TILE_COLS;
                    const int8_t* row = A + r * C;
                    for (int64_t c = 0; c < TSVD_TILE_COLS; ++c) {
                        const int64_t col = rank_cols ? tsvd_rank_logical(c0 + c, rank_cols) : c0 + c;
                        if (col >= C) continue;
                        const int v = row[col];
                        if (v == 0) continue;
                        if (v != 1 && v != -1) { bad.store(true); return; }
                        int word, bit;
                        tsvd_code_position(i, (int)c, &word, &bit);
                        tile[word] |= (v > 0 ? 1u : 3u) << bit;
                        ++count;
                    }
                }
                nnz[s * nkt + T] = (uint16_t)count;
                local_total += count;
            }
        }
        total.fetch_add(local_total);
    };
    const unsigned nw = worker_count(strips);
    if (nw <= 1) {
        work(0, strips);
    } else {
        std::vector<std::thread> th;
        const int64_t per = (strips + nw - 1) / nw;
        for (unsigned w = 0; w < nw; ++w) {
            const int64_t a = w * per, b = std::min<int64_t>(strips, a + per);
            if (a < b) th.emplace_back(work, a, b);
        }
        for (auto& t : th) t.join();
    }
    *nnz_total = total.load();
    return !bad.load();
}

// Inverse of pack_matrix for the valid R x C part; verifies padding is zero, no code is 10b
// and the stored counts match.  Returns false on any corruption.
bool unpack_matrix(int8_t* A, int64_t R, int64_t C, int64_t Rp, int64_t Cp, int64_t rank_rows, int64_t rank_cols,
                   const uint32_t* tiles, const uint16_t* nnz, bool check_only) {
    const int64_t strips = Rp / TSVD_TILE_ROWS, nkt = Cp / TSVD_TILE_COLS;
    std::atomic<bool> bad(false);
    auto work = [&](int64_t s0, int64_t s1) {
        for (int64_t s = s0; s < s1 && !bad.load(std::memory_order_relaxed); ++s) {
            for (int64_t T = 0; T < nkt; ++T) {
                const uint32_t* tile = tiles + (s * nkt + T) * (TSVD_TILE_BYTES / 4);
                int count = 0;
                for (int i = 0; i < TSVD_TILE_ROWS; ++i) {
                    const int64_t pr = s * TSVD_TILE_ROWS + i;
                    const int64_t r = rank_rows ? tsvd_rank_logical(pr, rank_rows) : pr;
                    for (int c = 0; c < TSVD_TILE_COLS; ++c) {
                        int word, bit;
                        tsvd_code_position(i, c, &word, &bit);
                        const unsigned code = (tile[word] >> bit) & 3u;
                        const int64_t pc = T * TSVD_TILE_COLS + c;
                        const int64_t col = rank_cols ? tsvd_rank_logical(pc, rank_cols) : pc;
                        const bool inside = r < R && col < C;
                        if (code == 2u || (!inside && code != 0u)) { bad.store(true); return; }
                        if (code) ++count;
                        if (inside && !check_only) A[r * C + col] = code == 0u ? 0 : (code == 1u ? 1 : -1);
                    }
                }
                if (count != nnz[s * nkt + T]) { bad.store(true); return; }
            }
        }
    };
    const unsigned nw = worker_count(strips);
    if (nw <= 1) {
        work(0, strips);
    } else {
        std::vector<std::thread> th;
        const int64_t per = (strips + nw - 1) / nw;
        for (unsigned w = 0; w < nw; ++w) {
            const int64_t a = w * per, b = std::min<int64_t>(strips, a + per);
            if (a < b) th.emplace_back(work, a, b);
        }
        for (auto& t : th) t.join();
    }
    return !bad.load();
}

}  // namespace

extern "C" size_t tsvd_packed_bytes(int64_t M, int64_t K, int64_t N) {
    Sections s;
    return sections(M, K, N, &s) ? (size_t)s.total : 0;
}

extern "C" tsvd_status tsvd_pack_host(const int8_t* U, const float* S, const int8_t* V,
                                      int64_t M, int64_t K, int64_t N, void* blob, size_t blob_bytes) {
    Sections sc;
    if (!U || !S || !V || !blob || !sections(M, K, N, &sc)) return TSVD_EINVAL;
    if (blob_bytes < sc.total) return TSVD_EINVAL;
    uint8_t* base = static_cast<uint8_t*>(blob);

    // Validate before touching the output so that a failure leaves it untouched.
    // (pack_matrix re-validates while packing; this pass is cheap next to it.)
    for (int64_t i = 0; i < M * K; ++i)
        if (U[i] < -1 || U[i] > 1) return TSVD_EVALUE;
    for (int64_t i = 0; i < K * N; ++i)
        if (V[i] < -1 || V[i] > 1) return TSVD_EVALUE;

    std::memset(base, 0, sc.total);
    tsvd_blob_header hd;
    std::memset(&hd, 0, sizeof hd);
    hd.magic = TSVD_MAGIC;
    hd.version = TSVD_FORMAT_VERSION;
    hd.header_bytes = sizeof hd;
    hd.M = M; hd.K = K; hd.N = N;
    hd.Mp = sc.Mp; hd.Kp = sc.Kp; hd.Np = sc.Np;
    hd.off_S = sc.off_S; hd.off_U = sc.off_U; hd.off_V = sc.off_V;
    hd.off_nnzU = sc.off_nnzU; hd.off_nnzV = sc.off_nnzV;
    hd.total_bytes = sc.total;

    {
        float* Sp = reinterpret_cast<float*>(base + sc.off_S);
        for (int64_t k = 0; k < K; ++k) Sp[tsvd_rank_position(k, K)] = S[k];
    }
    if (!pack_matrix(U, M, K, sc.Mp, sc.Kp, 0, K, reinterpret_cast<uint32_t*>(base + sc.off_U),
                     reinterpret_cast<uint16_t*>(base + sc.off_nnzU), &hd.nnzU))
        return TSVD_EVALUE;
    if (!pack_matrix(V, K, N, sc.Kp, sc.Np, K, 0, reinterpret_cast<uint32_t*>(base + sc.off_V),
                     reinterpret_cast<uint16_t*>(base + sc.off_nnzV), &hd.nnzV))
        return TSVD_EVALUE;
    std::memcpy(base, &hd, sizeof hd);
    return TSVD_OK;
}

extern "C" tsvd_status tsvd_unpack_host(const void* blob, size_t blob_bytes, int8_t* U, float* S,
                                        int8_t* V, int64_t* M, int64_t* K, int64_t* N) {
    if (!blob || blob_bytes < sizeof(tsvd_blob_header)) return TSVD_EINVAL;
    tsvd_blob_header hd;
    std::memcpy(&hd, blob, sizeof hd);
    if (hd.magic != TSVD_MAGIC || hd.version != TSVD_FORMAT_VERSION || hd.header_bytes != sizeof hd)
        return TSVD_EINVAL;
    Sections sc;
    if (!sections(hd.M, hd.K, hd.N, &sc)) return TSVD_EINVAL;
    if (sc.total != hd.total_bytes || blob_bytes < sc.total || sc.Mp != hd.Mp || sc.Kp != hd.Kp ||
        sc.Np != hd.Np || sc.off_S != hd.off_S || sc.off_U != hd.off_U || sc.off_V != hd.off_V ||
        sc.off_nnzU != hd.off_nnzU || sc.off_nnzV != hd.off_nnzV)
        return TSVD_EINVAL;
    const uint8_t* base = static_cast<const uint8_t*>(blob);
    if (U || S || V) {
        // S padding must be zero: the kernels rely on it.
        const float* Sp = reinterpret_cast<const float*>(base + sc.off_S);
        for (int64_t pos = 0; pos < sc.Kp; ++pos) {
            if (tsvd_rank_logical(pos, hd.K) < hd.K) continue;
            uint32_t bits;
            std::memcpy(&bits, Sp + pos, 4);
            if (bits != 0) return TSVD_EVALUE;
        }
        if (!unpack_matrix(U, hd.M, hd.K, sc.Mp, sc.Kp, 0, hd.K, reinterpret_cast<const uint32_t*>(base + sc.off_U),
                           reinterpret_cast<const uint16_t*>(base + sc.off_nnzU), U == nullptr))
            return TSVD_EVALUE;
        if (!unpack_matrix(V, hd.K, hd.N, sc.Kp, sc.Np, hd.K, 0, reinterpret_cast<const uint32_t*>(base + sc.off_V),
                           reinterpret_cast<const uint16_t*>(base + sc.off_nnzV), V == nullptr))
            return TSVD_EVALUE;
        if (S)
            for (int64_t k = 0; k < hd.K; ++k) std::memcpy(S + k, Sp + tsvd_rank_position(k, hd.K), sizeof(float));
    }
    if (M) *M = hd.M;
    if (K) *K = hd.K;
    if (N) *N = hd.N;
    return TSVD_OK;
}

// ---- denser code of U: five ternary elements per byte (3^5 = 243 <= 256), 1.6 bits per element --------
// Layout: groups of five consecutive 16-row strips; group-tile (G, T) = the five 1-KiB tiles (strips 5 G .. 5 G + 4,
// tile column T) recoded into 4 KiB: [4 chunks][64 lanes][16 bytes].  A lane's 64 bytes hold its 320 codes
// q = 64 t + 16 w + n (t = strip in the group, w = word of the lane in the 2-bit tile, n = code in the word), five
// per byte: byte j = sum_i trit(q = 5 j + i) 3^i with trit 0 / 1 / 2 for the elements 0 / +1 / -1.
namespace {
constexpr int DENSE_GROUP = 5;
int64_t dense_groups(int64_t M) { return (tsvd_round_up(M, TSVD_DIM_ALIGN) / TSVD_TILE_ROWS + DENSE_GROUP - 1) / DENSE_GROUP; }

void dense_from_tiles(const uint32_t* tiles, int64_t strips, int64_t nkt, uint8_t* out) {
    const int64_t groups = (strips + DENSE_GROUP - 1) / DENSE_GROUP;
    for (int64_t G = 0; G < groups; ++G)
        for (int64_t T = 0; T < nkt; ++T) {
            uint8_t* gt = out + (G * nkt + T) * 4096;
            for (int lane = 0; lane < 64; ++lane)
                for (int j = 0; j < 64; ++j) {
                    unsigned value = 0, pw = 1;
                    for (int i = 0; i < 5; ++i, pw *= 3) {
                        const int q = 5 * j + i, t = q >> 6, w = (q >> 4) & 3, n = q & 15;
                        const int64_t strip = G * DENSE_GROUP + t;
                        unsigned code = 0;
                        if (strip < strips) code = (tiles[(strip * nkt + T) * 256 + lane * 4 + w] >> (2 * n)) & 3u;
                        value += (code == 0 ? 0u : code == 1 ? 1u : 2u) * pw;
                    }
                    gt[(j >> 4) * 1024 + lane * 16 + (j & 15)] = (uint8_t)value;
                }
        }
}

// Inverse; false if a byte is not a valid code (>= 243) or a padding strip is not empty.
bool tiles_from_dense(const uint8_t* in, int64_t strips, int64_t nkt, uint32_t* tiles) {
    const int64_t groups = (strips + DENSE_GROUP - 1) / DENSE_GROUP;
    std::memset(tiles, 0, (size_t)(strips * nkt) * 1024);
    for (int64_t G = 0; G < groups; ++G)
        for (int64_t T = 0; T < nkt; ++T) {
            const uint8_t* gt = in + (G * nkt + T) * 4096;
            for (int lane = 0; lane < 64; ++lane)
                for (int j = 0; j < 64; ++j) {
                    unsigned value = gt[(j >> 4) * 1024 + lane * 16 + (j & 15)];
                    if (value >= 243u) return false;
                    for (int i = 0; i < 5; ++i, value /= 3) {
                        const unsigned trit = value % 3u;
                        if (!trit) continue;
                        const int q = 5 * j + i, t = q >> 6, w = (q >> 4) & 3, n = q & 15;
                        const int64_t strip = G * DENSE_GROUP + t;
                        if (strip >= strips) return false;
                        tiles[(strip * nkt + T) * 256 + lane * 4 + w] |= (trit == 1 ? 1u : 3u) << (2 * n);
                    }
                }
        }
    return true;
}
}  // namespace

extern "C" size_t tsvd_dense_bytes(int64_t M, int64_t K) {
    if (M <= 0 || K <= 0 || M > (int64_t(1) << 30) || K > (int64_t(1) << 30)) return 0;
    return (size_t)(dense_groups(M) * (tsvd_round_up(K, TSVD_DIM_ALIGN) / TSVD_TILE_COLS)) * 4096;
}

extern "C" tsvd_status tsvd_dense_pack_host(const int8_t* U, int64_t M, int64_t K, void* blob, size_t blob_bytes) {
    const size_t need = tsvd_dense_bytes(M, K);
    if (!U || !blob || need == 0 || blob_bytes < need) return TSVD_EINVAL;
    for (int64_t i = 0; i < M * K; ++i)
        if (U[i] < -1 || U[i] > 1) return TSVD_EVALUE;
    const int64_t Mp = tsvd_round_up(M, TSVD_DIM_ALIGN), Kp = tsvd_round_up(K, TSVD_DIM_ALIGN);
    const int64_t strips = Mp / TSVD_TILE_ROWS, nkt = Kp / TSVD_TILE_COLS;
    std::vector<uint32_t> tiles((size_t)(strips * nkt) * 256);
    std::vector<uint16_t> nnz((size_t)(strips * nkt));
    int64_t total = 0;
    if (!pack_matrix(U, M, K, Mp, Kp, 0, K, tiles.data(), nnz.data(), &total)) return TSVD_EVALUE;
    dense_from_tiles(tiles.data(), strips, nkt, static_cast<uint8_t*>(blob));
    return TSVD_OK;
}

extern "C" tsvd_status tsvd_dense_unpack_host(const void* blob, size_t blob_bytes, int8_t* U, int64_t M, int64_t K) {
    const size_t need = tsvd_dense_bytes(M, K);
    if (!U || !blob || need == 0 || blob_bytes < need) return TSVD_EINVAL;
    const int64_t Mp = tsvd_round_up(M, TSVD_DIM_ALIGN), Kp = tsvd_round_up(K, TSVD_DIM_ALIGN);
    const int64_t strips = Mp / TSVD_TILE_ROWS, nkt = Kp / TSVD_TILE_COLS;
    std::vector<uint32_t> tiles((size_t)(strips * nkt) * 256);
    if (!tiles_from_dense(static_cast<const uint8_t*>(blob), strips, nkt, tiles.data())) return TSVD_EVALUE;
    std::vector<uint16_t> nnz((size_t)(strips * nkt));
    for (int64_t t = 0; t < strips * nkt; ++t) {                 // the counts unpack_matrix checks against
        int c = 0;
        for (int w = 0; w < 256; ++w) {
            const uint32_t v = tiles[(size_t)t * 256 + w];
            c += __builtin_popcount(v & 0x55555555u);
        }
        nnz[(size_t)t] = (uint16_t)c;
    }
    return unpack_matrix(U, M, K, Mp, Kp, 0, K, tiles.data(), nnz.data(), false) ? TSVD_OK : TSVD_EVALUE;
}

// Recodes the packed tiles of U inside a blob of tsvd_pack_host (internal: tsvd_pack uploads the result).
void tsvd_internal_dense_from_blob(const void* blob, void* out) {
    tsvd_blob_header hd;
    std::memcpy(&hd, blob, sizeof hd);
    dense_from_tiles(reinterpret_cast<const uint32_t*>(static_cast<const uint8_t*>(blob) + hd.off_U), hd.Mp / TSVD_TILE_ROWS,
                     hd.Kp / TSVD_TILE_COLS, static_cast<uint8_t*>(out));
}

extern "C" const char* tsvd_strerror(tsvd_status s) {
    switch (s) {
        case TSVD_OK: return "ok";
        case TSVD_EINVAL: return "invalid argument";
        case TSVD_EVALUE: return "entry of U or V outside {-1,0,+1}, or corrupt packed code";
        case TSVD_ENOMEM: return "host memory allocation failed";
        case TSVD_EDEVICE: return "HIP call failed";
        case TSVD_EUNSUPPORTED: return "unsupported request";
        case TSVD_ETOOLARGE: return "the call needs more workspace than the fixed array of tsvd_forward_noalloc holds";
    }
    return "unknown status";
}
