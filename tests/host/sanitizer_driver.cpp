// Host-only driver for the packer (tsvd_pack.cpp), built with -fsanitize=address,undefined by
// tests/test_host_sanitizers.py: round trips on ragged shapes, every error path, corrupted blobs.
// Exit status 0 = all checks passed and no sanitizer report (the sanitizers abort the process).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/tsvd.h"

static uint64_t rng_state = 0x2308076412345678ull;
static uint32_t rnd() {                       // xorshift64*: inputs only, no arithmetic of the method
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (uint32_t)((rng_state * 0x2545F4914F6CDD1Dull) >> 32);
}
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static int round_trip(int64_t M, int64_t K, int64_t N) {
    std::vector<int8_t> U((size_t)(M * K)), V((size_t)(K * N)), U2(U.size()), V2(V.size());
    std::vector<float> S((size_t)K), S2((size_t)K);
    for (auto& v : U) v = (int8_t)((int)(rnd() % 3) - 1);
    for (auto& v : V) v = (int8_t)((int)(rnd() % 3) - 1);
    for (auto& v : S) v = (float)(rnd() % 1000) * 0.001f - 0.5f;
    const size_t bytes = tsvd_packed_bytes(M, K, N);
    CHECK(bytes > 0);
    std::vector<unsigned char> blob(bytes);            // exactly as large as promised: an overrun is a report
    CHECK(tsvd_pack_host(U.data(), S.data(), V.data(), M, K, N, blob.data(), bytes) == TSVD_OK);
    int64_t m = 0, k = 0, n = 0;
    CHECK(tsvd_unpack_host(blob.data(), bytes, U2.data(), S2.data(), V2.data(), &m, &k, &n) == TSVD_OK);
    CHECK(m == M && k == K && n == N);
    CHECK(std::memcmp(U.data(), U2.data(), U.size()) == 0 && std::memcmp(V.data(), V2.data(), V.size()) == 0);
    CHECK(std::memcmp(S.data(), S2.data(), S.size() * sizeof(float)) == 0);
    // error paths: short buffers, null pointers, bad values leave the output untouched
    std::vector<unsigned char> small(bytes - 1, 0xAB);
    CHECK(tsvd_pack_host(U.data(), S.data(), V.data(), M, K, N, small.data(), small.size()) == TSVD_EINVAL);
    for (unsigned char c : small) CHECK(c == 0xAB);
    CHECK(tsvd_pack_host(nullptr, S.data(), V.data(), M, K, N, blob.data(), bytes) == TSVD_EINVAL);
    CHECK(tsvd_unpack_host(blob.data(), bytes - 1, U2.data(), S2.data(), V2.data(), nullptr, nullptr, nullptr) == TSVD_EINVAL);
    CHECK(tsvd_unpack_host(blob.data(), 100, nullptr, nullptr, nullptr, &m, &k, &n) == TSVD_EINVAL);
    std::vector<int8_t> Ub = U;
    Ub[(size_t)(rnd() % Ub.size())] = 2;
    std::vector<unsigned char> keep(bytes, 0xCD);
    CHECK(tsvd_pack_host(Ub.data(), S.data(), V.data(), M, K, N, keep.data(), bytes) == TSVD_EVALUE);
    for (unsigned char c : keep) CHECK(c == 0xCD);
    // corrupted blobs: a flipped bit in the code area gives the unused code 10, a non-zero padding code or a
    // count mismatch; a non-zero scale in the padding is refused as well; a damaged header is refused
    for (int t = 0; t < 64; ++t) {
        std::vector<unsigned char> bad = blob;
        const size_t at = 256 + rnd() % (bytes - 256);
        bad[at] ^= (unsigned char)(1u << (rnd() % 8));
        const tsvd_status st = tsvd_unpack_host(bad.data(), bytes, U2.data(), S2.data(), V2.data(), nullptr, nullptr, nullptr);
        CHECK(st == TSVD_OK || st == TSVD_EVALUE);      // (a flipped bit of a valid scale is not detectable)
    }
    {
        std::vector<unsigned char> bad = blob;
        bad[rnd() % 200] ^= 0x55;
        const tsvd_status st = tsvd_unpack_host(bad.data(), bytes, nullptr, nullptr, nullptr, &m, &k, &n);
        CHECK(st == TSVD_OK || st == TSVD_EINVAL);
    }
    return 0;
}

int main() {
    const int64_t shapes[][3] = {{1, 1, 1}, {3, 7, 5}, {16, 16, 256}, {17, 33, 257}, {40, 70, 300}, {300, 513, 70},
                                 {5, 2, 1000}, {260, 345, 129}, {64, 1545, 48}, {33, 128, 31}, {20, 2415, 9}};
    for (const auto& s : shapes)
        if (round_trip(s[0], s[1], s[2])) { std::fprintf(stderr, "shape %lld %lld %lld\n", (long long)s[0], (long long)s[1], (long long)s[2]); return 1; }
    CHECK(tsvd_packed_bytes(0, 1, 1) == 0 && tsvd_packed_bytes(1, -1, 1) == 0);
    for (int s = 0; s < 8; ++s) CHECK(tsvd_strerror((tsvd_status)s) != nullptr);
    std::puts("host sanitizer driver: ok");
    return 0;
}
