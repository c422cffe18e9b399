// Host-sanitizer driver (tests/test_host_sanitizers.py compiles this with g++ -fsanitize=address,undefined
// together with the library's host sources and the C oracle, and runs it): every host entry point on
// ragged and extreme shapes, with outputs in exactly-sized heap buffers so that any access past an end
// is caught.  Agreement between the library and the oracle is checked too; exit status 0 = clean.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <vector>

#include "spqt.h"
#include "spqt_colblock.h"

extern "C" {
int64_t spqt_oracle_packed_bytes_g(int64_t M, int64_t K, int G);
int spqt_oracle_pack_g(const uint8_t *q_rowmajor, const uint16_t *scales, int64_t M, int64_t K, int G, uint8_t *out);
int spqt_oracle_unpack_g(const uint8_t *packed, int64_t M, int64_t K, int G, uint8_t *q_rowmajor, uint16_t *scales);
int64_t spqt_oracle_gather(const uint16_t *x, int64_t K, int batch, float thr, int32_t *idx);
void spqt_oracle_gemv(const uint8_t *q_rowmajor, const uint16_t *scales, int64_t M, int64_t K, int G, const uint16_t *x,
                      int batch, float thr, double *y);
}

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "sanitize_driver: %s failed at line %d\n", #c, __LINE__); std::exit(1); } } while (0)

static void group_layout(int64_t M, int64_t K, int G) {
    // exact-size heap buffers: M need not be a multiple of 256
    std::vector<uint8_t> q((size_t)M * K / 2);
    std::vector<uint16_t> sc((size_t)M * (K / G));
    for (auto &b : q) b = (uint8_t)rnd();
    for (auto &s : sc) s = (uint16_t)rnd();
    size_t nbytes = 0;
    REQUIRE(spqt_packed_bytes(M, K, G, &nbytes) == SPQT_OK);
    const bool whole = M % 256 == 0;
    if (whole) REQUIRE((int64_t)nbytes == spqt_oracle_packed_bytes_g(M, K, G));
    std::vector<uint8_t> packed(nbytes), q2(q.size());
    std::vector<uint16_t> sc2(sc.size());
    REQUIRE(spqt_pack(q.data(), sc.data(), M, K, G, packed.data(), nbytes) == SPQT_OK);
    REQUIRE(spqt_pack(q.data(), sc.data(), M, K, G, packed.data(), nbytes - 1) == SPQT_ESIZE);
    REQUIRE(spqt_unpack(packed.data(), M, K, G, q2.data(), sc2.data()) == SPQT_OK);
    REQUIRE(q == q2 && sc == sc2);
    if (whole) {
        std::vector<uint8_t> ref(nbytes);
        REQUIRE(spqt_oracle_pack_g(q.data(), sc.data(), M, K, G, ref.data()) == 0);
        REQUIRE(ref == packed);
        REQUIRE(spqt_oracle_unpack_g(ref.data(), M, K, G, q2.data(), sc2.data()) == 0);
        REQUIRE(q == q2 && sc == sc2);
    }
}

static void oracle_gemv(int64_t M, int64_t K) {
    std::vector<uint8_t> q((size_t)M * K / 2);
    std::vector<uint16_t> sc((size_t)M * (K / 128)), x((size_t)2 * K);
    for (auto &b : q) b = (uint8_t)rnd();
    for (auto &s : sc) s = (uint16_t)(0x2000 + rnd() % 0x400);      // small positive fp16
    for (auto &v : x) v = (uint16_t)(rnd() & 0xBFFF);                 // finite fp16, both signs
    x[3] = 0x7C00; x[5] = 0x7E00; x[7] = 0xFC00;                      // +inf, NaN, -inf
    std::vector<int32_t> idx((size_t)K);
    std::vector<double> y((size_t)2 * M);
    for (float thr : {0.0f, 0.5f, std::numeric_limits<float>::infinity()}) {
        const int64_t n = spqt_oracle_gather(x.data(), K, 2, thr, idx.data());
        REQUIRE(n >= 0 && n <= K);
        spqt_oracle_gemv(q.data(), sc.data(), M, K, 128, x.data(), 2, thr, y.data());
    }
}

static void column_blocks(int64_t M, int64_t K) {
    std::vector<float> w((size_t)M * K), back((size_t)M * K);
    for (auto &v : w) v = ((int)(rnd() % 2001) - 1000) * 1e-4f;
    // extremes: zero blocks, one huge value, tiny values that underflow the fp16 scale, negative zero
    for (int64_t k = 0; k < K && k < 64; ++k) w[k] = 0.0f;
    w[(size_t)(M > 1 ? 1 : 0) * K + 1] = 6.0e4f;
    w[(size_t)(M > 2 ? 2 : 0) * K + 2] = 1e-30f;
    w[(size_t)(M > 3 ? 3 : 0) * K + 3] = -0.0f;
    size_t nb = 0;
    REQUIRE(spqt_cb_packed_bytes(M, K, &nb) == SPQT_OK);
    std::vector<uint8_t> p(nb);
    REQUIRE(spqt_cb_quantize(w.data(), M, K, p.data(), nb) == SPQT_OK);
    REQUIRE(spqt_cb_quantize(w.data(), M, K, p.data(), nb - 1) == SPQT_ESIZE);
    REQUIRE(spqt_cb_dequantize(p.data(), M, K, back.data()) == SPQT_OK);
    for (size_t i = 0; i < back.size(); ++i) REQUIRE(std::isfinite(back[i]));
    REQUIRE(spqt_cbk_quantize(w.data(), M, K, p.data(), nb) == SPQT_OK);
    REQUIRE(spqt_cbk_dequantize(p.data(), M, K, back.data()) == SPQT_OK);
    for (size_t i = 0; i < back.size(); ++i) REQUIRE(std::isfinite(back[i]));
    size_t nb8 = 0;
    REQUIRE(spqt_cb8_packed_bytes(M, K, &nb8) == SPQT_OK);
    std::vector<uint8_t> p8(nb8);
    REQUIRE(spqt_cb8_quantize(w.data(), M, K, p8.data(), nb8) == SPQT_OK);
    REQUIRE(spqt_cb8_dequantize(p8.data(), M, K, back.data()) == SPQT_OK);
    for (size_t i = 0; i < back.size(); ++i) REQUIRE(std::isfinite(back[i]));
    size_t nb2 = 0;
    REQUIRE(spqt_cb2_packed_bytes(M, K, &nb2) == SPQT_OK);
    std::vector<uint8_t> p2(nb2);
    REQUIRE(spqt_cb2_quantize(w.data(), M, K, p2.data(), nb2) == SPQT_OK);
    REQUIRE(spqt_cb2_quantize(w.data(), M, K, p2.data(), nb2 - 1) == SPQT_ESIZE);
    REQUIRE(spqt_cb2_dequantize(p2.data(), M, K, back.data()) == SPQT_OK);
    for (size_t i = 0; i < back.size(); ++i) REQUIRE(std::isfinite(back[i]));
}

int main() {
    const int64_t shapes[][2] = {{256, 128}, {1, 128}, {255, 256}, {257, 128}, {300, 384}, {512, 1024}, {1000, 256}};
    for (auto &s : shapes) {
        group_layout(s[0], s[1], 128);
        group_layout(s[0], s[1], 64);
        column_blocks(s[0], s[1]);
    }
    oracle_gemv(256, 128);
    oracle_gemv(512, 384);
    // argument errors are answered, not executed
    size_t n = 0;
    REQUIRE(spqt_packed_bytes(0, 128, 128, &n) == SPQT_ESHAPE);
    REQUIRE(spqt_packed_bytes(256, 100, 128, &n) == SPQT_ESHAPE);
    REQUIRE(spqt_packed_bytes(256, 128, 32, &n) == SPQT_ESHAPE);
    REQUIRE(spqt_pack(nullptr, nullptr, 256, 128, 128, nullptr, 0) == SPQT_EINVAL);
    std::puts("sanitize_driver: clean");
    return 0;
}
