// Exercises the host-side (integer-only) part of the library and the CPU oracle under
// AddressSanitizer + UndefinedBehaviorSanitizer: round trips on ragged shapes, every
// bit-width, both layouts, and the error paths.  Built and run by tests/test_host_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "kmq.h"

extern "C" {
int oracle_pack(const uint8_t*, int64_t, int64_t, int, uint32_t*);
int oracle_unpack(const uint32_t*, int64_t, int64_t, int, uint8_t*);
int oracle_gemm(const uint32_t*, const uint16_t*, const uint16_t*, int64_t, int64_t, int, int64_t, int64_t, int64_t,
                double*, double*, uint16_t*);
int oracle_gemm_blockscaled(const uint32_t*, const uint16_t*, const uint16_t*, const uint16_t*, int64_t, int64_t, int,
                            int64_t, int64_t, int64_t, int64_t, int, double*, double*, uint16_t*);
}

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); return 1; } } while (0)

int main() {
    const int64_t Ns[] = {1, 3, 16, 17, 33};
    const int64_t Ks[] = {1, 5, 31, 32, 33, 100, 512, 1024};
    for (int bits = 1; bits <= 4; ++bits)
        for (int64_t N : Ns)
            for (int64_t K : Ks) {
                std::vector<uint8_t> idx(N * K), back(N * K);
                for (auto& v : idx) v = static_cast<uint8_t>(rnd() & ((1u << bits) - 1u));
                const int64_t wpr = kmq_words_per_row(bits, K);
                CHECK(wpr == (K * bits + 31) / 32);
                std::vector<uint32_t> p(N * wpr), po(N * wpr);
                CHECK(kmq_pack(idx.data(), N, K, bits, p.data()) == KMQ_OK);
                CHECK(oracle_pack(idx.data(), N, K, bits, po.data()) == 0);
                CHECK(p == po);                                   // two independent packers agree
                CHECK(kmq_unpack(p.data(), N, K, bits, back.data()) == KMQ_OK);
                CHECK(back == idx);
                const int64_t tw = kmq_tiled_words(N, K, bits, KMQ_LAYOUT_TILED);
                if (tw > 0) {
                    std::vector<uint32_t> t(tw), c(N * wpr);
                    CHECK(kmq_repack(p.data(), N, K, bits, KMQ_LAYOUT_TILED, t.data()) == KMQ_OK);
                    CHECK(kmq_unrepack(t.data(), N, K, bits, KMQ_LAYOUT_TILED, c.data()) == KMQ_OK);
                    CHECK(c == p);
                } else {
                    std::vector<uint32_t> t(1);
                    CHECK(kmq_repack(p.data(), N, K, bits, KMQ_LAYOUT_TILED, t.data()) == KMQ_ERR_LAYOUT);
                }
                // the oracle on the same buffers (reads every word it is entitled to and no more)
                std::vector<uint16_t> cb(N * (1 << bits), 0x3F80), X(2 * K, 0x3F80), yb(2 * N);
                std::vector<double> Y(2 * N), A(2 * N);
                CHECK(oracle_gemm(p.data(), cb.data(), X.data(), N, K, bits, 2, 0, N, Y.data(), A.data(), yb.data()) == 0);
                CHECK(Y[0] == static_cast<double>(K));            // every centroid and every x is 1.0
                if (K % 64 == 0) {
                    std::vector<uint16_t> sc(N * (K / 64), 0x4000), cbs(1 << bits, 0x3F80);
                    CHECK(oracle_gemm_blockscaled(p.data(), cbs.data(), sc.data(), X.data(), N, K, bits, 64, 2, 0, N, 1,
                                                  Y.data(), A.data(), yb.data()) == 0);
                    CHECK(Y[N] == 2.0 * static_cast<double>(K));
                }
            }
    // error paths
    uint8_t one = 9;
    uint32_t w = 0;
    CHECK(kmq_pack(&one, 1, 1, 2, &w) == KMQ_ERR_INDEX_RANGE);
    CHECK(kmq_pack(nullptr, 1, 1, 2, &w) == KMQ_ERR_NULL);
    CHECK(kmq_pack(&one, 1, 1, 7, &w) == KMQ_ERR_BITS);
    CHECK(kmq_pack(&one, 0, 1, 2, &w) == KMQ_ERR_SHAPE);
    CHECK(kmq_words_per_row(5, 10) == -1 && kmq_tiled_words(4, 100, 2, KMQ_LAYOUT_TILED) == -1);
    std::puts("host sanitizer run: ok");
    return 0;
}
