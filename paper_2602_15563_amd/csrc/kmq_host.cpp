// Host-side, integer-only part of the kmq library: canonical packing (the
// element stream of App. E's reference routine, widened to 32-bit words and to
// 3-bit fields) and the reversible GPU tile order.  See include/kmq.h for the
// format and the contract of every function.
#include <cstdint>
#include <cstring>

#include "kmq.h"
#include "kmq_internal.h"

extern "C" {

int64_t kmq_words_per_row(int bits, int64_t K) {
    if (!kmq::bits_valid(bits) || K < 0 || K > kmq::kMaxDim) return -1;
    return kmq::words_per_row(bits, K);
}

kmq_status kmq_pack(const uint8_t* idx, int64_t N, int64_t K, int bits, uint32_t* packed) {
    if (!idx || !packed) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K)) return KMQ_ERR_SHAPE;
    const int64_t wpr = kmq::words_per_row(bits, K);
    const uint32_t limit = 1u << bits;
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t* src = idx + n * K;
        uint32_t* dst = packed + n * wpr;
        // 64-bit shift register: fields are appended at `fill`, whole words drained.
        uint64_t reg = 0;
        int fill = 0;
        int64_t w = 0;
        for (int64_t k = 0; k < K; ++k) {
            const uint32_t v = src[k];
            if (v >= limit) return KMQ_ERR_INDEX_RANGE;
            reg |= static_cast<uint64_t>(v) << fill;
            fill += bits;
            if (fill >= 32) {
                dst[w++] = static_cast<uint32_t>(reg);
                reg >>= 32;
                fill -= 32;
            }
        }
        if (fill > 0) dst[w++] = static_cast<uint32_t>(reg);   // zero-padded tail
    }
    return KMQ_OK;
}

kmq_status kmq_unpack(const uint32_t* packed, int64_t N, int64_t K, int bits, uint8_t* idx) {
    if (!idx || !packed) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K)) return KMQ_ERR_SHAPE;
    const int64_t wpr = kmq::words_per_row(bits, K);
    const uint32_t mask = (1u << bits) - 1u;
    for (int64_t n = 0; n < N; ++n) {
        const uint32_t* src = packed + n * wpr;
        uint8_t* dst = idx + n * K;
        uint64_t reg = 0;
        int have = 0;
        int64_t w = 0;
        for (int64_t k = 0; k < K; ++k) {
            if (have < bits) {
                reg |= static_cast<uint64_t>(src[w++]) << have;
                have += 32;
            }
            dst[k] = static_cast<uint8_t>(reg & mask);
            reg >>= bits;
            have -= bits;
        }
    }
    return KMQ_OK;
}

int64_t kmq_tiled_words(int64_t N, int64_t K, int bits, int layout) {
    if (!kmq::bits_valid(bits) || !kmq::dims_valid(N, K)) return -1;
    const int64_t wpr = kmq::words_per_row(bits, K);
    if (layout == KMQ_LAYOUT_CANONICAL) return N * wpr;
    if (layout == KMQ_LAYOUT_TILED) {
        if (!kmq::tiled_valid(bits, K)) return -1;
        return kmq::round_up(N, kmq::kTileRows) * wpr;
    }
    if (layout == KMQ_LAYOUT_ROWLANE) {
        if (!kmq::rowlane_valid(bits, K)) return -1;
        return kmq::round_up(N, kmq::kTileRows) * wpr;
    }
    return -1;
}

static kmq_status repack_impl(const uint32_t* src, int64_t N, int64_t K, int bits, int layout,
                              uint32_t* dst, bool forward) {
    if (!src || !dst) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K)) return KMQ_ERR_SHAPE;
    const int64_t wpr = kmq::words_per_row(bits, K);
    if (layout == KMQ_LAYOUT_CANONICAL) {
        std::memcpy(dst, src, static_cast<size_t>(N * wpr) * sizeof(uint32_t));
        return KMQ_OK;
    }
    if (layout == KMQ_LAYOUT_ROWLANE) {
        if (!kmq::rowlane_valid(bits, K)) return KMQ_ERR_LAYOUT;
    } else if (layout != KMQ_LAYOUT_TILED || !kmq::tiled_valid(bits, K)) {
        return KMQ_ERR_LAYOUT;
    }
    const int64_t nrows_padded = kmq::round_up(N, kmq::kTileRows);
    if (forward) std::memset(dst, 0, static_cast<size_t>(nrows_padded * wpr) * sizeof(uint32_t));
    else         std::memset(dst, 0, static_cast<size_t>(N * wpr) * sizeof(uint32_t));
    const uint32_t* canon = forward ? src : dst;
    uint32_t* canon_out = forward ? nullptr : dst;
    const uint32_t* tiled_in = forward ? nullptr : src;
    uint32_t* tiled_out = forward ? dst : nullptr;
    const bool rowlane = layout == KMQ_LAYOUT_ROWLANE;
    const int gpg = rowlane ? 1 : kmq::tiled_groups_per_granule(bits);
    const int64_t ce = rowlane ? kmq::kRowlaneChunk : 1;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = (k % (32 * gpg)) / 8;
            const int j = static_cast<int>(g / 4), e = static_cast<int>(k % 8);
            const int64_t gd = rowlane ? kmq::rowlane_chunk_dword(bits, K, n, k) : kmq::tiled_granule_dword(bits, K, n, k);
            for (int t = 0; t < bits; ++t) {
                const int64_t cp = k * bits + t;                       // canonical stream bit of this row
                const int tp = rowlane ? kmq::rowlane_bit_position(bits, static_cast<int>(k % ce), t)
                                       : kmq::tiled_bit_position(bits, j, e, t);
                if (forward) {
                    const uint32_t bit = (canon[n * wpr + (cp >> 5)] >> (cp & 31)) & 1u;
                    tiled_out[gd + (tp >> 5)] |= bit << (tp & 31);
                } else {
                    const uint32_t bit = (tiled_in[gd + (tp >> 5)] >> (tp & 31)) & 1u;
                    canon_out[n * wpr + (cp >> 5)] |= bit << (cp & 31);
                }
            }
        }
    }
    return KMQ_OK;
}

kmq_status kmq_repack(const uint32_t* canonical, int64_t N, int64_t K, int bits, int layout,
                      uint32_t* tiled) {
    return repack_impl(canonical, N, K, bits, layout, tiled, true);
}

kmq_status kmq_unrepack(const uint32_t* tiled, int64_t N, int64_t K, int bits, int layout,
                        uint32_t* canonical) {
    return repack_impl(tiled, N, K, bits, layout, canonical, false);
}

const char* kmq_status_string(kmq_status s) {
    switch (s) {
        case KMQ_OK: return "ok";
        case KMQ_ERR_NULL: return "null pointer";
        case KMQ_ERR_BITS: return "bits must be 1, 2, 3, 4 or 8";
        case KMQ_ERR_SHAPE: return "bad shape (N, K >= 1; 1 <= M <= 16)";
        case KMQ_ERR_ALIGN: return "misaligned pointer";
        case KMQ_ERR_INDEX_RANGE: return "index out of range for this bit-width";
        case KMQ_ERR_WORKSPACE: return "workspace missing or too small";
        case KMQ_ERR_LAYOUT: return "unknown layout, or layout invalid for this shape";
        case KMQ_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

}  // extern "C"
