// Shared constants of the kmq library's own translation units (host packing,
// launch heuristics, kernels).  Not part of the public ABI.
#ifndef KMQ_INTERNAL_H
#define KMQ_INTERNAL_H

#include <cstdint>

#if defined(__HIPCC__)
#define KMQ_HD __host__ __device__
#else
#define KMQ_HD
#endif

namespace kmq {

constexpr int64_t kMaxDim = int64_t(1) << 24;   // N and K are capped so N*K*bits cannot overflow
constexpr int64_t kTileRows = 16;               // KMQ_LAYOUT_TILED: rows per block
constexpr int64_t kTileColWords = 4;            // KMQ_LAYOUT_TILED: words per column block (16 bytes)

inline bool bits_valid(int bits) { return bits >= 1 && bits <= 4; }
inline bool dims_valid(int64_t N, int64_t K) { return N >= 1 && K >= 1 && N <= kMaxDim && K <= kMaxDim; }
KMQ_HD inline int64_t words_per_row(int bits, int64_t K) { return (K * bits + 31) >> 5; }
inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

}  // namespace kmq

#endif
