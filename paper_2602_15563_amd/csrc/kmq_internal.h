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

inline bool bits_valid(int bits) { return bits >= 1 && bits <= 4; }
inline bool dims_valid(int64_t N, int64_t K) { return N >= 1 && K >= 1 && N <= kMaxDim && K <= kMaxDim; }
KMQ_HD inline int64_t words_per_row(int bits, int64_t K) { return (K * bits + 31) >> 5; }

// KMQ_LAYOUT_TILED (see include/kmq.h).  A group is 8 consecutive elements of a
// row = `bits` bytes of the canonical stream; a granule is the `gpg` groups
// {q, q+4, q+8, ...} of one super-block (4*gpg groups) of one row.
KMQ_HD inline int tiled_groups_per_granule(int bits) { return bits == 1 ? 16 : bits == 2 ? 8 : 4; }
KMQ_HD inline int64_t tiled_superblock_elems(int bits) { return 32 * tiled_groups_per_granule(bits); }
KMQ_HD inline bool tiled_valid(int bits, int64_t K) { return K % tiled_superblock_elems(bits) == 0; }
// Byte offset in the tiled stream of canonical byte `byte_in_row` of row n.
KMQ_HD inline int64_t tiled_byte_index(int bits, int64_t K, int64_t n, int64_t byte_in_row) {
    const int64_t gpg = tiled_groups_per_granule(bits);
    const int64_t gb = gpg * bits;                 // bytes per granule
    const int64_t sbb = 4 * gb;                    // bytes per super-block and row
    const int64_t nsb = (K * bits / 8) / sbb;
    const int64_t sb = byte_in_row / sbb, r = byte_in_row % sbb;
    const int64_t g = r / bits, o = r % bits;
    const int64_t q = g % 4, j = g / 4;
    const int64_t rb = n / kTileRows, nn = n % kTileRows;
    return ((rb * nsb + sb) * 64 + q * 16 + nn) * gb + j * bits + o;
}
inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

}  // namespace kmq

#endif
