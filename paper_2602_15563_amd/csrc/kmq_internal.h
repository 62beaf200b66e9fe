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

// 1..4 bits everywhere; 8 bits (a 256-entry codebook, one of the element widths of the paper's
// lookup-table kernel, Sec. 3.3) on the canonical layout through the shape-agnostic kernels
inline bool bits_valid(int bits) { return (bits >= 1 && bits <= 4) || bits == 8; }
inline bool dims_valid(int64_t N, int64_t K) { return N >= 1 && K >= 1 && N <= kMaxDim && K <= kMaxDim; }
KMQ_HD inline int64_t words_per_row(int bits, int64_t K) { return (K * bits + 31) >> 5; }
inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

// KMQ_LAYOUT_TILED (see include/kmq.h).  A group is 8 consecutive elements of a
// row; a granule is the `gpg` groups {q, q+4, q+8, ...} of one super-block
// (4*gpg groups) of one row, stored as gpg*bits/4 dwords.
KMQ_HD inline int tiled_groups_per_granule(int bits) { return bits == 1 ? 16 : bits == 2 ? 8 : 4; }
KMQ_HD inline int64_t tiled_superblock_elems(int bits) { return 32 * tiled_groups_per_granule(bits); }
KMQ_HD inline bool tiled_valid(int bits, int64_t K) { return bits <= 4 && K % tiled_superblock_elems(bits) == 0; }

// Dword offset in the tiled stream of the granule that holds element k of row n.
KMQ_HD inline int64_t tiled_granule_dword(int bits, int64_t K, int64_t n, int64_t k) {
    const int64_t gpg = tiled_groups_per_granule(bits);
    const int64_t gw = gpg * bits / 4;             // dwords per granule
    const int64_t sbe = 32 * gpg;
    const int64_t nsb = K / sbe;
    const int64_t sb = k / sbe, g = (k % sbe) / 8, q = g % 4;
    const int64_t rb = n / kTileRows, nn = n % kTileRows;
    return ((rb * nsb + sb) * 64 + q * 16 + nn) * gw;
}

// Inside a granule: bit position (0 .. 32*gw-1, dword-major) of bit t of the index
// of element e (0..7) of step j (0..gpg-1).  1- and 4-bit granules keep the
// canonical order of their groups; 2- and 3-bit granules spread the fields so
// that at most one shift and one AND put four indices into the four bytes of a
// register (a v_perm_b32 selector).
KMQ_HD inline int tiled_bit_position(int bits, int j, int e, int t) {
    switch (bits) {
        case 1: return 8 * j + e;
        case 4: return 32 * j + 4 * e + t;
        case 2: {
            const int c = 2 * j + e / 4, k = e % 4;
            return 32 * (c / 4) + 8 * k + 2 * (c % 4) + t;
        }
        default: {  // 3: steps 0..2 fill bits 0..5 of the bytes of dwords 0..2, step 3 the spare top bits
            const int h = e / 4, p = 8 * (e % 4);
            if (j < 3) return 32 * j + p + 3 * h + t;
            if (h == 0) return t < 2 ? p + 6 + t : 32 + p + 6;
            return t == 0 ? 32 + p + 7 : 64 + p + 5 + t;
        }
    }
}

// KMQ_LAYOUT_ROWLANE (see include/kmq.h).  A chunk is 64 consecutive elements of one row (2*bits
// dwords); a tile is 16 rows x 4 consecutive chunks, stored lane-major: lane kp*16 + r holds chunk
// kp of row r.  The tiles of a 16-row block follow each other along K.
KMQ_HD inline bool rowlane_bits(int bits) { return bits == 1 || bits == 2; }
constexpr int64_t kRowlaneChunk = 64, kRowlaneTile = 4 * kRowlaneChunk;
KMQ_HD inline bool rowlane_valid(int bits, int64_t K) { return rowlane_bits(bits) && K % kRowlaneTile == 0; }

// Dword offset in the row-lane stream of the chunk that holds element k of row n.
KMQ_HD inline int64_t rowlane_chunk_dword(int bits, int64_t K, int64_t n, int64_t k) {
    const int64_t tiles = K / kRowlaneTile;
    const int64_t t = k / kRowlaneTile, kp = (k % kRowlaneTile) / kRowlaneChunk;
    const int64_t rb = n / kTileRows, r = n % kTileRows;
    return ((rb * tiles + t) * 64 + kp * 16 + r) * (2 * bits);
}

// Inside a chunk: bit position (dword-major) of bit t of the index of element c (0..63) of the chunk.
// 2-bit: pairs of elements travel as nibbles; nibble slot s = 8*word + position is consumed against
//        the activation pair that lane s % 16 holds in register s / 16 after an 8-byte load per lane,
//        i.e. pair 2*(s % 16) + s / 16 of the chunk.
// 1-bit: four elements travel as a nibble; slot s = 8*word + 2*byte + view holds elements 4s..4s+3.
//        View 0 nibbles sit at bits 3..6 of each byte; view 1 nibbles at bits 7, 8, 9, 10 (mod 32)
//        above the byte's start, which a rotation of the word by 4 brings to bits 3..6 as well.
KMQ_HD inline int rowlane_bit_position(int bits, int c, int t) {
    if (bits == 2) {
        const int p = c >> 1, e = c & 1;
        const int s = (p >> 1) + 16 * (p & 1);
        return 4 * s + 2 * e + t;
    }
    const int s = c >> 2, i = c & 3;
    const int q = s >> 3, b = (s & 7) >> 1, view = s & 1;
    return 32 * q + (view ? (8 * b + 7 + i) % 32 : 8 * b + 3 + i);
}

}  // namespace kmq

#endif
