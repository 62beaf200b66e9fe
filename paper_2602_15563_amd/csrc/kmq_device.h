// Device-side helpers shared by the kmq kernels (gfx950 only).
#ifndef KMQ_DEVICE_H
#define KMQ_DEVICE_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "kmq.h"
#include "kmq_internal.h"

namespace kmq {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((ext_vector_type(3))) uint32_t u32x3_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16 bit pattern, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16, quiet = (u >> 16) | 0x40u;
    return static_cast<uint16_t>((u & 0x7FFFFFFFu) > 0x7F800000u ? quiet : rounded);   // (a select, not a branch)
}

// acc + w.lo*x.lo + w.hi*x.hi on packed bf16 pairs, fp32 accumulate (v_dot2c_f32_bf16).
__device__ __forceinline__ float dot2_bf16(uint32_t w, uint32_t x, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w),
                                           __builtin_bit_cast(bf16x2_t, x), acc, false);
}

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, true));
}

// Sum over groups of LANES consecutive lanes (16, 32 or 64) with DPP adds.
// The result is valid in the LAST lane of each group.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror: every lane of a 16-lane row holds the row sum
    if (LANES >= 32) v += dpp_move<0x142, 0xA>(v);   // row_bcast15 into rows 1 and 3
    if (LANES >= 64) v += dpp_move<0x143, 0xC>(v);   // row_bcast31 into rows 2 and 3
    return v;
}

// Index of element k of row n read from the tiled stream (slow path: used by the
// shape-agnostic kernels only).
__device__ __forceinline__ uint32_t tiled_fetch_index(const uint32_t* W, int bits, int64_t K, int64_t n, int64_t k) {
    const int gpg = tiled_groups_per_granule(bits);
    const int64_t g = (k % (32 * gpg)) / 8;
    const int j = static_cast<int>(g / 4), e = static_cast<int>(k % 8);
    const uint32_t* gr = W + tiled_granule_dword(bits, K, n, k);
    uint32_t v = 0;
    for (int t = 0; t < bits; ++t) {
        const int tp = tiled_bit_position(bits, j, e, t);
        v |= ((gr[tp >> 5] >> (tp & 31)) & 1u) << t;
    }
    return v;
}

}  // namespace kmq

#endif
