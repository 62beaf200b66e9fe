// Hand-scheduled lookup / multiply-accumulate blocks of the batch-1 table kernels (canonical layout):
// the lookup of paper App. E, "Kernel implementations", as LDS reads issued and consumed in a fixed,
// hand-counted order.  Shared by the kernels specialised on K and by the kernel that loops over K.
#ifndef KMQ_LUT_BLOCKS_H
#define KMQ_LUT_BLOCKS_H

#include <type_traits>

#include "kmq_device.h"

namespace kmq {

typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;

// ---- hand-scheduled blocks -----------------------------------------------------
// `a` holds four address registers whose bytes 1..3 are the table base.

// The LGKM counter of a wave has 4 bits: at most 15 LDS/scalar-memory operations
// may be outstanding, or s_waitcnt lgkmcnt(n) stops meaning what it says.  The
// pipeline below therefore issues lookups in groups of four and never has more
// than 12 in flight.

// 2-bit / 4-bit: four 4-byte lookups, nibbles 4H..4H+3 of `word` (H = 0, 1), into
// v[4H..4H+3]; v[2i] belongs to nibble 2i (even).  re/ro are the rotated words,
// produced when H == 0 and reused when H == 1.
template <int OFF, int H>
__device__ __forceinline__ void issue4_b32(uint32_t word, uint32_t& re, uint32_t& ro, uint32_t (&a)[4],
                                           uint32_t (&v)[8], uint32_t mask) {
    if constexpr (H == 0) {
        asm volatile(
            "v_alignbit_b32 %4, %10, %10, 30\n\t"
            "v_alignbit_b32 %5, %10, %10, 2\n\t"
            "v_and_b32_sdwa %6, %4, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %7, %5, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %8, %4, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %9, %5, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:DWORD\n\t"
            "ds_read_b32 %0, %6 offset:%c12\n\t"
            "ds_read_b32 %1, %7 offset:%c12\n\t"
            "ds_read_b32 %2, %8 offset:%c12\n\t"
            "ds_read_b32 %3, %9 offset:%c12"
            : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(re), "=&v"(ro),
              "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(word), "v"(mask), "n"(OFF));
    } else {
        asm volatile(
            "v_and_b32_sdwa %4, %8, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %5, %9, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %6, %8, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %7, %9, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:DWORD\n\t"
            "ds_read_b32 %0, %4 offset:%c11\n\t"
            "ds_read_b32 %1, %5 offset:%c11\n\t"
            "ds_read_b32 %2, %6 offset:%c11\n\t"
            "ds_read_b32 %3, %7 offset:%c11"
            : "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7]),
              "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(re), "v"(ro), "v"(mask), "n"(OFF));
    }
}

// 3-bit: two neighbouring fields (6 bits) index a table of 64 centroid pairs, so the lookups and
// dot instructions per weight are those of the 2-bit kernel.  Three words hold 16 such pairs;
// quarter Q (0..3) issues pairs 4Q..4Q+3 into v[0..3].  A pair's six bits are moved to bits 2..7
// of some byte by a shift (or a funnel shift where the pair straddles two words), from where the
// byte-select AND drops them into the address.  Pair p starts at bit 6p of the 96:
//   Q0: 0, 6, 12, 18 of w0      Q1: 24 of w0, 30 (w0|w1), 4 and 10 of w1
//   Q2: 16, 22 of w1, 28 (w1|w2), 2 of w2      Q3: 8, 14, 20, 26 of w2
template <int OFF, int Q>
__device__ __forceinline__ void issue4_p6(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t (&a)[4], uint32_t* v,
                                          uint32_t mask) {
    uint32_t t0, t1, t2;
#define KMQ_SDWA(dst, src, byte) \
    "v_and_b32_sdwa " dst ", " src ", %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_" byte " src1_sel:DWORD\n\t"
#define KMQ_READ4 \
    "ds_read_b32 %0, %7 offset:%c12\n\t" \
    "ds_read_b32 %1, %8 offset:%c12\n\t" \
    "ds_read_b32 %2, %9 offset:%c12\n\t" \
    "ds_read_b32 %3, %10 offset:%c12"
#define KMQ_OPERANDS \
    : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(t0), "=&v"(t1), "=&v"(t2), \
      "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]) \
    : "v"(mask), "n"(OFF)
    if constexpr (Q == 0) {
        asm volatile(
            "v_lshlrev_b32 %4, 2, %13\n\t"
            "v_lshlrev_b32 %5, 4, %13\n\t"
            "v_lshlrev_b32 %6, 6, %13\n\t"
            KMQ_SDWA("%7", "%4", "0") KMQ_SDWA("%8", "%5", "1") KMQ_SDWA("%9", "%6", "2") KMQ_SDWA("%10", "%13", "2")
            KMQ_READ4 KMQ_OPERANDS, "v"(w0));
    } else if constexpr (Q == 1) {
        asm volatile(
            "v_lshlrev_b32 %4, 2, %13\n\t"
            "v_alignbit_b32 %5, %14, %13, 28\n\t"
            "v_lshrrev_b32 %6, 2, %14\n\t"
            KMQ_SDWA("%7", "%4", "3") KMQ_SDWA("%8", "%5", "0") KMQ_SDWA("%9", "%6", "0") KMQ_SDWA("%10", "%14", "1")
            KMQ_READ4 KMQ_OPERANDS, "v"(w0), "v"(w1));
    } else if constexpr (Q == 2) {
        asm volatile(
            "v_lshlrev_b32 %4, 2, %13\n\t"
            "v_lshlrev_b32 %5, 4, %13\n\t"
            "v_alignbit_b32 %6, %14, %13, 26\n\t"
            KMQ_SDWA("%7", "%4", "2") KMQ_SDWA("%8", "%5", "3") KMQ_SDWA("%9", "%6", "0") KMQ_SDWA("%10", "%14", "0")
            KMQ_READ4 KMQ_OPERANDS, "v"(w1), "v"(w2));
    } else {
        asm volatile(
            "v_lshlrev_b32 %4, 2, %13\n\t"
            "v_lshlrev_b32 %5, 4, %13\n\t"
            "v_lshlrev_b32 %6, 6, %13\n\t"
            KMQ_SDWA("%7", "%4", "1") KMQ_SDWA("%8", "%5", "2") KMQ_SDWA("%9", "%6", "3") KMQ_SDWA("%10", "%13", "3")
            KMQ_READ4 KMQ_OPERANDS, "v"(w2));
    }
#undef KMQ_SDWA
#undef KMQ_READ4
#undef KMQ_OPERANDS
}

// A dot instruction's result may feed the accumulator of the next dot at once, but any OTHER
// vector instruction reading it needs three wait states (gfx90a and later).  The compiler
// inserts those for its own code; it cannot see inside an asm block, so accumulators written
// by the blocks below pass through this before ordinary code reads them.
__device__ __forceinline__ void settle_dot(float& a0, float& a1) {
    asm volatile("s_nop 2" : "+v"(a0), "+v"(a1));
}

// 2-bit: eight dot2 (two accumulator chains).  PENDING = LDS reads issued after
// the eight this block consumes.
template <int PENDING>
__device__ __forceinline__ void consume8_dot2(const uint32_t (&v)[8], const uint32_t* xr, float& a0, float& a1) {
    asm volatile(
        "s_waitcnt lgkmcnt(%c18)\n\t"
        "v_dot2c_f32_bf16 %0, %2, %10\n\t"
        "v_dot2c_f32_bf16 %1, %3, %11\n\t"
        "v_dot2c_f32_bf16 %0, %4, %12\n\t"
        "v_dot2c_f32_bf16 %1, %5, %13\n\t"
        "v_dot2c_f32_bf16 %0, %6, %14\n\t"
        "v_dot2c_f32_bf16 %1, %7, %15\n\t"
        "v_dot2c_f32_bf16 %0, %8, %16\n\t"
        "v_dot2c_f32_bf16 %1, %9, %17"
        : "+v"(a0), "+v"(a1)
        : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]),
          "v"(xr[0]), "v"(xr[1]), "v"(xr[2]), "v"(xr[3]), "v"(xr[4]), "v"(xr[5]), "v"(xr[6]), "v"(xr[7]),
          "n"(PENDING));
}

// 4-bit: eight FMAs, weights and activations as fp32.
template <int PENDING>
__device__ __forceinline__ void consume8_fma(const uint32_t (&v)[8], const uint32_t* xr, float& a0, float& a1) {
    asm volatile(
        "s_waitcnt lgkmcnt(%c18)\n\t"
        "v_fmac_f32 %0, %2, %10\n\t"
        "v_fmac_f32 %1, %3, %11\n\t"
        "v_fmac_f32 %0, %4, %12\n\t"
        "v_fmac_f32 %1, %5, %13\n\t"
        "v_fmac_f32 %0, %6, %14\n\t"
        "v_fmac_f32 %1, %7, %15\n\t"
        "v_fmac_f32 %0, %8, %16\n\t"
        "v_fmac_f32 %1, %9, %17"
        : "+v"(a0), "+v"(a1)
        : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]),
          "v"(xr[0]), "v"(xr[1]), "v"(xr[2]), "v"(xr[3]), "v"(xr[4]), "v"(xr[5]), "v"(xr[6]), "v"(xr[7]),
          "n"(PENDING));
}

// 1-bit: four 8-byte lookups for nibbles 4H..4H+3 of `word` (H = 0, 1); each
// returns four bf16 {0,1} masks.  re/ro are the rotated words, produced when
// H == 0 and reused when H == 1.  vv[2i] belongs to the even nibble.
template <int H>
__device__ __forceinline__ void issue4_b64(uint32_t word, uint32_t& re, uint32_t& ro, uint32_t (&a)[4],
                                           u32x2_t (&vv)[4], uint32_t mask) {
    if constexpr (H == 0) {
        asm volatile(
            "v_alignbit_b32 %4, %10, %10, 29\n\t"
            "v_alignbit_b32 %5, %10, %10, 1\n\t"
            "v_and_b32_sdwa %6, %4, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %7, %5, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %8, %4, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %9, %5, %11 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:DWORD\n\t"
            "ds_read_b64 %0, %6\n\t"
            "ds_read_b64 %1, %7\n\t"
            "ds_read_b64 %2, %8\n\t"
            "ds_read_b64 %3, %9"
            : "=&v"(vv[0]), "=&v"(vv[1]), "=&v"(vv[2]), "=&v"(vv[3]), "=&v"(re), "=&v"(ro),
              "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(word), "v"(mask));
    } else {
        asm volatile(
            "v_and_b32_sdwa %4, %8, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %5, %9, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %6, %8, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:DWORD\n\t"
            "v_and_b32_sdwa %7, %9, %10 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:DWORD\n\t"
            "ds_read_b64 %0, %4\n\t"
            "ds_read_b64 %1, %5\n\t"
            "ds_read_b64 %2, %6\n\t"
            "ds_read_b64 %3, %7"
            : "=&v"(vv[0]), "=&v"(vv[1]), "=&v"(vv[2]), "=&v"(vv[3]),
              "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(re), "v"(ro), "v"(mask));
    }
}

// 1-bit: eight dot2 of mask pairs against activation pairs.
template <int PENDING>
__device__ __forceinline__ void consume4_b64(const u32x2_t (&vv)[4], const uint32_t* xr, float& a0, float& a1) {
    asm volatile(
        "s_waitcnt lgkmcnt(%c18)\n\t"
        "v_dot2c_f32_bf16 %0, %2, %10\n\t"
        "v_dot2c_f32_bf16 %1, %3, %11\n\t"
        "v_dot2c_f32_bf16 %0, %4, %12\n\t"
        "v_dot2c_f32_bf16 %1, %5, %13\n\t"
        "v_dot2c_f32_bf16 %0, %6, %14\n\t"
        "v_dot2c_f32_bf16 %1, %7, %15\n\t"
        "v_dot2c_f32_bf16 %0, %8, %16\n\t"
        "v_dot2c_f32_bf16 %1, %9, %17"
        : "+v"(a0), "+v"(a1)
        : "v"(vv[0][0]), "v"(vv[0][1]), "v"(vv[1][0]), "v"(vv[1][1]), "v"(vv[2][0]), "v"(vv[2][1]), "v"(vv[3][0]), "v"(vv[3][1]),
          "v"(xr[0]), "v"(xr[1]), "v"(xr[2]), "v"(xr[3]), "v"(xr[4]), "v"(xr[5]), "v"(xr[6]), "v"(xr[7]),
          "n"(PENDING));
}

template <int I, int END, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < END) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, END>(f);
    }
}

template <int G> struct WordVec;
template <> struct WordVec<1> { using type = uint32_t; };
template <> struct WordVec<2> { using type = u32x2_t; };
struct alignas(4) Words3 { uint32_t v[3]; __device__ uint32_t operator[](int j) const { return v[j]; } };
template <> struct WordVec<3> { using type = Words3; };
template <> struct WordVec<4> { using type = u32x4_t; };

template <int G>
__device__ __forceinline__ void load_words(const uint32_t* p, uint32_t (&w)[G]) {
    if constexpr (G == 1) {
        w[0] = __builtin_nontemporal_load(p);
    } else if constexpr (G % 3 == 0) {
        typedef u32x3_t __attribute__((aligned(4))) u32x3_a4_t;      // 12-byte slices sit 4-byte aligned
#pragma unroll
        for (int i = 0; i < G / 3; ++i) {
            const u32x3_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x3_a4_t*>(p + 3 * i));   // (a 3-vector is 16 bytes wide as a type)
#pragma unroll
            for (int j = 0; j < 3; ++j) w[3 * i + j] = v[j];
        }
    } else {
        using V = typename WordVec<G>::type;
        const V v = __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
#pragma unroll
        for (int j = 0; j < G; ++j) w[j] = v[j];
    }
}

}  // namespace kmq

#endif
