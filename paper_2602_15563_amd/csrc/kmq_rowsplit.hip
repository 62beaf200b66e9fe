// Batch-1 kernels specialised on (bits, K), canonical layout.
//
// Operation: y = W x with w = codebook lookup (paper App. E, "Kernel
// implementations"; batch-1 is the memory-bound regime of App. D).  The packed
// index stream is the only large operand, so the kernel is organised around
// reading it exactly once with wide coalesced loads:
//
//   * a row is cut into S chunks of LPR lanes x G words; lane `pos` of a chunk
//     owns G consecutive words = EL = G*32/bits consecutive elements, so one
//     vector load per (row, chunk) and per lane, contiguous across the lanes;
//   * with LPR < 64 a wave covers 64/LPR rows per load; every wave owns
//     RS such row steps and issues all its index loads before using any;
//   * the activations the lane needs (S*EL values) stay in VGPRs for all rows;
//   * weights come from a small table in LDS that is conflict-free because all
//     lanes of a row read the same 16-bank table:
//       2-bit  per-row table nibble -> two bf16 weights (16 x 4 B), one
//              v_dot2c_f32_bf16 per pair against a packed pair of activations;
//       1-bit  one row-independent table nibble -> four bf16 {0,1} masks
//              (16 x 8 B); the kernel accumulates S1 = sum_{idx=1} x and
//              finishes with y = c0*sum(x) + (c1 - c0)*S1 (two-centroid closed form);
//       3/4-bit per-row table index -> fp32 centroid, one lookup and one FMA
//              per weight against fp32 activations;
//   * K-reduction with DPP adds inside the LPR-lane group, fp32 -> bf16 RNE.
#include "kmq_device.h"
#include "kmq_launch.h"

namespace kmq {

template <int G> struct WordVec;
template <> struct WordVec<1> { using type = uint32_t; };
template <> struct WordVec<2> { using type = u32x2_t; };
struct alignas(4) Words3 { uint32_t v[3]; __device__ uint32_t operator[](int j) const { return v[j]; } };
template <> struct WordVec<3> { using type = Words3; };
template <> struct WordVec<4> { using type = u32x4_t; };

template <int G>
__device__ __forceinline__ void load_words(const uint32_t* p, uint32_t (&w)[G]) {
    using V = typename WordVec<G>::type;
    const V v = *reinterpret_cast<const V*>(p);
    if constexpr (G == 1) {
        w[0] = v;
    } else {
#pragma unroll
        for (int j = 0; j < G; ++j) w[j] = v[j];
    }
}

template <int BITS, int G, int S, int LPR, int RS>
__global__ __launch_bounds__(256) void gemv_rowsplit_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    const uint16_t* __restrict__ x, uint16_t* __restrict__ y, int64_t N) {
    constexpr int C = 1 << BITS;
    constexpr int EL = G * 32 / BITS;          // elements per lane and chunk
    constexpr int K = S * LPR * EL;
    constexpr int WPR = K * BITS / 32;
    constexpr int RPL = kWave / LPR;           // rows per load step
    constexpr int RPW = RPL * RS;              // rows per wave
    constexpr int WAVES = 4;
    constexpr bool kPairs = BITS <= 2;         // activations kept as packed bf16 pairs
    constexpr int XR = kPairs ? S * EL / 2 : S * EL;
    static_assert(BITS != 3 || G == 3, "3-bit chunks are 96 bits");
    static_assert(EL % 8 == 0, "activation slices load as 16-byte vectors");

    // LDS tables.
    constexpr int LUT_ENTRIES = BITS == 2 ? 16 : C;
    __shared__ uint32_t lut[BITS == 1 ? 1 : WAVES][BITS == 1 ? 1 : RPW][LUT_ENTRIES];
    __shared__ u32x2_t mask_table[16];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane / LPR, pos = lane % LPR;
    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * WAVES + wave) * RPW;

    // ---- 1. issue every index load of this wave ------------------------------
    uint32_t w[RS][S][G];
#pragma unroll
    for (int t = 0; t < RS; ++t) {
        const int64_t row = row0 + t * RPL + sub;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (row < N) {
                load_words<G>(W + row * WPR + (s * LPR + pos) * G, w[t][s]);
            } else {
#pragma unroll
                for (int j = 0; j < G; ++j) w[t][s][j] = 0u;
            }
        }
    }

    // ---- 2. activations of this lane's K-slices -------------------------------
    uint32_t xr[XR];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(x + (s * LPR + pos) * EL);
#pragma unroll
        for (int q = 0; q < EL / 8; ++q) {
            const u32x4_t v = xp[q];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (kPairs) {
                    xr[s * (EL / 2) + q * 4 + j] = v[j];
                } else {
                    xr[s * EL + q * 8 + 2 * j] = v[j] << 16;
                    xr[s * EL + q * 8 + 2 * j + 1] = v[j] & 0xFFFF0000u;
                }
            }
        }
    }

    // ---- 3. lookup tables ------------------------------------------------------
    if constexpr (BITS == 1) {
        if (threadIdx.x < 16) {
            const uint32_t e = threadIdx.x;
            u32x2_t m;
            m[0] = ((e & 1u) ? 0x3F80u : 0u) | ((e & 2u) ? 0x3F800000u : 0u);
            m[1] = ((e & 4u) ? 0x3F80u : 0u) | ((e & 8u) ? 0x3F800000u : 0u);
            mask_table[e] = m;
        }
    } else if constexpr (BITS == 2) {
        // entry e = (c[e & 3], c[e >> 2]) as a packed bf16 pair; 4 rows per pass
#pragma unroll
        for (int p = 0; p < (RPW + 3) / 4; ++p) {
            const int r = p * 4 + (lane >> 4), e = lane & 15;
            const int64_t row = row0 + r;
            if (r < RPW && row < N) {
                const uint16_t* c = codebook + row * C;
                lut[wave][r][e] = static_cast<uint32_t>(c[e & 3]) | (static_cast<uint32_t>(c[e >> 2]) << 16);
            }
        }
    } else {
        constexpr int ROWS_PER_PASS = kWave / C;
#pragma unroll
        for (int p = 0; p < (RPW + ROWS_PER_PASS - 1) / ROWS_PER_PASS; ++p) {
            const int r = p * ROWS_PER_PASS + lane / C, e = lane % C;
            const int64_t row = row0 + r;
            if (r < RPW && row < N) lut[wave][r][e] = static_cast<uint32_t>(codebook[row * C + e]) << 16;
        }
    }
    __syncthreads();

    // ---- 4. decode + multiply-accumulate ---------------------------------------
    float acc[RS];
#pragma unroll
    for (int t = 0; t < RS; ++t) {
        float a = 0.f;
        [[maybe_unused]] const uint32_t* lrow = nullptr;
        if constexpr (BITS != 1) lrow = &lut[wave][t * RPL + sub][0];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if constexpr (BITS == 1) {
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    const uint32_t word = w[t][s][j];
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const u32x2_t m = mask_table[(word >> (4 * q)) & 15u];
                        const int xi = s * (EL / 2) + j * 16 + q * 2;
                        a = dot2_bf16(m[0], xr[xi], a);
                        a = dot2_bf16(m[1], xr[xi + 1], a);
                    }
                }
            } else if constexpr (BITS == 2) {
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    const uint32_t word = w[t][s][j];
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        a = dot2_bf16(lrow[(word >> (4 * q)) & 15u], xr[s * (EL / 2) + j * 8 + q], a);
                }
            } else if constexpr (BITS == 4) {
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    const uint32_t word = w[t][s][j];
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        a = fmaf(__uint_as_float(lrow[(word >> (4 * q)) & 15u]),
                                 __uint_as_float(xr[s * EL + j * 8 + q]), a);
                }
            } else {   // BITS == 3: 96 bits = 32 fields, two of which straddle words
                const uint64_t lo = static_cast<uint64_t>(w[t][s][0]) | (static_cast<uint64_t>(w[t][s][1]) << 32);
                const uint64_t hi = static_cast<uint64_t>(w[t][s][1]) | (static_cast<uint64_t>(w[t][s][2]) << 32);
#pragma unroll
                for (int e = 0; e < 32; ++e) {
                    const uint32_t f = e < 21 ? static_cast<uint32_t>(lo >> (3 * e)) & 7u
                                              : static_cast<uint32_t>(hi >> (3 * e - 32)) & 7u;
                    a = fmaf(__uint_as_float(lrow[f]), __uint_as_float(xr[s * EL + e]), a);
                }
            }
        }
        acc[t] = a;
    }

    // ---- 5. K-reduction and epilogue -------------------------------------------
    [[maybe_unused]] float sx = 0.f;
    if constexpr (BITS == 1) {
#pragma unroll
        for (int i = 0; i < XR; ++i) sx = dot2_bf16(0x3F803F80u, xr[i], sx);
        sx = group_sum<LPR>(sx);
    }
#pragma unroll
    for (int t = 0; t < RS; ++t) {
        const float s1 = group_sum<LPR>(acc[t]);
        const int64_t row = row0 + t * RPL + sub;
        if (pos == LPR - 1 && row < N) {
            float out = s1;
            if constexpr (BITS == 1) {
                const float c0 = bf16_to_f32(codebook[row * 2]), c1 = bf16_to_f32(codebook[row * 2 + 1]);
                out = fmaf(c1 - c0, s1, c0 * sx);
            }
            y[row] = f32_to_bf16(out);
        }
    }
}

// ---- specialisation table ---------------------------------------------------------

struct RowsplitEntry {
    int bits;
    int64_t K;
    int rows_per_block;
    const char* name;
    void (*launch)(const GemmArgs&, hipStream_t);
};

template <int BITS, int G, int S, int LPR, int RS>
static void launch_one(const GemmArgs& a, hipStream_t s) {
    constexpr int rows_per_block = 4 * (kWave / LPR) * RS;
    const dim3 grid(static_cast<unsigned>((a.N + rows_per_block - 1) / rows_per_block)), block(256);
    hipLaunchKernelGGL((gemv_rowsplit_kernel<BITS, G, S, LPR, RS>), grid, block, 0, s,
                       a.W, a.codebook, a.X, a.Y, a.N);
}

#define KMQ_ROWSPLIT(BITS, G, S, LPR, RS) \
    { BITS, int64_t(S) * LPR * (G * 32 / BITS), 4 * (64 / LPR) * RS, \
      "rowsplit_b" #BITS "_g" #G "_s" #S "_l" #LPR "_r" #RS, &launch_one<BITS, G, S, LPR, RS> }

// Only the 3-bit shapes are instantiated: 1-, 2- and 4-bit batch-1 products take the
// hand-scheduled table kernels (kmq_lut.hip), which supersede this kernel's paths for them.
static const RowsplitEntry kRowsplit[] = {
    KMQ_ROWSPLIT(3, 3, 1, 64, 4),   // K = 2048
    KMQ_ROWSPLIT(3, 3, 2, 64, 4),   // K = 4096
};
constexpr int kRowsplitCount = sizeof(kRowsplit) / sizeof(kRowsplit[0]);

int rowsplit_find(int64_t K, int bits, int layout) {
    if (layout != KMQ_LAYOUT_CANONICAL) return -1;
    for (int i = 0; i < kRowsplitCount; ++i)
        if (kRowsplit[i].bits == bits && kRowsplit[i].K == K) return i;
    return -1;
}

const char* rowsplit_name(int i) { return kRowsplit[i].name; }

hipError_t launch_rowsplit(int i, const GemmArgs& a, hipStream_t s) {
    kRowsplit[i].launch(a, s);
    return hipGetLastError();
}

}  // namespace kmq
