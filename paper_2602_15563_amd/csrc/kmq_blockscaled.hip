// Shape-agnostic kernel for the paper's own weight format (Sec. 2.2 "Nonlinear
// k-means quantization": centroids shared by the whole tensor, one bf16 scale per
// block of 64 consecutive elements along K; App. E "Kernel implementations"):
//
//     Y[m][n] = sum_g scale[n][g] * sum_{k in block g} codebook[idx[n][k]] * X[m][k]
//
// i.e. the appendix's deferred-scaling variant, with the block sums and the sum
// over blocks in fp32.  Canonical layout, any N, any K that is a multiple of 64,
// batch 1..16.  The shape-specialised batch-1 kernels live in kmq_lut.hip.
#include "kmq_device.h"
#include "kmq_launch.h"

namespace kmq {

// b-bit field `e` (0..63) of a 64-element block held in 2*BITS consecutive words
// (64*BITS bits: a block starts and ends on a word boundary for every bit-width).
template <int BITS>
__device__ __forceinline__ uint32_t block_field(const uint32_t (&w)[2 * BITS], int e) {
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int p = e * BITS;
    const int wi = p >> 5, sh = p & 31;
    uint32_t v = w[wi] >> sh;
    if constexpr (BITS == 3) {
        if (sh > 29) v |= w[wi + 1] << (32 - sh);   // field straddles two words (never the block's last word)
    }
    return v & mask;
}

// One wave per output row, four rows per workgroup; each lane walks over whole
// blocks, so a block's scale is applied once, to the lane's fp32 block sum.
template <int BITS, int MT>
__global__ __launch_bounds__(256) void gemm_blockscaled_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    const uint16_t* __restrict__ scales, const uint16_t* __restrict__ X, uint16_t* __restrict__ Y,
    int64_t N, int64_t K, int M) {
    constexpr int C = 1 << BITS;
    __shared__ float lut[C];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (threadIdx.x < C) lut[threadIdx.x] = bf16_to_f32(codebook[threadIdx.x]);
    __syncthreads();
    const int64_t n = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    if (n >= N) return;

    const int64_t wpr = words_per_row(BITS, K);
    const int64_t nblocks = K / KMQ_BLOCK;
    float acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = 0.f;

    for (int64_t g = lane; g < nblocks; g += kWave) {
        uint32_t w[2 * BITS];
#pragma unroll
        for (int j = 0; j < 2 * BITS; ++j) w[j] = W[n * wpr + g * (2 * BITS) + j];
        const float s = bf16_to_f32(scales[n * nblocks + g]);
        float z[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) z[m] = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {              // eight elements (16 bytes of x) at a time
            float c[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) c[e] = lut[block_field<BITS>(w, q * 8 + e)];
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (m < M) {
                    const u32x4_t xv = *reinterpret_cast<const u32x4_t*>(X + m * K + g * KMQ_BLOCK + q * 8);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        z[m] = fmaf(c[2 * t], __uint_as_float(xv[t] << 16), z[m]);
                        z[m] = fmaf(c[2 * t + 1], __uint_as_float(xv[t] & 0xFFFF0000u), z[m]);
                    }
                }
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = fmaf(s, z[m], acc[m]);
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const float s = group_sum<64>(acc[m]);
        if (lane == 63 && m < M) Y[static_cast<int64_t>(m) * N + n] = f32_to_bf16(s);
    }
}

// Dense weights of the format, Wd[n][k] = bf16( codebook[idx[n][k]] * scale[n][k / 64] ): one thread per
// 8 consecutive elements, so that a wave's store is 1 KB of consecutive bytes.  The fp32 product of two
// bf16 values is exact, so the result carries one rounding, to nearest even.
template <int BITS>
__global__ __launch_bounds__(256) void dequant_blockscaled_kernel(const uint32_t* __restrict__ W,
                                                                  const uint16_t* __restrict__ codebook,
                                                                  const uint16_t* __restrict__ scales, int64_t nchunks,
                                                                  int64_t total_words, uint16_t* __restrict__ Wd) {
    constexpr int C = 1 << BITS;
    constexpr uint32_t mask = C - 1;
    __shared__ float lut[C];
    if (threadIdx.x < C) lut[threadIdx.x] = bf16_to_f32(codebook[threadIdx.x]);
    __syncthreads();
    const int64_t c8 = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;   // chunk of 8 elements, row-major over N x K/8
    if (c8 >= nchunks) return;
    // K % 64 == 0: rows are whole words, so the matrix is one bit stream and chunk c8 starts at bit c8 * 8 * BITS
    const int64_t bit0 = c8 * (8 * BITS);
    const int64_t wi = bit0 >> 5;
    const int sh = static_cast<int>(bit0 & 31);
    const uint64_t lo = W[wi], hi = wi + 1 < total_words ? W[wi + 1] : 0u;
    const uint64_t v = (lo | (hi << 32)) >> sh;
    const float s = bf16_to_f32(scales[c8 >> 3]);
    uint32_t out[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        const uint32_t a = f32_to_bf16(lut[static_cast<uint32_t>(v >> (e * BITS)) & mask] * s);
        const uint32_t b = f32_to_bf16(lut[static_cast<uint32_t>(v >> ((e + 1) * BITS)) & mask] * s);
        out[e >> 1] = a | (b << 16);
    }
    // written once and read by a later kernel: no reason to keep it in this kernel's caches
    __builtin_nontemporal_store(u32x4_t{out[0], out[1], out[2], out[3]}, reinterpret_cast<u32x4_t*>(Wd + (c8 << 3)));
}

hipError_t launch_dequant_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales, uint16_t* Wd,
                                      int64_t N, int64_t K, int bits, hipStream_t s) {
    const int64_t nchunks = N * (K / 8), words = N * (K * bits / 32);
    const dim3 grid(static_cast<unsigned>((nchunks + 255) / 256)), block(256);
#define KMQ_DQ(B) hipLaunchKernelGGL(dequant_blockscaled_kernel<B>, grid, block, 0, s, W, codebook, scales, nchunks, words, Wd)
    switch (bits) {
        case 1: KMQ_DQ(1); break;
        case 2: KMQ_DQ(2); break;
        case 3: KMQ_DQ(3); break;
        case 8: KMQ_DQ(8); break;
        default: KMQ_DQ(4); break;
    }
#undef KMQ_DQ
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_blockscaled_bits(const GemmArgs& a, hipStream_t s) {
    const dim3 grid(static_cast<unsigned>((a.N + 3) / 4)), block(256);
#define KMQ_BS_LAUNCH(MT) \
    hipLaunchKernelGGL((gemm_blockscaled_kernel<BITS, MT>), grid, block, 0, s, a.W, a.codebook, a.scales, a.X, a.Y, a.N, a.K, a.M)
    if (a.M == 1) KMQ_BS_LAUNCH(1);
    else if (a.M <= 4) KMQ_BS_LAUNCH(4);
    else if (a.M <= 8) KMQ_BS_LAUNCH(8);
    else KMQ_BS_LAUNCH(16);
#undef KMQ_BS_LAUNCH
    return hipGetLastError();
}

hipError_t launch_blockscaled_generic(const GemmArgs& a, hipStream_t s) {
    switch (a.bits) {
        case 1: return launch_blockscaled_bits<1>(a, s);
        case 2: return launch_blockscaled_bits<2>(a, s);
        case 3: return launch_blockscaled_bits<3>(a, s);
        case 8: return launch_blockscaled_bits<8>(a, s);
        default: return launch_blockscaled_bits<4>(a, s);
    }
}

}  // namespace kmq
