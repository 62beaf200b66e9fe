// Dense bf16 GEMV: the unquantised baseline of the paper's micro-benchmark table
// (App. E, Table of m = 1, h = 8192, the 16-bit rows), so that speed-ups of the quantised
// kernels can be quoted against a bf16 product on the same machine.
//   y[n] = sum_k W[n][k] * x[k],  W N x K bf16 row-major, fp32 accumulation, bf16 output.
// HBM-bound stream of 2*N*K bytes: x is staged once per workgroup in LDS, every wave owns
// ROWS rows at a time and its lanes walk K in 16-byte pieces (1 KB contiguous per wave load).
#include "kmq_device.h"
#include "kmq_launch.h"

namespace kmq {

#ifndef KMQ_DENSE_ROWS
#define KMQ_DENSE_ROWS 2
#endif
#ifndef KMQ_DENSE_UNROLL
#define KMQ_DENSE_UNROLL 4
#endif
constexpr int kDenseRows = KMQ_DENSE_ROWS;       // rows per wave
constexpr int kDenseUnroll = KMQ_DENSE_UNROLL;   // steps of K whose loads are issued together
constexpr int kDenseWaves = 4;

template <bool VEC>
__global__ __launch_bounds__(kDenseWaves * 64) void gemv_bf16_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ x, uint16_t* __restrict__ y,
    int64_t N, int64_t K) {
    extern __shared__ u32x4_t xs[];                                  // ceil(K / 8) pieces of x
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t pieces = (K + 7) >> 3;
    for (int64_t c = threadIdx.x; c < pieces; c += kDenseWaves * 64) {
        u32x4_t v = u32x4_t{0u, 0u, 0u, 0u};
        if (VEC) {
            v = reinterpret_cast<const u32x4_t*>(x)[c];
        } else {                                                     // K % 8 != 0 or unaligned rows: element-wise, zero tail
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = c * 8 + e < K ? x[c * 8 + e] : 0u;
            v = u32x4_t{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        }
        xs[c] = v;
    }
    __syncthreads();

    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * kDenseWaves + wave) * kDenseRows;
    if (row0 >= N) return;
    float acc[kDenseRows];
#pragma unroll
    for (int r = 0; r < kDenseRows; ++r) acc[r] = 0.f;
    const uint16_t* wrow[kDenseRows];
#pragma unroll
    for (int r = 0; r < kDenseRows; ++r) {
        int64_t row = row0 + r;
        row = row < N ? row : N - 1;                                 // clamped: loads stay unconditional
        wrow[r] = W + row * K;
    }
    // kDenseUnroll steps of 64 pieces at a time: all their loads are issued before the first
    // multiply, so kDenseRows * kDenseUnroll 16-byte loads per lane are in flight
    int64_t c = lane;
    if (VEC) {
        for (; c + 64 * (kDenseUnroll - 1) < pieces; c += 64 * kDenseUnroll) {
            u32x4_t wv[kDenseUnroll][kDenseRows];
#pragma unroll
            for (int u = 0; u < kDenseUnroll; ++u)
#pragma unroll
                for (int r = 0; r < kDenseRows; ++r)
                    wv[u][r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow[r]) + c + 64 * u);
#pragma unroll
            for (int u = 0; u < kDenseUnroll; ++u) {
                const u32x4_t xv = xs[c + 64 * u];
#pragma unroll
                for (int r = 0; r < kDenseRows; ++r)
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[r] = dot2_bf16(wv[u][r][t], xv[t], acc[r]);
            }
        }
    }
    for (; c < pieces; c += 64) {
        const u32x4_t xv = xs[c];
#pragma unroll
        for (int r = 0; r < kDenseRows; ++r) {
            u32x4_t wv;
            if (VEC) {
                wv = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wrow[r]) + c);
            } else {
                uint32_t h[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) h[e] = c * 8 + e < K ? wrow[r][c * 8 + e] : 0u;
                wv = u32x4_t{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[r] = dot2_bf16(wv[t], xv[t], acc[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < kDenseRows; ++r) {
        const float s = group_sum<64>(acc[r]);
        if (lane == 63 && row0 + r < N) y[row0 + r] = f32_to_bf16(s);
    }
}

hipError_t launch_gemv_bf16(const uint16_t* W, const uint16_t* x, uint16_t* y, int64_t N, int64_t K, hipStream_t s) {
    const int64_t rows_wg = kDenseWaves * kDenseRows;
    const dim3 grid(static_cast<unsigned>((N + rows_wg - 1) / rows_wg)), block(kDenseWaves * 64);
    const size_t lds = static_cast<size_t>((K + 7) / 8) * sizeof(u32x4_t);
    const bool vec = (K % 8) == 0;
    if (vec) hipLaunchKernelGGL(gemv_bf16_kernel<true>, grid, block, lds, s, W, x, y, N, K);
    else hipLaunchKernelGGL(gemv_bf16_kernel<false>, grid, block, lds, s, W, x, y, N, K);
    return hipGetLastError();
}

}  // namespace kmq
