// Shape-agnostic kernel for the decoder-layer fusions at batch 1 (paper App. E "Model
// benchmarks": token generation runs the projections of a decoder layer back to back, and
// at low bit-widths the elementwise work between them -- RMSNorm, the activation function,
// the residual sums -- is a visible share of the time).  One launch computes
//
//     xn[k] = bf16( x[k] * g[k] )                       RMSNorm in front (optional; xn = x for unit gains)
//     r     = 1 / sqrt( mean_k x[k]^2 + eps )           (1 without the norm)
//     p[n]  = r * sum_k w[n][k] * xn[k]                 the product of kmq_gemv
//     y[n]  = bf16( residual[n] + p[n] )                residual behind (optional), or
//     y[n]  = bf16( silu(p_gate[n]) * p_up[n] )         for a pair of matrices (gate, up)
//
// The scalar r commutes with the sum, so the normalised activations enter the product as
// bf16(x * g) and r is applied once per row.  Canonical layout, any N and K; the
// shape-specialised kernels (kmq_lut.hip) carry the same fusions for their shapes.
#include "kmq_device.h"
#include "kmq_launch.h"

namespace kmq {

template <int BITS>
__device__ __forceinline__ uint32_t stream_field(const uint32_t* row, int64_t k) {
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int64_t p = k * BITS;
    const int64_t wi = p >> 5;
    const int sh = static_cast<int>(p & 31);
    uint32_t v = row[wi] >> sh;
    if (sh + BITS > 32) v |= row[wi + 1] << (32 - sh);
    return v & mask;
}

// One wave per output element, four per workgroup; lanes stride over K.
template <int BITS, bool PAIR>
__global__ __launch_bounds__(256) void gemv_fused_generic_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    const uint32_t* __restrict__ W2, const uint16_t* __restrict__ codebook2,
    const uint16_t* __restrict__ x, bool norm, const uint16_t* __restrict__ norm_w, float eps,
    const uint16_t* residual, uint16_t* y, int64_t N, int64_t K) {   // (may be one buffer: no __restrict__)
    constexpr int C = 1 << BITS;
    __shared__ float lut[4][2][C];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t n = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    const bool live = n < N;
    if (live)
        for (int e = lane; e < C; e += kWave) {
            lut[wave][0][e] = bf16_to_f32(codebook[n * C + e]);
            if constexpr (PAIR) lut[wave][1][e] = bf16_to_f32(codebook2[n * C + e]);
        }
    __syncthreads();
    if (!live) return;

    const int64_t wpr = words_per_row(BITS, K);
    const uint32_t* r0 = W + n * wpr;
    [[maybe_unused]] const uint32_t* r1 = PAIR ? W2 + n * wpr : nullptr;
    float acc0 = 0.f, acc1 = 0.f, ss = 0.f;
    for (int64_t k = lane; k < K; k += kWave) {
        float xv = bf16_to_f32(x[k]);
        if (norm) {
            ss = fmaf(xv, xv, ss);
            if (norm_w) xv = bf16_to_f32(f32_to_bf16(xv * bf16_to_f32(norm_w[k])));
        }
        acc0 = fmaf(lut[wave][0][stream_field<BITS>(r0, k)], xv, acc0);
        if constexpr (PAIR) acc1 = fmaf(lut[wave][1][stream_field<BITS>(r1, k)], xv, acc1);
    }
    acc0 = group_sum<64>(acc0);
    if constexpr (PAIR) acc1 = group_sum<64>(acc1);
    ss = group_sum<64>(ss);
    if (lane != 63) return;
    const float r = norm ? 1.f / sqrtf(ss * (1.f / static_cast<float>(K)) + eps) : 1.f;
    float out = acc0 * r;
    if constexpr (PAIR) {
        out = out / (1.f + __expf(-out)) * (acc1 * r);
    } else {
        if (residual) out += bf16_to_f32(residual[n]);
    }
    y[n] = f32_to_bf16(out);
}

template <int BITS>
static hipError_t launch_fused_bits(const GemmArgs& a, hipStream_t s) {
    const dim3 grid(static_cast<unsigned>((a.N + 3) / 4)), block(256);
    if (a.W2)
        hipLaunchKernelGGL((gemv_fused_generic_kernel<BITS, true>), grid, block, 0, s, a.W, a.codebook, a.W2, a.codebook2, a.X,
                           a.norm, a.norm_w, a.eps, static_cast<const uint16_t*>(nullptr), a.Y, a.N, a.K);
    else
        hipLaunchKernelGGL((gemv_fused_generic_kernel<BITS, false>), grid, block, 0, s, a.W, a.codebook,
                           static_cast<const uint32_t*>(nullptr), static_cast<const uint16_t*>(nullptr), a.X, a.norm, a.norm_w, a.eps,
                           a.residual, a.Y, a.N, a.K);
    return hipGetLastError();
}

hipError_t launch_fused_generic(const GemmArgs& a, hipStream_t s) {
    switch (a.bits) {
        case 1: return launch_fused_bits<1>(a, s);
        case 2: return launch_fused_bits<2>(a, s);
        case 3: return launch_fused_bits<3>(a, s);
        case 8: return launch_fused_bits<8>(a, s);
        default: return launch_fused_bits<4>(a, s);
    }
}

}  // namespace kmq
