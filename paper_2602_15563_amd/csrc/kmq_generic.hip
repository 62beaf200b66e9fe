// Shape-agnostic kernels: any K >= 1, any bit-width, both layouts, batch 1..16.
// They are the fallback behind the shape-specialised kernels and the
// bit-exact dequantiser.  Operation: paper App. E, "Kernel implementations"
// (lookup, then multiply-accumulate), per-row codebooks, fp32 accumulation.
#include <mutex>

#include "kmq_device.h"
#include "kmq_launch.h"

// Scratch of kmq_gemm_smallbatch_noalloc: the split-K partial sums of callers that cannot allocate.
// Every GPU the library runs on holds its own copy at its own address until the process ends.  In host
// code this name is a stand-in, not a device address: the address comes from hipGetSymbolAddress below.
static __device__ __align__(256) unsigned char scratch[KMQ_NOALLOC_SCRATCH_BYTES];

namespace kmq {

// Device address of this GPU's scratch array (looked up once per device, with that device current).
hipError_t noalloc_scratch(void** ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

// b-bit field `e` (0..31) of a 32-element group held in BITS consecutive words.
template <int BITS>
__device__ __forceinline__ uint32_t group_field(const uint32_t (&w)[BITS], int e) {
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int p = e * BITS;               // bit position inside the group
    const int wi = p >> 5, sh = p & 31;
    uint32_t v = w[wi] >> sh;
    if constexpr (BITS == 3) {
        if (sh > 29) v |= w[wi + 1] << (32 - sh);   // field straddles two words
    }
    return v & mask;
}

// One wave per output row, four rows per workgroup.  Each lane walks over
// 32-element groups (BITS words each, so groups start on a word boundary for
// every bit-width), looks weights up in the row's codebook (fp32 copy in LDS)
// and accumulates MT batch columns.
//
// Split-K (few rows, long rows: too few workgroups to fill the CUs otherwise): blockIdx.y
// selects one of gridDim.y slices of K (whole 32-element groups); the slice's fp32 partial
// sums go to partial[slice][m][n] and splitk_reduce_kernel adds the slices in index order, so
// the result does not depend on which workgroup finishes first.  partial == nullptr: one
// slice, bf16 output written directly.
template <int BITS, int MT>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    const uint16_t* __restrict__ X, uint16_t* __restrict__ Y,
    int64_t N, int64_t K, int M, int layout, float* __restrict__ partial) {
    constexpr int C = 1 << BITS;
    __shared__ float lut[4][C];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t n = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    const bool live = n < N;
    if (live)
        for (int e = lane; e < C; e += kWave) lut[wave][e] = bf16_to_f32(codebook[n * C + e]);
    __syncthreads();
    if (!live) return;

    const int64_t wpr = words_per_row(BITS, K);
    const int64_t ngroups = (K + 31) >> 5;
    const bool vec_x = (K & 7) == 0;      // rows of X start 16-byte aligned
    float acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = 0.f;

    const int64_t gps = (ngroups + gridDim.y - 1) / gridDim.y;     // groups per slice
    const int64_t g_begin = blockIdx.y * gps, g_end = g_begin + gps < ngroups ? g_begin + gps : ngroups;
    for (int64_t g = g_begin + lane; g < g_end; g += kWave) {
        const int64_t k0 = g << 5;
        const bool full = k0 + 32 <= K;
        float wt[32];
        if (layout == KMQ_LAYOUT_CANONICAL) {
            uint32_t w[BITS];
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const int64_t wi = g * BITS + j;
                w[j] = wi < wpr ? W[n * wpr + wi] : 0u;
            }
#pragma unroll
            for (int e = 0; e < 32; ++e) wt[e] = lut[wave][group_field<BITS>(w, e)];
        } else {
            for (int e = 0; e < 32; ++e) wt[e] = lut[wave][tiled_fetch_index(W, BITS, K, n, k0 + e)];   // K % 128 == 0 here
        }
        if (full && vec_x) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (m < M) {
                    const u32x4_t* xp = reinterpret_cast<const u32x4_t*>(X + m * K + k0);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const u32x4_t xv = xp[q];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            acc[m] = fmaf(wt[q * 8 + t * 2], __uint_as_float(xv[t] << 16), acc[m]);
                            acc[m] = fmaf(wt[q * 8 + t * 2 + 1], __uint_as_float(xv[t] & 0xFFFF0000u), acc[m]);
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                if (k0 + e < K) {
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        if (m < M) acc[m] = fmaf(wt[e], bf16_to_f32(X[m * K + k0 + e]), acc[m]);
                }
            }
        }
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const float s = group_sum<64>(acc[m]);
        if (lane == 63 && m < M) {
            if (partial) partial[(static_cast<int64_t>(blockIdx.y) * M + m) * N + n] = s;
            else Y[static_cast<int64_t>(m) * N + n] = f32_to_bf16(s);
        }
    }
}

// Second pass of split-K: Y[m][n] = bf16( partial[0][m][n] + partial[1][m][n] + ... ), slices in order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, uint16_t* __restrict__ Y,
                                                            int64_t MN, int slices) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= MN) return;
    float s = 0.f;
    for (int k = 0; k < slices; ++k) s += partial[static_cast<int64_t>(k) * MN + i];
    Y[i] = f32_to_bf16(s);
}

// Fused pair, any K, canonical layout, batch 1: y[n] = silu(W[n] . x) * (W2[n] . x), the
// SwiGLU of a decoder MLP's gate and up projections (both products share x).  One wave per
// output element walks both rows.
template <int BITS>
__global__ __launch_bounds__(256) void gemv_pair_generic_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    const uint32_t* __restrict__ W2, const uint16_t* __restrict__ codebook2,
    const uint16_t* __restrict__ x, uint16_t* __restrict__ y, int64_t N, int64_t K) {
    constexpr int C = 1 << BITS;
    __shared__ float lut[4][2][C];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t n = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    const bool live = n < N;
    if (live)
        for (int e = lane; e < 2 * C; e += kWave)
            lut[wave][e / C][e % C] = bf16_to_f32((e < C ? codebook : codebook2)[n * C + e % C]);
    __syncthreads();
    if (!live) return;
    const int64_t wpr = words_per_row(BITS, K);
    const int64_t ngroups = (K + 31) >> 5;
    float acc[2] = {0.f, 0.f};
    for (int64_t g = lane; g < ngroups; g += kWave) {
        const int64_t k0 = g << 5;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t* row = (h ? W2 : W) + n * wpr;
            uint32_t w[BITS];
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const int64_t wi = g * BITS + j;
                w[j] = wi < wpr ? row[wi] : 0u;
            }
#pragma unroll
            for (int e = 0; e < 32; ++e)
                if (k0 + e < K) acc[h] = fmaf(lut[wave][h][group_field<BITS>(w, e)], bf16_to_f32(x[k0 + e]), acc[h]);
        }
    }
    const float gate = group_sum<64>(acc[0]), up = group_sum<64>(acc[1]);
    if (lane == 63) y[n] = f32_to_bf16(gate / (1.f + __expf(-gate)) * up);
}

hipError_t launch_pair_generic(const GemmArgs& a, hipStream_t s) {
    const dim3 grid(static_cast<unsigned>((a.N + 3) / 4)), block(256);
    switch (a.bits) {
        case 1: hipLaunchKernelGGL(gemv_pair_generic_kernel<1>, grid, block, 0, s, a.W, a.codebook, a.W2, a.codebook2, a.X, a.Y, a.N, a.K); break;
        case 2: hipLaunchKernelGGL(gemv_pair_generic_kernel<2>, grid, block, 0, s, a.W, a.codebook, a.W2, a.codebook2, a.X, a.Y, a.N, a.K); break;
        case 3: hipLaunchKernelGGL(gemv_pair_generic_kernel<3>, grid, block, 0, s, a.W, a.codebook, a.W2, a.codebook2, a.X, a.Y, a.N, a.K); break;
        case 8: hipLaunchKernelGGL(gemv_pair_generic_kernel<8>, grid, block, 0, s, a.W, a.codebook, a.W2, a.codebook2, a.X, a.Y, a.N, a.K); break;
        default: hipLaunchKernelGGL(gemv_pair_generic_kernel<4>, grid, block, 0, s, a.W, a.codebook, a.W2, a.codebook2, a.X, a.Y, a.N, a.K); break;
    }
    return hipGetLastError();
}

// One thread per (row, 32-element group): Wdense[n][k] = codebook[n][idx[n][k]].
template <int BITS>
__global__ __launch_bounds__(256) void dequant_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    uint16_t* __restrict__ Wd, int64_t N, int64_t K, int layout) {
    constexpr int C = 1 << BITS;
    const int64_t wpr = words_per_row(BITS, K);
    const int64_t ngroups = (K + 31) >> 5;
    const int64_t total = N * ngroups;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t n = i / ngroups, g = i % ngroups;
        uint32_t w[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j) {
            const int64_t wi = g * BITS + j;
            w[j] = (layout == KMQ_LAYOUT_CANONICAL && wi < wpr) ? W[n * wpr + wi] : 0u;
        }
        [[maybe_unused]] uint16_t c[BITS <= 4 ? C : 1];
        if constexpr (BITS <= 4) {
#pragma unroll
            for (int j = 0; j < C; ++j) c[j] = codebook[n * C + j];
        }
        const int64_t k0 = g << 5;
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const uint32_t f = layout == KMQ_LAYOUT_CANONICAL ? group_field<BITS>(w, e)
                                                              : tiled_fetch_index(W, BITS, K, n, k0 + e);
            uint16_t v;
            if constexpr (BITS <= 4) {
                v = c[0];
#pragma unroll
                for (int j = 1; j < C; ++j) v = f == static_cast<uint32_t>(j) ? c[j] : v;
            } else {
                v = codebook[n * C + f];     // 256 entries: read through the caches instead of held in registers
            }
            if (k0 + e < K) Wd[n * K + k0 + e] = v;
        }
    }
}

// The same for the canonical layout with K % 8 == 0: one thread per 8 consecutive elements, one 16-byte
// store per thread (a wave writes 1 KB of consecutive bytes, past the caches: the matrix is read by a later
// kernel).  The row's centroids are read through the caches.
template <int BITS>
__global__ __launch_bounds__(256) void dequant_rows8_kernel(const uint32_t* __restrict__ W,
                                                            const uint16_t* __restrict__ codebook,
                                                            uint16_t* __restrict__ Wd, int64_t N, int64_t K) {
    constexpr int C = 1 << BITS;
    constexpr uint32_t mask = C - 1;
    const int64_t cpr = K >> 3;                                   // chunks per row
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= N * cpr) return;
    const int64_t n = i / cpr, c8 = i % cpr;
    const int64_t wpr = words_per_row(BITS, K);
    const int64_t bit0 = c8 * (8 * BITS);
    const int64_t wi = bit0 >> 5;
    const int sh = static_cast<int>(bit0 & 31);
    const uint32_t* row = W + n * wpr;
    const uint64_t lo = row[wi], hi = wi + 1 < wpr ? row[wi + 1] : 0u;
    const uint64_t v = (lo | (hi << 32)) >> sh;
    const uint16_t* c = codebook + n * C;
    uint32_t out[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        const uint32_t a = c[static_cast<uint32_t>(v >> (e * BITS)) & mask];
        const uint32_t b = c[static_cast<uint32_t>(v >> ((e + 1) * BITS)) & mask];
        out[e >> 1] = a | (b << 16);
    }
    __builtin_nontemporal_store(u32x4_t{out[0], out[1], out[2], out[3]}, reinterpret_cast<u32x4_t*>(Wd + n * K + (c8 << 3)));
}

template <int BITS>
static hipError_t launch_generic_bits(const GemmArgs& a, int slices, hipStream_t s) {
    const dim3 grid(static_cast<unsigned>((a.N + 3) / 4), static_cast<unsigned>(slices)), block(256);
    float* partial = slices > 1 ? static_cast<float*>(a.workspace) : nullptr;
#define KMQ_GEN_LAUNCH(MT) \
    hipLaunchKernelGGL((gemm_generic_kernel<BITS, MT>), grid, block, 0, s, a.W, a.codebook, a.X, a.Y, a.N, a.K, a.M, a.layout, partial)
    if (a.M == 1) KMQ_GEN_LAUNCH(1);
    else if (a.M <= 4) KMQ_GEN_LAUNCH(4);
    else if (a.M <= 8) KMQ_GEN_LAUNCH(8);
    else KMQ_GEN_LAUNCH(16);
#undef KMQ_GEN_LAUNCH
    if (slices > 1) {
        const int64_t mn = static_cast<int64_t>(a.M) * a.N;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(static_cast<unsigned>((mn + 255) / 256)), dim3(256), 0, s,
                           partial, a.Y, mn, slices);
    }
    return hipGetLastError();
}

// Slices of K for the shape-agnostic kernel: 1 unless its one-wave-per-row grid would leave more
// than half of the 256 CUs idle on a product with long rows; then enough slices to fill them, each
// at least 4096 elements long.
int generic_splitk_slices(int64_t N, int64_t K, int layout) {
    if (layout != KMQ_LAYOUT_CANONICAL) return 1;
    const int64_t wgs = (N + 3) / 4;
    if (wgs * 2 > 256 || K < 16384) return 1;   // measured: at K = 8192 the second launch costs more than the split saves
    int64_t s = 256 / wgs;
    if (s > K / 4096) s = K / 4096;
    if (s > 64) s = 64;
    return s < 2 ? 1 : static_cast<int>(s);
}

hipError_t launch_generic(const GemmArgs& a, hipStream_t s) {
    const int slices = (a.workspace && a.workspace_bytes > 0) ? generic_splitk_slices(a.N, a.K, a.layout) : 1;
    switch (a.bits) {
        case 1: return launch_generic_bits<1>(a, slices, s);
        case 2: return launch_generic_bits<2>(a, slices, s);
        case 3: return launch_generic_bits<3>(a, slices, s);
        case 8: return launch_generic_bits<8>(a, slices, s);
        default: return launch_generic_bits<4>(a, slices, s);
    }
}

hipError_t launch_dequant(const uint32_t* W, const uint16_t* codebook, uint16_t* Wd, int64_t N,
                          int64_t K, int bits, int layout, hipStream_t s) {
    if (layout == KMQ_LAYOUT_CANONICAL && (K & 7) == 0 && (reinterpret_cast<uintptr_t>(Wd) & 15) == 0 &&
        N * (K >> 3) <= (int64_t(1) << 38)) {                  // one workgroup per 256 chunks must fit the grid
        const int64_t chunks = N * (K >> 3);
        const dim3 grid8(static_cast<unsigned>((chunks + 255) / 256)), block8(256);
        switch (bits) {
            case 1: hipLaunchKernelGGL(dequant_rows8_kernel<1>, grid8, block8, 0, s, W, codebook, Wd, N, K); break;
            case 2: hipLaunchKernelGGL(dequant_rows8_kernel<2>, grid8, block8, 0, s, W, codebook, Wd, N, K); break;
            case 3: hipLaunchKernelGGL(dequant_rows8_kernel<3>, grid8, block8, 0, s, W, codebook, Wd, N, K); break;
            case 8: hipLaunchKernelGGL(dequant_rows8_kernel<8>, grid8, block8, 0, s, W, codebook, Wd, N, K); break;
            default: hipLaunchKernelGGL(dequant_rows8_kernel<4>, grid8, block8, 0, s, W, codebook, Wd, N, K); break;
        }
        return hipGetLastError();
    }
    const int64_t total = N * ((K + 31) >> 5);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    const dim3 grid(static_cast<unsigned>(blocks)), block(256);
    switch (bits) {
        case 1: hipLaunchKernelGGL(dequant_kernel<1>, grid, block, 0, s, W, codebook, Wd, N, K, layout); break;
        case 2: hipLaunchKernelGGL(dequant_kernel<2>, grid, block, 0, s, W, codebook, Wd, N, K, layout); break;
        case 3: hipLaunchKernelGGL(dequant_kernel<3>, grid, block, 0, s, W, codebook, Wd, N, K, layout); break;
        case 8: hipLaunchKernelGGL(dequant_kernel<8>, grid, block, 0, s, W, codebook, Wd, N, K, layout); break;
        default: hipLaunchKernelGGL(dequant_kernel<4>, grid, block, 0, s, W, codebook, Wd, N, K, layout); break;
    }
    return hipGetLastError();
}

}  // namespace kmq
