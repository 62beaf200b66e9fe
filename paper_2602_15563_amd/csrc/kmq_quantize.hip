// The quantiser that produces the k-means weight formats from dense bf16 weights
// (paper Sec. 2.1 "Rounding to nearest centroids": f_c(x) = argmin_{c_i} |x - c_i| with
// the centroids from 1-D k-means clustering; "Block formats"; Sec. 2.2 "Nonlinear
// k-means quantization": per tensor, on weights normalised by a 16-bit scale per block
// of 64 elements).  The paper names Lloyd's algorithm and leaves its details open; the
// rules fixed here (kmq.h states them for callers):
//
//   * fp64 throughout; centroids stay sorted; a value is assigned to the cluster whose
//     index is the number of boundaries (c_i + c_{i+1}) / 2 below it (a value on a boundary
//     goes down); an empty cluster keeps its centroid; exactly `iters` rounds;
//   * start: 2^b points evenly spaced over the data's range (row min..max, or [-1, 1]
//     for normalised weights);
//   * the stored codebook is the centroids rounded to bf16 (nearest even) and the indices
//     are nearest STORED centroids.
//
// Sums of a cluster's members are formed per lane, then over a wave's lanes, then over
// waves (and workgroups) in a fixed order: deterministic, and exact whenever the members'
// exponents span fewer than 53 - log2(count) bits (always so for rows of bf16 weights of
// one layer), in which case the result does not depend on the order at all.
//
// Compiled with floating-point contraction off: the arithmetic is specified operation by
// operation.
#include "kmq_device.h"
#include "kmq_launch.h"

#pragma clang fp contract(off)

namespace kmq {

__device__ __forceinline__ double bf16_to_f64(uint32_t h) { return static_cast<double>(__uint_as_float(h << 16)); }

// Nearest-even rounding of a finite double to bf16, decided on the double's own bits.
// Magnitudes below bf16's normal range give zero.
__device__ __forceinline__ uint16_t f64_to_bf16(double c) {
    const uint64_t u = static_cast<uint64_t>(__double_as_longlong(c));
    const uint32_t sign = static_cast<uint32_t>(u >> 63) << 15;
    const int e32 = static_cast<int>((u >> 52) & 0x7FF) - 1023 + 127;
    if (e32 <= 0) return static_cast<uint16_t>(sign);
    const uint64_t mant = u & ((1ull << 52) - 1);
    uint32_t m7 = static_cast<uint32_t>(mant >> 45);
    const uint64_t rem = mant & ((1ull << 45) - 1), half = 1ull << 44;
    if (rem > half || (rem == half && (m7 & 1u))) ++m7;
    return static_cast<uint16_t>(sign | ((static_cast<uint32_t>(e32) << 7) + m7));   // m7 == 128 carries into the exponent
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ long long wave_sum(long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int C>
struct Clusters {
    double b[C > 1 ? C - 1 : 1];   // boundaries
    double s[C];
    int n[C];                      // per lane: at most a few thousand members, widened when lanes are added up
    __device__ __forceinline__ void begin(const double* c) {
#pragma unroll
        for (int i = 0; i + 1 < C; ++i) b[i] = 0.5 * (c[i] + c[i + 1]);
#pragma unroll
        for (int j = 0; j < C; ++j) { s[j] = 0.0; n[j] = 0; }
    }
    __device__ __forceinline__ int assign(double v) const {
        int a = 0;
#pragma unroll
        for (int i = 0; i + 1 < C; ++i) a += v > b[i] ? 1 : 0;
        return a;
    }
    __device__ __forceinline__ void add(double v) {
        const int a = assign(v);
#pragma unroll
        for (int j = 0; j < C; ++j) {       // compile-time j: the sums stay in registers
            s[j] += a == j ? v : 0.0;
            n[j] += a == j ? 1 : 0;
        }
    }
};

// 32 consecutive indices -> BITS words of the canonical stream (LSB first, 3-bit fields may straddle).
template <int BITS>
struct GroupPacker {
    uint32_t w[BITS];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int j = 0; j < BITS; ++j) w[j] = 0;
    }
    template <int E>
    __device__ __forceinline__ void put(uint32_t a) {
        constexpr int p = E * BITS, wi = p >> 5, sh = p & 31;
        w[wi] |= a << sh;
        if constexpr (sh + BITS > 32) w[wi + 1] |= a >> (32 - sh);
    }
};

template <int BITS, int E = 0, typename F>
__device__ __forceinline__ void pack_group(GroupPacker<BITS>& g, F&& index_of) {
    if constexpr (E < 32) {
        g.template put<E>(index_of(E));
        pack_group<BITS, E + 1>(g, index_of);
    }
}

// ---- one codebook per row ------------------------------------------------------------------------
// One workgroup of four waves per row; the row is re-read from the caches each round.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const uint16_t* __restrict__ W, int64_t K, int iters,
                                                            uint32_t* __restrict__ packed,
                                                            uint16_t* __restrict__ codebook) {
    constexpr int C = 1 << BITS;
    __shared__ double cs[C];
    __shared__ double ps[4][C];
    __shared__ long long pn[4][C];
    __shared__ double plo[4], phi[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n = blockIdx.x;
    const uint16_t* w = W + n * K;

    double lo = __builtin_huge_val(), hi = -__builtin_huge_val();
    for (int64_t k = tid; k < K; k += 256) {
        const double v = bf16_to_f64(w[k]);
        lo = v < lo ? v : lo;
        hi = v > hi ? v : hi;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double l2 = __shfl_xor(lo, off, 64), h2 = __shfl_xor(hi, off, 64);
        lo = l2 < lo ? l2 : lo;
        hi = h2 > hi ? h2 : hi;
    }
    if (lane == 0) { plo[wave] = lo; phi[wave] = hi; }
    __syncthreads();
    if (tid < C) {
        double l = plo[0], h = phi[0];
#pragma unroll
        for (int q = 1; q < 4; ++q) { l = plo[q] < l ? plo[q] : l; h = phi[q] > h ? phi[q] : h; }
        cs[tid] = l + (tid + 0.5) * (h - l) / C;
    }
    __syncthreads();

    Clusters<C> cl;
    double c[C];
    for (int t = 0; t < iters; ++t) {
#pragma unroll
        for (int j = 0; j < C; ++j) c[j] = cs[j];
        cl.begin(c);
        for (int64_t k = tid; k < K; k += 256) cl.add(bf16_to_f64(w[k]));
#pragma unroll
        for (int j = 0; j < C; ++j) {
            const double s = wave_sum(cl.s[j]);
            const long long m = wave_sum(static_cast<long long>(cl.n[j]));
            if (lane == 0) { ps[wave][j] = s; pn[wave][j] = m; }
        }
        __syncthreads();
        if (tid < C) {
            const double s = ((ps[0][tid] + ps[1][tid]) + ps[2][tid]) + ps[3][tid];
            const long long m = pn[0][tid] + pn[1][tid] + pn[2][tid] + pn[3][tid];
            if (m > 0) cs[tid] = s / static_cast<double>(m);
        }
        __syncthreads();
    }

    if (tid < C) {
        const uint16_t h = f64_to_bf16(cs[tid]);
        codebook[n * C + tid] = h;
        cs[tid] = bf16_to_f64(h);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < C; ++j) c[j] = cs[j];
    cl.begin(c);
    const int64_t wpr = words_per_row(BITS, K), ngroups = (K + 31) >> 5;
    for (int64_t g = tid; g < ngroups; g += 256) {
        GroupPacker<BITS> gp;
        gp.clear();
        const int64_t k0 = g << 5;
        pack_group<BITS>(gp, [&](int e) -> uint32_t {
            return k0 + e < K ? static_cast<uint32_t>(cl.assign(bf16_to_f64(w[k0 + e]))) : 0u;
        });
#pragma unroll
        for (int j = 0; j < BITS; ++j)
            if (g * BITS + j < wpr) packed[n * wpr + g * BITS + j] = gp.w[j];
    }
}

// ---- the paper's format: scale per 64-element block, one codebook per tensor -------------------------
constexpr int kQuantPartials = 1024;   // workgroups of a clustering pass = partial sums per cluster

struct QuantScratch {                  // layout of the caller's workspace
    double cent[16];
    double psum[kQuantPartials][16];
    long long pcnt[kQuantPartials][16];
};

// scale = largest magnitude of the block (bf16 magnitudes order like their bit patterns); wave per block
__global__ __launch_bounds__(256) void bs_scales_kernel(const uint16_t* __restrict__ W, int64_t nblocks,
                                                        uint16_t* __restrict__ scales, QuantScratch* q, int C) {
    const int lane = threadIdx.x & 63;
    const int64_t blk = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (blockIdx.x == 0 && threadIdx.x < C) q->cent[threadIdx.x] = -1.0 + (2 * static_cast<int>(threadIdx.x) + 1) / static_cast<double>(C);
    if (blk >= nblocks) return;
    int mag = W[blk * KMQ_BLOCK + lane] & 0x7FFF;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const int o = __shfl_xor(mag, off, 64);
        mag = o > mag ? o : mag;
    }
    if (lane == 0) scales[blk] = static_cast<uint16_t>(mag);
}

__device__ __forceinline__ double normalised(uint32_t w, uint32_t scale) {
    const double s = bf16_to_f64(scale);
    return s > 0.0 ? bf16_to_f64(w) / s : 0.0;
}

// one clustering round, first half: every workgroup sums the members of each cluster over its blocks
template <int BITS>
__global__ __launch_bounds__(256) void bs_lloyd_pass_kernel(const uint16_t* __restrict__ W,
                                                            const uint16_t* __restrict__ scales, int64_t nblocks,
                                                            QuantScratch* q) {
    constexpr int C = 1 << BITS;
    __shared__ double ps[4][C];
    __shared__ long long pn[4][C];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double c[C];
#pragma unroll
    for (int j = 0; j < C; ++j) c[j] = q->cent[j];
    Clusters<C> cl;
    cl.begin(c);
    // a lane takes 8 consecutive elements (one 16-byte load; eight lanes share a block's scale), a wave 8 blocks
    const int64_t nchunks = nblocks * (KMQ_BLOCK / 8);
    for (int64_t c = (static_cast<int64_t>(blockIdx.x) * 4 + wave) * kWave + lane; c < nchunks;
         c += static_cast<int64_t>(gridDim.x) * 4 * kWave) {
        const u32x4_t w8 = *reinterpret_cast<const u32x4_t*>(W + c * 8);
        const uint32_t scale = scales[c >> 3];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            cl.add(normalised(w8[e] & 0xFFFFu, scale));
            cl.add(normalised(w8[e] >> 16, scale));
        }
    }
#pragma unroll
    for (int j = 0; j < C; ++j) {
        const double s = wave_sum(cl.s[j]);
        const long long m = wave_sum(static_cast<long long>(cl.n[j]));
        if (lane == 0) { ps[wave][j] = s; pn[wave][j] = m; }
    }
    __syncthreads();
    if (tid < C) {
        q->psum[blockIdx.x][tid] = ((ps[0][tid] + ps[1][tid]) + ps[2][tid]) + ps[3][tid];
        q->pcnt[blockIdx.x][tid] = pn[0][tid] + pn[1][tid] + pn[2][tid] + pn[3][tid];
    }
}

// second half: partial sums added in workgroup order, centroids updated; on the last round the
// codebook is written as well
__global__ __launch_bounds__(64) void bs_lloyd_update_kernel(QuantScratch* q, int C, int partials, bool update,
                                                             uint16_t* __restrict__ codebook) {
    const int j = threadIdx.x;
    if (j >= C) return;
    if (update) {
        double s = 0.0;
        long long m = 0;
        for (int p = 0; p < partials; ++p) { s += q->psum[p][j]; m += q->pcnt[p][j]; }
        if (m > 0) q->cent[j] = s / static_cast<double>(m);
    }
    if (codebook) codebook[j] = f64_to_bf16(q->cent[j]);
}

// nearest stored centroid for every element, packed; one thread per 32 elements
template <int BITS>
__global__ __launch_bounds__(256) void bs_assign_pack_kernel(const uint16_t* __restrict__ W,
                                                             const uint16_t* __restrict__ scales,
                                                             const uint16_t* __restrict__ codebook, int64_t ngroups,
                                                             uint32_t* __restrict__ packed) {
    constexpr int C = 1 << BITS;
    const int64_t g = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (g >= ngroups) return;
    double c[C];
#pragma unroll
    for (int j = 0; j < C; ++j) c[j] = bf16_to_f64(codebook[j]);
    Clusters<C> cl;
    cl.begin(c);
    const uint32_t scale = scales[g >> 1];
    const uint16_t* w = W + (g << 5);
    GroupPacker<BITS> gp;
    gp.clear();
    pack_group<BITS>(gp, [&](int e) -> uint32_t { return static_cast<uint32_t>(cl.assign(normalised(w[e], scale))); });
#pragma unroll
    for (int j = 0; j < BITS; ++j) packed[g * BITS + j] = gp.w[j];
}

size_t quantize_blockscaled_workspace_bytes() { return sizeof(QuantScratch); }

template <int BITS>
static hipError_t quantize_rows_bits(const uint16_t* W, int64_t N, int64_t K, int iters, uint32_t* packed,
                                     uint16_t* codebook, hipStream_t s) {
    hipLaunchKernelGGL((quantize_rows_kernel<BITS>), dim3(static_cast<unsigned>(N)), dim3(256), 0, s, W, K, iters, packed,
                       codebook);
    return hipGetLastError();
}

hipError_t launch_quantize_rows(const uint16_t* W, int64_t N, int64_t K, int bits, int iters, uint32_t* packed,
                                uint16_t* codebook, hipStream_t s) {
    switch (bits) {
        case 1: return quantize_rows_bits<1>(W, N, K, iters, packed, codebook, s);
        case 2: return quantize_rows_bits<2>(W, N, K, iters, packed, codebook, s);
        case 3: return quantize_rows_bits<3>(W, N, K, iters, packed, codebook, s);
        default: return quantize_rows_bits<4>(W, N, K, iters, packed, codebook, s);
    }
}

template <int BITS>
static hipError_t quantize_blockscaled_bits(const uint16_t* W, int64_t N, int64_t K, int iters, uint32_t* packed,
                                            uint16_t* codebook, uint16_t* scales, QuantScratch* q, hipStream_t s) {
    constexpr int C = 1 << BITS;
    const int64_t nblocks = N * (K / KMQ_BLOCK), ngroups = nblocks * 2;
    const int64_t want = (nblocks + 31) / 32;          // a wave takes 8 blocks at a time
    const int partials = static_cast<int>(want < kQuantPartials ? want : kQuantPartials);
    hipLaunchKernelGGL(bs_scales_kernel, dim3(static_cast<unsigned>((nblocks + 3) / 4)), dim3(256), 0, s, W, nblocks, scales, q, C);
    for (int t = 0; t < iters; ++t) {
        hipLaunchKernelGGL((bs_lloyd_pass_kernel<BITS>), dim3(partials), dim3(256), 0, s, W, scales, nblocks, q);
        hipLaunchKernelGGL(bs_lloyd_update_kernel, dim3(1), dim3(64), 0, s, q, C, partials, true,
                           t + 1 == iters ? codebook : static_cast<uint16_t*>(nullptr));
    }
    if (iters == 0)
        hipLaunchKernelGGL(bs_lloyd_update_kernel, dim3(1), dim3(64), 0, s, q, C, 0, false, codebook);
    hipLaunchKernelGGL((bs_assign_pack_kernel<BITS>), dim3(static_cast<unsigned>((ngroups + 255) / 256)), dim3(256), 0, s, W,
                       scales, codebook, ngroups, packed);
    return hipGetLastError();
}

hipError_t launch_quantize_blockscaled(const uint16_t* W, int64_t N, int64_t K, int bits, int iters, uint32_t* packed,
                                       uint16_t* codebook, uint16_t* scales, void* workspace, hipStream_t s) {
    QuantScratch* q = static_cast<QuantScratch*>(workspace);
    switch (bits) {
        case 1: return quantize_blockscaled_bits<1>(W, N, K, iters, packed, codebook, scales, q, s);
        case 2: return quantize_blockscaled_bits<2>(W, N, K, iters, packed, codebook, scales, q, s);
        case 3: return quantize_blockscaled_bits<3>(W, N, K, iters, packed, codebook, scales, q, s);
        default: return quantize_blockscaled_bits<4>(W, N, K, iters, packed, codebook, scales, q, s);
    }
}

}  // namespace kmq
