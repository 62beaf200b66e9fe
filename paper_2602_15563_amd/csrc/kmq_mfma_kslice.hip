// Small-batch product Y = X W^T on the matrix cores, tiled layout, 2- and 3-bit per-row codebooks,
// for rows short enough that a wave can keep its slice of the activations in registers
// (K <= 16 waves x 8 matrix steps x 32 columns = 4096): the batch-8 / batch-16 shapes of the
// benchmark contract (paper App. D: up to a batch of a few tens the product stays bound by the
// transfer of W provided every weight is dequantised once; App. E "Micro-benchmarks").
//
// The general matrix-core kernel (kmq_mfma.hip) gives every wave a run of super-blocks of ONE or two
// row blocks and re-stages the activations of every chunk through LDS for them, which leaves a CU
// with two waves per SIMD and an LDS round trip in front of every fourth matrix instruction.  Here
// the work is cut the other way round:
//   * a workgroup is NWK waves that split K; wave w owns the same SPW super-blocks (STEPS = SPW *
//     steps-per-super-block matrix steps) of EVERY row block of the workgroup;
//   * the wave's B operands (the X^T slices of its STEPS steps: 4 VGPRs each) are fetched ONCE,
//     transposed through a wave-private LDS tile exactly as in the general kernel, and then stay in
//     registers for all row blocks;
//   * the grid is at most 256 workgroups (one per CU, 4 waves per SIMD with NWK = 16); workgroup b
//     takes the RPW adjacent row blocks b * RPW ..; every index granule of all its row blocks is
//     requested before the first one is decoded;
//   * the main loop is then nothing but decode (v_perm_b32 on the lane's codebook pools, as in the
//     general kernel) and v_mfma_f32_16x16x32_bf16, with no memory or LDS instruction in it.
// Partial 16x16 tiles of the waves are summed through LDS in a fixed order (deterministic).
#include <cstdlib>

#include "kmq_device.h"
#include "kmq_launch.h"

namespace kmq {

namespace kslice {

template <int BITS> struct Tiled {
    static constexpr int GPG = BITS == 2 ? 8 : 4;        // matrix steps per super-block (granule)
    static constexpr int GW = GPG * BITS / 4;            // dwords per granule
    static constexpr int SBE = 32 * GPG;                 // elements per super-block
};

template <int GW>
__device__ __forceinline__ void load_granule(const uint32_t* p, uint32_t (&g)[GW]) {
    if constexpr (GW == 3) {
        typedef u32x3_t __attribute__((aligned(4))) u32x3_a4_t;
        const u32x3_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x3_a4_t*>(p));
        g[0] = t[0]; g[1] = t[1]; g[2] = t[2];
    } else {
        const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        g[0] = t[0]; g[1] = t[1]; g[2] = t[2]; g[3] = t[3];
    }
}

// The eight weights of matrix step j of a granule as four registers of bf16 pairs.  The tiled layout
// (include/kmq.h) spreads the index fields so that a shift and an AND leave four indices in the four
// bytes of a register, a v_perm_b32 selector into the low-byte and high-byte pools of the lane's
// centroids; two more permutes interleave the gathered bytes.
template <int BITS>
__device__ __forceinline__ u32x4_t decode_step(const uint32_t* D, int j, uint32_t lo0, uint32_t lo1, uint32_t hi0, uint32_t hi1) {
    u32x4_t a;
#pragma unroll
    for (int h = 0; h < 2; ++h) {      // elements 4h..4h+3 of this step
        uint32_t sel;
        if constexpr (BITS == 2) {
            const int c = 2 * j + h;
            sel = (D[c >> 2] >> (2 * (c & 3))) & 0x03030303u;
        } else {
            if (j < 3) sel = (h == 0 ? D[j] : D[j] >> 3) & 0x07070707u;
            else if (h == 0) sel = ((D[0] >> 6) & 0x03030303u) | ((D[1] >> 4) & 0x04040404u);
            else sel = ((D[1] >> 7) & 0x01010101u) | ((D[2] >> 5) & 0x06060606u);
        }
        const uint32_t lo = __builtin_amdgcn_perm(lo1, lo0, sel);
        const uint32_t hi = __builtin_amdgcn_perm(hi1, hi0, sel);
        a[2 * h] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
        a[2 * h + 1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
    }
    return a;
}

}  // namespace kslice

constexpr int kKsliceMaxWaves = 16;
#ifndef KMQ_KS_DBG
#define KMQ_KS_DBG 0     // instrumented builds: 1 no index loads, 2 one decode + matrix step per granule instead of all
#endif

// BITS 2 or 3; SPW super-blocks per wave; RPW row blocks per workgroup at most.  blockDim.x = 64 * NWK with
// NWK * SPW super-blocks = K; workgroup b owns row blocks b * RPW + i, i < RPW.
template <int BITS, int SPW, int RPW>
__global__ __launch_bounds__(1024) void gemm_mfma_kslice_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int64_t N, int64_t K, int M) {
    using namespace kslice;
    using T = Tiled<BITS>;
    constexpr int GPG = T::GPG, GW = T::GW, SBE = T::SBE, C = 1 << BITS;
    constexpr int STEPS = SPW * GPG;                        // matrix steps of a wave per row block
    constexpr int CHUNKS = STEPS / 4;                       // 128-column chunks of the wave's slice
    static_assert(STEPS % 4 == 0 && STEPS <= 8, "the wave's B operands stay in registers");
    static_assert(RPW >= 1 && RPW <= 4, "row blocks per workgroup");
    struct alignas(256) Smem {
        // per wave: 16 batch rows x (16 + 1 pad) 16-byte pieces of activations; afterwards the same memory
        // holds the wave's RPW partial 16x16 tiles ([batch column][row, padded to 17] floats)
        u32x4_t xstage[kKsliceMaxWaves][16 * 17];
    };
    __shared__ Smem sm;
    static_assert(RPW * 16 * 17 * sizeof(float) <= 16 * 17 * sizeof(u32x4_t), "partial tiles reuse the activation tile");

    const int wk = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nwk = static_cast<int>(blockDim.x >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int64_t nrb = (N + 15) >> 4;
    const int nsb = static_cast<int>(K / SBE);
    const int sb0 = wk * SPW;
    // row blocks of this workgroup (clamped copies past the end keep every load in bounds; they are never stored)
    int cnt = 0;
    int64_t rbs[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int64_t rb = static_cast<int64_t>(blockIdx.x) * RPW + r;      // adjacent row blocks: a batch column's outputs of the workgroup are one run of RPW * 32 bytes
        if (rb < nrb) cnt = r + 1;
        rbs[r] = rb < nrb ? rb : nrb - 1;
    }

    // ---- loads: codebooks, activations of the wave's slice, then every granule, in the order of use ----
    uint32_t lo0[RPW], lo1[RPW], hi0[RPW], hi1[RPW];        // perm pools: low / high bytes of the lane's centroids
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        int row = static_cast<int>(rbs[r]) * 16 + n;         // (row numbers fit 32 bits: the library caps N at 2^24)
        row = row < static_cast<int>(N) ? row : static_cast<int>(N) - 1;
        const uint32_t* cw = reinterpret_cast<const uint32_t*>(codebook + static_cast<int64_t>(row) * C);
        // v_perm_b32(S0, S1, sel): selector values 0..3 pick bytes of S1, 4..7 bytes of S0
        lo0[r] = __builtin_amdgcn_perm(cw[1], cw[0], 0x06040200u);
        hi0[r] = __builtin_amdgcn_perm(cw[1], cw[0], 0x07050301u);
        if constexpr (BITS == 3) {
            lo1[r] = __builtin_amdgcn_perm(cw[3], cw[2], 0x06040200u);
            hi1[r] = __builtin_amdgcn_perm(cw[3], cw[2], 0x07050301u);
        } else {
            lo1[r] = lo0[r];
            hi1[r] = hi0[r];
        }
    }
    // activations: 256 contiguous bytes per batch row and chunk (lane (n, q) fetches bytes 16n.. of row 4i + q);
    // batch columns >= M are fed row M - 1 and dropped at the end
    const char* xbase = reinterpret_cast<const char*>(X + static_cast<int64_t>(sb0) * SBE);
    u32x4_t bfrag[STEPS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int m = 4 * i + q;
            m = m < M ? m : M - 1;
            const uint32_t off = (static_cast<uint32_t>(m) * static_cast<uint32_t>(K) + 8u * n) * 2u + static_cast<uint32_t>(c) * 256u;
            bfrag[4 * c + i] = *reinterpret_cast<const u32x4_t*>(xbase + off);
        }
    }
    const int64_t gstride = 64 * GW;                        // dwords per (row block, super-block) tile
    uint32_t gran[RPW][SPW][GW];
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
        for (int s = 0; s < SPW; ++s)
#if KMQ_KS_DBG == 1
            { for (int g = 0; g < GW; ++g) gran[r][s][g] = (lane * 0x9E3779B9u + r * 77u + s * 1315423911u + g) * 2654435761u; }
#else
            load_granule<GW>(W + (rbs[r] * nsb + sb0 + s) * gstride + lane * GW, gran[r][s]);
#endif

    __builtin_amdgcn_sched_barrier(0);                      // every load is requested before anything waits for one

    // ---- B operands: through the wave's LDS tile, piece (q + 4i) of batch row n for step i of the chunk ----
    u32x4_t* xtile = &sm.xstage[wk][0];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
        for (int i = 0; i < 4; ++i) xtile[(4 * i + q) * 17 + n] = bfrag[4 * c + i];
#pragma unroll
        for (int i = 0; i < 4; ++i) bfrag[4 * c + i] = xtile[n * 17 + q + 4 * i];
    }

    // ---- decode and multiply: no memory instruction in here ----
    f32x4_t acc[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) acc[r] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        // no `r < cnt` test here: only the last workgroup has clamped copies to skip, and a load whose only use
        // sits behind a branch is sunk into it by the compiler, i.e. requested a whole memory latency late
#pragma unroll
        for (int s = 0; s < SPW; ++s)
#pragma unroll
            for (int j = 0; j < GPG; ++j) {
#if KMQ_KS_DBG == 2
                if (j > 0) { acc[r][0] += __uint_as_float(gran[r][s][j % GW] & 0x3FFFFFFFu); continue; }
#endif
                const u32x4_t a = decode_step<BITS>(gran[r][s], j, lo0[r], lo1[r], hi0[r], hi1[r]);
                acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                                __builtin_bit_cast(bf16x8_t, bfrag[s * GPG + j]), acc[r], 0, 0, 0);
            }
    }

    // ---- K-reduction across the waves, fixed order: lane holds D[row 4q + i][batch column n] ----
    // (one output per thread, every thread busy: four rows per thread with 16-byte LDS accesses and 8-byte
    // stores leaves three quarters of the waves idle behind a chain of 16 loads and measured 3 % slower; a
    // reduction per row block, overlapped with the next block's decode, costs a barrier per block and
    // measured 19 % slower)
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) reinterpret_cast<float*>(xtile)[(r * 16 + n) * 17 + 4 * q + i] = acc[r][i];
    __syncthreads();
    for (int o = threadIdx.x; o < RPW * 256; o += blockDim.x) {
        const int m = o / (RPW * 16), nl = o % (RPW * 16);  // consecutive threads -> consecutive rows
        const int r = nl >> 4, nn = nl & 15;
        float s = 0.f;
        for (int k = 0; k < nwk; ++k) s += reinterpret_cast<const float*>(&sm.xstage[k][0])[(r * 16 + m) * 17 + nn];
        const int row = (static_cast<int>(blockIdx.x) * RPW + r) * 16 + nn;
        if (r < cnt && m < M && row < static_cast<int>(N)) Y[static_cast<int64_t>(m) * N + row] = f32_to_bf16(s);
    }
}

// ---- launch ------------------------------------------------------------------------------------

struct KsliceShape { int nwk, spw, rpw, grid; };

// NWK = the most waves (<= 16) that divide the super-blocks with at most 8 matrix steps each; the grid is one
// workgroup per CU at most, each with ceil(row blocks / grid) <= 4 row blocks.
static bool kslice_shape(int64_t N, int64_t K, int bits, KsliceShape& s) {
    if (bits != 2 && bits != 3) return false;
    // rows of 3072 and 4096 columns: 12 to 16 waves with eight matrix steps each.  Shorter rows leave a wave too
    // little work per row block next to its share of the 16-way reduction (batch 8, 14336 rows, K = 2048,
    // 2 bits: 5.4 us here against 5.25 us in the general kernel; at K = 3072 this kernel is ahead at 2 and 3 bits).
    if (K < 3072) return false;
    const int64_t sbe = tiled_superblock_elems(bits);
    if (K % sbe != 0) return false;
    const int64_t nsb = K / sbe;
    const int max_spw = bits == 2 ? 1 : 2;                  // 8 steps per wave
    int nwk = 0, spw = 0;
    for (int w = kKsliceMaxWaves; w >= 1; --w)
        if (nsb % w == 0 && nsb / w <= max_spw) { nwk = w; spw = static_cast<int>(nsb / w); break; }
    if (!nwk || spw != max_spw) return false;               // (eight steps per wave: the only instances built)
    const int64_t nrb = (N + 15) / 16;
    const int64_t grid = nrb < 256 ? nrb : 256;
    const int64_t rpw = (nrb + grid - 1) / grid;
    // one row block per workgroup is the general kernel's ground (3-bit 4096 x 4096, batch 8: 4.55 us there, 4.76 us here:
    // sixteen waves for eight matrix steps each); a grid that leaves a quarter of the CUs idle is not worth it either
    if (rpw < 2 || rpw > 4 || (nrb + rpw - 1) / rpw < 192) return false;
    // no more workgroups than rpw row blocks each need: 14336 rows are 224 workgroups of four row blocks rather than 256 of
    // three or four (5 % slower at batch 8 and 16 of the 3-bit 14336 x 4096 shape) -- every workgroup
    // fetches all of X
    s = {nwk, spw, static_cast<int>(rpw), static_cast<int>((nrb + rpw - 1) / rpw)};
    return true;
}

bool mfma_kslice_has_kernel(int64_t N, int64_t K, int bits) {
#ifdef KMQ_TUNING
    static const char* const off = std::getenv("KMQ_MFMA_NO_KSLICE");       // sweeps only: builds with -DKMQ_TUNING
    if (off) return false;
#endif
    KsliceShape s;
    return kslice_shape(N, K, bits, s);
}

template <int BITS, int SPW>
static void launch_kslice_rpw(const GemmArgs& a, const KsliceShape& s, hipStream_t st) {
    const dim3 grid(s.grid), block(64 * s.nwk);
#define KMQ_KS(RPW) hipLaunchKernelGGL((gemm_mfma_kslice_kernel<BITS, SPW, RPW>), grid, block, 0, st, a.W, a.codebook, a.X, a.Y, a.N, a.K, a.M)
    switch (s.rpw) { case 1: KMQ_KS(1); break; case 2: KMQ_KS(2); break; case 3: KMQ_KS(3); break; default: KMQ_KS(4); break; }
#undef KMQ_KS
}

hipError_t launch_mfma_kslice(const GemmArgs& a, hipStream_t st) {
    KsliceShape s;
    if (!kslice_shape(a.N, a.K, a.bits, s) || a.scales) return hipErrorInvalidValue;
    if (a.bits == 2 && s.spw == 1) launch_kslice_rpw<2, 1>(a, s, st);
    else if (a.bits == 3 && s.spw == 2) launch_kslice_rpw<3, 2>(a, s, st);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace kmq
