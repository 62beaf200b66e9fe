// Small-batch product Y = X W^T on the matrix cores, tiled layout, any batch
// 1..16 (paper App. D/E: up to a batch of a few tens the product is still bound
// by the transfer of W, provided each weight is dequantised once and reused for
// every batch column).
//
// One v_mfma_f32_16x16x32_bf16 step multiplies a 16-row x 32-column tile of
// dequantised W (A operand) by the matching 32 x 16 slice of X^T (B operand;
// batch columns beyond M are computed and dropped).  Lane (n, q) = (lane & 15,
// lane >> 4) supplies 8 weights of row n and 8 activations of batch column n,
// both for columns 8*(q + 4j)..+7 of the current super-block at step j: the
// tiled layout stores exactly those groups contiguously per lane (a granule),
// so the index stream is read with one 12- or 16-byte load per lane and
// super-block, and the activation loads of a step cover 64 contiguous bytes of
// each batch row.
//
// Dequantisation per step and lane (8 weights -> 4 VGPRs of bf16 pairs):
//   2/3-bit  the lane's row codebook (8 or 16 bytes) lives in VGPRs, split into a
//            low-byte and a high-byte pool; the tiled granule stores the index
//            fields spread so that one shift + AND yields four indices in the
//            four bytes of a register, which is a v_perm_b32 selector: two byte
//            gathers (low, high) and two interleaves per four weights, no LDS;
//   4-bit    16 centroids do not fit a perm pool: tables in LDS, one column (= bank) per lane so that
//            lookups never collide, the index dropped into byte 1 of the address by one instruction;
//            with a tensor-wide codebook and long rows, a table of centroid pairs indexed by a whole byte;
//   1-bit    no per-row table: the A operand is the {0,1} mask of the bits
//            (row-independent nibble table in LDS), a second MFMA with an all-ones
//            A operand accumulates sum_k x, and the epilogue applies the closed
//            form y = c0*sum(x) + (c1 - c0)*sum_{idx=1} x.
//
// A workgroup is NWK waves that split K (whole super-blocks each) for RBW blocks
// of 16 rows; partial 16x16 tiles are summed through LDS in a fixed order.
#include <cstdlib>
#include <type_traits>

#include "kmq_device.h"
#include "kmq_launch.h"

namespace kmq {

constexpr int kPrefetch = 4;   // super-blocks of index granules in flight per wave

template <int BITS> struct Tiled {
    static constexpr int GPG = BITS == 1 ? 16 : BITS == 2 ? 8 : 4;   // groups (MFMA steps) per granule
    static constexpr int GW = GPG * BITS / 4;                        // dwords per granule
    static constexpr int SBE = 32 * GPG;                             // elements per super-block
};

template <int GW>
__device__ __forceinline__ void load_granule(const uint32_t* p, uint32_t (&g)[GW]) {
    if constexpr (GW == 3) {
        // 12-byte granules sit 4-byte aligned; read once, so kept out of the caches like the others
        typedef u32x3_t __attribute__((aligned(4))) u32x3_a4_t;
        const u32x3_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x3_a4_t*>(p));
        g[0] = t[0]; g[1] = t[1]; g[2] = t[2];
    } else {
        const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        g[0] = t[0]; g[1] = t[1]; g[2] = t[2]; g[3] = t[3];
    }
}

// 1- and 4-bit granules: the bits*8 index bits of group j, in the low bits of the result.
template <int BITS, int GW>
__device__ __forceinline__ uint32_t group_bits(const uint32_t (&g)[GW], int j) {
    if constexpr (BITS == 4) return g[j];
    if constexpr (BITS == 1) return (g[j >> 2] >> (8 * (j & 3))) & 0xFFu;
    return 0;
}

// SPW > 0 fixes the number of super-blocks per wave at compile time: the K loop is then
// fully unrolled and has no back edge.  That matters beyond loop overhead: with loads in
// flight across a back edge the compiler's s_waitcnt vmcnt() placement becomes
// conservative and drains the whole prefetch queue at every iteration.  SPW = 0 is the
// general (runtime trip count) version.
//
// SC selects the paper's own weight format (Sec. 2.2 "Nonlinear k-means quantization"; App. E
// "Kernel implementations", deferred scaling): `codebook` is one table for the whole tensor and
// `scales` holds one bf16 per 64 elements of a row.  A block of 64 columns is two MFMA steps:
// their 16x16 product starts from zero and is added to the running tile multiplied by the
// scales of its four output rows.  The workgroup's scales are staged once, transposed, in LDS
// (kMaxScaledBlocks blocks of K at most).
constexpr int kMaxScaledBlocks = 256;          // K <= 16384 for the scaled matrix-core path
// Staged scales: 16 rows of a K block take 20 entries, not 16.  Staging transposes (a lane reads eight
// consecutive blocks of one row and writes them 8 x kSctRow entries apart); with 16 lanes on 16 rows and
// the wave's four lane groups on four runs of eight blocks, a stride of 20 puts the groups 16 banks
// apart, so the 64 two-byte writes of an instruction fall into 32 distinct dwords in 32 banks.  A stride
// of 16 would put all of them into the same eight banks.  (Multiple of four: the reader's 8-byte loads.)
constexpr int kSctRow = 20;

typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;

// byte 1 of `a` <- (byte BYTE of src) & mask, other bytes of `a` kept: drops a table index into
// bits 8.. of an LDS address with one instruction
template <typename F>
__device__ __forceinline__ void static_for_bytes(F&& f) {
    f(std::integral_constant<int, 0>{});
    f(std::integral_constant<int, 1>{});
    f(std::integral_constant<int, 2>{});
    f(std::integral_constant<int, 3>{});
}

template <int BYTE>
__device__ __forceinline__ void index_to_byte1(uint32_t& a, uint32_t src, uint32_t mask) {
    static_assert(BYTE >= 0 && BYTE < 4, "byte select");
    if constexpr (BYTE == 0)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:DWORD" : "+v"(a) : "v"(src), "v"(mask));
    else if constexpr (BYTE == 1)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:DWORD" : "+v"(a) : "v"(src), "v"(mask));
    else if constexpr (BYTE == 2)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:DWORD" : "+v"(a) : "v"(src), "v"(mask));
    else
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:DWORD" : "+v"(a) : "v"(src), "v"(mask));
}

//
// PT (4-bit block-scaled only) selects the table of centroid PAIRS described at the table layout below.
template <int BITS, int NWK, int RBW, int SPW, bool SC, bool PT = false>
__global__ __launch_bounds__(NWK * 64) void gemm_mfma_kernel(
    const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
    const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int64_t N, int64_t K, int M,
    const uint16_t* __restrict__ scales) {
    using T = Tiled<BITS>;
    constexpr int GPG = T::GPG, GW = T::GW, SBE = T::SBE, C = 1 << BITS;
    constexpr int THREADS = NWK * 64;

    // 4-bit: the centroid tables are laid out [entry][lane]: lane l keeps its row's 16 centroids (as
    // bf16 in both halves of a dword) in column l, i.e. in LDS bank l, so a wave's 64 lookups never
    // collide whatever the indices are, and the address is (entry << 8) | (lane << 2): the index
    // goes into byte 1 of a register that holds lane * 4.
    // With the tensor-wide codebook of the block-scaled format one table serves every row, and it can be
    // a table of PAIRS (PT: 256 entries, 64 KB with a column per lane): a byte of the index stream is then
    // the address of two weights, already packed as the matrix instruction wants them -- half the
    // lookups and a third of the vector instructions, for a 64 KB fill per workgroup and one workgroup
    // per CU: it pays on long rows (8192 x 8192, batch 16: 16.1 -> 13.5 us) and costs on short ones
    // (4096 x 4096: 6.7 -> 7.5 us), so the launcher decides.
    static_assert(!PT || (BITS == 4 && SC), "pair table: 4-bit, tensor-wide codebook");
    constexpr int PT_RB = BITS == 4 ? (SC ? 1 : RBW) : 1, PT_ENT = BITS == 4 ? (PT ? 256 : 16) : 1;
    struct alignas(256) Smem {
        uint32_t ptab[PT_RB][PT_ENT][64];
        u32x2_t masks[16];                                  // 1-bit: nibble -> four bf16 {0,1}
        // per wave: 16 batch rows x (16 + 1 pad) 16-byte pieces of activations; when the wave is
        // done with them the same memory holds its RBW partial 16x16 tiles ([m][n padded to 17] floats)
        u32x4_t xstage[NWK][16 * 17];
        float redx[BITS == 1 ? NWK : 1][16];                // 1-bit: partial sum_k x per batch column
        uint32_t cpair[BITS == 1 ? RBW * 16 : 1];           // 1-bit: the rows' centroid pairs, fetched at the start for the epilogue
        // block-scaled: scales of the workgroup's rows, [row block][K block][row in block, padded to kSctRow]
        // (kept as bf16: an fp32 table saves four conversions per tile and block but doubles the
        // staging writes and the footprint, and measured slower)
        uint16_t sct[SC ? RBW * kMaxScaledBlocks * kSctRow : 1];
    };
    __shared__ Smem sm;

    // the wave index is uniform: telling the compiler so moves the address arithmetic to the scalar unit
    const int wk = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int n = lane & 15, q = lane >> 4;
    const int64_t rb0 = static_cast<int64_t>(blockIdx.x) * RBW;
    const int64_t nrb = (N + 15) >> 4;
    const int nsb = static_cast<int>(K / SBE);
    constexpr int kOuterUnroll = SPW > 0 ? (SPW + kPrefetch - 1) / kPrefetch : 1;
    const int spw = SPW > 0 ? SPW : nsb / NWK;              // super-blocks per wave (host guarantees divisibility)
    const int sb0 = wk * spw;

    // ---- tables ---------------------------------------------------------------------------
    if constexpr (BITS == 1) {
        if (threadIdx.x < 16) {
            const uint32_t e = threadIdx.x;
            u32x2_t m;
            m[0] = ((e & 1u) ? 0x3F80u : 0u) | ((e & 2u) ? 0x3F800000u : 0u);
            m[1] = ((e & 4u) ? 0x3F80u : 0u) | ((e & 8u) ? 0x3F800000u : 0u);
            sm.masks[e] = m;
        }
        if constexpr (!SC) {
            // a load issued in the epilogue would put a whole memory latency behind the last reduction
            if (threadIdx.x < RBW * 16) {
                int64_t row = rb0 * 16 + threadIdx.x;
                row = row < N ? row : N - 1;
                sm.cpair[threadIdx.x] = *reinterpret_cast<const uint32_t*>(codebook + row * 2);
            }
        }
    } else if constexpr (PT) {
        const uint32_t cv = codebook[lane & 15];             // lane l holds centroid l mod 16; entries are wave-uniform
        for (int e = wk; e < 256; e += NWK)
            sm.ptab[0][e][lane] = static_cast<uint32_t>(__builtin_amdgcn_readlane(cv, e & 15)) |
                                  (static_cast<uint32_t>(__builtin_amdgcn_readlane(cv, e >> 4)) << 16);
    } else if constexpr (BITS == 4) {
#pragma unroll
        for (int r = 0; r < PT_RB; ++r) {
            int64_t row = (rb0 + r) * 16 + n;
            row = row < N ? row : N - 1;
            if constexpr (SC) row = 0;
            const uint32_t* cw = reinterpret_cast<const uint32_t*>(codebook + row * C);
            for (int e2 = wk; e2 < C / 2; e2 += NWK) {       // the waves share the entries; every lane fills its own column
                const uint32_t dw = cw[e2];
                sm.ptab[r][2 * e2][lane] = __builtin_amdgcn_perm(dw, dw, 0x01000100u);
                sm.ptab[r][2 * e2 + 1][lane] = __builtin_amdgcn_perm(dw, dw, 0x03020302u);
            }
        }
    }

    if constexpr (SC) {
        const int nblk = static_cast<int>(K / KMQ_BLOCK);
        if ((nblk & 7) == 0 && (reinterpret_cast<uintptr_t>(scales) & 15) == 0) {
            // eight scales (16 bytes) of one row per load: an eighth of the load instructions
            const int nb8 = nblk >> 3;
            for (int e = threadIdx.x; e < RBW * 16 * nb8; e += THREADS) {
                // 16 consecutive lanes: the 16 rows of a row block; the next 16 lanes: the next eight blocks
                const int r16 = e & 15, b8 = (e >> 4) % nb8, rb = (e >> 4) / nb8;
                int64_t row = (rb0 + rb) * 16 + r16;
                row = row < N ? row : N - 1;
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(scales + row * nblk + b8 * 8);
                uint16_t* dst = &sm.sct[(rb * nblk + b8 * 8) * kSctRow + r16];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    dst[(2 * i) * kSctRow] = static_cast<uint16_t>(v[i]);
                    dst[(2 * i + 1) * kSctRow] = static_cast<uint16_t>(v[i] >> 16);
                }
            }
        } else {
            for (int e = threadIdx.x; e < RBW * 16 * nblk; e += THREADS) {
                const int rl = e / nblk, blk = e % nblk;        // consecutive threads: consecutive blocks of a row
                int64_t row = rb0 * 16 + rl;
                row = row < N ? row : N - 1;
                sm.sct[((rl >> 4) * nblk + blk) * kSctRow + (rl & 15)] = scales[row * nblk + blk];
            }
        }
    }

    // Activations of a chunk (16 batch rows x 128 columns) go through a wave-private LDS
    // tile: global loads take 256 contiguous bytes per row (rows of X are K*2 bytes apart,
    // so gathering 16 rows x 64 bytes per instruction thrashes one memory channel), and
    // lane (m = n, q) then reads the 16 bytes of columns 8*(q + 4i)..+7 for step i.
    // Batch columns >= M are fed row M-1 and dropped at the end.
    const char* xbase = reinterpret_cast<const char*>(X + static_cast<int64_t>(sb0) * SBE);   // uniform
    uint32_t xoff[4];                                       // per-lane byte offsets (M*K*2 < 2^30)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = 4 * i + q;
        m = m < M ? m : M - 1;
        xoff[i] = (static_cast<uint32_t>(m) * static_cast<uint32_t>(K) + 8u * n) * 2u;
    }
    u32x4_t* xtile = &sm.xstage[wk][0];
    // partial tiles: [row block][batch column][row, padded to 17] floats -- the threads that sum them read 16
    // consecutive rows of two batch columns at once; unpadded (and row-major) that was a 16-way bank conflict
    static_assert(RBW * 16 * 17 * sizeof(float) <= 16 * 17 * sizeof(u32x4_t), "partial tiles reuse the activation tile");

    f32x4_t acc[RBW];
#pragma unroll
    for (int r = 0; r < RBW; ++r) acc[r] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    [[maybe_unused]] f32x4_t accx = f32x4_t{0.f, 0.f, 0.f, 0.f};
    [[maybe_unused]] f32x4_t accxs[RBW];                    // 1-bit block-scaled: sum over blocks of scale * (block sum of x)
    if constexpr (SC && BITS == 1) {
#pragma unroll
        for (int r = 0; r < RBW; ++r) accxs[r] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    [[maybe_unused]] uint32_t areg[8];                      // 4-bit: lookup addresses, byte 0 = lane * 4, byte 1 = index
#pragma unroll
    for (int e = 0; e < 8; ++e) areg[e] = static_cast<uint32_t>(lane) * 4u;
    [[maybe_unused]] uint32_t lo0[RBW], lo1[RBW], hi0[RBW], hi1[RBW];   // perm pools: low / high bytes of the lane's centroids
    if constexpr (BITS == 2 || BITS == 3) {
#pragma unroll
        for (int r = 0; r < RBW; ++r) {
            int64_t row = (rb0 + r) * 16 + n;
            row = row < N ? row : N - 1;
            if constexpr (SC) row = 0;
            const uint32_t* cw = reinterpret_cast<const uint32_t*>(codebook + row * C);
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
    }

    [[maybe_unused]] float c0s = 0.f, cdiff = 0.f;          // 1-bit block-scaled: c0 and c1 - c0 of the tensor-wide pair
    if constexpr (SC && BITS == 1) {
        const uint32_t cc2 = *reinterpret_cast<const uint32_t*>(codebook);
        c0s = bf16_to_f32(cc2 & 0xFFFFu);
        cdiff = bf16_to_f32(cc2 >> 16) - c0s;
    }

    // Activations are fetched kXAhead chunks (of 4 steps) ahead of the chunk being multiplied.
    constexpr int CPG = GPG / 4;                            // chunks per super-block
#ifndef KMQ_XAHEAD
#define KMQ_XAHEAD 2
#endif
    constexpr int kXAhead = KMQ_XAHEAD;                      // divides kPrefetch * CPG, so ring slots are static
    const int nchunks = spw * CPG;
    u32x4_t xg[kXAhead][4];
#pragma unroll
    for (int c = 0; c < kXAhead; ++c) {
        const int cn = c < nchunks ? c : nchunks - 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) xg[c][i] = *reinterpret_cast<const u32x4_t*>(xbase + (xoff[i] + static_cast<uint32_t>(cn) * 256u));
    }

    // Issue order matters: vmcnt retires loads in order, and the memory system serves the
    // whole grid's requests roughly first come first served.  Small operands (codebook rows,
    // first activation chunks) were requested above; granules follow in the order they are
    // consumed, so a wave can start on super-block 0 when a quarter of its data is there.
    const int64_t gstride = 64 * GW;                        // dwords per (row block, super-block) tile
    const uint32_t* wbase[RBW];
#pragma unroll
    for (int r = 0; r < RBW; ++r) {
        int64_t rb = rb0 + r;
        rb = rb < nrb ? rb : nrb - 1;
        wbase[r] = W + (rb * nsb + sb0) * gstride;           // uniform; the lane adds lane * GW dwords
    }
    uint32_t gran[kPrefetch][RBW][GW];
#pragma unroll
    for (int p = 0; p < kPrefetch; ++p) {
        const int s = p < spw ? p : spw - 1;
#pragma unroll
        for (int r = 0; r < RBW; ++r) load_granule<GW>(wbase[r] + s * gstride + lane * GW, gran[p][r]);
    }

    __syncthreads();                                        // tables visible; every load above is in flight

#pragma unroll kOuterUnroll
    for (int s0 = 0; s0 < spw; s0 += kPrefetch) {
#pragma unroll
        for (int p = 0; p < kPrefetch; ++p) {
            const int s = s0 + p;
            if (s < spw) {
#pragma unroll
                for (int cc = 0; cc < CPG; ++cc) {
                    // this chunk: registers -> LDS tile -> B fragments; chunk + kXAhead: global -> registers
                    const int slot = (p * CPG + cc) % kXAhead;
#pragma unroll
                    for (int i = 0; i < 4; ++i) xtile[(4 * i + q) * 17 + n] = xg[slot][i];
                    if (const int cn = s * CPG + cc + kXAhead; cn < nchunks) {   // wave-uniform
#pragma unroll
                        for (int i = 0; i < 4; ++i) xg[slot][i] = *reinterpret_cast<const u32x4_t*>(xbase + (xoff[i] + static_cast<uint32_t>(cn) * 256u));
                    }
                    u32x4_t xf[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) xf[i] = xtile[n * 17 + q + 4 * i];
                    auto decode = [&](int r, int j) -> u32x4_t {
                        u32x4_t a;
                        if constexpr (BITS == 1) {
                            const uint32_t gb = group_bits<BITS, GW>(gran[p][r], j);
                            const u32x2_t lo = sm.masks[gb & 15u], hi = sm.masks[gb >> 4];
                            a = u32x4_t{lo[0], lo[1], hi[0], hi[1]};
                        } else if constexpr (BITS == 4) {
                            const uint32_t gb = group_bits<BITS, GW>(gran[p][r], j);
                            const uint32_t toff = static_cast<uint32_t>(reinterpret_cast<size_t>((lds_cu32_t*)(&sm.ptab[SC ? 0 : r][0][0])));
                            if constexpr (PT) {                // a byte = two indices = one entry of the pair table
                                static_for_bytes([&](auto bc) {
                                    constexpr int b = decltype(bc)::value;
                                    index_to_byte1<b>(areg[b], gb, 0xFFu);
                                    a[b] = *reinterpret_cast<lds_cu32_t*>(static_cast<size_t>(areg[b] + toff));
                                });
                                return a;
                            }
                            // even nibbles sit in the low four bits of the bytes of gb, odd ones of gb >> 4
                            const uint32_t go = gb >> 4;
                            uint32_t wv[8];
                            static_for_bytes([&](auto bc) {
                                constexpr int b = decltype(bc)::value;
                                index_to_byte1<b>(areg[2 * b], gb, 0x0Fu);
                                wv[2 * b] = *reinterpret_cast<lds_cu32_t*>(static_cast<size_t>(areg[2 * b] + toff));
                                index_to_byte1<b>(areg[2 * b + 1], go, 0x0Fu);
                                wv[2 * b + 1] = *reinterpret_cast<lds_cu32_t*>(static_cast<size_t>(areg[2 * b + 1] + toff));
                            });
                            a = u32x4_t{__builtin_amdgcn_perm(wv[1], wv[0], 0x07060100u), __builtin_amdgcn_perm(wv[3], wv[2], 0x07060100u),
                                        __builtin_amdgcn_perm(wv[5], wv[4], 0x07060100u), __builtin_amdgcn_perm(wv[7], wv[6], 0x07060100u)};
                        } else {
#pragma unroll
                            for (int h = 0; h < 2; ++h) {      // elements 4h..4h+3 of this step
                                uint32_t sel;
                                if constexpr (BITS == 2) {
                                    const int c = 2 * j + h;
                                    sel = (gran[p][r][c >> 2] >> (2 * (c & 3))) & 0x03030303u;
                                } else {
                                    const uint32_t* D = gran[p][r];
                                    if (j < 3) sel = (h == 0 ? D[j] : D[j] >> 3) & 0x07070707u;
                                    else if (h == 0) sel = ((D[0] >> 6) & 0x03030303u) | ((D[1] >> 4) & 0x04040404u);
                                    else sel = ((D[1] >> 7) & 0x01010101u) | ((D[2] >> 5) & 0x06060606u);
                                }
                                const uint32_t lo = __builtin_amdgcn_perm(lo1[r], lo0[r], sel);
                                const uint32_t hi = __builtin_amdgcn_perm(hi1[r], hi0[r], sel);
                                a[2 * h] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
                                a[2 * h + 1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
                            }
                        }
                        return a;
                    };
                    const u32x4_t ones = u32x4_t{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
                    if constexpr (!SC) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int j = cc * 4 + i;
                            const bf16x8_t b = __builtin_bit_cast(bf16x8_t, xf[i]);
#pragma unroll
                            for (int r = 0; r < RBW; ++r)
                                acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, decode(r, j)), b, acc[r], 0, 0, 0);
                            if constexpr (BITS == 1)
                                accx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ones), b, accx, 0, 0, 0);
                        }
                    } else {
#pragma unroll
                        for (int g2 = 0; g2 < 2; ++g2) {           // the chunk's two 64-column blocks
                            const bf16x8_t b0 = __builtin_bit_cast(bf16x8_t, xf[2 * g2]), b1 = __builtin_bit_cast(bf16x8_t, xf[2 * g2 + 1]);
                            const int j0 = cc * 4 + 2 * g2;
                            const int blk = (sb0 + s) * (SBE / KMQ_BLOCK) + cc * 2 + g2;      // wave-uniform
                            const f32x4_t zero = f32x4_t{0.f, 0.f, 0.f, 0.f};
                            [[maybe_unused]] f32x4_t tx = zero;
                            if constexpr (BITS == 1) {
                                tx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ones), b0, zero, 0, 0, 0);
                                tx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ones), b1, tx, 0, 0, 0);
                            }
#pragma unroll
                            for (int r = 0; r < RBW; ++r) {
                                f32x4_t t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, decode(r, j0)), b0, zero, 0, 0, 0);
                                t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, decode(r, j0 + 1)), b1, t, 0, 0, 0);
                                // scales of output rows 4q..4q+3 of this row block, one 8-byte read
                                const u32x2_t s4 = *reinterpret_cast<const u32x2_t*>(&sm.sct[((r * static_cast<int>(K / KMQ_BLOCK)) + blk) * kSctRow + 4 * q]);
                                const float sc[4] = {bf16_to_f32(s4[0] & 0xFFFFu), bf16_to_f32(s4[0] >> 16),
                                                     bf16_to_f32(s4[1] & 0xFFFFu), bf16_to_f32(s4[1] >> 16)};
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    acc[r][i] = fmaf(sc[i], t[i], acc[r][i]);
                                    // 1-bit: the scaled block sums of x are kept apart and combined with
                                    // the two centroids once, after the loop
                                    if constexpr (BITS == 1) accxs[r][i] = fmaf(sc[i], tx[i], accxs[r][i]);
                                }
                            }
                        }
                    }
                }
                // refill this slot with the granule kPrefetch super-blocks ahead
                if (const int sn = s + kPrefetch; sn < spw) {
#pragma unroll
                    for (int r = 0; r < RBW; ++r) load_granule<GW>(wbase[r] + sn * gstride + lane * GW, gran[p][r]);
                }
            }
        }
    }

    // ---- K-reduction across the waves, fixed order ---------------------------------------------
    // lane holds D[row 4*q + i][batch column n], i = 0..3
    if constexpr (SC && BITS == 1) {
#pragma unroll
        for (int r = 0; r < RBW; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[r][i] = fmaf(cdiff, acc[r][i], c0s * accxs[r][i]);
    }
#pragma unroll
    for (int r = 0; r < RBW; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) reinterpret_cast<float*>(xtile)[(r * 16 + n) * 17 + 4 * q + i] = acc[r][i];
    if constexpr (BITS == 1 && !SC) {
        if (q == 0) sm.redx[wk][n] = accx[0];               // every row of the all-ones tile is sum_k x[m][k]
    }
    __syncthreads();

    for (int o = threadIdx.x; o < RBW * 256; o += THREADS) {
        const int m = o / (RBW * 16), nl = o % (RBW * 16);  // consecutive threads -> consecutive rows
        const int r = nl >> 4, nn = nl & 15;
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < NWK; ++k) s += reinterpret_cast<const float*>(&sm.xstage[k][0])[(r * 16 + m) * 17 + nn];
        const int64_t row = (rb0 + r) * 16 + nn;
        if (m < M && row < N) {
            if constexpr (BITS == 1 && !SC) {
                float sx = 0.f;
#pragma unroll
                for (int k = 0; k < NWK; ++k) sx += sm.redx[k][m];
                const uint32_t cc = sm.cpair[nl];
                const float c0 = bf16_to_f32(cc & 0xFFFFu), c1 = bf16_to_f32(cc >> 16);
                s = fmaf(c1 - c0, s, c0 * sx);
            }
            Y[static_cast<int64_t>(m) * N + row] = f32_to_bf16(s);
        }
    }
}

// ---- launch ------------------------------------------------------------------------------------

template <int BITS, int NWK, int RBW, int SPW>
static void launch_mfma_one(const GemmArgs& a, hipStream_t s) {
    const int64_t nrb = (a.N + 15) / 16;
    const dim3 grid(static_cast<unsigned>((nrb + RBW - 1) / RBW)), block(NWK * 64);
    if constexpr (BITS == 4) {
        // pair table: long rows (the 64 KB fill is amortised) and a grid of one round (one workgroup per CU)
        if (a.scales && a.K >= 8192 && grid.x <= 256) {
            hipLaunchKernelGGL((gemm_mfma_kernel<BITS, NWK, RBW, SPW, true, true>), grid, block, 0, s,
                               a.W, a.codebook, a.X, a.Y, a.N, a.K, a.M, a.scales);
            return;
        }
    }
    if (a.scales)
        hipLaunchKernelGGL((gemm_mfma_kernel<BITS, NWK, RBW, SPW, true>), grid, block, 0, s,
                           a.W, a.codebook, a.X, a.Y, a.N, a.K, a.M, a.scales);
    else
        hipLaunchKernelGGL((gemm_mfma_kernel<BITS, NWK, RBW, SPW, false>), grid, block, 0, s,
                           a.W, a.codebook, a.X, a.Y, a.N, a.K, a.M, a.scales);
}

// Launch shapes (waves along K, row blocks per wave, super-blocks per wave) with a
// compile-time K loop, and the (waves, row blocks) pairs that also exist with a runtime loop.
#define KMQ_MFMA_SHAPES(X) \
    X(8, 1, 1) X(8, 1, 2) X(8, 1, 4) X(4, 1, 3) X(4, 1, 4) X(2, 1, 3) \
    X(6, 1, 1) X(6, 1, 2) X(3, 1, 2) \
    X(4, 2, 2) X(4, 2, 4) X(4, 2, 8) X(6, 2, 1) X(8, 2, 2) X(8, 2, 4) X(8, 2, 8) X(8, 1, 8) \
    X(6, 3, 1) X(8, 3, 2)
#define KMQ_MFMA_RT_SHAPES(X) \
    X(8, 1) X(4, 1) X(2, 1) X(1, 1) X(8, 2) X(4, 2) X(2, 2) X(1, 2)

template <int BITS>
static void launch_mfma_bits(const GemmArgs& a, int nwk, int rbw, int spw, hipStream_t s) {
#define X(NWK_, RBW_, SPW_) \
    if (nwk == NWK_ && rbw == RBW_ && spw == SPW_) { launch_mfma_one<BITS, NWK_, RBW_, SPW_>(a, s); return; }
    KMQ_MFMA_SHAPES(X)
#undef X
#define X(NWK_, RBW_) \
    if (nwk == NWK_ && rbw == RBW_) { launch_mfma_one<BITS, NWK_, RBW_, 0>(a, s); return; }
    KMQ_MFMA_RT_SHAPES(X)
#undef X
    launch_mfma_one<BITS, 1, 1, 0>(a, s);                  // any K the layout allows, one wave per row block
}

static bool mfma_has_shape(int nwk, int rbw, int spw) {
#define X(NWK_, RBW_, SPW_) if (nwk == NWK_ && rbw == RBW_ && spw == SPW_) return true;
    KMQ_MFMA_SHAPES(X)
#undef X
#define X(NWK_, RBW_) if (nwk == NWK_ && rbw == RBW_) return true;
    KMQ_MFMA_RT_SHAPES(X)
#undef X
    return false;
}

// Tuning override for sweeps, in builds with -DKMQ_TUNING only: KMQ_MFMA_NWK / KMQ_MFMA_RBW in the
// environment (read once).  An ordinary build never looks at the environment.
static int env_int(const char* name) {
#ifdef KMQ_TUNING
    const char* v = std::getenv(name);
    return v ? std::atoi(v) : 0;
#else
    (void)name;
    return 0;
#endif
}

// Waves along K for `rbw` row blocks per wave: the largest of 8, 6, 4, 3, 2, 1 that divides
// the number of super-blocks and has a kernel.  With two or more row blocks per wave and
// 2- or 3-bit decoding, more than 4 waves measured slower (registers); the 4-bit decode goes
// through LDS lookups and wants every wave it can get (8192 x 8192, M = 16: 25.6 us with 4
// waves, 20.8 with 8).
static int waves_along_k(int64_t K, int bits, int rbw) {
    static const int forced = env_int("KMQ_MFMA_NWK");
    const int nsb = static_cast<int>(K / tiled_superblock_elems(bits));
    const int cap = forced ? forced : (((bits == 2 || bits == 3) && rbw >= 2) ? 4 : 8);
    static const int kChoices[] = {8, 6, 4, 3, 2};
    for (int w : kChoices)
        if (nsb % w == 0 && w <= cap && mfma_has_shape(w, rbw, nsb / w)) return w;
    return 1;
}

// Row blocks per wave.  Every workgroup reads all of X through the L1, so fewer, fatter
// workgroups cut that traffic (it is 16x the index bytes at 1 bit with one row block), but
// the grid should still come out even over the 256 CUs: the cost model is (rounds of 256
// workgroups) x (row blocks per workgroup), ties go to the fatter workgroup.  Measured
// (us): 9216 x 3072, 1-bit, M = 16: 7.8 / 7.9 / 6.6 / 7.6 for 1 / 2 / 3 / 4 row blocks;
// 14336 x 4096, 3-bit, M = 16: 13.2 / 11.1 / - / 12.5.
int mfma_row_blocks(int64_t N, int64_t K, int bits) {
    static const int forced = env_int("KMQ_MFMA_RBW");
    const int64_t nrb = (N + 15) / 16;
    const int max_rbw = bits == 1 ? 3 : 2;
    int best = 1;
    int64_t best_cost = 0;
    for (int r = 1; r <= max_rbw; ++r) {
        if (forced && r != forced) continue;
        const int w = waves_along_k(K, bits, r);
        if (r > 1 && !mfma_has_shape(w, r, static_cast<int>(K / tiled_superblock_elems(bits) / w))) continue;
        const int64_t wgs = (nrb + r - 1) / r, cost = ((wgs + 255) / 256) * r;
        if (best_cost == 0 || cost <= best_cost) { best = r; best_cost = cost; }
    }
    return best;
}

int mfma_waves_along_k(int64_t N, int64_t K, int bits) { return waves_along_k(K, bits, mfma_row_blocks(N, K, bits)); }

hipError_t launch_mfma(const GemmArgs& a, hipStream_t s) {
    // short 2- and 3-bit rows: the kernel whose waves keep their slice of the activations in registers
    if (!a.scales && mfma_kslice_has_kernel(a.N, a.K, a.bits)) return launch_mfma_kslice(a, s);
    const int rbw = mfma_row_blocks(a.N, a.K, a.bits), nwk = waves_along_k(a.K, a.bits, rbw);
    const int spw = static_cast<int>(a.K / tiled_superblock_elems(a.bits) / nwk);
    switch (a.bits) {
        case 1: launch_mfma_bits<1>(a, nwk, rbw, spw, s); break;
        case 2: launch_mfma_bits<2>(a, nwk, rbw, spw, s); break;
        case 3: launch_mfma_bits<3>(a, nwk, rbw, spw, s); break;
        default: launch_mfma_bits<4>(a, nwk, rbw, spw, s); break;
    }
    return hipGetLastError();
}

}  // namespace kmq
