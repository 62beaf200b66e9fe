// Batch-1 kernels specialised on (bits, K), canonical layout: y = W x with
// w = codebook lookup (paper App. E, "Kernel implementations"; batch 1 is the
// memory-bound regime of App. D).
//
// Work split.  A row is cut into NWK slices along K, one per wave; inside a
// slice LPR lanes each own G consecutive words (EL = G*32/bits elements), so the
// index stream is read once with one contiguous vector load per lane and
// (row, slice).  With LPR < 64 a wave covers RPL = 64/LPR rows per load.  A
// workgroup is NWK x NWR waves and owns NWR*RPL*RS consecutive rows.  Every
// wave issues all of its index loads before it uses any of them.
//
// Operands on chip.  The activations a lane needs stay in VGPRs for all of its
// rows; the workgroup stages x through LDS once so that global reads of x are
// coalesced.  Weights come from 16-entry tables in LDS, which are conflict-free
// because the lanes of a row read one 64- or 128-byte table:
//   2-bit  per-row table: nibble (two indices) -> two bf16 weights, one
//          v_dot2c_f32_bf16 against a packed pair of activations per lookup;
//   4-bit  per-row table: index -> centroid as fp32, one FMA per lookup;
//   1-bit  one row-independent table: nibble -> four bf16 {0,1} masks (8 bytes);
//          the kernel accumulates S1 = sum_{idx=1} x and finishes with the
//          two-centroid closed form y = c0*sum(x) + (c1 - c0)*S1.
//
// Inner loop.  The table address of a lookup is 4*nibble (8*nibble for 1-bit)
// plus the table base.  Rotating the word by +-2 (+3/-1) bits puts the even/odd
// nibbles at bits 2..5 (3..6) of every byte, and one SDWA byte-select AND then
// produces the address byte; it writes only byte 0 of a register whose upper
// bytes hold the 256-byte-aligned table base, so there is no add.  Eight
// addresses and eight LDS reads are issued per word, about one word ahead of the
// multiply-accumulates that consume them (in two groups of four, so that no more
// than 12 LDS reads are ever outstanding).  These blocks are inline assembly
// with explicit s_waitcnt lgkmcnt(), because the compiler cannot see LDS reads
// issued from assembly and its own schedule exposed the LDS latency.
//
// K-reduction: DPP adds inside the LPR-lane group, then across the NWK slices
// through LDS; fp32 -> bf16 round-to-nearest-even; one coalesced store per
// workgroup.
#include <cstdlib>
#include <type_traits>

#include "kmq_device.h"
#include "kmq_launch.h"
#include "kmq_lut_blocks.h"

namespace kmq {

// ---- the kernel ----------------------------------------------------------------------

// SC selects the paper's own weight format (Sec. 2.2 "Nonlinear k-means quantization"):
// `codebook` is one table of 2^BITS centroids shared by all rows and `scales` holds one bf16
// per block of 64 elements of a row; a lane's slice is a whole number of blocks (or half of
// one), so its fp32 block sums are scaled once, before the reduction over lanes (the
// deferred-scaling variant of App. E "Kernel implementations").
//
// PAIR fuses two products that share x, as a decoder MLP's gate and up projections do, with the
// SwiGLU that consumes them: y[n] = silu(W[n] . x) * (W2[n] . x).  The kernel then walks 2N
// "virtual" rows, row 2n from (W, codebook) and row 2n + 1 from (W2, codebook2); N is passed as
// the virtual count, and the thread that would store a pair of outputs stores their combination.
// FUSE: decoder-layer fusions around the product (paper App. E "Model benchmarks": at one bit
// the elementwise work between the projections is a visible share of a token's time).
//   bit 0  RMSNorm in front: the activations entering the product are bf16(x * g), and the
//          result is multiplied by 1 / sqrt(mean(x^2) + eps), a scalar that commutes with the sum;
//   bit 1  residual behind: y = residual + product;
//   bit 2  RMSNorm with unit gains (gains folded into the weights before quantisation): only the
//          scalar, taken from the activations the workgroup stages anyway -- no second vector to
//          fetch per workgroup, which is what bit 0 costs.
template <int BITS, int G, int LPR, int NWK, int NWR, int RS, int WPE, bool SC, bool PAIR, int FUSE>
__global__ __launch_bounds__(NWK * NWR * 64) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemv_lut_kernel(const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
                     const uint16_t* __restrict__ x, uint16_t* y, int64_t N,
                     const uint16_t* __restrict__ scales,
                     const uint32_t* __restrict__ W2, const uint16_t* __restrict__ codebook2,
                     const uint16_t* __restrict__ norm_w, float eps, const uint16_t* residual, int mcols) {
    // (y and residual carry no __restrict__: the fused call documents that they may be the same buffer)
    static_assert(!(SC && PAIR), "the fused pair is offered for the per-row-codebook format");
    static_assert(FUSE == 0 || !SC, "decoder fusions are offered for the per-row-codebook format");
    static_assert(!(PAIR && (FUSE & 2)), "the fused pair has no residual input");
    static_assert((FUSE & 5) != 5, "gains or unit gains");
    constexpr bool NORM_G = (FUSE & 1) != 0, NORM = (FUSE & 5) != 0, RES = (FUSE & 2) != 0;
    static_assert(BITS >= 1 && BITS <= 4, "bit-width");
    static_assert(BITS != 3 || G % 3 == 0, "3-bit: lane slices are whole groups of three words");
    constexpr int C = 1 << BITS;
    constexpr int EL = G * 32 / BITS;              // elements per lane and row slice
    constexpr int K = NWK * LPR * EL;
    constexpr int WPR = K * BITS / 32;
    constexpr int RPL = kWave / LPR;               // rows per wave-wide load
    constexpr int ROWS_WAVE = RPL * RS;
    constexpr int ROWS_WG = NWR * ROWS_WAVE;
    constexpr int THREADS = NWK * NWR * 64;
    constexpr int U = BITS == 1 ? 2 * G : BITS == 3 ? 2 * G / 3 : G;   // lookup units (8 activation registers each) per row slice
    constexpr int XR = 8 * U;                      // activation registers: bf16 pairs (1/2/3-bit) or fp32 (4-bit)
    constexpr int C16 = EL * 2 / 16;               // 16-byte chunks of x per lane slice
    // Every wave builds the tables of its own rows (ENT lanes per row, LUT_PASSES passes of 64
    // lanes) in its own row groups; lanes past the last row write into padding: no branch.
    constexpr int ENT = BITS == 3 ? 64 : 16;       // table entries per row (3-bit: one per PAIR of fields)
    constexpr int LUT_PASSES = BITS == 1 ? 0 : (ROWS_WAVE * ENT + 63) / 64;
    constexpr int LUT_TABLES = BITS == 1 ? 1 : (LUT_PASSES * (64 / ENT) + RPL - 1) / RPL;   // tables per row group incl. padding
    constexpr int LUT_GROUPS = BITS == 1 ? 1 : NWK * NWR * RPL;
    constexpr int TBL = ((LUT_TABLES > RS ? LUT_TABLES : RS) * ENT + 63) / 64 * 64;   // dwords per row group: bases stay 256-byte aligned
    constexpr int XCHUNKS = K / 8;
    constexpr int XPT = (XCHUNKS + NWK * NWR * 64 - 1) / (NWK * NWR * 64);   // 16-byte chunks of x staged per thread
    constexpr int XSLOTS = XPT * NWK * NWR * 64;
    static_assert(RS <= 8 && (ROWS_WG % 2) == 0 && THREADS <= 1024, "launch shape");
    static_assert(EL % 8 == 0, "x slices are whole 16-byte chunks");
    constexpr int NSC = EL >= KMQ_BLOCK ? EL / KMQ_BLOCK : 1;      // scales per lane and row slice
    static_assert(!SC || EL % KMQ_BLOCK == 0 || KMQ_BLOCK % EL == 0, "lane slices must not straddle blocks");
    static_assert(!SC || NSC == 1 || (BITS == 1 && NSC == 2), "block sums kept by the pipeline");

    // Staged x is padded per lane slice so that a wave's 16-byte reads spread over the banks: a slice of C16
    // chunks takes XSTR chunks (an odd number), chunk q of slice sl sits at sl * XSTR + q -- one base
    // register per lane, the chunk number goes into the instruction's offset field.
    constexpr int XSTR = C16 | 1;

    struct alignas(256) Smem {
        // 2/3/4-bit: per wave and row group, RS tables of ENT x 4 B; 1-bit: lut[0] holds the 16 x 8 B mask table
        uint32_t lut[LUT_GROUPS][TBL];
        // staged activations, padded per lane slice; threads past the end of x (the
        // thread count need not divide the chunk count) write clamped data into the tail,
        // so that staging has no branch for the loads to be sunk into
        u32x4_t xs[(XSLOTS + C16 - 1) / C16 * XSTR];
        float part[NWK][ROWS_WG];                  // per-slice partial sums
        float sxp[NWK * NWR];                      // 1-bit: per-wave sum of the x the wave staged
        float ssq[NWK * NWR];                      // RMSNorm: per-wave sum of x^2 over the chunks the wave staged
    };
    __shared__ Smem sm;

    // the wave index is uniform: telling the compiler so moves address arithmetic to the scalar unit
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wk = wave % NWK, wr = wave / NWK;
    const int sub = lane / LPR, pos = lane % LPR;
    // mcols > 1: a batch of mcols activation rows in one launch, every workgroup still one column (x and y are
    // K and N elements apart per column).  Workgroup ids go round-robin over the 8 XCDs, each with its own L2;
    // the id is cut so that the mcols workgroups that read the same rows of W sit on one XCD, one after the
    // other: the first fetches those rows from memory, the others find them in that L2.
    // Row numbers are 32-bit (the library caps N at 2^24 rows, the fused pair at 2^25 virtual rows): clamps and
    // comparisons on 64-bit values cost two to three vector instructions each, ahead of the first load.
    const int Nr = static_cast<int>(N);
    int wg = blockIdx.x;
    if (mcols > 1) {
        const int t = wg >> 3;
        const int col = t % mcols;
        wg = (t / mcols) * 8 + (wg & 7);
        if (wg * ROWS_WG >= Nr) return;                      // the grid is padded to a multiple of 8 row groups
        x += static_cast<int64_t>(col) * K;
        y += static_cast<int64_t>(col) * (PAIR ? N / 2 : N);
    }
    const int wg_row0 = wg * ROWS_WG;
    const int wave_row0 = wg_row0 + wr * ROWS_WAVE;
    // start of a row's packed words / codebook (PAIR: even virtual rows first matrix, odd rows second)
    // PAIR: even virtual rows come from the first matrix, odd rows from the second.  The choice
    // is plain integer arithmetic on the addresses: a select between two pointer arguments can
    // end up as a two-entry table in scratch memory, and a kernel that uses scratch pays for
    // its set-up at every launch (measured: +15 us per call).
    const uintptr_t w_a = reinterpret_cast<uintptr_t>(W), w_d = PAIR ? reinterpret_cast<uintptr_t>(W2) - w_a : 0;
    const uintptr_t c_a = reinterpret_cast<uintptr_t>(codebook), c_d = PAIR ? reinterpret_cast<uintptr_t>(codebook2) - c_a : 0;
    auto wrow = [=](int row) -> const uint32_t* {
        if constexpr (PAIR)
            return reinterpret_cast<const uint32_t*>(w_a + (w_d & (uintptr_t(0) - uintptr_t(row & 1)))) + static_cast<int64_t>(row >> 1) * WPR;
        else
            return reinterpret_cast<const uint32_t*>(w_a) + static_cast<int64_t>(row) * WPR;
    };
    auto cbrow = [=](int row) -> const uint16_t* {
        if constexpr (PAIR)
            return reinterpret_cast<const uint16_t*>(c_a + (c_d & (uintptr_t(0) - uintptr_t(row & 1)))) + static_cast<int64_t>(row >> 1) * C;
        else
            return reinterpret_cast<const uint16_t*>(c_a) + static_cast<int64_t>(row) * C;
    };

    // ---- 1. small operands first: x chunks, then the codebook rows of this wave's own rows ----
    // Loads return in issue order.  x comes from the L2 and is there early; the codebook
    // rows are DRAM reads that queue behind other waves' index loads like the index loads
    // themselves, so they go second and nothing before the lookups waits for them.
    // Each thread stages XPT consecutive 16-byte chunks of x, fetched as ONE wide load: separate
    // loads get reordered behind the index loads by instruction selection.
    static_assert(XPT == 1 || XPT == 2 || XPT == 4, "x chunks per thread");
    typedef __attribute__((ext_vector_type(4 * XPT))) uint32_t xwide_t;
    static_assert(XCHUNKS % XPT == 0, "a thread's chunks are all inside x or all past its end");
    xwide_t xt;
    [[maybe_unused]] xwide_t gt;                   // RMSNorm weights of the same elements
    [[maybe_unused]] uint16_t resv[2];             // residual of the two rows this thread stores
    [[maybe_unused]] uint32_t ccv[2];              // 1-bit: centroid pair of the two rows this thread stores
    {
        int c = threadIdx.x * XPT;
        c = c < XCHUNKS ? c : XCHUNKS - XPT;
        xt = *reinterpret_cast<const xwide_t*>(x + c * 8);
        if constexpr (NORM_G) gt = *reinterpret_cast<const xwide_t*>(norm_w + c * 8);
        if constexpr (RES) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {          // fetched with the first loads: long there when the epilogue runs
                int rl = threadIdx.x * 2 + h;          // (only threads below ROWS_WG / 2 store)
                rl = rl < ROWS_WG ? rl : ROWS_WG - 1;
                int row = wg_row0 + rl;
                row = row < Nr ? row : Nr - 1;
                resv[h] = residual[row];
            }
        }
        if constexpr (BITS == 1 && !SC) {
            // the two centroids of the rows this thread stores: the epilogue's closed form needs them, and a
            // load issued there would put a whole memory latency behind the last reduction
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                int rl = threadIdx.x * 2 + h;          // (only threads below ROWS_WG / 2 store)
                rl = rl < ROWS_WG ? rl : ROWS_WG - 1;
                int row = wg_row0 + rl;
                row = row < Nr ? row : Nr - 1;
                ccv[h] = *reinterpret_cast<const uint32_t*>(cbrow(row));
            }
        }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    uint32_t cbv[LUT_PASSES > 0 ? LUT_PASSES : 1][BITS == 4 ? 1 : BITS == 3 ? 4 : 2];
#pragma unroll
    for (int p = 0; p < LUT_PASSES; ++p) {
        int rw = (lane + p * 64) / ENT;                                // row inside the wave: t * RPL + sub
        rw = rw < ROWS_WAVE ? rw : ROWS_WAVE - 1;
        int row = wave_row0 + rw;
        row = row < Nr ? row : Nr - 1;
        if constexpr (SC) row = 0;                                     // one table for the whole tensor
        if constexpr (BITS == 2) {
            // (codebooks are 4-byte aligned by contract: the vector types say so)
            typedef u32x2_t __attribute__((aligned(4))) u32x2_a4_t;
            const u32x2_t c = *reinterpret_cast<const u32x2_a4_t*>(cbrow(row));
            cbv[p][0] = c[0];
            cbv[p][1] = c[1];
        } else if constexpr (BITS == 3) {
            typedef u32x4_t __attribute__((aligned(4))) u32x4_a4_t;
            const u32x4_t c = *reinterpret_cast<const u32x4_a4_t*>(cbrow(row));
#pragma unroll
            for (int j = 0; j < 4; ++j) cbv[p][j] = c[j];
        } else {
            cbv[p][0] = cbrow(row)[lane & 15];
        }
    }

    // The small loads must be ahead of the index loads in the wave's (in-order) load queue:
    // staging x then waits for x only, with everything else still in flight.  Left to
    // itself the compiler sinks small loads below the index loads (or into a branch) and the
    // barrier ends up waiting for the whole index stream.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // ---- 2. every index load of this wave -------------------------------------------------
    uint32_t w[RS][G];
#pragma unroll
    for (int t = 0; t < RS; ++t) {
        int row = wave_row0 + t * RPL + sub;
        row = row < Nr ? row : Nr - 1;                                 // clamped: loads stay unconditional
        load_words<G>(wrow(row) + (wk * LPR + pos) * G, w[t]);
    }
    // block scales of this lane's slices: last in the queue, used after the lookups
    [[maybe_unused]] uint16_t sv[RS][NSC];
    if constexpr (SC) {
        const int blk0 = ((wk * LPR + pos) * EL) / KMQ_BLOCK;
#pragma unroll
        for (int t = 0; t < RS; ++t) {
            int row = wave_row0 + t * RPL + sub;
            row = row < Nr ? row : Nr - 1;
#pragma unroll
            for (int i = 0; i < NSC; ++i) sv[t][i] = __builtin_nontemporal_load(&scales[static_cast<int64_t>(row) * (K / KMQ_BLOCK) + blk0 + i]);
        }
    }
    // where this lane will read its slice of x from: computed now, while the loads are in flight,
    // and pinned here so that it is not scheduled behind the wait for x
    int xbase = (wk * LPR + pos) * XSTR;
    asm volatile("" : "+v"(xbase));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // ---- 3. staged activations into LDS ----------------------------------------------------------
    if constexpr (NORM) {
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < 4 * XPT; ++i) {
            ss = dot2_bf16(xt[i], xt[i], ss);
            if constexpr (NORM_G) {
                const float x0 = __uint_as_float(xt[i] << 16), x1 = __uint_as_float(xt[i] & 0xFFFF0000u);
                const float g0 = __uint_as_float(gt[i] << 16), g1 = __uint_as_float(gt[i] & 0xFFFF0000u);
                // a product of two bf16 values is exact in fp32: one rounding (to nearest even, the
                // hardware's packed conversion), to the bf16 activation
                typedef __attribute__((ext_vector_type(2))) float f32x2_t;
                const f32x2_t p = {x0 * g0, x1 * g1};
                xt[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2_t));
            }
        }
        ss = threadIdx.x * XPT < XCHUNKS ? ss : 0.f;       // threads past the end restaged a neighbour's chunks
        ss = group_sum<64>(ss);
        if (lane == 63) sm.ssq[wave] = ss;
    }
    if constexpr (BITS == 1 && !SC) {
        // sum of the activations for the two-centroid closed form, taken here from the chunks every thread stages anyway
        // (4 * XPT dots per thread) rather than from each wave's activation registers behind the lookups
        float sxl = 0.f;
#pragma unroll
        for (int i = 0; i < 4 * XPT; ++i) sxl = dot2_bf16(0x3F803F80u, xt[i], sxl);
        sxl = threadIdx.x * XPT < XCHUNKS ? sxl : 0.f;     // threads past the end restaged a neighbour's chunks
        sxl = group_sum<64>(sxl);
        if (lane == 63) sm.sxp[wave] = sxl;
    }
#pragma unroll
    for (int h = 0; h < XPT; ++h) {
        const int c = threadIdx.x * XPT + h;
        const int sl = c / C16, q = c % C16;
        sm.xs[sl * XSTR + q] = u32x4_t{xt[4 * h], xt[4 * h + 1], xt[4 * h + 2], xt[4 * h + 3]};
    }
    if constexpr (BITS == 1) {
        if (threadIdx.x < 16) {
            const uint32_t e = threadIdx.x;
            u32x2_t m;
            m[0] = ((e & 1u) ? 0x3F80u : 0u) | ((e & 2u) ? 0x3F800000u : 0u);
            m[1] = ((e & 4u) ? 0x3F80u : 0u) | ((e & 8u) ? 0x3F800000u : 0u);
            reinterpret_cast<u32x2_t*>(&sm.lut[0][0])[e] = m;
        }
    }
    __syncthreads();

    // ---- 4. this lane's activations into registers ---------------------------------------------
    uint32_t xr[XR];
    {
#pragma unroll
        for (int q = 0; q < C16; ++q) {
            const u32x4_t v = sm.xs[xbase + q];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (BITS == 4) {
                    xr[q * 8 + 2 * j] = v[j] << 16;
                    xr[q * 8 + 2 * j + 1] = v[j] & 0xFFFF0000u;
                } else {
                    xr[q * 4 + j] = v[j];
                }
            }
        }
    }

    // 1-bit block-scaled: the sums of x over this lane's two blocks, taken now, while the index words are still in
    // flight, rather than behind the lookups
    [[maybe_unused]] float sx0 = 0.f, sx1 = 0.f;
    if constexpr (SC && BITS == 1) {
#pragma unroll
        for (int i = 0; i < XR / 2; ++i) {
            sx0 = dot2_bf16(0x3F803F80u, xr[i], sx0);
            sx1 = dot2_bf16(0x3F803F80u, xr[XR / 2 + i], sx1);
        }
    }

    // ---- 4b. this wave's tables, once its codebook rows have arrived --------------------------------
    // (the wave reads back only what it wrote itself: LDS serves a wave's instructions in order)
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (BITS != 1) {
#pragma unroll
        for (int p = 0; p < LUT_PASSES; ++p) {
            const int rw = (lane + p * 64) / ENT, e = lane % ENT;
            const int t2 = rw / RPL, sub2 = rw % RPL;
            uint32_t entry;
            if constexpr (BITS == 2) {
                const uint64_t c64 = static_cast<uint64_t>(cbv[p][0]) | (static_cast<uint64_t>(cbv[p][1]) << 32);
                entry = (static_cast<uint32_t>(c64 >> (16 * (e & 3))) & 0xFFFFu) |
                        ((static_cast<uint32_t>(c64 >> (16 * (e >> 2))) & 0xFFFFu) << 16);
            } else if constexpr (BITS == 3) {
                // entry e: centroid e mod 8 for the even element, centroid e div 8 for the odd one
                auto pick = [&](int i) -> uint32_t {
                    const uint32_t lo2 = (i & 2) ? cbv[p][1] : cbv[p][0], hi2 = (i & 2) ? cbv[p][3] : cbv[p][2];
                    const uint32_t d = (i & 4) ? hi2 : lo2;
                    return (i & 1) ? d >> 16 : d & 0xFFFFu;
                };
                entry = pick(e & 7) | (pick(e >> 3) << 16);
            } else {
                entry = cbv[p][0] << 16;
            }
            sm.lut[wave * RPL + sub2][t2 * ENT + e] = entry;
        }
    }

    // ---- 5. lookups and multiply-accumulate, one unit ahead -------------------------------------
    const uint32_t lut_base = static_cast<uint32_t>(reinterpret_cast<size_t>(
        (lds_cu32_t*)(&sm.lut[BITS == 1 ? 0 : wave * RPL + sub][0])));
    // Four address registers serve both halves of a unit: a DS instruction has read its
    // address when it issues, so the next half may overwrite the low byte right behind it.
    uint32_t ar[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ar[i] = lut_base;
    // Everything the compiler itself has in flight on the LGKM counter (the reads of
    // x above) must have landed before the hand-counted pipeline starts.
    // That includes scalar loads: the two centroids of the 1-bit block-scaled form are fetched
    // here, ahead of the pipeline, because a scalar load issued in its middle would count on
    // the same LGKM counter as the lookups and return out of order with them.
    [[maybe_unused]] uint32_t cpair = 0;
    if constexpr (SC && BITS == 1) cpair = *reinterpret_cast<const uint32_t*>(codebook);
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(cpair) : : "memory");
    const uint32_t mask = BITS == 1 ? 0x78u : BITS == 3 ? 0xFCu : 0x3Cu;
    float acc[RS];
    [[maybe_unused]] float accb[RS];               // 1-bit with scales: the first block's sum
    float a0 = 0.f, a1 = 0.f;
    constexpr int NU = RS * U;
    if constexpr (BITS == 1) {
        u32x2_t vv[2][4];
        uint32_t re = 0, ro = 0;
        issue4_b64<0>(w[0][0], re, ro, ar, vv[0], mask);
        static_for<0, NU>([&](auto ic) {
            constexpr int n = decltype(ic)::value;
            constexpr int t = n / U, u = n % U;
            if constexpr (n + 1 < NU) {
                constexpr int t1 = (n + 1) / U, u1 = (n + 1) % U;
                issue4_b64<u1 % 2>(w[t1][u1 / 2], re, ro, ar, vv[(n + 1) & 1], mask);
                consume4_b64<4>(vv[n & 1], &xr[u * 8], a0, a1);
            } else {
                consume4_b64<0>(vv[n & 1], &xr[u * 8], a0, a1);
            }
            if constexpr (SC && u == U / 2 - 1) { settle_dot(a0, a1); accb[t] = a0 + a1; a0 = 0.f; a1 = 0.f; }
            if constexpr (u == U - 1) { settle_dot(a0, a1); acc[t] = a0 + a1; a0 = 0.f; a1 = 0.f; }
        });
    } else {
        uint32_t v[2][8];
        uint32_t re = 0, ro = 0;
        // half H (0, 1) of unit uu of row slice tt into vd[4H..4H+3]
        auto issue_half = [&](auto tc, auto uc, auto hc, uint32_t (&vd)[8]) {
            constexpr int tt = decltype(tc)::value, uu = decltype(uc)::value, hh = decltype(hc)::value;
            if constexpr (BITS == 3) {
                constexpr int g3 = 3 * (uu / 2);
                issue4_p6<tt * ENT * 4, 2 * (uu % 2) + hh>(w[tt][g3], w[tt][g3 + 1], w[tt][g3 + 2], ar, &vd[4 * hh], mask);
            } else {
                issue4_b32<tt * ENT * 4, hh>(w[tt][uu], re, ro, ar, vd, mask);
            }
        };
        using std::integral_constant;
        issue_half(integral_constant<int, 0>{}, integral_constant<int, 0>{}, integral_constant<int, 0>{}, v[0]);
        issue_half(integral_constant<int, 0>{}, integral_constant<int, 0>{}, integral_constant<int, 1>{}, v[0]);
        static_for<0, NU>([&](auto ic) {
            constexpr int n = decltype(ic)::value;
            constexpr int t = n / U, u = n % U;
            if constexpr (n + 1 < NU) {
                constexpr int t1 = (n + 1) / U, u1 = (n + 1) % U;
                issue_half(integral_constant<int, t1>{}, integral_constant<int, u1>{}, integral_constant<int, 0>{}, v[(n + 1) & 1]);
                if constexpr (BITS != 4) consume8_dot2<4>(v[n & 1], &xr[u * 8], a0, a1);
                else consume8_fma<4>(v[n & 1], &xr[u * 8], a0, a1);
                issue_half(integral_constant<int, t1>{}, integral_constant<int, u1>{}, integral_constant<int, 1>{}, v[(n + 1) & 1]);
            } else {
                if constexpr (BITS != 4) consume8_dot2<0>(v[n & 1], &xr[u * 8], a0, a1);
                else consume8_fma<0>(v[n & 1], &xr[u * 8], a0, a1);
            }
            if constexpr (u == U - 1) { settle_dot(a0, a1); acc[t] = a0 + a1; a0 = 0.f; a1 = 0.f; }
        });
    }

    // ---- 6. K-reduction: lanes of the group, then slices through LDS ------------------------------
    // (nothing of what follows may be scheduled into the hand-counted pipeline above)
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (SC) {
        if constexpr (BITS == 1) {
            // two blocks per lane: s0*(c0*X0 + d*S0) + s1*(c0*X1 + d*S1), X = the block's sum of x
            const float c0 = bf16_to_f32(cpair & 0xFFFFu), d = bf16_to_f32(cpair >> 16) - c0;
#pragma unroll
            for (int t = 0; t < RS; ++t)
                acc[t] = bf16_to_f32(sv[t][0]) * fmaf(d, accb[t], c0 * sx0) + bf16_to_f32(sv[t][1]) * fmaf(d, acc[t], c0 * sx1);
        } else {
#pragma unroll
            for (int t = 0; t < RS; ++t) acc[t] *= bf16_to_f32(sv[t][0]);
        }
    }
#pragma unroll
    for (int t = 0; t < RS; ++t) {
        const float s = group_sum<LPR>(acc[t]);
        if (pos == LPR - 1) sm.part[wk][wr * ROWS_WAVE + t * RPL + sub] = s;
    }
    __syncthreads();

    // ---- 7. epilogue: two rows per thread, one coalesced store per workgroup ----------------------
    if (threadIdx.x < ROWS_WG / 2) {
        float out[2];
        [[maybe_unused]] float rnorm = 1.f;
        if constexpr (NORM) {
            float ss = 0.f;
#pragma unroll
            for (int i = 0; i < NWK * NWR; ++i) ss += sm.ssq[i];
            rnorm = 1.f / sqrtf(ss * (1.f / K) + eps);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int rl = threadIdx.x * 2 + h;
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < NWK; ++k) s += sm.part[k][rl];
            if constexpr (BITS == 1 && !SC) {
                float sx = 0.f;
#pragma unroll
                for (int k = 0; k < NWK * NWR; ++k) sx += sm.sxp[k];
                const uint32_t cc = ccv[h];
                const float c0 = bf16_to_f32(cc & 0xFFFFu), c1 = bf16_to_f32(cc >> 16);
                s = fmaf(c1 - c0, s, c0 * sx);
            }
            if constexpr (NORM) s *= rnorm;
            if constexpr (RES) s += bf16_to_f32(resv[h]);
            out[h] = s;
        }
        const int r2 = wg_row0 + threadIdx.x * 2;
        if constexpr (PAIR) {
            // out[0] = gate, out[1] = up of output element r2 / 2: silu(gate) * up in fp32
            if (r2 < Nr) y[r2 >> 1] = f32_to_bf16(out[0] / (1.f + __expf(-out[0])) * out[1]);
            return;
        }
        const uint32_t packed = static_cast<uint32_t>(f32_to_bf16(out[0])) | (static_cast<uint32_t>(f32_to_bf16(out[1])) << 16);
        if (r2 + 1 < Nr && (reinterpret_cast<uintptr_t>(y) & 3u) == 0) {
            *reinterpret_cast<uint32_t*>(y + r2) = packed;
        } else {
            if (r2 < Nr) y[r2] = static_cast<uint16_t>(packed);
            if (r2 + 1 < Nr) y[r2 + 1] = static_cast<uint16_t>(packed >> 16);
        }
    }
}

// ---- specialisation table ------------------------------------------------------------------

struct LutEntry {
    int bits;
    int64_t K;
    int rows_wg;
    bool scaled;             // block scales + tensor-wide codebook
    const char* name;
    void (*launch)(const GemmArgs&, hipStream_t);
};

template <int BITS, int G, int LPR, int NWK, int NWR, int RS, int WPE, bool SC>
static void launch_lut(const GemmArgs& a, hipStream_t s) {
    constexpr int rows_wg = NWR * (kWave / LPR) * RS;
    const dim3 block(NWK * NWR * 64);
    if constexpr (!SC) {
        if (a.W2) {                                           // fused pair: 2N virtual rows
            const int64_t nv = 2 * a.N;
            const dim3 grid(static_cast<unsigned>((nv + rows_wg - 1) / rows_wg));
            if (a.norm && a.norm_w) {
                hipLaunchKernelGGL((gemv_lut_kernel<BITS, G, LPR, NWK, NWR, RS, WPE, false, true, 1>), grid, block, 0, s,
                                   a.W, a.codebook, a.X, a.Y, nv, a.scales, a.W2, a.codebook2, a.norm_w, a.eps, nullptr, 1);
                return;
            }
            if (a.norm) {
                hipLaunchKernelGGL((gemv_lut_kernel<BITS, G, LPR, NWK, NWR, RS, WPE, false, true, 4>), grid, block, 0, s,
                                   a.W, a.codebook, a.X, a.Y, nv, a.scales, a.W2, a.codebook2, nullptr, a.eps, nullptr, 1);
                return;
            }
            hipLaunchKernelGGL((gemv_lut_kernel<BITS, G, LPR, NWK, NWR, RS, WPE, false, true, 0>), grid, block, 0, s,
                               a.W, a.codebook, a.X, a.Y, nv, a.scales, a.W2, a.codebook2, nullptr, 0.f, nullptr, 1);
            return;
        }
    }
    const dim3 grid(static_cast<unsigned>((a.N + rows_wg - 1) / rows_wg));
    if constexpr (!SC) {                                      // decoder fusions (per-row-codebook format)
#define KMQ_LUT_FUSED(F) \
        hipLaunchKernelGGL((gemv_lut_kernel<BITS, G, LPR, NWK, NWR, RS, WPE, false, false, F>), grid, block, 0, s, \
                           a.W, a.codebook, a.X, a.Y, a.N, a.scales, nullptr, nullptr, a.norm_w, a.eps, a.residual, 1)
        const int fuse = (a.norm ? (a.norm_w ? 1 : 4) : 0) | (a.residual ? 2 : 0);
        switch (fuse) {
            case 1: KMQ_LUT_FUSED(1); return;
            case 2: KMQ_LUT_FUSED(2); return;
            case 3: KMQ_LUT_FUSED(3); return;
            case 4: KMQ_LUT_FUSED(4); return;
            case 6: KMQ_LUT_FUSED(6); return;
            default: break;
        }
#undef KMQ_LUT_FUSED
    }
    if (a.M > 1) {                                            // batch: one workgroup per (row group, column)
        const int64_t groups = (a.N + rows_wg - 1) / rows_wg;
        const dim3 grid_m(static_cast<unsigned>((groups + 7) / 8 * 8 * a.M));
        hipLaunchKernelGGL((gemv_lut_kernel<BITS, G, LPR, NWK, NWR, RS, WPE, SC, false, 0>), grid_m, block, 0, s,
                           a.W, a.codebook, a.X, a.Y, a.N, a.scales, nullptr, nullptr, nullptr, 0.f, nullptr, a.M);
        return;
    }
    hipLaunchKernelGGL((gemv_lut_kernel<BITS, G, LPR, NWK, NWR, RS, WPE, SC, false, 0>), grid, block, 0, s,
                       a.W, a.codebook, a.X, a.Y, a.N, a.scales, nullptr, nullptr, nullptr, 0.f, nullptr, 1);
}

#define KMQ_LUT(BITS, G, LPR, NWK, NWR, RS, WPE) \
    { BITS, int64_t(NWK) * LPR * (G * 32 / BITS), NWR * (64 / LPR) * RS, false, \
      "lut_b" #BITS "_g" #G "_l" #LPR "_k" #NWK "_r" #NWR "x" #RS, &launch_lut<BITS, G, LPR, NWK, NWR, RS, WPE, false> }
#define KMQ_LUT_SC(BITS, G, LPR, NWK, NWR, RS, WPE) \
    { BITS, int64_t(NWK) * LPR * (G * 32 / BITS), NWR * (64 / LPR) * RS, true, \
      "lut_sc_b" #BITS "_g" #G "_l" #LPR "_k" #NWK "_r" #NWR "x" #RS, &launch_lut<BITS, G, LPR, NWK, NWR, RS, WPE, true> }

static const LutEntry kLut[] = {
    // Several shapes may serve one (bits, K): lut_find takes the one whose grid comes out
    // most even over the CUs for the given N; the first listed wins ties.
    // 1-bit
    KMQ_LUT(1, 3, 16, 1, 4, 1, 4),   // K = 1536, 16 rows per workgroup
    KMQ_LUT(1, 4, 16, 1, 4, 1, 4),   // K = 2048, 16 rows per workgroup
    KMQ_LUT(1, 4, 16, 1, 2, 1, 4),   //            8
    KMQ_LUT(1, 3, 32, 1, 4, 2, 4),   // K = 3072, 16
    KMQ_LUT(1, 3, 32, 1, 3, 3, 4),   //           18
    KMQ_LUT(1, 3, 32, 1, 3, 2, 4),   //           12
    KMQ_LUT(1, 4, 32, 1, 4, 2, 4),   // K = 4096
    KMQ_LUT(1, 3, 64, 1, 6, 2, 4),   // K = 6144, 12
    KMQ_LUT(1, 4, 64, 1, 4, 2, 4),   // K = 8192,  8
    KMQ_LUT(1, 4, 64, 1, 4, 3, 4),   //           12
    // 2-bit
    KMQ_LUT(2, 3, 32, 1, 4, 2, 6),   // K = 1536
    KMQ_LUT(2, 4, 32, 1, 4, 2, 6),   // K = 2048
    KMQ_LUT(2, 3, 64, 1, 4, 2, 6),   // K = 3072
    KMQ_LUT(2, 4, 64, 1, 4, 2, 7),   // K = 4096
    KMQ_LUT(2, 3, 64, 2, 3, 2, 6),   // K = 6144: two slices of 12-byte loads, 6 rows per workgroup
    KMQ_LUT(2, 4, 64, 2, 2, 4, 4),   // K = 8192: 16 rows per workgroup (x, staged once per workgroup, is 16 KB here)
    KMQ_LUT(2, 4, 64, 2, 2, 2, 7),   //            8
    KMQ_LUT(2, 4, 32, 7, 1, 4, 4),   // K = 14336: 16-byte loads, 8 rows per workgroup (6.6 us on 4096 rows; 7.1 with 3 or 8 rows per wave)
    KMQ_LUT(2, 2, 64, 7, 1, 4, 7),   //            8-byte loads, 4 rows per workgroup (7.05 us; taken for few rows)
    // 3-bit (lane slices are whole groups of three words = 32 elements)
    KMQ_LUT(3, 3, 16, 3, 1, 2, 6),   // K = 1536: three slices of 12-byte loads, 8 rows per workgroup
    KMQ_LUT(3, 6, 32, 1, 4, 2, 6),   // K = 2048
    KMQ_LUT(3, 3, 32, 3, 1, 4, 6),   // K = 3072: three slices of 12-byte loads (9216 rows: 5.2 us; 6.1 with one slice of 36-byte loads)
    KMQ_LUT(3, 6, 64, 1, 4, 2, 7),   // K = 4096 (14336 rows: 7.7 us; 8.0 with 4 rows per wave)
    KMQ_LUT(3, 3, 64, 3, 2, 4, 6),   // K = 6144: three slices of 12-byte loads, 8 rows per workgroup
    KMQ_LUT(3, 6, 64, 2, 2, 4, 4),   // K = 8192: 16 rows per workgroup
    KMQ_LUT(3, 6, 64, 2, 2, 2, 6),   //            8
    KMQ_LUT(3, 3, 64, 7, 1, 4, 6),   // K = 14336: 12-byte loads, 4 rows per workgroup (4096 rows: 8.7 us; 9.0-9.2 with 24-byte loads)
    // 4-bit
    KMQ_LUT(4, 3, 64, 1, 4, 2, 6),   // K = 1536: 12-byte loads
    KMQ_LUT(4, 4, 64, 1, 4, 2, 6),   // K = 2048
    KMQ_LUT(4, 3, 64, 2, 2, 2, 6),   // K = 3072: two slices of 12-byte loads
    KMQ_LUT(4, 4, 64, 2, 2, 2, 6),   // K = 4096
    KMQ_LUT(4, 4, 64, 3, 2, 2, 6),   // K = 6144
    KMQ_LUT(4, 4, 64, 4, 1, 4, 4),   // K = 8192: 4 rows per workgroup (4096 rows: 6.6 us; 7.0 with 2 or 6)
    KMQ_LUT(4, 4, 64, 4, 1, 2, 6),   //           2
    KMQ_LUT(4, 4, 64, 7, 1, 4, 4),   // K = 14336: 4 rows per workgroup (4096 rows: 10.5 us; 12.2 with 2, 10.9 with 6)
    KMQ_LUT(4, 4, 64, 7, 1, 2, 6),   //            2
    // block-scaled format (lane slices of 32, 64 or 128 elements only)
    KMQ_LUT_SC(1, 4, 16, 1, 4, 1, 4),   // K = 2048
    KMQ_LUT_SC(1, 4, 16, 1, 2, 1, 4),
    KMQ_LUT_SC(1, 4, 32, 1, 4, 2, 4),   // K = 4096
    KMQ_LUT_SC(1, 4, 64, 1, 4, 2, 4),   // K = 8192
    KMQ_LUT_SC(1, 4, 64, 1, 4, 3, 4),
    KMQ_LUT_SC(2, 4, 32, 1, 4, 2, 6),   // K = 2048
    KMQ_LUT_SC(2, 4, 64, 1, 4, 2, 7),   // K = 4096
    KMQ_LUT_SC(2, 4, 64, 2, 2, 4, 4),   // K = 8192
    KMQ_LUT_SC(2, 4, 64, 2, 2, 2, 7),
    KMQ_LUT_SC(2, 4, 32, 7, 1, 4, 4),   // K = 14336
    KMQ_LUT_SC(2, 2, 64, 7, 1, 4, 7),
    KMQ_LUT_SC(3, 6, 32, 1, 4, 2, 6),   // K = 2048
    KMQ_LUT_SC(3, 6, 64, 1, 4, 2, 7),   // K = 4096
    KMQ_LUT_SC(3, 6, 64, 2, 2, 4, 4),   // K = 8192
    KMQ_LUT_SC(3, 6, 64, 2, 2, 2, 6),
    KMQ_LUT_SC(3, 6, 32, 7, 1, 4, 4),   // K = 14336 (lane slices of 64 elements: one block)
    KMQ_LUT_SC(4, 4, 64, 1, 4, 2, 6),   // K = 2048
    KMQ_LUT_SC(4, 4, 64, 2, 2, 2, 6),   // K = 4096
    KMQ_LUT_SC(4, 4, 64, 4, 2, 4, 4),   // K = 8192: 8 rows per workgroup (8192 rows: 10.8 us; 11.3 with 4 rows, 12.8 with 16 rows and 16 waves)
    KMQ_LUT_SC(4, 4, 64, 4, 1, 4, 4),   //           4
    KMQ_LUT_SC(4, 4, 64, 4, 1, 2, 6),
    KMQ_LUT_SC(4, 4, 64, 7, 1, 4, 4),   // K = 14336
    KMQ_LUT_SC(4, 4, 64, 7, 1, 2, 6),
};
constexpr int kLutCount = sizeof(kLut) / sizeof(kLut[0]);

// Cost of a shape for N rows: the most rows any CU gets when the workgroups are dealt
// round-robin over 256 CUs.
int lut_find(int64_t N, int64_t K, int bits, int layout, bool scaled) {
    if (layout != KMQ_LAYOUT_CANONICAL) return -1;
    int pick = -1;
#ifdef KMQ_TUNING
    // sweeps only (builds with -DKMQ_TUNING): KMQ_LUT_PICK=n takes the n-th shape listed for (bits, K)
    static const char* const pick_env = std::getenv("KMQ_LUT_PICK");
    if (pick_env) pick = std::atoi(pick_env);
#endif
    int best = -1;
    int64_t best_cost = 0;
    for (int i = 0; i < kLutCount; ++i) {
        if (kLut[i].bits != bits || kLut[i].K != K || kLut[i].scaled != scaled) continue;
        if (pick >= 0) {
            if (pick-- == 0) return i;
            continue;
        }
        const int64_t wgs = (N + kLut[i].rows_wg - 1) / kLut[i].rows_wg;
        const int64_t cost = ((wgs + 255) / 256) * kLut[i].rows_wg;
        if (best < 0 || cost < best_cost) { best = i; best_cost = cost; }
    }
    return best;
}

const char* lut_name(int i) { return kLut[i].name; }
bool lut_has_fusions(int i) { return !kLut[i].scaled; }

hipError_t launch_lut_entry(int i, const GemmArgs& a, hipStream_t s) {
    kLut[i].launch(a, s);
    return hipGetLastError();
}

}  // namespace kmq
