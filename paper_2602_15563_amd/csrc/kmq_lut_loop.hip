// Batch-1 table kernel for rows of any length that is a multiple of 32 (up to 24576), canonical layout:
// y = W x with w = codebook lookup (paper App. E, "Kernel implementations"; the hidden sizes of the
// paper's models, App. A table of architectural hyperparameters, are only some of the lengths a caller
// may bring).  The kernels specialised on K unroll a row completely; this one walks it in rounds.
//
// Work split.  A round is LPR * 32 consecutive elements of 64 / LPR rows: LPR lanes per row, 32
// elements (BITS words) per lane, so a wave-wide load fetches 64 / LPR runs of LPR * 4 * BITS bytes.  A
// wave owns RS such groups of rows, which share the activations it holds in registers; the NWK waves
// along K of a workgroup take contiguous ranges of a row's rounds, the 8 / NWK waves across take further
// rows.  Lanes past the end of a row (its last round need not be full) read clamped words and zeros for x.
// Few lanes per row waste little of a short row's last round; many keep the lookups free of bank
// conflicts, because lanes of one row read one table.
// Rounds are processed PF at a time: the words of the next PF rounds are requested before the lookups
// of the current ones start, the activations of the current ones are read from the workgroup's staged
// copy of x, and one hand-counted pipeline (the blocks shared with the specialised kernels) runs over
// all of them.  A range that is no multiple of PF ends in rounds whose loads are clamped to the row's
// last words and whose activations come from a slice of zeros.  The lookup tables of a workgroup's
// rows are built once, by all of its waves together, and shared by the waves along K.
//
// K-reduction: DPP adds over the lanes of a row, then across the NWK waves through LDS in fixed
// order; fp32 -> bf16 round-to-nearest-even; one coalesced store per workgroup.
#include <cstdlib>

#include "kmq_device.h"
#include "kmq_launch.h"
#include "kmq_lut_blocks.h"

namespace kmq {

namespace {

constexpr int kLoopMaxK = 24576;          // the staged copy of x: 60 KB of LDS with its padding (the launcher keeps tables + x within 64 KB)
constexpr int kLoopUnrolledK = 16384;     // x up to here is staged with loads that are all in flight at once
constexpr int kLoopThreads = 512;

template <int BITS, int LPR, int NWK, int RS, int PF, int WPE>
__global__ __launch_bounds__(kLoopThreads) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemv_lut_loop_kernel(const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
                          const uint16_t* __restrict__ X, uint16_t* Y, int64_t N, int K, const uint16_t* residual, int mcols) {
    // (Y and residual carry no __restrict__: the fused call documents that they may be the same buffer)
    static_assert(BITS >= 1 && BITS <= 4 && 8 % NWK == 0 && (LPR == 16 || LPR == 32 || LPR == 64), "shape");
    constexpr int C = 1 << BITS;
    constexpr int G = BITS;                        // words per lane and round: 32 elements
    constexpr int NWR = 8 / NWK;
    constexpr int RPL = kWave / LPR;               // rows per wave-wide load
    constexpr int ROWS_WAVE = RPL * RS;
    constexpr int ROWS_WG = NWR * ROWS_WAVE;
    constexpr int U = BITS == 1 ? 2 : BITS == 3 ? 2 : BITS;          // lookup units (8 activation registers each) per round
    constexpr int XR = 8 * U;                      // activation registers per round: bf16 pairs (1/2/3-bit) or fp32 (4-bit)
    constexpr int ENT = BITS == 3 ? 64 : 16;       // table entries per row (3-bit: one per pair of fields)
    constexpr int LUT_TOTAL = BITS == 1 ? 0 : ROWS_WG * ENT;        // table entries of the workgroup's rows
    constexpr int LUT_PASSES = (LUT_TOTAL + kLoopThreads - 1) / kLoopThreads;
    constexpr int TBL = RS * ENT < 64 ? 64 : RS * ENT;              // dwords per (wave across, row of the load): bases stay 256-byte aligned
    constexpr int XSTR = 5;                        // a lane slice of four 16-byte chunks takes five: reads spread over the banks
    constexpr int XPT = kLoopUnrolledK / 8 / kLoopThreads;          // 16-byte chunks of x staged per thread (4); longer rows: a loop for the rest

    struct alignas(256) Smem {
        uint32_t lut[NWR][RPL][TBL];               // per wave across and row of the load: RS tables (1-bit: lut[0][0] holds the mask table)
        float part[NWK][ROWS_WG];
        float sxw[8];                              // 1-bit: per-wave sum of the x it staged
    };
    __shared__ Smem sm;
    // staged activations, K / 32 + 1 slices of XSTR chunks: the last slice is zeros
    extern __shared__ __attribute__((aligned(16))) unsigned char xs_raw[];
    u32x4_t* const xs = reinterpret_cast<u32x4_t*>(xs_raw);
    const int xslices = K >> 5;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wk = wave % NWK, wr = wave / NWK;
    const int sub = lane / LPR, pos = lane % LPR;
    // A batch of mcols activation rows is one launch, every workgroup one column.  Workgroup ids go round-robin over
    // the 8 XCDs, each with its own L2; the id is cut so that the mcols workgroups that read the same rows of W sit on
    // one XCD, one after the other: the first fetches those rows from memory, the others find them in that L2.
    int wg = blockIdx.x, col = 0;
    if (mcols > 1) {
        const int t = wg >> 3;
        col = t % mcols;
        wg = (t / mcols) * 8 + (wg & 7);
        if (static_cast<int64_t>(wg) * ROWS_WG >= N) return;    // the grid is padded to a multiple of 8 row groups
    }
    const uint16_t* x = X + static_cast<int64_t>(col) * K;
    uint16_t* y = Y + static_cast<int64_t>(col) * N;
    const int Nr = static_cast<int>(N);            // row numbers fit 32 bits (the library caps N at 2^24)
    const int wg_row0 = wg * ROWS_WG;
    const int R = (xslices + LPR - 1) / LPR;       // rounds per row (the last one may be partly past the end)
    const int rw = (R + NWK - 1) / NWK;            // rounds per wave, contiguous
    const int r_begin = wk * rw;
    const int r_end = r_begin + rw < R ? r_begin + rw : R;          // (may be <= r_begin for the last waves of a short row)
    const int nit = (rw + PF - 1) / PF;
    const int64_t wpr = static_cast<int64_t>(K) * BITS / 32;
    const uint32_t* wlane[RS];
#pragma unroll
    for (int t = 0; t < RS; ++t) {
        int row = wg_row0 + wr * ROWS_WAVE + t * RPL + sub;
        row = row < Nr ? row : Nr - 1;             // clamped: loads stay unconditional
        wlane[t] = W + static_cast<int64_t>(row) * wpr;
    }
    auto load_rounds = [&](int r0, uint32_t (&w)[PF][RS][G]) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            int sl = (r0 + p) * LPR + pos;         // this lane's slice of 32 elements, clamped into the row
            sl = sl < xslices ? sl : xslices - 1;
#pragma unroll
            for (int t = 0; t < RS; ++t) load_words<G>(wlane[t] + sl * G, w[p][t]);
        }
    };

    // ---- 1. loads, small operands first: x, codebook rows, then the first rounds' words ----
    const int nch = K >> 3;
    u32x4_t xt[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        int c = threadIdx.x + i * kLoopThreads;
        c = c < nch ? c : nch - 1;
        xt[i] = *reinterpret_cast<const u32x4_t*>(x + c * 8);
    }
    // residual behind the product (a decoder layer's down projection, paper App. E "Model benchmarks"): the two
    // rows this thread stores, fetched with the first loads so that they are long there when the epilogue runs
    uint32_t resv[2] = {0u, 0u};
    if (residual) {                                // uniform
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int rl = threadIdx.x * 2 + h;          // (only threads below ROWS_WG / 2 store)
            rl = rl < ROWS_WG ? rl : ROWS_WG - 1;
            int r2 = wg_row0 + rl;
            r2 = r2 < Nr ? r2 : Nr - 1;
            resv[h] = residual[r2];
        }
    }
    [[maybe_unused]] uint32_t ccv[2];              // 1-bit: centroid pair of the two rows this thread stores
    if constexpr (BITS == 1) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int rl = threadIdx.x * 2 + h;          // (only threads below ROWS_WG / 2 store)
            rl = rl < ROWS_WG ? rl : ROWS_WG - 1;
            int r2 = wg_row0 + rl;
            r2 = r2 < Nr ? r2 : Nr - 1;
            ccv[h] = *reinterpret_cast<const uint32_t*>(codebook + static_cast<int64_t>(r2) * C);
        }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    // codebook rows of the table entries this thread builds: entry q of the workgroup = (row q / ENT, entry q % ENT)
    uint32_t cbv[LUT_PASSES > 0 ? LUT_PASSES : 1][BITS == 4 ? 1 : BITS == 3 ? 4 : 2];
#pragma unroll
    for (int p = 0; p < LUT_PASSES; ++p) {
        int q = threadIdx.x + p * kLoopThreads;
        q = q < LUT_TOTAL ? q : LUT_TOTAL - 1;
        int r2 = wg_row0 + q / ENT;
        r2 = r2 < Nr ? r2 : Nr - 1;
        const uint16_t* cb = codebook + static_cast<int64_t>(r2) * C;
        if constexpr (BITS == 2) {
            typedef u32x2_t __attribute__((aligned(4))) u32x2_a4_t;
            const u32x2_t c = *reinterpret_cast<const u32x2_a4_t*>(cb);
            cbv[p][0] = c[0];
            cbv[p][1] = c[1];
        } else if constexpr (BITS == 3) {
            typedef u32x4_t __attribute__((aligned(4))) u32x4_a4_t;
            const u32x4_t c = *reinterpret_cast<const u32x4_a4_t*>(cb);
#pragma unroll
            for (int j = 0; j < 4; ++j) cbv[p][j] = c[j];
        } else {
            cbv[p][0] = cb[q % ENT];
        }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    uint32_t w[PF][RS][G], wn[PF][RS][G];
    load_rounds(r_begin, w);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // ---- 2. x into LDS (its loads are the oldest in the queue: this waits for them only) ----
    [[maybe_unused]] float sxl = 0.f;
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        // the value is pinned ahead of the branch: a load whose only use sits behind a branch is sunk into it
        asm volatile("" : "+v"(xt[i]));
    }
    asm volatile("" : "+v"(resv[0]), "+v"(resv[1]));
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        const int c = threadIdx.x + i * kLoopThreads;
        if (c < nch) {
            xs[(c >> 2) * XSTR + (c & 3)] = xt[i];
            if constexpr (BITS == 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) sxl = dot2_bf16(0x3F803F80u, xt[i][j], sxl);
            }
        }
    }
    for (int c = threadIdx.x + XPT * kLoopThreads; c < nch; c += kLoopThreads) {      // rows beyond 16384 elements
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(x + c * 8);
        xs[(c >> 2) * XSTR + (c & 3)] = v;
        if constexpr (BITS == 1) {
#pragma unroll
            for (int j = 0; j < 4; ++j) sxl = dot2_bf16(0x3F803F80u, v[j], sxl);
        }
    }
    if (threadIdx.x < XSTR) xs[xslices * XSTR + threadIdx.x] = u32x4_t{0u, 0u, 0u, 0u};
    if constexpr (BITS == 1) {
        sxl = group_sum<64>(sxl);
        if (lane == 63) sm.sxw[wave] = sxl;
        if (threadIdx.x < 16) {
            const uint32_t e = threadIdx.x;
            u32x2_t m;
            m[0] = ((e & 1u) ? 0x3F80u : 0u) | ((e & 2u) ? 0x3F800000u : 0u);
            m[1] = ((e & 4u) ? 0x3F80u : 0u) | ((e & 8u) ? 0x3F800000u : 0u);
            reinterpret_cast<u32x2_t*>(&sm.lut[0][0][0])[e] = m;
        }
    }
    // the tables of the workgroup's rows: row rl of the workgroup belongs to wave across rl / ROWS_WAVE, table t of load row sb
    if constexpr (BITS != 1) {
#pragma unroll
        for (int p = 0; p < LUT_PASSES; ++p) {
            const int q = threadIdx.x + p * kLoopThreads;
            const int rl = q / ENT, e = q % ENT;
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
            const int wr2 = rl / ROWS_WAVE, t2 = (rl % ROWS_WAVE) / RPL, sb = rl % RPL;
            if (LUT_TOTAL % kLoopThreads == 0 || q < LUT_TOTAL) sm.lut[wr2][sb][t2 * ENT + e] = entry;
        }
    }
    __syncthreads();

    // ---- 3. rounds ----
    const uint32_t lut_base = static_cast<uint32_t>(reinterpret_cast<size_t>(
        (lds_cu32_t*)(&sm.lut[BITS == 1 ? 0 : wr][BITS == 1 ? 0 : sub][0])));
    uint32_t ar[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ar[i] = lut_base;
    const uint32_t mask = BITS == 1 ? 0x78u : BITS == 3 ? 0xFCu : 0x3Cu;
    float acc[RS][2];                              // two accumulator chains per row, kept across all rounds
#pragma unroll
    for (int t = 0; t < RS; ++t) acc[t][0] = acc[t][1] = 0.f;
    // One iteration = PF rounds.  MORE: the words of the next iteration are requested first and become the
    // current ones at the end.  The last iteration is a copy of the code without those loads rather than a
    // branch around them: with a branch, the number of loads in flight would depend on the path and every
    // wait for the current words would have to assume the fewest, i.e. wait for the loads just issued.
    auto iteration = [&](int it, auto more) {
        constexpr bool MORE = decltype(more)::value;
        const int r0 = r_begin + it * PF;
        if constexpr (MORE) load_rounds(r0 + PF, wn);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        uint32_t xr[PF][XR];
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            int sl = (r0 + p) * LPR + pos;
            sl = sl < (r0 + p < r_end ? xslices : 0) ? sl : xslices;     // past the wave's range or the row's end: the slice of zeros
            const u32x4_t* xp = xs + sl * XSTR;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32x4_t v = xp[q];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if constexpr (BITS == 4) {
                        xr[p][q * 8 + 2 * j] = v[j] << 16;
                        xr[p][q * 8 + 2 * j + 1] = v[j] & 0xFFFF0000u;
                    } else {
                        xr[p][q * 4 + j] = v[j];
                    }
                }
            }
        }
        // everything the compiler itself has in flight on the LGKM counter must have landed before the
        // hand-counted pipeline starts
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        constexpr int NU = PF * RS * U;                              // unit n: round n / (RS * U), row group (n / U) % RS
        if constexpr (BITS == 1) {
            u32x2_t vv[2][4];
            uint32_t re = 0, ro = 0;
            issue4_b64<0>(w[0][0][0], re, ro, ar, vv[0], mask);
            static_for<0, NU>([&](auto ic) {
                constexpr int n = decltype(ic)::value;
                constexpr int p = n / (RS * U), t = (n / U) % RS, u = n % U;
                if constexpr (n + 1 < NU) {
                    constexpr int p1 = (n + 1) / (RS * U), t1 = ((n + 1) / U) % RS, u1 = (n + 1) % U;
                    issue4_b64<u1 % 2>(w[p1][t1][u1 / 2], re, ro, ar, vv[(n + 1) & 1], mask);
                    consume4_b64<4>(vv[n & 1], &xr[p][u * 8], acc[t][0], acc[t][1]);
                } else {
                    consume4_b64<0>(vv[n & 1], &xr[p][u * 8], acc[t][0], acc[t][1]);
                }
            });
        } else {
            uint32_t v[2][8];
            uint32_t re = 0, ro = 0;
            // half hh (0, 1) of unit nn into vd[4 hh .. 4 hh + 3]
            auto issue_half = [&](auto nc, auto hc, uint32_t (&vd)[8]) {
                constexpr int nn = decltype(nc)::value, hh = decltype(hc)::value;
                constexpr int pp = nn / (RS * U), tt = (nn / U) % RS, uu = nn % U;
                if constexpr (BITS == 3) {
                    issue4_p6<tt * ENT * 4, 2 * (uu % 2) + hh>(w[pp][tt][0], w[pp][tt][1], w[pp][tt][2], ar, &vd[4 * hh], mask);
                } else {
                    issue4_b32<tt * ENT * 4, hh>(w[pp][tt][uu], re, ro, ar, vd, mask);
                }
            };
            using std::integral_constant;
            issue_half(integral_constant<int, 0>{}, integral_constant<int, 0>{}, v[0]);
            issue_half(integral_constant<int, 0>{}, integral_constant<int, 1>{}, v[0]);
            static_for<0, NU>([&](auto ic) {
                constexpr int n = decltype(ic)::value;
                constexpr int p = n / (RS * U), t = (n / U) % RS, u = n % U;
                if constexpr (n + 1 < NU) {
                    issue_half(integral_constant<int, n + 1>{}, integral_constant<int, 0>{}, v[(n + 1) & 1]);
                    if constexpr (BITS != 4) consume8_dot2<4>(v[n & 1], &xr[p][u * 8], acc[t][0], acc[t][1]);
                    else consume8_fma<4>(v[n & 1], &xr[p][u * 8], acc[t][0], acc[t][1]);
                    issue_half(integral_constant<int, n + 1>{}, integral_constant<int, 1>{}, v[(n + 1) & 1]);
                } else {
                    if constexpr (BITS != 4) consume8_dot2<0>(v[n & 1], &xr[p][u * 8], acc[t][0], acc[t][1]);
                    else consume8_fma<0>(v[n & 1], &xr[p][u * 8], acc[t][0], acc[t][1]);
                }
            });
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (MORE) {
#pragma unroll
            for (int p = 0; p < PF; ++p)
#pragma unroll
                for (int t = 0; t < RS; ++t)
#pragma unroll
                    for (int g = 0; g < G; ++g) w[p][t][g] = wn[p][t][g];
        }
    };
    for (int it = 0; it + 1 < nit; ++it) iteration(it, std::true_type{});
    iteration(nit - 1, std::false_type{});

    // ---- 4. K-reduction: the lanes of a row, then the waves along K through LDS ----
#pragma unroll
    for (int t = 0; t < RS; ++t) {
        settle_dot(acc[t][0], acc[t][1]);
        float s = acc[t][0] + acc[t][1];
        s = group_sum<LPR>(s);         // valid in the last lane of the group
        if (pos == LPR - 1) sm.part[wk][wr * ROWS_WAVE + t * RPL + sub] = s;
    }
    __syncthreads();

    // ---- 5. epilogue: two rows per thread, one coalesced store per workgroup ----
    if (threadIdx.x < ROWS_WG / 2) {
        float out[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int rl = threadIdx.x * 2 + h;
            float t = 0.f;
#pragma unroll
            for (int k = 0; k < NWK; ++k) t += sm.part[k][rl];
            if constexpr (BITS == 1) {
                // two centroids: y = c0 * sum(x) + (c1 - c0) * sum of the x whose index is 1
                float sx = 0.f;
#pragma unroll
                for (int k = 0; k < 8; ++k) sx += sm.sxw[k];
                const float c0 = bf16_to_f32(ccv[h] & 0xFFFFu), c1 = bf16_to_f32(ccv[h] >> 16);
                t = fmaf(c1 - c0, t, c0 * sx);
            }
            if (residual) t += bf16_to_f32(resv[h]);
            out[h] = t;
        }
        const int r2 = wg_row0 + threadIdx.x * 2;
        const uint32_t packed = static_cast<uint32_t>(f32_to_bf16(out[0])) | (static_cast<uint32_t>(f32_to_bf16(out[1])) << 16);
        if (r2 + 1 < Nr && (reinterpret_cast<uintptr_t>(y + r2) & 3u) == 0) {
            *reinterpret_cast<uint32_t*>(y + r2) = packed;
        } else {
            if (r2 < Nr) y[r2] = static_cast<uint16_t>(packed);
            if (r2 + 1 < Nr) y[r2 + 1] = static_cast<uint16_t>(packed >> 16);
        }
    }
}

struct LoopShape { int lpr, nwk; size_t x_bytes; };

constexpr int kRS = 2;                                            // groups of rows per wave
constexpr int kPF(int bits) { return bits == 4 ? 1 : 2; }         // rounds per iteration (4-bit keeps x as fp32: 32 registers per round)

// Lanes per row and waves along K for N rows of K elements: the shape with the lowest estimate of the time of
// the fullest CU, workgroups per CU x (a workgroup's fixed cost + its rounds x the cost of a round).  The unit is
// one wave's round over one group of rows; the constants are fits to measurements (14336 x 4096, 28672 x 5120,
// 4096 x {2560, 4096, 11008}, every shape): the fixed cost -- staging x, building the tables, two barriers -- is
// 19 / 11.5 / 5.5 / 4 units at 1 / 2 / 3 / 4 bits, and the tables of the 64 / LPR rows a wave looks up at once
// collide in the LDS banks: a round costs 1.27 (2 rows) or 2 (4 rows) units at 2 and 4 bits, 1.5 or 1.7 at 3 bits.
LoopShape loop_shape(int64_t N, int64_t K, int bits) {
    LoopShape best{64, 1, static_cast<size_t>((K / 32 + 1) * 5 * 16)};
#ifdef KMQ_TUNING
    static const char* const env = std::getenv("KMQ_LOOP_SHAPE");       // sweeps only: "<lanes per row / 8><nwk>", e.g. 84
    if (env && env[0] && env[1]) { best.lpr = (env[0] - '0') * 8; best.nwk = env[1] - '0'; return best; }
#endif
    const int pf = kPF(bits);
    static const int64_t fixed_x100[4] = {1900, 1150, 550, 400};
    static const int64_t round_x100[4][3] = {{100, 100, 100}, {100, 127, 200}, {100, 150, 170}, {100, 127, 200}};   // LPR = 64, 32, 16
    int64_t best_cost = -1;
    int li = 0;
    for (int lpr = 64; lpr >= 16; lpr /= 2, ++li) {
        const int64_t R = (K / 32 + lpr - 1) / lpr;
        for (int nwk = 1; nwk <= 8; nwk *= 2) {
            const int64_t rows_wg = 8 / nwk * (64 / lpr) * kRS;
            // static LDS: the tables (256-byte aligned slots per wave across and row of the load) and the partial sums
            const int64_t ent = bits == 3 ? 64 : 16, slot = kRS * ent < 64 ? 256 : kRS * ent * 4;
            const int64_t static_bytes = (bits == 1 ? 256 : 8 / nwk * (64 / lpr) * slot) + 8 * rows_wg * 4 + 512;
            if (static_bytes + static_cast<int64_t>(best.x_bytes) > 65536) continue;
            const int64_t wgs = (N + rows_wg - 1) / rows_wg;
            const int64_t per_cu_x100 = wgs * 100 / 256 < 100 ? 100 : wgs * 100 / 256;
            const int64_t rw = (R + nwk - 1) / nwk;
            const int64_t cost = per_cu_x100 * (fixed_x100[bits - 1] + (rw + pf - 1) / pf * pf * kRS * round_x100[bits - 1][li]);
            if (best_cost < 0 || cost < best_cost) { best.lpr = lpr; best.nwk = nwk; best_cost = cost; }
        }
    }
    return best;
}

template <int BITS, int WPE>
void launch_loop_bits(const GemmArgs& a, hipStream_t s) {
    const LoopShape sh = loop_shape(a.N, a.K, a.bits);
    const int rows_wg = 8 / sh.nwk * (64 / sh.lpr) * kRS;
    const int64_t groups = (a.N + rows_wg - 1) / rows_wg;
    const dim3 grid(static_cast<unsigned>(a.M > 1 ? (groups + 7) / 8 * 8 * a.M : groups)), block(kLoopThreads);
#define KMQ_LOOP(LPR, NWK) hipLaunchKernelGGL((gemv_lut_loop_kernel<BITS, LPR, NWK, kRS, kPF(BITS), WPE>), grid, block, sh.x_bytes, s, \
                                              a.W, a.codebook, a.X, a.Y, a.N, static_cast<int>(a.K), a.residual, a.M)
#define KMQ_LOOP_NWK(LPR) \
    switch (sh.nwk) { case 1: KMQ_LOOP(LPR, 1); break; case 2: KMQ_LOOP(LPR, 2); break; case 4: KMQ_LOOP(LPR, 4); break; default: KMQ_LOOP(LPR, 8); break; }
    switch (sh.lpr) {
        case 16: KMQ_LOOP_NWK(16) break;
        case 32: KMQ_LOOP_NWK(32) break;
        default: KMQ_LOOP_NWK(64) break;
    }
#undef KMQ_LOOP_NWK
#undef KMQ_LOOP
}

}  // namespace

bool lut_loop_has_kernel(int64_t N, int64_t K, int bits, int layout) {
    return layout == KMQ_LAYOUT_CANONICAL && bits >= 1 && bits <= 4 && K >= 32 && K % 32 == 0 && K <= kLoopMaxK && N >= 1;
}

const char* lut_loop_name(int bits) {
    static const char* const names[4] = {"lut_loop_b1", "lut_loop_b2", "lut_loop_b3", "lut_loop_b4"};
    return names[bits - 1];
}

hipError_t launch_lut_loop(const GemmArgs& a, hipStream_t s) {
    if (!lut_loop_has_kernel(a.N, a.K, a.bits, a.layout) || a.scales || a.W2 || a.norm || (a.residual && a.M != 1)) return hipErrorInvalidValue;
    switch (a.bits) {
        case 1: launch_loop_bits<1, 4>(a, s); break;
        case 2: launch_loop_bits<2, 4>(a, s); break;
        case 3: launch_loop_bits<3, 4>(a, s); break;
        default: launch_loop_bits<4, 4>(a, s); break;
    }
    return hipGetLastError();
}

}  // namespace kmq
