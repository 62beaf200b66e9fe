// Batch 1..4 kernels on the row-lane layout (KMQ_LAYOUT_ROWLANE, include/kmq.h): y = W x with
// w = codebook lookup (paper App. E, "Kernel implementations"), for the small-batch regime the
// paper calls memory-bound (App. D) on a machine where the decode, not the memory, is the longer
// side of a call.
//
// Work split.  A workgroup owns one block of 16 rows; its waves split K.  A wave-wide load of
// index words is one TILE (16 rows x 256 columns): lane (kp, r) = (lane / 16, lane % 16) gets
// chunk kp (64 columns: 8 bytes at 1 bit, 16 bytes at 2 bits) of row r, so the 16 lanes of a DPP
// row hold 16 different rows over the SAME 64 columns.
//
// Activations never pass through LDS and are never duplicated per row: the lanes of DPP row kp
// hold the 32 bf16 pairs of chunk kp, two per lane (one 8-byte load per lane, 512 contiguous
// bytes per wave), and a multiply-accumulate reads the pair it needs from its row of lanes with
// the DPP broadcast of v_dot2c_f32_bf16 (row_newbcast:j: every lane of a 16-lane row sees lane
// j's register).  The layout's bit order is chosen so that the j-th lookup of a register pairs
// with lane j.
//
// Weights.  2-bit: a nibble (two indices) addresses a 16-entry table of bf16 PAIRS, one column
// per lane ([entry][lane], 4 KB per workgroup, so a wave's 64 lookups never meet in a bank); the
// address is one SDWA byte-AND that drops the nibble into byte 1 of a register holding lane*4.
// 1-bit: a nibble addresses a row-independent table of four bf16 {0,1} masks (one copy per wave,
// so nothing waits for it); the kernel accumulates S1 = sum_{idx=1} x and finishes with the
// two-centroid closed form y = c0*sum(x) + (c1 - c0)*S1.
//
// K-reduction: every lane keeps one fp32 sum per batch column; lanes and waves are summed
// through LDS in a fixed order (deterministic), rounded to bf16 (nearest even), and stored as
// one contiguous run per workgroup and batch column.
#include <cstdlib>
#include <type_traits>

#include "kmq_device.h"
#include "kmq_launch.h"

namespace kmq {

namespace rowlane {

typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;
typedef __attribute__((address_space(1))) const char global_cchar_t;     // a global (not generic) pointer survives the integer round trip below

template <int I, int END, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < END) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, END>(f);
    }
}

// Four lookups per call, at most 12 in flight (the LGKM counter of a wave has 4 bits).
//
// 2-bit pair table: nibbles of bytes 2H and 2H + 1 of `w` (even nibbles) and of `ws` = w >> 4
// (odd nibbles).  `a` holds lane*4 in byte 0; byte 1 receives the nibble: entry*256 + lane*4.
#define KMQ_RL_SDWA(dst, src, dbyte, sbyte) \
    "v_and_b32_sdwa " dst ", " src ", %10 dst_sel:BYTE_" dbyte " dst_unused:UNUSED_PRESERVE src0_sel:BYTE_" sbyte " src1_sel:DWORD\n\t"
// OFF: byte offset of the table inside the workgroup's LDS (an immediate of the read: byte 1 of the
// address register belongs to the nibble).
template <int H, int OFF = 0>
__device__ __forceinline__ void issue4_pair(uint32_t w, uint32_t ws, uint32_t (&a)[4], uint32_t* v, uint32_t mask) {
    static_assert(OFF >= 0 && OFF < 65536, "16-bit offset field");
    if constexpr (H == 0) {
        asm volatile(
            KMQ_RL_SDWA("%4", "%8", "1", "0") KMQ_RL_SDWA("%5", "%9", "1", "0") KMQ_RL_SDWA("%6", "%8", "1", "1") KMQ_RL_SDWA("%7", "%9", "1", "1")
            "ds_read_b32 %0, %4 offset:%c11\n\tds_read_b32 %1, %5 offset:%c11\n\tds_read_b32 %2, %6 offset:%c11\n\tds_read_b32 %3, %7 offset:%c11"
            : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(w), "v"(ws), "v"(mask), "n"(OFF));
    } else {
        asm volatile(
            KMQ_RL_SDWA("%4", "%8", "1", "2") KMQ_RL_SDWA("%5", "%9", "1", "2") KMQ_RL_SDWA("%6", "%8", "1", "3") KMQ_RL_SDWA("%7", "%9", "1", "3")
            "ds_read_b32 %0, %4 offset:%c11\n\tds_read_b32 %1, %5 offset:%c11\n\tds_read_b32 %2, %6 offset:%c11\n\tds_read_b32 %3, %7 offset:%c11"
            : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(w), "v"(ws), "v"(mask), "n"(OFF));
    }
}

// 1-bit mask table (16 entries of 8 bytes): a nibble sits at bits 3..6 of a byte of `w` (view 0)
// or of `wr` = w rotated right by 4 (view 1), which is the entry's byte offset; `a` holds the
// 256-byte-aligned table base in bytes 1..3.  vv[i] = masks of elements 0,1 and of elements 2,3
// of nibble 4H + i of the word (byte 2H + i/2, view i%2).
template <int H>
__device__ __forceinline__ void issue4_mask(uint32_t w, uint32_t wr, uint32_t (&a)[4], u32x2_t* vv, uint32_t mask) {
    if constexpr (H == 0) {
        asm volatile(
            KMQ_RL_SDWA("%4", "%8", "0", "0") KMQ_RL_SDWA("%5", "%9", "0", "0") KMQ_RL_SDWA("%6", "%8", "0", "1") KMQ_RL_SDWA("%7", "%9", "0", "1")
            "ds_read_b64 %0, %4\n\tds_read_b64 %1, %5\n\tds_read_b64 %2, %6\n\tds_read_b64 %3, %7"
            : "=&v"(vv[0]), "=&v"(vv[1]), "=&v"(vv[2]), "=&v"(vv[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(w), "v"(wr), "v"(mask));
    } else {
        asm volatile(
            KMQ_RL_SDWA("%4", "%8", "0", "2") KMQ_RL_SDWA("%5", "%9", "0", "2") KMQ_RL_SDWA("%6", "%8", "0", "3") KMQ_RL_SDWA("%7", "%9", "0", "3")
            "ds_read_b64 %0, %4\n\tds_read_b64 %1, %5\n\tds_read_b64 %2, %6\n\tds_read_b64 %3, %7"
            : "=&v"(vv[0]), "=&v"(vv[1]), "=&v"(vv[2]), "=&v"(vv[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(w), "v"(wr), "v"(mask));
    }
}
#undef KMQ_RL_SDWA

// 2-bit: eight multiply-accumulates of looked-up weight pairs against the activation pairs that
// lanes BC .. BC + 7 of this lane's DPP row hold in `x`.  PENDING >= 0: first wait until at most
// that many LDS reads are outstanding.
#define KMQ_RL_DOT(acc, xx, vv, j) "v_dot2c_f32_bf16_dpp " acc ", " xx ", " vv " row_newbcast:" j " row_mask:0xf bank_mask:0xf\n\t"
template <int PENDING, int BC>
__device__ __forceinline__ void dot8_pair(const uint32_t* v, uint32_t x, float& a0, float& a1) {
    static_assert(BC == 0 || BC == 8, "half of a 16-lane row");
    if constexpr (PENDING >= 0) asm volatile("s_waitcnt lgkmcnt(%c0)" : : "n"(PENDING) : "memory");
    if constexpr (BC == 0) {
        asm volatile(
            KMQ_RL_DOT("%0", "%10", "%2", "0") KMQ_RL_DOT("%1", "%10", "%3", "1") KMQ_RL_DOT("%0", "%10", "%4", "2") KMQ_RL_DOT("%1", "%10", "%5", "3")
            KMQ_RL_DOT("%0", "%10", "%6", "4") KMQ_RL_DOT("%1", "%10", "%7", "5") KMQ_RL_DOT("%0", "%10", "%8", "6") KMQ_RL_DOT("%1", "%10", "%9", "7")
            : "+v"(a0), "+v"(a1)
            : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]), "v"(x));
    } else {
        asm volatile(
            KMQ_RL_DOT("%0", "%10", "%2", "8") KMQ_RL_DOT("%1", "%10", "%3", "9") KMQ_RL_DOT("%0", "%10", "%4", "10") KMQ_RL_DOT("%1", "%10", "%5", "11")
            KMQ_RL_DOT("%0", "%10", "%6", "12") KMQ_RL_DOT("%1", "%10", "%7", "13") KMQ_RL_DOT("%0", "%10", "%8", "14") KMQ_RL_DOT("%1", "%10", "%9", "15")
            : "+v"(a0), "+v"(a1)
            : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]), "v"(x));
    }
}

// 1-bit: the four nibbles S0 .. S0 + 3 of a chunk (sixteen elements): nibble s multiplies the
// masks of its elements 0,1 with the pair lane s holds in x0 and those of elements 2,3 with the
// pair lane s holds in x1.
template <int PENDING, int S0>
__device__ __forceinline__ void dot8_mask(const u32x2_t* vv, uint32_t x0, uint32_t x1, float& a0, float& a1) {
    static_assert(S0 == 0 || S0 == 4 || S0 == 8 || S0 == 12, "a group of four nibbles");
    if constexpr (PENDING >= 0) asm volatile("s_waitcnt lgkmcnt(%c0)" : : "n"(PENDING) : "memory");
#define KMQ_RL_DOT8(j0, j1, j2, j3) \
        asm volatile( \
            KMQ_RL_DOT("%0", "%10", "%2", j0) KMQ_RL_DOT("%1", "%11", "%3", j0) KMQ_RL_DOT("%0", "%10", "%4", j1) KMQ_RL_DOT("%1", "%11", "%5", j1) \
            KMQ_RL_DOT("%0", "%10", "%6", j2) KMQ_RL_DOT("%1", "%11", "%7", j2) KMQ_RL_DOT("%0", "%10", "%8", j3) KMQ_RL_DOT("%1", "%11", "%9", j3) \
            : "+v"(a0), "+v"(a1) \
            : "v"(vv[0][0]), "v"(vv[0][1]), "v"(vv[1][0]), "v"(vv[1][1]), "v"(vv[2][0]), "v"(vv[2][1]), "v"(vv[3][0]), "v"(vv[3][1]), \
              "v"(x0), "v"(x1))
    if constexpr (S0 == 0) KMQ_RL_DOT8("0", "1", "2", "3");
    else if constexpr (S0 == 4) KMQ_RL_DOT8("4", "5", "6", "7");
    else if constexpr (S0 == 8) KMQ_RL_DOT8("8", "9", "10", "11");
    else KMQ_RL_DOT8("12", "13", "14", "15");
#undef KMQ_RL_DOT8
}
#undef KMQ_RL_DOT

// A dot instruction's result may feed the next dot's accumulator at once; any other vector
// instruction reading it needs three wait states, which the compiler cannot count across an
// asm block.
__device__ __forceinline__ void settle(float& a0, float& a1) { asm volatile("s_nop 2" : "+v"(a0), "+v"(a1)); }

template <int G> struct WordVec;
template <> struct WordVec<2> { using type = u32x2_t; };
template <> struct WordVec<4> { using type = u32x4_t; };

}  // namespace rowlane

#ifdef KMQ_TIMESTAMPS
// Instrumented builds only: per-wave time stamps (100 MHz wall clock), [workgroup][wave][8].
__device__ unsigned long long kmq_rowlane_ts[1024 * 16 * 8];
#define KMQ_TS(i) do { if (ts_on) { const unsigned long long t_ = __builtin_amdgcn_s_memrealtime(); \
    if (lane == 0) kmq_rowlane_ts[(blockIdx.x * 16 + wave) * 8 + (i)] = t_; } } while (0)
#else
#define KMQ_TS(i) do { } while (0)
#endif

// BITS 1 or 2; CPW tiles per wave; MB batch columns; WPE waves per SIMD the register budget is
// sized for.  K = 256 * CPW * (waves per workgroup); the grid is one workgroup per 16-row block.
// LOOP: any K that is a multiple of 256: the workgroup walks K in rounds of CPW * (waves) tiles;
// a tile past the end of the last round is read from a valid address and meets activations
// forced to zero.  (The loads of a round are issued when the round starts, nothing is in flight
// across rounds: the shapes with a kernel of their own do not take this path.)
// DBG (instrumented builds only) takes parts of the kernel out, to time the rest: 1 no loads of
// x, 2 no loads of the codebook, 16 no lookups, 32 no loads of the index words, 64 no store.
// PAIR: the fused gate / up / SwiGLU call: the workgroup decodes the same 16 rows of TWO matrices (W, W2)
// against the same activations -- a wave's tiles of W2 follow its tiles of W through the same pipeline,
// with a second pair table -- and stores silu(W x) * (W2 x).
template <int BITS, int CPW, int MB, int WPE, bool LOOP = false, int DBG = 0, bool PAIR = false>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemv_rowlane_kernel(const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
                         const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int64_t N, int64_t K,
                         const uint32_t* __restrict__ W2 = nullptr, const uint16_t* __restrict__ codebook2 = nullptr) {
    using namespace rowlane;
    static_assert(BITS == 1 || BITS == 2, "bit-width");
    static_assert(!PAIR || (MB == 1 && !LOOP), "the fused pair: one activation vector, shapes with a kernel of their own");
    constexpr int NMAT = PAIR ? 2 : 1;
    constexpr int G = 2 * BITS;                     // index words per lane and tile
    constexpr int TILE_BYTES = 256 * G;
    struct alignas(256) Smem {
        // 2-bit: per matrix, [entry][lane] bf16 pairs (centroid of the even element, of the odd element);
        // 1-bit: per wave, at a 256-byte stride, 16 entries of four bf16 {0,1} masks
        uint32_t lut[NMAT * 16 * 64];
        float part[NMAT * MB][16][64];  // [matrix, column][wave][lane] partial sums
        float sx[MB][16];               // 1-bit: per column and wave, the sum of the wave's activations
    };
    __shared__ Smem sm;

    // Everything that can be is computed on the scalar unit: the waves of a launch all start at once,
    // and every vector instruction ahead of the loads delays the moment the memory system gets to work.
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t nwk = blockDim.x >> 6;
    const uint32_t rb = blockIdx.x;
    const uint32_t tiles = static_cast<uint32_t>(K >> 8);
#ifdef KMQ_TIMESTAMPS
    const bool ts_on = blockIdx.x < 1024 && MB == 1;
#endif
    KMQ_TS(0);

    // ---- loads, small operands first (a wave's loads return in issue order) ----------------
    // byte offsets inside a tile: 8*BITS per lane of W, 8 per lane of x (chunk kp starts 128 bytes
    // after chunk kp - 1, so lane kp*16 + r reads at lane*8), 2^BITS * 2 per row of the codebook
    const uint32_t off_x = lane * 8, off_w = BITS == 1 ? off_x : lane * 16;
    const int64_t rows_left = N - static_cast<int64_t>(rb) * 16;
    constexpr uint32_t CB_ROW = 4u << (BITS - 1);                               // bytes of a row's codebook
    const uint32_t last_c = __builtin_amdgcn_readfirstlane(rows_left < 16 ? static_cast<uint32_t>(rows_left - 1) * CB_ROW : 15u * CB_ROW);
    uint32_t off_c = BITS == 1 ? (lane * 4) & 0x3Cu : off_x & 0x78u;
    off_c = off_c < last_c ? off_c : last_c;                                   // rows past N read the last row
    const char* const cb_base = reinterpret_cast<const char*>(codebook) + static_cast<uint64_t>(rb) * (16 * CB_ROW);
    const char* const x_base = reinterpret_cast<const char*>(X) + static_cast<uint32_t>(wave) * 512;
    const char* const w_base = reinterpret_cast<const char*>(W) + (static_cast<uint64_t>(rb) * tiles + static_cast<uint32_t>(wave)) * TILE_BYTES;
    uint32_t cb[2];                                                            // 2-bit: four centroids; 1-bit: cb[0] = (c0, c1)
    [[maybe_unused]] uint32_t cb2[2] = {0, 0};                                  // PAIR: the same row of the second matrix
    if constexpr (DBG & 2) {
        cb[0] = 0x3C003B00u + lane;
        cb[1] = 0x3E003D00u;
    } else if constexpr (BITS == 2) {
        typedef u32x2_t __attribute__((aligned(4))) u32x2_a4_t;
        const u32x2_t c = *reinterpret_cast<const u32x2_a4_t*>(cb_base + off_c);
        cb[0] = c[0];
        cb[1] = c[1];
        if constexpr (PAIR) {
            const u32x2_t c2 = *reinterpret_cast<const u32x2_a4_t*>(reinterpret_cast<const char*>(codebook2) + static_cast<uint64_t>(rb) * (16 * CB_ROW) + off_c);
            cb2[0] = c2[0];
            cb2[1] = c2[1];
        }
    } else {
        cb[0] = *reinterpret_cast<const uint32_t*>(cb_base + off_c);
        cb[1] = 0;
        if constexpr (PAIR) cb2[0] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(codebook2) + static_cast<uint64_t>(rb) * (16 * CB_ROW) + off_c);
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);      // (left alone, the compiler sinks this load below the index loads)
    u32x2_t xv[MB][CPW];
    using wvec_t = typename WordVec<G>::type;
    wvec_t wv[NMAT * CPW];                                                      // PAIR: slots CPW .. 2 CPW - 1 hold the second matrix
    float acc[NMAT * MB][2];
#pragma unroll
    for (int m = 0; m < NMAT * MB; ++m) acc[m][0] = acc[m][1] = 0.f;
    [[maybe_unused]] float sxl[MB];                                            // LOOP, 1-bit: this lane's share of the sum of x
#pragma unroll
    for (int m = 0; m < MB; ++m) sxl[m] = 0.f;
    uint32_t lut_base = static_cast<uint32_t>(reinterpret_cast<size_t>((lds_cu32_t*)(&sm.lut[0])));
    if constexpr (BITS == 1) lut_base += static_cast<uint32_t>(wave) * 256;
    uint32_t t0 = 0;                                                           // first tile of the round
    do {
    // tile of slot j in this round: t0 + j * nwk + wave (LOOP: clamped, and x masked, past the end)
    uint32_t tile_of[CPW];
    [[maybe_unused]] uint32_t live[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        const uint32_t t = t0 + static_cast<uint32_t>(j) * nwk + static_cast<uint32_t>(wave);
        if constexpr (LOOP) {
            const bool in = t < tiles;
            tile_of[j] = __builtin_amdgcn_readfirstlane(in ? t : tiles - 1);
            live[j] = __builtin_amdgcn_readfirstlane(in ? 0xFFFFFFFFu : 0u);
        } else {
            tile_of[j] = t;
        }
    }
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            // (the tile's base stays on the scalar side: pinned, or the sum is re-associated into vector adds)
            uint64_t xb = LOOP ? reinterpret_cast<uint64_t>(X) + static_cast<uint64_t>(m) * K * 2 + static_cast<uint64_t>(tile_of[j]) * 512
                               : reinterpret_cast<uint64_t>(x_base) + static_cast<uint64_t>(m) * K * 2 + static_cast<uint64_t>(j) * nwk * 512;
            asm volatile("" : "+s"(xb));
            if constexpr (DBG & 1) xv[m][j] = u32x2_t{0x3F803F80u + off_x, 0x3F803F80u};
            else xv[m][j] = *reinterpret_cast<const __attribute__((address_space(1))) u32x2_t*>(reinterpret_cast<global_cchar_t*>(xb) + off_x);
        }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        uint64_t wb = LOOP ? reinterpret_cast<uint64_t>(W) + (static_cast<uint64_t>(rb) * tiles + tile_of[j]) * TILE_BYTES
                           : reinterpret_cast<uint64_t>(w_base) + static_cast<uint64_t>(j) * nwk * TILE_BYTES;
        asm volatile("" : "+s"(wb));
        if constexpr (DBG & 32) {
#pragma unroll
            for (int q = 0; q < G; ++q) wv[j][q] = (off_w + 0x12345u * (q + 1)) * 0x9E3779B9u;
        } else {
            wv[j] = __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) wvec_t*>(reinterpret_cast<global_cchar_t*>(wb) + off_w));
        }
    }
    if constexpr (PAIR) {
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            uint64_t wb = reinterpret_cast<uint64_t>(W2) + (static_cast<uint64_t>(rb) * tiles + static_cast<uint32_t>(wave) + static_cast<uint64_t>(j) * nwk) * TILE_BYTES;
            asm volatile("" : "+s"(wb));
            wv[CPW + j] = __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) wvec_t*>(reinterpret_cast<global_cchar_t*>(wb) + off_w));
        }
    }
    if constexpr (LOOP) {
#pragma unroll
        for (int j = 0; j < CPW; ++j)
#pragma unroll
            for (int m = 0; m < MB; ++m) { xv[m][j][0] &= live[j]; xv[m][j][1] &= live[j]; }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    KMQ_TS(1);

    // ---- tables (first round) ---------------------------------------------------------------------------
    if (!LOOP || t0 == 0) {
        if constexpr (BITS == 2) {
            // the workgroup's pair table: wave w writes entries w, w + nwk, ...
            // (a loop that always runs once: a load whose only use sits behind a branch gets sunk into it)
            int e = wave;
            do {
                const uint32_t a = (e & 3) * 2, b = (e >> 2) * 2;
                const uint32_t sel = a | ((a + 1) << 8) | (b << 16) | ((b + 1) << 24);
                sm.lut[e * 64 + lane] = __builtin_amdgcn_perm(cb[1], cb[0], sel);
                if constexpr (PAIR) sm.lut[1024 + e * 64 + lane] = __builtin_amdgcn_perm(cb2[1], cb2[0], sel);
                e += nwk;
            } while (e < 16);
            KMQ_TS(2);
            __syncthreads();
        } else {
            // this wave's copy of the mask table; a wave reads back only what it wrote itself (LDS serves a
            // wave's instructions in order), so no barrier
            if (lane < 16) {
                u32x2_t m;
                m[0] = ((lane & 1u) ? 0x3F80u : 0u) | ((lane & 2u) ? 0x3F800000u : 0u);
                m[1] = ((lane & 4u) ? 0x3F80u : 0u) | ((lane & 8u) ? 0x3F800000u : 0u);
                *reinterpret_cast<u32x2_t*>(&sm.lut[wave * 64 + lane * 2]) = m;
            }
            KMQ_TS(2);
        }
    }
    if constexpr (BITS == 1) {
        // the closed form's sum of x, taken while the index words are still on their way: every pair of
        // the wave's tiles sits in exactly one lane
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            float s = LOOP ? sxl[m] : 0.f;
#pragma unroll
            for (int j = 0; j < CPW; ++j) {
                s = dot2_bf16(0x3F803F80u, xv[m][j][0], s);
                s = dot2_bf16(0x3F803F80u, xv[m][j][1], s);
            }
            if constexpr (LOOP) {
                sxl[m] = s;
            } else {
                s = group_sum<64>(s);
                if (lane == 63) sm.sx[m][wave] = s;
            }
        }
    }
    KMQ_TS(3);

    // ---- lookups and multiply-accumulate, four lookups ahead -----------------------------------------
    uint32_t ar[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ar[i] = BITS == 2 ? lut_base + lane * 4 : lut_base;
    // what the compiler itself has in flight on the LGKM counter must have landed before the
    // hand-counted pipeline starts
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    constexpr int NW = CPW * G;
    if constexpr (DBG & 16) {
        uint32_t t = 0;
#pragma unroll
        for (int j = 0; j < CPW; ++j)
#pragma unroll
            for (int q = 0; q < G; ++q) t ^= wv[j][q];
        acc[0][0] = __uint_as_float(t & 0x3FFFFFFFu) * __uint_as_float(xv[0][0][0] & 0x3FFFFFFFu);
    } else if constexpr (BITS == 2) {
        const uint32_t mask = 0x0Fu;
        uint32_t v[2][8];
        uint32_t ws[2];
        ws[0] = wv[0][0] >> 4;
#ifdef KMQ_TIMESTAMPS
        if (ts_on) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); KMQ_TS(4); asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
#endif
        issue4_pair<0>(wv[0][0], ws[0], ar, &v[0][0], mask);
        issue4_pair<1>(wv[0][0], ws[0], ar, &v[0][4], mask);
        // word n of the wave: slot n / 4 (tile j = slot % CPW of matrix slot / CPW), word n % 4 of the lane's chunk
        static_for<0, NMAT * NW>([&](auto ic) {
            constexpr int n = decltype(ic)::value;
            constexpr int slot = n / 4, q = n % 4, j = slot % CPW, mat = slot / CPW;
            if constexpr (n + 1 < NMAT * NW) {
                constexpr int slot1 = (n + 1) / 4, q1 = (n + 1) % 4, off1 = (slot1 / CPW) * 4096;
                ws[(n + 1) & 1] = wv[slot1][q1] >> 4;
                issue4_pair<0, off1>(wv[slot1][q1], ws[(n + 1) & 1], ar, &v[(n + 1) & 1][0], mask);
                dot8_pair<4, 8 * (q % 2)>(v[n & 1], xv[0][j][q / 2], acc[mat * MB][0], acc[mat * MB][1]);
#pragma unroll
                for (int m = 1; m < MB; ++m) dot8_pair<-1, 8 * (q % 2)>(v[n & 1], xv[m][j][q / 2], acc[m][0], acc[m][1]);
                issue4_pair<1, off1>(wv[slot1][q1], ws[(n + 1) & 1], ar, &v[(n + 1) & 1][4], mask);
            } else {
                dot8_pair<0, 8 * (q % 2)>(v[n & 1], xv[0][j][q / 2], acc[mat * MB][0], acc[mat * MB][1]);
#pragma unroll
                for (int m = 1; m < MB; ++m) dot8_pair<-1, 8 * (q % 2)>(v[n & 1], xv[m][j][q / 2], acc[m][0], acc[m][1]);
            }
        });
    } else {
        // a group is four nibbles (half a word, sixteen elements); group g of the wave: word g / 2, half g % 2
        const uint32_t mask = 0x78u;
        constexpr int NG = 2 * NW;
        u32x2_t vv[2][4];
        uint32_t wr[2];
        wr[0] = __builtin_amdgcn_alignbit(wv[0][0], wv[0][0], 4);
#ifdef KMQ_TIMESTAMPS
        if (ts_on) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); KMQ_TS(4); asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
#endif
        issue4_mask<0>(wv[0][0], wr[0], ar, vv[0], mask);
        // group g of the wave: word g / 2 (slot word / 2: tile j = slot % CPW of matrix slot / CPW), half g % 2
        static_for<0, NMAT * NG>([&](auto ic) {
            constexpr int g = decltype(ic)::value;
            constexpr int n = g / 2, h = g % 2, slot = n / 2, q = n % 2, j = slot % CPW, mat = slot / CPW;
            if constexpr (g + 1 < NMAT * NG) {
                constexpr int n1 = (g + 1) / 2, h1 = (g + 1) % 2, slot1 = n1 / 2, q1 = n1 % 2;
                if constexpr (h1 == 0) wr[n1 & 1] = __builtin_amdgcn_alignbit(wv[slot1][q1], wv[slot1][q1], 4);
                issue4_mask<h1>(wv[slot1][q1], wr[n1 & 1], ar, vv[(g + 1) & 1], mask);
                dot8_mask<4, 8 * q + 4 * h>(vv[g & 1], xv[0][j][0], xv[0][j][1], acc[mat * MB][0], acc[mat * MB][1]);
            } else {
                dot8_mask<0, 8 * q + 4 * h>(vv[g & 1], xv[0][j][0], xv[0][j][1], acc[mat * MB][0], acc[mat * MB][1]);
            }
#pragma unroll
            for (int m = 1; m < MB; ++m) dot8_mask<-1, 8 * q + 4 * h>(vv[g & 1], xv[m][j][0], xv[m][j][1], acc[m][0], acc[m][1]);
        });
    }
    t0 += CPW * nwk;
    } while (LOOP && t0 < tiles);
    if constexpr (LOOP && BITS == 1) {
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            const float s = group_sum<64>(sxl[m]);
            if (lane == 63) sm.sx[m][wave] = s;
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    KMQ_TS(5);

    // ---- K-reduction through LDS, fixed order ---------------------------------------------------------
#pragma unroll
    for (int m = 0; m < NMAT * MB; ++m) {
        settle(acc[m][0], acc[m][1]);
        sm.part[m][wave][lane] = acc[m][0] + acc[m][1];
    }
    __syncthreads();
    KMQ_TS(6);
    // wave m finishes batch column m: each lane adds its own column of partial sums over the waves, then the
    // four 16-lane rows (the four chunks of a tile) are added lane by lane with two half-swaps
    for (uint32_t m = wave; m < MB; m += nwk) {
        float res[NMAT];
#pragma unroll
        for (int mat = 0; mat < NMAT; ++mat) {
            float s = 0.f;
            for (uint32_t w = 0; w < nwk; ++w) s += sm.part[mat * MB + m][w][lane];
            const auto h16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(s), __float_as_uint(s), false, false);
            s = __uint_as_float(h16[0]) + __uint_as_float(h16[1]);                 // rows 0+1 | 0+1 | 2+3 | 2+3
            const auto h32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(s), false, false);
            s = __uint_as_float(h32[0]) + __uint_as_float(h32[1]);                 // all four, in every lane
            if constexpr (BITS == 1) {
                float sx = 0.f;
                for (uint32_t w = 0; w < nwk; ++w) sx += sm.sx[m][w];
                // (every lane loaded the centroids of row lane % 16 of the block)
                const uint32_t c01 = mat == 0 ? cb[0] : cb2[0];
                const float c0 = bf16_to_f32(c01 & 0xFFFFu), c1 = bf16_to_f32(c01 >> 16);
                s = fmaf(c1 - c0, s, c0 * sx);
            }
            res[mat] = s;
        }
        float s = res[0];
        if constexpr (PAIR) s = res[0] / (1.f + __expf(-res[0])) * res[NMAT - 1];   // silu(gate) * up
        const uint32_t rr = lane & 15;
        const int64_t n0 = static_cast<int64_t>(rb) * 16 + rr;
        const uint32_t mine = f32_to_bf16(s);
        // even lanes store two rows at once where the pair is whole and aligned
        const uint32_t other = __builtin_amdgcn_update_dpp(0, static_cast<int>(mine), 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
        uint16_t* yp = Y + static_cast<int64_t>(m) * N + n0;
        const bool pairable = (reinterpret_cast<uintptr_t>(yp) & 3u) == 0 && n0 + 1 < N;
        if (lane < 16) {
            if constexpr (DBG & 64) {
                if (s == 1.2345e-30f) *yp = 1;
            } else if ((rr & 1) == 0) {
                if (pairable) *reinterpret_cast<uint32_t*>(yp) = mine | (other << 16);
                else if (n0 < N) *yp = static_cast<uint16_t>(mine);
            } else {
                // the even neighbour could not pair (misaligned y or last row): store alone
                const bool neighbour_pairs = (reinterpret_cast<uintptr_t>(yp - 1) & 3u) == 0 && n0 < N;
                if (!neighbour_pairs && n0 < N) *yp = static_cast<uint16_t>(mine);
            }
        }
    }
    KMQ_TS(7);
}

#ifdef KMQ_TIMESTAMPS
extern "C" int kmq_debug_rowlane_timestamps(unsigned long long* host, size_t count) {
    return static_cast<int>(hipMemcpyFromSymbol(host, HIP_SYMBOL(kmq_rowlane_ts), count * sizeof(unsigned long long)));
}
#endif

// ---- launch ----------------------------------------------------------------------------------------

struct RowlaneShape { int cpw, nwk; bool loop; };

// K / 256 tiles = cpw * nwk with nwk <= 16 waves; many thin waves first (occupancy hides the LDS latency
// of the lookups better than a deeper per-wave queue, which the 4-bit LGKM counter caps anyway).
// A tile count with no such factorisation (17, 19, 34, 43, ... or beyond 128) takes the kernel that
// walks K in rounds of 2 * nwk tiles -- and so does every 2-bit row of more than 32 tiles: three and
// more 16-byte index loads per lane in flight at once measured slower than rounds of two (4096 x 14336:
// 6.9 us with four tiles per wave, 6.1 us in two rounds; 8192 x 28672: 19.8 against 17.3 us; fetching a
// round ahead: 6.7 us).  1-bit rows (8-byte loads) keep the instances with everything in flight
// (4096 x 14336: 5.1 against 5.5 us in rounds).
static bool rowlane_shape(int64_t K, int bits, RowlaneShape& s, bool pair = false) {
    const int64_t tiles = K / 256;
    static const int cpws[] = {2, 1, 3, 4, 6, 7, 8};
#ifdef KMQ_TUNING
    static const char* const force = std::getenv("KMQ_RL_CPW");     // sweeps only: builds with -DKMQ_TUNING
    if (force) {
        const int c = std::atoi(force);
        if (c >= 1 && tiles % c == 0 && tiles / c <= 16) { s = {c, static_cast<int>(tiles / c), false}; return true; }
        if (c == 0 && tiles >= 1) { const int64_t r = (tiles + 31) / 32; s = {2, static_cast<int>((tiles + 2 * r - 1) / (2 * r)), true}; return true; }    // KMQ_RL_CPW=0: the round loop
    }
#endif
    // 1-bit rows of 12 or 24 tiles (3072, 6144 columns): three tiles per wave leave 4 or 8 waves, one or two per SIMD
    // from every workgroup, where two tiles per wave leave 6 or 12 (9216 x 3072: 3.90 against 4.00 us, batch 4: 6.5
    // against 7.0; 8192 x 6144: 4.24 against 4.42)
    if (bits == 1 && !pair && tiles % 3 == 0 && (tiles / 3) % 4 == 0 && tiles / 3 <= 16) { s = {3, static_cast<int>(tiles / 3), false}; return true; }
    for (int c : cpws) {
        if (bits == 2 && c > 2 && !pair) continue;       // (the fused pair has no round loop: it keeps the instances)
        if (tiles % c == 0 && tiles / c <= 16 && tiles / c >= 1) { s = {c, static_cast<int>(tiles / c), false}; return true; }
    }
    if (tiles < 1) return false;
    // rounds of at most 32 tiles (16 waves x 2), the waves spread evenly over the rounds
    const int64_t rounds = (tiles + 31) / 32;
    s = {2, static_cast<int>((tiles + 2 * rounds - 1) / (2 * rounds)), true};
    return true;
}

bool rowlane_has_kernel(int64_t K, int bits, int M) {
    RowlaneShape s;
    return rowlane_valid(bits, K) && M >= 1 && M <= KMQ_MAX_BATCH && rowlane_shape(K, bits, s);
}

bool rowlane_loops(int64_t K, int bits) {
    RowlaneShape s;
    return rowlane_shape(K, bits, s) && s.loop;
}

template <int BITS>
static hipError_t launch_rowlane_bits(const GemmArgs& a, const RowlaneShape& s, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>((a.N + 15) / 16)), block(64 * s.nwk);
#define KMQ_RL_LAUNCH(CPW, MB, WPE) \
    hipLaunchKernelGGL((gemv_rowlane_kernel<BITS, CPW, MB, WPE>), grid, block, 0, st, a.W, a.codebook, a.X, a.Y, a.N, a.K)
#define KMQ_RL_CPW(CPW, WPE) \
    switch (a.M) { case 1: KMQ_RL_LAUNCH(CPW, 1, WPE); break; case 2: KMQ_RL_LAUNCH(CPW, 2, WPE); break; \
                   case 3: KMQ_RL_LAUNCH(CPW, 3, WPE); break; default: KMQ_RL_LAUNCH(CPW, 4, WPE); break; }
#ifdef KMQ_TUNING
    static const char* const dbg_env = std::getenv("KMQ_RL_DBG");
    const int dbg = dbg_env ? std::atoi(dbg_env) : 0;
    if (dbg && s.cpw == 2 && a.M == 1) {
#define KMQ_RL_DBG_CASE(D) case D: hipLaunchKernelGGL((gemv_rowlane_kernel<BITS, 2, 1, 8, false, D>), grid, block, 0, st, a.W, a.codebook, a.X, a.Y, a.N, a.K); return hipGetLastError();
        switch (dbg) {
            KMQ_RL_DBG_CASE(1) KMQ_RL_DBG_CASE(2) KMQ_RL_DBG_CASE(3) KMQ_RL_DBG_CASE(16) KMQ_RL_DBG_CASE(32) KMQ_RL_DBG_CASE(19)
            KMQ_RL_DBG_CASE(35) KMQ_RL_DBG_CASE(64) KMQ_RL_DBG_CASE(80)
            default: break;
        }
#undef KMQ_RL_DBG_CASE
    }
#endif
    if (s.loop) {
#define KMQ_RL_LOOP(MB) hipLaunchKernelGGL((gemv_rowlane_kernel<BITS, 2, MB, 8, true>), grid, block, 0, st, a.W, a.codebook, a.X, a.Y, a.N, a.K)
        switch (a.M) { case 1: KMQ_RL_LOOP(1); break; case 2: KMQ_RL_LOOP(2); break; case 3: KMQ_RL_LOOP(3); break; default: KMQ_RL_LOOP(4); break; }
#undef KMQ_RL_LOOP
        return hipGetLastError();
    }
    if (s.cpw == 1) { KMQ_RL_CPW(1, 8); }
    else if (s.cpw == 2) { KMQ_RL_CPW(2, 8); }
    else if constexpr (BITS == 1) {                 // (2-bit rows of more than two tiles per wave walk K in rounds)
        switch (s.cpw) {
            case 3: KMQ_RL_CPW(3, 6); break;
            case 4: KMQ_RL_CPW(4, 4); break;
            case 6: KMQ_RL_CPW(6, 4); break;
            case 7: KMQ_RL_CPW(7, 4); break;
            default: KMQ_RL_CPW(8, 4); break;
        }
    } else {
        return hipErrorInvalidValue;
    }
#undef KMQ_RL_CPW
#undef KMQ_RL_LAUNCH
    return hipGetLastError();
}

// The fused gate / up / SwiGLU call: shapes with at most four tiles per wave (a wave then holds eight).
bool rowlane_pair_has_kernel(int64_t K, int bits) {
    RowlaneShape s;
    return rowlane_valid(bits, K) && rowlane_shape(K, bits, s, true) && !s.loop && s.cpw <= 4;
}

template <int BITS>
static hipError_t launch_rowlane_pair_bits(const GemmArgs& a, const RowlaneShape& s, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>((a.N + 15) / 16)), block(64 * s.nwk);
#define KMQ_RL_PAIR(CPW, WPE) \
    hipLaunchKernelGGL((gemv_rowlane_kernel<BITS, CPW, 1, WPE, false, 0, true>), grid, block, 0, st, a.W, a.codebook, a.X, a.Y, a.N, a.K, a.W2, a.codebook2)
    switch (s.cpw) {
        case 1: KMQ_RL_PAIR(1, 8); break;
        case 2: KMQ_RL_PAIR(2, 8); break;
        case 3: KMQ_RL_PAIR(3, 4); break;
        default: KMQ_RL_PAIR(4, 4); break;
    }
#undef KMQ_RL_PAIR
    return hipGetLastError();
}

hipError_t launch_rowlane_pair(const GemmArgs& a, hipStream_t st) {
    RowlaneShape s;
    if (!rowlane_shape(a.K, a.bits, s, true) || s.loop || s.cpw > 4 || !a.W2 || !a.codebook2) return hipErrorInvalidValue;
    return a.bits == 1 ? launch_rowlane_pair_bits<1>(a, s, st) : launch_rowlane_pair_bits<2>(a, s, st);
}

// A launch decodes every weight once for up to four batch columns (the registers that hold the
// activation pairs and the sums set the limit); wider batches take one launch per four columns.
hipError_t launch_rowlane(const GemmArgs& a, hipStream_t st) {
    RowlaneShape s;
    if (!rowlane_shape(a.K, a.bits, s)) return hipErrorInvalidValue;
    for (int m0 = 0; m0 < a.M; m0 += 4) {
        GemmArgs b = a;
        b.M = a.M - m0 < 4 ? a.M - m0 : 4;
        b.X = a.X + static_cast<int64_t>(m0) * a.K;
        b.Y = a.Y + static_cast<int64_t>(m0) * a.N;
        const hipError_t e = a.bits == 1 ? launch_rowlane_bits<1>(b, s, st) : launch_rowlane_bits<2>(b, s, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace kmq
