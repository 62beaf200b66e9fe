// Batch 1..4 kernels on the row-lane layout (KMQ_LAYOUT_ROWLANE, include/kmq.h): y = W x with
// w = codebook lookup (paper App. E, "Kernel implementations"), built for the regime the paper
// calls memory-bound (App. D) on a machine where the decode, not the memory, is the longer side.
//
// Work split.  A workgroup owns one block of 16 rows; its waves split K.  A wave-wide 16-byte
// load is one TILE: lane (kp, r) = (lane / 16, lane % 16) gets chunk kp (of 4) of row r, so the
// 16 lanes of a DPP row hold 16 different rows over the SAME 64 (2-bit) or 128 (1-bit) columns.
//
// Activations never pass through LDS and are never duplicated per row: the lanes of DPP row kp
// hold the bf16 pairs of chunk kp, one or two pairs per register, and the multiply-accumulate
// reads the pair it needs from its row of lanes with the DPP broadcast of v_dot2c_f32_bf16
// (row_newbcast:j: every lane of a 16-lane row sees lane j's register).  The layout's bit order
// is chosen so that the j-th lookup of a register pairs with lane j.
//
// Weights.  2-bit: a nibble (two indices) addresses a 16-entry table of bf16 PAIRS, one column
// per lane ([entry][lane], 4 KB per workgroup: a wave's 64 lookups fall into 64 different
// banks-times-lanes, never colliding); the address is one SDWA byte-AND that drops the nibble
// into byte 1 of a register holding lane*4.  1-bit: a nibble addresses a row-independent table
// of four bf16 {0,1} masks; the kernel accumulates S1 = sum_{idx=1} x and finishes with the
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

// Four lookups of the 2-bit pair table: nibbles of bytes B0 and B0 + 1 of `w` (even nibbles)
// and of `ws` = w >> 4 (odd nibbles).  `a` holds lane*4 in byte 0; byte 1 receives the nibble,
// i.e. the address is entry*256 + lane*4.  At most 12 lookups are kept in flight (the LGKM
// counter has 4 bits).
#define KMQ_RL_SDWA1(dst, src, byte) \
    "v_and_b32_sdwa " dst ", " src ", %10 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_" byte " src1_sel:DWORD\n\t"
template <int H>
__device__ __forceinline__ void issue4_pair(uint32_t w, uint32_t ws, uint32_t (&a)[4], uint32_t* v, uint32_t mask) {
    if constexpr (H == 0) {
        asm volatile(
            KMQ_RL_SDWA1("%4", "%8", "0") KMQ_RL_SDWA1("%5", "%9", "0") KMQ_RL_SDWA1("%6", "%8", "1") KMQ_RL_SDWA1("%7", "%9", "1")
            "ds_read_b32 %0, %4\n\tds_read_b32 %1, %5\n\tds_read_b32 %2, %6\n\tds_read_b32 %3, %7"
            : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(w), "v"(ws), "v"(mask));
    } else {
        asm volatile(
            KMQ_RL_SDWA1("%4", "%8", "2") KMQ_RL_SDWA1("%5", "%9", "2") KMQ_RL_SDWA1("%6", "%8", "3") KMQ_RL_SDWA1("%7", "%9", "3")
            "ds_read_b32 %0, %4\n\tds_read_b32 %1, %5\n\tds_read_b32 %2, %6\n\tds_read_b32 %3, %7"
            : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
            : "v"(w), "v"(ws), "v"(mask));
    }
}
#undef KMQ_RL_SDWA1

// Eight multiply-accumulates of looked-up weight pairs against the activation pairs that lanes
// BC .. BC + 7 of this lane's DPP row hold in `x`.  PENDING >= 0: first wait until at most that
// many LDS reads are outstanding.
#define KMQ_RL_DOT(acc, vv, j) "v_dot2c_f32_bf16_dpp " acc ", %10, " vv " row_newbcast:" j " row_mask:0xf bank_mask:0xf\n\t"
template <int PENDING, int BC>
__device__ __forceinline__ void dot8(const uint32_t* v, uint32_t x, float& a0, float& a1) {
    static_assert(BC == 0 || BC == 8, "half of a 16-lane row");
    if constexpr (PENDING >= 0) asm volatile("s_waitcnt lgkmcnt(%c0)" : : "n"(PENDING) : "memory");
    if constexpr (BC == 0) {
        asm volatile(
            KMQ_RL_DOT("%0", "%2", "0") KMQ_RL_DOT("%1", "%3", "1") KMQ_RL_DOT("%0", "%4", "2") KMQ_RL_DOT("%1", "%5", "3")
            KMQ_RL_DOT("%0", "%6", "4") KMQ_RL_DOT("%1", "%7", "5") KMQ_RL_DOT("%0", "%8", "6") KMQ_RL_DOT("%1", "%9", "7")
            : "+v"(a0), "+v"(a1)
            : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]), "v"(x));
    } else {
        asm volatile(
            KMQ_RL_DOT("%0", "%2", "8") KMQ_RL_DOT("%1", "%3", "9") KMQ_RL_DOT("%0", "%4", "10") KMQ_RL_DOT("%1", "%5", "11")
            KMQ_RL_DOT("%0", "%6", "12") KMQ_RL_DOT("%1", "%7", "13") KMQ_RL_DOT("%0", "%8", "14") KMQ_RL_DOT("%1", "%9", "15")
            : "+v"(a0), "+v"(a1)
            : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]), "v"(x));
    }
}
#undef KMQ_RL_DOT

// A dot instruction's result may feed the next dot's accumulator at once; any other vector
// instruction reading it needs three wait states, which the compiler cannot count across an
// asm block.
__device__ __forceinline__ void settle(float& a0, float& a1) { asm volatile("s_nop 2" : "+v"(a0), "+v"(a1)); }

}  // namespace rowlane

#ifdef KMQ_TIMESTAMPS
// Instrumented builds only: per-wave time stamps (100 MHz wall clock), [workgroup][wave][8].
__device__ unsigned long long kmq_rowlane_ts[1024 * 16 * 8];
#define KMQ_TS(i) do { if (ts_on) { const unsigned long long t_ = __builtin_amdgcn_s_memrealtime(); \
    if (lane == 0) kmq_rowlane_ts[(blockIdx.x * 16 + wave) * 8 + (i)] = t_; } } while (0)
#else
#define KMQ_TS(i) do { } while (0)
#endif

// CPW tiles per wave, MB batch columns, WPE waves per SIMD the register budget is sized for.
// K = 256 * CPW * (waves per workgroup); the grid is one workgroup per 16-row block.
template <int CPW, int MB, int WPE, int DBG = 0>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemv_rowlane_b2_kernel(const uint32_t* __restrict__ W, const uint16_t* __restrict__ codebook,
                            const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int64_t N, int64_t K) {
    using namespace rowlane;
    struct alignas(256) Smem {
        uint32_t lut[16 * 64];          // [entry][lane]: bf16 pair (centroid of the even element, of the odd element)
        float part[MB][16][64];         // [column][wave][lane] partial sums
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
    if constexpr (DBG & 8) __builtin_amdgcn_s_setprio(3);

    // ---- loads, small operands first (a wave's loads return in issue order) ----------------
    // byte offsets inside a tile: 16 per lane of W, 8 per lane of x (chunk kp starts 128 bytes after
    // chunk kp - 1, so lane kp*16 + r reads at lane*8), 8 per row of the codebook
    const uint32_t off_w = lane * 16, off_x = lane * 8;
    const int64_t rows_left = N - static_cast<int64_t>(rb) * 16;
    const uint32_t last_c = __builtin_amdgcn_readfirstlane(rows_left < 16 ? static_cast<uint32_t>(rows_left) * 8 - 8 : 120u);
    uint32_t off_c = off_x & 0x78u;
    off_c = off_c < last_c ? off_c : last_c;                                   // rows past N read the last row
    const char* const cb_base = reinterpret_cast<const char*>(codebook) + static_cast<uint64_t>(rb) * 128;
    const char* const x_base = reinterpret_cast<const char*>(X) + static_cast<uint32_t>(wave) * 512;
    const char* const w_base = reinterpret_cast<const char*>(W) + (static_cast<uint64_t>(rb) * tiles + static_cast<uint32_t>(wave)) * 1024;
    typedef u32x2_t __attribute__((aligned(4))) u32x2_a4_t;
    u32x4_t wv[CPW];
    if constexpr (DBG & 4) {
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            uint64_t wb = reinterpret_cast<uint64_t>(w_base) + static_cast<uint64_t>(j) * nwk * 1024;
            asm volatile("" : "+s"(wb));
            wv[j] = __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) u32x4_t*>(reinterpret_cast<global_cchar_t*>(wb) + off_w));
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    }
    u32x2_t cb;
    if constexpr (DBG & 2) cb = u32x2_t{0x3C003B00u + lane, 0x3E003D00u};
    else cb = *reinterpret_cast<const u32x2_a4_t*>(cb_base + off_c);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);      // (left alone, the compiler sinks this load below the index loads)
    u32x2_t xv[MB][CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
#pragma unroll
        for (int m = 0; m < MB; ++m)
        {
            // (the tile's base stays on the scalar side: pinned, or the sum is re-associated into vector adds)
            uint64_t xb = reinterpret_cast<uint64_t>(x_base) + static_cast<uint64_t>(m) * K * 2 + static_cast<uint64_t>(j) * nwk * 512;
            asm volatile("" : "+s"(xb));
            if constexpr (DBG & 1) xv[m][j] = u32x2_t{0x3F803F80u + off_x, 0x3F803F80u};
            else xv[m][j] = *reinterpret_cast<const __attribute__((address_space(1))) u32x2_t*>(reinterpret_cast<global_cchar_t*>(xb) + off_x);
        }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    if constexpr ((DBG & 4) == 0) {
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            uint64_t wb = reinterpret_cast<uint64_t>(w_base) + static_cast<uint64_t>(j) * nwk * 1024;
            asm volatile("" : "+s"(wb));
            if constexpr (DBG & 32) wv[j] = u32x4_t{off_w * 0x9E3779B9u, off_x * 0x85EBCA6Bu, off_w + 0x12345u, off_x ^ 0xABCDEFu};
            else wv[j] = __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) u32x4_t*>(reinterpret_cast<global_cchar_t*>(wb) + off_w));
        }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (DBG & 8) __builtin_amdgcn_s_setprio(0);

    KMQ_TS(1);
    // ---- the workgroup's pair table: wave w writes entries w, w + nwk, ... --------------------
    // (a loop that always runs once: a load whose only use sits behind a branch gets sunk into it)
    int e = wave;
    do {
        const uint32_t a = (e & 3) * 2, b = (e >> 2) * 2;
        const uint32_t sel = a | ((a + 1) << 8) | (b << 16) | ((b + 1) << 24);
        sm.lut[e * 64 + lane] = __builtin_amdgcn_perm(cb[1], cb[0], sel);
        e += nwk;
    } while (e < 16);
    KMQ_TS(2);
    __syncthreads();
    KMQ_TS(3);

    // ---- lookups and multiply-accumulate, one word ahead -------------------------------------------
    const uint32_t lut_base = static_cast<uint32_t>(reinterpret_cast<size_t>((lds_cu32_t*)(&sm.lut[0])));
    uint32_t ar[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ar[i] = lut_base + lane * 4;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const uint32_t mask = 0x0Fu;
    float acc[MB][2];
#pragma unroll
    for (int m = 0; m < MB; ++m) acc[m][0] = acc[m][1] = 0.f;
    constexpr int NW = CPW * 4;
    uint32_t v[2][8];
    uint32_t ws[2];
    if constexpr (DBG & 16) {
        uint32_t t = 0;
#pragma unroll
        for (int j = 0; j < CPW; ++j) t ^= wv[j][0] ^ wv[j][1] ^ wv[j][2] ^ wv[j][3];
        acc[0][0] = __uint_as_float(t & 0x3FFFFFFFu) * __uint_as_float(xv[0][0][0] & 0x3FFFFFFFu);
    } else {
    ws[0] = wv[0][0] >> 4;
#ifdef KMQ_TIMESTAMPS
    if (ts_on) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); KMQ_TS(4); asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
#endif
    issue4_pair<0>(wv[0][0], ws[0], ar, &v[0][0], mask);
    issue4_pair<1>(wv[0][0], ws[0], ar, &v[0][4], mask);
    static_for<0, NW>([&](auto ic) {
        constexpr int n = decltype(ic)::value;
        constexpr int j = n / 4, q = n % 4;
        if constexpr (n + 1 < NW) {
            constexpr int j1 = (n + 1) / 4, q1 = (n + 1) % 4;
            ws[(n + 1) & 1] = wv[j1][q1] >> 4;
            issue4_pair<0>(wv[j1][q1], ws[(n + 1) & 1], ar, &v[(n + 1) & 1][0], mask);
            dot8<4, 8 * (q % 2)>(v[n & 1], xv[0][j][q / 2], acc[0][0], acc[0][1]);
#pragma unroll
            for (int m = 1; m < MB; ++m) dot8<-1, 8 * (q % 2)>(v[n & 1], xv[m][j][q / 2], acc[m][0], acc[m][1]);
            issue4_pair<1>(wv[j1][q1], ws[(n + 1) & 1], ar, &v[(n + 1) & 1][4], mask);
        } else {
            dot8<0, 8 * (q % 2)>(v[n & 1], xv[0][j][q / 2], acc[0][0], acc[0][1]);
#pragma unroll
            for (int m = 1; m < MB; ++m) dot8<-1, 8 * (q % 2)>(v[n & 1], xv[m][j][q / 2], acc[m][0], acc[m][1]);
        }
    });
    }
    __builtin_amdgcn_sched_barrier(0);
    KMQ_TS(5);

    // ---- K-reduction through LDS, fixed order ---------------------------------------------------------
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        settle(acc[m][0], acc[m][1]);
        sm.part[m][wave][lane] = acc[m][0] + acc[m][1];
    }
    __syncthreads();
    KMQ_TS(6);
    if (threadIdx.x < 16 * MB) {
        const int m = threadIdx.x >> 4, rr = threadIdx.x & 15;
        float s = 0.f;
        for (int w = 0; w < nwk; ++w) {
#pragma unroll
            for (int c = 0; c < 4; ++c) s += sm.part[m][w][c * 16 + rr];
        }
        const int64_t n0 = static_cast<int64_t>(rb) * 16 + rr;
        const uint32_t mine = f32_to_bf16(s);
        // even lanes store two rows at once where the pair is whole and aligned
        const uint32_t other = __builtin_amdgcn_update_dpp(0, static_cast<int>(mine), 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
        uint16_t* yp = Y + static_cast<int64_t>(m) * N + n0;
        const bool pairable = (reinterpret_cast<uintptr_t>(yp) & 3u) == 0 && n0 + 1 < N;
        if ((rr & 1) == 0) {
            if (pairable) *reinterpret_cast<uint32_t*>(yp) = mine | (other << 16);
            else if (n0 < N) *yp = static_cast<uint16_t>(mine);
        } else {
            // the even neighbour could not pair (misaligned y or last row): store alone
            const bool neighbour_pairs = (reinterpret_cast<uintptr_t>(yp - 1) & 3u) == 0 && n0 < N;
            if (!neighbour_pairs && n0 < N) *yp = static_cast<uint16_t>(mine);
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



struct RowlaneShape { int cpw, nwk; };

// tiles = cpw * nwk with nwk <= 16 waves and cpw in {1, 2, 4, 7, 8}: prefer many thin waves
static bool rowlane_shape(int64_t K, RowlaneShape& s) {
    const int64_t tiles = K / 256;
    static const int cpws[] = {2, 1, 4, 3, 7, 8};
#ifdef KMQ_TUNING
    static const char* const force = std::getenv("KMQ_RL_CPW");     // sweeps only: builds with -DKMQ_TUNING
    if (force) {
        const int c = std::atoi(force);
        if (c >= 1 && tiles % c == 0 && tiles / c <= 16) { s = {c, static_cast<int>(tiles / c)}; return true; }
    }
#endif
    for (int c : cpws) {
        if (tiles % c == 0 && tiles / c <= 16 && tiles / c >= 1) { s = {c, static_cast<int>(tiles / c)}; return true; }
    }
    return false;
}

bool rowlane_has_kernel(int64_t K, int bits, int M) {
    RowlaneShape s;
    return bits == 2 && M >= 1 && M <= 4 && K % 256 == 0 && rowlane_shape(K, s);
}

hipError_t launch_rowlane(const GemmArgs& a, hipStream_t st) {
    RowlaneShape s;
    if (!rowlane_shape(a.K, s)) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>((a.N + 15) / 16)), block(64 * s.nwk);
#define KMQ_RL_LAUNCH(CPW, MB, WPE) \
    hipLaunchKernelGGL((gemv_rowlane_b2_kernel<CPW, MB, WPE>), grid, block, 0, st, a.W, a.codebook, a.X, a.Y, a.N, a.K)
#define KMQ_RL_CPW(CPW, WPE) \
    switch (a.M) { case 1: KMQ_RL_LAUNCH(CPW, 1, WPE); break; case 2: KMQ_RL_LAUNCH(CPW, 2, WPE); break; \
                   case 3: KMQ_RL_LAUNCH(CPW, 3, WPE); break; default: KMQ_RL_LAUNCH(CPW, 4, WPE); break; }
#ifdef KMQ_TUNING
    static const char* const dbg_env = std::getenv("KMQ_RL_DBG");
    const int dbg = dbg_env ? std::atoi(dbg_env) : 0;
    if (dbg && s.cpw == 2 && a.M == 1) {
#define KMQ_RL_DBG_CASE(D) case D: hipLaunchKernelGGL((gemv_rowlane_b2_kernel<2, 1, 8, D>), grid, block, 0, st, a.W, a.codebook, a.X, a.Y, a.N, a.K); return hipGetLastError();
        switch (dbg) {
            KMQ_RL_DBG_CASE(1) KMQ_RL_DBG_CASE(2) KMQ_RL_DBG_CASE(3) KMQ_RL_DBG_CASE(4) KMQ_RL_DBG_CASE(8) KMQ_RL_DBG_CASE(12)
            KMQ_RL_DBG_CASE(16) KMQ_RL_DBG_CASE(32) KMQ_RL_DBG_CASE(19) KMQ_RL_DBG_CASE(35)
            default: break;
        }
#undef KMQ_RL_DBG_CASE
    }
#endif
    switch (s.cpw) {
        case 1: KMQ_RL_CPW(1, 8); break;
        case 2: KMQ_RL_CPW(2, 8); break;
        case 3: KMQ_RL_CPW(3, 6); break;
        case 4: KMQ_RL_CPW(4, 4); break;
        case 7: KMQ_RL_CPW(7, 4); break;
        default: KMQ_RL_CPW(8, 4); break;
    }
#undef KMQ_RL_CPW
#undef KMQ_RL_LAUNCH
    return hipGetLastError();
}

}  // namespace kmq
