// C-ABI entry points of the device path: argument checks, launch-shape
// heuristic, dispatch.  Contract: include/kmq.h.
#include <cstdlib>
#include <hip/hip_runtime.h>

#include "kmq.h"
#include "kmq_internal.h"
#include "kmq_launch.h"

namespace kmq {

// On the canonical layout a batch above 1 runs the batch-1 table kernel, where the shape has one, over a
// grid of (row group, column) workgroups in ONE launch: the workgroups that share rows of W sit next to
// each other on one XCD, so W still comes from memory once and the other columns find it in that L2 (the
// tiled layout with its matrix-core kernel remains the fastest route for batch > 1: it also decodes each
// weight once).  Measured (us), every further column costs N*K / r with r = 20, 19, 14, 9.5 million
// weights per us at 1, 2, 3, 4 bits -- decode time, every column looks every weight up again -- against
// N*K / 9 for every column of the shape-agnostic kernel, which also starts later (about 5 us against 2.6
// + bytes / 3.3e6 for the first column): the table kernel wins at every batch.  Table / shape-agnostic:
// 9216x3072 1-bit, batch 4: 8.9 / 21.7; 14336x4096 2-bit, batch 16: 50.6 / 121; 8192x8192 block-scaled
// 4-bit, batch 16: 111 / 237; 4096x4096 4-bit, batch 4: 10.0 / 12.8.  (Builds with -DKMQ_TUNING
// read a cap on the batch from KMQ_PER_COLUMN_MAX in the environment, for sweeps.)
static bool per_column_faster(int M) {
#ifdef KMQ_TUNING
    static const char* const v = std::getenv("KMQ_PER_COLUMN_MAX");
    static const int cap = v ? std::atoi(v) : KMQ_MAX_BATCH;
#else
    constexpr int cap = KMQ_MAX_BATCH;
#endif
    return M >= 2 && M <= cap;
}

// Launch-shape heuristic (the paper autotunes chunk shapes per problem, App. E
// "Kernel implementations"; here the choice is a static function of the shape).
Plan make_plan(int64_t N, int64_t K, int bits, int M, int layout, bool scaled) {
    Plan p{kVariantInvalid, -1, 0, "invalid"};
    if (!bits_valid(bits) || !dims_valid(N, K) || M < 1 || M > KMQ_MAX_BATCH) return p;
    if (layout != KMQ_LAYOUT_CANONICAL && layout != KMQ_LAYOUT_TILED && layout != KMQ_LAYOUT_ROWLANE) return p;
    if (layout == KMQ_LAYOUT_ROWLANE) {
        if (scaled || !rowlane_valid(bits, K) || !rowlane_has_kernel(K, bits, M)) return p;
        static const char* const names[2][2] = {{"rowlane_b1", "rowlane_b2"}, {"rowlane_loop_b1", "rowlane_loop_b2"}};
        return Plan{kVariantRowlane, -1, 0, names[rowlane_loops(K, bits) ? 1 : 0][bits - 1]};
    }
    if (scaled) {
        if (K % KMQ_BLOCK != 0) return p;
        if (layout == KMQ_LAYOUT_TILED) {
            // matrix-core kernel; its LDS holds the scales of at most 256 blocks of K per row
            if (!tiled_valid(bits, K) || K > 256 * KMQ_BLOCK) return p;
            static const char* const names[4] = {"mfma_sc_b1", "mfma_sc_b2", "mfma_sc_b3", "mfma_sc_b4"};
            return Plan{kVariantMfma, -1, 0, names[bits - 1]};
        }
        if (M == 1 || per_column_faster(M)) {
            const int l = lut_find(N, K, bits, layout, true);
            if (l >= 0) return Plan{M == 1 ? kVariantLut : kVariantPerColumn, l, 0, lut_name(l)};
        }
        return Plan{kVariantBlockGeneric, -1, 0, "blockscaled_generic"};
    }
    if (layout == KMQ_LAYOUT_TILED && !tiled_valid(bits, K)) return p;
    if (layout == KMQ_LAYOUT_TILED) {
        static const char* const names[4] = {"mfma_b1", "mfma_b2", "mfma_b3", "mfma_b4"};
        if (mfma_kslice_has_kernel(N, K, bits)) return Plan{kVariantMfma, -1, 0, bits == 2 ? "mfma_kslice_b2" : "mfma_kslice_b3"};
        return Plan{kVariantMfma, -1, 0, names[bits - 1]};
    }
    bool use_loop = true, use_table = true;
#ifdef KMQ_TUNING
    static const char* const loop_env = std::getenv("KMQ_LOOP");      // sweeps only: 0 = never, 2 = instead of the specialised kernels
    if (loop_env) { use_loop = loop_env[0] != '0'; use_table = loop_env[0] != '2'; }
#endif
    if (use_table && (M == 1 || per_column_faster(M))) {
        const int l = lut_find(N, K, bits, layout);
        if (l >= 0) return Plan{M == 1 ? kVariantLut : kVariantPerColumn, l, 0, lut_name(l)};
    }
    const int slices = generic_splitk_slices(N, K, layout);
    if (slices > 1)
        return Plan{kVariantGeneric, slices, static_cast<size_t>(slices) * M * N * sizeof(float), "generic_splitk"};
    if (use_loop && (M == 1 || per_column_faster(M)) && lut_loop_has_kernel(N, K, bits, layout))
        return Plan{kVariantLutLoop, -1, 0, lut_loop_name(bits)};
    return Plan{kVariantGeneric, -1, 0, "generic"};
}

// Text of the last HIP error a launch reported on this thread ("" if none).
static thread_local const char* g_last_hip_error = "";

static kmq_status hip_status(hipError_t e) {
    if (e == hipSuccess) return KMQ_OK;
    g_last_hip_error = hipGetErrorString(e);
    return KMQ_ERR_HIP;
}

static bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// library_scratch: the caller brings no workspace; a plan that needs one takes this GPU's share of the
// library's own scratch array (kmq_gemm_smallbatch_noalloc), up to its fixed size.
static kmq_status check_and_run(const GemmArgs& a_in, void* stream, bool library_scratch = false) {
    GemmArgs a = a_in;
    if (!a.W || !a.codebook || !a.X || !a.Y) return KMQ_ERR_NULL;
    if (!bits_valid(a.bits)) return KMQ_ERR_BITS;
    if (!dims_valid(a.N, a.K) || a.M < 1 || a.M > KMQ_MAX_BATCH) return KMQ_ERR_SHAPE;
    if (a.layout != KMQ_LAYOUT_CANONICAL && a.layout != KMQ_LAYOUT_TILED && a.layout != KMQ_LAYOUT_ROWLANE) return KMQ_ERR_LAYOUT;
    if (a.layout == KMQ_LAYOUT_TILED && !tiled_valid(a.bits, a.K)) return KMQ_ERR_LAYOUT;
    if (a.layout == KMQ_LAYOUT_ROWLANE && (!rowlane_valid(a.bits, a.K) || a.scales)) return KMQ_ERR_LAYOUT;
    if (!aligned(a.W, 16) || !aligned(a.X, 16) || !aligned(a.codebook, 4) || !aligned(a.Y, 2)) return KMQ_ERR_ALIGN;
    const bool scaled = a.scales != nullptr;
    if (scaled) {
        if (a.K % KMQ_BLOCK != 0) return KMQ_ERR_SHAPE;
        if (a.layout == KMQ_LAYOUT_TILED && a.K > 256 * KMQ_BLOCK) return KMQ_ERR_LAYOUT;
        if (!aligned(a.scales, 2)) return KMQ_ERR_ALIGN;
    }
    const Plan plan = make_plan(a.N, a.K, a.bits, a.M, a.layout, scaled);
    if (plan.variant == kVariantInvalid) return a.layout == KMQ_LAYOUT_ROWLANE ? KMQ_ERR_LAYOUT : KMQ_ERR_SHAPE;
    if (plan.workspace_bytes > 0 && library_scratch) {
        if (plan.workspace_bytes > KMQ_NOALLOC_SCRATCH_BYTES) return KMQ_ERR_WORKSPACE;
        const hipError_t es = noalloc_scratch(&a.workspace);
        if (es != hipSuccess) return hip_status(es);
        a.workspace_bytes = KMQ_NOALLOC_SCRATCH_BYTES;
    }
    if (plan.workspace_bytes > 0 && (!a.workspace || a.workspace_bytes < plan.workspace_bytes)) return KMQ_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    switch (plan.variant) {
        case kVariantMfma: e = launch_mfma(a, s); break;
        case kVariantRowlane: e = launch_rowlane(a, s); break;
        case kVariantLut: e = launch_lut_entry(plan.table_index, a, s); break;
        case kVariantPerColumn:                               // one launch, a workgroup per (row group, column)
            e = launch_lut_entry(plan.table_index, a, s);   // K is a multiple of 8 for every table kernel: rows of X stay 16-byte aligned
            break;
        case kVariantLutLoop: e = launch_lut_loop(a, s); break;
        case kVariantBlockGeneric: e = launch_blockscaled_generic(a, s); break;
        default: e = launch_generic(a, s); break;
    }
    return hip_status(e);
}

}  // namespace kmq

extern "C" {

size_t kmq_workspace_bytes(int64_t N, int64_t K, int bits, int M, int layout) {
    return kmq::make_plan(N, K, bits, M, layout).workspace_bytes;
}

const char* kmq_kernel_name(int64_t N, int64_t K, int bits, int M, int layout) {
    return kmq::make_plan(N, K, bits, M, layout).name;
}

kmq_status kmq_gemm_smallbatch(const uint32_t* W, const uint16_t* codebook, const uint16_t* X,
                               uint16_t* Y, int64_t N, int64_t K, int M, int bits, int layout,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    const kmq::GemmArgs a{W, codebook, X, Y, N, K, M, bits, layout, workspace, workspace_bytes};
    return kmq::check_and_run(a, hip_stream);
}

kmq_status kmq_gemm_smallbatch_noalloc(const uint32_t* W, const uint16_t* codebook, const uint16_t* X,
                                       uint16_t* Y, int64_t N, int64_t K, int M, int bits, int layout,
                                       void* hip_stream) {
    const kmq::GemmArgs a{W, codebook, X, Y, N, K, M, bits, layout, nullptr, 0};
    return kmq::check_and_run(a, hip_stream, /*library_scratch=*/true);
}

kmq_status kmq_gemv(const uint32_t* W, const uint16_t* codebook, const uint16_t* x, uint16_t* y,
                    int64_t N, int64_t K, int bits, int layout,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
    const kmq::GemmArgs a{W, codebook, x, y, N, K, 1, bits, layout, workspace, workspace_bytes};
    return kmq::check_and_run(a, hip_stream);
}

kmq_status kmq_gemv_swiglu(const uint32_t* Wgate, const uint16_t* codebook_gate,
                           const uint32_t* Wup, const uint16_t* codebook_up,
                           const uint16_t* x, uint16_t* y, int64_t N, int64_t K, int bits, int layout,
                           void* hip_stream) {
    if (!Wgate || !codebook_gate || !Wup || !codebook_up || !x || !y) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K) || 2 * N > kmq::kMaxDim) return KMQ_ERR_SHAPE;
    const bool rowlane = layout == KMQ_LAYOUT_ROWLANE && kmq::rowlane_pair_has_kernel(K, bits);
    if (layout != KMQ_LAYOUT_CANONICAL && !rowlane) return KMQ_ERR_LAYOUT;
    if (!kmq::aligned(Wgate, 16) || !kmq::aligned(Wup, 16) || !kmq::aligned(x, 16) ||
        !kmq::aligned(codebook_gate, 4) || !kmq::aligned(codebook_up, 4) || !kmq::aligned(y, 2)) return KMQ_ERR_ALIGN;
    kmq::GemmArgs a{Wgate, codebook_gate, x, y, N, K, 1, bits, layout, nullptr, 0};
    a.W2 = Wup;
    a.codebook2 = codebook_up;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (rowlane) return kmq::hip_status(kmq::launch_rowlane_pair(a, s));
    const int l = kmq::lut_find(2 * N, K, bits, layout, false);
    const hipError_t e = l >= 0 ? kmq::launch_lut_entry(l, a, s) : kmq::launch_pair_generic(a, s);
    return kmq::hip_status(e);
}

const char* kmq_kernel_name_swiglu(int64_t N, int64_t K, int bits, int layout) {
    if (!kmq::bits_valid(bits) || !kmq::dims_valid(N, K)) return "invalid";
    if (layout == KMQ_LAYOUT_ROWLANE && kmq::rowlane_pair_has_kernel(K, bits)) return bits == 1 ? "rowlane_pair_b1" : "rowlane_pair_b2";
    if (layout != KMQ_LAYOUT_CANONICAL) return "invalid";
    const int l = kmq::lut_find(2 * N, K, bits, layout, false);
    return l >= 0 ? kmq::lut_name(l) : "pair_generic";
}

kmq_status kmq_gemv_fused(const uint32_t* W, const uint16_t* codebook, const uint16_t* x,
                          int rmsnorm, const uint16_t* norm_weight, float eps, const uint16_t* residual, uint16_t* y,
                          int64_t N, int64_t K, int bits, int layout, void* hip_stream) {
    if (!W || !codebook || !x || !y) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K) || (rmsnorm && !(eps >= 0.f)) || (rmsnorm != 0 && rmsnorm != 1)) return KMQ_ERR_SHAPE;
    if (!rmsnorm) norm_weight = nullptr;
    if (layout != KMQ_LAYOUT_CANONICAL) return KMQ_ERR_LAYOUT;
    if (!kmq::aligned(W, 16) || !kmq::aligned(x, 16) || !kmq::aligned(codebook, 4) || !kmq::aligned(y, 2) ||
        (norm_weight && !kmq::aligned(norm_weight, 16)) || (residual && !kmq::aligned(residual, 2))) return KMQ_ERR_ALIGN;
    kmq::GemmArgs a{W, codebook, x, y, N, K, 1, bits, layout, nullptr, 0};
    a.norm = rmsnorm != 0;
    a.norm_w = norm_weight;
    a.eps = eps;
    a.residual = residual;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int l = kmq::lut_find(N, K, bits, layout, false);
    hipError_t e;
    if (l >= 0 && kmq::lut_has_fusions(l)) e = kmq::launch_lut_entry(l, a, s);
    else if (!rmsnorm && kmq::lut_loop_has_kernel(N, K, bits, layout)) e = kmq::launch_lut_loop(a, s);   // residual behind: the K-loop table kernel
    else e = kmq::launch_fused_generic(a, s);
    return kmq::hip_status(e);
}

kmq_status kmq_gemv_swiglu_rmsnorm(const uint32_t* Wgate, const uint16_t* codebook_gate,
                                   const uint32_t* Wup, const uint16_t* codebook_up,
                                   const uint16_t* x, const uint16_t* norm_weight, float eps, uint16_t* y,
                                   int64_t N, int64_t K, int bits, int layout, void* hip_stream) {
    if (!Wgate || !codebook_gate || !Wup || !codebook_up || !x || !y) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K) || 2 * N > kmq::kMaxDim || !(eps >= 0.f)) return KMQ_ERR_SHAPE;
    if (layout != KMQ_LAYOUT_CANONICAL) return KMQ_ERR_LAYOUT;
    if (!kmq::aligned(Wgate, 16) || !kmq::aligned(Wup, 16) || !kmq::aligned(x, 16) || (norm_weight && !kmq::aligned(norm_weight, 16)) ||
        !kmq::aligned(codebook_gate, 4) || !kmq::aligned(codebook_up, 4) || !kmq::aligned(y, 2)) return KMQ_ERR_ALIGN;
    kmq::GemmArgs a{Wgate, codebook_gate, x, y, N, K, 1, bits, layout, nullptr, 0};
    a.W2 = Wup;
    a.codebook2 = codebook_up;
    a.norm = true;
    a.norm_w = norm_weight;
    a.eps = eps;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int l = kmq::lut_find(2 * N, K, bits, layout, false);
    const hipError_t e = (l >= 0 && kmq::lut_has_fusions(l)) ? kmq::launch_lut_entry(l, a, s) : kmq::launch_fused_generic(a, s);
    return kmq::hip_status(e);
}

const char* kmq_kernel_name_fused(int64_t N, int64_t K, int bits, int layout, int pair) {
    if (!kmq::bits_valid(bits) || !kmq::dims_valid(N, K) || layout != KMQ_LAYOUT_CANONICAL) return "invalid";
    const int l = kmq::lut_find(pair ? 2 * N : N, K, bits, layout, false);
    return (l >= 0 && kmq::lut_has_fusions(l)) ? kmq::lut_name(l) : "fused_generic";
}

kmq_status kmq_gemm_smallbatch_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales,
                                           const uint16_t* X, uint16_t* Y, int64_t N, int64_t K, int M, int bits,
                                           int layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!scales) return KMQ_ERR_NULL;
    const kmq::GemmArgs a{W, codebook, X, Y, N, K, M, bits, layout, workspace, workspace_bytes, scales};
    return kmq::check_and_run(a, hip_stream);
}

kmq_status kmq_gemv_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales,
                                const uint16_t* x, uint16_t* y, int64_t N, int64_t K, int bits, int layout,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
    return kmq_gemm_smallbatch_blockscaled(W, codebook, scales, x, y, N, K, 1, bits, layout, workspace,
                                           workspace_bytes, hip_stream);
}

const char* kmq_kernel_name_blockscaled(int64_t N, int64_t K, int bits, int M, int layout) {
    return kmq::make_plan(N, K, bits, M, layout, true).name;
}

kmq_status kmq_dequant(const uint32_t* W, const uint16_t* codebook, uint16_t* Wdense,
                       int64_t N, int64_t K, int bits, int layout, void* hip_stream) {
    if (!W || !codebook || !Wdense) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K)) return KMQ_ERR_SHAPE;
    if (layout != KMQ_LAYOUT_CANONICAL && layout != KMQ_LAYOUT_TILED) return KMQ_ERR_LAYOUT;
    if (layout == KMQ_LAYOUT_TILED && !kmq::tiled_valid(bits, K)) return KMQ_ERR_LAYOUT;
    if ((reinterpret_cast<uintptr_t>(W) & 15) || (reinterpret_cast<uintptr_t>(codebook) & 3) ||
        (reinterpret_cast<uintptr_t>(Wdense) & 1)) return KMQ_ERR_ALIGN;
    const hipError_t e = kmq::launch_dequant(W, codebook, Wdense, N, K, bits, layout,
                                             static_cast<hipStream_t>(hip_stream));
    return kmq::hip_status(e);
}

kmq_status kmq_gemv_bf16(const uint16_t* W, const uint16_t* x, uint16_t* y, int64_t N, int64_t K,
                         void* hip_stream) {
    if (!W || !x || !y) return KMQ_ERR_NULL;
    if (!kmq::dims_valid(N, K) || K > 32768) return KMQ_ERR_SHAPE;
    const uintptr_t a = (K % 8) == 0 ? 15 : 1;
    if ((reinterpret_cast<uintptr_t>(W) & a) || (reinterpret_cast<uintptr_t>(x) & a) ||
        (reinterpret_cast<uintptr_t>(y) & 1)) return KMQ_ERR_ALIGN;
    return kmq::hip_status(kmq::launch_gemv_bf16(W, x, y, N, K, static_cast<hipStream_t>(hip_stream)));
}

kmq_status kmq_quantize_rows(const uint16_t* Wdense, int64_t N, int64_t K, int bits, int iters,
                             uint32_t* packed, uint16_t* codebook, void* hip_stream) {
    if (!Wdense || !packed || !codebook) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits) || bits > 4) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K) || iters < 0 || N > 0x7FFFFFFF) return KMQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(Wdense) & 1) || (reinterpret_cast<uintptr_t>(codebook) & 1) ||
        (reinterpret_cast<uintptr_t>(packed) & 3)) return KMQ_ERR_ALIGN;
    return kmq::hip_status(kmq::launch_quantize_rows(Wdense, N, K, bits, iters, packed, codebook,
                                                     static_cast<hipStream_t>(hip_stream)));
}

size_t kmq_quantize_blockscaled_workspace_bytes(void) { return kmq::quantize_blockscaled_workspace_bytes(); }

kmq_status kmq_quantize_blockscaled(const uint16_t* Wdense, int64_t N, int64_t K, int bits, int iters,
                                    uint32_t* packed, uint16_t* codebook, uint16_t* scales,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!Wdense || !packed || !codebook || !scales) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits) || bits > 4) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K) || iters < 0 || K % KMQ_BLOCK != 0 || N * (K / KMQ_BLOCK) > (int64_t(1) << 32))
        return KMQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(Wdense) & 15) || (reinterpret_cast<uintptr_t>(codebook) & 1) ||
        (reinterpret_cast<uintptr_t>(scales) & 1) || (reinterpret_cast<uintptr_t>(packed) & 3) ||
        (reinterpret_cast<uintptr_t>(workspace) & 7)) return KMQ_ERR_ALIGN;
    if (!workspace || workspace_bytes < kmq::quantize_blockscaled_workspace_bytes()) return KMQ_ERR_WORKSPACE;
    return kmq::hip_status(kmq::launch_quantize_blockscaled(Wdense, N, K, bits, iters, packed, codebook, scales,
                                                            workspace, static_cast<hipStream_t>(hip_stream)));
}

kmq_status kmq_dequant_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales,
                                   uint16_t* Wdense, int64_t N, int64_t K, int bits, void* hip_stream) {
    if (!W || !codebook || !scales || !Wdense) return KMQ_ERR_NULL;
    if (!kmq::bits_valid(bits)) return KMQ_ERR_BITS;
    if (!kmq::dims_valid(N, K) || K % KMQ_BLOCK != 0 || N * (K / 8) > (int64_t(1) << 39)) return KMQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(W) & 15) || (reinterpret_cast<uintptr_t>(codebook) & 3) ||
        (reinterpret_cast<uintptr_t>(scales) & 1) || (reinterpret_cast<uintptr_t>(Wdense) & 15)) return KMQ_ERR_ALIGN;
    return kmq::hip_status(kmq::launch_dequant_blockscaled(W, codebook, scales, Wdense, N, K, bits,
                                                           static_cast<hipStream_t>(hip_stream)));
}

const char* kmq_last_hip_error(void) { return kmq::g_last_hip_error; }

}  // extern "C"
