// Internal launch interface between the C-ABI layer and the kernel files.
#ifndef KMQ_LAUNCH_H
#define KMQ_LAUNCH_H

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace kmq {

struct GemmArgs {
    const uint32_t* W;
    const uint16_t* codebook;
    const uint16_t* X;
    uint16_t* Y;
    int64_t N, K;
    int M, bits, layout;
    void* workspace;
    size_t workspace_bytes;
    const uint16_t* scales = nullptr;   // block-scaled format: N x K/64 bf16, and `codebook` is one tensor-wide table
    const uint32_t* W2 = nullptr;       // fused pair (gate, up): second matrix and its codebooks, same shape and format
    const uint16_t* codebook2 = nullptr;
    bool norm = false;                  // RMSNorm of x in front of the product, with eps ...
    const uint16_t* norm_w = nullptr;   // ... and these gains (K bf16); nullptr: unit gains
    float eps = 0.f;
    const uint16_t* residual = nullptr; // N bf16 added to the product
};

// Kernel variants the heuristic can pick (kmq_kernel_name reports them).
enum Variant {
    kVariantInvalid = 0,
    kVariantGeneric,     // any shape: wave per row, fp32 codebook in LDS
    kVariantLut,         // batch 1, K from a table: hand-scheduled LDS-table kernel
    kVariantMfma,        // tiled layout, batch 1..16: matrix-core kernel
    kVariantBlockGeneric,  // block-scaled format, any shape with K % 64 == 0
    kVariantPerColumn,     // canonical layout, batch > 1, shape with a batch-1 table kernel: that kernel over a (row group, column) grid
    kVariantRowlane,       // row-lane layout, batch 1..4: lane-per-row table kernel, activations through DPP broadcasts
    kVariantLutLoop,       // canonical layout, K % 32 == 0 (up to 24576) without a specialised table kernel: the table kernel that walks K in rounds
};

struct Plan {
    Variant variant;
    int table_index;         // which specialisation (variant-specific), -1 if none
    size_t workspace_bytes;  // device workspace this plan needs
    const char* name;
};

Plan make_plan(int64_t N, int64_t K, int bits, int M, int layout, bool scaled = false);

hipError_t launch_generic(const GemmArgs& a, hipStream_t s);   // split-K when a.workspace is given and the shape asks for it
int generic_splitk_slices(int64_t N, int64_t K, int layout);
hipError_t noalloc_scratch(void** ptr);   // this GPU's KMQ_NOALLOC_SCRATCH_BYTES of library-owned scratch (kmq_gemm_smallbatch_noalloc)
hipError_t launch_dequant(const uint32_t* W, const uint16_t* codebook, uint16_t* Wd, int64_t N,
                          int64_t K, int bits, int layout, hipStream_t s);

hipError_t launch_pair_generic(const GemmArgs& a, hipStream_t s);
hipError_t launch_fused_generic(const GemmArgs& a, hipStream_t s);   // batch 1, canonical layout, any shape; pair optional
hipError_t launch_blockscaled_generic(const GemmArgs& a, hipStream_t s);
hipError_t launch_dequant_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales, uint16_t* Wd,
                                      int64_t N, int64_t K, int bits, hipStream_t s);   // canonical, K % 64 == 0

// Dense bf16 baseline; K * 2 bytes of LDS, so K <= 32768.
hipError_t launch_gemv_bf16(const uint16_t* W, const uint16_t* x, uint16_t* y, int64_t N, int64_t K, hipStream_t s);

// Quantiser (dense bf16 -> indices + codebooks): per-row codebooks, and the block-scaled format
// whose workspace is quantize_blockscaled_workspace_bytes() bytes, 8-byte aligned.
hipError_t launch_quantize_rows(const uint16_t* W, int64_t N, int64_t K, int bits, int iters, uint32_t* packed,
                                uint16_t* codebook, hipStream_t s);
size_t quantize_blockscaled_workspace_bytes();
hipError_t launch_quantize_blockscaled(const uint16_t* W, int64_t N, int64_t K, int bits, int iters, uint32_t* packed,
                                       uint16_t* codebook, uint16_t* scales, void* workspace, hipStream_t s);

// Matrix-core kernel (tiled layout only).
hipError_t launch_mfma(const GemmArgs& a, hipStream_t s);
// 2- and 3-bit rows of at most 4096 columns: every wave keeps its slice of the activations in registers
bool mfma_kslice_has_kernel(int64_t N, int64_t K, int bits);
hipError_t launch_mfma_kslice(const GemmArgs& a, hipStream_t s);
int mfma_waves_along_k(int64_t N, int64_t K, int bits);
int mfma_row_blocks(int64_t N, int64_t K, int bits);

// Row-lane layout kernels (batch 1..4).
bool rowlane_has_kernel(int64_t K, int bits, int M);
bool rowlane_loops(int64_t K, int bits);              // K served by the kernel that walks K in rounds
hipError_t launch_rowlane(const GemmArgs& a, hipStream_t s);
bool rowlane_pair_has_kernel(int64_t K, int bits);     // fused gate / up / SwiGLU on the row-lane layout
hipError_t launch_rowlane_pair(const GemmArgs& a, hipStream_t s);

// Hand-scheduled table kernels (1/2/4-bit): -1 if (bits, K, layout) has none.
int lut_find(int64_t N, int64_t K, int bits, int layout, bool scaled = false);
const char* lut_name(int table_index);
bool lut_has_fusions(int table_index);   // RMSNorm in front / residual behind (GemmArgs::norm_w, residual)
hipError_t launch_lut_entry(int table_index, const GemmArgs& a, hipStream_t s);

// The table kernel that walks K in rounds (canonical layout, K % 32 == 0, K <= 24576, batches in one launch).
bool lut_loop_has_kernel(int64_t N, int64_t K, int bits, int layout);
const char* lut_loop_name(int bits);
hipError_t launch_lut_loop(const GemmArgs& a, hipStream_t s);

}  // namespace kmq

#endif
