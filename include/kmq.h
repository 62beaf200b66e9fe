/* kmq.h -- C ABI of the k-means-quantised matrix-vector / small-batch matrix
 * product for AMD MI355X (gfx950).
 *
 * The operation is the fused dequantise-multiply of the paper's App. E
 * ("Benchmarking": Y^T = dequantize(W~) X^T, and the reference routine under
 * "Kernel implementations"), with dequantisation by centroid lookup as in
 * Sec. 2.2 ("Nonlinear k-means quantization"), in the benchmark contract's
 * form: no block scales, one codebook of 2^b bf16 centroids per output row.
 *
 *     w[n][k] = codebook[n][ idx[n][k] ]                 (bf16, exact lookup)
 *     Y[m][n] = sum_k w[n][k] * X[m][k]                  (fp32 accumulation, bf16 out,
 *                                                         round-to-nearest-even)
 *
 * CANONICAL PACKED FORMAT (layout 0).  Row n of W is a little-endian bit
 * stream: element k occupies stream bits [k*b, k*b+b), stream bit p is bit
 * (p mod 32) of 32-bit word (p div 32).  For b = 3 a field may straddle two
 * words.  Every row starts on a fresh word and holds kmq_words_per_row(b, K)
 * words; pad bits are zero on output of kmq_pack and ignored on input
 * everywhere.  For b in {1,2,4} the byte view of this stream is the paper's
 * uint8 element stream `Wq` with an LSB-first byte table.
 *
 * BIT-WIDTHS.  b = 1, 2, 3, 4 everywhere.  b = 8 (256 centroids, the widest of the
 * element formats of the paper's lookup-table kernel, Sec. 3.3 "Software formats") is
 * accepted on the canonical layout by every product, fusion and dequantisation call
 * and served by the shape-agnostic kernels; there is no tiled layout for it
 * (KMQ_ERR_LAYOUT) and the quantiser does not produce it (KMQ_ERR_BITS).
 *
 * General rules.  No function allocates, frees or synchronises.  Device entry
 * points enqueue on `hip_stream` (a hipStream_t passed as void*, NULL = the
 * null stream) and return; they are legal under stream capture.  The caller
 * owns every buffer.  Inputs are never written; outputs are fully overwritten.
 * The same inputs give bit-identical outputs run to run (no floating-point
 * atomics).  Every argument is checked before anything is launched; a bad
 * argument returns an error code and touches nothing.  Nothing throws or aborts.
 */
#ifndef KMQ_H
#define KMQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t kmq_status;
enum {
    KMQ_OK = 0,
    KMQ_ERR_NULL = 1,        /* a required pointer is NULL */
    KMQ_ERR_BITS = 2,        /* bits not in {1,2,3,4,8} (the quantiser: {1,2,3,4}) */
    KMQ_ERR_SHAPE = 3,       /* N, K < 1, M outside 1..KMQ_MAX_BATCH, or size overflow */
    KMQ_ERR_ALIGN = 4,       /* pointer alignment (see each function) */
    KMQ_ERR_INDEX_RANGE = 5, /* kmq_pack: an index >= 2^bits */
    KMQ_ERR_WORKSPACE = 6,   /* workspace NULL or smaller than kmq_workspace_bytes */
    KMQ_ERR_LAYOUT = 7,      /* unknown layout id, or layout not valid for this (bits, K) */
    KMQ_ERR_HIP = 8          /* the HIP runtime refused a launch (hipGetLastError is left set) */
};

enum {
    KMQ_LAYOUT_CANONICAL = 0, /* the format above */
    KMQ_LAYOUT_TILED = 1,     /* matrix-core operand order, see kmq_repack */
    KMQ_LAYOUT_ROWLANE = 2    /* lane-per-row order of the batch 1..4 kernels, see kmq_repack */
};

#define KMQ_MAX_BATCH 16

/* ceil(K*bits/32): 32-bit words per row of the canonical stream; -1 on bad arguments. */
int64_t kmq_words_per_row(int bits, int64_t K);

/* Host, offline, integer only.  idx: N*K bytes, one index per element, row-major,
 * each < 2^bits.  packed: N*kmq_words_per_row words, canonical format, pad bits zero.
 * Both are host pointers.  KMQ_ERR_INDEX_RANGE leaves `packed` unspecified. */
kmq_status kmq_pack(const uint8_t* idx, int64_t N, int64_t K, int bits, uint32_t* packed);

/* Inverse of kmq_pack (host pointers).  Pad bits of `packed` are ignored. */
kmq_status kmq_unpack(const uint32_t* packed, int64_t N, int64_t K, int bits, uint8_t* idx);

/* Host, offline, integer only, reversible: permutes the index bits of the
 * canonical stream into the order named by `layout` (kmq_unrepack(kmq_repack(P))
 * == P).  Motivated by
 * the paper's remark (App. E, "Micro-benchmarks: Results") that custom code with
 * an optimised data layout is the route to faster low-bit kernels.
 *
 * KMQ_LAYOUT_TILED is the operand order of the matrix-core kernels.  A GROUP is
 * 8 consecutive elements of a row.  Let gpg = 16, 8, 4, 4 groups for bits = 1, 2,
 * 3, 4.  K is cut into super-blocks of 4*gpg groups (512, 256, 128, 128 elements)
 * and rows into blocks of 16 (the last block may be short; its missing rows are
 * zero).  The GRANULE (rb, sb, q, n) holds the groups q + 4j, j = 0..gpg-1, of
 * super-block sb of row 16*rb + n; it is gw = gpg*bits/4 dwords (4, 4, 3, 4) at
 * dword offset
 *     ((rb * nsb + sb) * 64 + q*16 + n) * gw,      nsb = K / (32*gpg),
 * so one 64-lane load of consecutive granules is 16 rows x one super-block, and
 * lane (n, q) of 16x16x32 matrix-core step j owns columns 8*(q+4j)..+7 of both
 * operands.  Inside a granule (bit positions count through its dwords, LSB
 * first), bit t of the index of element e (0..7) of step j sits at
 *     bits = 1:  8*j + e                               (groups in order, one byte each)
 *     bits = 4:  32*j + 4*e + t                        (groups in order, one dword each)
 *     bits = 2:  32*(c/4) + 8*(e%4) + 2*(c%4) + t,     c = 2*j + e/4
 *     bits = 3:  h = e/4, p = 8*(e%4):
 *                j < 3:          32*j + p + 3*h + t     (two 3-bit fields in bits 0..5 of each byte)
 *                j = 3, h = 0:   t < 2: p + 6 + t       (the bytes' two spare top bits, dword 0)
 *                                t = 2: 32 + p + 6
 *                j = 3, h = 1:   t = 0: 32 + p + 7
 *                                t > 0: 64 + p + 5 + t
 * The 2- and 3-bit orders spread the fields so that at most one shift and one
 * AND leave four indices in the four bytes of a register (3-bit, step 3: two of each).  Requires K % (32*gpg) == 0
 * (else KMQ_ERR_LAYOUT).  Same size as the canonical stream with rows padded
 * to 16: size `tiled` with kmq_tiled_words().
 *
 * KMQ_LAYOUT_ROWLANE (bits = 1 or 2, K % 256 == 0, else KMQ_ERR_LAYOUT) is the order of the
 * lane-per-row kernels that serve batches 1..4 without the matrix cores (a weight is decoded
 * once per launch of up to four batch columns; wider batches take several launches).  Every such K
 * has a kernel: K / 256 = c * w with c in {1,2,3,4,6,7,8} tiles per wave and w <= 16 waves is served
 * with every load in flight at once, any other tile count (17, 19, 43, ... or beyond 128) by a kernel
 * that walks K in rounds (kmq_kernel_name says "rowlane_loop_...").  A CHUNK is
 * 64 consecutive elements of a row (2*bits dwords); a TILE is 16 rows x 4 consecutive chunks,
 * 64 chunks stored one after the other, chunk kp of row 16*rb + r at dword offset
 *     ((rb * (K/256) + t) * 64 + kp*16 + r) * 2*bits          (t = tile number along K),
 * so a wave's load of one tile is contiguous, the 16 lanes that share a chunk number hold 16
 * different rows, and the activations of chunk kp are 32 bf16 pairs, two per lane.  Inside a chunk
 * (bit positions count through its dwords, LSB first), bit u of the index of element c (0..63):
 *     bits = 2:  p = c/2 (pair), s = p/2 + 16*(p%2):    4*s + 2*(c%2) + u
 *                (nibble slot s, 8 per dword, holds the pair whose activations sit in lane s%16,
 *                register s/16, after one 8-byte load per lane)
 *     bits = 1:  s = c/4, q = s/8, b = (s%8)/2, view = s%2, i = c%4:
 *                view 0:  32*q + 8*b + 3 + i
 *                view 1:  32*q + (8*b + 7 + i) % 32
 *                (a nibble sits at bits 3..6 of a byte, either of the dword itself or of the dword
 *                rotated right by 4: one byte-select AND yields its 8-byte table offset)
 * Rows are padded to a multiple of 16 with zeros, as for KMQ_LAYOUT_TILED; same size. */
kmq_status kmq_repack(const uint32_t* canonical, int64_t N, int64_t K, int bits, int layout,
                      uint32_t* tiled);
kmq_status kmq_unrepack(const uint32_t* tiled, int64_t N, int64_t K, int bits, int layout,
                        uint32_t* canonical);
/* Number of 32-bit words of W in `layout` (canonical: N*wpr); -1 on bad arguments. */
int64_t kmq_tiled_words(int64_t N, int64_t K, int bits, int layout);

/* Bytes of device workspace kmq_gemv / kmq_gemm_smallbatch need for this
 * problem: 0 unless the rows are too few to fill the compute units and long
 * (canonical layout, ceil(N/4) <= 128 and K >= 16384, no shape-specialised
 * kernel), where K is split over workgroups and the workspace holds
 * slices * M * N fp32 partial sums, added in slice order by a second kernel
 * (deterministic).  The workspace need not be initialised and may be reused
 * by later calls on the same stream.
 * Returns 0 on bad arguments (the compute call then reports the error). */
size_t kmq_workspace_bytes(int64_t N, int64_t K, int bits, int M, int layout);

/* y = W x.  All pointers are DEVICE pointers.
 *   W        packed indices in `layout` (16-byte aligned)
 *   codebook N x 2^bits bf16 bit patterns, row-major (4-byte aligned)
 *   x        K bf16 (16-byte aligned)
 *   y        N bf16, overwritten (2-byte aligned)
 *   workspace, workspace_bytes  >= kmq_workspace_bytes(N,K,bits,1,layout); may be NULL/0 if that is 0
 * Equivalent to kmq_gemm_smallbatch with M = 1.
 * Kernels on the canonical layout (kmq_kernel_name tells which one a shape gets): bits 1..4 with K one of
 * the row lengths the library has a fully unrolled table kernel for ("lut_b..."), any other K % 32 == 0 up
 * to 24576 through the table kernel that walks a row in rounds ("lut_loop_b..."), everything else (K not a
 * multiple of 32 or beyond 24576, bits = 8) through the shape-agnostic kernel ("generic", "generic_splitk"). */
kmq_status kmq_gemv(const uint32_t* W, const uint16_t* codebook, const uint16_t* x, uint16_t* y,
                    int64_t N, int64_t K, int bits, int layout,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Y = X W^T for 1 <= M <= KMQ_MAX_BATCH (paper App. D/E: the small-batch,
 * memory-bound regime; larger batches are better served by kmq_dequant plus a
 * dense GEMM, App. E "Model benchmarks").  X is M x K bf16 row-major (16-byte
 * aligned), Y is M x N bf16 row-major, overwritten.  Other arguments as kmq_gemv.
 * Every layout is accepted at every M.  KMQ_LAYOUT_TILED is the fast one for M >= 8
 * (matrix-core kernel: a weight is dequantised once for the whole batch);
 * KMQ_LAYOUT_ROWLANE serves M = 1..4 on the vector units, each weight dequantised once
 * (M > 4: one launch per four columns); on the canonical layout every batch column
 * looks the weights up again, in one launch. */
kmq_status kmq_gemm_smallbatch(const uint32_t* W, const uint16_t* codebook, const uint16_t* X,
                               uint16_t* Y, int64_t N, int64_t K, int M, int bits, int layout,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* kmq_gemm_smallbatch for callers that cannot allocate device memory and so cannot bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (without the workspace pair), same kernels, same results bit for bit.  Where the problem needs a
 * workspace (kmq_workspace_bytes > 0: K split over workgroups), the partial sums go to an array of
 * KMQ_NOALLOC_SCRATCH_BYTES that the library holds on every GPU it runs on, until the process ends;
 * a problem that needs more returns KMQ_ERR_WORKSPACE (64 KiB covers every shape the split currently
 * serves).  The call itself allocates and frees nothing.  The first call on a device looks the
 * array's address up (make that call outside stream capture).  All calls on one GPU share that
 * GPU's array: it keeps the last call's contents (nothing in it has to start at zero: every partial
 * sum is written before it is read), and calls that overlap on one GPU -- different streams, or graphs
 * replayed concurrently -- race on it; calls on one stream are ordered and safe. */
#define KMQ_NOALLOC_SCRATCH_BYTES 65536
kmq_status kmq_gemm_smallbatch_noalloc(const uint32_t* W, const uint16_t* codebook, const uint16_t* X,
                                       uint16_t* Y, int64_t N, int64_t K, int M, int bits, int layout,
                                       void* hip_stream);

/* Wdense[n][k] = codebook[n][idx[n][k]] as bf16 bit patterns, N x K row-major,
 * bit-exact (device pointers).  The separate-dequantise route the paper
 * suggests for large batches (App. E "Model benchmarks"), and the bit-exactness probe. */
kmq_status kmq_dequant(const uint32_t* W, const uint16_t* codebook, uint16_t* Wdense,
                       int64_t N, int64_t K, int bits, int layout, void* hip_stream);

/* ---- The paper's own weight format: tensor-wide codebook + block scales -------------
 * Sec. 2.2 "Nonlinear k-means quantization": the centroids (values in [-1, 1]) are shared
 * by the whole tensor and every block of KMQ_BLOCK = 64 consecutive elements of a row has
 * one 16-bit scale; App. E "Kernel implementations" gives the reference routine
 * (lookup, multiply by the block's scale, matrix product) and the deferred-scaling
 * variant (scale each block's partial sum), which is what these calls compute:
 *
 *     Y[m][n] = sum_g scale[n][g] * sum_{k in block g} codebook[idx[n][k]] * X[m][k]
 *
 * with both sums in fp32 and one rounding to bf16 at the end.
 *   W         packed indices, 16-byte aligned; KMQ_LAYOUT_CANONICAL, or KMQ_LAYOUT_TILED (the matrix-core
 *             kernel, any batch) for K <= 16384 (else KMQ_ERR_LAYOUT)
 *   codebook  2^bits bf16 bit patterns (4-byte aligned)
 *   scales    N x K/64 bf16 bit patterns, row-major (2-byte aligned); K % 64 != 0 -> KMQ_ERR_SHAPE
 *   x / X, y / Y, M, workspace, hip_stream: as kmq_gemv / kmq_gemm_smallbatch.
 * All pointers are DEVICE pointers owned by the caller; nothing is allocated or synchronised. */
#define KMQ_BLOCK 64
kmq_status kmq_gemv_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales,
                                const uint16_t* x, uint16_t* y, int64_t N, int64_t K, int bits, int layout,
                                void* workspace, size_t workspace_bytes, void* hip_stream);
kmq_status kmq_gemm_smallbatch_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales,
                                           const uint16_t* X, uint16_t* Y, int64_t N, int64_t K, int M, int bits,
                                           int layout, void* workspace, size_t workspace_bytes, void* hip_stream);
/* As kmq_kernel_name, for the block-scaled calls. */
const char* kmq_kernel_name_blockscaled(int64_t N, int64_t K, int bits, int M, int layout);

/* Fused gate / up / SwiGLU of a decoder MLP (App. E "Model benchmarks": token generation runs the
 * backbone's projections one after another, with the activation function between them as extra
 * cost): y[n] = silu(Wgate[n] . x) * (Wup[n] . x), silu(t) = t / (1 + exp(-t)), both products
 * and the combination in fp32, one rounding to bf16.  Both matrices are N x K in the per-row-codebook
 * format, same bits, same layout: KMQ_LAYOUT_CANONICAL, or KMQ_LAYOUT_ROWLANE for 1 and 2 bits where
 * K / 256 splits into at most four tiles per wave times at most 16 waves (kmq_kernel_name_swiglu says
 * "rowlane_pair_..."; every workgroup then decodes the same 16 rows of both matrices against one copy
 * of the activations); any other layout or shape of it: KMQ_ERR_LAYOUT.  Alignment as kmq_gemv;
 * 2N <= 2^24.  One launch instead of two products and an elementwise pass. */
kmq_status kmq_gemv_swiglu(const uint32_t* Wgate, const uint16_t* codebook_gate,
                           const uint32_t* Wup, const uint16_t* codebook_up,
                           const uint16_t* x, uint16_t* y, int64_t N, int64_t K, int bits, int layout,
                           void* hip_stream);
const char* kmq_kernel_name_swiglu(int64_t N, int64_t K, int bits, int layout);

/* Decoder-layer fusions at batch 1 (paper App. E "Model benchmarks": token generation runs a
 * layer's projections back to back; Sec. 3.3 "Software formats" attributes part of the 1-bit
 * model's lost speed to the elementwise work on the activations, RMSNorm and the activation
 * function).  One launch computes RMSNorm in front of the product and a residual sum behind it:
 *     r     = 1 / sqrt( (1/K) sum_k x[k]^2 + eps )           (rmsnorm; else 1)
 *     xn[k] = bf16( x[k] * r * norm_weight[k] )              (the normalised bf16 activations; else xn = x)
 *     y[n]  = bf16( residual[n] + sum_k w[n][k] xn[k] )      (residual optional)
 * The kernels let the scalar r commute with the sum: they round x[k] * norm_weight[k] to bf16
 * and multiply the fp32 sum by r.  Each activation then differs from xn[k] by at most 2^-7 of
 * itself (two roundings to 8 significant bits of the same exact value), so the result is within
 * 2^-7 * sum_k |w xn| of the definition above in the worst case and, the roundings being
 * independent, far inside 2e-3 * sum_k |w xn| for rows of hundreds of elements.
 *   rmsnorm      0: no normalisation (norm_weight and eps ignored); 1: RMSNorm
 *   norm_weight  K bf16 gains, 16-byte aligned, or NULL for unit gains -- the cheaper form: gains
 *                are per input channel and can be multiplied into the dense weights before they are
 *                quantised, and then no second vector is fetched by every workgroup
 *   eps          >= 0
 *   residual     N bf16, 2-byte aligned, or NULL; may alias y
 * Other arguments as kmq_gemv.  Canonical layout only (else KMQ_ERR_LAYOUT).  With rmsnorm = 0
 * and residual = NULL it equals kmq_gemv. */
kmq_status kmq_gemv_fused(const uint32_t* W, const uint16_t* codebook, const uint16_t* x,
                          int rmsnorm, const uint16_t* norm_weight, float eps, const uint16_t* residual,
                          uint16_t* y, int64_t N, int64_t K, int bits, int layout, void* hip_stream);
/* kmq_gemv_swiglu with the same RMSNorm in front of both products (norm_weight NULL: unit gains). */
kmq_status kmq_gemv_swiglu_rmsnorm(const uint32_t* Wgate, const uint16_t* codebook_gate,
                                   const uint32_t* Wup, const uint16_t* codebook_up,
                                   const uint16_t* x, const uint16_t* norm_weight, float eps, uint16_t* y,
                                   int64_t N, int64_t K, int bits, int layout, void* hip_stream);
/* Kernel the two calls above use (pair != 0: the SwiGLU form); static string, "invalid" on bad arguments.
 * "fused_generic" names the shape-agnostic path; kmq_gemv_fused with rmsnorm = 0 takes the kernel kmq_kernel_name
 * reports instead where that is a table kernel (the residual is added in its epilogue). */
const char* kmq_kernel_name_fused(int64_t N, int64_t K, int bits, int layout, int pair);

/* Dense bf16 GEMV, y = W x with W N x K bf16 bit patterns, row-major: the unquantised
 * baseline of the paper's micro-benchmark table (App. E, the 16-bit rows), provided so that
 * speed-ups can be quoted against a bf16 product on the same machine.  fp32 accumulation,
 * bf16 output.  Device pointers; W and x 16-byte aligned when K % 8 == 0 (else 2-byte),
 * y 2-byte aligned; 1 <= K <= 32768 (x is staged in 64 KB of LDS), else KMQ_ERR_SHAPE. */
kmq_status kmq_gemv_bf16(const uint16_t* W, const uint16_t* x, uint16_t* y, int64_t N, int64_t K,
                         void* hip_stream);

/* kmq_dequant for the block-scaled format (canonical layout, K % KMQ_BLOCK == 0):
 * Wdense[n][k] = bf16( codebook[idx[n][k]] * scale[n][k / KMQ_BLOCK] ), one rounding to nearest
 * even of the exact product -- the matrix the reference routine of paper App. E "Kernel
 * implementations" materialises, and the first half of the separate-dequantise route for large
 * batches (App. E "Model benchmarks").  Wdense N x K bf16, 16-byte aligned; other pointers as
 * kmq_gemv_blockscaled.  Device pointers; asynchronous on hip_stream. */
kmq_status kmq_dequant_blockscaled(const uint32_t* W, const uint16_t* codebook, const uint16_t* scales,
                                   uint16_t* Wdense, int64_t N, int64_t K, int bits, void* hip_stream);

/* ---- The quantiser: dense bf16 weights -> indices + codebooks ------------------------
 * (paper Sec. 2.1 "Rounding to nearest centroids": the quantiser rounds to the nearest of
 * 2^bits centroids obtained by 1-D k-means clustering; "Block formats"; Sec. 2.2 "Nonlinear
 * k-means quantization".)  The paper names Lloyd's algorithm and fixes neither its start nor
 * its stopping rule; this library's rules, the same for both calls:
 *   - arithmetic in fp64; the centroids stay sorted ascending;
 *   - a value belongs to cluster a = number of boundaries (c_i + c_{i+1}) / 2 that lie below it
 *     (nearest centroid; a value on a boundary goes to the lower cluster);
 *   - each round replaces a centroid by the mean of its members; a cluster without members
 *     keeps its centroid; exactly `iters` >= 0 rounds are run (a converged state is a fixed point);
 *   - start: 2^bits points evenly spaced over the range of the data,
 *     c_i = lo + (i + 1/2) (hi - lo) / 2^bits;
 *   - the codebook written is the centroids rounded to bf16 (nearest even) and the indices
 *     written are nearest centroids OF THAT CODEBOOK, packed in the canonical layout.
 * Results are deterministic run to run.  Device pointers; asynchronous on hip_stream. */

/* One codebook per row, no scales (the format kmq_gemv takes): row n of Wdense (N x K bf16,
 * row-major, 2-byte aligned) is clustered on its own, lo / hi = the row's min / max.
 *   packed    N * kmq_words_per_row(bits, K) words out (4-byte aligned), pad bits zero
 *   codebook  N x 2^bits bf16 out, ascending per row
 * Errors: KMQ_ERR_NULL, KMQ_ERR_BITS, KMQ_ERR_SHAPE (N, K < 1, iters < 0), KMQ_ERR_ALIGN. */
kmq_status kmq_quantize_rows(const uint16_t* Wdense, int64_t N, int64_t K, int bits, int iters,
                             uint32_t* packed, uint16_t* codebook, void* hip_stream);

/* The paper's format (the one kmq_gemv_blockscaled takes): scale[n][g] = the largest
 * magnitude of block g of row n (blocks of KMQ_BLOCK elements along K; itself a bf16 value),
 * normalised weight v = w / scale in fp64 (0 where the scale is 0), ONE clustering over all
 * N*K normalised weights with lo = -1, hi = 1.
 *   Wdense    N x K bf16, row-major, 16-byte aligned for this call
 *   packed    N * K * bits / 32 words out; codebook 2^bits bf16 out; scales N x K/KMQ_BLOCK bf16 out
 *   workspace device memory of kmq_quantize_blockscaled_workspace_bytes() bytes, 8-byte aligned
 *             (partial sums of the clustering rounds; contents undefined before and after)
 * K % KMQ_BLOCK != 0 -> KMQ_ERR_SHAPE; workspace NULL or too small -> KMQ_ERR_WORKSPACE. */
size_t kmq_quantize_blockscaled_workspace_bytes(void);
kmq_status kmq_quantize_blockscaled(const uint16_t* Wdense, int64_t N, int64_t K, int bits, int iters,
                                    uint32_t* packed, uint16_t* codebook, uint16_t* scales,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Name of the kernel variant the launch heuristic picks for this problem
 * (static string, never NULL; "invalid" on bad arguments).  For reports. */
const char* kmq_kernel_name(int64_t N, int64_t K, int bits, int M, int layout);

const char* kmq_status_string(kmq_status s);

/* Text the HIP runtime gave for the last KMQ_ERR_HIP on the calling thread
 * (static string, "" if there was none). */
const char* kmq_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KMQ_H */
