// kmq_oracle.cpp -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, slow, single-threaded CPU statement of what the k-means-quantised
// matrix product computes, used only to check the GPU library.  Only tests,
// the smoke check and the benchmark's cpu_baseline leg may call it.  It shares
// no source, header, table or helper with the GPU library.
//
// Operation (paper, App. E "Benchmarking", the fused dequantise-multiply
// Y^T = dequantize(W~) X^T and its reference routine in "Kernel
// implementations"; Sec. 2.2 "Nonlinear k-means quantization" for
// dequantisation = centroid lookup), specialised as the benchmark contract
// states it: no block scales, one codebook of 2^b bf16 centroids per output
// row, indices packed b bits each along K.
//
//     w[n][k] = real( codebook[n][ idx[n][k] ] )
//     Y[m][n] = sum_{k=0..K-1} w[n][k] * real( X[m][k] )      (fp64, k ascending)
//     A[m][n] = sum_{k=0..K-1} | w[n][k] * real( X[m][k] ) |  (tolerance scale)
//
// A bf16 x bf16 product has at most 16 significant bits, so every product is
// exact in fp64 and the fp64 sum of <= 2^14 of them is within ~1e-13*A of the
// real-number result: the method reaches exactly this value up to rounding
// order, so the oracle is the definition written out.
//
// Packed format (readings of the contract where it is silent are listed in the
// repository's design notes):
//   * element k of a row occupies stream bits [k*b, k*b + b) of that row;
//   * stream bit p lives in 32-bit word p/32 at bit position p%32 (LSB first);
//   * for b = 3 a field may straddle two consecutive words;
//   * every row starts on a fresh word, rows hold ceil(K*b/32) words, pad bits
//     are zero.
//
// A second entry point, oracle_gemm_blockscaled, states the paper's own weight
// format (Sec. 2.2 "Nonlinear k-means quantization": centroids shared by the whole
// tensor, one 16-bit scale per block of B consecutive elements along K; App. E
// "Kernel implementations", the reference routine and its deferred-scaling
// variant):
//
//     w[n][k] = real( codebook[ idx[n][k] ] ) * real( scale[n][k / B] )
//     Y[m][n] = sum_k w[n][k] * real( X[m][k] )
//
// The product of three bf16 values has at most 24 significant bits: still exact
// in fp64.  "Immediate" sums c*s*x over k ascending; "deferred" sums c*x inside a
// block and multiplies the block sum by s, the order the appendix gives as a
// variant.  Both are the same real number; they differ by fp64 rounding only.
//
// Pins (tests/test_oracle_*.py): literal hand-computed words, round trips,
// brute-force dense products from the unpacked uint8 indices, the 1-bit closed
// form, one-hot / constant-codebook / scaling / permutation invariants, and the
// shared-codebook special case that reduces to the paper's byte-LUT routine.
// Nothing here is "parity unpinned".

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// bf16 is the upper half of an IEEE binary32 pattern.
double bf16_to_double(uint16_t h) {
    uint32_t u = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

bool bits_ok(int bits) { return (bits >= 1 && bits <= 4) || bits == 8; }   // 8: a 256-entry codebook

int64_t words_per_row(int bits, int64_t K) { return (K * bits + 31) / 32; }

// Read the b-bit field of element k from one row's word stream, one bit at a
// time: deliberately the slowest and most literal form of the format rule.
uint32_t read_field(const uint32_t* row, int64_t k, int bits) {
    uint32_t v = 0;
    for (int j = 0; j < bits; ++j) {
        int64_t p = k * bits + j;             // stream bit position
        uint32_t bit = (row[p / 32] >> (p % 32)) & 1u;
        v |= bit << j;
    }
    return v;
}

}  // namespace

extern "C" {

int64_t oracle_words_per_row(int bits, int64_t K) {
    if (!bits_ok(bits) || K < 0) return -1;
    return words_per_row(bits, K);
}

// idx[N][K] (one uint8 per element, value < 2^bits) -> packed[N][wpr].
// Returns 0, or 1 on a bad argument, or 2 if an index is out of range.
int oracle_pack(const uint8_t* idx, int64_t N, int64_t K, int bits, uint32_t* packed) {
    if (!bits_ok(bits) || N < 0 || K < 0) return 1;
    const int64_t wpr = words_per_row(bits, K);
    for (int64_t n = 0; n < N; ++n) {
        uint32_t* row = packed + n * wpr;
        for (int64_t w = 0; w < wpr; ++w) row[w] = 0u;
        for (int64_t k = 0; k < K; ++k) {
            uint32_t v = idx[n * K + k];
            if (v >= (1u << bits)) return 2;
            for (int j = 0; j < bits; ++j) {
                int64_t p = k * bits + j;
                row[p / 32] |= ((v >> j) & 1u) << (p % 32);
            }
        }
    }
    return 0;
}

int oracle_unpack(const uint32_t* packed, int64_t N, int64_t K, int bits, uint8_t* idx) {
    if (!bits_ok(bits) || N < 0 || K < 0) return 1;
    const int64_t wpr = words_per_row(bits, K);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            idx[n * K + k] = static_cast<uint8_t>(read_field(packed + n * wpr, k, bits));
    return 0;
}

// Dequantised weights as bf16 bit patterns: Wd[n][k] = codebook[n][idx[n][k]].
int oracle_dequant(const uint32_t* packed, const uint16_t* codebook, int64_t N, int64_t K,
                   int bits, uint16_t* Wd) {
    if (!bits_ok(bits) || N < 0 || K < 0) return 1;
    const int64_t wpr = words_per_row(bits, K);
    const int64_t C = int64_t(1) << bits;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            Wd[n * K + k] = codebook[n * C + read_field(packed + n * wpr, k, bits)];
    return 0;
}

// Round a double to the nearest bf16 (ties to even).  Finite, normal-range
// inputs only (the synthetic workloads never leave it); NaN/Inf pass through.
uint16_t oracle_round_bf16(double y) {
    float f = static_cast<float>(y);
    uint32_t u;
    std::memcpy(&u, &f, sizeof u);
    if (!std::isfinite(f)) return static_cast<uint16_t>(u >> 16);
    // The two bf16 neighbours that bracket f in magnitude.
    uint32_t lo = u & 0xFFFF0000u, hi = lo + 0x00010000u;
    float flo, fhi;
    std::memcpy(&flo, &lo, sizeof flo);
    std::memcpy(&fhi, &hi, sizeof fhi);
    double dlo = std::fabs(y - static_cast<double>(flo));
    double dhi = std::fabs(y - static_cast<double>(fhi));
    uint32_t pick;
    if (dlo < dhi) pick = lo;
    else if (dhi < dlo) pick = hi;
    else pick = ((lo >> 16) & 1u) ? hi : lo;   // tie: even mantissa
    return static_cast<uint16_t>(pick >> 16);
}

// Rows [n0, n1) of Y = X * W^T.  X is M x K bf16 row-major; Y, A and Ybf16 are
// M x N row-major and only columns n0..n1-1 are written.  A and Ybf16 may be
// null.  M = 1 is the matrix-vector product.
int oracle_gemm(const uint32_t* packed, const uint16_t* codebook, const uint16_t* X,
                int64_t N, int64_t K, int bits, int64_t M, int64_t n0, int64_t n1,
                double* Y, double* A, uint16_t* Ybf16) {
    if (!bits_ok(bits) || N < 0 || K < 0 || M < 0 || n0 < 0 || n1 > N || n0 > n1) return 1;
    const int64_t wpr = words_per_row(bits, K);
    const int64_t C = int64_t(1) << bits;
    std::vector<double> w(static_cast<size_t>(K));
    for (int64_t n = n0; n < n1; ++n) {
        for (int64_t k = 0; k < K; ++k)
            w[k] = bf16_to_double(codebook[n * C + read_field(packed + n * wpr, k, bits)]);
        for (int64_t m = 0; m < M; ++m) {
            double y = 0.0, a = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double t = w[k] * bf16_to_double(X[m * K + k]);
                y += t;
                a += std::fabs(t);
            }
            Y[m * N + n] = y;
            if (A) A[m * N + n] = a;
            if (Ybf16) Ybf16[m * N + n] = oracle_round_bf16(y);
        }
    }
    return 0;
}

// Block-scaled product with a tensor-wide codebook of 2^bits bf16 centroids and
// scales[N][K/B] (bf16).  K must be a multiple of B.  deferred = 0: c*s*x summed
// over k ascending; deferred = 1: per-block sums of c*x, each multiplied by its
// scale, blocks ascending.  A = sum_k |c*s*x| either way.  Rows [n0, n1).
int oracle_gemm_blockscaled(const uint32_t* packed, const uint16_t* codebook, const uint16_t* scales,
                            const uint16_t* X, int64_t N, int64_t K, int bits, int64_t B, int64_t M,
                            int64_t n0, int64_t n1, int deferred, double* Y, double* A,
                            uint16_t* Ybf16) {
    if (!bits_ok(bits) || N < 0 || K < 0 || M < 0 || B < 1 || K % B != 0 || n0 < 0 || n1 > N || n0 > n1)
        return 1;
    const int64_t wpr = words_per_row(bits, K);
    const int64_t G = K / B;
    std::vector<double> c(static_cast<size_t>(K));
    for (int64_t n = n0; n < n1; ++n) {
        for (int64_t k = 0; k < K; ++k)
            c[k] = bf16_to_double(codebook[read_field(packed + n * wpr, k, bits)]);
        for (int64_t m = 0; m < M; ++m) {
            double y = 0.0, a = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                const double s = bf16_to_double(scales[n * G + g]);
                double z = 0.0;
                for (int64_t k = g * B; k < (g + 1) * B; ++k) {
                    const double x = bf16_to_double(X[m * K + k]);
                    if (deferred) z += c[k] * x;
                    else y += (c[k] * s) * x;
                    a += std::fabs((c[k] * s) * x);
                }
                if (deferred) y += z * s;
            }
            Y[m * N + n] = y;
            if (A) A[m * N + n] = a;
            if (Ybf16) Ybf16[m * N + n] = oracle_round_bf16(y);
        }
    }
    return 0;
}

// Dense weights of the block-scaled format (the separate-dequantise route the paper recommends
// for large batches, App. E "Model benchmarks"; the reference routine of "Kernel implementations"
// materialises the same matrix): Wd[n][k] = bf16( codebook[idx[n][k]] * scale[n][k / B] ).
// The product of two bf16 values is exact in fp64, so this is one rounding (to nearest even).
int oracle_dequant_blockscaled(const uint32_t* packed, const uint16_t* codebook, const uint16_t* scales,
                               int64_t N, int64_t K, int bits, int64_t B, uint16_t* Wd) {
    if (!packed || !codebook || !scales || !Wd || !bits_ok(bits) || N < 0 || K < 1 || B < 1 || K % B != 0) return 1;
    const int64_t wpr = words_per_row(bits, K), G = K / B;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const double c = bf16_to_double(codebook[read_field(packed + n * wpr, k, bits)]);
            Wd[n * K + k] = oracle_round_bf16(c * bf16_to_double(scales[n * G + k / B]));
        }
    return 0;
}

// SwiGLU of a decoder MLP's gate and up projections (Shazeer-style gated unit with the SiLU
// activation, as in the Llama-3 architecture the paper benchmarks, App. E "Model benchmarks"):
// y[i] = silu(g[i]) * u[i], silu(t) = t / (1 + exp(-t)), on fp64 inputs.
int oracle_swiglu(const double* gate, const double* up, int64_t n, double* y) {
    if (n < 0) return 1;
    for (int64_t i = 0; i < n; ++i) y[i] = gate[i] / (1.0 + std::exp(-gate[i])) * up[i];
    return 0;
}

// RMSNorm in front of a product (the normalisation of the Llama-3 decoder layers the paper
// benchmarks, App. E "Model benchmarks"; the paper fixes none of its arithmetic).  The plain
// definition, written out: r = 1 / sqrt(mean(x^2) + eps) and
//     xn[k] = bf16( x[k] * r * g[k] )
// evaluated in fp64 and rounded ONCE to the method's activation type; the product that follows
// sees xn.  r is returned as well, for the pins.  (A kernel may let the scalar r commute with the
// sum and apply it to the fp32 result instead; that is an approximation of this definition, and
// the parity tests bound it.)
int oracle_rmsnorm(const uint16_t* x, const uint16_t* g, int64_t K, double eps, uint16_t* xn, double* r) {
    if (!x || !g || !xn || !r || K < 1 || !(eps >= 0.0)) return 1;
    double ss = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        const double v = bf16_to_double(x[k]);
        ss += v * v;
    }
    *r = 1.0 / std::sqrt(ss / static_cast<double>(K) + eps);
    for (int64_t k = 0; k < K; ++k) xn[k] = oracle_round_bf16(bf16_to_double(x[k]) * *r * bf16_to_double(g[k]));
    return 0;
}

// Dense bf16 matrix times bf16 vectors, the unquantised baseline the paper compares
// against (App. E, Table of m = 1, h = 8192, the 16-bit rows): Y[m][n] = sum_k W[n][k]*X[m][k]
// in fp64, k ascending.  W is N x K bf16 bit patterns, row-major.
int oracle_gemm_dense(const uint16_t* W, const uint16_t* X, int64_t N, int64_t K, int64_t M,
                      int64_t n0, int64_t n1, double* Y, double* A, uint16_t* Ybf16) {
    if (N < 0 || K < 0 || M < 0 || n0 < 0 || n1 > N || n0 > n1) return 1;
    for (int64_t n = n0; n < n1; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double y = 0.0, a = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double t = bf16_to_double(W[n * K + k]) * bf16_to_double(X[m * K + k]);
                y += t;
                a += std::fabs(t);
            }
            Y[m * N + n] = y;
            if (A) A[m * N + n] = a;
            if (Ybf16) Ybf16[m * N + n] = oracle_round_bf16(y);
        }
    return 0;
}

}  // extern "C"
