// kmq_quantize_oracle.cpp -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, slow, single-threaded CPU statement of the quantiser that PRODUCES the
// k-means weight formats (paper, Sec. 2.1 "Rounding to nearest centroids", the
// quantiser f_c(x) = argmin_{c_i} |x - c_i| with centroids from 1-D k-means
// clustering (Lloyd); "Block formats"; Sec. 2.2 "Nonlinear k-means quantization":
// centroids in [-1, 1] computed per weight tensor on the normalised weights, one
// 16-bit scale per block of 64 elements).  Only tests may call it; it shares no
// source, header, table or helper with the GPU library.
//
// The paper names the algorithm and leaves its details open.  The reading taken
// here, identical on the GPU side by specification and not by shared code:
//
//   * Lloyd's iteration in fp64 on sorted centroids c_0 <= ... <= c_{C-1}, C = 2^b:
//       assignment  a(v) = number of boundaries m_i = (c_i + c_{i+1}) / 2, i = 0..C-2,
//                   with v > m_i   (nearest centroid; a value exactly on a boundary
//                   goes to the lower cluster)
//       update      c_j = (sum of the members of cluster j) / (their number);
//                   a cluster without members keeps its centroid
//     for exactly `iters` rounds (no early stop: a converged state is a fixed point
//     of the round, so further rounds change nothing).
//   * Start: C points evenly spaced in the data's range [lo, hi],
//     c_i = lo + (i + 1/2) (hi - lo) / C  (per row: the row's min and max; normalised
//     weights: lo = -1, hi = 1).
//   * Stored codebook: the centroids rounded to bf16 (round to nearest even); the
//     indices are the assignment against the STORED codebook, so that dequantising
//     returns the nearest stored centroid.
//   * Block scales (paper: lambda proportional to absmax, stored in 16 bits):
//     scale = absmax of the block (a bf16 value, so stored exactly); normalised
//     weight v = w / scale in fp64, v = 0 where the scale is 0.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

double bf16_value(uint16_t h) {
    const uint32_t u = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

// Round to nearest even to 8 significant bits, decided on the double itself (no intermediate
// fp32 rounding).  Finite inputs in bf16's normal range, which is all a centroid can be.
uint16_t round_to_bf16(double c) {
    if (c == 0.0) return std::signbit(c) ? 0x8000 : 0x0000;
    const double a = std::fabs(c);
    int e;
    const double m = std::frexp(a, &e);          // a = m * 2^e, m in [0.5, 1)
    // 8 significant bits: scale so that the integer part holds them.
    const double scaled = std::ldexp(m, 8);      // in [128, 256)
    double r = std::nearbyint(scaled);           // default rounding mode: to nearest even
    int e2 = e - 8;
    if (r == 256.0) { r = 128.0; e2 += 1; }
    const float f = static_cast<float>(std::ldexp(r, e2));   // exact: 8 bits (normal range)
    uint32_t u;
    std::memcpy(&u, &f, sizeof u);
    u = (u & 0x7FFFFFFFu) | (std::signbit(c) ? 0x80000000u : 0u);
    return static_cast<uint16_t>(u >> 16);
}

int assign(const double* c, int C, double v) {
    int a = 0;
    for (int i = 0; i + 1 < C; ++i)
        if (v > 0.5 * (c[i] + c[i + 1])) ++a;    // sorted centroids: the count of boundaries below v
    return a;
}

// `iters` Lloyd rounds over v[0..n), centroids c[0..C) updated in place.
void lloyd(const double* v, int64_t n, double* c, int C, int iters) {
    std::vector<double> sum(C);
    std::vector<int64_t> cnt(C);
    for (int t = 0; t < iters; ++t) {
        for (int j = 0; j < C; ++j) { sum[j] = 0.0; cnt[j] = 0; }
        for (int64_t k = 0; k < n; ++k) {
            const int a = assign(c, C, v[k]);
            sum[a] += v[k];
            cnt[a] += 1;
        }
        for (int j = 0; j < C; ++j)
            if (cnt[j] > 0) c[j] = sum[j] / static_cast<double>(cnt[j]);
    }
}

}  // namespace

extern "C" {

// Exposed so that tests can pin the rounding against an independent conversion.
uint16_t oracle_quantize_round_bf16(double c) { return round_to_bf16(c); }

// The bare iteration on caller-supplied values and start centroids (tests pin it against
// a library k-means and against brute force).
int oracle_lloyd(const double* v, int64_t n, double* c, int C, int iters) {
    if (!v || !c || n < 0 || C < 1 || iters < 0) return 1;
    lloyd(v, n, c, C, iters);
    return 0;
}

// One codebook per row, no scales (the benchmark contract's format).
//   W        N x K bf16 bit patterns
//   idx      N x K uint8 out, codebook N x 2^bits bf16 out (sorted ascending per row)
//   centroid N x 2^bits fp64 out (before rounding; may be NULL)
//   sse      N fp64 out: sum_k (w - dequantised w)^2 per row (may be NULL)
int oracle_quantize_rows(const uint16_t* W, int64_t N, int64_t K, int bits, int iters,
                         uint8_t* idx, uint16_t* codebook, double* centroid, double* sse) {
    if (!W || !idx || !codebook || N < 1 || K < 1 || bits < 1 || bits > 4 || iters < 0) return 1;
    const int C = 1 << bits;
    std::vector<double> v(K), c(C), cb(C);
    for (int64_t n = 0; n < N; ++n) {
        double lo = bf16_value(W[n * K]), hi = lo;
        for (int64_t k = 0; k < K; ++k) {
            v[k] = bf16_value(W[n * K + k]);
            if (v[k] < lo) lo = v[k];
            if (v[k] > hi) hi = v[k];
        }
        for (int i = 0; i < C; ++i) c[i] = lo + (i + 0.5) * (hi - lo) / C;
        lloyd(v.data(), K, c.data(), C, iters);
        for (int i = 0; i < C; ++i) {
            codebook[n * C + i] = round_to_bf16(c[i]);
            cb[i] = bf16_value(codebook[n * C + i]);
            if (centroid) centroid[n * C + i] = c[i];
        }
        double e2 = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const int a = assign(cb.data(), C, v[k]);
            idx[n * K + k] = static_cast<uint8_t>(a);
            e2 += (v[k] - cb[a]) * (v[k] - cb[a]);
        }
        if (sse) sse[n] = e2;
    }
    return 0;
}

// The paper's format: scale per block of B elements along K, one codebook for the tensor.
//   scales   N x K/B bf16 out; codebook 2^bits bf16 out; idx N x K uint8 out
//   centroid 2^bits fp64 out (may be NULL)
//   vnorm    N x K fp64 out, the normalised weights the clustering saw (may be NULL)
int oracle_quantize_blockscaled(const uint16_t* W, int64_t N, int64_t K, int bits, int64_t B, int iters,
                                uint8_t* idx, uint16_t* codebook, uint16_t* scales, double* centroid,
                                double* vnorm) {
    if (!W || !idx || !codebook || !scales || N < 1 || K < 1 || B < 1 || K % B != 0 || bits < 1 || bits > 4 ||
        iters < 0)
        return 1;
    const int C = 1 << bits;
    const int64_t G = K / B;
    std::vector<double> v(static_cast<size_t>(N) * K);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t g = 0; g < G; ++g) {
            uint16_t best = 0;                     // bit pattern of the largest magnitude (sign cleared)
            for (int64_t k = g * B; k < (g + 1) * B; ++k) {
                const uint16_t mag = W[n * K + k] & 0x7FFF;
                if (bf16_value(mag) > bf16_value(best)) best = mag;
            }
            scales[n * G + g] = best;
            const double s = bf16_value(best);
            for (int64_t k = g * B; k < (g + 1) * B; ++k)
                v[n * K + k] = s > 0.0 ? bf16_value(W[n * K + k]) / s : 0.0;
        }
    std::vector<double> c(C), cb(C);
    for (int i = 0; i < C; ++i) c[i] = -1.0 + (2 * i + 1) / static_cast<double>(C);
    lloyd(v.data(), N * K, c.data(), C, iters);
    for (int i = 0; i < C; ++i) {
        codebook[i] = round_to_bf16(c[i]);
        cb[i] = bf16_value(codebook[i]);
        if (centroid) centroid[i] = c[i];
    }
    for (int64_t i = 0; i < N * K; ++i) {
        idx[i] = static_cast<uint8_t>(assign(cb.data(), C, v[i]));
        if (vnorm) vnorm[i] = v[i];
    }
    return 0;
}

}  // extern "C"
