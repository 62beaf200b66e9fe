"""Pins of the quantiser oracle (1-D k-means / nearest-centroid rounding, paper Sec. 2.1 "Rounding to
nearest centroids" and Sec. 2.2 "Nonlinear k-means quantization") against things other than itself:
a library k-means started from the same centroids, the optimal 1-D clustering by dynamic programming
on tiny inputs, the fixed-point and monotonicity properties of Lloyd's iteration, hand-worked cases of
the tie and empty-cluster rules, exact rational rounding to bf16, numpy re-statements of the scale and
assignment rules, and the error bound that ties the quantised product to the dense one."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2602_15563_amd import synth


def sse_of(v, c):
    c = np.asarray(c, dtype=np.float64)
    return float(np.sum(np.min((v[:, None] - c[None, :]) ** 2, axis=1)))


def grid_start(lo, hi, C):
    return lo + (np.arange(C) + 0.5) * (hi - lo) / C


# ---- Lloyd's iteration -------------------------------------------------------------------------

def test_hand_worked_two_clusters():
    assert np.array_equal(oracle.lloyd([0, 1, 2, 10, 11, 12.0], [1.0, 9.0], 3), [1.0, 11.0])
    # one round from a poor start: boundary 3.5 -> {0,1,2} and {10,11,12}
    assert np.array_equal(oracle.lloyd([0, 1, 2, 10, 11, 12.0], [0.0, 7.0], 1), [1.0, 11.0])
    # zero rounds: the start is returned untouched
    assert np.array_equal(oracle.lloyd([0, 1, 2.0], [0.25, 0.75], 0), [0.25, 0.75])


def test_value_on_a_boundary_goes_to_the_lower_cluster():
    # boundary (0 + 2) / 2 = 1: the value 1 joins cluster 0 -> means 0.5 and 2
    assert np.array_equal(oracle.lloyd([0.0, 2.0, 1.0], [0.0, 2.0], 1), [0.5, 2.0])


def test_empty_cluster_keeps_its_centroid():
    c = oracle.lloyd([0.0, 0.0, 1.0, 1.0], [0.0, 0.5, 1.0, 5.0], 4)
    assert np.array_equal(c, [0.0, 0.5, 1.0, 5.0])


@pytest.mark.parametrize("C,n,seed", [(2, 500, 0), (4, 2000, 1), (8, 4096, 2), (16, 20000, 3)])
def test_against_library_kmeans(C, n, seed):
    """scikit-learn's Lloyd from the same start: same centroids to rounding (no cluster runs empty here,
    the one case where the library does something else)."""
    from sklearn.cluster import KMeans
    g = np.random.default_rng(seed)
    v = g.normal(0, 0.02, size=n) * g.uniform(0.5, 2.0)
    c0 = grid_start(v.min(), v.max(), C)
    for iters in (1, 7, 40):
        km = KMeans(n_clusters=C, init=c0.reshape(-1, 1), n_init=1, max_iter=iters, tol=0.0, algorithm="lloyd")
        km.fit(v.reshape(-1, 1))
        ours = oracle.lloyd(v, c0, iters)
        assert np.all(np.diff(ours) > 0)
        np.testing.assert_allclose(ours, km.cluster_centers_.ravel(), rtol=0, atol=1e-12 * np.abs(v).max() * n)


def optimal_sse(v, C):
    """Optimal 1-D C-clustering of sorted values by dynamic programming over contiguous segments."""
    v = np.sort(v)
    n = len(v)
    p1 = np.concatenate([[0.0], np.cumsum(v)])
    p2 = np.concatenate([[0.0], np.cumsum(v * v)])

    def cost(i, j):   # v[i:j]
        s = p1[j] - p1[i]
        return (p2[j] - p2[i]) - s * s / (j - i)
    best = np.full((C + 1, n + 1), np.inf)
    best[0, 0] = 0.0
    for k in range(1, C + 1):
        for j in range(k, n + 1):
            best[k, j] = min(best[k - 1, i] + cost(i, j) for i in range(k - 1, j))
    return best[C, n]


@pytest.mark.parametrize("seed", range(6))
def test_never_better_than_the_optimum_and_equal_on_separated_data(seed):
    g = np.random.default_rng(100 + seed)
    C = int(g.choice([2, 3, 4]))
    v = g.normal(0, 1, size=14)
    c = oracle.lloyd(v, grid_start(v.min(), v.max(), C), 50)
    opt = optimal_sse(v, C)
    assert sse_of(v, c) >= opt - 1e-12
    # well-separated equal-width clumps on the start grid: Lloyd finds the optimum
    centres = np.arange(C) * 10.0 + 5.0
    w = np.concatenate([m + g.uniform(-1, 1, size=5) for m in centres])
    c = oracle.lloyd(w, grid_start(0.0, 10.0 * C, C), 5)
    assert abs(sse_of(w, c) - optimal_sse(w, C)) <= 1e-9


@pytest.mark.parametrize("C", [2, 4, 8, 16])
def test_objective_never_increases_and_fixed_point(C):
    g = np.random.default_rng(C)
    v = np.concatenate([g.normal(0, 0.02, 3000), g.normal(0.05, 0.005, 500)])
    c0 = grid_start(v.min(), v.max(), C)
    prev = sse_of(v, c0)
    for t in range(1, 30):
        cur = sse_of(v, oracle.lloyd(v, c0, t))
        assert cur <= prev + 1e-15
        prev = cur
    c = oracle.lloyd(v, c0, 2000)
    a = np.argmin(np.abs(v[:, None] - c[None, :]), axis=1)
    for j in range(C):                       # converged: every centroid is the mean of its nearest values
        if np.any(a == j):
            assert abs(c[j] - v[a == j].mean()) <= 1e-15 + 1e-13 * abs(c[j])
    assert np.array_equal(oracle.lloyd(v, c, 1), c)


def test_as_many_distinct_values_as_centroids_gives_zero_error():
    vals = np.array([-0.75, -0.25, 0.25, 0.75])
    v = np.repeat(vals, [3, 1, 5, 2])
    c = oracle.lloyd(v, grid_start(-1.0, 1.0, 4), 1)
    assert np.array_equal(c, vals) and sse_of(v, c) == 0.0


# ---- rounding of the centroids -----------------------------------------------------------------

def _bf16_exact(h):
    return Fraction(float(synth.bf16_to_f64(np.array([h], np.uint16))[0]))


def test_rounding_to_bf16_is_nearest_even_in_exact_arithmetic():
    g = np.random.default_rng(5)
    xs = list(g.normal(0, 0.02, 300)) + list(g.uniform(-1, 1, 300)) + [1.0, -1.0, 0.0, 0.00390625, 1.00390625,
                                                                     1.01171875, 0.998046875, -0.5009765625]
    for x in xs:
        h = oracle.quantize_round_bf16(x)
        got, fx = _bf16_exact(h), Fraction(x)
        if x == 0:
            assert h == 0
            continue
        mag = h & 0x7FFF
        lo, hi = _bf16_exact((h & 0x8000) | (mag - 1)) if mag > 0 else None, _bf16_exact((h & 0x8000) | (mag + 1))
        for nb in (lo, hi):
            if nb is None:
                continue
            assert abs(got - fx) <= abs(nb - fx)
            if abs(got - fx) == abs(nb - fx):          # a tie: the even significand wins
                assert h & 1 == 0
    # the three tie cases above, spelled out: 1 + 2^-8 -> 1 (even), 1 + 3*2^-8 -> 1 + 2^-6 (even)
    assert oracle.quantize_round_bf16(1.00390625) == 0x3F80 and oracle.quantize_round_bf16(1.01171875) == 0x3F82
    assert oracle.quantize_round_bf16(0.998046875) == 0x3F80    # 1 - 2^-9: tie between 0x3F7F and 0x3F80


# ---- per-row quantiser ---------------------------------------------------------------------------

@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_rows_restated_in_numpy(bits):
    C, N, K, iters = 1 << bits, 5, 777, 12
    W = synth.make_dense_weights(11, bits, N, K)
    idx, cb, cen, sse = oracle.quantize_rows(W, bits, iters)
    v = synth.bf16_to_f64(W)
    for n in range(N):
        c = oracle.lloyd(v[n], grid_start(v[n].min(), v[n].max(), C), iters)
        assert np.array_equal(cen[n], c)
        assert [oracle.quantize_round_bf16(x) for x in c] == list(cb[n])
        cbv = synth.bf16_to_f64(cb[n])
        assert np.all(np.diff(cbv) >= 0)
        d = np.abs(v[n][:, None] - cbv[None, :])
        assert np.array_equal(idx[n], np.argmin(d, axis=1))      # nearest stored centroid, first of equals
        assert abs(sse[n] - np.sum(np.min(d, axis=1) ** 2)) <= 1e-12 * sse[n]
    assert idx.max() < C


def test_rows_error_shrinks_with_bits_and_beats_a_uniform_grid():
    W = synth.make_dense_weights(12, 0, 8, 4096)
    v = synth.bf16_to_f64(W)
    last = None
    for bits in (1, 2, 3, 4):
        _, cb, _, sse = oracle.quantize_rows(W, bits, 25)
        if last is not None:
            assert np.all(sse < last)
        last = sse
        for n in range(8):
            grid = grid_start(v[n].min(), v[n].max(), 1 << bits)
            assert sse[n] <= sse_of(v[n], grid)


def test_rows_feed_the_product_oracle_within_the_quantisation_error():
    """Quantise, pack, multiply: the result differs from the dense product by at most
    ||w - w_hat|| * ||x|| per row (Cauchy-Schwarz), and the dequantised weights are the stored centroids."""
    bits, N, K = 3, 6, 1024
    W = synth.make_dense_weights(13, 0, N, K)
    X = synth.make_x(13, 0, 2, K)
    idx, cb, _, sse = oracle.quantize_rows(W, bits, 20)
    packed = oracle.pack(idx, bits)
    Yq, _, _ = oracle.gemm(packed, cb, X, K, bits)
    Yd, _, _ = oracle.gemm_dense(W, X)
    xn = np.linalg.norm(synth.bf16_to_f64(X), axis=1)
    assert np.all(np.abs(Yq - Yd) <= np.sqrt(sse)[None, :] * xn[:, None] * (1 + 1e-12))
    assert np.any(np.abs(Yq - Yd) > 0)
    assert np.array_equal(oracle.dequant(packed, cb, K, bits), np.take_along_axis(cb, idx.astype(np.int64), axis=1))


# ---- the paper's format: block scales, one codebook per tensor -----------------------------------

@pytest.mark.parametrize("bits", [1, 2, 4])
def test_blockscaled_restated_in_numpy(bits):
    C, N, K, iters = 1 << bits, 6, 512, 15
    W = synth.make_dense_weights(14, bits, N, K)
    W[2, 64:128] = 0                       # an all-zero block: scale 0, normalised weights 0
    W[3, 5] |= 0x8000                      # signs do not matter to the scale
    idx, cb, sc, cen, vn = oracle.quantize_blockscaled(W, bits, iters)
    w = synth.bf16_to_f64(W)
    s = np.abs(w).reshape(N, K // 64, 64).max(axis=2)
    assert np.array_equal(synth.bf16_to_f64(sc), s)               # absmax is itself a bf16 value
    with np.errstate(divide="ignore", invalid="ignore"):
        v = np.where(np.repeat(s, 64, axis=1) > 0, w / np.repeat(s, 64, axis=1), 0.0)
    assert np.array_equal(vn, v) and np.abs(v).max() == 1.0
    c = oracle.lloyd(v.ravel(), -1.0 + (2 * np.arange(C) + 1) / C, iters)
    assert np.array_equal(cen, c) and np.all(np.abs(c) <= 1.0)
    assert [oracle.quantize_round_bf16(x) for x in c] == list(cb)
    cbv = synth.bf16_to_f64(cb)
    assert np.array_equal(idx, np.argmin(np.abs(v[:, :, None] - cbv[None, None, :]), axis=2))


def test_blockscaled_feeds_the_product_oracle():
    bits, N, K = 4, 4, 512
    W = synth.make_dense_weights(15, 0, N, K)
    X = synth.make_x(15, 0, 1, K)
    idx, cb, sc, _, vn = oracle.quantize_blockscaled(W, bits, 20)
    Yq, _, _ = oracle.gemm_blockscaled(oracle.pack(idx, bits), cb, sc, X, K, bits)
    Yd, _, _ = oracle.gemm_dense(W, X)
    w_hat = synth.bf16_to_f64(cb)[idx] * np.repeat(synth.bf16_to_f64(sc), 64, axis=1)
    err = np.linalg.norm(synth.bf16_to_f64(W) - w_hat, axis=1)
    assert np.all(np.abs(Yq - Yd) <= err[None, :] * np.linalg.norm(synth.bf16_to_f64(X)) * (1 + 1e-12))
    # 16 levels on normalised weights: relative error of the reconstruction well under 10 %
    assert np.all(err / np.linalg.norm(synth.bf16_to_f64(W), axis=1) < 0.1)


def test_bad_arguments():
    W = synth.make_dense_weights(1, 0, 2, 64)
    with pytest.raises(ValueError):
        oracle.quantize_rows(W, 5, 3)
    with pytest.raises(ValueError):
        oracle.quantize_blockscaled(W[:, :63], 2, 3)
