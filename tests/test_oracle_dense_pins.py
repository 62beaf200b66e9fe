"""Pins for the oracle's dense bf16 product (the unquantised baseline of the paper's
App. E micro-benchmark table).  CPU only."""
import numpy as np

import oracle
from paper_2602_15563_amd import synth


def test_dense_product_equals_numpy_and_explicit_loops():
    g = np.random.default_rng(3)
    N, K, M = 7, 45, 3
    W = synth.f32_to_bf16(g.normal(0, 0.02, size=(N, K)).astype(np.float32))
    X = synth.f32_to_bf16(g.normal(0, 1, size=(M, K)).astype(np.float32))
    Y, A, Yb = oracle.gemm_dense(W, X)
    w, x = synth.bf16_to_f64(W), synth.bf16_to_f64(X)
    want = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += w[n, k] * x[m, k]
            want[m, n] = acc
    assert np.array_equal(Y, want)
    assert np.allclose(Y, x @ w.T, rtol=0, atol=1e-15 * np.abs(x) @ np.abs(w).T)
    assert np.allclose(A, np.abs(x) @ np.abs(w).T, rtol=1e-13)
    assert np.array_equal(Yb, np.array([[oracle.round_bf16(v) for v in row] for row in Y], dtype=np.uint16))


def test_quantised_product_is_the_dense_product_of_the_dequantised_weights():
    """Two entry points of the oracle, one statement: Y(packed, codebook) == Y(dense(dequant))."""
    bits, N, K, M = 3, 11, 96, 2
    idx = synth.make_indices(8, 0, N, K, bits)
    cb = synth.make_codebook(8, 0, N, bits)
    X = synth.make_x(8, 0, M, K)
    p = oracle.pack(idx, bits)
    Yq, Aq, _ = oracle.gemm(p, cb, X, K, bits)
    Yd, Ad, _ = oracle.gemm_dense(oracle.dequant(p, cb, K, bits), X)
    assert np.array_equal(Yq, Yd) and np.array_equal(Aq, Ad)


def test_hand_values_and_rows_argument():
    W = synth.f32_to_bf16(np.array([[1, 2, -4], [0.5, 0, 8]], dtype=np.float32))
    x = synth.f32_to_bf16(np.array([3, -1, 0.25], dtype=np.float32))
    Y, A, _ = oracle.gemm_dense(W, x)
    assert Y.tolist() == [0.0, 3.5] and A.tolist() == [6.0, 3.5]
    Yr, _, _ = oracle.gemm_dense(W, x, rows=(1, 2))
    assert np.isnan(Yr[0]) and Yr[1] == 3.5


def test_swiglu_pins():
    """silu by its textbook properties: value at 0 and 1, the identity silu(t) - silu(-t) = t,
    the limits, the slope 1/2 at the origin, and the product with `up`."""
    t = np.array([0.0, 1.0, -1.0, 3.5, -3.5, 30.0, -30.0, 1e-6])
    one = np.ones_like(t)
    y = oracle.swiglu(t, one)
    assert y[0] == 0.0
    assert abs(y[1] - 0.7310585786300049) < 1e-15            # 1 / (1 + e^-1)
    assert np.allclose(oracle.swiglu(t, one) - oracle.swiglu(-t, one), t, rtol=0, atol=1e-15 * (1 + np.abs(t)))
    assert abs(y[5] - 30.0) < 1e-11 and abs(y[6]) < 1e-11
    assert abs(y[7] / 1e-6 - 0.5) < 1e-6
    assert np.array_equal(oracle.swiglu(t, -2.5 * one), -2.5 * y)
    assert abs(oracle.swiglu(np.array([2.0]), np.array([3.0]))[0] - 2.0 / (1.0 + np.exp(-2.0)) * 3.0) < 1e-15
