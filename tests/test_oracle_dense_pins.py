"""Pins for the oracle's dense bf16 product (the unquantised baseline of the paper's
App. E micro-benchmark table), SwiGLU, and RMSNorm / residual around a product.  CPU only."""
import numpy as np
import pytest

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


# ---- RMSNorm in front of a product, residual behind (the fused decoder call's definition) ----

def test_rmsnorm_against_torch_and_numpy():
    import torch
    g0 = np.random.default_rng(21)
    for K, eps in [(64, 1e-5), (3072, 1e-6), (515, 0.0), (8192, 1e-5)]:
        x = synth.make_x(21, K, 1, K)[0]
        g = synth.f32_to_bf16((1.0 + 0.1 * g0.standard_normal(K)).astype(np.float32))
        xn, r = oracle.rmsnorm(x, g, eps)
        xd, gd = synth.bf16_to_f64(x), synth.bf16_to_f64(g)
        # the scalar: torch's rms_norm of x with unit weights is x * r
        ref = torch.nn.functional.rms_norm(torch.from_numpy(xd), (K,), eps=eps).numpy()
        nz = xd != 0
        np.testing.assert_allclose(ref[nz] / xd[nz], r, rtol=1e-12)
        assert abs(r - 1.0 / np.sqrt(np.mean(xd * xd) + eps)) <= 1e-14 * r
        # the activations: the library's weighted rms_norm in fp64, rounded once to bf16.  torch's value
        # and the oracle's can differ in the last bits of the fp64 product, which moves the rounding only
        # for values within 1e-12 of a tie: every element must be one of the (at most two) bf16 values
        # that round-to-nearest could give for torch's value, and all but a handful must be equal.
        full = torch.nn.functional.rms_norm(torch.from_numpy(xd), (K,), weight=torch.from_numpy(gd), eps=eps)
        want = full.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)      # torch's own nearest-even rounding
        xnd = synth.bf16_to_f64(xn)
        assert np.count_nonzero(xn != want) <= 2
        assert np.all(np.abs(xnd - full.numpy()) <= 2.0 ** -8 * np.abs(full.numpy()) * (1 + 1e-9) + 1e-300)    # half an ulp of 8 significant bits


def test_rmsnorm_closed_forms():
    K = 128
    c = synth.f32_to_bf16(np.full(K, 0.75, np.float32))
    one = synth.f32_to_bf16(np.ones(K, np.float32))
    xn, r = oracle.rmsnorm(c, one, 0.25)
    assert r == 1.0 / np.sqrt(0.75 ** 2 + 0.25)
    assert np.array_equal(xn, synth.f32_to_bf16(np.full(K, 0.75 * r, np.float32)))     # 0.75 / sqrt(0.8125) = 0.832..., rounded once
    two = synth.f32_to_bf16(np.full(K, 2.0, np.float32))
    xn2, r2 = oracle.rmsnorm(two, one, 0.0)                                              # mean(x^2) = 4: r = 1/2, xn = 1 exactly
    assert r2 == 0.5 and np.array_equal(xn2, one)
    gains = synth.f32_to_bf16(np.linspace(-2, 2, K).astype(np.float32))
    xn3, _ = oracle.rmsnorm(two, gains, 0.0)                                             # xn = g exactly
    assert np.array_equal(xn3, gains)
    x = synth.make_x(22, 0, 1, K)[0]
    x2 = synth.f32_to_bf16(2.0 * synth.bf16_to_f32(x))                    # exact doubling
    (_, r1), (_, r2) = oracle.rmsnorm(x, one, 0.0), oracle.rmsnorm(x2, one, 0.0)
    assert abs(r1 - 2.0 * r2) <= 1e-15 * r1                                 # scale invariance without eps
    with pytest.raises(ValueError):
        oracle.rmsnorm(x, one, -1.0)


def test_fused_call_is_the_product_with_the_scalar_and_the_residual():
    bits, N, K = 2, 24, 640
    idx = synth.make_indices(23, 0, N, K, bits)
    cb = synth.make_codebook(23, 0, N, bits)
    x = synth.make_x(23, 0, 1, K)
    g = synth.f32_to_bf16((1.0 + 0.2 * np.random.default_rng(23).standard_normal(K)).astype(np.float32))
    res = synth.make_x(23, 1, 1, N)[0]
    packed = oracle.pack(idx, bits)
    Y0, A0, _ = oracle.gemm(packed, cb, x, K, bits)
    Yp, Ap = oracle.gemv_fused(packed, cb, x, K, bits)
    assert np.array_equal(Yp, Y0[0]) and np.array_equal(Ap, A0[0])          # no fusion: the plain product
    Yr, _ = oracle.gemv_fused(packed, cb, x, K, bits, residual=res)
    assert np.array_equal(Yr, Y0[0] + synth.bf16_to_f64(res))
    # dense restatement: W_hat (xn * r) + res, with W_hat from the uint8 indices
    Yf, Af = oracle.gemv_fused(packed, cb, x, K, bits, norm_weight=g, eps=1e-5, residual=res)
    W = np.take_along_axis(synth.bf16_to_f64(cb), idx.astype(np.int64), axis=1)
    import torch
    xd, gd = synth.bf16_to_f64(x[0]), synth.bf16_to_f64(g)
    xn = torch.nn.functional.rms_norm(torch.from_numpy(xd), (K,), weight=torch.from_numpy(gd), eps=1e-5).to(torch.bfloat16).double().numpy()
    np.testing.assert_allclose(Yf, W @ xn + synth.bf16_to_f64(res), rtol=0, atol=1e-12 * Af.max())
    np.testing.assert_allclose(Af, np.abs(W * xn[None, :]).sum(axis=1) + np.abs(synth.bf16_to_f64(res)), rtol=1e-12)
