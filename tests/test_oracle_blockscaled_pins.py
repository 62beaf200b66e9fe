"""Pins for the oracle's block-scaled entry point (the paper's own weight format:
Sec. 2.2 "Nonlinear k-means quantization"; App. E "Kernel implementations").
CPU only.  Each pin checks the oracle against something other than itself."""
import os

import numpy as np
import pytest

import oracle
from paper_2602_15563_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
ONE = np.uint16(0x3F80)


def _bf16(vals):
    h = synth.f32_to_bf16(np.asarray(vals, dtype=np.float32))
    assert np.array_equal(synth.bf16_to_f32(h), np.asarray(vals, dtype=np.float32)), "not exact in bf16"
    return h


def _case(seed, N, K, bits, M, block=64):
    idx = synth.make_indices(seed, 0, N, K, bits)
    cb = synth.make_shared_codebook(seed, 0, bits)
    sc = synth.make_scales(seed, 0, N, K, block)
    X = synth.make_x(seed, 0, M, K)
    return idx, cb, sc, X


def _dense(idx, cb, sc, block):
    """Dense fp64 weights from the UNPACKED indices: centroid * scale of the element's block."""
    N, K = idx.shape
    c = synth.bf16_to_f64(cb)[idx]
    s = np.repeat(synth.bf16_to_f64(sc), block, axis=1)
    return c * s


def test_hand_computed_examples():
    n = 0
    for line in open(os.path.join(HERE, "golden", "blockscaled_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = [p.split() for p in line.split("|")]
        bits, B = int(f[0][0]), int(f[0][1])
        cb = _bf16([float(v) for v in f[1]])
        idx = np.array([[int(v) for v in f[2]]], dtype=np.uint8)
        sc = _bf16([float(v) for v in f[3]]).reshape(1, -1)
        x = _bf16([float(v) for v in f[4]])
        y_want, a_want = float(f[5][0]), float(f[6][0])
        K = idx.shape[1]
        for deferred in (False, True):
            Y, A, Yb = oracle.gemm_blockscaled(oracle.pack(idx, bits), cb, sc, x, K, bits, block=B, deferred=deferred)
            assert Y[0] == y_want and A[0] == a_want
            assert synth.bf16_to_f32(Yb)[0] == np.float32(y_want)
        n += 1
    assert n == 3


@pytest.mark.parametrize("bits", (1, 2, 3, 4))
def test_unit_scales_and_replicated_codebook_reduce_to_the_per_row_product(bits):
    """scale = 1 everywhere and every row given the same codebook: the block-scaled
    product IS the per-row-codebook product, term by term (c*1*x = c*x), so bit-equal."""
    N, K, M = 9, 320, 3
    idx, cb, _, X = _case(11 + bits, N, K, bits, M)
    p = oracle.pack(idx, bits)
    ones = np.full((N, K // 64), ONE, dtype=np.uint16)
    Y, A, Yb = oracle.gemm_blockscaled(p, cb, ones, X, K, bits)
    Y0, A0, Yb0 = oracle.gemm(p, np.tile(cb, (N, 1)), X, K, bits)
    assert np.array_equal(Y, Y0) and np.array_equal(A, A0) and np.array_equal(Yb, Yb0)


@pytest.mark.parametrize("bits", (1, 2, 4))
def test_byte_view_of_the_stream_with_partial_sums_per_byte(bits):
    """The special case that meets the paper's uint8 element stream (App. E "Kernel implementations"): for
    1, 2 and 4 bits the little-endian bytes of the packed words hold 8/bits whole elements each, first
    element in the low bits.  Checked with a formulation of its own: for every byte POSITION of a row and
    every byte VALUE, the partial product of the 8/bits centroids that value selects with the activations
    at that position is tabulated once (an activation-side table); an output is then the sum, over the byte
    positions, of the tabulated entry its row's byte selects, times the scale of the block the byte lies in."""
    N, K, M = 12, 256, 2
    idx, cb, sc, X = _case(23 + bits, N, K, bits, M)
    p = oracle.pack(idx, bits)
    per_byte = 8 // bits
    field = (1 << bits) - 1
    centroid = synth.bf16_to_f64(cb)
    act = synth.bf16_to_f64(X)
    scale = synth.bf16_to_f64(sc)
    stream = p.view(np.uint8).reshape(N, -1)[:, :K // per_byte]          # byte j of row n
    # partial[m, j, v] = sum over the elements e of byte position j of centroid[field e of v] * act[m, j*per_byte + e]
    selected = np.array([[centroid[(v >> (e * bits)) & field] for e in range(per_byte)] for v in range(256)])    # [v][e]
    partial = np.einsum("mje,ve->mjv", act.reshape(M, K // per_byte, per_byte), selected)
    block_of_byte = (np.arange(K // per_byte) * per_byte) // 64
    want = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            picked = partial[m, np.arange(K // per_byte), stream[n]]                                              # one entry per byte
            want[m, n] = np.sum(picked * scale[n, block_of_byte])
    Y, A, _ = oracle.gemm_blockscaled(p, cb, sc, X, K, bits)
    assert np.all(np.abs(Y - want) <= 1e-13 * A)


@pytest.mark.parametrize("bits", (1, 2, 3, 4))
def test_brute_force_from_unpacked_indices_and_deferred_variant(bits):
    N, K, M, B = 7, 192, 2, 64
    idx, cb, sc, X = _case(31 + bits, N, K, bits, M, B)
    W = _dense(idx, cb, sc, B)
    x = synth.bf16_to_f64(X)
    want = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):                                   # same order as the immediate form
                acc += W[n, k] * x[m, k]
            want[m, n] = acc
    p = oracle.pack(idx, bits)
    Y, A, _ = oracle.gemm_blockscaled(p, cb, sc, X, K, bits, block=B)
    assert np.array_equal(Y, want)
    # deferred scaling (App. E): block sums of c*x times the block's scale
    c = synth.bf16_to_f64(cb)[idx].reshape(N, K // B, B)
    z = np.einsum("mGg,hGg->mhG", x.reshape(M, K // B, B), c)
    want_d = np.einsum("mhG,hG->mh", z, synth.bf16_to_f64(sc))
    Yd, Ad, _ = oracle.gemm_blockscaled(p, cb, sc, X, K, bits, block=B, deferred=True)
    assert np.all(np.abs(Yd - want_d) <= 1e-13 * A) and np.array_equal(Ad, A)
    assert np.all(np.abs(Yd - Y) <= 1e-13 * A)


def test_only_the_scaled_block_contributes():
    """All scales zero except block g of row r: y[r] is that block's sum alone, other rows 0.
    A wrong block boundary or a transposed scale index fails this."""
    bits, N, K, B = 2, 5, 256, 64
    idx, cb, sc, X = _case(5, N, K, bits, 1, B)
    x = synth.bf16_to_f64(X)[0]
    c = synth.bf16_to_f64(cb)
    for r, g in ((0, 0), (3, 2), (4, 3)):
        z = np.zeros_like(sc)
        z[r, g] = sc[r, g]
        Y, _, _ = oracle.gemm_blockscaled(oracle.pack(idx, bits), cb, z, X[0], K, bits, block=B)
        want = sum(c[idx[r, k]] * synth.bf16_to_f64(sc[r, g:g + 1])[0] * x[k] for k in range(g * B, (g + 1) * B))
        assert abs(Y[r] - want) <= 1e-15 * abs(want) + 1e-300
        assert not np.delete(Y, r).any()


def test_power_of_two_scaling_is_exact():
    bits, N, K = 4, 6, 128
    idx, cb, sc, X = _case(9, N, K, bits, 2)
    p = oracle.pack(idx, bits)
    Y, A, _ = oracle.gemm_blockscaled(p, cb, sc, X, K, bits)
    sc4 = (sc + np.uint16(2 << 7)).astype(np.uint16)              # bf16 exponent + 2: every scale times 4
    Y4, A4, _ = oracle.gemm_blockscaled(p, cb, sc4, X, K, bits)
    assert np.array_equal(Y4, 4.0 * Y) and np.array_equal(A4, 4.0 * A)


def test_rows_argument_and_bad_block():
    bits, N, K = 2, 10, 128
    idx, cb, sc, X = _case(3, N, K, bits, 1)
    p = oracle.pack(idx, bits)
    Y, _, _ = oracle.gemm_blockscaled(p, cb, sc, X[0], K, bits)
    Yr, _, _ = oracle.gemm_blockscaled(p, cb, sc, X[0], K, bits, rows=(4, 7))
    assert np.array_equal(Yr[4:7], Y[4:7]) and np.isnan(Yr[:4]).all() and np.isnan(Yr[7:]).all()
    with pytest.raises(ValueError):
        oracle.gemm_blockscaled(p, cb, sc[:, :1], X[0], K, bits, block=96)


def test_scale_generator_matches_the_block_maximum_it_stands_for():
    """make_scales inverts the distribution of max |z_j| over 64 normal samples: compare
    its quantiles with a literal simulation."""
    s = synth.bf16_to_f64(synth.make_scales(1, 0, 256, 64 * 64))
    z = np.abs(np.random.default_rng(0).normal(0.0, synth.SIGMA_W, size=(s.size, 64))).max(axis=1)
    for q in (0.1, 0.5, 0.9):
        assert abs(np.quantile(s, q) - np.quantile(z, q)) < 0.03 * np.quantile(z, q)
    cb = synth.bf16_to_f64(synth.make_shared_codebook(1, 0, 4))
    assert np.all(np.diff(cb) >= 0) and np.all(np.abs(cb) <= 1.0)


def test_dense_weights_of_the_format():
    """bf16(codebook[idx] * scale): one rounding of an exact product, re-stated with numpy's fp32 product
    (exact for two bf16 factors) and an independent rounding; unit scales give the bare centroids; and the
    dense product of these weights is the block-scaled product up to that rounding."""
    bits, N, K = 3, 9, 640
    idx = synth.make_indices(31, 0, N, K, bits)
    cb, sc = synth.make_shared_codebook(31, 0, bits), synth.make_scales(31, 0, N, K)
    packed = oracle.pack(idx, bits)
    Wd = oracle.dequant_blockscaled(packed, cb, sc, K, bits)
    want = synth.f32_to_bf16(synth.bf16_to_f32(cb)[idx] * np.repeat(synth.bf16_to_f32(sc), 64, axis=1))
    assert np.array_equal(Wd, want)
    ones = np.full_like(sc, 0x3F80)
    assert np.array_equal(oracle.dequant_blockscaled(packed, cb, ones, K, bits), cb[idx])
    X = synth.make_x(31, 0, 2, K)
    Yb, Ab, _ = oracle.gemm_blockscaled(packed, cb, sc, X, K, bits)
    Yd, _, _ = oracle.gemm_dense(Wd, X)
    assert np.all(np.abs(Yb - Yd) <= 2.0 ** -8 * Ab)        # each weight moved by at most half a bf16 ulp
    assert np.any(Yb != Yd)
