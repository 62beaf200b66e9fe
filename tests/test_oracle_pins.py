"""Pins for the CPU oracle: everything here checks oracle/ against something
that is not the oracle -- hand-computed words, numpy library routines on the
unpacked uint8 indices, closed forms and invariants.  No GPU involved."""
import math
import os

import numpy as np
import pytest

import oracle
from paper_2602_15563_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
BITS = (1, 2, 3, 4)
EDGE_K = (1, 2, 7, 10, 11, 21, 22, 31, 32, 33, 63, 64, 65, 67, 96, 100, 129)


def _golden_pack_vectors():
    out = []
    with open(os.path.join(GOLDEN, "pack_vectors.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, spec, words = [s.strip() for s in line.split("|")]
            bits, K = (int(t) for t in head.split())
            idx = np.zeros(K, dtype=np.uint8)
            if spec.startswith("seq:"):
                seq = [int(t) for t in spec[4:].split(",")]
                for k in range(K):
                    idx[k] = seq[k % len(seq)]
            else:
                for kv in spec.split(","):
                    k, v = kv.split(":")
                    idx[int(k)] = int(v)
            out.append((bits, K, idx, np.array([int(w, 16) for w in words.split(",")], dtype=np.uint32)))
    return out


def _numpy_pack(idx, bits):
    """Independent packer built on np.packbits (little bit order)."""
    N, K = idx.shape
    bitplanes = ((idx[:, :, None] >> np.arange(bits, dtype=np.uint8)) & 1).astype(np.uint8)
    stream = bitplanes.reshape(N, K * bits)
    wpr = (K * bits + 31) // 32
    padded = np.zeros((N, wpr * 32), dtype=np.uint8)
    padded[:, :K * bits] = stream
    by = np.packbits(padded, axis=1, bitorder="little")          # N x wpr*4 bytes
    return np.ascontiguousarray(by).view("<u4").astype(np.uint32)


def _rand_case(seed, N, K, bits, M, shared=False):
    g = np.random.default_rng(seed)
    idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    cb = synth.f32_to_bf16(g.normal(0, 0.02, size=(N, 1 << bits)).astype(np.float32))
    if shared:
        cb[:] = cb[0]
    X = synth.f32_to_bf16(g.standard_normal(size=(M, K)).astype(np.float32))
    return idx, cb, X


def _dense(idx, cb):
    """fp64 dense weights from the *unpacked* indices (never reads the packed stream)."""
    return np.take_along_axis(synth.bf16_to_f64(cb), idx.astype(np.int64), axis=1)


# ---------------------------------------------------------------- pack / unpack

@pytest.mark.parametrize("bits,K,idx,words", _golden_pack_vectors())
def test_pack_matches_hand_computed_words(bits, K, idx, words):
    got = oracle.pack(idx[None, :], bits)
    assert got.shape == (1, len(words))
    assert [hex(w) for w in got[0]] == [hex(w) for w in words]
    assert np.array_equal(oracle.unpack(words[None, :], K, bits)[0], idx)


@pytest.mark.parametrize("bits", BITS)
def test_words_per_row(bits):
    for K in EDGE_K + (2048, 4096, 14336):
        assert oracle.words_per_row(bits, K) == -(-K * bits // 32)
    with pytest.raises(ValueError):
        oracle.words_per_row(5, 8)
    with pytest.raises(ValueError):
        oracle.words_per_row(0, 8)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("K", EDGE_K)
def test_round_trip_and_numpy_packbits(bits, K):
    g = np.random.default_rng(1000 * bits + K)
    for N in (1, 3):
        idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        p = oracle.pack(idx, bits)
        assert np.array_equal(p, _numpy_pack(idx, bits))
        assert np.array_equal(oracle.unpack(p, K, bits), idx)


@pytest.mark.parametrize("bits", BITS)
def test_pad_bits_zero_and_all_ones(bits):
    for K in (1, 5, 11, 33, 50):
        idx = np.full((2, K), (1 << bits) - 1, dtype=np.uint8)
        p = oracle.pack(idx, bits)
        used = K * bits
        total = int(sum(bin(int(w)).count("1") for w in p[0]))
        assert total == used                       # every used bit set, every pad bit clear
        last = int(p[0, -1])
        tail = used - 32 * (p.shape[1] - 1)
        assert last == (1 << tail) - 1 if tail < 32 else last == 0xFFFFFFFF


@pytest.mark.parametrize("bits", BITS)
def test_pack_rejects_out_of_range_index(bits):
    idx = np.zeros((1, 8), dtype=np.uint8)
    idx[0, 3] = 1 << bits
    with pytest.raises(ValueError):
        oracle.pack(idx, bits)


def test_unpack_ignores_pad_bits():
    idx = np.array([[1, 0, 1]], dtype=np.uint8)
    p = oracle.pack(idx, 1)
    p[0, 0] |= np.uint32(0xFFFFFFF8)
    assert np.array_equal(oracle.unpack(p, 3, 1), idx)


# ---------------------------------------------------------------- dequant

@pytest.mark.parametrize("bits", BITS)
def test_dequant_is_codebook_lookup(bits):
    idx, cb, _ = _rand_case(7 + bits, 13, 67, bits, 1)
    Wd = oracle.dequant(oracle.pack(idx, bits), cb, 67, bits)
    assert np.array_equal(Wd, np.take_along_axis(cb, idx.astype(np.int64), axis=1))


@pytest.mark.parametrize("bits", BITS)
def test_dequant_relabelling_invariance(bits):
    idx, cb, _ = _rand_case(17 + bits, 9, 50, bits, 1)
    g = np.random.default_rng(5)
    Wd = oracle.dequant(oracle.pack(idx, bits), cb, 50, bits)
    perm = np.stack([g.permutation(1 << bits) for _ in range(9)])       # new label j holds old perm[j]
    cb2 = np.take_along_axis(cb, perm, axis=1)
    inv = np.argsort(perm, axis=1)
    idx2 = np.take_along_axis(inv, idx.astype(np.int64), axis=1).astype(np.uint8)
    assert np.array_equal(oracle.dequant(oracle.pack(idx2, bits), cb2, 50, bits), Wd)


# ---------------------------------------------------------------- product

@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("N,K,M", [(1, 1, 1), (5, 33, 1), (67, 64, 3), (16, 67, 2)])
def test_gemm_vs_bruteforce_same_order_bit_exact(bits, N, K, M):
    """Textbook triple loop in Python floats (IEEE double), k ascending."""
    idx, cb, X = _rand_case(31 * bits + N + K, N, K, bits, M)
    Y, A, _ = oracle.gemm(oracle.pack(idx, bits), cb, X, K, bits)
    W = _dense(idx, cb)
    Xd = synth.bf16_to_f64(X)
    for m in range(M):
        for n in range(N):
            y = 0.0
            a = 0.0
            for k in range(K):
                t = float(W[n, k]) * float(Xd[m, k])
                y += t
                a += abs(t)
            assert Y[m, n] == y
            assert A[m, n] == a


@pytest.mark.parametrize("bits", BITS)
def test_gemm_vs_numpy_dense(bits):
    N, K, M = 96, 515, 5
    idx, cb, X = _rand_case(77 + bits, N, K, bits, M)
    Y, A, Yb = oracle.gemm(oracle.pack(idx, bits), cb, X, K, bits)
    W = _dense(idx, cb)
    Xd = synth.bf16_to_f64(X)
    Aref = np.abs(Xd) @ np.abs(W).T
    assert np.all(np.abs(Y - Xd @ W.T) <= 1e-13 * Aref)
    assert np.allclose(A, Aref, rtol=1e-12, atol=0)
    # transposed-operand mistake would show here: X W^T is M x N, not N x M
    assert Y.shape == (M, N)
    # the rounded output is within half a bf16 ulp of the fp64 value
    mine = synth.bf16_to_f64(Yb)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(mine))) - 7)
    assert np.all(np.abs(mine - Y) <= 0.5 * ulp)


def test_one_bit_closed_form():
    """y = c0*sum(x) + (c1 - c0)*sum_{idx=1} x   (two-centroid rows)."""
    N, K, M = 40, 1000, 3
    idx, cb, X = _rand_case(5, N, K, 1, M)
    Y, A, _ = oracle.gemm(oracle.pack(idx, 1), cb, X, K, 1)
    c = synth.bf16_to_f64(cb)
    Xd = synth.bf16_to_f64(X)
    for m in range(M):
        sx = math.fsum(Xd[m])
        for n in range(N):
            s1 = math.fsum(Xd[m][idx[n] == 1])
            y = c[n, 0] * sx + (c[n, 1] - c[n, 0]) * s1
            assert abs(Y[m, n] - y) <= 1e-12 * A[m, n]


def test_one_bit_symmetric_form():
    """cfg0 recipe: (-t, +t) gives y = t*(2*sum_{idx=1}x - sum x)."""
    N, K = 32, 2048
    idx = synth.make_indices(0, 0, N, K, 1)
    cb = synth.make_codebook(0, 0, N, 1, symmetric=True)
    x = synth.make_x(0, 0, 1, K)[0]
    Y, A, _ = oracle.gemm(oracle.pack(idx, 1), cb, x, K, 1)
    t = synth.bf16_to_f64(cb[:, 1])
    xd = synth.bf16_to_f64(x)
    for n in range(N):
        y = t[n] * (2.0 * math.fsum(xd[idx[n] == 1]) - math.fsum(xd))
        assert abs(Y[n] - y) <= 1e-12 * A[n]


@pytest.mark.parametrize("bits", BITS)
def test_one_hot_x_reads_a_single_weight(bits):
    N, K = 11, 70
    idx, cb, _ = _rand_case(3 + bits, N, K, bits, 1)
    p = oracle.pack(idx, bits)
    W = _dense(idx, cb)
    one = np.uint16(0x3F80)                          # bf16 1.0
    for k in (0, 1, 10, 21, 31, 32, 63, 64, 69):
        x = np.zeros(K, dtype=np.uint16)
        x[k] = one
        Y, A, Yb = oracle.gemm(p, cb, x, K, bits)
        assert np.array_equal(Y, W[:, k])
        assert np.array_equal(A, np.abs(W[:, k]))
        assert np.array_equal(Yb, np.take_along_axis(cb, idx[:, k:k + 1].astype(np.int64), axis=1)[:, 0])


@pytest.mark.parametrize("bits", BITS)
def test_constant_codebook_row_and_zero_x(bits):
    N, K = 6, 333
    idx, cb, X = _rand_case(9 + bits, N, K, bits, 2)
    cb[2, :] = cb[2, 0]
    p = oracle.pack(idx, bits)
    Y, A, _ = oracle.gemm(p, cb, X, K, bits)
    Xd = synth.bf16_to_f64(X)
    c = float(synth.bf16_to_f64(cb[2, :1])[0])
    for m in range(2):
        assert abs(Y[m, 2] - c * math.fsum(Xd[m])) <= 1e-13 * A[m, 2]
    Y0, A0, Yb0 = oracle.gemm(p, cb, np.zeros((2, K), np.uint16), K, bits)
    assert not Y0.any() and not A0.any() and not Yb0.any()


@pytest.mark.parametrize("bits", BITS)
def test_power_of_two_scaling_is_exact(bits):
    N, K = 8, 257
    idx, cb, X = _rand_case(19 + bits, N, K, bits, 2)
    p = oracle.pack(idx, bits)
    Y, _, _ = oracle.gemm(p, cb, X, K, bits)
    X4 = synth.f32_to_bf16(synth.bf16_to_f32(X) * np.float32(4.0))
    Y4, _, _ = oracle.gemm(p, cb, X4, K, bits)
    assert np.array_equal(Y4, 4.0 * Y)
    Xn = X ^ np.uint16(0x8000)                       # negate every activation
    Yn, _, _ = oracle.gemm(p, cb, Xn, K, bits)
    assert np.array_equal(Yn, -Y)


@pytest.mark.parametrize("bits", BITS)
def test_row_and_column_permutations(bits):
    N, K = 12, 130
    idx, cb, X = _rand_case(23 + bits, N, K, bits, 2)
    g = np.random.default_rng(2)
    Y, A, _ = oracle.gemm(oracle.pack(idx, bits), cb, X, K, bits)
    rp = g.permutation(N)
    Yr, _, _ = oracle.gemm(oracle.pack(idx[rp], bits), cb[rp], X, K, bits)
    assert np.array_equal(Yr, Y[:, rp])
    cp = g.permutation(K)
    Yc, _, _ = oracle.gemm(oracle.pack(idx[:, cp], bits), cb, X[:, cp], K, bits)
    assert np.all(np.abs(Yc - Y) <= 1e-13 * A)


@pytest.mark.parametrize("bits", (1, 2, 4))
def test_shared_codebook_reduces_to_byte_lut_routine(bits):
    """With one codebook for every row and unit block scales, the format is the
    paper's reference routine (App. E, "Kernel implementations"): a 256-entry
    table maps each packed byte to its 8/bits decoded elements, the table is
    gathered by the byte stream, and the batch is multiplied by the transpose."""
    N, K, M = 24, 256, 4
    idx, cb, X = _rand_case(41 + bits, N, K, bits, M, shared=True)
    p = oracle.pack(idx, bits)
    epb = 8 // bits
    c = synth.bf16_to_f64(cb[0])
    byte_values = np.arange(256)
    table = np.stack([c[(byte_values >> (bits * j)) & ((1 << bits) - 1)] for j in range(epb)], axis=1)
    stream = np.ascontiguousarray(p.astype("<u4")).view(np.uint8).reshape(N, -1)   # N x K/epb
    Wfull = table[stream].reshape(N, K)
    Yref = synth.bf16_to_f64(X) @ Wfull.T
    Y, A, _ = oracle.gemm(p, cb, X, K, bits)
    assert np.all(np.abs(Y - Yref) <= 1e-13 * A)


@pytest.mark.parametrize("bits", BITS)
def test_batch_rows_equal_single_vector_calls_and_row_ranges(bits):
    N, K, M = 10, 99, 4
    idx, cb, X = _rand_case(51 + bits, N, K, bits, M)
    p = oracle.pack(idx, bits)
    Y, A, Yb = oracle.gemm(p, cb, X, K, bits)
    for m in range(M):
        y, a, yb = oracle.gemm(p, cb, X[m], K, bits)
        assert np.array_equal(y, Y[m]) and np.array_equal(a, A[m]) and np.array_equal(yb, Yb[m])
    Ys, As, _ = oracle.gemm(p, cb, X, K, bits, rows=(3, 7))
    assert np.array_equal(Ys[:, 3:7], Y[:, 3:7]) and np.isnan(Ys[:, :3]).all() and np.isnan(Ys[:, 7:]).all()


# ---------------------------------------------------------------- bf16 rounding

def test_round_bf16_known_values_and_ties():
    assert oracle.round_bf16(1.0) == 0x3F80
    assert oracle.round_bf16(-2.0) == 0xC000
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 0x3F80            # tie -> even (down)
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82        # tie -> even (up)
    assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == 0x3F81   # no double rounding through fp32
    assert oracle.round_bf16(1.0 + 2.0 ** -8 - 2.0 ** -30) == 0x3F80
    assert oracle.round_bf16(0.0) == 0


def test_round_bf16_vs_torch_on_fp32_values():
    import torch
    g = np.random.default_rng(8)
    v = (g.standard_normal(4000) * np.exp(g.uniform(-20, 20, 4000))).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.round_bf16(float(t)) for t in v], dtype=np.uint16)
    assert np.array_equal(got, ref)
    assert np.array_equal(synth.f32_to_bf16(v), ref)             # the generator's converter too
