"""The 8-bit element width (256 centroids; the widest element format of the paper's lookup-table kernel,
Sec. 3.3 "Software formats"): oracle pins and host code on the CPU, the shape-agnostic kernels on the GPU."""
import numpy as np
import pytest

import oracle
from paper_2602_15563_amd import kmq, synth

BITS = 8


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    return gpu_util


def _codebook(seed, N):
    c = synth.f32_to_bf16(synth.rng(seed, 0, synth.KIND_CODEBOOK).normal(0.0, 0.02, size=(N, 256)).astype(np.float32))
    return np.take_along_axis(c, np.argsort(synth.bf16_to_f32(c), axis=1, kind="stable"), axis=1)


# ---- CPU: format and oracle ------------------------------------------------------------------------

def test_packed_words_are_the_index_bytes_little_endian():
    """Element k of a row is byte k of the row's stream (LSB first): hand-written words."""
    idx = np.array([[0x00, 0x14, 0x28, 0x3C, 0x50, 0xFF, 0x01]], np.uint8)
    want = np.array([[0x3C281400, 0x0001FF50]], np.uint32)
    assert np.array_equal(oracle.pack(idx, BITS), want) and np.array_equal(kmq.pack(idx, BITS), want)
    assert np.array_equal(oracle.unpack(want, 7, BITS), idx) and np.array_equal(kmq.unpack(want, 7, BITS), idx)
    assert oracle.words_per_row(BITS, 7) == 2 == kmq.words_per_row(BITS, 7)


@pytest.mark.parametrize("K", [1, 3, 4, 5, 63, 64, 257])
def test_round_trip_and_byte_view(K):
    idx = synth.make_indices(80, K, 5, K, BITS)
    p = oracle.pack(idx, BITS)
    assert np.array_equal(kmq.pack(idx, BITS), p)
    assert np.array_equal(p.view(np.uint8).reshape(5, -1)[:, :K], idx)          # the stream IS the bytes
    assert not p.view(np.uint8).reshape(5, -1)[:, K:].any()                      # pad bits zero
    assert np.array_equal(oracle.unpack(p, K, BITS), idx) and np.array_equal(kmq.unpack(p, K, BITS), idx)


def test_oracle_product_against_dense_numpy():
    N, K, M = 6, 67, 3
    idx, cb, X = synth.make_indices(81, 0, N, K, BITS), _codebook(81, N), synth.make_x(81, 0, M, K)
    p = oracle.pack(idx, BITS)
    Y, A, _ = oracle.gemm(p, cb, X, K, BITS)
    W = np.take_along_axis(synth.bf16_to_f64(cb), idx.astype(np.int64), axis=1)
    Xd = synth.bf16_to_f64(X)
    np.testing.assert_allclose(Y, Xd @ W.T, rtol=0, atol=1e-13 * A.max())
    np.testing.assert_allclose(A, np.abs(Xd) @ np.abs(W).T, rtol=1e-12)
    assert np.array_equal(oracle.dequant(p, cb, K, BITS), np.take_along_axis(cb, idx.astype(np.int64), axis=1))
    # one-hot activations read single weights back
    e = np.zeros((1, K), np.uint16)
    e[0, 41] = 0x3F80
    Y1, _, _ = oracle.gemm(p, cb, e, K, BITS)
    assert np.array_equal(Y1[0], W[:, 41])


def test_no_tiled_layout_and_no_quantiser_for_eight_bits():
    assert kmq.kernel_name(64, 4096, BITS, 8, 1) == "invalid" and kmq.kernel_name(64, 4096, BITS, 8, 0) == "generic"
    assert kmq.workspace_bytes(4, 65536, BITS, 1) > 0                              # split-K applies as for any width


# ---- GPU ------------------------------------------------------------------------------------------

@pytest.mark.gpu
@pytest.mark.parametrize("N,K,M", [(5, 33, 1), (64, 4096, 1), (100, 515, 3), (40, 1000, 16), (9, 4096, 8), (3, 40000, 2)])
def test_gpu_product(gpu, N, K, M):
    idx, cb, X = synth.make_indices(82, N, N, K, BITS), _codebook(82 + N, N), synth.make_x(82, N, M, K)
    p = oracle.pack(idx, BITS)
    Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X, N, K, BITS)
    gpu.check_against_oracle(Yg, p, cb, X, K, BITS, label=f"b8 {N}x{K} M{M}")


@pytest.mark.gpu
def test_gpu_dequant_bit_exact_and_one_hot(gpu):
    import torch
    N, K = 37, 300
    idx, cb = synth.make_indices(83, 0, N, K, BITS), _codebook(83, N)
    p = oracle.pack(idx, BITS)
    Wd = torch.full((N, K), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.dequant(gpu.dev(p), gpu.dev(cb), Wd, N, K, BITS)
    torch.cuda.synchronize()
    want = oracle.dequant(p, cb, K, BITS)
    assert np.array_equal(gpu.host_u16(Wd), want)
    X = np.zeros((16, K), np.uint16)
    for m in range(16):
        X[m, 100 + m] = 0x3F80
    Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X, N, K, BITS)
    assert np.array_equal(Yg, want[:, 100:116].T)                  # single-term sums: the weights themselves


@pytest.mark.gpu
@pytest.mark.parametrize("N,K,M", [(7, 64, 1), (50, 4096, 1), (20, 640, 5)])
def test_gpu_blockscaled(gpu, N, K, M):
    import torch
    idx = synth.make_indices(84, N, N, K, BITS)
    cb = np.sort(synth.f32_to_bf16(np.clip(synth.rng(84, N, synth.KIND_SHARED_CODEBOOK).normal(0, 0.45, 256), -1, 1).astype(np.float32)).view(np.int16)).view(np.uint16)
    sc, X = synth.make_scales(84, N, N, K), synth.make_x(84, N, M, K)
    p = oracle.pack(idx, BITS)
    Yg = gpu.run_gemm_blockscaled(gpu.dev(p), gpu.dev(cb), gpu.dev(sc), X, N, K, BITS)
    gpu.check_blockscaled_against_oracle(Yg, p, cb, sc, X, K, BITS, label=f"b8 scaled {N}x{K} M{M}")
    Wd = torch.full((N, K), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.dequant_blockscaled(gpu.dev(p), gpu.dev(cb), gpu.dev(sc), Wd, N, K, BITS)
    torch.cuda.synchronize()
    assert np.array_equal(gpu.host_u16(Wd), oracle.dequant_blockscaled(p, cb, sc, K, BITS))


@pytest.mark.gpu
def test_gpu_fusions(gpu):
    import torch
    N, K = 48, 1024
    idx, cb = synth.make_indices(85, 0, N, K, BITS), _codebook(85, N)
    x, g, res = synth.make_x(85, 0, 1, K)[0], synth.make_norm_weight(85, 0, K), synth.make_residual(85, 0, N)
    p = oracle.pack(idx, BITS)
    y = torch.full((N,), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.gemv_fused(gpu.dev(p), gpu.dev(cb), gpu.dev(x), y, N, K, BITS, norm_weight=gpu.dev(g), eps=1e-5, residual=gpu.dev(res))
    torch.cuda.synchronize()
    Y, A = oracle.gemv_fused(p, cb, x, K, BITS, norm_weight=g, eps=1e-5, residual=res)
    yg = synth.bf16_to_f64(gpu.host_u16(y))
    # (+ 2^-7 of the product's magnitude: the oracle rounds x*r*g, the kernel rounds x*g and scales the sum)
    Ap = A - np.abs(synth.bf16_to_f64(res))
    assert np.all(np.abs(yg - Y) <= gpu.arithmetic_bound(A, Y, K + 16) + gpu.rmsnorm_commute_bound(Ap))
    assert np.all(np.abs(yg - Y) <= gpu.TOL * A + 2.0 ** -8 * np.abs(Y))
    kmq.gemv_swiglu(gpu.dev(p), gpu.dev(cb), gpu.dev(p), gpu.dev(cb), gpu.dev(x), y, N, K, BITS)
    torch.cuda.synchronize()
    G, Ag, _ = oracle.gemm(p, cb, x.reshape(1, -1), K, BITS)
    want = oracle.swiglu(G[0], G[0])
    yg = synth.bf16_to_f64(gpu.host_u16(y))
    assert np.all(np.abs(yg - want) <= gpu.swiglu_bound(G[0], G[0], Ag[0], Ag[0], oracle.swiglu(G[0], np.ones_like(G[0])), want, K))


@pytest.mark.gpu
def test_gpu_errors(gpu):
    import torch
    N, K = 16, 128
    idx, cb = synth.make_indices(86, 0, N, K, BITS), _codebook(86, N)
    W, C, X = gpu.dev(oracle.pack(idx, BITS)), gpu.dev(cb), gpu.dev(synth.make_x(86, 0, 1, K))
    y = torch.zeros(N, dtype=torch.int16, device="cuda")
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv(W, C, X, y, N, K, BITS, 1)
    assert e.value.status == 7
    dense = gpu.dev(synth.make_dense_weights(86, 0, N, K))
    with pytest.raises(kmq.KmqError) as e:
        kmq.quantize_rows(dense, N, K, BITS, 3, W, C)
    assert e.value.status == 2
