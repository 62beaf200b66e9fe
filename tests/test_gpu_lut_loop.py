"""GPU parity of the table kernel that walks a row in rounds (canonical layout, any K % 32 == 0 up to 24576
that has no kernel specialised on it): through the C ABI against the CPU oracle -- every bit-width, every
number of lanes per row and split of K over the waves of a workgroup, rows that end inside a round, row counts
that end inside a workgroup, ranges of rounds that end in padded rounds, batches as grid rows, one-hot probes
(bit-exact), determinism."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_15563_amd import kmq, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    assert torch.cuda.is_available()
    return gpu_util


def _case(seed, N, K, bits, M):
    g = np.random.default_rng(seed)
    idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    cb = synth.f32_to_bf16(np.sort(g.normal(0, 0.02, size=(N, 1 << bits)).astype(np.float32), axis=1))
    X = synth.f32_to_bf16(g.standard_normal(size=(M, K)).astype(np.float32))
    return idx, cb, X


# K: a single slice (32), less than one round (96, 256), rows that end inside a round (1056 = 33 slices, 4000,
# 11008, 12320), round counts the waves along K do not divide (2560, 5120, 7168), the longest rows (16384; 21504 and
# 24576, whose x is staged in two steps)
# N: 1 and 7 rows (one partly filled wave), 250 (ragged), 1000 / 4099 (several waves along K), 20000 / 40001
# (one wave along K)
@pytest.mark.parametrize("bits", (1, 2, 3, 4))
@pytest.mark.parametrize("N,K", [(1, 256), (7, 768), (250, 1280), (1000, 2560), (4099, 2816), (4096, 5120), (2048, 7168),
                                 (20000, 512), (40001, 1024), (4099, 11008), (513, 16384), (9000, 3584),
                                 (300, 32), (5000, 96), (1000, 1056), (4097, 4000), (2000, 12320), (1000, 21504), (600, 24576)])
def test_loop_kernel_vs_oracle(gpu, bits, N, K):
    if kmq.kernel_name(N, K, bits, 1, kmq.LAYOUT_CANONICAL) != f"lut_loop_b{bits}":
        pytest.skip("this (bits, K) has a kernel specialised on K")
    idx, cb, X = _case(31 * bits + N + K, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X, N, K, bits)
    ranges = gpu.sample_ranges(N, N + K)
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, ranges, label=f"lut_loop b{bits} {N}x{K}")


# the launcher's choice of lanes per row and waves along K depends on N as well as K, and long rows leave little LDS beside
# the staged x: every bit-width at the longest row and just below, with few and with many rows
@pytest.mark.parametrize("bits", (1, 2, 3, 4))
@pytest.mark.parametrize("N,K", [(3, 24576), (2600, 24576), (2600, 24544), (700, 20512), (6000, 8224), (30000, 2080), (70000, 288)])
def test_loop_kernel_launch_shapes(gpu, bits, N, K):
    if kmq.kernel_name(N, K, bits, 1, kmq.LAYOUT_CANONICAL) != f"lut_loop_b{bits}":
        pytest.skip("few long rows: split over K by the shape-agnostic kernel")
    idx, cb, X = _case(3 * bits + N + K, N, K, bits, 1)
    Yg = gpu.run_gemm(gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb), X, N, K, bits)
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, gpu.sample_ranges(N, N + K, nblocks=3),
                             label=f"lut_loop b{bits} {N}x{K}")


@pytest.mark.parametrize("bits,N,K,M", [(3, 1000, 2560, 3), (4, 4099, 5120, 2), (2, 513, 7168, 16), (1, 2048, 1280, 5)])
def test_loop_kernel_batches(gpu, bits, N, K, M):
    assert kmq.kernel_name(N, K, bits, M, kmq.LAYOUT_CANONICAL) == f"lut_loop_b{bits}"
    idx, cb, X = _case(7 * bits + N + K + M, N, K, bits, M)
    Yg = gpu.run_gemm(gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb), X, N, K, bits)
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, gpu.sample_ranges(N, N + K + M),
                             label=f"lut_loop b{bits} {N}x{K} M{M}")


@pytest.mark.parametrize("bits", (1, 2, 3, 4))
def test_loop_kernel_one_hot_probe_is_bit_exact(gpu, bits):
    """x = e_k: a sum with one non-zero term, so y[n] is the dequantised weight W[n][k] exactly."""
    N, K = 1003, 2816
    idx, cb, _ = _case(5 * bits, N, K, bits, 1)
    assert kmq.kernel_name(N, K, bits, 1, kmq.LAYOUT_CANONICAL) == f"lut_loop_b{bits}"
    pd, cd = gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb)
    Wd = oracle.dequant(oracle.pack(idx, bits), cb, K, bits)
    for k0 in (0, 31, 32, 255, 256, 1407, 1408, 2047, 2048, 2559, 2560, K - 1):
        x = np.zeros(K, dtype=np.uint16)
        x[k0] = 0x3F80
        Yg = gpu.run_gemm(pd, cd, x, N, K, bits)
        assert np.array_equal(Yg[0], Wd[:, k0]), f"k0={k0}"


def test_loop_kernel_is_deterministic(gpu):
    bits, N, K = 3, 4099, 5120
    idx, cb, X = _case(99, N, K, bits, 1)
    pd, cd = gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb)
    a = gpu.run_gemm(pd, cd, X, N, K, bits)
    for _ in range(3):
        assert np.array_equal(a, gpu.run_gemm(pd, cd, X, N, K, bits))
