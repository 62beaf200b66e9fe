"""GPU parity of the matrix-core kernel whose waves keep their slice of the activations in registers
(tiled layout, 2 and 3 bits, K <= 4096, at least 6144 rows): through the C ABI against the CPU oracle on
sampled row blocks -- two, three and four row blocks per workgroup, ragged last blocks, every batch size,
every split of K over the waves, one-hot probes (bit-exact), determinism."""
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


# rows: 6144 (384 row blocks: 2 per workgroup, 192 workgroups), 8190 (ragged, 2 x 256), 9216 (3 x 192),
# 12281 (ragged, 3 x 256), 14336 (4 x 224), 16377 (ragged, 4 x 256)
@pytest.mark.parametrize("bits,K", [(2, 3072), (2, 3584), (2, 4096), (3, 3072), (3, 3584), (3, 4096)])
@pytest.mark.parametrize("N,M", [(6144, 8), (8190, 16), (9216, 1), (12281, 5), (14336, 16), (16377, 8)])
def test_kslice_vs_oracle(gpu, bits, K, N, M):
    idx, cb, X = _case(17 * bits + N + K + M, N, K, bits, M)
    p = kmq.pack(idx, bits)
    assert kmq.kernel_name(N, K, bits, M, kmq.LAYOUT_TILED) == f"mfma_kslice_b{bits}"
    Yg = gpu.run_gemm(gpu.dev(kmq.repack(p, K, bits, kmq.LAYOUT_TILED)), gpu.dev(cb), X, N, K, bits, layout=kmq.LAYOUT_TILED,
                      use_gemv=(M == 1))
    ranges = gpu.sample_ranges(N, N + K + M)
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, ranges, label=f"kslice b{bits} {N}x{K} M{M}")


@pytest.mark.parametrize("bits", (2, 3))
def test_kslice_one_hot_batch16_probe_is_bit_exact(gpu, bits):
    """x = e_k in every batch column: a sum with one non-zero term, so Y[m][n] is the dequantised weight."""
    N, K = 9216 + 5, 4096
    idx, cb, _ = _case(5 * bits, N, K, bits, 1)
    pd, cd = gpu.dev(kmq.repack(kmq.pack(idx, bits), K, bits, kmq.LAYOUT_TILED)), gpu.dev(cb)
    for k0 in (0, 24, 255, 256, 2047, K - 16):
        X = np.zeros((16, K), dtype=np.uint16)
        for m in range(16):
            X[m, k0 + m] = 0x3F80
        Yg = gpu.run_gemm(pd, cd, X, N, K, bits, layout=kmq.LAYOUT_TILED)
        want = cb[np.arange(N)[:, None], idx[:, k0:k0 + 16]].T        # [m][n] = codebook[n][idx[n][k0 + m]]
        Wd = oracle.dequant(oracle.pack(idx[:64], bits), cb[:64], K, bits)
        assert np.array_equal(want[:, :64], Wd[:, k0:k0 + 16].T)      # the expected values are the oracle's
        assert np.array_equal(Yg, want), f"k0={k0}"


def test_kslice_is_deterministic(gpu):
    bits, N, K, M = 3, 14336, 4096, 16
    idx, cb, X = _case(99, N, K, bits, M)
    pd, cd = gpu.dev(kmq.repack(kmq.pack(idx, bits), K, bits, kmq.LAYOUT_TILED)), gpu.dev(cb)
    a = gpu.run_gemm(pd, cd, X, N, K, bits, layout=kmq.LAYOUT_TILED)
    for _ in range(3):
        assert np.array_equal(a, gpu.run_gemm(pd, cd, X, N, K, bits, layout=kmq.LAYOUT_TILED))
