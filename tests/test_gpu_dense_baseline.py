"""GPU parity of the dense bf16 GEMV baseline (the 16-bit rows of the paper's App. E
micro-benchmark table) against the oracle's dense product."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_15563_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    return gpu_util


def _run(gpu, W, x):
    from paper_2602_15563_amd import kmq
    N, K = W.shape
    y = torch.full((N,), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.gemv_bf16(gpu.dev(W), gpu.dev(x), y, N, K)
    torch.cuda.synchronize()
    return gpu.host_u16(y)


@pytest.mark.parametrize("N,K", [(1, 8), (3, 64), (17, 1000), (64, 4096), (333, 515), (100, 8192), (16, 32768), (5, 1)])
def test_dense_gemv_vs_oracle(gpu, N, K):
    g = np.random.default_rng(N * 7 + K)
    W = synth.f32_to_bf16(g.normal(0, 0.02, size=(N, K)).astype(np.float32))
    x = synth.f32_to_bf16(g.normal(0, 1, size=K).astype(np.float32))
    yg = synth.bf16_to_f64(_run(gpu, W, x))
    Y, A, _ = oracle.gemm_dense(W, x)
    err = np.abs(yg - Y)
    assert np.all(err <= gpu.arithmetic_bound(A, Y, K))
    if K >= 512:
        assert np.all(err <= gpu.TOL * A)


def test_dense_gemv_equals_the_quantised_gemv_of_the_same_weights(gpu):
    """Dequantise on the GPU (bit-exact), multiply densely: same weights, same x -> the two
    kernels agree to fp32 summation order."""
    from paper_2602_15563_amd import kmq
    bits, N, K = 2, 128, 4096
    idx = synth.make_indices(42, 0, N, K, bits)
    cb = synth.make_codebook(42, 0, N, bits)
    x = synth.make_x(42, 0, 1, K)[0]
    p = gpu.dev(kmq.pack(idx, bits))
    Wd = torch.zeros((N, K), dtype=torch.int16, device="cuda")
    kmq.dequant(p, gpu.dev(cb), Wd, N, K, bits)
    yq = synth.bf16_to_f64(gpu.run_gemm(p, gpu.dev(cb), x, N, K, bits)[0])
    yd = synth.bf16_to_f64(_run(gpu, gpu.host_u16(Wd), x))
    _, A, _ = oracle.gemm(oracle.pack(idx, bits), cb, x, K, bits)
    assert np.all(np.abs(yq - yd) <= 2 * gpu.arithmetic_bound(A, np.maximum(np.abs(yq), np.abs(yd)), K))


def test_errors(gpu):
    from paper_2602_15563_amd import kmq
    W = torch.zeros((4, 64), dtype=torch.int16, device="cuda")
    x = torch.zeros(64, dtype=torch.int16, device="cuda")
    y = torch.zeros(4, dtype=torch.int16, device="cuda")
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv_bf16(W, x, y, 4, 32769)
    assert e.value.status == 3
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv_bf16(None, x, y, 4, 64)
    assert e.value.status == 1
