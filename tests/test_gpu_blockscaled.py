"""GPU parity of the block-scaled calls (the paper's own weight format: Sec. 2.2
"Nonlinear k-means quantization", App. E "Kernel implementations") against the oracle,
through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_2602_15563_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    return gpu_util


def _case(seed, N, K, bits, M):
    return (synth.make_indices(seed, 0, N, K, bits), synth.make_shared_codebook(seed, 0, bits),
            synth.make_scales(seed, 0, N, K), synth.make_x(seed, 0, M, K))


@pytest.mark.parametrize("bits", (1, 2, 3, 4))
@pytest.mark.parametrize("N,K,M", [(1, 64, 1), (5, 128, 1), (64, 320, 3), (333, 192, 16), (17, 4160, 8), (40, 1024, 4)])
def test_generic_shapes_vs_oracle(gpu, bits, N, K, M):
    from paper_2602_15563_amd import kmq
    idx, cb, sc, X = _case(3 * bits + N + K + M, N, K, bits, M)
    p = kmq.pack(idx, bits)
    assert kmq.kernel_name_blockscaled(N, K, bits, M) == "blockscaled_generic"
    Yg = gpu.run_gemm_blockscaled(gpu.dev(p), gpu.dev(cb), gpu.dev(sc), X, N, K, bits)
    gpu.check_blockscaled_against_oracle(Yg, oracle.pack(idx, bits), cb, sc, X, K, bits, label=f"b{bits} {N}x{K} M{M}")


SC_SHAPES = [(1, 2048), (1, 4096), (1, 8192), (2, 2048), (2, 4096), (2, 8192), (2, 14336),
             (3, 2048), (3, 4096), (3, 8192), (3, 14336), (4, 2048), (4, 4096), (4, 8192), (4, 14336)]


@pytest.mark.parametrize("bits,K", SC_SHAPES)
@pytest.mark.parametrize("N", (1, 3, 17, 64, 333))
def test_specialised_gemv_vs_oracle(gpu, bits, K, N):
    from paper_2602_15563_amd import kmq
    idx, cb, sc, X = _case(11 * bits + N + K, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    assert kmq.kernel_name_blockscaled(N, K, bits, 1).startswith("lut_sc_"), kmq.kernel_name_blockscaled(N, K, bits, 1)
    Yg = gpu.run_gemm_blockscaled(gpu.dev(p), gpu.dev(cb), gpu.dev(sc), X[0], N, K, bits)
    gpu.check_blockscaled_against_oracle(Yg, oracle.pack(idx, bits), cb, sc, X, K, bits, label=f"b{bits} {N}x{K}")


@pytest.mark.parametrize("bits,K", [(2, 4096), (4, 8192)])
def test_unit_scales_reproduce_the_per_row_kernel_bit_for_bit(gpu, bits, K):
    """scale = 1 and the shared codebook copied to every row: the same table entries, the same
    products in the same order, one exact multiplication by 1.0 -> identical bf16 outputs."""
    from paper_2602_15563_amd import kmq
    N = 96
    idx, cb, _, X = _case(5 + bits, N, K, bits, 1)
    p = gpu.dev(kmq.pack(idx, bits))
    ones = np.full((N, K // 64), 0x3F80, dtype=np.uint16)
    Ys = gpu.run_gemm_blockscaled(p, gpu.dev(cb), gpu.dev(ones), X[0], N, K, bits)
    Yr = gpu.run_gemm(p, gpu.dev(np.tile(cb, (N, 1))), X[0], N, K, bits)
    assert np.array_equal(Ys, Yr)


def test_only_the_scaled_block_contributes(gpu):
    """One non-zero scale: the output is that block's sum alone (block boundaries and the
    scale's index as the kernels see them)."""
    from paper_2602_15563_amd import kmq
    bits, N, K = 4, 24, 8192
    idx, cb, sc, X = _case(77, N, K, bits, 1)
    p = gpu.dev(kmq.pack(idx, bits))
    for r, g in ((0, 0), (5, 63), (23, 127), (7, 64)):
        z = np.zeros_like(sc)
        z[r, g] = sc[r, g]
        Yg = gpu.run_gemm_blockscaled(p, gpu.dev(cb), gpu.dev(z), X[0], N, K, bits)
        gpu.check_blockscaled_against_oracle(Yg, oracle.pack(idx, bits), cb, z, X, K, bits, strict=False, label=f"r{r} g{g}")
        assert not np.delete(synth.bf16_to_f32(Yg[0]), r).any()


@pytest.mark.parametrize("bits", (4, 1))
def test_papers_benchmark_shape_full_size(gpu, bits):
    """App. E, Table "perf_micro_m1_impl": m = 1, h = 8192, 4-bit and 1-bit elements with B = 64
    scales; sampled row blocks of the full-size product."""
    from paper_2602_15563_amd import kmq
    N = K = 8192
    idx, cb, sc, X = _case(100 + bits, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    Yg = gpu.run_gemm_blockscaled(gpu.dev(p), gpu.dev(cb), gpu.dev(sc), X[0], N, K, bits)
    worst = gpu.check_blockscaled_against_oracle(Yg, oracle.pack(idx, bits), cb, sc, X, K, bits, strict=True,
                                                 row_ranges=gpu.sample_ranges(N, bits), label=f"h8192 b{bits}")
    assert worst < 2e-3


@pytest.mark.parametrize("bits", (1, 2, 3, 4))
@pytest.mark.parametrize("N,K,M", [(16, 512, 16), (40, 1024, 4), (97, 4096, 8), (333, 3072, 1), (64, 8192, 16), (130, 2048, 2),
                                   (20, 384, 5), (70, 640, 16), (5000, 8192, 3), (33, 16384, 16), (50, 1536, 7)])
def test_tiled_layout_matrix_core_vs_oracle(gpu, bits, N, K, M):
    """The block-scaled product on the tiled layout (matrix-core kernel), ragged row counts, every
    batch kind, K with 1..16 super-blocks per wave; numbers of blocks that are and are not multiples of
    eight (two ways of staging the scales); long rows with few and with many row blocks (4-bit: with and
    without the table of centroid pairs)."""
    from paper_2602_15563_amd import kmq
    if kmq.tiled_words(N, K, bits, 1) < 0:
        pytest.skip("K is not a whole number of super-blocks at this bit-width")
    idx, cb, sc, X = _case(19 * bits + N + K + M, N, K, bits, M)
    p = kmq.pack(idx, bits)
    t = kmq.repack(p, K, bits, 1)
    assert kmq.kernel_name_blockscaled(N, K, bits, M, 1) == f"mfma_sc_b{bits}"
    import torch
    Y = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.gemm_smallbatch_blockscaled(gpu.dev(t), gpu.dev(cb), gpu.dev(sc), gpu.dev(X), Y, N, K, M, bits, 1)
    torch.cuda.synchronize()
    gpu.check_blockscaled_against_oracle(gpu.host_u16(Y), oracle.pack(idx, bits), cb, sc, X, K, bits,
                                         label=f"tiled b{bits} {N}x{K} M{M}")


def test_tiled_only_the_scaled_block_contributes(gpu):
    from paper_2602_15563_amd import kmq
    import torch
    bits, N, K, M = 3, 48, 4096, 16
    idx, cb, sc, X = _case(91, N, K, bits, M)
    t = gpu.dev(kmq.repack(kmq.pack(idx, bits), K, bits, 1))
    for r, g in ((0, 0), (17, 1), (47, 63), (33, 30)):
        z = np.zeros_like(sc)
        z[r, g] = sc[r, g]
        Y = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")
        kmq.gemm_smallbatch_blockscaled(t, gpu.dev(cb), gpu.dev(z), gpu.dev(X), Y, N, K, M, bits, 1)
        torch.cuda.synchronize()
        Yg = gpu.host_u16(Y)
        gpu.check_blockscaled_against_oracle(Yg, oracle.pack(idx, bits), cb, z, X, K, bits, strict=False, label=f"r{r} g{g}")
        assert not np.delete(synth.bf16_to_f32(Yg), r, axis=1).any()


def test_errors(gpu):
    from paper_2602_15563_amd import kmq
    import torch
    N, K, bits = 8, 128, 2
    idx, cb, sc, X = _case(1, N, K, bits, 1)
    p, cbd, scd, xd = gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb), gpu.dev(sc), gpu.dev(X[0])
    y = torch.zeros(N, dtype=torch.int16, device="cuda")
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv_blockscaled(p, cbd, scd, xd, y, N, K - 32, bits)       # K not a multiple of 64
    assert e.value.status == 3
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv_blockscaled(p, cbd, scd, xd, y, N, K, bits, layout=1)  # K = 128 is not a whole 2-bit super-block
    assert e.value.status == 7
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv_blockscaled(p, cbd, None, xd, y, N, K, bits)
    assert e.value.status == 1


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("N,K", [(1, 64), (7, 640), (300, 4096), (33, 64 * 257)])
def test_dequant_blockscaled_bit_exact(gpu, N, K, bits):
    import torch
    from paper_2602_15563_amd import kmq
    idx, cb, sc, _ = _case(900 + bits + N, N, K, bits, 1)
    packed = oracle.pack(idx, bits)
    Wd = torch.full((N, K), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.dequant_blockscaled(gpu.dev(packed), gpu.dev(cb), gpu.dev(sc), Wd, N, K, bits)
    torch.cuda.synchronize()
    assert np.array_equal(gpu.host_u16(Wd), oracle.dequant_blockscaled(packed, cb, sc, K, bits))


def test_dequant_blockscaled_then_dense_product_matches_the_fused_one(gpu):
    """The separate-dequantise route: dense weights from kmq_dequant_blockscaled through the dense bf16 GEMV against
    the fused block-scaled GEMV of the same buffers; they differ by the rounding of the dense weights."""
    import torch
    from paper_2602_15563_amd import kmq
    bits, N, K = 4, 512, 4096
    idx, cb, sc, x = _case(940, N, K, bits, 1)
    packed = oracle.pack(idx, bits)
    Wd = torch.empty((N, K), dtype=torch.int16, device="cuda")
    kmq.dequant_blockscaled(gpu.dev(packed), gpu.dev(cb), gpu.dev(sc), Wd, N, K, bits)
    y = torch.empty(N, dtype=torch.int16, device="cuda")
    kmq.gemv_bf16(Wd, gpu.dev(x), y, N, K)
    torch.cuda.synchronize()
    fused = synth.bf16_to_f64(gpu.run_gemm_blockscaled(gpu.dev(packed), gpu.dev(cb), gpu.dev(sc), x, N, K, bits)[0])
    _, A, _ = oracle.gemm_blockscaled(packed, cb, sc, x, K, bits)
    dense = synth.bf16_to_f64(gpu.host_u16(y))
    assert np.all(np.abs(dense - fused) <= 2.0 ** -8 * A[0] + 2.0 ** -7 * np.abs(fused) + 2 * gpu.TOL * A[0])


def test_dequant_blockscaled_errors(gpu):
    import torch
    from paper_2602_15563_amd import kmq
    idx, cb, sc, _ = _case(950, 4, 128, 2, 1)
    W, C, S = gpu.dev(oracle.pack(idx, 2)), gpu.dev(cb), gpu.dev(sc)
    Wd = torch.zeros((4, 128), dtype=torch.int16, device="cuda")
    for call, status in [(lambda: kmq.dequant_blockscaled(W, C, S, Wd, 4, 100, 2), 3),
                         (lambda: kmq.dequant_blockscaled(W, C, S, Wd, 4, 128, 7), 2),
                         (lambda: kmq.dequant_blockscaled(W, C, None, Wd, 4, 128, 2), 1),
                         (lambda: kmq.dequant_blockscaled(W, C, S, Wd.view(-1)[1:], 4, 128, 2), 4)]:
        with pytest.raises(kmq.KmqError) as e:
            call()
        assert e.value.status == status
