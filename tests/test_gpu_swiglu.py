"""GPU parity of the fused gate / up / SwiGLU call against the oracle: two fp64 products and
the fp64 definition of silu(g) * u."""
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


def _check(gpu, bits, N, K, seed, layout=0):
    from paper_2602_15563_amd import kmq
    ig, iu = synth.make_indices(seed, 0, N, K, bits), synth.make_indices(seed, 1, N, K, bits)
    sym = bits == 1
    cg, cu = synth.make_codebook(seed, 0, N, bits, symmetric=sym), synth.make_codebook(seed, 1, N, bits, symmetric=sym)
    # activations scaled so that the gate spans the interesting range of silu (|g| up to a few units)
    x = synth.f32_to_bf16((synth.bf16_to_f32(synth.make_x(seed, 0, 1, K)[0]) * np.float32(40.0 / np.sqrt(K))))
    y = torch.full((N,), 0x7FC1, dtype=torch.int16, device="cuda")
    pg, pu = kmq.pack(ig, bits), kmq.pack(iu, bits)
    if layout:
        pg, pu = kmq.repack(pg, K, bits, layout), kmq.repack(pu, K, bits, layout)
    kmq.gemv_swiglu(gpu.dev(pg), gpu.dev(cg), gpu.dev(pu), gpu.dev(cu), gpu.dev(x), y, N, K, bits, layout)
    torch.cuda.synchronize()
    yg = synth.bf16_to_f64(gpu.host_u16(y))
    G, Ag, _ = oracle.gemm(oracle.pack(ig, bits), cg, x, K, bits)
    U, Au, _ = oracle.gemm(oracle.pack(iu, bits), cu, x, K, bits)
    want = oracle.swiglu(G, U)
    silu = oracle.swiglu(G, np.ones_like(G))
    bound = gpu.swiglu_bound(G, U, Ag, Au, silu, want, K)
    err = np.abs(yg - want)
    assert np.all(err <= bound), f"b{bits} {N}x{K}: max err/bound {np.max(err / np.maximum(bound, 1e-300)):.2f}"
    if N >= 64:
        assert np.abs(G).max() > 0.5       # the test does exercise the non-linear part


LUT_SHAPES = [(1, 1536), (1, 2048), (1, 3072), (1, 4096), (1, 6144), (1, 8192), (2, 1536), (2, 2048), (2, 3072), (2, 4096), (2, 6144),
              (2, 8192), (2, 14336), (3, 1536), (3, 2048), (3, 3072), (3, 4096), (3, 6144), (3, 8192), (3, 14336),
              (4, 1536), (4, 2048), (4, 4096), (4, 6144), (4, 8192), (4, 14336)]


@pytest.mark.parametrize("bits,K", LUT_SHAPES)
@pytest.mark.parametrize("N", (1, 2, 5, 17, 64, 333))
def test_fused_pair_on_the_table_kernels(gpu, bits, K, N):
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name_swiglu(N, K, bits).startswith("lut_"), kmq.kernel_name_swiglu(N, K, bits)
    _check(gpu, bits, N, K, 7 * bits + N + K)


# row-lane layout: 1, 2, 3 and 4 tiles per wave (K / 256 = 1 .. 56 tiles)
@pytest.mark.parametrize("bits", (1, 2))
@pytest.mark.parametrize("K", (256, 1024, 1536, 2048, 3072, 4096, 6144, 8192, 12288, 14336))
@pytest.mark.parametrize("N", (1, 16, 17, 64, 333))
def test_fused_pair_on_the_rowlane_kernels(gpu, bits, K, N):
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name_swiglu(N, K, bits, kmq.LAYOUT_ROWLANE) == f"rowlane_pair_b{bits}"
    _check(gpu, bits, N, K, 11 * bits + N + K, layout=kmq.LAYOUT_ROWLANE)


def test_fused_pair_rowlane_rejections(gpu):
    """3 and 4 bits have no row-lane layout; tile counts that need more than four tiles per wave or the round loop
    have no fused kernel: KMQ_ERR_LAYOUT before any launch."""
    from paper_2602_15563_amd import kmq
    z = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    y = torch.zeros(64, dtype=torch.int16, device="cuda")
    for bits, K in ((3, 4096), (4, 4096), (2, 256 * 17), (1, 256 * 96), (2, 4000)):
        assert kmq.kernel_name_swiglu(16, K, bits, kmq.LAYOUT_ROWLANE) == "invalid"
        with pytest.raises(kmq.KmqError) as e:
            kmq.gemv_swiglu(z, z, z, z, z, y, 16, K, bits, kmq.LAYOUT_ROWLANE)
        assert e.value.status == 7          # KMQ_ERR_LAYOUT


@pytest.mark.parametrize("bits,N,K", [(3, 40, 1024), (2, 9, 515), (4, 100, 33), (1, 7, 1), (3, 130, 1000)])
def test_fused_pair_any_shape(gpu, bits, N, K):
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name_swiglu(N, K, bits) == "pair_generic"
    _check(gpu, bits, N, K, 3 * bits + N + K)


def test_decoder_shape_and_two_separate_calls_agree(gpu):
    """gate/up of the 1-bit decoder layer (8192 x 3072): the fused call against two kmq_gemv calls
    combined on the host in fp64; they differ by the bf16 rounding of the two intermediate vectors."""
    from paper_2602_15563_amd import kmq
    bits, N, K = 1, 8192, 3072
    ig, iu = synth.make_indices(4, 2, N, K, bits), synth.make_indices(4, 3, N, K, bits)
    cg, cu = synth.make_codebook(4, 2, N, bits, symmetric=True), synth.make_codebook(4, 3, N, bits, symmetric=True)
    x = synth.make_x(4, 2, 1, K)[0]
    pg, pu = gpu.dev(kmq.pack(ig, bits)), gpu.dev(kmq.pack(iu, bits))
    y = torch.full((N,), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.gemv_swiglu(pg, gpu.dev(cg), pu, gpu.dev(cu), gpu.dev(x), y, N, K, bits)
    torch.cuda.synchronize()
    fused = synth.bf16_to_f64(gpu.host_u16(y))
    g = synth.bf16_to_f64(gpu.run_gemm(pg, gpu.dev(cg), x, N, K, bits)[0])
    u = synth.bf16_to_f64(gpu.run_gemm(pu, gpu.dev(cu), x, N, K, bits)[0])
    two = oracle.swiglu(g, u)
    # g and u each carry one bf16 rounding (relative 2^-8) in the two-call form, the fused result one
    assert np.all(np.abs(fused - two) <= 2.0 ** -7 * np.abs(two) + 1.1 * 2.0 ** -8 * np.abs(u * g) + 1e-9)


def test_errors(gpu):
    from paper_2602_15563_amd import kmq
    z = torch.zeros(4096, dtype=torch.int16, device="cuda")
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv_swiglu(z, z, None, z, z, z, 4, 64, 2)
    assert e.value.status == 1
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv_swiglu(z, z, z, z, z, z, 4, 256, 2, layout=1)
    assert e.value.status == 7
