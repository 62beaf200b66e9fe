"""GPU parity of the decoder-layer fusions (RMSNorm in front of a product, residual behind it, and the
RMSNorm + gate / up / SwiGLU call) against the oracle's definition, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_15563_amd import synth

pytestmark = pytest.mark.gpu
EPS = 1e-5


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    return gpu_util


def _inputs(seed, bits, N, K):
    idx = synth.make_indices(seed, 0, N, K, bits)
    cb = synth.make_codebook(seed, 0, N, bits, symmetric=(bits == 1))
    x = synth.make_x(seed, 0, 1, K)[0]
    return idx, cb, x, synth.make_norm_weight(seed, 0, K), synth.make_residual(seed, 0, N)


def _run(gpu, idx, cb, x, bits, g=None, res=None, alias=False, unit=False):
    from paper_2602_15563_amd import kmq
    N, K = idx.shape
    y = gpu.dev(res) if alias else torch.full((N,), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.gemv_fused(gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb), gpu.dev(x), y, N, K, bits,
                   norm_weight=None if g is None else gpu.dev(g), eps=EPS,
                   residual=None if res is None else (y if alias else gpu.dev(res)), rmsnorm=True if unit else None)
    torch.cuda.synchronize()
    return synth.bf16_to_f64(gpu.host_u16(y))


def _check(gpu, yg, idx, cb, x, bits, g, res, label, unit=False):
    N, K = idx.shape
    Y, A = oracle.gemv_fused(oracle.pack(idx, bits), cb, x, K, bits, norm_weight=g, eps=EPS, residual=res,
                             rmsnorm=True if unit else None)
    err = np.abs(yg - Y)
    # fp32 sums in any order, the scalar in fp32 (a few roundings), one bf16 rounding of the result
    bound = gpu.arithmetic_bound(A, Y, K + 16)
    if g is not None or unit:
        # the oracle rounds x*r*g to bf16, the kernels round x*g and apply r to the sum (tolerance.py, item 4)
        Ap = A - (np.abs(synth.bf16_to_f64(res)) if res is not None else 0.0)
        bound = bound + gpu.rmsnorm_commute_bound(Ap)
    bad = err > bound
    if K >= 512:
        bad |= err > gpu.TOL * A + 2.0 ** -8 * np.abs(Y)
    assert not bad.any(), f"{label}: {int(bad.sum())} beyond tolerance, worst err/A {np.max(err / np.maximum(A, 1e-300)):.3e}"


MODES = [("norm", True, False), ("res", False, True), ("both", True, True), ("plain", False, False),
         ("unit", "unit", False), ("unit+res", "unit", True)]
LUT_SHAPES = [(1, 2048, 64), (1, 2048, 333), (1, 3072, 100), (1, 3072, 3072), (1, 4096, 50), (1, 8192, 96), (1, 8192, 3072),
              (2, 2048, 40), (2, 3072, 77), (2, 4096, 1000), (2, 8192, 64), (2, 14336, 130),
              (3, 2048, 90), (3, 3072, 50), (3, 4096, 333), (3, 8192, 64), (3, 14336, 70),
              (4, 2048, 40), (4, 4096, 333), (4, 8192, 64), (4, 14336, 70),
              (1, 1536, 70), (1, 6144, 50), (2, 1536, 33), (2, 6144, 40), (3, 1536, 50), (3, 6144, 30), (4, 1536, 20), (4, 6144, 45)]


@pytest.mark.parametrize("mode,use_g,use_r", MODES)
@pytest.mark.parametrize("bits,K,N", LUT_SHAPES)
def test_fused_on_the_table_kernels(gpu, bits, K, N, mode, use_g, use_r):
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name_fused(N, K, bits).startswith(f"lut_b{bits}")
    idx, cb, x, g, res = _inputs(500 + K // 64 + N, bits, N, K)
    print(f"fused {mode} b{bits} {N}x{K}", flush=True)
    unit = use_g == "unit"
    gg = g if use_g is True else None
    yg = _run(gpu, idx, cb, x, bits, gg, res if use_r else None, unit=unit)
    _check(gpu, yg, idx, cb, x, bits, gg, res if use_r else None, f"{mode} b{bits} {N}x{K}", unit=unit)


@pytest.mark.parametrize("mode,use_g,use_r", MODES)
# (row lengths that are multiples of 32 without a specialised kernel: with no RMSNorm in front, the table kernel that
# walks K in rounds takes the residual; 5120 and 21504 are SwiGLU widths of App. A's architectures)
@pytest.mark.parametrize("bits,N,K", [(3, 40, 1024), (3, 33, 515), (4, 100, 33), (1, 7, 1), (1, 9, 1000), (2, 64, 1024),
                                      (4, 1001, 5120), (3, 300, 21504), (1, 515, 7168)])
def test_fused_any_shape(gpu, bits, N, K, mode, use_g, use_r):
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name_fused(N, K, bits) == "fused_generic"
    idx, cb, x, g, res = _inputs(600 + bits + N, bits, N, K)
    unit = use_g == "unit"
    gg = g if use_g is True else None
    yg = _run(gpu, idx, cb, x, bits, gg, res if use_r else None, unit=unit)
    _check(gpu, yg, idx, cb, x, bits, gg, res if use_r else None, f"{mode} b{bits} {N}x{K}", unit=unit)


def test_plain_mode_equals_kmq_gemv_bit_for_bit(gpu):
    for bits, K, N in [(1, 3072, 200), (1, 8192, 64), (2, 4096, 300), (4, 4096, 100)]:
        idx, cb, x, _, _ = _inputs(700 + N, bits, N, K)
        from paper_2602_15563_amd import kmq
        a = _run(gpu, idx, cb, x, bits)
        b = synth.bf16_to_f64(gpu.run_gemm(gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb), x, N, K, bits)[0])
        assert np.array_equal(a, b)


def test_residual_may_alias_the_output(gpu):
    idx, cb, x, g, res = _inputs(710, 1, 3072, 3072)
    a = _run(gpu, idx, cb, x, 1, g, res)
    b = _run(gpu, idx, cb, x, 1, g, res, alias=True)
    assert np.array_equal(a, b)


def test_residual_may_alias_the_output_in_the_kernel_that_walks_k(gpu):
    """No RMSNorm, a row length without a specialised kernel: the residual goes to the epilogue of the table kernel
    that walks K in rounds; y = residual + product with the residual read from y itself."""
    from paper_2602_15563_amd import kmq
    bits, N, K = 3, 1001, 5120
    assert kmq.kernel_name(N, K, bits, 1) == "lut_loop_b3"
    idx, cb, x, _, res = _inputs(715, bits, N, K)
    a = _run(gpu, idx, cb, x, bits, None, res)
    b = _run(gpu, idx, cb, x, bits, None, res, alias=True)
    assert np.array_equal(a, b)
    plain = _run(gpu, idx, cb, x, bits)
    assert not np.array_equal(a, plain)


def test_unit_weights_reduce_to_a_scaled_product(gpu):
    """g = 1: the activations pass unchanged and the result is the plain product times r."""
    N, K = 128, 3072
    idx, cb, x, _, _ = _inputs(720, 1, N, K)
    one = synth.f32_to_bf16(np.ones(K, np.float32))
    yg = _run(gpu, idx, cb, x, 1, one, None)
    Y0, A0, _ = oracle.gemm(oracle.pack(idx, 1), cb, x.reshape(1, -1), K, 1)
    xd = synth.bf16_to_f64(x)
    r = 1.0 / np.sqrt(np.mean(xd * xd) + EPS)       # (the kernels apply the scalar to the sum: with unit gains that is exactly this)
    assert np.all(np.abs(yg - Y0[0] * r) <= gpu.arithmetic_bound(A0[0] * r, Y0[0] * r, K + 16))


def _swiglu_norm(gpu, bits, N, K, seed, unit=False):
    from paper_2602_15563_amd import kmq
    ig, iu = synth.make_indices(seed, 0, N, K, bits), synth.make_indices(seed, 1, N, K, bits)
    sym = bits == 1
    cg, cu = synth.make_codebook(seed, 0, N, bits, symmetric=sym), synth.make_codebook(seed, 1, N, bits, symmetric=sym)
    x = synth.f32_to_bf16(synth.bf16_to_f32(synth.make_x(seed, 0, 1, K)[0]) * np.float32(3.0))
    # gains large enough that the gate spans the non-linear range of silu after normalisation
    g = None if unit else synth.make_norm_weight(seed, 0, K, gain=40.0 / np.sqrt(K))
    y = torch.full((N,), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.gemv_swiglu_rmsnorm(gpu.dev(kmq.pack(ig, bits)), gpu.dev(cg), gpu.dev(kmq.pack(iu, bits)), gpu.dev(cu), gpu.dev(x),
                            None if unit else gpu.dev(g), EPS, y, N, K, bits)
    torch.cuda.synchronize()
    yg = synth.bf16_to_f64(gpu.host_u16(y))
    G, Ag = oracle.gemv_fused(oracle.pack(ig, bits), cg, x, K, bits, norm_weight=g, eps=EPS, rmsnorm=True)
    U, Au = oracle.gemv_fused(oracle.pack(iu, bits), cu, x, K, bits, norm_weight=g, eps=EPS, rmsnorm=True)
    want = oracle.swiglu(G, U)
    silu = oracle.swiglu(G, np.ones_like(G))
    err = np.abs(yg - want)
    # guarantee: fp32 sums plus the rounding-point difference of the normalised activations (2^-7 of
    # sum |w xn|: the oracle rounds x*r*g, the kernels round x*g and scale the sum), through silu' in [-0.1, 1.1]
    for dg, du, what in (((K + 24) * 2.0 ** -23 * Ag + 2.0 ** -7 * Ag, (K + 24) * 2.0 ** -23 * Au + 2.0 ** -7 * Au, "guaranteed"),
                         (2e-3 * Ag, 2e-3 * Au, "contract (independent roundings add in quadrature)")):
        inner = 1.1 * np.abs(U) * dg + np.abs(silu) * du + 1.1 * dg * du + 8 * 2.0 ** -23 * np.abs(want)
        bound = inner + 2.0 ** -8 * (np.abs(want) + inner)
        assert np.all(err <= bound), f"b{bits} {N}x{K}, {what}: max err/bound {np.max(err / np.maximum(bound, 1e-300)):.2f}"


@pytest.mark.parametrize("bits,K,N", [(1, 2048, 40), (1, 3072, 64), (1, 3072, 8192), (1, 4096, 333), (1, 8192, 17),
                                      (2, 4096, 14336), (2, 14336, 50), (4, 4096, 100), (4, 8192, 33)])
def test_swiglu_rmsnorm_on_the_table_kernels(gpu, bits, K, N):
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name_fused(N, K, bits, pair=True).startswith(f"lut_b{bits}")
    _swiglu_norm(gpu, bits, N, K, 800 + N)
    _swiglu_norm(gpu, bits, N, K, 850 + N, unit=True)


@pytest.mark.parametrize("bits,N,K", [(3, 40, 1024), (3, 33, 515), (4, 20, 33), (1, 9, 1000)])
def test_swiglu_rmsnorm_any_shape(gpu, bits, N, K):
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name_fused(N, K, bits, pair=True) == "fused_generic"
    _swiglu_norm(gpu, bits, N, K, 900 + N)
    _swiglu_norm(gpu, bits, N, K, 950 + N, unit=True)


def test_errors(gpu):
    from paper_2602_15563_amd import kmq
    idx, cb, x, g, res = _inputs(950, 2, 8, 64)
    W, cbd, xd, gd = gpu.dev(kmq.pack(idx, 2)), gpu.dev(cb), gpu.dev(x), gpu.dev(g)
    y = torch.zeros(8, dtype=torch.int16, device="cuda")
    for call, status in [
        (lambda: kmq.gemv_fused(W, cbd, xd, y, 8, 64, 2, layout=1), 7),
        (lambda: kmq.gemv_fused(W, cbd, xd, y, 8, 64, 5), 2),
        (lambda: kmq.gemv_fused(W, cbd, xd, y, 8, 64, 2, norm_weight=gd, eps=-1.0), 3),
        (lambda: kmq.gemv_fused(W, cbd, None, y, 8, 64, 2), 1),
        (lambda: kmq.gemv_swiglu_rmsnorm(W, cbd, W, cbd, None, gd, EPS, y, 8, 64, 2), 1),
        (lambda: kmq.gemv_swiglu_rmsnorm(W, cbd, W, cbd, xd, gd, -1.0, y, 8, 64, 2), 3),
        (lambda: kmq.gemv_fused(W, cbd, xd, y, 8, 64, 2, norm_weight=gd[1:]), 4),
    ]:
        with pytest.raises(kmq.KmqError) as e:
            call()
        assert e.value.status == status
