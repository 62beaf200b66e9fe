"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer work (dequantised weights, one-hot probes)
must be bit-exact; products must satisfy |err| <= 2e-3 * sum_k |w x|."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_15563_amd import synth

pytestmark = pytest.mark.gpu

BITS = (1, 2, 3, 4)


def _small_case(seed, N, K, bits, M):
    g = np.random.default_rng(seed)
    idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    cb = synth.f32_to_bf16(g.normal(0, 0.02, size=(N, 1 << bits)).astype(np.float32))
    X = synth.f32_to_bf16(g.standard_normal(size=(M, K)).astype(np.float32))
    return idx, cb, X


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    assert torch.cuda.is_available()
    return gpu_util


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("layout", (0, 1))
@pytest.mark.parametrize("N,K", [(1, 1), (5, 33), (37, 100), (67, 515), (130, 4096), (16, 128), (33, 1024)])
def test_dequant_bit_exact(gpu, bits, layout, N, K):
    from paper_2602_15563_amd import kmq
    idx, cb, _ = _small_case(bits * 100 + N + K, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    if layout == 1:
        if kmq.tiled_words(N, K, bits, 1) < 0:
            pytest.skip("tiled layout needs K to be whole super-blocks")
        stored = kmq.repack(p, K, bits, 1)
    else:
        stored = p
    Wd = torch.full((N, K), 0x7FC1, dtype=torch.int16, device="cuda")
    kmq.dequant(gpu.dev(stored), gpu.dev(cb), Wd, N, K, bits, layout)
    torch.cuda.synchronize()
    assert np.array_equal(gpu.host_u16(Wd), oracle.dequant(oracle.pack(idx, bits), cb, K, bits))


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("M", (1, 2, 3, 4, 7, 8, 13, 16))
@pytest.mark.parametrize("N,K", [(1, 1), (3, 31), (67, 100), (300, 515), (130, 1024), (77, 2048)])
def test_generic_shapes_vs_oracle(gpu, bits, M, N, K):
    """Ragged shapes that only the shape-agnostic kernel handles (several tiles + tails)."""
    from paper_2602_15563_amd import kmq
    idx, cb, X = _small_case(7 * bits + M + N + K, N, K, bits, M)
    p = kmq.pack(idx, bits)
    Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X, N, K, bits)
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, label=f"b{bits} {N}x{K} M{M}")


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("N,K", [(1, 512), (15, 1024), (17, 1024), (33, 1536), (130, 1024), (48, 4096), (300, 3072)])
@pytest.mark.parametrize("M", (1, 2, 5, 8, 13, 16))
def test_tiled_layout_mfma_vs_oracle(gpu, bits, N, K, M):
    """The matrix-core kernel: every batch size, ragged row counts (short last
    16-row block), K with 1, 2, 3, 4, 6, 8 super-blocks per wave split."""
    from paper_2602_15563_amd import kmq
    idx, cb, X = _small_case(11 * bits + N + M + K, N, K, bits, M)
    p = kmq.pack(idx, bits)
    assert kmq.kernel_name(N, K, bits, M, 1).startswith("mfma")
    Yg = gpu.run_gemm(gpu.dev(kmq.repack(p, K, bits, 1)), gpu.dev(cb), X, N, K, bits, layout=1, use_gemv=(M == 1))
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, label=f"tiled b{bits} {N}x{K} M{M}")


@pytest.mark.parametrize("bits", (2, 3, 4))
def test_tiled_one_hot_batch16_probe_is_bit_exact(gpu, bits):
    from paper_2602_15563_amd import kmq
    N, K = 40, 1024
    idx, cb, _ = _small_case(3 * bits, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    Wd = oracle.dequant(oracle.pack(idx, bits), cb, K, bits)
    pd, cd = gpu.dev(kmq.repack(p, K, bits, 1)), gpu.dev(cb)
    for k0 in (0, 8, 24, 100, 511, K - 16):
        X = np.zeros((16, K), dtype=np.uint16)
        for m in range(16):
            X[m, k0 + m] = 0x3F80
        Yg = gpu.run_gemm(pd, cd, X, N, K, bits, layout=1)
        assert np.array_equal(Yg, Wd[:, k0:k0 + 16].T.copy()), f"k0={k0}"


@pytest.mark.parametrize("cfg", (3, 4))
def test_contract_configs_tiled(gpu, cfg):
    """The small-batch configurations at full size on the tiled layout (the
    launch configuration bench.py times for batch > 1)."""
    from paper_2602_15563_amd import kmq
    for case in synth.cases(cfg):
        idx, cb, X = case.tensors()
        p = kmq.pack(idx, case.bits)
        t = kmq.repack(p, case.K, case.bits, 1)
        assert np.array_equal(kmq.unrepack(t, case.N, case.K, case.bits, 1), p)
        Yg = gpu.run_gemm(gpu.dev(t), gpu.dev(cb), X, case.N, case.K, case.bits, layout=1, use_gemv=False)
        ranges = gpu.sample_ranges(case.N, case.seed + case.matrix)
        worst = gpu.check_against_oracle(Yg, p, cb, X, case.K, case.bits, ranges, label=case.name)
        print(f"{case.name}: kernel={kmq.kernel_name(case.N, case.K, case.bits, case.M, 1)} max err/A={worst:.2e}")


FAST_SHAPES = [(1, 1536), (1, 2048), (1, 3072), (1, 4096), (1, 6144), (1, 8192), (2, 1536), (2, 2048), (2, 3072), (2, 4096), (2, 6144),
               (2, 8192), (2, 14336), (3, 1536), (3, 2048), (3, 3072), (3, 4096), (3, 6144), (3, 8192), (3, 14336),
               (4, 1536), (4, 2048), (4, 4096), (4, 6144), (4, 8192), (4, 14336)]


@pytest.mark.parametrize("bits,K", FAST_SHAPES)
@pytest.mark.parametrize("N", (1, 2, 3, 15, 16, 17, 64, 333))
def test_specialised_gemv_vs_oracle(gpu, bits, K, N):
    """Every (bits, K) the batch-1 specialisations cover, with row counts around
    the rows-per-workgroup boundaries (ragged last workgroup)."""
    from paper_2602_15563_amd import kmq
    idx, cb, X = _small_case(13 * bits + N + K, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    assert kmq.kernel_name(N, K, bits, 1).startswith("lut_"), kmq.kernel_name(N, K, bits, 1)
    Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X[0], N, K, bits)
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, label=f"b{bits} {N}x{K}")


@pytest.mark.parametrize("bits,K,N,shape", [
    (1, 2048, 4090, "_r4x1"), (1, 2048, 2040, "_r2x1"),
    (1, 3072, 9209, "_r3x3"), (1, 3072, 8190, "_r4x2"), (1, 3072, 3070, "_r3x2"),
    (1, 8192, 3065, "_r4x3"), (1, 8192, 2047, "_r4x2"),
])
def test_gemv_shape_choice_by_rows(gpu, bits, K, N, shape):
    """Where several launch shapes serve one (bits, K), the row count picks the one whose
    grid is most even over the CUs; every such shape at an N that selects it, ragged."""
    from paper_2602_15563_amd import kmq
    assert kmq.kernel_name(N, K, bits, 1).endswith(shape), kmq.kernel_name(N, K, bits, 1)
    idx, cb, X = _small_case(7 * bits + N + K, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X[0], N, K, bits)
    gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb, X, K, bits, label=f"b{bits} {N}x{K}")


@pytest.mark.parametrize("bits,K", [(2, 4096), (2, 14336), (3, 4096), (4, 4096), (2, 100), (3, 515), (4, 33)])
def test_one_hot_probe_is_bit_exact(gpu, bits, K):
    """x = e_k makes every output a single weight: y[n] must equal the bf16
    centroid exactly, which checks unpack + lookup inside the production kernels."""
    from paper_2602_15563_amd import kmq
    N = 40
    idx, cb, _ = _small_case(17 * bits + K, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    Wd = oracle.dequant(oracle.pack(idx, bits), cb, K, bits)
    pd, cd = gpu.dev(p), gpu.dev(cb)
    for k in sorted({0, 1, 10, 21, 31, 32, K // 2 + 1, K - 2 if K > 2 else 0, K - 1}):
        x = np.zeros(K, dtype=np.uint16)
        x[k] = 0x3F80
        Yg = gpu.run_gemm(pd, cd, x, N, K, bits)
        assert np.array_equal(Yg[0], Wd[:, k]), f"k={k}"


def test_one_hot_batch16_probe_is_bit_exact(gpu):
    from paper_2602_15563_amd import kmq
    bits, N, K = 3, 48, 4096
    idx, cb, _ = _small_case(99, N, K, bits, 1)
    p = kmq.pack(idx, bits)
    Wd = oracle.dequant(oracle.pack(idx, bits), cb, K, bits)
    pd, cd = gpu.dev(p), gpu.dev(cb)
    for k0 in (0, 20, 1000, K - 16):
        X = np.zeros((16, K), dtype=np.uint16)
        for m in range(16):
            X[m, k0 + m] = 0x3F80
        Yg = gpu.run_gemm(pd, cd, X, N, K, bits)
        assert np.array_equal(Yg, Wd[:, k0:k0 + 16].T.copy())


@pytest.mark.parametrize("cfg", range(5))
def test_contract_configs_full_size(gpu, cfg):
    """The five benchmark configurations at full size, in the launch
    configuration bench.py times; compared on sampled row blocks (first, last,
    random), and on every row when the matrix is small."""
    from paper_2602_15563_amd import kmq
    for case in synth.cases(cfg):
        idx, cb, X = case.tensors()
        p = kmq.pack(idx, case.bits)
        Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X if case.M > 1 else X[0], case.N, case.K, case.bits)
        full = case.N * case.K * case.M <= 20_000_000
        ranges = None if full else gpu.sample_ranges(case.N, case.seed + case.matrix)
        worst = gpu.check_against_oracle(Yg, p, cb, X, case.K, case.bits, ranges, label=case.name)
        print(f"{case.name}: kernel={kmq.kernel_name(case.N, case.K, case.bits, case.M)} max err/A={worst:.2e}")


def test_full_rows_headline_shape(gpu):
    """Every output of the headline shape (2-bit 14336 x 4096, batch 1)."""
    from paper_2602_15563_amd import kmq
    case = synth.cases(2)[0]
    idx, cb, X = case.tensors()
    p = kmq.pack(idx, case.bits)
    Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X[0], case.N, case.K, case.bits)
    gpu.check_against_oracle(Yg, p, cb, X, case.K, case.bits, label=case.name)


def test_run_to_run_determinism(gpu):
    from paper_2602_15563_amd import kmq
    for bits, N, K, M in [(2, 999, 4096, 1), (1, 500, 3072, 1), (3, 300, 4096, 16), (4, 200, 515, 4)]:
        idx, cb, X = _small_case(5, N, K, bits, M)
        pd, cd = gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb)
        a = gpu.run_gemm(pd, cd, X, N, K, bits)
        for _ in range(3):
            assert np.array_equal(gpu.run_gemm(pd, cd, X, N, K, bits), a)


def test_gemv_equals_gemm_with_batch_one(gpu):
    from paper_2602_15563_amd import kmq
    bits, N, K = 2, 100, 4096
    idx, cb, X = _small_case(6, N, K, bits, 1)
    pd, cd = gpu.dev(kmq.pack(idx, bits)), gpu.dev(cb)
    assert np.array_equal(gpu.run_gemm(pd, cd, X, N, K, bits, use_gemv=True),
                          gpu.run_gemm(pd, cd, X, N, K, bits, use_gemv=False))


def test_degenerate_inputs(gpu):
    """Zero activations, constant codebooks, all-max indices."""
    from paper_2602_15563_amd import kmq
    for bits, K in [(1, 2048), (2, 4096), (3, 100), (4, 4096)]:
        N = 20
        idx, cb, X = _small_case(8, N, K, bits, 1)
        pd = gpu.dev(kmq.pack(idx, bits))
        y0 = synth.bf16_to_f64(gpu.run_gemm(pd, gpu.dev(cb), np.zeros(K, np.uint16), N, K, bits))
        assert not y0.any()                                      # +-0 allowed
        cb2 = cb.copy()
        cb2[:] = cb2[:, :1]
        Yg = gpu.run_gemm(pd, gpu.dev(cb2), X[0], N, K, bits)
        gpu.check_against_oracle(Yg, oracle.pack(idx, bits), cb2, X, K, bits, label="const codebook", strict=False)
        idx[:] = (1 << bits) - 1
        p = kmq.pack(idx, bits)
        Yg = gpu.run_gemm(gpu.dev(p), gpu.dev(cb), X[0], N, K, bits)
        gpu.check_against_oracle(Yg, p, cb, X, K, bits, label="all-max indices")


@pytest.mark.parametrize("bits,N,K,M", [(1, 9216, 3072, 4), (1, 300, 3072, 2), (2, 1000, 4096, 3), (2, 333, 14336, 4),
                                        (4, 4096, 4096, 2), (4, 77, 8192, 4), (1, 64, 8192, 3),
                                        (3, 1000, 4096, 2), (3, 4096, 14336, 4), (3, 130, 2048, 3),
                                        (2, 14336, 4096, 16), (1, 9216, 3072, 7), (3, 17, 4096, 16), (4, 64, 8192, 9),
                                        (2, 7, 2048, 5), (1, 4090, 2048, 16), (3, 1500, 3072, 8)])
def test_batches_on_the_canonical_layout_per_column(gpu, bits, N, K, M):
    """Batches on the canonical layout may run the batch-1 table kernel over a (row group, column) grid in one
    launch (a cost model in the heuristic decides): whatever is chosen must match the oracle, and a per-column
    result is the batch-1 result of each column bit for bit.  Row counts that leave the padded grid (a multiple
    of 8 row groups per column) partly empty are part of the list."""
    from paper_2602_15563_amd import kmq
    seed = 900 + bits + M
    idx = synth.make_indices(seed, 0, N, K, bits)
    cb = synth.make_codebook(seed, 0, N, bits, symmetric=(bits == 1))
    X = synth.make_x(seed, 0, M, K)
    packed = oracle.pack(idx, bits)
    name = kmq.kernel_name(N, K, bits, M)
    Wd, cbd = gpu.dev(packed), gpu.dev(cb)
    Yg = gpu.run_gemm(Wd, cbd, X, N, K, bits)
    ranges = gpu.sample_ranges(N, seed)
    gpu.check_against_oracle(Yg, packed, cb, X, K, bits, row_ranges=ranges, label=f"b{bits} {N}x{K} M{M} ({name})")
    if name.startswith("lut_"):
        for m in range(M):
            assert np.array_equal(Yg[m], gpu.run_gemm(Wd, cbd, X[m], N, K, bits)[0])


@pytest.mark.parametrize("bits,N,K,M,layout", [(1, 70, 3072, 1, 0), (2, 130, 4096, 1, 0), (3, 90, 4096, 1, 0), (3, 50, 3072, 1, 0),
                                               (4, 64, 8192, 1, 0), (3, 33, 515, 1, 0), (2, 40, 1000, 3, 0),
                                               (2, 100, 4096, 2, 0), (3, 64, 4096, 8, 1), (4, 48, 2048, 16, 1)])
def test_operands_at_their_minimum_alignment(gpu, bits, N, K, M, layout):
    """The contract asks 16 bytes of W and X but only 4 of the codebook and 2 of Y: the kernels' vector loads of
    codebook rows and their paired output stores must cope with exactly that."""
    import torch
    from paper_2602_15563_amd import kmq
    seed = 1300 + bits + M
    idx = synth.make_indices(seed, 0, N, K, bits)
    cb = synth.make_codebook(seed, 0, N, bits, symmetric=(bits == 1))
    X = synth.make_x(seed, 0, M, K)
    packed = oracle.pack(idx, bits)
    Wd = gpu.dev(kmq.repack(packed, K, bits, kmq.LAYOUT_TILED) if layout else packed)
    cbuf = torch.zeros(cb.size + 8, dtype=torch.int16, device="cuda")
    ybuf = torch.full((M * N + 8,), 0x7FC1, dtype=torch.int16, device="cuda")
    for c_off, y_off in ((2, 1), (6, 3), (4, 0)):             # int16 elements: 4, 12, 8 and 2, 6, 0 bytes
        cbd = cbuf[c_off:c_off + cb.size].view(N, -1)
        cbd.copy_(gpu.dev(cb))
        ybuf.fill_(0x7FC1)
        Y = ybuf[y_off:y_off + M * N].view(M, N)
        assert cbd.data_ptr() % 16 == (2 * c_off) % 16 and Y.data_ptr() % 4 == (2 * y_off) % 4
        ws_bytes = kmq.workspace_bytes(N, K, bits, M, layout)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda") if ws_bytes else None
        if M == 1:
            kmq.gemv(Wd, cbd, gpu.dev(X), Y, N, K, bits, layout, ws)
        else:
            kmq.gemm_smallbatch(Wd, cbd, gpu.dev(X), Y, N, K, M, bits, layout, ws)
        torch.cuda.synchronize()
        gpu.check_against_oracle(gpu.host_u16(Y), packed, cb, X, K, bits,
                                 label=f"b{bits} {N}x{K} M{M} codebook+{2 * c_off}B y+{2 * y_off}B")
        assert int(ybuf[y_off + M * N]) == 0x7FC1 and (y_off == 0 or int(ybuf[y_off - 1]) == 0x7FC1)   # nothing outside Y
