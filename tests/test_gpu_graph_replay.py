"""The device calls are legal inside HIP graph capture (nothing allocates, nothing
synchronises): capture one call of each kind, replay the graph several times with eager work
and synchronisations in between, and compare every replay with the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2602_15563_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    return gpu_util


def test_graph_replays_match_eager(gpu):
    from paper_2602_15563_amd import kmq
    dev = gpu.dev
    # batch-1 table kernel, matrix-core kernel on the tiled layout, block-scaled GEMV, shape-agnostic kernel
    N1, K1, b1 = 300, 4096, 2
    N2, K2, b2, M2 = 96, 4096, 3, 8
    N3, K3, b3 = 130, 8192, 4
    N4, K4, b4, M4 = 77, 515, 4, 3
    idx1, cb1, x1 = synth.make_indices(1, 0, N1, K1, b1), synth.make_codebook(1, 0, N1, b1), synth.make_x(1, 0, 1, K1)
    idx2, cb2, X2 = synth.make_indices(2, 0, N2, K2, b2), synth.make_codebook(2, 0, N2, b2), synth.make_x(2, 0, M2, K2)
    idx3, cb3, sc3, x3 = (synth.make_indices(3, 0, N3, K3, b3), synth.make_shared_codebook(3, 0, b3),
                          synth.make_scales(3, 0, N3, K3), synth.make_x(3, 0, 1, K3))
    idx4, cb4, X4 = synth.make_indices(4, 0, N4, K4, b4), synth.make_codebook(4, 0, N4, b4), synth.make_x(4, 0, M4, K4)
    W1, C1, Xd1 = dev(kmq.pack(idx1, b1)), dev(cb1), dev(x1)
    W2, C2, Xd2 = dev(kmq.repack(kmq.pack(idx2, b2), K2, b2, 1)), dev(cb2), dev(X2)
    W3, C3, S3, Xd3 = dev(kmq.pack(idx3, b3)), dev(cb3), dev(sc3), dev(x3)
    W4, C4, Xd4 = dev(kmq.pack(idx4, b4)), dev(cb4), dev(X4)

    def outputs():
        return (torch.full((1, N1), 0x7FC1, dtype=torch.int16, device="cuda"),
                torch.full((M2, N2), 0x7FC1, dtype=torch.int16, device="cuda"),
                torch.full((1, N3), 0x7FC1, dtype=torch.int16, device="cuda"),
                torch.full((M4, N4), 0x7FC1, dtype=torch.int16, device="cuda"))

    def run(Y):
        kmq.gemv(W1, C1, Xd1, Y[0], N1, K1, b1)
        kmq.gemm_smallbatch(W2, C2, Xd2, Y[1], N2, K2, M2, b2, 1)
        kmq.gemv_blockscaled(W3, C3, S3, Xd3, Y[2], N3, K3, b3)
        kmq.gemm_smallbatch(W4, C4, Xd4, Y[3], N4, K4, M4, b4)

    eager = outputs()
    run(eager)
    torch.cuda.synchronize()
    want = [y.clone() for y in eager]

    captured = outputs()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        run(captured)                         # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            run(captured)
    for replay in range(4):
        for y in captured:                    # poison the outputs, with a fill kernel
            y.fill_(0x7FC1)
        run(eager)                            # eager work of the program between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (y, w) in enumerate(zip(captured, want)):
            assert torch.equal(y, w), f"replay {replay}, call {i}"
        for y, w in zip(eager, want):
            assert torch.equal(y, w)


def test_graph_replays_of_the_multi_kernel_and_fused_calls(gpu):
    """The calls that launch more than one kernel (split-K with its workspace, the per-tensor quantiser)
    and the decoder fusions, captured together; every replay against the eager result."""
    from paper_2602_15563_amd import kmq
    dev = gpu.dev
    N1, K1 = 3072, 3072                         # fused RMSNorm + residual on a 1-bit table kernel
    idx1, cb1 = synth.make_indices(11, 0, N1, K1, 1), synth.make_codebook(11, 0, N1, 1, symmetric=True)
    x1, g1, r1 = synth.make_x(11, 0, 1, K1), synth.make_norm_weight(11, 0, K1), synth.make_residual(11, 0, N1)
    N2, K2, b2, M2 = 6, 40000, 3, 2             # split-K: partial sums in the workspace, second kernel adds them
    idx2, cb2, X2 = synth.make_indices(12, 0, N2, K2, b2), synth.make_codebook(12, 0, N2, b2), synth.make_x(12, 0, M2, K2)
    N3, K3, b3 = 64, 1024, 2                    # the quantiser in the paper's format: 2 * rounds + 3 kernels
    Wd3 = synth.make_dense_weights(13, 0, N3, K3)
    W1, C1, Xd1, G1, R1 = dev(kmq.pack(idx1, 1)), dev(cb1), dev(x1), dev(g1), dev(r1)
    W2, C2, Xd2 = dev(kmq.pack(idx2, b2)), dev(cb2), dev(X2)
    ws2 = torch.empty(kmq.workspace_bytes(N2, K2, b2, M2), dtype=torch.uint8, device="cuda")
    assert ws2.numel() > 0
    D3 = dev(Wd3)
    ws3 = torch.empty(kmq.quantize_blockscaled_workspace_bytes(), dtype=torch.uint8, device="cuda")

    def outputs():
        return (torch.full((N1,), 0x7FC1, dtype=torch.int16, device="cuda"),
                torch.full((N1,), 0x7FC1, dtype=torch.int16, device="cuda"),
                torch.full((M2, N2), 0x7FC1, dtype=torch.int16, device="cuda"),
                torch.full((N3, K3 * b3 // 32), -1, dtype=torch.int32, device="cuda"),
                torch.full((1 << b3,), 0x7FC1, dtype=torch.int16, device="cuda"),
                torch.full((N3, K3 // 64), 0x7FC1, dtype=torch.int16, device="cuda"))

    def run(Y):
        kmq.gemv_fused(W1, C1, Xd1, Y[0], N1, K1, 1, norm_weight=G1, eps=1e-5, residual=R1)
        kmq.gemv_swiglu_rmsnorm(W1, C1, W1, C1, Xd1, G1, 1e-5, Y[1], N1, K1, 1)
        kmq.gemm_smallbatch(W2, C2, Xd2, Y[2], N2, K2, M2, b2, 0, ws2)
        kmq.quantize_blockscaled(D3, N3, K3, b3, 5, Y[3], Y[4], Y[5], ws3)

    eager = outputs()
    run(eager)
    torch.cuda.synchronize()
    want = [y.clone() for y in eager]
    captured = outputs()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        run(captured)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            run(captured)
    for replay in range(3):
        for y in captured:
            y.fill_(0x7FC1 if y.dtype == torch.int16 else -1)
        ws2.fill_(0xFF)                        # the workspaces carry nothing from one call to the next
        ws3.fill_(0xFF)
        run(eager)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (y, w) in enumerate(zip(captured, want)):
            assert torch.equal(y, w), f"replay {replay}, output {i}"


def test_graph_replays_of_the_rowlane_and_kslice_calls(gpu):
    """The lane-per-row kernels (batch 1, a batch of seven = two launches, the round loop, the fused pair), the
    matrix-core kernel with register-resident activations, the call that allocates nothing and the canonical
    layout's kernel that walks K in rounds, captured together; every replay against the eager result."""
    from paper_2602_15563_amd import kmq
    dev = gpu.dev
    RL, T = kmq.LAYOUT_ROWLANE, kmq.LAYOUT_TILED
    g = np.random.default_rng(77)

    def case(N, K, bits, M):
        idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        cb = synth.f32_to_bf16(g.normal(0, 0.02, size=(N, 1 << bits)).astype(np.float32))
        X = synth.f32_to_bf16(g.standard_normal(size=(M, K)).astype(np.float32))
        return kmq.pack(idx, bits), cb, X

    p1, c1, x1 = case(330, 4096, 2, 1)                 # rowlane_b2
    p2, c2, x2 = case(100, 3072, 1, 7)                 # rowlane_b1, 4 + 3 columns
    p3, c3, x3 = case(50, 256 * 19, 2, 2)              # rowlane_loop_b2
    p4, c4, x4 = case(64, 2048, 2, 1)                  # rowlane_pair_b2 (gate = up weights differ below)
    p4u, c4u, _ = case(64, 2048, 2, 1)
    p5, c5, x5 = case(6144 + 3, 3072, 3, 8)            # mfma_kslice_b3
    p6, c6, x6 = case(40, 32768, 2, 2)                 # split over K: the static scratch of the no-allocation call
    p7, c7, x7 = case(1001, 2848, 3, 3)                # lut_loop_b3: rounds over K, a row that ends inside a round, batch as grid rows
    assert kmq.kernel_name(6147, 3072, 3, 8, T) == "mfma_kslice_b3" and kmq.kernel_name(40, 32768, 2, 2) == "generic_splitk"
    assert kmq.kernel_name(1001, 2848, 3, 3) == "lut_loop_b3"
    W1, W2, W3 = dev(kmq.repack(p1, 4096, 2, RL)), dev(kmq.repack(p2, 3072, 1, RL)), dev(kmq.repack(p3, 256 * 19, 2, RL))
    W4, W4u = dev(kmq.repack(p4, 2048, 2, RL)), dev(kmq.repack(p4u, 2048, 2, RL))
    W5, W6, W7 = dev(kmq.repack(p5, 3072, 3, T)), dev(p6), dev(p7)
    C = [dev(c) for c in (c1, c2, c3, c4, c4u, c5, c6, c7)]
    Xd = [dev(x) for x in (x1, x2, x3, x4, x5, x6, x7)]

    def outputs():
        shapes = ((1, 330), (7, 100), (2, 50), (1, 64), (8, 6147), (2, 40), (3, 1001))
        return [torch.full(s, 0x7FC1, dtype=torch.int16, device="cuda") for s in shapes]

    def run(Y):
        kmq.gemv(W1, C[0], Xd[0], Y[0], 330, 4096, 2, RL)
        kmq.gemm_smallbatch(W2, C[1], Xd[1], Y[1], 100, 3072, 7, 1, RL)
        kmq.gemm_smallbatch(W3, C[2], Xd[2], Y[2], 50, 256 * 19, 2, 2, RL)
        kmq.gemv_swiglu(W4, C[3], W4u, C[4], Xd[3], Y[3], 64, 2048, 2, RL)
        kmq.gemm_smallbatch(W5, C[5], Xd[4], Y[4], 6147, 3072, 8, 3, T)
        kmq.gemm_smallbatch_noalloc(W6, C[6], Xd[5], Y[5], 40, 32768, 2, 2, 0)
        kmq.gemm_smallbatch(W7, C[7], Xd[6], Y[6], 1001, 2848, 3, 3, 0)

    eager = outputs()
    run(eager)
    torch.cuda.synchronize()
    want = [y.clone() for y in eager]
    captured = outputs()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        run(captured)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            run(captured)
    for replay in range(4):
        for y in captured:
            y.fill_(0x7FC1)
        run(eager)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (y, w) in enumerate(zip(captured, want)):
            assert torch.equal(y, w), f"replay {replay}, call {i}"
