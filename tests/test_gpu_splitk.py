"""Split-K over workgroups (few rows, long rows): partial sums in the caller's workspace, added in a
fixed order by a second kernel, so the result is deterministic.  Parity against the oracle through
the C ABI, the workspace contract and the shapes on both sides of the heuristic's threshold."""
import numpy as np
import pytest

import oracle
from paper_2602_15563_amd import kmq, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    return gpu_util


CASES = [  # N, K, bits, M
    (3, 65536, 2, 1),
    (5, 40000, 3, 4),          # K not a multiple of 32: ragged last group in the last slice
    (17, 3 * 8192 + 7, 1, 16),
    (40, 100000, 4, 8),
    (128, 16384, 2, 2),        # threshold case: two slices over 32 workgroups
    (1, 262144, 3, 1),
]


def slices_expected(N, K):
    wgs = (N + 3) // 4
    if wgs * 2 > 256 or K < 16384:
        return 1
    s = min(256 // wgs, K // 4096, 64)
    return s if s >= 2 else 1


@pytest.mark.parametrize("N,K,bits,M", CASES)
def test_splitk_matches_oracle(gpu, N, K, bits, M):
    seed = 4100 + N
    idx = synth.make_indices(seed, 0, N, K, bits)
    cb = synth.make_codebook(seed, 0, N, bits)
    X = synth.make_x(seed, 0, M, K)
    packed = oracle.pack(idx, bits)
    s = slices_expected(N, K)
    assert s > 1
    assert kmq.kernel_name(N, K, bits, M) == "generic_splitk"
    assert kmq.workspace_bytes(N, K, bits, M) == s * M * N * 4
    Wd, cbd = gpu.dev(packed), gpu.dev(cb)
    print(f"split-K N={N} K={K} b={bits} M={M} slices={s}", flush=True)
    Y1 = gpu.run_gemm(Wd, cbd, X, N, K, bits)
    worst = gpu.check_against_oracle(Y1, packed, cb, X, K, bits, label=f"splitk {N}x{K} b{bits} m{M}")
    assert worst <= 2e-3
    Y2 = gpu.run_gemm(Wd, cbd, X, N, K, bits)
    assert np.array_equal(Y1, Y2)           # fixed summation order: bit-identical on every call


def test_splitk_needs_workspace(gpu):
    import torch
    dev = gpu.dev
    N, K, bits = 4, 32768, 2
    idx = synth.make_indices(7, 0, N, K, bits)
    Wd, cbd = dev(oracle.pack(idx, bits)), dev(synth.make_codebook(7, 0, N, bits))
    xd = dev(synth.make_x(7, 0, 1, K))
    y = torch.zeros(N, dtype=torch.int16, device="cuda")
    need = kmq.workspace_bytes(N, K, bits, 1)
    assert need > 0
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv(Wd, cbd, xd, y, N, K, bits)
    assert e.value.status == 6
    small = torch.empty(need - 4, dtype=torch.uint8, device="cuda")
    with pytest.raises(kmq.KmqError) as e:
        kmq.gemv(Wd, cbd, xd, y, N, K, bits, 0, small)
    assert e.value.status == 6
    torch.cuda.synchronize()
    assert not y.any().item()               # nothing was launched


@pytest.mark.parametrize("N,K,M", [(600, 16384, 2), (8, 4100, 2), (128, 8192, 2)])
def test_no_split_beyond_threshold(gpu, N, K, M):
    """Enough rows to fill the chip, or short rows: single pass, no workspace."""
    if slices_expected(N, K) == 1:
        name = kmq.kernel_name(N, K, 2, M)
        assert kmq.workspace_bytes(N, K, 2, M) == 0 and (name == "generic" or name.startswith("lut_b2") or name == "lut_loop_b2"), name
    idx = synth.make_indices(9, 0, N, K, 2)
    cb = synth.make_codebook(9, 0, N, 2)
    X = synth.make_x(9, 0, M, K)
    packed = oracle.pack(idx, 2)
    Y = gpu.run_gemm(gpu.dev(packed), gpu.dev(cb), X, N, K, 2)
    gpu.check_against_oracle(Y, packed, cb, X, K, 2, label=f"nosplit {N}x{K}")
