"""The entry point for callers that cannot allocate (kmq_gemm_smallbatch_noalloc): split-K partial sums
in the library's own per-GPU scratch array instead of a workspace argument.  Called through the C ABI
and compared bit for bit with kmq_gemm_smallbatch on a caller's workspace -- same kernels, same fixed
summation order -- on two calls in a row, the second with a smaller input, and with the oracle.
The file name sorts after every other test file, so it is collected last."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_15563_amd import kmq, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from tests import gpu_util
    return gpu_util


def _both(gpu, N, K, bits, M, seed):
    idx = synth.make_indices(seed, 0, N, K, bits)
    cb = synth.make_codebook(seed, 0, N, bits)
    X = synth.make_x(seed, 0, M, K)
    packed = oracle.pack(idx, bits)
    Wd, cbd, Xd = gpu.dev(packed), gpu.dev(cb), gpu.dev(X)
    need = kmq.workspace_bytes(N, K, bits, M)
    print(f"no-alloc N={N} K={K} b={bits} M={M} workspace={need} kernel={kmq.kernel_name(N, K, bits, M)}", flush=True)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
    Y_ws = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")
    Y_na = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")
    lib = kmq.raw()
    st = torch.cuda.current_stream().cuda_stream
    rc = lib.kmq_gemm_smallbatch(Wd.data_ptr(), cbd.data_ptr(), Xd.data_ptr(), Y_ws.data_ptr(), N, K, M, bits, 0,
                                 ws.data_ptr() if need else None, need, st)
    assert rc == 0, kmq.status_string(rc)
    rc = lib.kmq_gemm_smallbatch_noalloc(Wd.data_ptr(), cbd.data_ptr(), Xd.data_ptr(), Y_na.data_ptr(), N, K, M, bits, 0, st)
    assert rc == 0, kmq.status_string(rc)
    torch.cuda.synchronize()
    a, b = gpu.host_u16(Y_ws), gpu.host_u16(Y_na)
    assert np.array_equal(a, b), "no-alloc entry point differs from the workspace entry point"
    gpu.check_against_oracle(b, packed, cb, X, K, bits, label=f"noalloc {N}x{K} b{bits} m{M}")
    return need


def test_two_calls_in_a_row_the_second_smaller(gpu):
    assert _both(gpu, 64, 32768, 3, 4, 9100) > 0          # split-K: 8 slices, 8 KiB of partial sums
    assert _both(gpu, 16, 16384, 2, 2, 9101) > 0          # smaller: 4 slices over the same array
    assert _both(gpu, 5, 40000, 1, 16, 9102) > 0          # ragged K, widest batch
    assert _both(gpu, 512, 16384, 4, 16, 9103) == kmq.NOALLOC_SCRATCH_BYTES     # the largest workspace the split asks for
    assert _both(gpu, 300, 4096, 2, 3, 9104) == 0         # a problem without workspace takes the ordinary path


def test_argument_errors_and_the_size_limit(gpu):
    lib = kmq.raw()
    z = torch.zeros(4096, dtype=torch.int32, device="cuda")
    p = z.data_ptr()
    assert lib.kmq_gemm_smallbatch_noalloc(None, p, p, p, 4, 64, 1, 2, 0, None) == 1
    assert lib.kmq_gemm_smallbatch_noalloc(p, p, p, p, 4, 64, 1, 7, 0, None) == 2
    assert lib.kmq_gemm_smallbatch_noalloc(p, p, p, p, 4, 64, 17, 2, 0, None) == 3
    assert lib.kmq_gemm_smallbatch_noalloc(p, p, p, p, 4, 64, 1, 2, 9, None) == 7
    assert lib.kmq_gemm_smallbatch_noalloc(p + 4, p, p, p, 4, 64, 1, 2, 0, None) == 4
    # no shape the split currently serves needs more than the array holds
    for N in (1, 4, 100, 256, 300, 508, 512):
        for K in (16384, 65536, 1 << 22):
            assert kmq.workspace_bytes(N, K, 2, 16) <= kmq.NOALLOC_SCRATCH_BYTES
