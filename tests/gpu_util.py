"""Helpers shared by the GPU parity tests: move numpy buffers to the device,
call the C ABI through the binding, compare with the oracle's fp64 result."""
import numpy as np
import torch

import oracle
from paper_2602_15563_amd import kmq, synth

# every acceptance bound lives in one module, shared with bench.py
from paper_2602_15563_amd.tolerance import TOL, arithmetic_bound, rmsnorm_commute_bound, swiglu_bound, swiglu_contract_bound  # noqa: E402,F401


def dev(a: np.ndarray) -> torch.Tensor:
    """numpy uint32/uint16/uint8 -> device tensor with the same bytes."""
    a = np.ascontiguousarray(a)
    view = {np.dtype(np.uint32): np.int32, np.dtype(np.uint16): np.int16, np.dtype(np.uint8): np.uint8}[a.dtype]
    return torch.from_numpy(a.view(view)).cuda()


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


def run_gemm(packed_dev, cb_dev, X: np.ndarray, N, K, bits, layout=0, use_gemv=None):
    """Run the product on the GPU; returns uint16 bf16 patterns, shape (M, N)."""
    X2 = X.reshape(1, -1) if X.ndim == 1 else X
    M = X2.shape[0]
    Xd = dev(X2)
    Y = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")   # NaN pattern: must be overwritten
    ws_bytes = kmq.workspace_bytes(N, K, bits, M, layout)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device="cuda") if ws_bytes else None
    if use_gemv is None:
        use_gemv = M == 1
    if use_gemv:
        kmq.gemv(packed_dev, cb_dev, Xd, Y, N, K, bits, layout, ws)
    else:
        kmq.gemm_smallbatch(packed_dev, cb_dev, Xd, Y, N, K, M, bits, layout, ws)
    torch.cuda.synchronize()
    return host_u16(Y)


def check_against_oracle(Yg_u16, packed, cb, X, K, bits, row_ranges=None, label="", strict=None):
    """Element-by-element comparison on the given row ranges (default: all rows).
    strict: also assert the contract's |err| <= 2e-3*A (default: when K >= 512)."""
    if strict is None:
        strict = K >= 512
    N = packed.shape[0]
    X2 = X.reshape(1, -1) if X.ndim == 1 else X
    ranges = row_ranges or [(0, N)]
    worst = 0.0
    for n0, n1 in ranges:
        Y, A, _ = oracle.gemm(packed, cb, X2, K, bits, rows=(n0, n1))
        yg = synth.bf16_to_f64(Yg_u16[:, n0:n1])
        err = np.abs(yg - Y[:, n0:n1])
        a = A[:, n0:n1]
        bad = err > arithmetic_bound(a, Y[:, n0:n1], K)
        if strict:
            bad |= err > TOL * a
        assert not bad.any(), (
            f"{label}: {int(bad.sum())} outputs beyond tolerance in rows [{n0},{n1}); "
            f"first at {np.argwhere(bad)[0]}, err={err[bad][0]:.3e}, A={a[bad][0]:.3e}")
        with np.errstate(divide="ignore", invalid="ignore"):
            r = np.where(a > 0, err / a, 0.0)
        worst = max(worst, float(r.max()) if r.size else 0.0)
    return worst


def sample_ranges(N, seed, block=64, nblocks=6):
    """First and last rows plus a few random blocks: covers both grid edges."""
    if N <= block * (nblocks + 2):
        return [(0, N)]
    g = np.random.default_rng(seed)
    starts = sorted(int(s) for s in g.integers(block, N - 2 * block, size=nblocks))
    return [(0, block)] + [(s, s + block) for s in starts] + [(N - block, N)]


def run_gemm_blockscaled(packed_dev, cb_dev, sc_dev, X: np.ndarray, N, K, bits, use_gemv=None):
    """Block-scaled product on the GPU; returns uint16 bf16 patterns, shape (M, N)."""
    X2 = X.reshape(1, -1) if X.ndim == 1 else X
    M = X2.shape[0]
    Xd = dev(X2)
    Y = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")
    if use_gemv is None:
        use_gemv = M == 1
    if use_gemv:
        kmq.gemv_blockscaled(packed_dev, cb_dev, sc_dev, Xd, Y, N, K, bits)
    else:
        kmq.gemm_smallbatch_blockscaled(packed_dev, cb_dev, sc_dev, Xd, Y, N, K, M, bits)
    torch.cuda.synchronize()
    return host_u16(Y)


def check_blockscaled_against_oracle(Yg_u16, packed, cb, sc, X, K, bits, row_ranges=None, label="", strict=None):
    """As check_against_oracle, for the block-scaled format.  The arithmetic bound counts
    one more rounding per block (the multiplication by the scale)."""
    if strict is None:
        strict = K >= 512
    N = packed.shape[0]
    X2 = X.reshape(1, -1) if X.ndim == 1 else X
    worst = 0.0
    for n0, n1 in (row_ranges or [(0, N)]):
        Y, A, _ = oracle.gemm_blockscaled(packed, cb, sc, X2, K, bits, rows=(n0, n1))
        yg = synth.bf16_to_f64(Yg_u16[:, n0:n1])
        err = np.abs(yg - Y[:, n0:n1])
        a = A[:, n0:n1]
        bad = err > arithmetic_bound(a, Y[:, n0:n1], K + 2 * (K // 64))
        if strict:
            bad |= err > TOL * a
        assert not bad.any(), (
            f"{label}: {int(bad.sum())} outputs beyond tolerance in rows [{n0},{n1}); "
            f"first at {np.argwhere(bad)[0]}, err={err[bad][0]:.3e}, A={a[bad][0]:.3e}")
        with np.errstate(divide="ignore", invalid="ignore"):
            r = np.where(a > 0, err / a, 0.0)
        worst = max(worst, float(r.max()) if r.size else 0.0)
    return worst
