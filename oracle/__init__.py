"""CPU oracle for the k-means-quantised matrix product -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg may import this package.  It wraps ``kmq_oracle.cpp`` (plain C++, fp64,
single-threaded) with numpy marshalling and nothing else; it never touches the
GPU library and shares no code with it.

The operation is the fused dequantise-multiply of the paper's App. E
("Kernel implementations"), with per-output-row codebooks and no block scales
(``gemm``), and in the paper's own format, a tensor-wide codebook with one bf16
scale per block of 64 elements along K (``gemm_blockscaled``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "kmq_oracle.cpp"), os.path.join(_HERE, "kmq_quantize_oracle.cpp")]
_LIB = os.path.join(_HERE, "libkmq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no GPU involved)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB] + _SRCS
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, ci, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_words_per_row.restype = i64
        lib.oracle_words_per_row.argtypes = [ci, i64]
        lib.oracle_pack.restype = ci
        lib.oracle_pack.argtypes = [vp, i64, i64, ci, vp]
        lib.oracle_unpack.restype = ci
        lib.oracle_unpack.argtypes = [vp, i64, i64, ci, vp]
        lib.oracle_dequant.restype = ci
        lib.oracle_dequant.argtypes = [vp, vp, i64, i64, ci, vp]
        lib.oracle_round_bf16.restype = ctypes.c_uint16
        lib.oracle_round_bf16.argtypes = [ctypes.c_double]
        lib.oracle_gemm.restype = ci
        lib.oracle_gemm.argtypes = [vp, vp, vp, i64, i64, ci, i64, i64, i64, vp, vp, vp]
        lib.oracle_gemm_blockscaled.restype = ci
        lib.oracle_gemm_blockscaled.argtypes = [vp, vp, vp, vp, i64, i64, ci, i64, i64, i64, i64, ci, vp, vp, vp]
        lib.oracle_swiglu.restype = ci
        lib.oracle_swiglu.argtypes = [vp, vp, i64, vp]
        lib.oracle_gemm_dense.restype = ci
        lib.oracle_gemm_dense.argtypes = [vp, vp, i64, i64, i64, i64, i64, vp, vp, vp]
        lib.oracle_dequant_blockscaled.restype = ci
        lib.oracle_dequant_blockscaled.argtypes = [vp, vp, vp, i64, i64, ci, i64, vp]
        lib.oracle_rmsnorm.restype = ci
        lib.oracle_rmsnorm.argtypes = [vp, vp, i64, ctypes.c_double, vp, vp]
        lib.oracle_quantize_round_bf16.restype = ctypes.c_uint16
        lib.oracle_quantize_round_bf16.argtypes = [ctypes.c_double]
        lib.oracle_lloyd.restype = ci
        lib.oracle_lloyd.argtypes = [vp, i64, vp, ci, ci]
        lib.oracle_quantize_rows.restype = ci
        lib.oracle_quantize_rows.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp]
        lib.oracle_quantize_blockscaled.restype = ci
        lib.oracle_quantize_blockscaled.argtypes = [vp, i64, i64, ci, i64, ci, vp, vp, vp, vp, vp]
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _arr(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def words_per_row(bits: int, K: int) -> int:
    r = _load().oracle_words_per_row(bits, K)
    if r < 0:
        raise ValueError("bad bits or K")
    return int(r)


def pack(idx: np.ndarray, bits: int) -> np.ndarray:
    """uint8 idx[N][K] -> uint32 packed[N][ceil(K*bits/32)]."""
    idx = _arr(idx, np.uint8)
    N, K = idx.shape
    out = np.empty((N, words_per_row(bits, K)), dtype=np.uint32)
    rc = _load().oracle_pack(_p(idx), N, K, bits, _p(out))
    if rc == 2:
        raise ValueError("index out of range for this bit-width")
    if rc:
        raise ValueError("bad argument")
    return out


def unpack(packed: np.ndarray, K: int, bits: int) -> np.ndarray:
    N = packed.shape[0]
    packed = _arr(packed, np.uint32, (N, words_per_row(bits, K)))
    out = np.empty((N, K), dtype=np.uint8)
    if _load().oracle_unpack(_p(packed), N, K, bits, _p(out)):
        raise ValueError("bad argument")
    return out


def dequant(packed: np.ndarray, codebook: np.ndarray, K: int, bits: int) -> np.ndarray:
    """bf16 bit patterns (uint16) of the dequantised weights, N x K."""
    N = packed.shape[0]
    packed = _arr(packed, np.uint32, (N, words_per_row(bits, K)))
    codebook = _arr(codebook, np.uint16, (N, 1 << bits))
    out = np.empty((N, K), dtype=np.uint16)
    if _load().oracle_dequant(_p(packed), _p(codebook), N, K, bits, _p(out)):
        raise ValueError("bad argument")
    return out


def round_bf16(y: float) -> int:
    return int(_load().oracle_round_bf16(float(y)))


def gemm(packed: np.ndarray, codebook: np.ndarray, X: np.ndarray, K: int, bits: int,
         rows: tuple[int, int] | None = None):
    """Y = X W^T in fp64.  X: uint16 bf16 patterns, shape (M, K) or (K,).

    Returns (Y, A, Ybf16), each M x N (or N for a vector X); with ``rows=(n0, n1)``
    only those output columns are computed and the rest are NaN / 0.
    """
    N = packed.shape[0]
    packed = _arr(packed, np.uint32, (N, words_per_row(bits, K)))
    codebook = _arr(codebook, np.uint16, (N, 1 << bits))
    X = np.ascontiguousarray(X, dtype=np.uint16)
    vec = X.ndim == 1
    X2 = X.reshape(1, -1) if vec else X
    M = X2.shape[0]
    if X2.shape[1] != K:
        raise ValueError("X has the wrong K")
    n0, n1 = (0, N) if rows is None else rows
    Y = np.full((M, N), np.nan, dtype=np.float64)
    A = np.full((M, N), np.nan, dtype=np.float64)
    Yb = np.zeros((M, N), dtype=np.uint16)
    if _load().oracle_gemm(_p(packed), _p(codebook), _p(X2), N, K, bits, M, n0, n1,
                           _p(Y), _p(A), _p(Yb)):
        raise ValueError("bad argument")
    if vec:
        return Y[0], A[0], Yb[0]
    return Y, A, Yb


def gemm_blockscaled(packed: np.ndarray, codebook: np.ndarray, scales: np.ndarray, X: np.ndarray,
                     K: int, bits: int, block: int = 64, rows: tuple[int, int] | None = None,
                     deferred: bool = False):
    """Y = X W^T with w[n][k] = codebook[idx[n][k]] * scales[n][k // block], fp64.

    codebook: uint16 bf16 patterns, shape (2^bits,), shared by all rows; scales:
    uint16 bf16 patterns, shape (N, K // block).  Returns (Y, A, Ybf16) as ``gemm``.
    """
    N = packed.shape[0]
    packed = _arr(packed, np.uint32, (N, words_per_row(bits, K)))
    codebook = _arr(codebook, np.uint16, (1 << bits,))
    if K % block:
        raise ValueError("K must be a multiple of the block size")
    scales = _arr(scales, np.uint16, (N, K // block))
    X = np.ascontiguousarray(X, dtype=np.uint16)
    vec = X.ndim == 1
    X2 = X.reshape(1, -1) if vec else X
    M = X2.shape[0]
    if X2.shape[1] != K:
        raise ValueError("X has the wrong K")
    n0, n1 = (0, N) if rows is None else rows
    Y = np.full((M, N), np.nan, dtype=np.float64)
    A = np.full((M, N), np.nan, dtype=np.float64)
    Yb = np.zeros((M, N), dtype=np.uint16)
    if _load().oracle_gemm_blockscaled(_p(packed), _p(codebook), _p(scales), _p(X2), N, K, bits, block, M,
                                       n0, n1, int(deferred), _p(Y), _p(A), _p(Yb)):
        raise ValueError("bad argument")
    if vec:
        return Y[0], A[0], Yb[0]
    return Y, A, Yb


def gemm_dense(W: np.ndarray, X: np.ndarray, rows: tuple[int, int] | None = None):
    """Y = X W^T for a dense bf16 W (uint16 patterns, N x K), fp64: the unquantised baseline."""
    W = np.ascontiguousarray(W, dtype=np.uint16)
    N, K = W.shape
    X = np.ascontiguousarray(X, dtype=np.uint16)
    vec = X.ndim == 1
    X2 = X.reshape(1, -1) if vec else X
    M = X2.shape[0]
    if X2.shape[1] != K:
        raise ValueError("X has the wrong K")
    n0, n1 = (0, N) if rows is None else rows
    Y = np.full((M, N), np.nan, dtype=np.float64)
    A = np.full((M, N), np.nan, dtype=np.float64)
    Yb = np.zeros((M, N), dtype=np.uint16)
    if _load().oracle_gemm_dense(_p(W), _p(X2), N, K, M, n0, n1, _p(Y), _p(A), _p(Yb)):
        raise ValueError("bad argument")
    if vec:
        return Y[0], A[0], Yb[0]
    return Y, A, Yb


def swiglu(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    """silu(gate) * up element-wise on fp64 arrays (the fused call's definition)."""
    g = np.ascontiguousarray(gate, dtype=np.float64)
    u = np.ascontiguousarray(up, dtype=np.float64)
    if g.shape != u.shape:
        raise ValueError("shapes differ")
    y = np.empty_like(g)
    if _load().oracle_swiglu(_p(g), _p(u), g.size, _p(y)):
        raise ValueError("bad argument")
    return y


def dequant_blockscaled(packed, codebook, scales, K: int, bits: int, block: int = 64) -> np.ndarray:
    """Dense bf16 weights (uint16 patterns, N x K) of the block-scaled format: bf16(codebook[idx] * scale)."""
    packed = _arr(packed, np.uint32)
    N = packed.shape[0]
    codebook = _arr(codebook, np.uint16, (1 << bits,))
    scales = _arr(scales, np.uint16, (N, K // block))
    Wd = np.empty((N, K), np.uint16)
    if _load().oracle_dequant_blockscaled(_p(packed), _p(codebook), _p(scales), N, K, bits, block, _p(Wd)):
        raise ValueError("oracle_dequant_blockscaled: bad arguments")
    return Wd


def rmsnorm(x, g, eps: float):
    """(xn, r): r = 1 / sqrt(mean(x^2) + eps) in fp64 and the normalised activations
    xn = bf16(x * r * g) as uint16 patterns (one rounding of the fp64 value)."""
    x = _arr(x, np.uint16).reshape(-1)
    g = np.full(x.shape, 0x3F80, np.uint16) if g is None else _arr(g, np.uint16, x.shape)   # None: unit gains
    xn = np.empty_like(x)
    r = np.empty(1, np.float64)
    if _load().oracle_rmsnorm(_p(x), _p(g), x.size, float(eps), _p(xn), _p(r)):
        raise ValueError("oracle_rmsnorm: bad arguments")
    return xn, float(r[0])


_rmsnorm = rmsnorm     # gemv_fused has a parameter of that name


def gemv_fused(packed, codebook, x, K: int, bits: int, norm_weight=None, eps: float = 0.0, residual=None, rows=None,
               rmsnorm=None):
    """The fused decoder call's definition, composed from the pieces above:
    Y[n] = residual[n] + sum_k w[n][k] xn[k] with xn = rmsnorm(x) (bf16); returns (Y, A) with
    A = |residual| + sum |w xn|.
    rmsnorm defaults to "gains were given"; rmsnorm=True without gains normalises with unit gains."""
    x = _arr(x, np.uint16).reshape(1, -1)
    if rmsnorm is None:
        rmsnorm = norm_weight is not None
    if rmsnorm:
        xn, _ = _rmsnorm(x[0], norm_weight, eps)
        x = xn.reshape(1, -1)
    Y, A, _ = gemm(packed, codebook, x, K, bits, rows=rows)
    Y, A = Y[0], A[0]
    if residual is not None:
        res = (np.ascontiguousarray(residual, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        Y, A = Y + res, A + np.abs(res)
    return Y, A


# ---- the quantiser that produces the formats (kmq_quantize_oracle.cpp) ----

def quantize_round_bf16(c: float) -> int:
    return int(_load().oracle_quantize_round_bf16(float(c)))


def lloyd(v, c0, iters: int) -> np.ndarray:
    """`iters` rounds of 1-D Lloyd on values v from sorted start centroids c0; returns the centroids (fp64)."""
    v = _arr(v, np.float64)
    c = np.array(c0, dtype=np.float64, copy=True)
    if _load().oracle_lloyd(_p(v), v.size, _p(c), c.size, iters):
        raise ValueError("oracle_lloyd: bad arguments")
    return c


def quantize_rows(W, bits: int, iters: int):
    """Per-row k-means of dense bf16 weights (uint16 bit patterns, N x K).
    Returns (idx uint8 N x K, codebook uint16 N x 2^bits, centroid fp64 N x 2^bits, sse fp64 N)."""
    W = _arr(W, np.uint16)
    N, K = W.shape
    C = 1 << bits
    idx = np.empty((N, K), np.uint8)
    cb = np.empty((N, C), np.uint16)
    cen = np.empty((N, C), np.float64)
    sse = np.empty(N, np.float64)
    if _load().oracle_quantize_rows(_p(W), N, K, bits, iters, _p(idx), _p(cb), _p(cen), _p(sse)):
        raise ValueError("oracle_quantize_rows: bad arguments")
    return idx, cb, cen, sse


def quantize_blockscaled(W, bits: int, iters: int, block: int = 64):
    """The paper's format from dense bf16 weights: absmax scale per block, tensor-wide k-means on the
    normalised weights.  Returns (idx uint8 N x K, codebook uint16 2^bits, scales uint16 N x K/block,
    centroid fp64 2^bits, vnorm fp64 N x K)."""
    W = _arr(W, np.uint16)
    N, K = W.shape
    C = 1 << bits
    idx = np.empty((N, K), np.uint8)
    cb = np.empty(C, np.uint16)
    sc = np.empty((N, K // block), np.uint16)
    cen = np.empty(C, np.float64)
    vn = np.empty((N, K), np.float64)
    if _load().oracle_quantize_blockscaled(_p(W), N, K, bits, block, iters, _p(idx), _p(cb), _p(sc), _p(cen), _p(vn)):
        raise ValueError("oracle_quantize_blockscaled: bad arguments")
    return idx, cb, sc, cen, vn
