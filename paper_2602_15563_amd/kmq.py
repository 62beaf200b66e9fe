"""Thin binding over the C-ABI library (include/kmq.h): argument marshalling
only.  Host functions take numpy arrays; device functions take torch tensors
that already live on the GPU and enqueue on torch's current stream.  There is
no fallback: if libkmq.so is missing, importing this module fails."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkmq.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2602_15563_amd.build`")


def _preload_torch_hip_runtime():
    """PyTorch's ROCm wheel bundles its own HIP runtime (same soname as the
    system one).  Streams and device pointers handed to libkmq.so come from
    that runtime, so it must be the one libkmq.so binds to: load it first, and
    the dynamic loader resolves libkmq.so's dependency to it by soname."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.submodule_search_locations:
        return
    cand = os.path.join(list(spec.submodule_search_locations)[0], "lib", "libamdhip64.so")
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


_preload_torch_hip_runtime()
_lib = ctypes.CDLL(LIB_PATH)

OK = 0
LAYOUT_CANONICAL, LAYOUT_TILED, LAYOUT_ROWLANE = 0, 1, 2
MAX_BATCH = 16

_i64, _int, _vp, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
_lib.kmq_words_per_row.restype = _i64
_lib.kmq_words_per_row.argtypes = [_int, _i64]
_lib.kmq_pack.restype = ctypes.c_int32
_lib.kmq_pack.argtypes = [_vp, _i64, _i64, _int, _vp]
_lib.kmq_unpack.restype = ctypes.c_int32
_lib.kmq_unpack.argtypes = [_vp, _i64, _i64, _int, _vp]
_lib.kmq_repack.restype = ctypes.c_int32
_lib.kmq_repack.argtypes = [_vp, _i64, _i64, _int, _int, _vp]
_lib.kmq_unrepack.restype = ctypes.c_int32
_lib.kmq_unrepack.argtypes = [_vp, _i64, _i64, _int, _int, _vp]
_lib.kmq_tiled_words.restype = _i64
_lib.kmq_tiled_words.argtypes = [_i64, _i64, _int, _int]
_lib.kmq_workspace_bytes.restype = _sz
_lib.kmq_workspace_bytes.argtypes = [_i64, _i64, _int, _int, _int]
_lib.kmq_gemv.restype = ctypes.c_int32
_lib.kmq_gemv.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _vp, _sz, _vp]
_lib.kmq_gemm_smallbatch.restype = ctypes.c_int32
_lib.kmq_gemm_smallbatch.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _int, _vp, _sz, _vp]
_lib.kmq_gemm_smallbatch_noalloc.restype = ctypes.c_int32
_lib.kmq_gemm_smallbatch_noalloc.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _int, _vp]
_lib.kmq_dequant.restype = ctypes.c_int32
_lib.kmq_dequant.argtypes = [_vp, _vp, _vp, _i64, _i64, _int, _int, _vp]
_lib.kmq_kernel_name.restype = ctypes.c_char_p
_lib.kmq_kernel_name.argtypes = [_i64, _i64, _int, _int, _int]
_lib.kmq_gemv_blockscaled.restype = ctypes.c_int32
_lib.kmq_gemv_blockscaled.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _vp, _sz, _vp]
_lib.kmq_gemm_smallbatch_blockscaled.restype = ctypes.c_int32
_lib.kmq_gemm_smallbatch_blockscaled.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _int, _vp, _sz, _vp]
_lib.kmq_kernel_name_blockscaled.restype = ctypes.c_char_p
_lib.kmq_kernel_name_blockscaled.argtypes = [_i64, _i64, _int, _int, _int]
_lib.kmq_gemv_swiglu.restype = ctypes.c_int32
_lib.kmq_gemv_swiglu.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _vp]
_lib.kmq_kernel_name_swiglu.restype = ctypes.c_char_p
_lib.kmq_kernel_name_swiglu.argtypes = [_i64, _i64, _int, _int]
_lib.kmq_gemv_bf16.restype = ctypes.c_int32
_lib.kmq_gemv_bf16.argtypes = [_vp, _vp, _vp, _i64, _i64, _vp]
_lib.kmq_dequant_blockscaled.restype = ctypes.c_int32
_lib.kmq_dequant_blockscaled.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _int, _vp]
_lib.kmq_gemv_fused.restype = ctypes.c_int32
_lib.kmq_gemv_fused.argtypes = [_vp, _vp, _vp, _int, _vp, ctypes.c_float, _vp, _vp, _i64, _i64, _int, _int, _vp]
_lib.kmq_gemv_swiglu_rmsnorm.restype = ctypes.c_int32
_lib.kmq_gemv_swiglu_rmsnorm.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _i64, _i64, _int, _int, _vp]
_lib.kmq_kernel_name_fused.restype = ctypes.c_char_p
_lib.kmq_kernel_name_fused.argtypes = [_i64, _i64, _int, _int, _int]
_lib.kmq_quantize_rows.restype = ctypes.c_int32
_lib.kmq_quantize_rows.argtypes = [_vp, _i64, _i64, _int, _int, _vp, _vp, _vp]
_lib.kmq_quantize_blockscaled_workspace_bytes.restype = _sz
_lib.kmq_quantize_blockscaled_workspace_bytes.argtypes = []
_lib.kmq_quantize_blockscaled.restype = ctypes.c_int32
_lib.kmq_quantize_blockscaled.argtypes = [_vp, _i64, _i64, _int, _int, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.kmq_last_hip_error.restype = ctypes.c_char_p
_lib.kmq_last_hip_error.argtypes = []
_lib.kmq_status_string.restype = ctypes.c_char_p
_lib.kmq_status_string.argtypes = [ctypes.c_int32]


class KmqError(RuntimeError):
    def __init__(self, status: int):
        self.status = int(status)
        detail = f" ({_lib.kmq_last_hip_error().decode()})" if self.status == 8 else ""
        super().__init__(f"kmq status {status}: {status_string(status)}{detail}")


def raw():
    """The ctypes library object (for tests that call the C ABI directly)."""
    return _lib


def status_string(status: int) -> str:
    return _lib.kmq_status_string(int(status)).decode()


def _check(status: int):
    if status != OK:
        raise KmqError(status)


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _npp(a):
    return a.ctypes.data_as(_vp)


def words_per_row(bits: int, K: int) -> int:
    return int(_lib.kmq_words_per_row(bits, K))


def tiled_words(N: int, K: int, bits: int, layout: int) -> int:
    return int(_lib.kmq_tiled_words(N, K, bits, layout))


def pack(idx: np.ndarray, bits: int) -> np.ndarray:
    idx = _np(idx, np.uint8)
    N, K = idx.shape
    wpr = words_per_row(bits, K)
    if wpr < 0:
        raise KmqError(2 if not 1 <= bits <= 4 else 3)
    out = np.empty((N, wpr), dtype=np.uint32)
    _check(_lib.kmq_pack(_npp(idx), N, K, bits, _npp(out)))
    return out


def unpack(packed: np.ndarray, K: int, bits: int) -> np.ndarray:
    packed = _np(packed, np.uint32)
    N = packed.shape[0]
    out = np.empty((N, K), dtype=np.uint8)
    _check(_lib.kmq_unpack(_npp(packed), N, K, bits, _npp(out)))
    return out


def repack(canonical: np.ndarray, K: int, bits: int, layout: int) -> np.ndarray:
    canonical = _np(canonical, np.uint32)
    N = canonical.shape[0]
    n = tiled_words(N, K, bits, layout)
    if n < 0:
        raise KmqError(7)
    out = np.empty(n, dtype=np.uint32)
    _check(_lib.kmq_repack(_npp(canonical), N, K, bits, layout, _npp(out)))
    return out


def unrepack(tiled: np.ndarray, N: int, K: int, bits: int, layout: int) -> np.ndarray:
    tiled = _np(tiled, np.uint32)
    out = np.empty((N, words_per_row(bits, K)), dtype=np.uint32)
    _check(_lib.kmq_unrepack(_npp(tiled), N, K, bits, layout, _npp(out)))
    return out


def workspace_bytes(N: int, K: int, bits: int, M: int, layout: int = 0) -> int:
    return int(_lib.kmq_workspace_bytes(N, K, bits, M, layout))


def kernel_name(N: int, K: int, bits: int, M: int, layout: int = 0) -> str:
    return _lib.kmq_kernel_name(N, K, bits, M, layout).decode()


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def gemv(W, codebook, x, y, N: int, K: int, bits: int, layout: int = 0, workspace=None):
    """y[N] = W x on torch's current stream.  All tensors are device tensors
    (W int32/uint32 words, codebook/x/y int16 or bfloat16 storage)."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.kmq_gemv(_ptr(W), _ptr(codebook), _ptr(x), _ptr(y), N, K, bits, layout,
                         _ptr(workspace), ws_bytes, _stream()))


def gemm_smallbatch(W, codebook, X, Y, N: int, K: int, M: int, bits: int, layout: int = 0, workspace=None):
    """Y[M][N] = X[M][K] W^T on torch's current stream."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.kmq_gemm_smallbatch(_ptr(W), _ptr(codebook), _ptr(X), _ptr(Y), N, K, M, bits, layout,
                                    _ptr(workspace), ws_bytes, _stream()))


NOALLOC_SCRATCH_BYTES = 65536


def gemm_smallbatch_noalloc(W, codebook, X, Y, N: int, K: int, M: int, bits: int, layout: int = 0):
    """gemm_smallbatch without a workspace argument: split-K partial sums go to the library's own per-GPU array."""
    _check(_lib.kmq_gemm_smallbatch_noalloc(_ptr(W), _ptr(codebook), _ptr(X), _ptr(Y), N, K, M, bits, layout, _stream()))


def kernel_name_blockscaled(N: int, K: int, bits: int, M: int, layout: int = 0) -> str:
    return _lib.kmq_kernel_name_blockscaled(N, K, bits, M, layout).decode()


def gemv_blockscaled(W, codebook, scales, x, y, N: int, K: int, bits: int, layout: int = 0, workspace=None):
    """y[N] = W x in the block-scaled format (codebook: 2^bits shared centroids, scales: N x K/64),
    on torch's current stream."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.kmq_gemv_blockscaled(_ptr(W), _ptr(codebook), _ptr(scales), _ptr(x), _ptr(y), N, K, bits, layout,
                                     _ptr(workspace), ws_bytes, _stream()))


def gemm_smallbatch_blockscaled(W, codebook, scales, X, Y, N: int, K: int, M: int, bits: int, layout: int = 0,
                                workspace=None):
    """Y[M][N] = X[M][K] W^T in the block-scaled format, on torch's current stream."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.kmq_gemm_smallbatch_blockscaled(_ptr(W), _ptr(codebook), _ptr(scales), _ptr(X), _ptr(Y), N, K, M,
                                                bits, layout, _ptr(workspace), ws_bytes, _stream()))


def kernel_name_swiglu(N: int, K: int, bits: int, layout: int = 0) -> str:
    return _lib.kmq_kernel_name_swiglu(N, K, bits, layout).decode()


def gemv_swiglu(Wgate, codebook_gate, Wup, codebook_up, x, y, N: int, K: int, bits: int, layout: int = 0):
    """y[N] = silu(Wgate x) * (Wup x) in one launch, on torch's current stream."""
    _check(_lib.kmq_gemv_swiglu(_ptr(Wgate), _ptr(codebook_gate), _ptr(Wup), _ptr(codebook_up), _ptr(x), _ptr(y),
                                N, K, bits, layout, _stream()))


def gemv_bf16(W, x, y, N: int, K: int):
    """y[N] = W x for a dense bf16 W (N x K, row-major) on torch's current stream: the unquantised baseline."""
    _check(_lib.kmq_gemv_bf16(_ptr(W), _ptr(x), _ptr(y), N, K, _stream()))


def gemv_fused(W, codebook, x, y, N: int, K: int, bits: int, norm_weight=None, eps: float = 0.0, residual=None,
               layout: int = 0, rmsnorm=None):
    """y = residual + W rmsnorm(x; norm_weight, eps) on torch's current stream; both fusions optional.
    rmsnorm defaults to "gains were given"; rmsnorm=True with norm_weight=None normalises with unit gains."""
    if rmsnorm is None:
        rmsnorm = norm_weight is not None
    _check(_lib.kmq_gemv_fused(_ptr(W), _ptr(codebook), _ptr(x), 1 if rmsnorm else 0, _ptr(norm_weight), eps,
                               _ptr(residual), _ptr(y), N, K, bits, layout, _stream()))


def gemv_swiglu_rmsnorm(Wgate, cb_gate, Wup, cb_up, x, norm_weight, eps: float, y, N: int, K: int, bits: int,
                        layout: int = 0):
    """y = silu(Wgate xn) * (Wup xn), xn = rmsnorm(x; norm_weight, eps), one launch."""
    _check(_lib.kmq_gemv_swiglu_rmsnorm(_ptr(Wgate), _ptr(cb_gate), _ptr(Wup), _ptr(cb_up), _ptr(x), _ptr(norm_weight),
                                        eps, _ptr(y), N, K, bits, layout, _stream()))


def kernel_name_fused(N: int, K: int, bits: int, layout: int = 0, pair: bool = False) -> str:
    return _lib.kmq_kernel_name_fused(N, K, bits, layout, 1 if pair else 0).decode()


def quantize_rows(Wdense, N: int, K: int, bits: int, iters: int, packed, codebook):
    """Per-row k-means of dense bf16 weights -> canonical packed indices and N x 2^bits codebooks (device tensors)."""
    _check(_lib.kmq_quantize_rows(_ptr(Wdense), N, K, bits, iters, _ptr(packed), _ptr(codebook), _stream()))


def quantize_blockscaled_workspace_bytes() -> int:
    return int(_lib.kmq_quantize_blockscaled_workspace_bytes())


def quantize_blockscaled(Wdense, N: int, K: int, bits: int, iters: int, packed, codebook, scales, workspace):
    """The paper's format from dense bf16 weights: absmax block scales, one tensor-wide codebook (device tensors)."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.kmq_quantize_blockscaled(_ptr(Wdense), N, K, bits, iters, _ptr(packed), _ptr(codebook), _ptr(scales),
                                         _ptr(workspace), ws_bytes, _stream()))


def dequant(W, codebook, Wdense, N: int, K: int, bits: int, layout: int = 0):
    """Wdense[N][K] (bf16 storage) = codebook[n][idx[n][k]] on torch's current stream."""
    _check(_lib.kmq_dequant(_ptr(W), _ptr(codebook), _ptr(Wdense), N, K, bits, layout, _stream()))


def dequant_blockscaled(W, codebook, scales, Wdense, N: int, K: int, bits: int):
    """Wdense[N][K] (bf16 storage) = bf16(codebook[idx] * scale) of the block-scaled format, on torch's current stream."""
    _check(_lib.kmq_dequant_blockscaled(_ptr(W), _ptr(codebook), _ptr(scales), _ptr(Wdense), N, K, bits, _stream()))
