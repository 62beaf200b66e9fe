"""Binding over libkmq_probe.so (include/kmq_probe.h): an empty kernel and pure reads,
used by bench.py to measure the launch floor and the read ceiling.  Not part of the product
path: nothing in paper_2602_15563_amd.kmq depends on it."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkmq_probe.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2602_15563_amd.build`")

from .. import kmq as _kmq   # loads torch's HIP runtime first, and shares the stream / pointer helpers

_lib = ctypes.CDLL(LIB_PATH)
_vp, _sz, _int = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_lib.kmq_probe_empty.restype = _int
_lib.kmq_probe_empty.argtypes = [_int, _int, _vp, _vp]
_lib.kmq_probe_read_variants.restype = _int
_lib.kmq_probe_read_name.restype = ctypes.c_char_p
_lib.kmq_probe_read_name.argtypes = [_int]
_lib.kmq_probe_read.restype = _int
_lib.kmq_probe_read.argtypes = [_vp, _sz, _int, _vp, _vp]


def read_variants() -> list[str]:
    return [_lib.kmq_probe_read_name(i).decode() for i in range(_lib.kmq_probe_read_variants())]


def empty(grid: int, block: int, sink=None):
    rc = _lib.kmq_probe_empty(grid, block, _kmq._ptr(sink), _kmq._stream())
    if rc:
        raise RuntimeError(f"kmq_probe_empty failed ({rc})")


def read(t, variant: int, sink=None):
    rc = _lib.kmq_probe_read(_kmq._ptr(t), t.numel() * t.element_size(), variant, _kmq._ptr(sink), _kmq._stream())
    if rc:
        raise RuntimeError(f"kmq_probe_read failed ({rc})")
