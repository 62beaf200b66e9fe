"""Build libkmq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Cross-compiles without a GPU.  Every source is compiled to an object under
``_build/`` (in parallel) and linked into ``paper_2602_15563_amd/libkmq.so``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libkmq.so")
PROBE_OUT = os.path.join(HERE, "probe", "libkmq_probe.so")
OBJ_DIR = os.path.join(ROOT, "_build")

SOURCES = ["kmq_host.cpp", "kmq_generic.hip", "kmq_lut.hip", "kmq_lut_loop.hip", "kmq_rowlane.hip", "kmq_mfma.hip", "kmq_mfma_kslice.hip", "kmq_blockscaled.hip", "kmq_dense.hip", "kmq_quantize.hip", "kmq_fused.hip", "kmq_api.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-fp32 code generation is switched off on purpose: some packed forms have given
         # wrong results on this hardware; ordinary float code loses nothing measurable here
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
if os.environ.get("KMQ_TUNING"):      # launch-shape overrides from the environment, for sweeps; never in a normal build
    FLAGS.append("-DKMQ_TUNING")
if os.environ.get("KMQ_TIMESTAMPS"):  # per-wave time stamps in the row-lane kernel (slower; for taking a kernel apart)
    FLAGS.append("-DKMQ_TIMESTAMPS")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    extra = os.environ.get("KMQ_EXTRA_FLAGS_" + os.path.splitext(src)[0].upper(), "").split()
    cmd = ["hipcc", *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops' is not a recognized" not in l)
    if r.returncode:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def _build_probe() -> str:
    """libkmq_probe.so: the measurement probes bench.py uses (an empty kernel, pure reads); its own
    library, so that the product library exports nothing that is not the product."""
    src = os.path.join(HERE, "probe", "kmq_probe.hip")
    cmd = ["hipcc", *FLAGS, "-shared", "-x", "hip", src, "-o", PROBE_OUT]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("hipcc failed on kmq_probe.hip:\n" + r.stderr)
    return PROBE_OUT


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        probe = ex.submit(_build_probe)
        objs = list(ex.map(_compile, SOURCES))
        probe.result()
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", OUT, "and", PROBE_OUT)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
