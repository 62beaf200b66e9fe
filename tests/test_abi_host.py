"""CPU-side checks of the product library: it loads, exports every symbol the
header declares, its host functions agree with the oracle, and every argument
error is reported before anything touches the GPU.  No compute calls."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2602_15563_amd import kmq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BITS = (1, 2, 3, 4)


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "kmq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(kmq_[a-z0-9_]+)\s*\(", text))
    assert {"kmq_pack", "kmq_gemv", "kmq_gemm_smallbatch", "kmq_unpack", "kmq_repack", "kmq_unrepack",
            "kmq_dequant", "kmq_workspace_bytes", "kmq_words_per_row", "kmq_status_string"} <= names
    lib = kmq.raw()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in kmq.h but not exported"


def test_the_probe_library_is_apart_from_the_product():
    """The measurement probes live in their own library: every symbol its header declares is exported
    there, and the product library exports none of them."""
    from paper_2602_15563_amd import probe
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "kmq_probe.h")).read(), flags=re.S)
    names = set(re.findall(r"\b(kmq_probe_[a-z0-9_]+)\s*\(", text))
    assert names == {"kmq_probe_empty", "kmq_probe_read_variants", "kmq_probe_read_name", "kmq_probe_read"}
    for n in sorted(names):
        assert hasattr(probe._lib, n), f"{n} declared in kmq_probe.h but not exported"
        assert not hasattr(kmq.raw(), n)
    assert not hasattr(kmq.raw(), "kmq_stream_read")
    v = probe.read_variants()
    assert len(v) == len(set(v)) >= 8 and all(n.startswith(("oneshot_", "persist_")) for n in v)
    assert probe._lib.kmq_probe_read(None, 4096, 0, None, None) == -1        # argument errors before any launch
    assert probe._lib.kmq_probe_empty(0, 256, None, None) == -1 and probe._lib.kmq_probe_empty(4, 100, None, None) == -1


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("K", (1, 2, 7, 10, 11, 21, 22, 31, 32, 33, 63, 64, 65, 100, 515, 4096))
def test_host_pack_matches_oracle_and_round_trips(bits, K):
    g = np.random.default_rng(bits * 1000 + K)
    for N in (1, 4):
        idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        p = kmq.pack(idx, bits)
        assert np.array_equal(p, oracle.pack(idx, bits))
        assert np.array_equal(kmq.unpack(p, K, bits), idx)
        assert kmq.words_per_row(bits, K) == oracle.words_per_row(bits, K)


def test_unpack_ignores_pad_bits():
    idx = np.array([[3, 1, 2]], dtype=np.uint8)
    p = kmq.pack(idx, 2)
    p[0, 0] |= np.uint32(0xFFFFFFC0)
    assert np.array_equal(kmq.unpack(p, 3, 2), idx)


@pytest.mark.parametrize("bits", BITS)
def test_pack_rejects_out_of_range(bits):
    idx = np.zeros((2, 9), dtype=np.uint8)
    idx[1, 8] = 1 << bits
    with pytest.raises(kmq.KmqError) as e:
        kmq.pack(idx, bits)
    assert e.value.status == 5


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("N", (1, 15, 16, 17, 40))
def test_repack_is_a_reversible_permutation(bits, N):
    K = 1024
    g = np.random.default_rng(N + bits)
    idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    p = kmq.pack(idx, bits)
    t = kmq.repack(p, K, bits, kmq.LAYOUT_TILED)
    wpr = kmq.words_per_row(bits, K)
    assert t.size == -(-N // 16) * 16 * wpr == kmq.tiled_words(N, K, bits, 1)
    assert np.array_equal(kmq.unrepack(t, N, K, bits, kmq.LAYOUT_TILED), p)
    # the documented position formula, element by element
    gpg = {1: 16, 2: 8, 3: 4, 4: 4}[bits]
    gw, nsb = gpg * bits // 4, K // (32 * gpg)

    def position(j, e, tbit):
        if bits == 1:
            return 8 * j + e
        if bits == 4:
            return 32 * j + 4 * e + tbit
        if bits == 2:
            c = 2 * j + e // 4
            return 32 * (c // 4) + 8 * (e % 4) + 2 * (c % 4) + tbit
        h, p = e // 4, 8 * (e % 4)
        if j < 3:
            return 32 * j + p + 3 * h + tbit
        if h == 0:
            return p + 6 + tbit if tbit < 2 else 32 + p + 6
        return 32 + p + 7 if tbit == 0 else 64 + p + 5 + tbit

    for _ in range(300):
        n, k = int(g.integers(0, N)), int(g.integers(0, K))
        sb, grp, e = k // (32 * gpg), (k % (32 * gpg)) // 8, k % 8
        q, j = grp % 4, grp // 4
        rb, nn = divmod(n, 16)
        base = ((rb * nsb + sb) * 64 + q * 16 + nn) * gw
        v = 0
        for tbit in range(bits):
            pos = position(j, e, tbit)
            v |= ((int(t[base + pos // 32]) >> (pos % 32)) & 1) << tbit
        assert v == idx[n, k]
    # rows of a short last block are zero
    if N % 16:
        rb, nn = divmod(N, 16)                            # first missing row
        off = ((rb * nsb) * 64 + nn) * gw
        assert not t[off:off + gw].any()
    assert np.array_equal(kmq.repack(p, K, bits, kmq.LAYOUT_CANONICAL).reshape(N, wpr), p)


@pytest.mark.parametrize("bits", (1, 2))
@pytest.mark.parametrize("N", (1, 15, 16, 17, 40))
def test_rowlane_repack_is_a_reversible_permutation(bits, N):
    """KMQ_LAYOUT_ROWLANE: the position formula of kmq.h, element by element, and the inverse."""
    K = 1024
    g = np.random.default_rng(100 * N + bits)
    idx = g.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    p = kmq.pack(idx, bits)
    t = kmq.repack(p, K, bits, kmq.LAYOUT_ROWLANE)
    wpr = kmq.words_per_row(bits, K)
    assert t.size == -(-N // 16) * 16 * wpr == kmq.tiled_words(N, K, bits, kmq.LAYOUT_ROWLANE)
    assert np.array_equal(kmq.unrepack(t, N, K, bits, kmq.LAYOUT_ROWLANE), p)

    def position(c, u):
        if bits == 2:
            pr = c // 2
            s = pr // 2 + 16 * (pr % 2)
            return 4 * s + 2 * (c % 2) + u
        s, i = c // 4, c % 4
        q, b, view = s // 8, (s % 8) // 2, s % 2
        return 32 * q + ((8 * b + 7 + i) % 32 if view else 8 * b + 3 + i)

    seen = set()
    for _ in range(400):
        n, k = int(g.integers(0, N)), int(g.integers(0, K))
        tile, kp, c = k // 256, (k % 256) // 64, k % 64
        rb, r = divmod(n, 16)
        base = ((rb * (K // 256) + tile) * 64 + kp * 16 + r) * 2 * bits
        v = 0
        for u in range(bits):
            pos = position(c, u)
            assert 0 <= pos < 64 * bits
            seen.add((c, u, pos))
            v |= ((int(t[base + pos // 32]) >> (pos % 32)) & 1) << u
        assert v == idx[n, k]
    # the formula is a bijection of the chunk's bits
    assert len({position(c, u) for c in range(64) for u in range(bits)}) == 64 * bits
    if N % 16:                                            # rows of a short last block are zero
        rb, r = divmod(N, 16)
        off = ((rb * (K // 256)) * 64 + r) * 2 * bits
        assert not t[off:off + 2 * bits].any()


@pytest.mark.parametrize("bits,K", [(1, 128), (2, 320), (3, 1024), (4, 1024), (8, 1024)])
def test_rowlane_repack_rejects_other_bit_widths_and_ragged_k(bits, K):
    idx = np.zeros((4, K), dtype=np.uint8)
    p = kmq.pack(idx, bits)
    assert kmq.tiled_words(4, K, bits, kmq.LAYOUT_ROWLANE) == -1
    with pytest.raises(kmq.KmqError) as e:
        kmq.repack(p, K, bits, kmq.LAYOUT_ROWLANE)
    assert e.value.status == 7
    assert kmq.kernel_name(4, K, bits, 1, kmq.LAYOUT_ROWLANE) == "invalid"


@pytest.mark.parametrize("bits,K", [(1, 256), (2, 128), (3, 64), (4, 96), (2, 33)])
def test_repack_rejects_k_that_is_not_whole_superblocks(bits, K):
    idx = np.zeros((4, K), dtype=np.uint8)
    p = kmq.pack(idx, bits)
    assert kmq.tiled_words(4, K, bits, kmq.LAYOUT_TILED) == -1
    with pytest.raises(kmq.KmqError) as e:
        kmq.repack(p, K, bits, kmq.LAYOUT_TILED)
    assert e.value.status == 7


def test_argument_errors_are_reported_before_any_launch():
    """These calls return an error code from the host-side checks, so they are
    safe (and meaningful) on a machine without a GPU."""
    lib = kmq.raw()
    buf = (ctypes.c_uint8 * 4096)()
    base = ctypes.addressof(buf)
    a16 = (base + 15) & ~15
    W, cb, x, y = a16, a16 + 256, a16 + 512, a16 + 1024
    ok = dict(N=4, K=64, bits=2, layout=0)

    def gemv(W=W, cb=cb, x=x, y=y, N=ok["N"], K=ok["K"], bits=ok["bits"], layout=ok["layout"], ws=None, wsb=0):
        return lib.kmq_gemv(W, cb, x, y, N, K, bits, layout, ws, wsb, None)

    def gemm(M, W=W, x=x, N=4, K=64, bits=2):
        return lib.kmq_gemm_smallbatch(W, cb, x, y, N, K, M, bits, 0, None, 0, None)

    assert gemv(W=None) == 1 and gemv(cb=None) == 1 and gemv(x=None) == 1 and gemv(y=None) == 1
    assert gemv(bits=0) == 2 and gemv(bits=5) == 2
    assert gemv(N=0) == 3 and gemv(K=0) == 3 and gemv(N=-1) == 3 and gemv(K=1 << 30) == 3
    assert gemm(0) == 3 and gemm(17) == 3
    assert gemv(layout=3) == 7 and gemv(layout=-1) == 7
    assert gemv(layout=2) == 7                        # row-lane layout: K = 64 is not a whole number of 256-element tiles
    assert gemv(layout=2, K=1024, bits=3) == 7 and gemv(layout=2, K=1024, W=W + 4) == 4
    assert gemv(K=40, layout=1) == 7                  # 2-bit K=40 is not a whole number of 256-element super-blocks
    assert gemv(W=W + 4) == 4 and gemv(x=x + 2) == 4 and gemv(cb=cb + 2) == 4 and gemv(y=y + 1) == 4
    assert lib.kmq_dequant(None, cb, y, 4, 64, 2, 0, None) == 1
    assert lib.kmq_dequant(W, cb, y, 4, 64, 7, 0, None) == 2
    assert lib.kmq_dequant(W, cb, y, 0, 64, 2, 0, None) == 3
    assert lib.kmq_dequant(W, cb, y, 4, 64, 2, 3, None) == 7
    assert lib.kmq_pack(None, 1, 1, 1, W) == 1 and lib.kmq_unpack(W, 1, 1, 9, W) == 2
    assert kmq.workspace_bytes(0, 64, 2, 1) == 0 and kmq.kernel_name(4, 64, 9, 1) == "invalid"
    # the block-scaled calls and the dense baseline: same rule, checks before any launch
    sc = a16 + 2048

    def bs(W=W, cb=cb, sc=sc, x=x, y=y, N=4, K=64, bits=2, layout=0, M=1):
        return lib.kmq_gemm_smallbatch_blockscaled(W, cb, sc, x, y, N, K, M, bits, layout, None, 0, None)

    assert bs(sc=None) == 1 and bs(W=None) == 1 and bs(bits=9) == 2 and bs(M=17) == 3
    assert bs(K=96) == 3                               # not a whole number of 64-element blocks
    assert bs(layout=1, K=192) == 7 and bs(layout=1, K=32768) == 7 and bs(sc=sc + 1) == 4
    assert kmq.kernel_name_blockscaled(4096, 4096, 3, 16, 1) == "mfma_sc_b3"
    assert lib.kmq_gemv_blockscaled(W, cb, None, x, y, 4, 64, 2, 0, None, 0, None) == 1
    assert kmq.kernel_name_blockscaled(4, 96, 2, 1) == "invalid"
    assert kmq.kernel_name_blockscaled(8192, 8192, 4, 1).startswith("lut_sc_b4")
    assert kmq.kernel_name_blockscaled(8192, 8192, 4, 16).startswith("lut_sc_b4")    # canonical batch: table kernel over (row group, column)
    assert kmq.kernel_name_blockscaled(100, 8192 + 64, 4, 16) == "blockscaled_generic"
    assert lib.kmq_gemv_bf16(None, x, y, 4, 64, None) == 1 and lib.kmq_gemv_bf16(W, x, y, 4, 40000, None) == 3
    assert lib.kmq_gemv_bf16(W + 2, x, y, 4, 64, None) == 4 and lib.kmq_gemv_bf16(W, x, y, 0, 64, None) == 3
    for s in range(9):
        assert kmq.status_string(s) and kmq.status_string(s) != "unknown status"
    assert kmq.status_string(99) == "unknown status"


def test_heuristic_names():
    assert kmq.kernel_name(14336, 4096, 2, 1).startswith("lut_b2")
    assert kmq.kernel_name(4096, 14336, 2, 1).startswith("lut_b2")
    assert kmq.kernel_name(2048, 2048, 1, 1).startswith("lut_b1")
    assert kmq.kernel_name(4096, 4096, 3, 1).startswith("lut_b3")
    assert kmq.kernel_name(4096, 1024, 3, 1) == "lut_loop_b3" and kmq.kernel_name(4096, 1000, 3, 1) == "generic"
    # no row length that is a multiple of 32 (up to 24576) falls to the shape-agnostic kernel on the canonical layout
    for bits in (1, 2, 3, 4):
        for K in range(32, 24576 + 1, 32):
            name = kmq.kernel_name(4096, K, bits, 1)
            assert name.startswith("lut_b") or name == f"lut_loop_b{bits}", (bits, K, name)
    assert kmq.kernel_name(4096, 3072, 4, 1).startswith("lut_b4") and kmq.kernel_name(4096, 24576 + 32, 4, 1) == "generic"
    assert kmq.kernel_name(4096, 11008, 4, 7) == "lut_loop_b4"                                # batches: grid rows
    assert kmq.kernel_name(77, 515, 2, 1) == "generic"
    assert kmq.kernel_name(4096, 4096, 3, 16, kmq.LAYOUT_TILED) == "mfma_b3"
    assert kmq.kernel_name(4096, 4000, 3, 16, kmq.LAYOUT_TILED) == "invalid"
    assert kmq.kernel_name(14336, 4096, 3, 16, kmq.LAYOUT_TILED) == "mfma_kslice_b3" and kmq.kernel_name(14336, 8192, 3, 16, kmq.LAYOUT_TILED) == "mfma_b3"
    assert kmq.kernel_name(14336, 4096, 2, 1, kmq.LAYOUT_ROWLANE) == "rowlane_b2"
    assert kmq.kernel_name(9216, 3072, 1, 4, kmq.LAYOUT_ROWLANE) == "rowlane_b1"
    assert kmq.kernel_name(9216, 3072, 1, 16, kmq.LAYOUT_ROWLANE) == "rowlane_b1"     # four launches of four columns
    assert kmq.kernel_name(64, 256 * 17, 2, 1, kmq.LAYOUT_ROWLANE) == "rowlane_loop_b2"      # 17 tiles: no even split over <= 16 waves
    assert kmq.kernel_name(64, 11008, 1, 3, kmq.LAYOUT_ROWLANE) == "rowlane_loop_b1" and kmq.kernel_name(64, 65536, 2, 1, kmq.LAYOUT_ROWLANE) == "rowlane_loop_b2"
    assert kmq.kernel_name(64, 28672, 1, 1, kmq.LAYOUT_ROWLANE) == "rowlane_b1"              # 112 tiles = 7 x 16 waves
    assert kmq.kernel_name(64, 28672, 2, 1, kmq.LAYOUT_ROWLANE) == "rowlane_loop_b2"         # 2-bit rows beyond 32 tiles: rounds of two tiles
    assert kmq.kernel_name(4096, 14336, 2, 1, kmq.LAYOUT_ROWLANE) == "rowlane_loop_b2" and kmq.kernel_name(4096, 8192, 2, 1, kmq.LAYOUT_ROWLANE) == "rowlane_b2"
    assert kmq.kernel_name(64, 4000, 2, 1, kmq.LAYOUT_ROWLANE) == "invalid"                  # the layout needs whole tiles
    assert kmq.kernel_name_swiglu(14336, 4096, 2, kmq.LAYOUT_ROWLANE) == "rowlane_pair_b2"
    assert kmq.kernel_name_swiglu(8192, 3072, 1, kmq.LAYOUT_ROWLANE) == "rowlane_pair_b1"
    assert kmq.kernel_name_swiglu(64, 256 * 17, 2, kmq.LAYOUT_ROWLANE) == "invalid" and kmq.kernel_name_swiglu(64, 4096, 3, kmq.LAYOUT_ROWLANE) == "invalid"
    assert kmq.workspace_bytes(14336, 4096, 2, 4, kmq.LAYOUT_ROWLANE) == 0


def test_workspace_bytes_split_k():
    """Few long rows: the shape-agnostic kernel splits K over workgroups and needs slices * M * N floats."""
    assert kmq.workspace_bytes(3, 65536, 2, 1) == 16 * 1 * 3 * 4 and kmq.kernel_name(3, 65536, 2, 1) == "generic_splitk"
    assert kmq.workspace_bytes(128, 16384, 2, 2) == 4 * 2 * 128 * 4 and kmq.workspace_bytes(128, 8192, 2, 2) == 0
    assert kmq.workspace_bytes(1, 1 << 20, 4, 16) == 64 * 16 * 1 * 4
    assert kmq.workspace_bytes(600, 16384, 2, 2) == 0       # enough rows
    assert kmq.workspace_bytes(8, 4100, 2, 2) == 0          # short rows
    assert kmq.workspace_bytes(16, 65536, 2, 2, 1) == 0     # tiled layout: matrix-core kernel


def test_argument_errors_of_the_later_calls_and_the_size_limits():
    """Fused decoder calls, quantiser, block-scaled dequantisation: host-side checks only, nothing is launched."""
    lib = kmq.raw()
    buf = (ctypes.c_uint8 * 8192)()
    a16 = (ctypes.addressof(buf) + 15) & ~15
    W, cb, x, y, g, res, sc, ws = a16, a16 + 256, a16 + 512, a16 + 1024, a16 + 1536, a16 + 2048, a16 + 2560, a16 + 3072
    f32 = ctypes.c_float

    def fused(W=W, x=x, norm=1, g=g, eps=1e-5, res=res, y=y, N=4, K=64, bits=2, layout=0):
        return lib.kmq_gemv_fused(W, cb, x, norm, g, f32(eps), res, y, N, K, bits, layout, None)

    assert fused(W=None) == 1 and fused(x=None) == 1 and fused(y=None) == 1
    assert fused(bits=6) == 2 and fused(N=0) == 3 and fused(eps=-1.0) == 3 and fused(norm=2) == 3
    assert fused(layout=1) == 7 and fused(g=g + 2) == 4 and fused(res=res + 1) == 4
    assert fused(norm=0, eps=-1.0, g=None, res=None, N=0) == 3            # still a bad shape
    assert lib.kmq_gemv_swiglu_rmsnorm(W, cb, None, cb, x, g, f32(1e-5), y, 4, 64, 2, 0, None) == 1
    assert lib.kmq_gemv_swiglu_rmsnorm(W, cb, W, cb, x, g, f32(1e-5), y, 4, 64, 2, 1, None) == 7
    assert kmq.kernel_name_fused(8192, 3072, 1).startswith("lut_b1") and kmq.kernel_name_fused(8, 100, 3) == "fused_generic"
    assert kmq.kernel_name_fused(8, 100, 7) == "invalid"

    def qrows(Wd=W, N=4, K=64, bits=2, iters=3, packed=x, cbk=cb):
        return lib.kmq_quantize_rows(Wd, N, K, bits, iters, packed, cbk, None)

    assert qrows(Wd=None) == 1 and qrows(bits=8) == 2 and qrows(bits=0) == 2 and qrows(iters=-1) == 3 and qrows(K=0) == 3
    assert qrows(packed=x + 2) == 4 and qrows(Wd=W + 1) == 4
    need = kmq.quantize_blockscaled_workspace_bytes()
    assert need > 0 and need % 8 == 0

    def qbs(Wd=W, N=4, K=64, bits=2, iters=3, ws=ws, wsb=need, scales=sc):
        return lib.kmq_quantize_blockscaled(Wd, N, K, bits, iters, x, cb, scales, ws, wsb, None)

    assert qbs(scales=None) == 1 and qbs(bits=8) == 2 and qbs(K=96) == 3 and qbs(ws=None) == 6 and qbs(wsb=need - 1) == 6
    assert qbs(ws=ws + 4) == 4
    assert lib.kmq_dequant_blockscaled(W, cb, None, y, 4, 64, 2, None) == 1
    assert lib.kmq_dequant_blockscaled(W, cb, sc, y, 4, 96, 2, None) == 3
    assert lib.kmq_dequant_blockscaled(W, cb, sc, y + 2, 4, 64, 2, None) == 4
    # size limits: N and K up to 2^24 each
    top = 1 << 24
    assert kmq.words_per_row(4, top) == top // 8 and kmq.words_per_row(8, top) == top // 4
    assert lib.kmq_words_per_row(4, top + 1) == -1
    assert lib.kmq_gemv(W, cb, x, y, top + 1, 64, 2, 0, None, 0, None) == 3
    assert lib.kmq_gemv(W, cb, x, y, 4, top + 1, 2, 0, None, 0, None) == 3
    assert kmq.kernel_name(top, 4096, 2, 1).startswith("lut_b2") and kmq.kernel_name(top + 1, 4096, 2, 1) == "invalid"
    assert kmq.workspace_bytes(1, top, 2, 16) == 64 * 16 * 1 * 4


def test_batches_on_the_canonical_layout_take_the_table_kernels():
    assert kmq.kernel_name(9216, 3072, 1, 4).startswith("lut_b1")          # table kernel, one workgroup per (row group, column)
    assert kmq.kernel_name(14336, 4096, 2, 4).startswith("lut_b2") and kmq.kernel_name(14336, 4096, 2, 16).startswith("lut_b2")
    assert kmq.kernel_name(4096, 4096, 4, 2).startswith("lut_b4")
    assert kmq.kernel_name(4096, 4096, 4, 16).startswith("lut_b4") and kmq.kernel_name(2048, 2048, 1, 8).startswith("lut_b1")
    assert kmq.kernel_name(100, 515, 2, 2) == "generic"                     # no table kernel for this K
    assert kmq.kernel_name_blockscaled(8192, 8192, 4, 4).startswith("lut_sc_b4")
    assert kmq.kernel_name_blockscaled(8192, 8192, 4, 16).startswith("lut_sc_b4")


def test_matrix_core_kernel_choice():
    """The kernel whose waves keep their slice of the activations in registers is taken only where it was measured faster."""
    T = kmq.LAYOUT_TILED
    assert kmq.kernel_name(4096, 4096, 3, 8, T) == "mfma_b3"             # one row block per workgroup: the general kernel
    assert kmq.kernel_name(4800, 4096, 3, 8, T) == "mfma_b3"             # 300 row blocks: 150 workgroups would idle 106 CUs
    assert kmq.kernel_name(14336, 8192, 3, 8, T) == "mfma_b3"            # a wave's slice of X would not fit in registers
    assert kmq.kernel_name(14336, 2048, 3, 8, T) == "mfma_b3" and kmq.kernel_name(14336, 2048, 2, 8, T) == "mfma_b2"   # too little work per wave
    assert kmq.kernel_name(14336, 4096, 1, 8, T) == "mfma_b1" and kmq.kernel_name(14336, 4096, 4, 8, T) == "mfma_b4"
    assert kmq.kernel_name(70000, 4096, 3, 8, T) == "mfma_b3"            # more than four row blocks per workgroup
    assert kmq.kernel_name(14336, 4096, 2, 16, T) == "mfma_kslice_b2"


def test_the_built_library_is_not_an_instrumented_build():
    """Launch-shape overrides read from the environment exist only in builds with -DKMQ_TUNING (used for sweeps);
    the library in the tree must be an ordinary build, which never looks at the environment."""
    import os
    path = os.path.join(os.path.dirname(kmq.__file__), "libkmq.so")
    blob = open(path, "rb").read()
    for name in (b"KMQ_LUT_PICK", b"KMQ_RL_CPW", b"KMQ_RL_DBG", b"KMQ_MFMA_NWK", b"KMQ_MFMA_NO_KSLICE", b"kmq_debug_rowlane_timestamps"):
        assert name not in blob, name.decode()
