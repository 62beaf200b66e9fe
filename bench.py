"""Benchmark of the k-means-quantised GEMV hot path on one MI355X.

A step is one call of the whole hot path (index stream load, unpack + codebook
lookup, multiply-accumulate, K-reduction, bf16 store) on the headline workload
of the benchmark contract: 2-bit 14336 x 4096 GEMV at batch 1.  Inputs are
resident in HBM before the timed region.  Calls rotate over enough distinct
(W, codebook, x, y) instances to exceed the 256 MB last-level cache, and are
replayed from a HIP graph so that launch overhead from Python is not measured
(the protocol of the paper's App. E "Micro-benchmarks", adapted to HIP).

Prints ONE JSON line on stdout.  `--table` additionally writes per-shape
numbers for every contract configuration to bench_table.json in the output folder (--out).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2602_15563_amd import tolerance  # noqa: E402  (acceptance bounds; numpy only -- the HIP library is loaded in main)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E peak, GB/s
LLC_BYTES = 256 << 20          # last-level (memory-side) cache
CALLS_PER_GRAPH = 100

WORKLOADS = {
    # name: (bits, N, K, M, cfg seed, matrix number, symmetric 1-bit codebook)
    "cfg2_gateup_b2_14336x4096_m1": (2, 14336, 4096, 1, 2, 0, False),
    "cfg2_down_b2_4096x14336_m1": (2, 4096, 14336, 1, 2, 1, False),
    "cfg0_b1_2048x2048_m1": (1, 2048, 2048, 1, 0, 0, True),
    "cfg1_b4_4096x4096_m1": (4, 4096, 4096, 1, 1, 0, False),
    "cfg3_b3_4096x4096_m8": (3, 4096, 4096, 8, 3, 0, False),
    "cfg3_b3_4096x4096_m16": (3, 4096, 4096, 16, 3, 0, False),
    "cfg3_b3_14336x4096_m8": (3, 14336, 4096, 8, 3, 1, False),
    "cfg3_b3_14336x4096_m16": (3, 14336, 4096, 16, 3, 1, False),
    # the same two 3-bit matrices at batch 1 (canonical layout; not a contract row: token generation at 3 bits)
    "b3_4096x4096_m1": (3, 4096, 4096, 1, 3, 0, False),
    "b3_14336x4096_m1": (3, 14336, 4096, 1, 3, 1, False),
    "cfg4_qkv_b1_9216x3072_m1": (1, 9216, 3072, 1, 4, 0, True),
    "cfg4_o_b1_3072x3072_m1": (1, 3072, 3072, 1, 4, 1, True),
    "cfg4_gate_b1_8192x3072_m1": (1, 8192, 3072, 1, 4, 2, True),
    "cfg4_up_b1_8192x3072_m1": (1, 8192, 3072, 1, 4, 3, True),
    "cfg4_down_b1_3072x8192_m1": (1, 3072, 8192, 1, 4, 4, True),
    "cfg4_qkv_b1_9216x3072_m4": (1, 9216, 3072, 4, 4, 0, True),
    "cfg4_qkv_b1_9216x3072_m16": (1, 9216, 3072, 16, 4, 0, True),
    "cfg4_down_b1_3072x8192_m16": (1, 3072, 8192, 16, 4, 4, True),
    # down projection of the largest architecture of App. A's table (d = 6144, SwiGLU width 1.3 * 8d/3 rounded to a
    # multiple of 1024 = 21504) at 3 and 4 bits: a row length without a specialised kernel (not a contract row)
    "arch_d6144_down_b3_6144x21504_m1": (3, 6144, 21504, 1, 8, 0, False),
    "arch_d6144_down_b4_6144x21504_m1": (4, 6144, 21504, 1, 8, 1, False),
    # the paper's own format and micro-benchmark shape (App. E, table of m = 1, h = 8192):
    # tensor-wide codebook, one bf16 scale per 64 elements; 8th field = block-scaled
    "paper_b4s_8192x8192_m1": (4, 8192, 8192, 1, 5, 0, False, True),
    "paper_b1s_8192x8192_m1": (1, 8192, 8192, 1, 6, 0, False, True),
    "paper_b2s_8192x8192_m1": (2, 8192, 8192, 1, 7, 0, False, True),
    "paper_b4s_8192x8192_m16": (4, 8192, 8192, 16, 5, 0, False, True),
    "paper_b1s_8192x8192_m16": (1, 8192, 8192, 16, 6, 0, False, True),
}
TABLE_WORKLOADS = list(WORKLOADS)      # what --table times: the contract's shapes and the paper's h = 8192 rows
# the rest of the paper's micro-benchmark grid (square h x h, block-scaled format), used by --micro-sweep
for _h in (2048, 4096, 8192):
    for _b, _seed in ((4, 5), (2, 7), (1, 6)):
        WORKLOADS.setdefault(f"paper_b{_b}s_{_h}x{_h}_m1", (_b, _h, _h, 1, _seed, 0, False, True))
        WORKLOADS.setdefault(f"paper_b{_b}s_{_h}x{_h}_m16", (_b, _h, _h, 16, _seed, 0, False, True))
# The paper's published numbers for those two workloads (App. E, table "perf_micro_m1_impl":
# Triton kernels on an NVIDIA L40S, 864 GB/s): effective GB/s, us per call.
PAPER_NUMBERS = {"paper_b4s_8192x8192_m1": (721.0, 49.5), "paper_b1s_8192x8192_m1": (438.0, 24.0)}
HEADLINE = "cfg2_gateup_b2_14336x4096_m1"
LAYOUT_NAMES = {0: "canonical", 1: "tiled", 2: "rowlane"}
PROFILE_SUMMARIES = {HEADLINE: "gemv_b2_14336x4096_m1_rowlane.txt"}


def _dev(a):
    import numpy as np
    import torch
    view = {np.dtype(np.uint32): np.int32, np.dtype(np.uint16): np.int16}[a.dtype]
    return torch.from_numpy(np.ascontiguousarray(a).view(view)).cuda()


class Instances:
    """R rotating device-resident instances of one workload.  Instance 0 follows
    the seeded recipe exactly (host generator) and is the one checked against the
    oracle; the others are drawn on the device with the same distributions
    (uniform index bits, sorted N(0, 0.02) centroids, N(0, 1) activations)."""

    def __init__(self, name, rotate=True, layout=None, R=None, M=None):
        import numpy as np
        import torch

        from paper_2602_15563_amd import kmq, synth
        self.name = name
        self.bits, self.N, self.K, self.M, seed, matrix, sym = WORKLOADS[name][:7]
        self.scaled = len(WORKLOADS[name]) > 7 and WORKLOADS[name][7]
        if M is not None:
            self.M = M
        bits, N, K, M = self.bits, self.N, self.K, self.M
        # Default layouts (the offline, reversible repack is outside the timed region), by what was measured
        # fastest within the contract's rule that the matrix cores serve batches of 8 and more:
        #   batch 1: the row-lane layout for 2-bit matrices (14336 x 4096: 5.4 us against 6.0 us canonical;
        #            4096 x 14336: 6.0 against 6.5), canonical for the rest (1-bit: both within 0.2 us);
        #   batch 2..7: the row-lane layout where it exists (1 and 2 bits: every weight decoded once, on the
        #            vector units), else tiled;
        #   batch >= 8: tiled (matrix-core kernel).
        if layout is None:
            from paper_2602_15563_amd import kmq as _k
            has_rowlane = not self.scaled and _k.kernel_name(N, K, bits, M, 2) != "invalid"
            if M == 1:
                layout = 2 if (has_rowlane and bits == 2) else 0
            elif M < 8:
                layout = 2 if has_rowlane else 1
            else:
                layout = 1
        self.layout = layout
        self.bytes = (synth.algorithmic_bytes_blockscaled if self.scaled else synth.algorithmic_bytes)(N, K, bits, M)
        self.R = max(2, -(-2 * LLC_BYTES // self.bytes)) if rotate else 1
        self.R = min(self.R, 2048) if R is None else R
        self.idx = synth.make_indices(seed, matrix, N, K, bits)
        self.cb = synth.make_shared_codebook(seed, matrix, bits) if self.scaled else \
            synth.make_codebook(seed, matrix, N, bits, symmetric=sym)
        self.sc = synth.make_scales(seed, matrix, N, K) if self.scaled else None
        self.X = synth.make_x(seed, matrix, M, K)
        t0 = time.perf_counter()
        self.packed = kmq.pack(self.idx, bits)
        self.pack_ms = (time.perf_counter() - t0) * 1e3
        self.repack_ms = None
        wpr = self.packed.shape[1]
        stored = self.packed
        if self.layout != 0:
            t0 = time.perf_counter()
            stored = kmq.repack(self.packed, K, bits, self.layout).reshape(-1, wpr)
            self.repack_ms = (time.perf_counter() - t0) * 1e3
            assert np.array_equal(kmq.unrepack(stored, N, K, bits, self.layout), self.packed)
        nrows_stored = stored.shape[0]
        g = torch.Generator(device="cuda")
        g.manual_seed(1234 + seed)
        self.W, self.C, self.Xd, self.Y = [_dev(stored)], [_dev(self.cb)], [_dev(self.X)], []
        self.S = [_dev(self.sc)] if self.scaled else None
        for _ in range(1, self.R):
            self.W.append(torch.randint(-2**31, 2**31, (nrows_stored, wpr), dtype=torch.int32, device="cuda", generator=g))
            if self.scaled:
                # same distributions as the host recipe: clipped N(0, 0.45) centroids, block-maximum scales
                c = torch.sort((torch.randn(1 << bits, device="cuda", generator=g) * 0.45).clamp(-1, 1)).values.to(torch.bfloat16)
                u = torch.rand((N, K // 64), device="cuda", generator=g, dtype=torch.float64)
                t = 0.02 * torch.special.ndtri(0.5 * (1.0 + u ** (1.0 / 64)))
                self.S.append(t.clamp_min(1e-6).to(torch.bfloat16).view(torch.int16).contiguous())
            elif sym:
                t = (torch.randn(N, device="cuda", generator=g) * 0.02).abs().to(torch.bfloat16)
                c = torch.stack([-t, t], dim=1)
            else:
                c = (torch.randn((N, 1 << bits), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
                c = torch.sort(c.float(), dim=1).values.to(torch.bfloat16)
            self.C.append(c.view(torch.int16).contiguous())
            self.Xd.append(torch.randn((M, K), device="cuda", generator=g).to(torch.bfloat16).view(torch.int16))
        for _ in range(self.R):
            self.Y.append(torch.zeros((M, N), dtype=torch.int16, device="cuda"))
        ws = kmq.workspace_bytes(N, K, bits, M, self.layout)
        self.ws = torch.empty(ws, dtype=torch.uint8, device="cuda") if ws else None
        self.kernel = (kmq.kernel_name_blockscaled if self.scaled else kmq.kernel_name)(N, K, bits, M, self.layout)

    def call(self, i):
        from paper_2602_15563_amd import kmq
        r = i % self.R
        if self.scaled:
            kmq.gemm_smallbatch_blockscaled(self.W[r], self.C[r], self.S[r], self.Xd[r], self.Y[r], self.N, self.K,
                                            self.M, self.bits, self.layout, self.ws)
        elif self.M == 1:
            kmq.gemv(self.W[r], self.C[r], self.Xd[r], self.Y[r], self.N, self.K, self.bits, self.layout, self.ws)
        else:
            kmq.gemm_smallbatch(self.W[r], self.C[r], self.Xd[r], self.Y[r], self.N, self.K, self.M,
                                self.bits, self.layout, self.ws)

    def check(self):
        """Instance 0 against the oracle on sampled row blocks; returns max err/A."""
        import numpy as np
        import torch

        import oracle
        from paper_2602_15563_amd import synth
        self.call(0)
        torch.cuda.synchronize()
        yg = synth.bf16_to_f64(self.Y[0].cpu().numpy().view(np.uint16))
        worst = 0.0
        rng = np.random.default_rng(0)
        starts = [0, self.N - 64] + [int(s) for s in rng.integers(0, self.N - 64, size=4)]
        for n0 in starts:
            if self.scaled:
                Yo, A, _ = oracle.gemm_blockscaled(self.packed, self.cb, self.sc, self.X, self.K, self.bits, rows=(n0, n0 + 64))
            else:
                Yo, A, _ = oracle.gemm(self.packed, self.cb, self.X, self.K, self.bits, rows=(n0, n0 + 64))
            err = np.abs(yg[:, n0:n0 + 64] - Yo[:, n0:n0 + 64])
            if not np.all(err <= tolerance.TOL * A[:, n0:n0 + 64]):
                raise SystemExit(f"bench: {self.name} does not match the oracle in rows {n0}..{n0 + 64}")
            worst = max(worst, float(np.max(err / np.maximum(A[:, n0:n0 + 64], 1e-300))))
        return worst


def time_workload(inst: Instances, steps: int, warmup: int, use_graph: bool = True, per_replay: list | None = None):
    """Returns (seconds for `steps` calls, steps actually timed).  per_replay, if given, receives the
    microseconds per call of every graph replay (an event between replays), for the spread."""
    import torch
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for i in range(max(warmup, 1)):
            inst.call(i)
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if use_graph:
            n_replays = max(10, steps // CALLS_PER_GRAPH)    # never fewer than ten replays: the spread is part of the result
            steps = n_replays * CALLS_PER_GRAPH
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(CALLS_PER_GRAPH):
                    inst.call(i)
            graph.replay()                      # untimed first replay
            stream.synchronize()
            torch.cuda.synchronize()
            marks = []
            e0.record(stream)
            for _ in range(n_replays):
                graph.replay()
                if per_replay is not None:
                    marks.append(torch.cuda.Event(enable_timing=True))
                    marks[-1].record(stream)
            e1.record(stream)
        else:
            torch.cuda.synchronize()
            e0.record(stream)
            for i in range(steps):
                inst.call(i)
            e1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
    if use_graph and per_replay is not None:
        prev = e0
        for m in marks:
            per_replay.append(prev.elapsed_time(m) * 1e3 / CALLS_PER_GRAPH)
            prev = m
    return e0.elapsed_time(e1) * 1e-3, steps


def clock_snapshot():
    """Clock and performance-level state of GPU 0 as rocm-smi reports it.  Taken before this process
    touches the GPU (so: the idle state the run starts from; device settings are read-only here)."""
    import subprocess
    # under a profiler the GPU runtime is already up when this process starts: start no child then
    if "rocprof" in os.environ.get("LD_PRELOAD", "").lower() or any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ):
        return {"unavailable": "profiler attached"}
    try:
        r = subprocess.run(["rocm-smi", "--showclocks", "--showperflevel", "--json"], capture_output=True, text=True,
                           timeout=30)
        line = next(ln for ln in r.stdout.splitlines() if ln.startswith("{"))
        card = json.loads(line).get("card0", {})
        return {k.rstrip(":").replace(" clock", ""): v.strip("()") for k, v in card.items()}
    except Exception as e:   # the tool is absent or refused: say so rather than fail the measurement
        return {"unavailable": type(e).__name__}


SWEEP_LAYERS = 28
SWEEP_SHAPES = ["cfg4_qkv_b1_9216x3072_m1", "cfg4_o_b1_3072x3072_m1", "cfg4_gate_b1_8192x3072_m1",
                "cfg4_up_b1_8192x3072_m1", "cfg4_down_b1_3072x8192_m1"]         # gate and up are two matrices


def run_sweep(M: int, replays: int, fuse: str = "", layout=None):
    """The 1-bit decoder-layer sweep of the fifth contract configuration: 28 layers x
    (fused QKV, O, gate, up, down), every matrix with its own weights (396 MB of indices, so
    each pass streams from HBM), captured as one HIP graph of 140 calls on one stream."""
    import numpy as np
    import torch

    import oracle
    from paper_2602_15563_amd import synth
    insts = [Instances(n, R=SWEEP_LAYERS, M=M, layout=layout) for n in SWEEP_SHAPES]
    worst = max(it.check() for it in insts)
    gate, up = insts[2], insts[3]
    fuse_gate_up = fuse == "gate_up"
    if fuse in ("decoder", "decoder_unit_gains"):
        unit = fuse == "decoder_unit_gains"      # gains multiplied into the weights before quantisation: scalar only
        # the whole layer's elementwise work folded into four launches (attention itself is not part of
        # this path): RMSNorm -> QKV; O + residual; RMSNorm -> gate, up -> SwiGLU; down + residual
        from paper_2602_15563_amd import kmq
        assert M == 1
        qkv, o, down = insts[0], insts[1], insts[4]
        eps = 1e-5
        gn_host = [synth.make_norm_weight(4, 100 + l, qkv.K) for l in range(2)]
        res_host = synth.make_residual(4, 100, o.N)
        gn1 = [_dev(synth.make_norm_weight(4, 100 + 2 * l, qkv.K)) for l in range(SWEEP_LAYERS)]
        gn2 = [_dev(synth.make_norm_weight(4, 101 + 2 * l, qkv.K)) for l in range(SWEEP_LAYERS)]
        hres = [_dev(synth.make_residual(4, 100 + l, o.N)) for l in range(SWEEP_LAYERS)]
        ysw = [torch.zeros(gate.N, dtype=torch.int16, device="cuda") for _ in range(SWEEP_LAYERS)]

        def decoder_layer(l):
            kmq.gemv_fused(qkv.W[l], qkv.C[l], qkv.Xd[l], qkv.Y[l], qkv.N, qkv.K, qkv.bits,
                           norm_weight=None if unit else gn1[l], eps=eps, rmsnorm=True)
            kmq.gemv_fused(o.W[l], o.C[l], o.Xd[l], o.Y[l], o.N, o.K, o.bits, residual=hres[l])
            kmq.gemv_swiglu_rmsnorm(gate.W[l], gate.C[l], up.W[l], up.C[l], gate.Xd[l], None if unit else gn2[l], eps, ysw[l],
                                    gate.N, gate.K, gate.bits)
            kmq.gemv_fused(down.W[l], down.C[l], down.Xd[l], down.Y[l], down.N, down.K, down.bits, residual=hres[l])
        decoder_layer(0)
        torch.cuda.synchronize()

        def close(yg, Y, A, what):
            if not np.all(np.abs(yg - Y) <= tolerance.TOL * A + 2.0 ** -8 * np.abs(Y)):
                raise SystemExit(f"bench: fused decoder call ({what}) does not match the oracle")
        if unit:
            gn_host = [None, None]
        for it, g_, r_ in ((qkv, gn_host[0], None), (o, None, res_host), (down, None, res_host)):
            yg = synth.bf16_to_f64(it.Y[0].cpu().numpy().view(np.uint16)).reshape(-1)
            for n0 in (0, it.N // 2, it.N - 64):
                Y, A = oracle.gemv_fused(it.packed, it.cb, it.X, it.K, it.bits, norm_weight=g_, eps=eps, residual=r_,
                                         rows=(n0, n0 + 64), rmsnorm=it is qkv)
                close(yg[n0:n0 + 64], Y[n0:n0 + 64], A[n0:n0 + 64], it.name)
        yg = synth.bf16_to_f64(ysw[0].cpu().numpy().view(np.uint16))
        for n0 in (0, gate.N // 2, gate.N - 64):
            G, Ag = oracle.gemv_fused(gate.packed, gate.cb, gate.X, gate.K, gate.bits, norm_weight=gn_host[1], eps=eps,
                                      rows=(n0, n0 + 64), rmsnorm=True)
            U, Au = oracle.gemv_fused(up.packed, up.cb, gate.X, gate.K, gate.bits, norm_weight=gn_host[1], eps=eps,
                                      rows=(n0, n0 + 64), rmsnorm=True)
            G, Ag, U, Au = G[n0:n0 + 64], Ag[n0:n0 + 64], U[n0:n0 + 64], Au[n0:n0 + 64]
            want = oracle.swiglu(G, U)
            tol = tolerance.swiglu_contract_bound(U, Ag, Au, oracle.swiglu(G, np.ones_like(G)), want)
            if not np.all(np.abs(yg[n0:n0 + 64] - want) <= tol):
                raise SystemExit("bench: the fused RMSNorm / gate / up / SwiGLU call does not match the oracle")
    if fuse_gate_up:
        # gate and up in one launch with the SwiGLU that consumes them (batch 1, canonical layout)
        from paper_2602_15563_amd import kmq
        assert M == 1
        ysw = [torch.zeros(gate.N, dtype=torch.int16, device="cuda") for _ in range(SWEEP_LAYERS)]

        def fused_call(layer):
            kmq.gemv_swiglu(gate.W[layer], gate.C[layer], up.W[layer], up.C[layer], gate.Xd[layer], ysw[layer],
                            gate.N, gate.K, gate.bits)
        fused_call(0)
        torch.cuda.synchronize()
        yg = synth.bf16_to_f64(ysw[0].cpu().numpy().view(np.uint16))
        for n0 in (0, gate.N // 2, gate.N - 64):
            G, Ag, _ = oracle.gemm(gate.packed, gate.cb, gate.X, gate.K, gate.bits, rows=(n0, n0 + 64))
            U, Au, _ = oracle.gemm(up.packed, up.cb, gate.X, gate.K, gate.bits, rows=(n0, n0 + 64))
            G, Ag, U, Au = G[0, n0:n0 + 64], Ag[0, n0:n0 + 64], U[0, n0:n0 + 64], Au[0, n0:n0 + 64]
            want = oracle.swiglu(G, U)
            tol = tolerance.swiglu_contract_bound(U, Ag, Au, oracle.swiglu(G, np.ones_like(G)), want)
            if not np.all(np.abs(yg[n0:n0 + 64] - want) <= tol):
                raise SystemExit("bench: the fused gate/up/SwiGLU call does not match the oracle")
    # one later layer (device-drawn weights) against the oracle as well, on sampled rows
    layer = 17
    for it in insts:
        it.call(layer)
    torch.cuda.synchronize()
    for it in insts[:1] + insts[4:]:
        if it.layout:                     # repacked: bring the words back to canonical order on the host
            from paper_2602_15563_amd import kmq
            packed = kmq.unrepack(it.W[layer].cpu().numpy().view(np.uint32).reshape(-1), it.N, it.K, it.bits, it.layout)
        else:
            packed = it.W[layer].cpu().numpy().view(np.uint32)
        cb = it.C[layer].cpu().numpy().view(np.uint16)
        X = it.Xd[layer].cpu().numpy().view(np.uint16)
        yg = synth.bf16_to_f64(it.Y[layer].cpu().numpy().view(np.uint16))
        for n0 in (0, it.N // 2, it.N - 64):
            Yo, A, _ = oracle.gemm(packed, cb, X, it.K, it.bits, rows=(n0, n0 + 64))
            err = np.abs(yg[:, n0:n0 + 64] - Yo[:, n0:n0 + 64])
            if not np.all(err <= tolerance.TOL * A[:, n0:n0 + 64]):
                raise SystemExit(f"bench: sweep layer {layer} of {it.name} does not match the oracle")
            worst = max(worst, float(np.max(err / np.maximum(A[:, n0:n0 + 64], 1e-300))))
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        def one_pass():
            for layer in range(SWEEP_LAYERS):
                if fuse.startswith("decoder"):
                    decoder_layer(layer)
                elif fuse_gate_up:
                    insts[0].call(layer)
                    insts[1].call(layer)
                    fused_call(layer)
                    insts[4].call(layer)
                else:
                    for it in insts:
                        it.call(layer)
        one_pass()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            one_pass()
        graph.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(replays):
            graph.replay()
        e1.record(stream)
        stream.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / replays
    nbytes = SWEEP_LAYERS * sum(it.bytes for it in insts)
    calls = SWEEP_LAYERS * (len(insts) - (1 if fuse else 0))
    suffix = {"": "", "gate_up": "_fused_gate_up_swiglu", "decoder": "_fused_rmsnorm_swiglu_residual",
              "decoder_unit_gains": "_fused_rmsnorm_unit_gains_swiglu_residual"}[fuse]
    return {"workload": f"cfg4_sweep_28layers_m{M}" + suffix, "us_per_sweep": round(us, 2), "us_per_call": round(us / calls, 3),
            "passes_per_s": round(1e6 / us, 1),
            "calls": calls, "GBps": round(nbytes / us * 1e-3, 1), "pct_peak": round(100 * nbytes / us * 1e-3 / HBM_PEAK_GBS, 2),
            "bytes": nbytes, "kernels": sorted({it.kernel for it in insts}),
            "layout": LAYOUT_NAMES[insts[0].layout], "max_err_over_A": float(f"{worst:.3e}")}


def run_pair(name: str, layout: int, replays: int = 20):
    """The fused gate / up / SwiGLU call (kmq_gemv_swiglu) on two matrices of workload `name`'s shape:
    y = silu(Wgate x) * (Wup x) in one launch, rotating instances, same graph protocol.  Instance 0 of
    both matrices follows the host recipe and is checked against the oracle on sampled rows."""
    import numpy as np
    import torch

    import oracle
    from paper_2602_15563_amd import kmq, synth
    spec = WORKLOADS[name]
    up_name = name + "__up"
    WORKLOADS[up_name] = spec[:5] + (spec[5] + 7,) + spec[6:]        # the same shape, another matrix number
    gate = Instances(name, layout=layout, M=1)
    up = Instances(up_name, layout=layout, M=1, R=gate.R)
    R = gate.R
    ys = [torch.zeros(gate.N, dtype=torch.int16, device="cuda") for _ in range(R)]

    def call(i):
        r = i % R
        kmq.gemv_swiglu(gate.W[r], gate.C[r], up.W[r], up.C[r], gate.Xd[r], ys[r], gate.N, gate.K, gate.bits, layout)
    call(0)
    torch.cuda.synchronize()
    yg = synth.bf16_to_f64(ys[0].cpu().numpy().view(np.uint16))
    for n0 in (0, gate.N // 2, gate.N - 64):
        G, Ag, _ = oracle.gemm(gate.packed, gate.cb, gate.X, gate.K, gate.bits, rows=(n0, n0 + 64))
        U, Au, _ = oracle.gemm(up.packed, up.cb, gate.X, gate.K, gate.bits, rows=(n0, n0 + 64))
        G, Ag, U, Au = G[0, n0:n0 + 64], Ag[0, n0:n0 + 64], U[0, n0:n0 + 64], Au[0, n0:n0 + 64]
        want = oracle.swiglu(G, U)
        tol = tolerance.swiglu_contract_bound(U, Ag, Au, oracle.swiglu(G, np.ones_like(G)), want)
        if not np.all(np.abs(yg[n0:n0 + 64] - want) <= tol):
            raise SystemExit(f"bench: the fused gate/up/SwiGLU call on {name} (layout {layout}) does not match the oracle")
    us = _graph_us_per_call(call, replays)
    nbytes = gate.bytes + up.bytes - 2 * gate.K - 2 * gate.N        # one x, one y
    return {"workload": name.replace("_m1", "") + "_pair_swiglu_m1", "kernel": kmq.kernel_name_swiglu(gate.N, gate.K, gate.bits, layout),
            "layout": LAYOUT_NAMES[layout], "us_per_call": round(us, 3), "GBps": round(nbytes / us * 1e-3, 1),
            "pct_peak": round(100 * nbytes / us * 1e-3 / HBM_PEAK_GBS, 2), "bytes": nbytes, "R": R}


def time_bf16_baseline(N: int, K: int, steps: int):
    """The unquantised product on the same machine: dense bf16 W (2*N*K bytes), rotating
    instances, same graph replay.  Returns us per call and effective GB/s."""
    import torch

    from paper_2602_15563_amd import kmq
    nbytes = 2 * N * K + 2 * K + 2 * N
    R = max(2, -(-2 * LLC_BYTES // nbytes))
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    Ws = [(torch.randn((N, K), device="cuda", generator=g) * 0.02).to(torch.bfloat16).view(torch.int16) for _ in range(R)]
    xs = [torch.randn(K, device="cuda", generator=g).to(torch.bfloat16).view(torch.int16) for _ in range(R)]
    ys = [torch.zeros(N, dtype=torch.int16, device="cuda") for _ in range(R)]
    # one instance against the oracle, sampled rows
    import numpy as np

    import oracle
    from paper_2602_15563_amd import synth
    kmq.gemv_bf16(Ws[0], xs[0], ys[0], N, K)
    torch.cuda.synchronize()
    yg = synth.bf16_to_f64(ys[0].cpu().numpy().view(np.uint16))
    Wh, xh = Ws[0][:64].cpu().numpy().view(np.uint16), xs[0].cpu().numpy().view(np.uint16)
    Yo, A, _ = oracle.gemm_dense(Wh, xh)
    if not np.all(np.abs(yg[:64] - Yo) <= tolerance.TOL * A):
        raise SystemExit("bench: the dense bf16 baseline does not match the oracle")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        graph = torch.cuda.CUDAGraph()
        for i in range(R):
            kmq.gemv_bf16(Ws[i], xs[i], ys[i], N, K)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(CALLS_PER_GRAPH):
                kmq.gemv_bf16(Ws[i % R], xs[i % R], ys[i % R], N, K)
        graph.replay()
        stream.synchronize()
        n = max(1, steps // CALLS_PER_GRAPH)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            graph.replay()
        e1.record(stream)
        stream.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (n * CALLS_PER_GRAPH)
    return {"us_per_call": round(us, 3), "GB/s": round(nbytes / us * 1e-3, 1), "bytes": nbytes, "rotating_instances": R}


def _graph_us_per_call(launch, replays: int):
    """us per call of launch(i), i = 0..99, captured into one HIP graph and replayed."""
    import torch
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for i in range(20):
            launch(i)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(CALLS_PER_GRAPH):
                launch(i)
        graph.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(replays):
            graph.replay()
        e1.record(stream)
        stream.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (replays * CALLS_PER_GRAPH)


def time_launch_floor(replays: int = 20):
    """What a call costs when the kernel does nothing: empty kernels (kmq_probe_empty) through the same
    100-call graph protocol, at the launch shapes the product kernels use."""
    import torch

    from paper_2602_15563_amd import probe
    sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
    shapes = {"1x64": (1, 64), "896x512": (896, 512), "1792x256": (1792, 256), "256x1024": (256, 1024), "3584x256": (3584, 256)}
    return {k: round(_graph_us_per_call(lambda i, g=g, b=b: probe.empty(g, b, sink), replays), 3) for k, (g, b) in shapes.items()}


def time_read_ceiling(inst: Instances, replays: int = 20):
    """Pure reads (kmq_probe_read: no decode, no store) of the same rotating index streams, and of a
    134 MB buffer, through the same graph protocol: every probe variant, the best one reported."""
    import torch

    from paper_2602_15563_amd import probe
    names = probe.read_variants()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    big = [torch.empty(134217728 // 4, dtype=torch.int32, device="cuda").random_() for _ in range(5)]
    for label, bufs, rep in (("same_bytes", inst.W, replays), ("134MB", big, 3)):
        nbytes = bufs[0].numel() * 4
        rows = {}
        for v, name in enumerate(names):
            rows[name] = round(_graph_us_per_call(lambda i, v=v: probe.read(bufs[i % len(bufs)], v, sink), rep), 3)
        best = min(rows, key=rows.get)
        out[label] = {"bytes": nbytes, "best_variant": best, "us_per_call": rows[best],
                      "GB/s": round(nbytes / rows[best] * 1e-3, 1), "all_variants_us": rows}
    del big
    torch.cuda.empty_cache()
    out["us_per_call"] = out["same_bytes"]["us_per_call"]
    out["GB/s"] = out["same_bytes"]["GB/s"]
    out["what"] = "kmq_probe_read (libkmq_probe.so): reads only, no decode, no store; best of the listed variants"
    return out


def committed_profile(workload: str, kernel: str):
    """Figures of the committed rocprofv3 summaries for this workload, or None where there is no summary or
    it was taken with another kernel than the one this run times (then the figures do not describe it).
    The summaries state: kernel = <name>, traffic_bytes_per_launch = <HBM bytes from FETCH_SIZE + WRITE_SIZE,
    scaled by a copy of known size>, kernel_us_avg / kernel_us_median = <kernel-trace durations>."""
    path = os.path.join(ROOT, "profiles", PROFILE_SUMMARIES.get(workload, "_none_"))
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.startswith(("#", " ")):
            k, v = line.split("=", 1)
            vals[k.strip()] = v.strip()
    if vals.get("kernel") != kernel:
        return None
    out = {"file": "profiles/" + PROFILE_SUMMARIES[workload]}
    for k in ("traffic_bytes_per_launch", "kernel_us_avg", "kernel_us_median"):
        if k in vals:
            out[k] = float(vals[k]) if "us" in k else int(vals[k])
    return out


def run_large_batch(h: int = 8192, batches=(16, 64, 256), replays: int = 5):
    """Batches above the fused kernels' range, by the route the paper recommends there (App. E
    "Model benchmarks"): dequantise in a separate kernel (kmq_dequant_blockscaled), then a dense bf16
    GEMM -- the GEMM is torch.matmul, i.e. the vendor library, used here as the stand-in for "any
    dense GEMM" and timed alone as the unquantised baseline.  Block-scaled format, h x h, rotating
    weights; eager launches timed with events on the launch stream (library GEMMs pick workspaces
    at run time, so they are kept out of graphs)."""
    import numpy as np
    import torch

    import oracle
    from paper_2602_15563_amd import kmq, synth
    rows = []
    R = 3
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    Wd = [torch.empty((h, h), dtype=torch.bfloat16, device="cuda") for _ in range(R)]
    dense = [(torch.randn((h, h), device="cuda", generator=g) * 0.02).to(torch.bfloat16) for _ in range(R)]
    for bits in (4, 1):
        wpr = h * bits // 32
        Wp = [torch.randint(-2**31, 2**31, (h, wpr), dtype=torch.int32, device="cuda", generator=g) for _ in range(R)]
        cb = _dev(synth.make_shared_codebook(5, bits, bits))
        sc = [_dev(synth.make_scales(5, i, h, h)) for i in range(R)]
        # the dequantised matrix of instance 0 against the oracle, first rows
        kmq.dequant_blockscaled(Wp[0], cb, sc[0], Wd[0].view(torch.int16), h, h, bits)
        torch.cuda.synchronize()
        want = oracle.dequant_blockscaled(Wp[0][:8].cpu().numpy().view(np.uint32), synth.make_shared_codebook(5, bits, bits),
                                          sc[0][:8].cpu().numpy().view(np.uint16), h, bits)
        if not np.array_equal(Wd[0][:8].view(torch.int16).cpu().numpy().view(np.uint16), want):
            raise SystemExit("bench: kmq_dequant_blockscaled does not match the oracle")
        for M in batches:
            X = torch.randn((M, h), device="cuda", generator=g).to(torch.bfloat16)
            stream = torch.cuda.Stream()

            def timed(fn, n):
                with torch.cuda.stream(stream):
                    for i in range(R):
                        fn(i)
                    stream.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for i in range(n):
                        fn(i % R)
                    e1.record(stream)
                    stream.synchronize()
                return e0.elapsed_time(e1) * 1e3 / n

            def route(i):
                kmq.dequant_blockscaled(Wp[i], cb, sc[i], Wd[i].view(torch.int16), h, h, bits)
                torch.matmul(X, Wd[i].t())
            t_route = timed(route, 30 * replays)
            t_deq = timed(lambda i: kmq.dequant_blockscaled(Wp[i], cb, sc[i], Wd[i].view(torch.int16), h, h, bits), 30 * replays)
            t_gemm = timed(lambda i: torch.matmul(X, dense[i].t()), 30 * replays)
            row = {"workload": f"paper_b{bits}s_{h}x{h}_m{M}_dequant_then_gemm", "us_route": round(t_route, 2),
                   "us_dequant": round(t_deq, 2), "us_bf16_gemm": round(t_gemm, 2), "speedup_vs_bf16": round(t_gemm / t_route, 3)}
            if M <= 16:
                it = Instances(f"paper_b{bits}s_{h}x{h}_m16", M=M)
                sec, n = time_workload(it, 2000, 50)
                row["us_fused_tiled"] = round(sec / n * 1e6, 2)
                row["fused_speedup_vs_bf16"] = round(t_gemm / row["us_fused_tiled"], 3)
                del it
            rows.append(row)
        del Wp, sc
        torch.cuda.empty_cache()
    return rows


def run_micro_sweep():
    """The paper's micro-benchmark grid on this machine (App. E "Micro-benchmarks": square h x h products swept
    over batch, hidden size and bit-width, figure only): block-scaled format, h in {2048, 4096, 8192}, bits in
    {4, 2, 1}, batch 1 (canonical layout, against the dense bf16 GEMV) and batch 16 (tiled layout, against the
    vendor library's bf16 GEMM through torch.matmul), with the paper's roofline model evaluated beside each."""
    import torch

    from paper_2602_15563_amd import model
    nu = 2.5e15 / (HBM_PEAK_GBS * 1e9)
    rows = []
    for h in (2048, 4096, 8192):
        base1 = time_bf16_baseline(h, h, 2000)["us_per_call"]
        g = torch.Generator(device="cuda")
        g.manual_seed(11)
        R = max(2, -(-2 * LLC_BYTES // (2 * h * h)))
        Wd = [(torch.randn((h, h), device="cuda", generator=g) * 0.02).to(torch.bfloat16) for _ in range(R)]
        X = torch.randn((16, h), device="cuda", generator=g).to(torch.bfloat16)
        # the library GEMM replayed from a graph like everything else here (its results are not used: eager
        # launches of it are bound by the host at these sizes, which would flatter the comparison)
        Yb = [torch.empty((16, h), dtype=torch.bfloat16, device="cuda") for _ in range(R)]
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for i in range(R):
                torch.matmul(X, Wd[i].t(), out=Yb[i])
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(CALLS_PER_GRAPH):
                    torch.matmul(X, Wd[i % R].t(), out=Yb[i % R])
            graph.replay()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                graph.replay()
            e1.record(stream)
            stream.synchronize()
        base16 = e0.elapsed_time(e1) * 1e3 / (10 * CALLS_PER_GRAPH)
        del graph, Yb
        del Wd
        torch.cuda.empty_cache()
        for bits in (4, 2, 1):
            for M, base in ((1, base1), (16, base16)):
                it = Instances(f"paper_b{bits}s_{h}x{h}_m{M}")
                w = it.check()
                sec, n = time_workload(it, 3000, 100)
                us = sec / n * 1e6
                rows.append({"h": h, "bits": bits, "P_w": bits + 0.25, "batch": M, "kernel": it.kernel,
                             "us_per_call": round(us, 3), "GBps": round(it.bytes / us * 1e-3, 1),
                             "us_bf16": round(base, 3), "speedup_vs_bf16": round(base / us, 2),
                             "model_max_speedup": round(model.speedup(16.0, bits + 0.25, M, nu), 2),
                             "max_err_over_A": float(f"{w:.3e}")})
                print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
                del it
                torch.cuda.empty_cache()
    return rows


def cpu_baseline(inst: Instances):
    """The oracle, as it stands, single-threaded, on the same matrix."""
    import oracle
    best = None
    n_rows = inst.N
    def run(rows=None):
        if inst.scaled:
            oracle.gemm_blockscaled(inst.packed, inst.cb, inst.sc, inst.X, inst.K, inst.bits, rows=rows)
        else:
            oracle.gemm(inst.packed, inst.cb, inst.X, inst.K, inst.bits, rows=rows)
    run((0, min(64, n_rows)))   # warm-up
    t_total = 0.0
    runs = 0
    while runs < 3 or (t_total < 10.0 and runs < 20):
        t = time.perf_counter()
        run()
        dt = time.perf_counter() - t
        best = dt if best is None else min(best, dt)
        t_total += dt
        runs += 1
    return {"value": round(inst.bytes / best / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "ms_per_call": round(best * 1e3, 2),
            "sample": f"the whole {inst.name} matrix ({inst.N}x{inst.K}, batch {inst.M}), best of {runs} calls"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(WORKLOADS))
    ap.add_argument("--no-graph", action="store_true", help="launch directly instead of replaying a HIP graph")
    ap.add_argument("--no-rotate", action="store_true", help="reuse one instance (cache-resident, NOT the headline)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-probes", action="store_true", help="skip the launch-floor and read-ceiling probes")
    ap.add_argument("--no-cache-resident", action="store_true",
                    help="skip the secondary same-matrix-every-call timing (keeps a kernel trace to the cold calls)")
    ap.add_argument("--layout", type=int, default=None, choices=(0, 1, 2),
                    help="0 canonical, 1 tiled (matrix-core order), 2 row-lane (default: per workload, see Instances)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the timed region, launch a plain 64 MiB device copy 10 times: a kernel of known "
                         "traffic against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--sweep", action="store_true",
                    help="also run the 28-layer 1-bit decoder sweep at batch 1, 4 and 16 -> <out>/bench_sweep.json")
    ap.add_argument("--micro-sweep", action="store_true",
                    help="also run the paper's micro-benchmark grid (h x bits x batch 1 / 16) -> <out>/bench_micro_sweep.json")
    ap.add_argument("--large-batch", action="store_true",
                    help="also time batches 16 / 64 / 256 at h = 8192 by dequantise + dense GEMM -> <out>/bench_large_batch.json")
    ap.add_argument("--table", action="store_true", help="also time every contract shape and the paper's h = 8192 rows -> <out>/bench_table.json")
    ap.add_argument("--no-contract-shapes", action="store_true",
                    help="skip the short timing of the contract's other shapes and of the batch-1 decoder sweep (config.contract_shapes)")
    ap.add_argument("--out", default=os.path.join(ROOT, "bench_out"), help="folder for the json files of --table, --sweep, --micro-sweep and --large-batch")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on exactly one GPU (--gpus 1); "
                         "the path shards by rows or by K across GPUs but no multi-GPU leg exists here")

    clocks = clock_snapshot()
    import numpy as np
    import torch

    from paper_2602_15563_amd import kmq  # noqa: F401  (fails loudly if the HIP library is missing)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    inst = Instances(args.workload, rotate=not args.no_rotate, layout=args.layout)
    worst = inst.check()
    if args.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
    replay_us = []
    secs, steps = time_workload(inst, args.steps, args.warmup, use_graph=not args.no_graph, per_replay=replay_us)
    us = secs / steps * 1e6
    gbs = inst.bytes / (secs / steps) / 1e9
    out = {
        "metric": "effective HBM GB/s (% of peak) and us/call, 2-bit 14336x4096 GEMV bs=1"
                  if args.workload == HEADLINE else f"effective HBM GB/s, {args.workload}",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(us * 1e-3, 6), "us_per_call": round(us, 3),
        "us_per_call_se": round(float(np.std(replay_us, ddof=1) / np.sqrt(len(replay_us))), 4) if len(replay_us) > 1 else None,
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": round(gbs / PAPER_NUMBERS[args.workload][0], 3) if args.workload in PAPER_NUMBERS else None,
        "dtype": "bf16", "accumulate_dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "bits": inst.bits, "N": inst.N, "K": inst.K, "batch": inst.M,
                   "kernel": inst.kernel, "layout": LAYOUT_NAMES[inst.layout],
                   "rotating_instances": inst.R, "hip_graph": not args.no_graph,
                   "algorithmic_bytes_per_call": inst.bytes, "max_err_over_A_vs_oracle": float(f"{worst:.3e}"),
                   "clocks_before_run": clocks,
                   "offline_host_ms": {"kmq_pack": round(inst.pack_ms, 2),
                                       "kmq_repack": None if inst.repack_ms is None else round(inst.repack_ms, 2)}},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "note": "achieved = algorithmic bytes per launch / average launch-to-launch time "
                             "(HIP events on the launch stream around the timed region); traffic and kernel_us_* come "
                             "from the committed rocprofv3 summary named in profile_file, and are null when that summary "
                             "was taken with another kernel than this run's"},
    }
    prof = committed_profile(args.workload, inst.kernel)
    if prof:
        out["roofline"]["traffic"] = prof.get("traffic_bytes_per_launch")
        out["roofline"]["kernel_us_avg"] = prof.get("kernel_us_avg")
        out["roofline"]["kernel_us_median"] = prof.get("kernel_us_median")
        out["roofline"]["profile_file"] = prof["file"]
    if args.workload in PAPER_NUMBERS:
        out["config"]["paper"] = {"GB/s": PAPER_NUMBERS[args.workload][0], "us_per_call": PAPER_NUMBERS[args.workload][1],
                                  "hardware": "NVIDIA L40S (864 GB/s), Triton kernel, paper App. E; another machine: context only"}
    if inst.scaled and inst.M == 1:
        # speed-up over an unquantised bf16 product on this machine, next to the paper's roofline
        # model (Sec. 3.3, eq. "theoretical-speedup") evaluated for it: nu = dense bf16 op/s / HBM byte/s
        from paper_2602_15563_amd import model
        base = time_bf16_baseline(inst.N, inst.K, 2000)
        nu = 2.5e15 / (HBM_PEAK_GBS * 1e9)
        out["config"]["bf16_baseline"] = base
        out["config"]["speedup_vs_bf16"] = round(base["us_per_call"] / us, 2)
        out["config"]["model_max_speedup"] = round(model.speedup(16.0, inst.bits + 0.25, inst.M, nu), 2)
    if not args.no_probes:
        out["roofline"]["floor_us"] = time_launch_floor()
        out["roofline"]["read_ceiling"] = time_read_ceiling(inst)
    if not args.no_rotate and not args.no_graph and not args.no_cache_resident:
        # secondary figure, NOT the headline: the same matrix every call, so it is served from the caches
        one = Instances(args.workload, rotate=False, layout=args.layout)
        s1, n1 = time_workload(one, 5000, 100)
        out["config"]["cache_resident_us_per_call"] = round(s1 / n1 * 1e6, 3)
        del one
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(inst)

    if not args.no_contract_shapes and args.workload == HEADLINE and not args.table:
        # the contract's other configurations, briefly (the headline above is the metric; --table and --sweep
        # time these at length): same protocol, 2000 calls each, instance 0 checked against the oracle
        rows = []
        for name in WORKLOADS:
            if not name.startswith("cfg") or name == HEADLINE:
                continue
            it = Instances(name)
            w = it.check()
            s, n = time_workload(it, 2000, 100)
            rows.append({"workload": name, "kernel": it.kernel, "layout": LAYOUT_NAMES[it.layout],
                         "us_per_call": round(s / n * 1e6, 3),
                         "pct_peak": round(100 * it.bytes / (s / n) / 1e9 / HBM_PEAK_GBS, 2),
                         "max_err_over_A": float(f"{w:.3e}")})
            M_, lay_ = it.M, it.layout
            del it
            torch.cuda.empty_cache()
            if 2 <= M_ < 8 and lay_ != 1:
                # batches below 8 run on the vector units by the contract's rule; the matrix-core kernel on the
                # tiled layout next to it, for comparison
                it = Instances(name, layout=1)
                it.check()
                s, n = time_workload(it, 2000, 100)
                rows[-1]["tiled_matrix_core"] = {"kernel": it.kernel, "us_per_call": round(s / n * 1e6, 3)}
                del it
                torch.cuda.empty_cache()
        out["config"]["contract_shapes"] = rows
        if not args.sweep:
            sw = run_sweep(1, 50)
            out["config"]["decoder_sweep_batch1"] = {k: sw[k] for k in ("us_per_sweep", "us_per_call", "passes_per_s", "calls", "pct_peak", "layout", "max_err_over_A")}
            torch.cuda.empty_cache()

    if args.table:
        rows = []
        for name in TABLE_WORKLOADS:
            it = Instances(name)
            w = it.check()
            s, n = time_workload(it, 5000, 100)
            rows.append({"workload": name, "kernel": it.kernel, "layout": LAYOUT_NAMES[it.layout],
                         "us_per_call": round(s / n * 1e6, 3),
                         "GBps": round(it.bytes / (s / n) / 1e9, 1),
                         "pct_peak": round(100 * it.bytes / (s / n) / 1e9 / HBM_PEAK_GBS, 2),
                         "bytes": it.bytes, "R": it.R, "max_err_over_A": float(f"{w:.3e}")})
            print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
            del it
            torch.cuda.empty_cache()
        # the 2-bit gate / up pair of the third configuration as ONE fused launch (an extra measurement, not a
        # contract row: the contract times the two products separately), on both layouts that serve it
        for lay in (0, 2):
            rows.append(run_pair(HEADLINE, lay))
            print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
            torch.cuda.empty_cache()
        os.makedirs(args.out, exist_ok=True)
        with open(os.path.join(args.out, "bench_table.json"), "w") as f:
            json.dump(rows, f, indent=1)

    if args.sweep:
        rows = []
        for M, fused, lay in ((1, "", None), (1, "gate_up", None), (1, "decoder", None), (1, "decoder_unit_gains", None),
                              (4, "", 2), (4, "", 1), (16, "", None)):
            rows.append(run_sweep(M, 200, fuse=fused, layout=lay))
            print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
            torch.cuda.empty_cache()
        os.makedirs(args.out, exist_ok=True)
        with open(os.path.join(args.out, "bench_sweep.json"), "w") as f:
            json.dump(rows, f, indent=1)
        out["config"]["decoder_sweep"] = rows

    if args.micro_sweep:
        rows = run_micro_sweep()
        os.makedirs(args.out, exist_ok=True)
        with open(os.path.join(args.out, "bench_micro_sweep.json"), "w") as f:
            json.dump(rows, f, indent=1)
        out["config"]["micro_sweep"] = rows

    if args.large_batch:
        rows = run_large_batch()
        for r in rows:
            print(json.dumps(r), file=sys.stderr, flush=True)
        os.makedirs(args.out, exist_ok=True)
        with open(os.path.join(args.out, "bench_large_batch.json"), "w") as f:
            json.dump(rows, f, indent=1)
        out["config"]["large_batch"] = rows

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
