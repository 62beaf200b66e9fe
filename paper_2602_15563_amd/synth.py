"""Seeded synthetic inputs shaped like the paper's LLM linear layers.

Data plumbing only: this module draws random indices, codebooks and activations
and converts them to bf16 bit patterns.  It holds none of the method's
arithmetic (no packing, no dequantisation, no products) and imports neither the
GPU binding nor the CPU oracle, so both can be fed the same buffers.

The paper (App. E, "Micro-benchmarks" and "Model benchmarks") measures on the
linear layers of Llama-style models; its checkpoints are not used here.
Uniform-random indices stand in for k-means indices of trained weights and
N(0, 0.02) centroids for learned centroids.

For the paper's own weight format (Sec. 2.2 "Nonlinear k-means quantization":
centroids in [-1, 1] shared by the tensor, one bf16 scale per block of 64
elements) the stand-ins are: centroids ~ N(0, 0.45) clipped to [-1, 1] and
sorted (1-bit: (-t, +t), t ~ U(0.5, 0.9)), and scales distributed like the
absolute maximum of 64 samples of N(0, 0.02), the scale an absmax-normalised
block of such weights would get.

Generator: numpy's counter-based Philox, keyed by (seed, stream) where
stream = matrix_number * 16 + kind, kind in {0: indices, 1: codebook, 2: x,
3: block scales, 4: tensor-wide codebook, 5: dense weights, 6: RMSNorm gains,
7: residual stream}.
Normal samples are drawn in fp64, narrowed to fp32, then rounded to bf16 with
round-to-nearest-even; codebooks are sorted after rounding.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

KIND_IDX, KIND_CODEBOOK, KIND_X, KIND_SCALE, KIND_SHARED_CODEBOOK, KIND_DENSE, KIND_NORM, KIND_RESIDUAL = range(8)
BLOCK = 64      # elements per scale along K
SIGMA_W = 0.02  # standard deviation of the centroid distribution


def rng(seed: int, matrix: int, kind: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(matrix) * 16 + int(kind)]))


# ---- bf16 <-> float conversions on bit patterns (uint16) ---------------------

def f32_to_bf16(a) -> np.ndarray:
    """Round fp32 values to bf16 bit patterns, ties to even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_to_f32(h) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32)


def bf16_to_f64(h) -> np.ndarray:
    return bf16_to_f32(h).astype(np.float64)


# ---- tensors -----------------------------------------------------------------

def make_indices(seed: int, matrix: int, N: int, K: int, bits: int) -> np.ndarray:
    """uint8 idx[N][K], uniform in [0, 2^bits)."""
    return rng(seed, matrix, KIND_IDX).integers(0, 1 << bits, size=(N, K), dtype=np.uint8)


def make_codebook(seed: int, matrix: int, N: int, bits: int, symmetric: bool = False) -> np.ndarray:
    """uint16 bf16 codebook[N][2^bits].

    symmetric (1-bit only): (-t, +t) with t = bf16(|a|), a ~ N(0, SIGMA_W).
    otherwise: 2^bits samples of N(0, SIGMA_W), rounded to bf16, sorted ascending.
    """
    g = rng(seed, matrix, KIND_CODEBOOK)
    if symmetric:
        if bits != 1:
            raise ValueError("symmetric codebooks are the 1-bit recipe")
        t = f32_to_bf16(np.abs(g.normal(0.0, SIGMA_W, size=N)).astype(np.float32))
        return np.stack([t | np.uint16(0x8000), t], axis=1).astype(np.uint16)
    c = f32_to_bf16(g.normal(0.0, SIGMA_W, size=(N, 1 << bits)).astype(np.float32))
    order = np.argsort(bf16_to_f32(c), axis=1, kind="stable")
    return np.take_along_axis(c, order, axis=1)


def make_x(seed: int, matrix: int, M: int, K: int) -> np.ndarray:
    """uint16 bf16 X[M][K] ~ N(0, 1)."""
    return f32_to_bf16(rng(seed, matrix, KIND_X).standard_normal(size=(M, K)).astype(np.float32))


def make_dense_weights(seed: int, matrix: int, N: int, K: int) -> np.ndarray:
    """uint16 bf16 W[N][K]: unquantised weights for the quantiser, N(0, SIGMA_W) with a per-row gain
    in [0.5, 2) (rows of trained layers differ in scale, which is what per-row codebooks and block
    scales adapt to)."""
    g = rng(seed, matrix, KIND_DENSE)
    gain = g.uniform(0.5, 2.0, size=(N, 1))
    return f32_to_bf16((g.normal(0.0, SIGMA_W, size=(N, K)) * gain).astype(np.float32))


def make_norm_weight(seed: int, matrix: int, K: int, gain: float = 1.0) -> np.ndarray:
    """uint16 bf16 g[K]: RMSNorm gains, gain * (1 + 0.2 z), z ~ N(0, 1) (trained gains sit around a common level)."""
    return f32_to_bf16((gain * (1.0 + 0.2 * rng(seed, matrix, KIND_NORM).standard_normal(K))).astype(np.float32))


def make_residual(seed: int, matrix: int, N: int) -> np.ndarray:
    """uint16 bf16 residual[N] ~ N(0, 1): the hidden state a projection's output is added to."""
    return f32_to_bf16(rng(seed, matrix, KIND_RESIDUAL).standard_normal(N).astype(np.float32))


def make_shared_codebook(seed: int, matrix: int, bits: int) -> np.ndarray:
    """uint16 bf16 codebook[2^bits] shared by all rows, values in [-1, 1], sorted ascending."""
    g = rng(seed, matrix, KIND_SHARED_CODEBOOK)
    if bits == 1:
        t = f32_to_bf16(np.array([g.uniform(0.5, 0.9)], dtype=np.float32))[0]
        return np.array([t | np.uint16(0x8000), t], dtype=np.uint16)
    c = f32_to_bf16(np.clip(g.normal(0.0, 0.45, size=1 << bits), -1.0, 1.0).astype(np.float32))
    return c[np.argsort(bf16_to_f32(c), kind="stable")]


def make_scales(seed: int, matrix: int, N: int, K: int, block: int = BLOCK) -> np.ndarray:
    """uint16 bf16 scales[N][K // block] > 0, distributed like max |z_j|, j < block, z ~ N(0, SIGMA_W).

    Drawn by inverting the distribution function of that maximum,
    P(max <= t) = (2 Phi(t / sigma) - 1)^block, so one uniform sample per block suffices.
    """
    from scipy.special import ndtri
    if K % block:
        raise ValueError("K must be a multiple of the block size")
    u = rng(seed, matrix, KIND_SCALE).uniform(0.0, 1.0, size=(N, K // block))
    t = SIGMA_W * ndtri(0.5 * (1.0 + u ** (1.0 / block)))
    return f32_to_bf16(np.maximum(t, 1e-6).astype(np.float32))


# ---- the benchmark contract's five configurations ----------------------------

@dataclass(frozen=True)
class Case:
    """One (matrix shape, bit-width, batch) instance of a configuration."""
    cfg: int
    name: str
    seed: int
    matrix: int          # matrix number inside the configuration (RNG stream)
    bits: int
    N: int
    K: int
    M: int
    symmetric: bool = False

    def tensors(self):
        """(idx uint8 N x K, codebook uint16 N x 2^b, X uint16 M x K)."""
        return (make_indices(self.seed, self.matrix, self.N, self.K, self.bits),
                make_codebook(self.seed, self.matrix, self.N, self.bits, self.symmetric),
                make_x(self.seed, self.matrix, self.M, self.K))


def algorithmic_bytes(N: int, K: int, bits: int, M: int) -> int:
    """Bytes the method itself must move per call: packed indices + codebooks +
    activations in + outputs (paper App. E: effective bandwidth = operand sizes / time)."""
    wpr = (K * bits + 31) // 32
    return 4 * N * wpr + 2 * N * (1 << bits) + 2 * M * K + 2 * M * N


def algorithmic_bytes_blockscaled(N: int, K: int, bits: int, M: int, block: int = BLOCK) -> int:
    """Operand bytes of one block-scaled call: indices, the tensor-wide codebook, one bf16
    scale per block, X and Y (the paper's "effective bandwidth" numerator, App. E)."""
    wpr = (K * bits + 31) // 32
    return 4 * N * wpr + 2 * (1 << bits) + 2 * N * (K // block) + 2 * M * K + 2 * M * N


def cases(cfg: int) -> list[Case]:
    """All (shape, batch) instances of configuration ``cfg`` (0..4).

    cfg 4 lists one decoder layer (fused QKV, O, gate, up, down); the 28 layers
    of the sweep share these shapes and differ only in the matrix number.
    """
    if cfg == 0:
        return [Case(0, "b1 2048x2048 M1", 0, 0, 1, 2048, 2048, 1, True)]
    if cfg == 1:
        return [Case(1, "b4 4096x4096 M1", 1, 0, 4, 4096, 4096, 1)]
    if cfg == 2:
        return [Case(2, "b2 gate/up 14336x4096 M1", 2, 0, 2, 14336, 4096, 1),
                Case(2, "b2 down 4096x14336 M1", 2, 1, 2, 4096, 14336, 1)]
    if cfg == 3:
        out = []
        for mi, (N, K) in enumerate([(4096, 4096), (14336, 4096)]):
            for M in (8, 16):
                out.append(Case(3, f"b3 {N}x{K} M{M}", 3, mi, 3, N, K, M))
        return out
    if cfg == 4:
        out = []
        shapes = [("qkv", 9216, 3072), ("o", 3072, 3072), ("gate", 8192, 3072),
                  ("up", 8192, 3072), ("down", 3072, 8192)]
        for M in (1, 4, 16):
            for mi, (nm, N, K) in enumerate(shapes):
                out.append(Case(4, f"b1 {nm} {N}x{K} M{M}", 4, mi, 1, N, K, M, True))
        return out
    raise ValueError("cfg must be 0..4")


LAYER_SHAPES_CFG4 = [(9216, 3072), (3072, 3072), (8192, 3072), (8192, 3072), (3072, 8192)]
N_LAYERS_CFG4 = 28
