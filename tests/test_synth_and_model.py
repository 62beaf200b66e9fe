"""Host-side checks: the seeded input generator and the paper's roofline model
(against the values the paper prints).  No GPU, no oracle."""
import math
import os

import numpy as np
import pytest

from paper_2602_15563_amd import model, synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_generator_is_deterministic_and_streams_differ():
    a = synth.make_indices(2, 0, 8, 64, 2)
    assert np.array_equal(a, synth.make_indices(2, 0, 8, 64, 2))
    assert not np.array_equal(a, synth.make_indices(2, 1, 8, 64, 2))
    assert not np.array_equal(a, synth.make_indices(3, 0, 8, 64, 2))
    assert np.array_equal(synth.make_x(1, 0, 2, 33), synth.make_x(1, 0, 2, 33))


@pytest.mark.parametrize("bits", (1, 2, 3, 4))
def test_indices_cover_the_range_uniformly(bits):
    idx = synth.make_indices(9, 0, 64, 4096, bits)
    assert idx.dtype == np.uint8 and idx.max() == (1 << bits) - 1 and idx.min() == 0
    counts = np.bincount(idx.ravel(), minlength=1 << bits) / idx.size
    assert np.all(np.abs(counts - 1.0 / (1 << bits)) < 0.01)


@pytest.mark.parametrize("bits", (2, 3, 4))
def test_codebooks_sorted_bf16_with_std_002(bits):
    cb = synth.make_codebook(5, 0, 4096, bits)
    v = synth.bf16_to_f64(cb)
    assert cb.shape == (4096, 1 << bits) and cb.dtype == np.uint16
    assert np.all(np.diff(v, axis=1) >= 0)
    assert abs(v.std() - 0.02) < 0.001 and abs(v.mean()) < 0.001


def test_symmetric_one_bit_codebook():
    cb = synth.make_codebook(0, 0, 2048, 1, symmetric=True)
    v = synth.bf16_to_f64(cb)
    assert np.array_equal(v[:, 0], -v[:, 1]) and np.all(v[:, 1] >= 0)
    # |N(0, s)| has mean s*sqrt(2/pi)
    assert abs(v[:, 1].mean() - 0.02 * math.sqrt(2 / math.pi)) < 0.001


def test_x_is_standard_normal_bf16():
    x = synth.bf16_to_f64(synth.make_x(2, 0, 4, 14336))
    assert abs(x.std() - 1.0) < 0.02 and abs(x.mean()) < 0.02


def test_bf16_round_trip_is_identity_on_bf16_values():
    h = np.arange(0x0080, 0x7F80, 37, dtype=np.uint16)             # positive normals
    assert np.array_equal(synth.f32_to_bf16(synth.bf16_to_f32(h)), h)


def test_config_shapes_and_algorithmic_bytes():
    """Byte counts of the benchmark contract's shapes (indices + codebooks + X + Y)."""
    assert synth.algorithmic_bytes(14336, 4096, 2, 1) == 14_831_616       # headline shape
    assert synth.algorithmic_bytes(4096, 14336, 2, 1) == 14_749_696
    assert synth.algorithmic_bytes(2048, 2048, 1, 1) == 540_672
    assert synth.algorithmic_bytes(4096, 4096, 4, 1) == 8_536_064
    assert synth.algorithmic_bytes(14336, 4096, 3, 16) == 22_839_296
    assert synth.algorithmic_bytes(9216, 3072, 1, 4) == 3_674_112
    assert [len(synth.cases(c)) for c in range(5)] == [1, 1, 2, 4, 15]
    layer = sum(N * K for N, K in synth.LAYER_SHAPES_CFG4)
    assert layer == 113_246_208 and abs(layer * synth.N_LAYERS_CFG4 / 1e9 - 3.17) < 0.01


def _golden_model_rows():
    rows = []
    with open(os.path.join(GOLDEN, "roofline_model.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def test_roofline_model_reproduces_the_papers_printed_values():
    nu = 362e12 / 864e9
    seen = set()
    for row in _golden_model_rows():
        kind = row[0]
        seen.add(kind)
        if kind == "peak_speedup":
            p1, p2, want = float(row[1]), float(row[2]), float(row[3])
            assert round(model.speedup(p1, p2, 1, nu), 1) == want
        elif kind == "membound_batch":
            assert math.floor(model.memory_bound_batch(float(row[1]), nu)) == int(row[2])
        elif kind == "no_speedup_batch":
            m = int(row[2])
            assert math.floor(model.memory_bound_batch(float(row[1]), nu)) == m
            assert model.speedup(16, 1.25, m + 1, nu) == 1.0
            assert model.speedup(16, 1.25, m, nu) > 1.0
        elif kind == "eff_bw":
            P, us, want = float(row[1]), float(row[2]), float(row[3])
            got = model.effective_bandwidth(8192 * 8192 * P / 8, us * 1e-6) / 1e9
            assert abs(got - want) <= 2.0
    assert seen == {"peak_speedup", "membound_batch", "no_speedup_batch", "eff_bw"}


def test_roofline_regimes():
    nu = 312.0
    assert model.speedup(16, 2, 1, nu) == 8.0                   # both memory-bound: ratio of precisions
    assert model.speedup(16, 2, 10_000, nu) == 1.0              # both compute-bound
    mid = model.speedup(16, 2, 100, nu)                         # in between: falls like 1/m
    assert abs(mid - 16 * nu / (16 * 100)) < 1e-12
    t = model.kernel_time(2, 4096, 1, 157e12, 8e12)
    assert t == 2 * 4096 * 4096 / (8 * 8e12)
