"""GPU parity on seeded random layer shapes: whatever kernel the library picks for a geometry
(MFMA plans with their tilings, the generic kernels), every output of the step agrees with
the oracle.  Shapes are small enough for the oracle and chosen to land on ragged tiles, edge
channel blocks, several images per pixel tile, odd row lengths and both strides."""
from __future__ import annotations

import numpy as np
import pytest

from paper_2409_11902_amd import synth
from test_gpu_parity import _check_step

pytestmark = pytest.mark.gpu


def _random_specs(count, seed):
    rng = np.random.Generator(np.random.Philox(key=seed))
    out = []
    while len(out) < count:
        R = int(rng.choice([1, 3, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 2]))
        pad = int(rng.integers(0, R // 2 + 1))
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        if H + 2 * pad < R or W + 2 * pad < R:
            continue
        N = int(rng.integers(1, 10))
        C = int(rng.choice([1, 3, 8, 16, 24, 32, 48, 64, 72, 96]))
        K = int(rng.choice([1, 5, 16, 32, 40, 64, 80, 128]))
        k = int(rng.choice([1, 2, 2, 2, 4]))
        dtype = synth.BF16 if rng.random() < 0.75 else synth.F32
        # keep the oracle's direct loops to a fraction of a second
        if N * C * K * H * W * R * R > 6e8:
            continue
        out.append(synth.LayerSpec(f"rnd{len(out)} N{N} C{C} K{K} {H}x{W} R{R} s{stride} p{pad} k{k} {dtype}",
                                   N, C, K, H, W, R, R, stride, pad, k, dtype))
    return out


def _mfma_leaning_specs(count, seed):
    """bf16 only, channel counts that fill MFMA tiles, odd maps (odd element counts, ragged pooling
    tiles), more images: the shapes the tiled kernels see in the workloads, shrunk."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    out = []
    while len(out) < count:
        R = int(rng.choice([1, 3, 3]))
        stride = int(rng.choice([1, 1, 2]))
        pad = R // 2 if rng.random() < 0.8 else 0
        H = int(rng.choice([4, 5, 7, 8, 9, 13, 14, 15, 16, 21, 28]))
        W = H if rng.random() < 0.6 else int(rng.choice([3, 7, 8, 12, 17, 24]))
        if H + 2 * pad < R or W + 2 * pad < R:
            continue
        N = int(rng.integers(1, 18))
        C = int(rng.choice([32, 33, 64, 65, 96, 128]))
        K = int(rng.choice([32, 63, 64, 96, 128, 160]))
        k = int(rng.choice([1, 2, 2, 4]))
        if N * C * K * H * W * R * R > 1.2e9:
            continue
        out.append(synth.LayerSpec(f"mf{len(out)} N{N} C{C} K{K} {H}x{W} R{R} s{stride} p{pad} k{k}",
                                   N, C, K, H, W, R, R, stride, pad, k, synth.BF16))
    return out


SPECS = _random_specs(48, seed=20240911) + _mfma_leaning_specs(40, seed=7)


@pytest.mark.parametrize("spec", SPECS, ids=[s.name for s in SPECS])
def test_random_shape(spec):
    from gpu_util import run_step
    t = synth.make_inputs(spec, "random_shapes")
    _check_step(spec, t, run_step(spec, t))
