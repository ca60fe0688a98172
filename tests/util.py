"""Helpers shared by the tests (no arithmetic of the method's kernels)."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2409_11902_amd import synth


def rel_l2(got, want) -> float:
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    den = float(np.linalg.norm(want))
    num = float(np.linalg.norm(got - want))
    return num / den if den > 0 else num


def geom(spec: synth.LayerSpec) -> oracle.ConvGeom:
    return oracle.ConvGeom(spec.N, spec.C, spec.K, spec.H, spec.W, spec.R, spec.S,
                           spec.stride, spec.stride, spec.pad, spec.pad)


def tile_constant_activation(spec: synth.LayerSpec, seed: int = 0) -> np.ndarray:
    """An activation that is constant on every k x k tile (test input for the
    lossless special case): a coarse map written out over its tiles."""
    k = spec.k
    hp, wp = -(-spec.H // k), -(-spec.W // k)
    rng = np.random.Generator(np.random.Philox(key=1234 + seed))
    coarse = np.maximum(rng.standard_normal((spec.N, spec.C, hp, wp), dtype=np.float32), 0)
    coarse = synth.to_storage(coarse, spec.dtype)
    full = np.empty((spec.N, spec.C, spec.H, spec.W), dtype=np.float32)
    for h in range(spec.H):
        for w in range(spec.W):
            full[:, :, h, w] = coarse[:, :, h // k, w // k]
    return full
