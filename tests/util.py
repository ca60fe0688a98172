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


def check_bf16_output(got, want, what: str) -> None:
    """A bfloat16 output (Y, dX) against the oracle's fp64 values.  The device sums in float and
    rounds once, so it must land on the oracle value rounded to bfloat16 by the harness or on a
    neighbour of it: rel-L2 <= 4e-3 over the elements given and, for every single one,
    |got - want| <= 2^-7 |want| + 2^-7 rms(want) (one bfloat16 ulp is at most 2^-7 of the value;
    the rms term covers sums that cancel to near zero).  One wrong pixel fails the second part."""
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    wr = synth.round_to_bf16(want.astype(np.float32)).astype(np.float64)
    err = rel_l2(got, wr)
    assert err <= 4e-3, f"{what}: rel-L2 against the bf16-rounded oracle {err:.3e}"
    rms = float(np.sqrt(np.mean(wr * wr))) if wr.size else 0.0
    bound = 2.0 ** -7 * np.abs(wr) + 2.0 ** -7 * rms
    bad = np.abs(got - wr) > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} elements off by more than a bf16 ulp, first at "
                           f"{int(np.argmax(bad))}: got {got[np.argmax(bad)]!r} want {wr[np.argmax(bad)]!r}")
