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


def _workload_like_specs(count, seed):
    """The workloads' layer shapes with smaller batches: long enough for several chunks per
    workgroup, several pixel slices and both workgroup shapes of the weight-gradient kernel."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    out = []
    while len(out) < count:
        R = int(rng.choice([1, 3, 3, 3]))
        stride = int(rng.choice([1, 1, 1, 2]))
        H = int(rng.choice([4, 7, 8, 14, 16, 28, 32, 56]))
        N = int(rng.choice([8, 12, 16, 24, 32]))
        C = int(rng.choice([64, 128, 256]))
        K = int(rng.choice([64, 128, 256]))
        k = int(rng.choice([1, 2, 2, 2, 4]))
        if N * C * K * H * H * R * R > 2.5e9 or N * C * H * H > 4e6:
            continue
        out.append(synth.LayerSpec(f"wl{len(out)} N{N} C{C} K{K} {H}x{H} R{R} s{stride} k{k}",
                                   N, C, K, H, H, R, R, stride, R // 2, k, synth.BF16))
    return out


def _few_tap_specs(count, seed):
    """1x1 and stride-2 layers with 96 to 320 channels on even and odd maps: launches with one, two or four
    taps, which stage several 32-channel groups per pass (the last group often only partly real)
    and, for a 1x1 stride-2 forward pass on rows of a multiple of 8 pixels, a decimated input copy."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    out = []
    while len(out) < count:
        R = int(rng.choice([1, 1, 3]))
        stride = int(rng.choice([1, 2, 2])) if R == 1 else 2
        H = int(rng.choice([4, 6, 7, 8, 12, 14, 16, 24, 28]))
        W = H if rng.random() < 0.5 else int(rng.choice([8, 16, 24, 12, 14, 6]))
        N = int(rng.integers(1, 12))
        C = int(rng.choice([96, 100, 112, 128, 160, 200, 256, 320]))
        K = int(rng.choice([32, 64, 96, 112, 128, 200, 256]))
        k = int(rng.choice([1, 2, 2, 2, 4]))
        if N * C * K * H * W * R * R > 1.5e9:
            continue
        out.append(synth.LayerSpec(f"ft{len(out)} N{N} C{C} K{K} {H}x{W} R{R} s{stride} k{k}",
                                   N, C, K, H, W, R, R, stride, 0 if R == 1 else 1, k, synth.BF16))
    return out


SPECS = (_random_specs(48, seed=20240911) + _mfma_leaning_specs(40, seed=7) + _workload_like_specs(24, seed=3) +
         _few_tap_specs(32, seed=5))


@pytest.mark.parametrize("spec", SPECS, ids=[s.name for s in SPECS])
def test_random_shape(spec):
    from gpu_util import run_step
    t = synth.make_inputs(spec, "random_shapes")
    _check_step(spec, t, run_step(spec, t))


def _anisotropic_cases(count, seed):
    """Descriptors the square LayerSpec shorthand cannot express: R != S, strides, paddings and
    pooling factors that differ per axis, with and without bias."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    out = []
    while len(out) < count:
        R, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        ph, pw = int(rng.integers(0, R)), int(rng.integers(0, S))
        H, W = int(rng.integers(1, 25)), int(rng.integers(1, 25))
        if H + 2 * ph < R or W + 2 * pw < S:
            continue
        kh, kw = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4, 8]))
        N, C, K = int(rng.integers(1, 6)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        dtype = synth.BF16 if rng.random() < 0.5 else synth.F32
        out.append(dict(N=N, C=C, K=K, H=H, W=W, R=R, S=S, sh=sh, sw=sw, ph=ph, pw=pw, kh=kh, kw=kw, dtype=dtype,
                        bias=bool(rng.random() < 0.7), seed=int(rng.integers(1 << 30))))
    return out


ANISO = _anisotropic_cases(40, seed=99)


@pytest.mark.parametrize("c", ANISO, ids=[f"an{i} " + " ".join(f"{k}{v}" for k, v in c.items() if k != "seed") for i, c in enumerate(ANISO)])
def test_random_anisotropic_descriptor(c):
    import torch
    import oracle
    from gpu_util import Guarded, upload, download, workspace
    from paper_2409_11902_amd import binding as B
    from test_gpu_parity import TOL
    from util import rel_l2
    g = oracle.ConvGeom(c["N"], c["C"], c["K"], c["H"], c["W"], c["R"], c["S"], c["sh"], c["sw"], c["ph"], c["pw"])
    rng = np.random.Generator(np.random.Philox(key=c["seed"]))
    dt = c["dtype"]
    t = dict(X=synth.to_storage(np.maximum(rng.standard_normal((c["N"], c["C"], c["H"], c["W"]), dtype=np.float32), 0), dt),
             W=synth.to_storage(0.2 * rng.standard_normal((c["K"], c["C"], c["R"], c["S"]), dtype=np.float32), dt),
             b=synth.to_storage(0.1 * rng.standard_normal((c["K"],), dtype=np.float32), dt),
             dY=synth.to_storage(rng.standard_normal((c["N"], c["K"], g.P, g.Q), dtype=np.float32), dt))
    d = B.make_desc(c["N"], c["C"], c["K"], c["H"], c["W"], c["R"], c["S"], c["sh"], c["sw"], c["ph"], c["pw"], c["kh"], c["kw"],
                    dtype=B.F32 if dt == synth.F32 else B.BF16, has_bias=int(c["bias"]))
    hp, wp, zb, xb = B.cac_pooled_shape(d)
    assert (hp, wp) == oracle.pooled_shape(c["H"], c["W"], c["kh"], c["kw"]) and B.cac_out_shape(d) == (g.P, g.Q)
    td = torch.float32 if dt == synth.F32 else torch.bfloat16
    X, Wt, b, dY = (upload(t[k], dt) for k in ("X", "W", "b", "dY"))
    Y, Z = Guarded((c["N"], c["K"], g.P, g.Q), td), Guarded((c["N"], c["C"], hp, wp), td)
    dW, dX = Guarded((c["K"], c["C"], c["R"], c["S"]), torch.float32), Guarded((c["N"], c["C"], c["H"], c["W"]), td)
    db = Guarded((c["K"],), torch.float32)
    B.conv_fwd_and_compress(d, X, Wt, b if c["bias"] else None, Y.t, Z.t, workspace(d, B.OP_FWD_AND_COMPRESS))
    B.conv_bwd_weight_compressed(d, Z.t, dY, dW.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
    B.conv_bwd_data(d, Wt, dY, dX.t, workspace(d, B.OP_BWD_DATA))
    B.conv_bwd_bias(d, dY, db.t)
    torch.cuda.synchronize()
    f = {k: v.astype(np.float64) for k, v in t.items()}
    Zo = oracle.avgpool(f["X"], c["kh"], c["kw"])
    want = dict(Y=oracle.conv_fwd(g, f["X"], f["W"], f["b"] if c["bias"] else None), Z=Zo,
                dW=oracle.conv_dw(g, oracle.inflate(Zo, c["H"], c["W"], c["kh"], c["kw"]), f["dY"]),
                dX=oracle.conv_dx(g, f["W"], f["dY"]), db=oracle.bias_grad(f["dY"]))
    got = dict(Y=Y, Z=Z, dW=dW, dX=dX, db=db)
    for name in want:
        got[name].check(name)
        w = want[name]
        e = rel_l2(download(got[name].t), w) if np.abs(w).max() > 0 else np.abs(download(got[name].t)).max()
        assert e <= TOL[dt], f"{name}: {e:.3e}"
