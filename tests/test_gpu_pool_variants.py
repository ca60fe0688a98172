"""GPU parity of the pooling variants: compression with the tile maximum (the compression section
names other forms of pooling as feasible; the maximum is the reading this library offers) and mean
tiles whose sides are not powers of two.  A maximum is one of the tile's own elements, so Z has to
agree with the oracle bit for bit in either storage type; everything downstream of Z is checked as
in the other parity tests."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_2409_11902_amd import binding as B
from paper_2409_11902_amd import synth
from test_gpu_parity import TOL
from util import rel_l2

pytestmark = pytest.mark.gpu


def _run(c, pool_mode):
    from gpu_util import Guarded, upload, download, workspace
    N, C, K, H, W, R, stride, pad, kh, kw, dt = c
    g = oracle.ConvGeom(N, C, K, H, W, R, R, stride, stride, pad, pad)
    rng = np.random.Generator(np.random.Philox(key=hash((N, C, K, H, W, R, kh, kw)) & 0xffffffff))
    # shifted below zero: a zero standing in for a missing element of a ragged tile would win the maximum
    X = synth.to_storage(rng.standard_normal((N, C, H, W), dtype=np.float32) - 0.75, dt)
    Wt = synth.to_storage(0.2 * rng.standard_normal((K, C, R, R), dtype=np.float32), dt)
    dY = synth.to_storage(rng.standard_normal((N, K, g.P, g.Q), dtype=np.float32), dt)
    d = B.make_desc(N, C, K, H, W, R, R, stride, stride, pad, pad, kh, kw,
                    dtype=B.F32 if dt == synth.F32 else B.BF16, has_bias=0, pool_mode=pool_mode)
    hp, wp, zb, xb = B.cac_pooled_shape(d)
    td = torch.float32 if dt == synth.F32 else torch.bfloat16
    Xd, Wd, dYd = upload(X, dt), upload(Wt, dt), upload(dY, dt)
    Y, Z, Z2 = Guarded((N, K, g.P, g.Q), td), Guarded((N, C, hp, wp), td), Guarded((N, C, hp, wp), td)
    dW, dX = Guarded((K, C, R, R), torch.float32), Guarded((N, C, H, W), td)
    B.conv_fwd_and_compress(d, Xd, Wd, None, Y.t, Z.t, workspace(d, B.OP_FWD_AND_COMPRESS))
    B.cac_compress(d, Xd, Z2.t)
    B.conv_bwd_weight_compressed(d, Z.t, dYd, dW.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
    B.conv_bwd_data(d, Wd, dYd, dX.t, workspace(d, B.OP_BWD_DATA))
    torch.cuda.synchronize()
    for name, buf in (("Y", Y), ("Z", Z), ("Z2", Z2), ("dW", dW), ("dX", dX)):
        buf.check(name)
    f = dict(X=X.astype(np.float64), W=Wt.astype(np.float64), dY=dY.astype(np.float64))
    return g, f, {k: download(v.t) for k, v in dict(Y=Y, Z=Z, Z2=Z2, dW=dW, dX=dX).items()}


# N, C, K, H, W, R, stride, pad, kh, kw, dtype
MAX_CASES = [
    (3, 5, 6, 7, 7, 3, 1, 1, 2, 2, synth.BF16),        # ragged tiles, odd rows
    (2, 8, 4, 14, 14, 3, 1, 1, 4, 4, synth.BF16),
    (4, 32, 32, 16, 16, 3, 1, 1, 2, 2, synth.BF16),    # a shape whose mean is formed inside the forward call
    (8, 64, 64, 8, 8, 3, 1, 1, 2, 2, synth.BF16),
    (2, 16, 16, 12, 20, 3, 1, 1, 2, 4, synth.BF16),
    (2, 6, 5, 9, 11, 3, 2, 1, 3, 3, synth.BF16),       # plain kernels
    (2, 4, 4, 10, 10, 1, 1, 0, 8, 8, synth.BF16),
    (2, 3, 3, 3, 3, 3, 1, 1, 4, 4, synth.BF16),        # tile larger than the map
    (3, 50, 8, 14, 14, 3, 1, 1, 2, 2, synth.BF16),     # narrow rows: a thread per row pair, last wave not full
    (2, 9, 8, 6, 10, 3, 1, 1, 2, 2, synth.BF16),
    (1, 1, 1, 1, 1, 1, 1, 0, 2, 2, synth.BF16),
    (3, 5, 6, 7, 9, 3, 1, 1, 2, 2, synth.F32),
    (2, 8, 4, 13, 16, 3, 1, 1, 4, 2, synth.F32),
    (2, 4, 4, 10, 7, 3, 1, 1, 3, 2, synth.F32),
    (2, 4, 4, 9, 9, 3, 1, 1, 1, 1, synth.BF16),        # k = 1: the maximum of one element
]


@pytest.mark.parametrize("c", MAX_CASES, ids=[" ".join(map(str, c)) for c in MAX_CASES])
def test_max_pool_compression(c):
    N, C, K, H, W, R, stride, pad, kh, kw, dt = c
    g, f, got = _run(c, B.POOL_MAX)
    Zo = oracle.maxpool(f["X"], kh, kw)
    assert np.array_equal(got["Z"].astype(np.float64), Zo), "Z from the forward call"
    assert np.array_equal(got["Z2"].astype(np.float64), Zo), "Z from the compress call"
    want = dict(Y=oracle.conv_fwd(g, f["X"], f["W"], None), dX=oracle.conv_dx(g, f["W"], f["dY"]),
                dW=oracle.conv_dw(g, oracle.inflate(Zo, H, W, kh, kw), f["dY"]))
    for name, w in want.items():
        e = rel_l2(got[name], w)
        assert e <= TOL[dt], f"{name}: {e:.3e}"
    if kh * kw > 1 and H * W > 1:
        # the mean of the same input gives another Z: the mode reaches the kernels
        assert not np.array_equal(Zo, oracle.avgpool(f["X"], kh, kw))


MEAN_CASES = [
    (2, 6, 5, 9, 11, 3, 2, 1, 3, 3, synth.BF16),
    (3, 16, 16, 12, 12, 3, 1, 1, 3, 3, synth.BF16),
    (2, 32, 32, 14, 14, 3, 1, 1, 3, 2, synth.BF16),
    (2, 8, 8, 10, 7, 1, 1, 0, 5, 3, synth.BF16),
    (2, 4, 4, 10, 7, 3, 1, 1, 3, 1, synth.F32),
    (2, 4, 6, 15, 15, 3, 1, 1, 3, 3, synth.F32),
    (1, 3, 3, 8, 8, 3, 1, 1, 6, 7, synth.F32),
]


@pytest.mark.parametrize("c", MEAN_CASES, ids=[" ".join(map(str, c)) for c in MEAN_CASES])
def test_mean_tiles_that_are_not_powers_of_two(c):
    N, C, K, H, W, R, stride, pad, kh, kw, dt = c
    g, f, got = _run(c, B.POOL_MEAN)
    Zo = oracle.avgpool(f["X"], kh, kw)
    want = dict(Y=oracle.conv_fwd(g, f["X"], f["W"], None), dX=oracle.conv_dx(g, f["W"], f["dY"]), Z=Zo, Z2=Zo,
                dW=oracle.conv_dw(g, oracle.inflate(Zo, H, W, kh, kw), f["dY"]))
    for name, w in want.items():
        e = rel_l2(got[name], w)
        assert e <= TOL[dt], f"{name}: {e:.3e}"


# Anisotropic and 8-wide tiles on shapes the MFMA weight-gradient kernel takes (3x3 pad 1 at
# stride 1 and 2, 1x1 stride 2; channels >= 32 with an edge block; odd W, so the last tile of a
# row is ragged; enough images for several chunks and pixel slices).
# N, C, K, H, W, R, stride, pad, kh, kw, dtype
MFMA_TILE_CASES = [
    (12, 40, 72, 16, 17, 3, 1, 1, 8, 8, synth.BF16),
    (12, 64, 33, 16, 19, 3, 1, 1, 2, 8, synth.BF16),
    (10, 40, 64, 24, 15, 3, 1, 1, 8, 1, synth.BF16),
    (10, 32, 72, 14, 21, 3, 1, 1, 1, 4, synth.BF16),
    (12, 72, 40, 12, 13, 3, 1, 1, 4, 2, synth.BF16),
    (12, 40, 72, 16, 17, 3, 2, 1, 8, 8, synth.BF16),
    (12, 64, 33, 16, 19, 3, 2, 1, 2, 8, synth.BF16),
    (10, 40, 64, 24, 15, 3, 2, 1, 8, 1, synth.BF16),
    (10, 32, 72, 14, 21, 3, 2, 1, 1, 4, synth.BF16),
    (12, 72, 40, 12, 13, 3, 2, 1, 4, 2, synth.BF16),
    (12, 40, 72, 16, 17, 1, 2, 0, 8, 8, synth.BF16),
    (12, 64, 33, 16, 19, 1, 2, 0, 2, 8, synth.BF16),
    (10, 72, 64, 24, 15, 1, 2, 0, 8, 1, synth.BF16),
    (10, 32, 72, 14, 21, 1, 2, 0, 1, 4, synth.BF16),
    (12, 72, 40, 12, 13, 1, 2, 0, 4, 2, synth.BF16),
]


@pytest.mark.parametrize("c", MFMA_TILE_CASES, ids=[" ".join(map(str, c)) for c in MFMA_TILE_CASES])
def test_anisotropic_and_wide_tiles_on_the_mfma_weight_gradient(c):
    N, C, K, H, W, R, stride, pad, kh, kw, dt = c
    d = B.make_desc(N, C, K, H, W, R, R, stride, stride, pad, pad, kh, kw, dtype=B.BF16, has_bias=0)
    plan = B.cac_describe_plan(d, B.OP_BWD_WEIGHT_COMPRESSED)
    assert plan.startswith("dw_mfma"), plan   # the case is here for that kernel's staging branches
    g, f, got = _run(c, B.POOL_MEAN)
    Zo = oracle.avgpool(f["X"], kh, kw)
    Zr = synth.round_to_bf16(Zo.astype(np.float32)).astype(np.float64)
    assert float((np.abs(got["Z"] - Zr) > np.abs(Zr) * 2.0 ** -7).mean()) == 0.0
    want = oracle.conv_dw(g, oracle.inflate(Zr, H, W, kh, kw), f["dY"])
    e = rel_l2(got["dW"], want)
    assert e <= 2e-4, f"dW (tight): {e:.3e}"
