"""Parity at the benchmark's full layer sizes, in the launch configuration the
benchmark times: EVERY layer of the bfloat16 workloads (the CIFAR-shaped list,
the bottleneck list, the pooling-factor sweep at k = 1, 2, 4 and the deep
small-spatial pair).  The oracle computes sampled outputs one by one at full
reduction length (every dW entry is an independent dot product over all N*P*Q
pixels, every Y / dX element one over the filter), plus properties that hold at
any size.  The combined backward call, which is what the benchmark's step calls,
has to reproduce the separate calls bit for bit at these sizes."""
import numpy as np
import pytest

import oracle
from paper_2409_11902_amd import synth
from util import check_bf16_output, geom, rel_l2

pytestmark = pytest.mark.gpu

N_SAMPLES = 4096
WORKLOADS = ("cfg2_resnet18_cifar", "cfg3_resnet50_imagenet", "cfg4_resnet18_imagenet_k1",
             "cfg4_resnet18_imagenet_k2", "cfg4_resnet18_imagenet_k4", "cfg5_deep_small_spatial")


def _layers():
    cfg = synth.configs()
    return [(w, s) for w in WORKLOADS for s in cfg[w]]


LAYERS = _layers()


def _dw_sample(spec, rng):
    """Flat indices into dW: a uniform sample plus, for every filter tap, the entries on the
    borders of the kernels' 32-, 64- and 128-wide channel tiles."""
    total = spec.K * spec.C * spec.R * spec.S
    edges = (0, 31, 32, 63, 64, 127, 128)
    os_ = sorted({e for e in edges if e < spec.K} | {spec.K - 1})
    cs_ = sorted({e for e in edges if e < spec.C} | {spec.C - 1})
    T = spec.R * spec.S
    forced = [(o * spec.C + c) * T + t for o in os_ for c in cs_ for t in range(T)]
    return np.unique(np.concatenate([rng.integers(0, total, N_SAMPLES), np.asarray(forced, dtype=np.int64)]))


@pytest.mark.parametrize("config,spec", LAYERS, ids=[f"{c.split('_')[0]}-{s.name}-k{s.k}" for c, s in LAYERS])
def test_layer_at_full_size(config, spec):
    import torch
    from gpu_util import Guarded, download, tdtype, upload, workspace
    from paper_2409_11902_amd import binding as B

    print(f"layer {config} {spec.name} k={spec.k}", flush=True)
    t = synth.make_inputs(spec, config)
    rng = np.random.Generator(np.random.Philox(key=99))
    t["b"] = synth.to_storage(0.1 * rng.standard_normal((spec.K,), dtype=np.float32), spec.dtype)  # (the recipe's bias is zero)
    d = B.desc_from_spec(spec)
    g = geom(spec)
    hp, wp, zb, xb = B.cac_pooled_shape(d)
    assert (hp, wp) == oracle.pooled_shape(spec.H, spec.W, spec.k, spec.k)
    td = tdtype(spec)
    X, Wt, b, dY = (upload(t[k], spec.dtype) for k in ("X", "W", "b", "dY"))
    Y = Guarded((spec.N, spec.K, g.P, g.Q), td)
    Z = Guarded((spec.N, spec.C, hp, wp), td)
    Z2 = Guarded((spec.N, spec.C, hp, wp), td)
    dW, dW2 = Guarded((spec.K, spec.C, spec.R, spec.S), torch.float32), Guarded((spec.K, spec.C, spec.R, spec.S), torch.float32)
    dX, dX2 = Guarded((spec.N, spec.C, spec.H, spec.W), td), Guarded((spec.N, spec.C, spec.H, spec.W), td)
    B.conv_fwd_and_compress(d, X, Wt, b, Y.t, Z.t, workspace(d, B.OP_FWD_AND_COMPRESS))
    B.cac_compress(d, X, Z2.t)
    del X
    B.conv_bwd_weight_compressed(d, Z.t, dY, dW.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
    B.conv_bwd_data(d, Wt, dY, dX.t, workspace(d, B.OP_BWD_DATA))
    ws = workspace(d, B.OP_BWD_WEIGHT_AND_DATA)
    if ws is not None:
        ws.fill_(0xFF)   # stale contents must not matter (all-ones floats are NaN)
    B.conv_bwd_weight_and_data(d, Z.t, Wt, dY, dW2.t, dX2.t, ws)
    torch.cuda.synchronize()
    for name, buf in (("Y", Y), ("Z", Z), ("Z2", Z2), ("dW", dW), ("dX", dX), ("dW2", dW2), ("dX2", dX2)):
        buf.check(name)
    # the forward call's Z is the stand-alone kernel's, the combined backward call's results are
    # the separate calls', bit for bit
    assert torch.equal(Z.t.view(torch.int16), Z2.t.view(torch.int16)), "Z of the forward call"
    assert torch.equal(dW.t, dW2.t), "dW of the combined call"
    assert torch.equal(dX.t.view(torch.int16), dX2.t.view(torch.int16)), "dX of the combined call"
    got_Z, got_dW, got_Y, got_dX = download(Z.t), download(dW.t), download(Y.t), download(dX.t)
    assert np.isfinite(got_dW).all() and np.isfinite(got_Y).all() and np.isfinite(got_dX).all()

    Xd, Wd, bd, dYd = (t[k].astype(np.float64) for k in ("X", "W", "b", "dY"))
    # ---- compress: every element, official tolerance and at most one bf16 ulp
    Zo = oracle.avgpool(Xd, spec.k, spec.k)
    assert rel_l2(got_Z, Zo) <= 2e-2
    Zr = synth.round_to_bf16(Zo.astype(np.float32)).astype(np.float64)
    assert float((np.abs(got_Z - Zr) > np.abs(Zr) * 2.0 ** -7).mean()) == 0.0
    if spec.k == 1:
        assert np.array_equal(got_Z, Xd)   # pooling factor 1 keeps X itself
    # channel sums survive pooling when the tile divides the map
    if spec.H % spec.k == 0 and spec.W % spec.k == 0:
        np.testing.assert_allclose(got_Z.sum(axis=(2, 3)) * spec.k ** 2, Xd.sum(axis=(2, 3)), rtol=5e-3, atol=1e-2)

    # ---- Y and dX: sampled elements, each within a bf16 ulp of the rounded oracle value
    idx = np.unique(rng.integers(0, got_Y.size, N_SAMPLES))
    want = oracle.conv_fwd_entries(g, Xd, Wd, bd, idx)
    assert rel_l2(got_Y.ravel()[idx], want) <= 2e-2
    check_bf16_output(got_Y.ravel()[idx], want, "Y sample")
    idx = np.unique(rng.integers(0, got_dX.size, N_SAMPLES))
    want = oracle.conv_dx_entries(g, Wd, dYd, idx)
    if np.abs(want).max() > 0:
        assert rel_l2(got_dX.ravel()[idx], want) <= 2e-2
    check_bf16_output(got_dX.ravel()[idx], want, "dX sample")
    del Xd

    # ---- dW: the sample with the tile borders forced in
    idx = _dw_sample(spec, rng)
    want = oracle.conv_dw_entries(g, oracle.inflate(Zo, spec.H, spec.W, spec.k, spec.k), dYd, idx)
    err = rel_l2(got_dW.ravel()[idx], want)
    assert err <= 2e-2, f"dW sample rel-L2 {err:.3e}"
    # tight: same storage rounding of Z on both sides leaves only summation order
    want_r = oracle.conv_dw_entries(g, oracle.inflate(Zr, spec.H, spec.W, spec.k, spec.k), dYd, idx)
    err = rel_l2(got_dW.ravel()[idx], want_r)
    assert err <= 2e-4, f"dW sample (tight) rel-L2 {err:.3e}"
    # and no single entry off: float accumulation of N*P*Q terms stays far below this
    scale = float(np.sqrt(np.mean(want_r * want_r)))
    worst = float(np.abs(got_dW.ravel()[idx] - want_r).max())
    assert worst <= 2e-3 * scale, f"dW worst sampled entry off by {worst:.3e} (rms {scale:.3e})"
