"""Parity at the benchmark's full layer sizes, in the launch configuration the
benchmark times.  The oracle computes sampled outputs one by one at full
reduction length (every dW entry is an independent dot product over all
N*P*Q pixels), plus properties that hold at any size."""
import numpy as np
import pytest

import oracle
from paper_2409_11902_amd import synth
from util import geom, rel_l2

pytestmark = pytest.mark.gpu

N_SAMPLES = 4096


def _layers():
    cfg = synth.configs()
    picks = []
    picks += [("cfg2_resnet18_cifar", s) for s in cfg["cfg2_resnet18_cifar"]]
    picks += [("cfg5_deep_small_spatial", s) for s in cfg["cfg5_deep_small_spatial"]]
    picks += [("cfg4_resnet18_imagenet_k2", s) for s in cfg["cfg4_resnet18_imagenet_k2"]]
    k1, k4 = cfg["cfg4_resnet18_imagenet_k1"], cfg["cfg4_resnet18_imagenet_k4"]
    picks += [("cfg4_resnet18_imagenet_k1", k1[0]), ("cfg4_resnet18_imagenet_k1", k1[9]),
              ("cfg4_resnet18_imagenet_k4", k4[0]), ("cfg4_resnet18_imagenet_k4", k4[2]),
              ("cfg4_resnet18_imagenet_k4", k4[6]), ("cfg4_resnet18_imagenet_k4", k4[9])]
    c3 = {s.name: s for s in cfg["cfg3_resnet50_imagenet"]}
    for name in ("s1.b0.1x1_64_256@56", "s1.b1.1x1_256_64@56", "s2.b0.3x3s2_128_128@56",
                 "s2.b0.down1x1s2_256_512@56", "s3.b1.3x3_256_256@14", "s4.b0.1x1_512_2048@7",
                 "s4.b1.3x3_512_512@7"):
        picks.append(("cfg3_resnet50_imagenet", c3[name]))
    return picks


LAYERS = _layers()


@pytest.mark.parametrize("config,spec", LAYERS, ids=[f"{c.split('_')[0]}-{s.name}-k{s.k}" for c, s in LAYERS])
def test_dw_and_compress_at_full_size(config, spec):
    import torch
    from gpu_util import Guarded, download, tdtype, upload, workspace
    from paper_2409_11902_amd import binding as B

    print(f"layer {config} {spec.name} k={spec.k}", flush=True)
    t = synth.make_inputs(spec, config, tensors=("X", "dY"))
    d = B.desc_from_spec(spec)
    hp, wp, zb, xb = B.cac_pooled_shape(d)
    assert (hp, wp) == oracle.pooled_shape(spec.H, spec.W, spec.k, spec.k)
    X, dY = upload(t["X"], spec.dtype), upload(t["dY"], spec.dtype)
    Z = Guarded((spec.N, spec.C, hp, wp), tdtype(spec))
    dW = Guarded((spec.K, spec.C, spec.R, spec.S), torch.float32)
    B.cac_compress(d, X, Z.t)
    del X
    B.conv_bwd_weight_compressed(d, Z.t, dY, dW.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
    torch.cuda.synchronize()
    Z.check("Z")
    dW.check("dW")
    got_Z, got_dW = download(Z.t), download(dW.t)
    assert np.isfinite(got_dW).all()

    Xd = t["X"].astype(np.float64)
    Zo = oracle.avgpool(Xd, spec.k, spec.k)
    # compress: every element, official tolerance and at most one bf16 ulp
    assert rel_l2(got_Z, Zo) <= 2e-2
    Zr = synth.round_to_bf16(Zo.astype(np.float32)).astype(np.float64)
    assert float((np.abs(got_Z - Zr) > np.abs(Zr) * 2.0 ** -7).mean()) == 0.0
    # channel sums survive pooling when the tile divides the map
    if spec.H % spec.k == 0 and spec.W % spec.k == 0:
        np.testing.assert_allclose(got_Z.sum(axis=(2, 3)) * spec.k ** 2, Xd.sum(axis=(2, 3)), rtol=5e-3, atol=1e-2)
    del Xd

    g = geom(spec)
    rng = np.random.Generator(np.random.Philox(key=99))
    idx = np.unique(rng.integers(0, got_dW.size, N_SAMPLES))
    dYd = t["dY"].astype(np.float64)
    want = oracle.conv_dw_entries(g, oracle.inflate(Zo, spec.H, spec.W, spec.k, spec.k), dYd, idx)
    err = rel_l2(got_dW.ravel()[idx], want)
    assert err <= 2e-2, f"dW sample rel-L2 {err:.3e}"
    # tight: same storage rounding of Z on both sides leaves only summation order
    want_r = oracle.conv_dw_entries(g, oracle.inflate(Zr, spec.H, spec.W, spec.k, spec.k), dYd, idx)
    err = rel_l2(got_dW.ravel()[idx], want_r)
    assert err <= 2e-4, f"dW sample (tight) rel-L2 {err:.3e}"


def _step_layers():
    """The benchmark's default workload plus the layer kinds whose forward / data-gradient launch
    differs in kind: stride 2 (four parity classes), 1x1, rows of 28 and 14 pixels (no pooled map
    from the repack), a deep layer on 7x7 maps."""
    cfg = synth.configs()
    picks = [("cfg2_resnet18_cifar", s) for s in cfg["cfg2_resnet18_cifar"]]
    k2 = cfg["cfg4_resnet18_imagenet_k2"]
    picks += [("cfg4_resnet18_imagenet_k2", k2[i]) for i in (1, 2, 3, 6, 9)]
    picks += [("cfg5_deep_small_spatial", s) for s in cfg["cfg5_deep_small_spatial"]]
    # the bottleneck blocks' layer kinds: narrow and wide 1x1, a stride-2 1x1 shortcut, stride-2 3x3,
    # thousands of channels on 7x7 maps (odd planes: the element-wise repack)
    c3 = {s.name: s for s in cfg["cfg3_resnet50_imagenet"]}
    for name in ("s1.b0.1x1_64_256@56", "s1.b1.1x1_256_64@56", "s2.b0.3x3s2_128_128@56", "s3.b0.down1x1s2_512_1024@28",
                 "s3.b1.1x1_1024_256@14", "s4.b0.1x1_512_2048@7", "s4.b1.1x1_2048_512@7"):
        picks.append(("cfg3_resnet50_imagenet", c3[name]))
    return picks


STEP_LAYERS = _step_layers()


@pytest.mark.parametrize("config,spec", STEP_LAYERS, ids=[f"{c.split('_')[0]}-{s.name}" for c, s in STEP_LAYERS])
def test_forward_and_data_gradient_at_full_size(config, spec):
    """Y (with bias), the Z the forward call leaves, and dX at the benchmark's sizes: sampled
    outputs against the oracle's entry-by-entry sums, Z against the stand-alone kernel bit for bit."""
    import torch
    from gpu_util import Guarded, download, tdtype, upload, workspace
    from paper_2409_11902_amd import binding as B

    print(f"layer {config} {spec.name}", flush=True)
    t = synth.make_inputs(spec, config)
    rng = np.random.Generator(np.random.Philox(key=7))
    t["b"] = synth.to_storage(0.1 * rng.standard_normal((spec.K,), dtype=np.float32), spec.dtype)  # (the recipe's bias is zero)
    d = B.desc_from_spec(spec)
    g = geom(spec)
    hp, wp, zb, xb = B.cac_pooled_shape(d)
    X, Wt, b, dY = (upload(t[k], spec.dtype) for k in ("X", "W", "b", "dY"))
    Y = Guarded((spec.N, spec.K, g.P, g.Q), tdtype(spec))
    Z = Guarded((spec.N, spec.C, hp, wp), tdtype(spec))
    dX = Guarded((spec.N, spec.C, spec.H, spec.W), tdtype(spec))
    Z2 = torch.empty_like(Z.t)
    B.conv_fwd_and_compress(d, X, Wt, b, Y.t, Z.t, workspace(d, B.OP_FWD_AND_COMPRESS))
    B.conv_bwd_data(d, Wt, dY, dX.t, workspace(d, B.OP_BWD_DATA))
    B.cac_compress(d, X, Z2)
    torch.cuda.synchronize()
    for name, buf in (("Y", Y), ("Z", Z), ("dX", dX)):
        buf.check(name)
    assert torch.equal(Z.t.view(torch.int16), Z2.view(torch.int16))
    got_Y, got_dX = download(Y.t), download(dX.t)
    assert np.isfinite(got_Y).all() and np.isfinite(got_dX).all()
    Xd, Wd, bd, dYd = (t[k].astype(np.float64) for k in ("X", "W", "b", "dY"))
    idx = np.unique(rng.integers(0, got_Y.size, N_SAMPLES))
    err = rel_l2(got_Y.ravel()[idx], oracle.conv_fwd_entries(g, Xd, Wd, bd, idx))
    assert err <= 2e-2, f"Y sample rel-L2 {err:.3e}"
    idx = np.unique(rng.integers(0, got_dX.size, N_SAMPLES))
    err = rel_l2(got_dX.ravel()[idx], oracle.conv_dx_entries(g, Wd, dYd, idx))
    assert err <= 2e-2, f"dX sample rel-L2 {err:.3e}"
