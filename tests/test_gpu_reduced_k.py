"""The weight gradient in its reduced-K form (dw_algo = CAC_DW_REDUCED_K) against the oracle.

It computes the same real number as the inflating kernel -- the pixel sum regrouped by pooling
tile -- so the official bound is the same 2e-2 against the oracle's dW from the inflated fp64 Z.
The tight bound isolates indexing from storage rounding as the other parity tests do: this form
keeps the tile sums of dY in bfloat16, so the oracle's regrouped form is run from Z and tile sums
rounded to bfloat16 by the harness, which leaves only float summation order (2e-4)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_2409_11902_amd import binding as B
from paper_2409_11902_amd import synth
from util import geom, rel_l2

pytestmark = pytest.mark.gpu


def _run_and_check(spec, config, full_check=True):
    from gpu_util import Guarded, download, tdtype, upload, workspace
    d = B.desc_from_spec(spec, dw_algo=B.DW_REDUCED_K)
    plan = B.cac_describe_plan(d, B.OP_BWD_WEIGHT_COMPRESSED)
    assert plan.startswith("dw_rk"), plan
    print(f"{spec.name}: {plan}", flush=True)
    t = synth.make_inputs(spec, config, tensors=("X", "dY"))
    hp, wp, _, _ = B.cac_pooled_shape(d)
    X, dY = upload(t["X"], spec.dtype), upload(t["dY"], spec.dtype)
    Z = torch.empty((spec.N, spec.C, hp, wp), dtype=tdtype(spec), device="cuda:0")
    B.cac_compress(d, X, Z)
    dW = Guarded((spec.K, spec.C, 3, 3), torch.float32)
    dW2 = Guarded((spec.K, spec.C, 3, 3), torch.float32)
    ws = workspace(d, B.OP_BWD_WEIGHT_COMPRESSED)
    if ws is not None:
        ws.fill_(0xFF)
    B.conv_bwd_weight_compressed(d, Z, dY, dW.t, ws)
    B.conv_bwd_weight_compressed(d, Z, dY, dW2.t, ws)      # again over its own leftovers: reproducible bit for bit
    torch.cuda.synchronize()
    dW.check("dW")
    dW2.check("dW2")
    assert torch.equal(dW.t, dW2.t)
    got = download(dW.t)
    assert np.isfinite(got).all()
    assert B.dw_rk_executed_flops(d) == 2 * 9 * spec.K * spec.C * spec.N * hp * wp
    g = geom(spec)
    Zg = download(Z)                                        # the stored Z (its own parity is tested elsewhere)
    Xd, dYd = t["X"].astype(np.float64), t["dY"].astype(np.float64)
    Zo = oracle.avgpool(Xd, 2, 2)
    Zr = synth.round_to_bf16(Zo.astype(np.float32)).astype(np.float64)
    assert float((np.abs(Zg - Zr) > np.abs(Zr) * 2.0 ** -7).mean()) == 0.0
    # tight: the oracle's regrouped form on the same storage roundings (Z and the tile sums in bfloat16)
    want_t = oracle.conv_dw_from_tile_sums(g, Zg, dYd, 2, 2, round_sums=lambda T: synth.round_to_bf16(T.astype(np.float32)))
    err = rel_l2(got, want_t)
    assert err <= 2e-4, f"{spec.name} dW (tight) rel-L2 {err:.3e}"
    scale = float(np.sqrt(np.mean(want_t * want_t)))
    worst = float(np.abs(got - want_t).max())
    assert worst <= 2e-3 * scale, f"{spec.name}: worst entry off by {worst:.3e} (rms {scale:.3e})"
    # official: the method's dW (inflated fp64 Z), regrouped form = inflated form (pinned on the CPU)
    want = oracle.conv_dw_from_tile_sums(g, Zo, dYd, 2, 2)
    if full_check and spec.N * spec.P * spec.Q * spec.K * spec.C <= 3e8:
        np.testing.assert_allclose(want, oracle.conv_dw(g, oracle.inflate(Zo, spec.H, spec.W, 2, 2), dYd), rtol=1e-10, atol=1e-10)
    err = rel_l2(got, want)
    assert err <= 2e-2, f"{spec.name} dW rel-L2 {err:.3e}"
    return got


# name, N, C, K, H, W: several channel tiles with edge blocks, odd batch sizes (a last unit or chunk
# that is only partly there), one and two blocks per tile-sum row, row blocks within an image
SMALL = [
    ("rk 14x14", 5, 128, 32, 14, 14),
    ("rk 14x14 edge channels", 7, 200, 72, 14, 14),
    ("rk 8x8", 9, 160, 40, 8, 8),
    ("rk 4x4", 11, 130, 33, 4, 4),
    ("rk 2x2", 6, 96, 16, 2, 2),
    ("rk 16x16", 3, 128, 64, 16, 16),
    ("rk 28x28", 2, 144, 48, 28, 28),
    ("rk 12x20", 4, 128, 32, 12, 20),
    ("rk 6x30", 3, 96, 32, 6, 30),
    ("rk 10x10 many images", 37, 128, 32, 10, 10),
]


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_reduced_k_small_shapes(case):
    name, N, C, K, H, W = case
    spec = synth.LayerSpec(name, N, C, K, H, W, 3, 3, 1, 1, 2, synth.BF16)
    _run_and_check(spec, "reduced_k")


def test_reduced_k_falls_back_where_it_has_no_kernel():
    """Odd maps, other strides, filters and tiles run on the inflating kernel under the same flag."""
    for spec in (synth.LayerSpec("odd", 2, 128, 32, 7, 7, 3, 3, 1, 1, 2, synth.BF16),
                 synth.LayerSpec("s2", 2, 128, 32, 14, 14, 3, 3, 2, 1, 2, synth.BF16),
                 synth.LayerSpec("k4", 2, 128, 32, 16, 16, 3, 3, 1, 1, 4, synth.BF16),
                 synth.LayerSpec("1x1", 2, 128, 32, 14, 14, 1, 1, 1, 0, 2, synth.BF16)):
        d = B.desc_from_spec(spec, dw_algo=B.DW_REDUCED_K)
        assert not B.cac_describe_plan(d, B.OP_BWD_WEIGHT_COMPRESSED).startswith("dw_rk")
        assert B.dw_rk_executed_flops(d) == spec.dw_flops


def _full_layers():
    cfg = synth.configs()
    out = []
    for w in ("cfg5_deep_small_spatial", "cfg2_resnet18_cifar", "cfg3_resnet50_imagenet", "cfg4_resnet18_imagenet_k2"):
        for s in cfg[w]:
            d = B.desc_from_spec(s, dw_algo=B.DW_REDUCED_K)
            if B.cac_describe_plan(d, B.OP_BWD_WEIGHT_COMPRESSED).startswith("dw_rk"):
                out.append((w, s))
    return out


FULL = _full_layers()


@pytest.mark.parametrize("config,spec", FULL, ids=[f"{c.split('_')[0]}-{s.name}" for c, s in FULL])
def test_reduced_k_at_full_size(config, spec):
    _run_and_check(spec, config, full_check=False)


def test_reduced_k_in_the_combined_backward_call():
    """conv_bwd_weight_and_data with the reduced-K flag: dW identical to the separate call's bit for
    bit (its slice sum then runs in the data gradient's repack launch), dX untouched by the flag."""
    from gpu_util import Guarded, tdtype, upload, workspace
    spec = synth.LayerSpec("rk both", 12, 128, 64, 14, 14, 3, 3, 1, 1, 2, synth.BF16)
    t = synth.make_inputs(spec, "reduced_k")
    d, d0 = B.desc_from_spec(spec, dw_algo=B.DW_REDUCED_K), B.desc_from_spec(spec)
    X, Wt, dY = (upload(t[k], spec.dtype) for k in ("X", "W", "dY"))
    Z = torch.empty((spec.N, spec.C, 7, 7), dtype=torch.bfloat16, device="cuda:0")
    B.cac_compress(d, X, Z)
    dW1, dW2 = Guarded((64, 128, 3, 3), torch.float32), Guarded((64, 128, 3, 3), torch.float32)
    dX1, dX2 = Guarded((12, 128, 14, 14), torch.bfloat16), Guarded((12, 128, 14, 14), torch.bfloat16)
    B.conv_bwd_weight_compressed(d, Z, dY, dW1.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
    B.conv_bwd_data(d0, Wt, dY, dX1.t, workspace(d0, B.OP_BWD_DATA))
    B.conv_bwd_weight_and_data(d, Z, Wt, dY, dW2.t, dX2.t, workspace(d, B.OP_BWD_WEIGHT_AND_DATA))
    torch.cuda.synchronize()
    for b in (dW1, dW2, dX1, dX2):
        b.check("rk both")
    assert torch.equal(dW1.t, dW2.t)
    assert torch.equal(dX1.t.view(torch.int16), dX2.t.view(torch.int16))


def test_auto_runs_the_kernel_its_plan_names():
    """dw_algo = AUTO: bit for bit the reduced-K result on a layer large enough for it, the
    inflating kernel's on a small one."""
    from gpu_util import Guarded, upload, workspace
    cfg = synth.configs()
    for config, spec, same_as in (("cfg5_deep_small_spatial", cfg["cfg5_deep_small_spatial"][0], B.DW_REDUCED_K),
                                  ("cfg2_resnet18_cifar", cfg["cfg2_resnet18_cifar"][1], B.DW_INFLATE)):
        t = synth.make_inputs(spec, config, tensors=("X", "dY"))
        X, dY = upload(t["X"], spec.dtype), upload(t["dY"], spec.dtype)
        da, db = B.desc_from_spec(spec, dw_algo=B.DW_AUTO), B.desc_from_spec(spec, dw_algo=same_as)
        hp, wp, _, _ = B.cac_pooled_shape(da)
        Z = torch.empty((spec.N, spec.C, hp, wp), dtype=torch.bfloat16, device="cuda:0")
        B.cac_compress(da, X, Z)
        shape = (spec.K, spec.C, spec.R, spec.S)
        dWa, dWb = Guarded(shape, torch.float32), Guarded(shape, torch.float32)
        B.conv_bwd_weight_compressed(da, Z, dY, dWa.t, workspace(da, B.OP_BWD_WEIGHT_COMPRESSED))
        B.conv_bwd_weight_compressed(db, Z, dY, dWb.t, workspace(db, B.OP_BWD_WEIGHT_COMPRESSED))
        torch.cuda.synchronize()
        dWa.check(spec.name)
        dWb.check(spec.name)
        assert torch.equal(dWa.t, dWb.t), spec.name
