"""The combined backward call against the two separate ones: it runs the same kernels with the
slice sum of the weight gradient moved into the data gradient's repack launch, so both outputs
have to be bit-identical to the separate calls' (which the other parity tests hold against the
oracle), whatever kernels a shape ends up on."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2409_11902_amd import binding as B
from paper_2409_11902_amd import synth
from test_gpu_parity import SMALL
from test_gpu_random_shapes import _workload_like_specs

pytestmark = pytest.mark.gpu


def _specs():
    out = [synth.LayerSpec(name, N, C, K, H, W, R, S, stride, pad, k, dt)
           for (name, N, C, K, H, W, R, S, stride, pad, k) in SMALL for dt in (synth.BF16, synth.F32)]
    out += _workload_like_specs(16, seed=11)
    cfg = synth.configs()
    out += cfg["cfg2_resnet18_cifar"]
    out += [cfg["cfg4_resnet18_imagenet_k2"][i] for i in (1, 2, 4, 9)]
    return out


SPECS = _specs()


@pytest.mark.parametrize("spec", SPECS, ids=[f"{s.name} {s.dtype}" for s in SPECS])
def test_combined_backward_is_bit_identical_to_the_separate_calls(spec):
    from gpu_util import Guarded, upload, workspace, tdtype
    d = B.desc_from_spec(spec)
    t = synth.make_inputs(spec, "bwd_both", tensors=("X", "W", "dY"))
    hp, wp, _, _ = B.cac_pooled_shape(d)
    td = tdtype(spec)
    X, Wt, dY = upload(t["X"], spec.dtype), upload(t["W"], spec.dtype), upload(t["dY"], spec.dtype)
    Z = torch.empty((spec.N, spec.C, hp, wp), dtype=td, device="cuda:0")
    B.cac_compress(d, X, Z)
    del X
    out = {}
    for mode in ("separate", "both"):
        dW, dX = Guarded((spec.K, spec.C, spec.R, spec.S), torch.float32), Guarded((spec.N, spec.C, spec.H, spec.W), td)
        if mode == "separate":
            B.conv_bwd_weight_compressed(d, Z, dY, dW.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
            B.conv_bwd_data(d, Wt, dY, dX.t, workspace(d, B.OP_BWD_DATA))
        else:
            ws = workspace(d, B.OP_BWD_WEIGHT_AND_DATA)
            if ws is not None:
                ws.fill_(0xFF)   # stale contents must not matter (all-ones floats are NaN)
            B.conv_bwd_weight_and_data(d, Z, Wt, dY, dW.t, dX.t, ws)
        torch.cuda.synchronize()
        dW.check(f"{mode} dW")
        dX.check(f"{mode} dX")
        assert dW.untouched_fraction() < 0.1 and dX.untouched_fraction() < 0.1   # (a result byte may equal the canary by chance)
        out[mode] = (dW.t.clone(), dX.t.clone())
    assert torch.equal(out["separate"][0], out["both"][0]), "dW"
    assert torch.equal(out["separate"][1].view(torch.uint8), out["both"][1].view(torch.uint8)), "dX"
