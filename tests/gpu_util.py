"""Device-side plumbing of the GPU parity tests: uploads, guarded output
buffers, one call of each entry point through the binding."""
from __future__ import annotations

import numpy as np
import torch

from paper_2409_11902_amd import binding as B
from paper_2409_11902_amd import synth

DEV = "cuda:0"
GUARD = 256  # bytes of canary on each side of every output buffer
CANARY = 0xA5


def upload(a: np.ndarray, dtype: str) -> torch.Tensor:
    return B.to_device(a, dtype, DEV)


def download(t: torch.Tensor) -> np.ndarray:
    return B.to_host(t)


class Guarded:
    """An output buffer with canary bytes before and after it."""

    def __init__(self, shape, torch_dtype):
        self.shape = tuple(shape)
        self.dtype = torch_dtype
        es = torch.empty((), dtype=torch_dtype).element_size()
        self.nbytes = int(np.prod(self.shape)) * es
        pad = (-self.nbytes) % 16
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), CANARY, dtype=torch.uint8, device=DEV)
        assert self.raw.data_ptr() % 16 == 0
        self.t = self.raw[GUARD:GUARD + self.nbytes].view(torch_dtype).view(self.shape)

    def check(self, what=""):
        head = self.raw[:GUARD]
        tail = self.raw[GUARD + self.nbytes:]
        assert bool((head == CANARY).all()) and bool((tail == CANARY).all()), f"{what}: write outside the buffer"

    def untouched_fraction(self):
        body = self.raw[GUARD:GUARD + self.nbytes]
        return float((body == CANARY).float().mean())


def tdtype(spec):
    return torch.float32 if spec.dtype == synth.F32 else torch.bfloat16


def workspace(d, op):
    n = B.cac_workspace_size(d, op)
    return None if n == 0 else torch.empty((n + 15) // 16 * 16, dtype=torch.uint8, device=DEV)


def run_step(spec: synth.LayerSpec, t: dict, has_bias: bool = True, desc_over=None):
    """One pass of the whole path for one layer.  Returns float64 host arrays
    Y, Z, dW, dX, db and the descriptor."""
    d = B.desc_from_spec(spec, has_bias=int(has_bias), **(desc_over or {}))
    hp, wp, zb, xb = B.cac_pooled_shape(d)
    td = tdtype(spec)
    X, Wt, dY = upload(t["X"], spec.dtype), upload(t["W"], spec.dtype), upload(t["dY"], spec.dtype)
    b = upload(t["b"], spec.dtype) if has_bias else None
    Y = Guarded((spec.N, spec.K, spec.P, spec.Q), td)
    Z = Guarded((spec.N, spec.C, hp, wp), td)
    dW = Guarded((spec.K, spec.C, spec.R, spec.S), torch.float32)
    dX = Guarded((spec.N, spec.C, spec.H, spec.W), td)
    db = Guarded((spec.K,), torch.float32)
    assert Z.nbytes == zb and dX.nbytes == xb
    B.conv_fwd_and_compress(d, X, Wt, b, Y.t, Z.t, workspace(d, B.OP_FWD_AND_COMPRESS))
    del X  # the layer input is not needed past this point: only Z is kept
    B.conv_bwd_weight_compressed(d, Z.t, dY, dW.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
    B.conv_bwd_data(d, Wt, dY, dX.t, workspace(d, B.OP_BWD_DATA))
    B.conv_bwd_bias(d, dY, db.t)
    torch.cuda.synchronize()
    out = {}
    for name, gbuf in (("Y", Y), ("Z", Z), ("dW", dW), ("dX", dX), ("db", db)):
        gbuf.check(f"{spec.name} {name}")
        out[name] = download(gbuf.t)
    out["desc"] = d
    return out
