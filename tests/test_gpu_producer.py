"""Compression at the producer of the activation (normalise + activate + pool in one pass) and
batch normalisation's backward pass from its compressed saved input, against the oracle."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_2409_11902_amd import binding as B
from paper_2409_11902_amd import synth
from util import check_bf16_output, rel_l2

pytestmark = pytest.mark.gpu

# N, C, H, W, kh, kw, dtype: the streaming kernel's tiles (1, 2, 4 in its mixes), odd and narrow
# rows, tiles the plain kernel takes, full-size layers
CASES = [
    (3, 5, 8, 8, 2, 2, synth.BF16), (2, 7, 7, 7, 2, 2, synth.BF16), (2, 3, 14, 14, 4, 4, synth.BF16), (4, 6, 9, 13, 2, 4, synth.BF16),
    (2, 4, 12, 20, 4, 2, synth.BF16), (2, 3, 5, 4, 2, 2, synth.BF16), (3, 4, 10, 10, 3, 3, synth.BF16), (2, 3, 9, 11, 1, 1, synth.BF16),
    (3, 5, 8, 8, 2, 2, synth.F32), (2, 7, 7, 9, 2, 2, synth.F32), (2, 4, 10, 7, 3, 2, synth.F32), (2, 3, 16, 12, 4, 4, synth.F32),
    (64, 64, 56, 56, 2, 2, synth.BF16), (128, 512, 7, 7, 2, 2, synth.BF16), (32, 256, 14, 14, 4, 4, synth.BF16),
    # rows of 10, 12, 14 elements (a thread per row pair): fewer records than a wave, whole waves, whole waves and a rest, full size
    (5, 3, 4, 12, 2, 2, synth.BF16), (16, 64, 14, 14, 2, 2, synth.BF16), (3, 50, 14, 14, 2, 2, synth.BF16), (2, 7, 6, 10, 2, 2, synth.BF16),
    (256, 512, 14, 14, 2, 2, synth.BF16), (9, 33, 28, 28, 2, 2, synth.BF16),
]


def _inputs(N, C, H, W, dt, seed):
    rng = np.random.Generator(np.random.Philox(key=seed))
    Y = synth.to_storage(rng.standard_normal((N, C, H, W), dtype=np.float32) * 1.5 + 0.2, dt)
    gamma = (1.0 + 0.3 * rng.standard_normal(C)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(C)).astype(np.float32)
    mean = Y.mean(axis=(0, 2, 3), dtype=np.float64).astype(np.float32)
    invstd = (1.0 / np.sqrt(Y.var(axis=(0, 2, 3), dtype=np.float64) + 1e-5)).astype(np.float32)
    return Y, gamma, beta, mean, invstd


@pytest.mark.parametrize("c", CASES, ids=[" ".join(map(str, c)) for c in CASES])
def test_normalise_activate_compress(c):
    from gpu_util import Guarded, download, upload
    N, C, H, W, kh, kw, dt = c
    Y, gamma, beta, mean, invstd = _inputs(N, C, H, W, dt, 11)
    scale = (gamma * invstd).astype(np.float32)
    shift = (beta - mean * scale).astype(np.float32)
    d = B.make_desc(N, C, 8, H, W, 1, 1, 1, 1, 0, 0, kh, kw, dtype=B.F32 if dt == synth.F32 else B.BF16)
    hp, wp, _, _ = B.cac_pooled_shape(d)
    td = torch.float32 if dt == synth.F32 else torch.bfloat16
    Yd = upload(Y, dt)
    sc, sh = torch.from_numpy(scale).cuda(), torch.from_numpy(shift).cuda()
    Xn, Zn, Zin = Guarded((N, C, H, W), td), Guarded((N, C, hp, wp), td), Guarded((N, C, hp, wp), td)
    Zn2, Zin2 = torch.empty_like(Zn.t), torch.empty_like(Zin.t)
    B.cac_bn_relu_fwd_compress(d, Yd, sc, sh, Xn.t, Zn.t, Zin.t)
    B.cac_compress(d, Xn.t, Zn2)
    B.cac_compress(d, Yd, Zin2)
    torch.cuda.synchronize()
    for b in (Xn, Zn, Zin):
        b.check("producer")
    # the records are, bit for bit, what compressing the stored tensors gives
    assert torch.equal(Zn.t.view(torch.uint8), Zn2.view(torch.uint8))
    assert torch.equal(Zin.t.view(torch.uint8), Zin2.view(torch.uint8))
    got_x = download(Xn.t)
    want_x = oracle.bn_relu(Y.astype(np.float64), scale, shift)
    if dt == synth.F32:
        assert np.abs(got_x - want_x).max() <= 1e-5 * max(1.0, np.abs(want_x).max())
    else:
        check_bf16_output(got_x, want_x, "X_next")
    # and they are the oracle's pooling of those tensors (to the storage type's rounding)
    tol = 1e-6 if dt == synth.F32 else 2.0 ** -8
    want_zn = oracle.avgpool(got_x, kh, kw)
    assert np.abs(download(Zn.t) - want_zn).max() <= tol * max(1e-30, np.abs(want_zn).max())
    want_zin = oracle.avgpool(Y.astype(np.float64), kh, kw)
    assert np.abs(download(Zin.t) - want_zin).max() <= tol * max(1e-30, np.abs(want_zin).max())
    # without the optional record
    Xn3, Zn3 = torch.empty_like(Xn.t), torch.empty_like(Zn.t)
    B.cac_bn_relu_fwd_compress(d, Yd, sc, sh, Xn3, Zn3, None)
    torch.cuda.synchronize()
    assert torch.equal(Xn3.view(torch.uint8), Xn.t.view(torch.uint8)) and torch.equal(Zn3.view(torch.uint8), Zn.t.view(torch.uint8))


BN_CASES = CASES[:12] + [(16, 64, 28, 28, 2, 2, synth.BF16), (64, 64, 56, 56, 2, 2, synth.BF16), (256, 512, 14, 14, 2, 2, synth.BF16),
                         (5, 3, 4, 12, 2, 2, synth.BF16), (16, 64, 14, 14, 2, 2, synth.BF16), (3, 50, 14, 14, 2, 2, synth.BF16),
                         (2, 7, 6, 10, 2, 2, synth.BF16), (2, 2100, 14, 14, 2, 2, synth.BF16), (9, 33, 28, 28, 2, 2, synth.BF16),
                         (64, 512, 28, 28, 2, 2, synth.BF16)]


@pytest.mark.parametrize("c", BN_CASES, ids=[" ".join(map(str, c)) for c in BN_CASES])
def test_batch_norm_backward_from_the_compressed_record(c):
    from gpu_util import Guarded, download, upload
    N, C, H, W, kh, kw, dt = c
    Y, gamma, beta, mean, invstd = _inputs(N, C, H, W, dt, 12)
    rng = np.random.Generator(np.random.Philox(key=13))
    dY = synth.to_storage(rng.standard_normal((N, C, H, W), dtype=np.float32), dt)
    d = B.make_desc(N, C, 8, H, W, 1, 1, 1, 1, 0, 0, kh, kw, dtype=B.F32 if dt == synth.F32 else B.BF16)
    hp, wp, _, _ = B.cac_pooled_shape(d)
    td = torch.float32 if dt == synth.F32 else torch.bfloat16
    Yd, dYd = upload(Y, dt), upload(dY, dt)
    Zin = torch.empty((N, C, hp, wp), dtype=td, device="cuda:0")
    B.cac_compress(d, Yd, Zin)
    dg, db, dX = Guarded((C,), torch.float32), Guarded((C,), torch.float32), Guarded((N, C, H, W), td)
    f = lambda a: torch.from_numpy(a).cuda()
    from gpu_util import workspace
    B.cac_bn_bwd_compressed(d, Zin, dYd, f(mean), f(invstd), f(gamma), dg.t, db.t, dX.t, workspace(d, B.OP_BN_BWD))
    torch.cuda.synchronize()
    for b in (dg, db, dX):
        b.check("bn backward")
    # the oracle from the same stored record (its own parity is the compress tests' subject)
    xs = oracle.inflate(download(Zin), H, W, kh, kw)
    want_dg, want_db, want_dx = oracle.bn_bwd(xs, dY.astype(np.float64), mean, invstd, gamma)
    M = N * H * W
    scale_g = np.sqrt(M) * max(1.0, float(np.abs(want_dg).max() / np.sqrt(M)))
    assert np.abs(download(dg.t) - want_dg).max() <= 2e-5 * scale_g
    assert np.abs(download(db.t) - want_db).max() <= 2e-5 * np.sqrt(M) * 4
    if dt == synth.F32:
        assert rel_l2(download(dX.t), want_dx) <= 1e-5
    else:
        check_bf16_output(download(dX.t), want_dx, "dX")
    if kh * kw == 1:
        # pooling factor 1 keeps the activation: the exact backward pass
        e_dg, e_db, e_dx = oracle.bn_bwd(Y.astype(np.float64), dY.astype(np.float64), mean, invstd, gamma)
        assert rel_l2(download(dX.t), e_dx) <= (1e-5 if dt == synth.F32 else 4e-3)
