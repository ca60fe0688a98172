"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches a GPU or the HIP library.  Each pin is chosen so
that a plausible slip in oracle/cac_oracle.c (a dropped term, a wrong sign or
index, swapped filter axes, a wrong divisor on ragged tiles) fails at least one.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import ConvGeom
from paper_2409_11902_amd import synth
from util import geom, rel_l2, tile_constant_activation

MiB = float(1 << 20)


def _rand(shape, seed, relu=False):
    rng = np.random.Generator(np.random.Philox(key=seed))
    a = rng.standard_normal(shape)
    return np.maximum(a, 0) if relu else a


# Asymmetric on purpose: H != W, R != S, strides and pads differ per axis, so a
# transposed axis or swapped stride/pad cannot cancel out.
GEOMS = [
    ConvGeom(2, 3, 4, 7, 9, 3, 3, 1, 1, 1, 1),
    ConvGeom(2, 3, 5, 8, 6, 3, 2, 2, 1, 1, 0),
    ConvGeom(1, 4, 3, 9, 7, 1, 1, 2, 2, 0, 0),
    ConvGeom(3, 2, 2, 5, 5, 3, 3, 2, 2, 1, 1),
    ConvGeom(2, 2, 3, 6, 10, 2, 3, 1, 2, 0, 2),
    ConvGeom(1, 5, 6, 4, 4, 1, 1, 1, 1, 0, 0),
    ConvGeom(2, 3, 2, 11, 6, 5, 3, 2, 1, 2, 1),
]


# ---------------------------------------------------------------- paper fixtures

def test_fig3_tile_membership(golden_dir):
    """Compression figure: which entries of the 4x4 X feed which mean of the 2x2 Z."""
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(golden_dir, "fig3_tiling.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 16
    assert oracle.pooled_shape(4, 4, 2, 2) == (2, 2)
    # indicator inputs: a single 1 at X[i,j] must land, as 1/4, only in mu[a,b]
    for (i, j, a, b) in rows:
        X = np.zeros((1, 1, 4, 4))
        X[0, 0, i, j] = 1.0
        Z = oracle.avgpool(X, 2, 2)
        want = np.zeros((1, 1, 2, 2))
        want[0, 0, a, b] = 0.25
        assert np.array_equal(Z, want)
        # and inflation paints mu[a,b] back over exactly the entries of that colour
        Zi = np.zeros((1, 1, 2, 2))
        Zi[0, 0, a, b] = 1.0
        Xh = oracle.inflate(Zi, 4, 4, 2, 2)
        members = {(r[0], r[1]) for r in rows if (r[2], r[3]) == (a, b)}
        got = {(int(h), int(w)) for h, w in zip(*np.nonzero(Xh[0, 0]))}
        assert got == members


def test_table1_bytes(golden_dir):
    """Per-layer memory table: X, Z(2x2), Z(4x4) MiB at mini-batch 32, 4-byte
    elements, reproduced by the floor/drop shape rule (the only one that gives the
    printed 0.28 / 0.56 / 0.06 MiB of the 14x14 and 7x7 layers)."""
    sums = np.zeros(3)
    paper_sum = None
    for line in open(os.path.join(golden_dir, "table1_memory.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "Sum":
            paper_sum = [float(v) for v in f[4:7]]
            continue
        C, H, W = int(f[1]), int(f[2]), int(f[3])
        printed = [float(v) for v in f[4:7]]
        xb, z2 = oracle.saved_bytes(32, C, H, W, 2, 2, 4, oracle.EDGE_FLOOR_DROP)
        _, z4 = oracle.saved_bytes(32, C, H, W, 4, 4, 4, oracle.EDGE_FLOOR_DROP)
        mine = [xb / MiB, z2 / MiB, z4 / MiB]
        sums += mine
        for m, p in zip(mine, printed):
            assert abs(m - p) <= 0.0051, (f[0], mine, printed)
    assert paper_sum is not None
    for m, p in zip(sums, paper_sum):
        assert abs(m - p) <= 0.0051, (sums, paper_sum)
    # reductions printed next to the sums: -75 % and -94 %
    assert round(100 * (1 - sums[1] / sums[0])) == 75
    assert round(100 * (1 - sums[2] / sums[0])) == 94


def test_reduction_fractions_when_k_divides():
    """Memory subsection: pooling cuts the saved bytes by 3/4 and 15/16."""
    for k, frac in ((2, 3 / 4), (4, 15 / 16)):
        for mode in (oracle.EDGE_CEIL_VALID, oracle.EDGE_FLOOR_DROP):
            xb, zb = oracle.saved_bytes(32, 64, 56, 56, k, k, 4, mode)
            assert xb - zb == int(frac * xb) and zb * k * k == xb


def test_ragged_shapes_ceil_valid():
    assert oracle.pooled_shape(7, 7, 2, 2) == (4, 4)
    assert oracle.pooled_shape(14, 14, 4, 4) == (4, 4)
    assert oracle.pooled_shape(7, 9, 4, 2) == (2, 5)
    xb, zb = oracle.saved_bytes(256, 512, 7, 7, 2, 2, 2)
    assert (xb, zb) == (256 * 512 * 49 * 2, 256 * 512 * 16 * 2)


# ---------------------------------------------------------------- invariants

@pytest.mark.parametrize("g", GEOMS)
def test_k1_is_identity_and_exact(g):
    """Pooling factor 1 stores X itself, so the weight gradient is the exact one
    (the uncompressed stem's gradient is unaffected: layer-sensitivity subsection)."""
    X = _rand((g.N, g.C, g.H, g.W), 1, relu=True)
    dY = _rand((g.N, g.K, g.P, g.Q), 2)
    Z = oracle.avgpool(X, 1, 1)
    assert np.array_equal(Z, X)
    Xh = oracle.inflate(Z, g.H, g.W, 1, 1)
    assert np.array_equal(Xh, X)
    assert np.array_equal(oracle.conv_dw(g, Xh, dY), oracle.conv_dw(g, X, dY))
    assert oracle.cosine(oracle.conv_dw(g, Xh, dY), oracle.conv_dw(g, X, dY)) == pytest.approx(1.0, abs=1e-15)


@pytest.mark.parametrize("k", [2, 4])
@pytest.mark.parametrize("hw", [(8, 8), (7, 7), (5, 9), (14, 6)])
def test_tile_constant_activation_is_lossless(k, hw):
    H, W = hw
    spec = synth.LayerSpec("t", 2, 3, 4, H, W, 3, 3, 1, 1, k=k, dtype=synth.F32)
    X = tile_constant_activation(spec).astype(np.float64)
    Z = oracle.avgpool(X, k, k)
    Xh = oracle.inflate(Z, H, W, k, k)
    assert np.array_equal(Xh, X)          # exact: sums of k*k equal values, power-of-two divisor
    g = geom(spec)
    dY = _rand((g.N, g.K, g.P, g.Q), 3)
    assert np.array_equal(oracle.conv_dw(g, Xh, dY), oracle.conv_dw(g, X, dY))


def test_ragged_tile_constant_lossless_nonpow2_counts():
    # ragged tiles have 2 or 1 valid elements at 7x7, k=2: mean of equal values is exact
    X = np.full((1, 1, 7, 7), 0.3)
    Xh = oracle.inflate(oracle.avgpool(X, 2, 2), 7, 7, 2, 2)
    assert np.array_equal(Xh, X)
    # k=4 on 7 wide: ragged tile has 3 columns: 3 equal values / 3
    Xh = oracle.inflate(oracle.avgpool(X, 4, 4), 7, 7, 4, 4)
    assert np.allclose(Xh, X, rtol=0, atol=1e-16)


@pytest.mark.parametrize("k", [2, 4])
@pytest.mark.parametrize("hw", [(8, 8), (7, 7), (5, 9), (14, 14)])
def test_average_pooling_preserves_channel_sums(k, hw):
    H, W = hw
    X = _rand((2, 3, H, W), 4, relu=True)
    Xh = oracle.inflate(oracle.avgpool(X, k, k), H, W, k, k)
    np.testing.assert_allclose(Xh.sum(axis=(2, 3)), X.sum(axis=(2, 3)), rtol=1e-13)
    # a wrong divisor on ragged tiles (k*k instead of the valid count) breaks this
    if H % k:
        Zbad = oracle.avgpool(np.pad(X, ((0, 0), (0, 0), (0, (-H) % k), (0, (-W) % k))), k, k)
        bad = oracle.inflate(Zbad, H + (-H) % k, W + (-W) % k, k, k)[:, :, :H, :W]
        assert not np.allclose(bad.sum(axis=(2, 3)), X.sum(axis=(2, 3)), rtol=1e-6)


@pytest.mark.parametrize("k", [2, 4])
def test_pointwise_conv_with_tile_constant_dy_is_exact(k):
    """1x1 stride-1 conv: if dY is constant on every tile, sum over a tile of x*g
    equals g * k*k * mean, so the compressed gradient equals the exact one."""
    g = ConvGeom(2, 3, 4, 8, 12, 1, 1, 1, 1, 0, 0)
    X = _rand((g.N, g.C, g.H, g.W), 5, relu=True)
    coarse = _rand((g.N, g.K, g.H // k, g.W // k), 6)
    dY = np.kron(coarse, np.ones((k, k)))
    Xh = oracle.inflate(oracle.avgpool(X, k, k), g.H, g.W, k, k)
    np.testing.assert_allclose(oracle.conv_dw(g, Xh, dY), oracle.conv_dw(g, X, dY), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("g", GEOMS)
def test_adjoint_identities(g):
    """<conv(X,W), dY> = <W, dW(X,dY)> = <X, dX(W,dY)>, and the bias pairs with db."""
    X = _rand((g.N, g.C, g.H, g.W), 7, relu=True)
    Wt = _rand((g.K, g.C, g.R, g.S), 8)
    b = _rand((g.K,), 9)
    dY = _rand((g.N, g.K, g.P, g.Q), 10)
    Y0 = oracle.conv_fwd(g, X, Wt, None)
    Yb = oracle.conv_fwd(g, X, Wt, b)
    lhs = float((Y0 * dY).sum())
    assert float((Wt * oracle.conv_dw(g, X, dY)).sum()) == pytest.approx(lhs, rel=1e-11)
    assert float((X * oracle.conv_dx(g, Wt, dY)).sum()) == pytest.approx(lhs, rel=1e-11)
    assert float(((Yb - Y0) * dY).sum()) == pytest.approx(float((b * oracle.bias_grad(dY)).sum()), rel=1e-10)


def test_dw_is_linear_in_the_activation():
    g = GEOMS[1]
    A1 = _rand((g.N, g.C, g.H, g.W), 11)
    A2 = _rand((g.N, g.C, g.H, g.W), 12)
    dY = _rand((g.N, g.K, g.P, g.Q), 13)
    lhs = oracle.conv_dw(g, 0.5 * A1 - 3.0 * A2, dY)
    rhs = 0.5 * oracle.conv_dw(g, A1, dY) - 3.0 * oracle.conv_dw(g, A2, dY)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- library special cases

@pytest.mark.parametrize("g", GEOMS)
def test_against_torch_cpu_fp64_autograd(g):
    """With k = 1 the step is an ordinary convolution layer: PyTorch's CPU fp64
    conv2d and its autograd give Y, dW, dX and db independently."""
    X = torch.tensor(_rand((g.N, g.C, g.H, g.W), 14, relu=True), requires_grad=True)
    Wt = torch.tensor(_rand((g.K, g.C, g.R, g.S), 15), requires_grad=True)
    b = torch.tensor(_rand((g.K,), 16), requires_grad=True)
    Y = F.conv2d(X, Wt, b, stride=(g.sh, g.sw), padding=(g.ph, g.pw))
    dY = torch.tensor(_rand(tuple(Y.shape), 17))
    Y.backward(dY)
    assert tuple(Y.shape) == (g.N, g.K, g.P, g.Q)
    xn, wn, bn, dyn = X.detach().numpy(), Wt.detach().numpy(), b.detach().numpy(), dY.numpy()
    np.testing.assert_allclose(oracle.conv_fwd(g, xn, wn, bn), Y.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_dw(g, xn, dyn), Wt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_dx(g, wn, dyn), X.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.bias_grad(dyn), b.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_torch_avgpool_ceil_mode_divides_by_valid_count():
    # establish the library's behaviour on a case small enough to do by hand first
    x = torch.arange(9, dtype=torch.float64).reshape(1, 1, 3, 3)
    z = F.avg_pool2d(x, 2, 2, ceil_mode=True, count_include_pad=False)
    want = torch.tensor([[(0 + 1 + 3 + 4) / 4, (2 + 5) / 2], [(6 + 7) / 2, 8.0]], dtype=torch.float64)
    assert torch.equal(z[0, 0], want)


@pytest.mark.parametrize("k", [(1, 1), (2, 2), (4, 4), (2, 4), (3, 3)])
@pytest.mark.parametrize("hw", [(8, 8), (7, 7), (5, 9), (14, 14), (3, 10)])
def test_pool_and_inflate_against_torch(k, hw):
    kh, kw = k
    H, W = hw
    X = _rand((2, 3, H, W), 18, relu=True)
    Z = oracle.avgpool(X, kh, kw)
    zt = F.avg_pool2d(torch.tensor(X), (kh, kw), (kh, kw), ceil_mode=True, count_include_pad=False)
    assert tuple(zt.shape[2:]) == oracle.pooled_shape(H, W, kh, kw)
    np.testing.assert_allclose(Z, zt.numpy(), rtol=1e-14, atol=0)
    Xh = oracle.inflate(Z, H, W, kh, kw)
    xt = torch.tensor(Z).repeat_interleave(kh, dim=2).repeat_interleave(kw, dim=3)[:, :, :H, :W]
    assert np.array_equal(Xh, xt.numpy())
    # floor/drop pooling equals the library's default floor-mode pooling
    if H >= kh and W >= kw:
        Zf = oracle.avgpool(X, kh, kw, oracle.EDGE_FLOOR_DROP)
        zf = F.avg_pool2d(torch.tensor(X), (kh, kw), (kh, kw))
        np.testing.assert_allclose(Zf, zf.numpy(), rtol=1e-14, atol=0)


def test_inflate_refuses_what_the_paper_leaves_undefined():
    """Floor/drop tiles that leave rows or columns uncovered: the paper says nothing about what
    those pixels inflate to, so the oracle has no value for them.  Where the tiles do cover the
    map the two edge modes are the same thing."""
    X = _rand((1, 2, 7, 8), 25, relu=True)
    Zf = oracle.avgpool(X, 2, 2, oracle.EDGE_FLOOR_DROP)
    assert Zf.shape == (1, 2, 3, 4)
    with pytest.raises(ValueError):
        oracle.inflate(Zf, 7, 8, 2, 2, oracle.EDGE_FLOOR_DROP)
    X = _rand((1, 2, 8, 12), 26, relu=True)
    Zf, Zc = oracle.avgpool(X, 2, 4, oracle.EDGE_FLOOR_DROP), oracle.avgpool(X, 2, 4)
    assert np.array_equal(Zf, Zc)
    assert np.array_equal(oracle.inflate(Zf, 8, 12, 2, 4, oracle.EDGE_FLOOR_DROP), oracle.inflate(Zc, 8, 12, 2, 4))


@pytest.mark.parametrize("g", GEOMS[:5])
@pytest.mark.parametrize("k", [2, 4])
def test_compressed_dw_against_unfold_matmul(g, k):
    """The whole compressed step, rebuilt with different machinery: library
    pooling, repeat + crop, an explicit patch matrix (unfold) and one matmul."""
    X = _rand((g.N, g.C, g.H, g.W), 19, relu=True)
    dY = _rand((g.N, g.K, g.P, g.Q), 20)
    mine = oracle.conv_dw(g, oracle.inflate(oracle.avgpool(X, k, k), g.H, g.W, k, k), dY)
    zt = F.avg_pool2d(torch.tensor(X), k, k, ceil_mode=True, count_include_pad=False)
    xh = zt.repeat_interleave(k, dim=2).repeat_interleave(k, dim=3)[:, :, :g.H, :g.W]
    cols = F.unfold(xh, (g.R, g.S), padding=(g.ph, g.pw), stride=(g.sh, g.sw))   # N, C*R*S, P*Q
    gy = torch.tensor(dY).reshape(g.N, g.K, g.P * g.Q)
    dw = torch.einsum("nkl,ncl->kc", gy, cols).reshape(g.K, g.C, g.R, g.S)
    np.testing.assert_allclose(mine, dw.numpy(), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- regrouped (tile-sum) form

@pytest.mark.parametrize("g", GEOMS)
@pytest.mark.parametrize("k", [(1, 1), (2, 2), (4, 4), (2, 4), (3, 2)])
def test_tile_sum_form_is_the_inflated_form(g, k):
    """Regrouping the pixel sum by pooling tile changes nothing: Z times the tile sums of dY equals
    the weight-gradient formula applied to the inflated Z, for every stride, padding and tile."""
    kh, kw = k
    X = _rand((g.N, g.C, g.H, g.W), 31, relu=True)
    dY = _rand((g.N, g.K, g.P, g.Q), 32)
    Z = oracle.avgpool(X, kh, kw)
    want = oracle.conv_dw(g, oracle.inflate(Z, g.H, g.W, kh, kw), dY)
    got = oracle.conv_dw_from_tile_sums(g, Z, dY, kh, kw)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_tile_sums_by_hand_and_by_mass():
    """3x3, stride 1, padding 1, 2x2 tiles on a 4x4 map: tap (0,0) reads input pixel (p-1, q-1), so
    tile (0,0) (input rows 0-1, columns 0-1) collects dY at p, q in {1,2}; tap (1,1) collects the
    aligned pairs.  Every dY value whose tap lies inside the image is counted exactly once."""
    g = oracle.ConvGeom(1, 1, 1, 4, 4, 3, 3, 1, 1, 1, 1)
    dY = np.arange(16, dtype=np.float64).reshape(1, 1, 4, 4)
    T00 = oracle.tile_sums(g, dY, 2, 2, 0, 0)[0, 0]
    assert T00[0, 0] == dY[0, 0, 1, 1] + dY[0, 0, 1, 2] + dY[0, 0, 2, 1] + dY[0, 0, 2, 2]
    assert T00[1, 1] == dY[0, 0, 3, 3]                   # p, q in {3, 4}: only 3 exists
    T11 = oracle.tile_sums(g, dY, 2, 2, 1, 1)[0, 0]
    assert T11[0, 1] == dY[0, 0, 0, 2] + dY[0, 0, 0, 3] + dY[0, 0, 1, 2] + dY[0, 0, 1, 3]
    assert T11.sum() == dY.sum()                         # the centre tap never leaves the image
    assert T00.sum() == dY[0, 0, 1:, 1:].sum()           # row 0 / column 0 fall into the padding
    g2 = oracle.ConvGeom(2, 1, 3, 9, 7, 3, 3, 2, 2, 1, 1)
    dY2 = _rand((2, 3, g2.P, g2.Q), 33)
    for r in range(3):
        for s in range(3):
            T = oracle.tile_sums(g2, dY2, 2, 4, r, s)
            rows = [p for p in range(g2.P) if 0 <= 2 * p + r - 1 < 9]
            cols = [q for q in range(g2.Q) if 0 <= 2 * q + s - 1 < 7]
            np.testing.assert_allclose(T.sum(axis=(2, 3)), dY2[:, :, rows][:, :, :, cols].sum(axis=(2, 3)), rtol=1e-13)


# ---------------------------------------------------------------- normalisation at the producer

def test_bn_backward_against_autograd_and_relu_form():
    """The batch-normalisation backward formulas from the saved activation itself equal library
    autograd through batch_norm in training mode; the producer's forward is the library's
    batch_norm + relu when scale and shift are built from the batch statistics."""
    rng = np.random.default_rng(5)
    N, C, H, W = 3, 4, 5, 6
    X = rng.standard_normal((N, C, H, W))
    dY = rng.standard_normal((N, C, H, W))
    gamma, beta = rng.standard_normal(C) + 1.5, rng.standard_normal(C)
    eps = 1e-5
    mean = X.mean(axis=(0, 2, 3))
    var = X.var(axis=(0, 2, 3))
    invstd = 1.0 / np.sqrt(var + eps)
    xt = torch.tensor(X, requires_grad=True)
    gt, bt = torch.tensor(gamma, requires_grad=True), torch.tensor(beta, requires_grad=True)
    yt = F.batch_norm(xt, None, None, gt, bt, training=True, eps=eps)
    yt.backward(torch.tensor(dY))
    dgamma, dbeta, dX = oracle.bn_bwd(X, dY, mean, invstd, gamma)
    np.testing.assert_allclose(dgamma, gt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dbeta, bt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dX, xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    scale = gamma * invstd
    shift = beta - mean * scale
    np.testing.assert_allclose(oracle.bn_relu(X, scale, shift), F.relu(yt).detach().numpy(), rtol=1e-11, atol=1e-12)
    # a tile-constant activation is its own inflated record: the compressed backward is then exact
    Xc = np.repeat(np.repeat(rng.standard_normal((N, C, 3, 3)), 2, axis=2), 2, axis=3)[:, :, :5, :6]
    Zc = oracle.avgpool(Xc, 2, 2)
    a = oracle.bn_bwd(oracle.inflate(Zc, 5, 6, 2, 2), dY, mean, invstd, gamma)
    b = oracle.bn_bwd(Xc, dY, mean, invstd, gamma)
    for u, v in zip(a, b):
        np.testing.assert_allclose(u, v, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- sampled-entry functions

@pytest.mark.parametrize("g", GEOMS[:4])
def test_entry_functions_match_full_tensors(g):
    X = _rand((g.N, g.C, g.H, g.W), 21, relu=True)
    Wt = _rand((g.K, g.C, g.R, g.S), 22)
    b = _rand((g.K,), 23)
    dY = _rand((g.N, g.K, g.P, g.Q), 24)
    rng = np.random.default_rng(0)
    dW = oracle.conv_dw(g, X, dY)
    idx = rng.integers(0, dW.size, 50)
    assert np.array_equal(oracle.conv_dw_entries(g, X, dY, idx), dW.ravel()[idx])
    dX = oracle.conv_dx(g, Wt, dY)
    idx = rng.integers(0, dX.size, 80)
    np.testing.assert_allclose(oracle.conv_dx_entries(g, Wt, dY, idx), dX.ravel()[idx], rtol=1e-12, atol=1e-13)
    Y = oracle.conv_fwd(g, X, Wt, b)
    idx = rng.integers(0, Y.size, 80)
    assert np.array_equal(oracle.conv_fwd_entries(g, X, Wt, b, idx), Y.ravel()[idx])


# ---------------------------------------------------------------- cosine similarity

def test_cosine_closed_forms():
    a = np.array([3.0, 4.0, 0.0])
    assert oracle.cosine(a, a) == pytest.approx(1.0, abs=1e-15)
    assert oracle.cosine(a, -2 * a) == pytest.approx(-1.0, abs=1e-15)
    assert oracle.cosine(a, np.array([-4.0, 3.0, 7.0])) == pytest.approx(0.0, abs=1e-15)
    assert oracle.cosine(np.array([1.0, 0.0]), np.array([1.0, 1.0])) == pytest.approx(np.sqrt(0.5), rel=1e-15)
    # a zero gradient has no direction: the convention taken is 0, for either argument
    assert oracle.cosine(np.zeros(3), a) == 0.0 and oracle.cosine(a, np.zeros(3)) == 0.0


def test_compression_lowers_cosine_but_keeps_direction():
    # not a paper number: a sanity bound that the approximation is an approximation
    spec = synth.LayerSpec("t", 4, 8, 8, 16, 16, 3, 3, 1, 1, k=2, dtype=synth.F32)
    t = synth.make_inputs(spec, "pins")
    g = geom(spec)
    X, dY = t["X"].astype(np.float64), t["dY"].astype(np.float64)
    exact = oracle.conv_dw(g, X, dY)
    c2 = oracle.cosine(oracle.conv_dw(g, oracle.inflate(oracle.avgpool(X, 2, 2), 16, 16, 2, 2), dY), exact)
    c4 = oracle.cosine(oracle.conv_dw(g, oracle.inflate(oracle.avgpool(X, 4, 4), 16, 16, 4, 4), dY), exact)
    assert 0.0 < c4 < c2 < 1.0
