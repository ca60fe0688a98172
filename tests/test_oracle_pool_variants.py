"""Pins of the oracle's pooling variants (no GPU): compression with the tile maximum and tiles
whose sides are not powers of two.  The compression section names other forms of pooling as
feasible without defining one; the reading pinned here is the textbook one (same tiles as the
mean, the largest element a tile really has, inflation unchanged), so a library routine, brute
force and a hand-worked map fix it."""
from __future__ import annotations

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import ConvGeom


def _rand(shape, seed, relu=False):
    x = np.random.Generator(np.random.Philox(key=seed)).standard_normal(shape)
    return np.maximum(x, 0) if relu else x


def test_maxpool_hand_worked_map():
    # 5 x 4 map, 2 x 2 tiles: the last tile row has one input row only
    x = np.array([[1, -2, 0, 7],
                  [3, 4, -5, 6],
                  [-1, -1, 2, 2],
                  [-9, -3, 8, -8],
                  [-4, -6, 5, 9]], dtype=np.float64).reshape(1, 1, 5, 4)
    want = np.array([[4, 7], [-1, 8], [-4, 9]], dtype=np.float64)
    assert np.array_equal(oracle.maxpool(x, 2, 2)[0, 0], want)
    # 4 x 2 tiles on the same map: tile rows 0-3 and 4
    assert np.array_equal(oracle.maxpool(x, 4, 2)[0, 0], np.array([[4, 8], [-4, 9]], dtype=np.float64))
    # floor/drop leaves the fifth row out
    assert np.array_equal(oracle.maxpool(x, 2, 2, oracle.EDGE_FLOOR_DROP)[0, 0], want[:2])


@pytest.mark.parametrize("k", [(1, 1), (2, 2), (4, 4), (2, 4), (3, 3), (3, 2), (8, 8)])
@pytest.mark.parametrize("hw", [(8, 8), (7, 7), (5, 9), (14, 14), (3, 10), (1, 1)])
def test_maxpool_against_torch(k, hw):
    kh, kw = k
    H, W = hw
    X = _rand((2, 3, H, W), 41) - 1.5        # mostly negative: a zero that stands in for a missing element would win
    Z = oracle.maxpool(X, kh, kw)
    # the library refuses windows that start outside the map; none does for ceil(H/k) tiles from the origin
    zt = F.max_pool2d(torch.tensor(X), (kh, kw), (kh, kw), ceil_mode=True)
    assert tuple(zt.shape[2:]) == oracle.pooled_shape(H, W, kh, kw) == Z.shape[2:]
    assert np.array_equal(Z, zt.numpy())
    if H >= kh and W >= kw:
        Zf = oracle.maxpool(X, kh, kw, oracle.EDGE_FLOOR_DROP)
        assert np.array_equal(Zf, F.max_pool2d(torch.tensor(X), (kh, kw), (kh, kw)).numpy())


def test_maxpool_brute_force():
    X = _rand((2, 2, 7, 5), 42)
    for kh, kw in [(2, 2), (3, 2), (4, 4)]:
        Z = oracle.maxpool(X, kh, kw)
        for n in range(2):
            for c in range(2):
                for i in range(-(-7 // kh)):
                    for j in range(-(-5 // kw)):
                        vals = [X[n, c, h, w] for h in range(i * kh, min(i * kh + kh, 7))
                                for w in range(j * kw, min(j * kw + kw, 5))]
                        assert Z[n, c, i, j] == max(vals)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_maxpool_properties(k):
    X = _rand((2, 3, 11, 13), 43)
    Zm, Za = oracle.maxpool(X, k, k), oracle.avgpool(X, k, k)
    assert (Zm >= Za - 1e-15).all() and (Zm > Za).any()
    # every maximum is an element of its own tile, and no element of the tile exceeds it
    Xh = oracle.inflate(Zm, 11, 13, k, k)
    assert (Xh >= X).all()
    hit = (Xh == X).reshape(2, 3, -1).sum(axis=2)
    assert (hit >= Zm.shape[2] * Zm.shape[3]).all()
    # shifting and positive scaling commute with the maximum; negation turns it into the minimum
    assert np.array_equal(oracle.maxpool(2.0 * X + 3.0, k, k), 2.0 * Zm + 3.0)
    assert (-oracle.maxpool(-X, k, k) <= Za + 1e-15).all()
    # k = 1 keeps the map
    assert np.array_equal(oracle.maxpool(X, 1, 1), X)


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("hw", [(8, 8), (7, 7), (5, 9)])
def test_tile_constant_maps_are_lossless_under_both_poolings(k, hw):
    H, W = hw
    hp, wp = oracle.pooled_shape(H, W, k, k)
    coarse = _rand((2, 3, hp, wp), 44)
    X = np.repeat(np.repeat(coarse, k, axis=2), k, axis=3)[:, :, :H, :W]
    assert np.array_equal(oracle.maxpool(X, k, k), coarse)
    np.testing.assert_allclose(oracle.avgpool(X, k, k), coarse, rtol=4e-16, atol=0)   # k = 3: nine equal terms / 9
    g = ConvGeom(2, 3, 4, H, W, 3, 3, 1, 1, 1, 1)
    dY = _rand((2, 4, g.P, g.Q), 45)
    Xh = oracle.inflate(oracle.maxpool(X, k, k), H, W, k, k)
    assert np.array_equal(oracle.conv_dw(g, Xh, dY), oracle.conv_dw(g, X, dY))


@pytest.mark.parametrize("k", [(3, 3), (3, 2), (5, 3)])
@pytest.mark.parametrize("hw", [(9, 9), (7, 7), (10, 4)])
def test_non_power_of_two_mean_tiles(k, hw):
    kh, kw = k
    H, W = hw
    X = _rand((2, 2, H, W), 46, relu=True)
    Z = oracle.avgpool(X, kh, kw)
    zt = F.avg_pool2d(torch.tensor(X), (kh, kw), (kh, kw), ceil_mode=True, count_include_pad=False)
    np.testing.assert_allclose(Z, zt.numpy(), rtol=1e-14, atol=0)
    Xh = oracle.inflate(Z, H, W, kh, kw)
    np.testing.assert_allclose(Xh.sum(axis=(2, 3)), X.sum(axis=(2, 3)), rtol=1e-13)
    # inflation: element (h, w) is the pooled value of tile (h // kh, w // kw)
    for h in range(H):
        for w in range(W):
            assert np.array_equal(Xh[:, :, h, w], Z[:, :, h // kh, w // kw])
