"""ctypes front end of cac_oracle.c (TEST INFRASTRUCTURE, not the product).

Every function takes and returns contiguous numpy float64 arrays.  The C file is
compiled with gcc on first use (or by build()); nothing here touches a GPU.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

EDGE_CEIL_VALID = 0
EDGE_FLOOR_DROP = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cac_oracle.c")
_LIB = os.path.join(_HERE, "libcac_oracle.so")
_lib = None

_i64 = ctypes.c_int64
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile cac_oracle.c into libcac_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_cosine.restype = ctypes.c_double
        _lib.oracle_inflate.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


@dataclass(frozen=True)
class ConvGeom:
    """Geometry of one convolution layer (notation of the compression figure)."""
    N: int
    C: int
    K: int
    H: int
    W: int
    R: int
    S: int
    sh: int = 1
    sw: int = 1
    ph: int = 0
    pw: int = 0

    @property
    def P(self) -> int:
        return out_shape(self)[0]

    @property
    def Q(self) -> int:
        return out_shape(self)[1]

    def _args(self):
        return [_i64(v) for v in (self.N, self.C, self.K, self.H, self.W, self.R, self.S,
                                  self.sh, self.sw, self.ph, self.pw)]


def _d(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def pooled_shape(H: int, W: int, kh: int, kw: int, edge_mode: int = EDGE_CEIL_VALID):
    hp, wp = _i64(), _i64()
    _load().oracle_pooled_shape(_i64(H), _i64(W), _i64(kh), _i64(kw), ctypes.c_int(edge_mode),
                                ctypes.byref(hp), ctypes.byref(wp))
    return int(hp.value), int(wp.value)


def out_shape(g: ConvGeom):
    p, q = _i64(), _i64()
    _load().oracle_out_shape(_i64(g.H), _i64(g.W), _i64(g.R), _i64(g.S), _i64(g.sh), _i64(g.sw),
                             _i64(g.ph), _i64(g.pw), ctypes.byref(p), ctypes.byref(q))
    return int(p.value), int(q.value)


def saved_bytes(N: int, C: int, H: int, W: int, kh: int, kw: int, elem_bytes: int,
                edge_mode: int = EDGE_CEIL_VALID):
    """(x_bytes, z_bytes) of the saved activation, exact integers."""
    hp, wp = pooled_shape(H, W, kh, kw, edge_mode)
    return N * C * H * W * elem_bytes, N * C * hp * wp * elem_bytes


def avgpool(X, kh: int, kw: int, edge_mode: int = EDGE_CEIL_VALID) -> np.ndarray:
    X = _f64(X)
    N, C, H, W = X.shape
    hp, wp = pooled_shape(H, W, kh, kw, edge_mode)
    Z = np.empty((N, C, hp, wp), dtype=np.float64)
    _load().oracle_avgpool(_d(X), _i64(N), _i64(C), _i64(H), _i64(W), _i64(kh), _i64(kw),
                           ctypes.c_int(edge_mode), _d(Z))
    return Z


def maxpool(X, kh: int, kw: int, edge_mode: int = EDGE_CEIL_VALID) -> np.ndarray:
    """Tile maxima over the same tiles as avgpool (a reading: the compression section names other
    poolings as feasible and defines none)."""
    X = _f64(X)
    N, C, H, W = X.shape
    hp, wp = pooled_shape(H, W, kh, kw, edge_mode)
    Z = np.empty((N, C, hp, wp), dtype=np.float64)
    _load().oracle_maxpool(_d(X), _i64(N), _i64(C), _i64(H), _i64(W), _i64(kh), _i64(kw),
                           ctypes.c_int(edge_mode), _d(Z))
    return Z


def inflate(Z, H: int, W: int, kh: int, kw: int, edge_mode: int = EDGE_CEIL_VALID) -> np.ndarray:
    Z = _f64(Z)
    N, C, hp, wp = Z.shape
    assert (hp, wp) == pooled_shape(H, W, kh, kw, edge_mode)
    Xh = np.empty((N, C, H, W), dtype=np.float64)
    rc = _load().oracle_inflate(_d(Z), _i64(N), _i64(C), _i64(H), _i64(W), _i64(kh), _i64(kw),
                                ctypes.c_int(edge_mode), _d(Xh))
    if rc != 0:
        raise ValueError("inflation is undefined where floor/drop tiles leave rows or columns uncovered")
    return Xh


def conv_fwd(g: ConvGeom, X, Wt, b=None) -> np.ndarray:
    X, Wt = _f64(X), _f64(Wt)
    assert X.shape == (g.N, g.C, g.H, g.W) and Wt.shape == (g.K, g.C, g.R, g.S)
    bb = None if b is None else _f64(b)
    Y = np.empty((g.N, g.K, g.P, g.Q), dtype=np.float64)
    _load().oracle_conv_fwd(_d(X), _d(Wt), _d(bb) if bb is not None else None, *g._args(), _d(Y))
    return Y


def conv_dw(g: ConvGeom, A, dY) -> np.ndarray:
    """dW from activation A (inflated Z for the compressed step, X for the exact one)."""
    A, dY = _f64(A), _f64(dY)
    assert A.shape == (g.N, g.C, g.H, g.W) and dY.shape == (g.N, g.K, g.P, g.Q)
    dW = np.empty((g.K, g.C, g.R, g.S), dtype=np.float64)
    _load().oracle_conv_dw(_d(A), _d(dY), *g._args(), _d(dW))
    return dW


def conv_dw_entries(g: ConvGeom, A, dY, flat_index) -> np.ndarray:
    A, dY = _f64(A), _f64(dY)
    assert A.shape == (g.N, g.C, g.H, g.W) and dY.shape == (g.N, g.K, g.P, g.Q)
    idx = np.ascontiguousarray(flat_index, dtype=np.int64)
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < g.K * g.C * g.R * g.S)
    out = np.empty(idx.shape, dtype=np.float64)
    _load().oracle_conv_dw_entries(_d(A), _d(dY), *g._args(), idx.ctypes.data_as(_ip),
                                   _i64(idx.size), _d(out))
    return out


def tile_sums(g: ConvGeom, dY, kh: int, kw: int, r: int, s: int) -> np.ndarray:
    """T[n,o,i,j]: sum of the dY values whose filter tap (r, s) lands in pooling tile (i, j)."""
    dY = _f64(dY)
    assert dY.shape == (g.N, g.K, g.P, g.Q) and 0 <= r < g.R and 0 <= s < g.S
    hp, wp = pooled_shape(g.H, g.W, kh, kw)
    T = np.empty((g.N, g.K, hp, wp), dtype=np.float64)
    _load().oracle_tile_sums(_d(dY), *g._args(), _i64(kh), _i64(kw), _i64(r), _i64(s), _d(T))
    return T


def conv_dw_from_tile_sums(g: ConvGeom, Z, dY, kh: int, kw: int, round_sums=None) -> np.ndarray:
    """The weight gradient of the compressed step in its regrouped form, tap by tap:
    dW[o,c,r,s] = sum_{n,i,j} Z[n,c,i,j] * T_rs[n,o,i,j] (a plain contraction; numpy's matmul is
    the step).  `round_sums`: applied to every T_rs first (the harness passes its storage-type
    rounding when it checks a kernel that keeps the sums in that type)."""
    Z = _f64(Z)
    dW = np.empty((g.K, g.C, g.R, g.S), dtype=np.float64)
    zf = Z.transpose(1, 0, 2, 3).reshape(g.C, -1)
    for r in range(g.R):
        for s in range(g.S):
            T = tile_sums(g, dY, kh, kw, r, s)
            if round_sums is not None:
                T = _f64(round_sums(T))
            dW[:, :, r, s] = T.transpose(1, 0, 2, 3).reshape(g.K, -1) @ zf.T
    return dW


def conv_dx(g: ConvGeom, Wt, dY) -> np.ndarray:
    Wt, dY = _f64(Wt), _f64(dY)
    assert Wt.shape == (g.K, g.C, g.R, g.S) and dY.shape == (g.N, g.K, g.P, g.Q)
    dX = np.empty((g.N, g.C, g.H, g.W), dtype=np.float64)
    _load().oracle_conv_dx(_d(Wt), _d(dY), *g._args(), _d(dX))
    return dX


def conv_dx_entries(g: ConvGeom, Wt, dY, flat_index) -> np.ndarray:
    Wt, dY = _f64(Wt), _f64(dY)
    assert Wt.shape == (g.K, g.C, g.R, g.S) and dY.shape == (g.N, g.K, g.P, g.Q)
    idx = np.ascontiguousarray(flat_index, dtype=np.int64)
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < g.N * g.C * g.H * g.W)
    out = np.empty(idx.shape, dtype=np.float64)
    _load().oracle_conv_dx_entries(_d(Wt), _d(dY), *g._args(), idx.ctypes.data_as(_ip),
                                   _i64(idx.size), _d(out))
    return out


def conv_fwd_entries(g: ConvGeom, X, Wt, b, flat_index) -> np.ndarray:
    X, Wt = _f64(X), _f64(Wt)
    assert X.shape == (g.N, g.C, g.H, g.W) and Wt.shape == (g.K, g.C, g.R, g.S)
    bb = None if b is None else _f64(b)
    idx = np.ascontiguousarray(flat_index, dtype=np.int64)
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < g.N * g.K * g.P * g.Q)
    out = np.empty(idx.shape, dtype=np.float64)
    _load().oracle_conv_fwd_entries(_d(X), _d(Wt), _d(bb) if bb is not None else None,
                                    *g._args(), idx.ctypes.data_as(_ip), _i64(idx.size), _d(out))
    return out


def bn_relu(Y, scale, shift) -> np.ndarray:
    """relu(scale[c] * Y + shift[c]): a normalisation with given per-channel statistics followed by
    the activation, i.e. what produces a convolution's input in the residual networks of the
    experiments (architecture figure)."""
    Y = _f64(Y)
    sc, sh = _f64(scale)[None, :, None, None], _f64(shift)[None, :, None, None]
    return np.maximum(sc * Y + sh, 0.0)


def bn_bwd(Xsaved, dY, mean, invstd, gamma):
    """Backward pass of y = gamma * xhat + beta, xhat = (x - mean) * invstd with batch statistics
    (the textbook formulas), from the saved activation the backward pass has: x itself for the
    exact step, the inflated record for the compressed one (the conclusion's extension of the
    method to batch normalisation; a reading, the paper gives no formulas).
    Returns (dgamma, dbeta, dX)."""
    X, dY = _f64(Xsaved), _f64(dY)
    N, C, H, W = X.shape
    mu, istd, g = (_f64(v)[None, :, None, None] for v in (mean, invstd, gamma))
    xh = (X - mu) * istd
    M = N * H * W
    dbeta = dY.sum(axis=(0, 2, 3))
    dgamma = (dY * xh).sum(axis=(0, 2, 3))
    dX = g * istd * (dY - dbeta[None, :, None, None] / M - xh * dgamma[None, :, None, None] / M)
    return dgamma, dbeta, dX


def bias_grad(dY) -> np.ndarray:
    dY = _f64(dY)
    N, K, P, Q = dY.shape
    db = np.empty((K,), dtype=np.float64)
    _load().oracle_bias_grad(_d(dY), _i64(N), _i64(K), _i64(P), _i64(Q), _d(db))
    return db


def cosine(a, b) -> float:
    a, b = _f64(a).ravel(), _f64(b).ravel()
    assert a.size == b.size
    return float(_load().oracle_cosine(_d(a), _d(b), _i64(a.size)))


def num_threads() -> int:
    return int(_load().oracle_num_threads())
