"""ctypes binding of libcac.so: argument marshalling only.

Function names and argument order follow include/cac.h.  Tensors are torch
tensors on the GPU (torch is used for device memory and streams, nothing else);
every computation happens inside the library's HIP kernels.  A missing library
is an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

from . import synth

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcac.so")

CAC_OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_ALIGNMENT, ERR_LAUNCH_FAILED = -1, -2, -3, -4, -5
F32, BF16 = 0, 1
DW_INFLATE, DW_REDUCED_K, DW_AUTO = 0, 1, 2
EDGE_CEIL_VALID, EDGE_FLOOR_DROP = 0, 1
POOL_MEAN, POOL_MAX = 0, 1
(OP_FWD_AND_COMPRESS, OP_BWD_WEIGHT_COMPRESSED, OP_BWD_DATA, OP_COMPRESS, OP_BWD_BIAS, OP_GRAD_COSINE,
 OP_BWD_WEIGHT_AND_DATA, OP_BN_BWD) = range(8)

EXPORTS = (
    "cac_version", "cac_last_error", "cac_out_shape", "cac_pooled_shape", "cac_workspace_size", "cac_describe_plan",
    "cac_dw_executed_flops",
    "conv_fwd_and_compress", "cac_compress", "conv_bwd_weight_compressed", "conv_bwd_data", "conv_bwd_bias", "cac_grad_cosine",
    "conv_bwd_weight_and_data", "conv_bwd_weight_compressed_noalloc", "cac_bn_relu_fwd_compress", "cac_bn_bwd_compressed", "cac_probe",
)
PROBE_MFMA, PROBE_COPY, PROBE_READ, PROBE_MFMA_16X16, PROBE_MFMA_1WAVE = 0, 1, 2, 3, 4
NOALLOC_SCRATCH_BYTES = 40 << 20


class cac_desc(ctypes.Structure):
    _fields_ = [("size", ctypes.c_uint32)] + [
        (n, ctypes.c_int32) for n in (
            "N", "C_in", "C_out", "H", "W", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w",
            "pool_kh", "pool_kw", "edge_mode", "dtype", "has_bias", "pool_mode", "dw_algo")
    ]


class CacError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"cac error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded native library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2409_11902_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        L.cac_version.restype = ctypes.c_int
        L.cac_last_error.restype = ctypes.c_char_p
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        dp = ctypes.POINTER(cac_desc)
        ip = ctypes.POINTER(ctypes.c_int32)
        szp = ctypes.POINTER(ctypes.c_size_t)
        L.cac_out_shape.argtypes = [dp, ip, ip]
        L.cac_pooled_shape.argtypes = [dp, ip, ip, szp, szp]
        L.cac_workspace_size.argtypes = [dp, ctypes.c_int, szp]
        L.cac_describe_plan.argtypes = [dp, ctypes.c_int, ctypes.c_char_p, sz]
        L.cac_dw_executed_flops.argtypes = [dp, ctypes.POINTER(ctypes.c_uint64)]
        L.conv_fwd_and_compress.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cac_compress.argtypes = [dp, vp, vp, vp]
        L.conv_bwd_weight_compressed.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.conv_bwd_weight_compressed_noalloc.argtypes = [dp, vp, vp, vp, vp]
        L.conv_bwd_data.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.conv_bwd_weight_and_data.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.conv_bwd_bias.argtypes = [dp, vp, vp, vp]
        L.cac_probe.argtypes = [ctypes.c_int, vp, vp, sz, ctypes.c_int, vp]
        L.cac_bn_relu_fwd_compress.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        L.cac_bn_bwd_compressed.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cac_grad_cosine.argtypes = [dp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        for n in EXPORTS[2:]:
            getattr(L, n).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(rc: int):
    if rc != CAC_OK:
        raise CacError(rc, lib().cac_last_error().decode())


def make_desc(N, C_in, C_out, H, W, R, S, stride_h=1, stride_w=1, pad_h=0, pad_w=0, pool_kh=2, pool_kw=2,
              edge_mode=EDGE_CEIL_VALID, dtype=BF16, has_bias=1, pool_mode=POOL_MEAN, dw_algo=DW_INFLATE) -> cac_desc:
    return cac_desc(ctypes.sizeof(cac_desc), N, C_in, C_out, H, W, R, S, stride_h, stride_w, pad_h, pad_w,
                    pool_kh, pool_kw, edge_mode, dtype, has_bias, pool_mode, dw_algo)


def desc_from_spec(spec: synth.LayerSpec, has_bias: int = 1, **over) -> cac_desc:
    kw = dict(N=spec.N, C_in=spec.C, C_out=spec.K, H=spec.H, W=spec.W, R=spec.R, S=spec.S,
              stride_h=spec.stride, stride_w=spec.stride, pad_h=spec.pad, pad_w=spec.pad,
              pool_kh=spec.k, pool_kw=spec.k, dtype=F32 if spec.dtype == synth.F32 else BF16,
              has_bias=has_bias)
    kw.update(over)
    return make_desc(**kw)


def cac_version() -> int:
    return lib().cac_version()


def cac_out_shape(d: cac_desc):
    p, q = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().cac_out_shape(ctypes.byref(d), ctypes.byref(p), ctypes.byref(q)))
    return p.value, q.value


def cac_pooled_shape(d: cac_desc):
    """(Hp, Wp, z_bytes, x_bytes)"""
    hp, wp = ctypes.c_int32(), ctypes.c_int32()
    zb, xb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().cac_pooled_shape(ctypes.byref(d), ctypes.byref(hp), ctypes.byref(wp), ctypes.byref(zb),
                                  ctypes.byref(xb)))
    return hp.value, wp.value, zb.value, xb.value


def cac_workspace_size(d: cac_desc, op: int) -> int:
    b = ctypes.c_size_t()
    _check(lib().cac_workspace_size(ctypes.byref(d), op, ctypes.byref(b)))
    return b.value


def cac_describe_plan(d: cac_desc, op: int) -> str:
    buf = ctypes.create_string_buffer(2048)
    _check(lib().cac_describe_plan(ctypes.byref(d), op, buf, len(buf)))
    return buf.value.decode()


def dw_rk_executed_flops(d: cac_desc) -> int:
    f = ctypes.c_uint64()
    _check(lib().cac_dw_executed_flops(ctypes.byref(d), ctypes.byref(f)))
    return f.value


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ws(ws):
    if ws is None:
        return None, 0
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def conv_fwd_and_compress(d, X, W, b, Y, Z, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv_fwd_and_compress(ctypes.byref(d), _ptr(X), _ptr(W), _ptr(b), _ptr(Y), _ptr(Z), wp, wb,
                                       _stream(stream)))


def cac_compress(d, X, Z, stream=None):
    _check(lib().cac_compress(ctypes.byref(d), _ptr(X), _ptr(Z), _stream(stream)))


def conv_bwd_weight_compressed(d, Z, dY, dW, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv_bwd_weight_compressed(ctypes.byref(d), _ptr(Z), _ptr(dY), _ptr(dW), wp, wb, _stream(stream)))


def conv_bwd_weight_compressed_noalloc(d, Z, dY, dW, stream=None):
    _check(lib().conv_bwd_weight_compressed_noalloc(ctypes.byref(d), _ptr(Z), _ptr(dY), _ptr(dW), _stream(stream)))


def conv_bwd_data(d, W, dY, dX, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv_bwd_data(ctypes.byref(d), _ptr(W), _ptr(dY), _ptr(dX), wp, wb, _stream(stream)))


def conv_bwd_weight_and_data(d, Z, W, dY, dW, dX, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv_bwd_weight_and_data(ctypes.byref(d), _ptr(Z), _ptr(W), _ptr(dY), _ptr(dW), _ptr(dX), wp, wb,
                                          _stream(stream)))


def cac_bn_relu_fwd_compress(d, Y, scale, shift, X_next, Z_next, Z_in=None, stream=None):
    _check(lib().cac_bn_relu_fwd_compress(ctypes.byref(d), _ptr(Y), _ptr(scale), _ptr(shift), _ptr(X_next), _ptr(Z_next),
                                          _ptr(Z_in), _stream(stream)))


def cac_bn_bwd_compressed(d, Z_in, dY, mean, invstd, gamma, dgamma, dbeta, dX, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().cac_bn_bwd_compressed(ctypes.byref(d), _ptr(Z_in), _ptr(dY), _ptr(mean), _ptr(invstd), _ptr(gamma),
                                       _ptr(dgamma), _ptr(dbeta), _ptr(dX), wp, wb, _stream(stream)))


def cac_probe(kind, src, dst, nbytes, iters=0, stream=None):
    _check(lib().cac_probe(kind, _ptr(src), _ptr(dst), nbytes, iters, _stream(stream)))


def conv_bwd_bias(d, dY, db, stream=None):
    _check(lib().conv_bwd_bias(ctypes.byref(d), _ptr(dY), _ptr(db), _stream(stream)))


def cac_grad_cosine(d, dW_a, dW_b, out, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().cac_grad_cosine(ctypes.byref(d), _ptr(dW_a), _ptr(dW_b), _ptr(out), wp, wb, _stream(stream)))


# ---- host <-> device marshalling (type conversion only, no arithmetic)

def to_device(a, dtype: str, device: str = "cuda:0"):
    """float32 host array already rounded to `dtype` -> device tensor of that dtype."""
    import numpy as np
    import torch
    if dtype == synth.F32:
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    bits = synth.bf16_bits(a).view(np.int16)
    return torch.from_numpy(bits).to(device).view(torch.bfloat16)


def to_host(t):
    """device tensor -> float64 host array (bfloat16 widened exactly)."""
    import numpy as np
    import torch
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return synth.bf16_from_bits(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)
