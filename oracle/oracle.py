"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Wraps ``dnb_oracle.c`` (float64, NCHW).  Nothing in the product package imports
this module; it is used by ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg.  It holds no arithmetic of its own: every number comes
from the C file, whose functions cite the paper passages they follow.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dnb_oracle.c")
_LIB = os.path.join(_HERE, "libdnb_oracle.so")

G1, B1, W1, G2, B2, W3 = range(6)
PARAM_NAMES = ("g1", "b1", "W1", "g2", "b2", "W3")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, -O2).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("c0", C.c_int32), ("h", C.c_int32), ("w", C.c_int32),
                ("layers", C.c_int32), ("growth", C.c_int32), ("bottleneck", C.c_int32),
                ("eps", C.c_double)]


class _Mem(C.Structure):
    _fields_ = [("peak_elems", C.c_int64), ("stored_elems", C.c_int64), ("live_elems", C.c_int64)]


_lib = None
_dp = C.POINTER(C.c_double)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.dnbo_param_count.restype = C.c_int64
        _lib.dnbo_param_count.argtypes = [C.POINTER(_Desc)]
        _lib.dnbo_param_offset.restype = C.c_int64
        _lib.dnbo_param_offset.argtypes = [C.POINTER(_Desc), C.c_int, C.c_int, C.POINTER(C.c_int64)]
        for name in ("dnbo_block_naive", "dnbo_block_shared", "dnbo_block_naive_bf16"):
            f = getattr(_lib, name)
            f.restype = C.c_int
            f.argtypes = [C.POINTER(_Desc), _dp, _dp, _dp, _dp, _dp, _dp, C.POINTER(_Mem)]
        _lib.dnbo_round_bf16.restype = C.c_double
        _lib.dnbo_round_bf16.argtypes = [C.c_double]
        _lib.dnbo_block_probe_layer.restype = C.c_int
        _lib.dnbo_block_probe_layer.argtypes = [C.POINTER(_Desc), _dp, _dp, C.c_int, _dp, _dp]
        i64 = C.c_int64
        _lib.dnbo_bn_forward.restype = None
        _lib.dnbo_bn_forward.argtypes = [_dp, i64, i64, i64, _dp, _dp, C.c_double, _dp, _dp, _dp]
        _lib.dnbo_bn_backward.restype = None
        _lib.dnbo_bn_backward.argtypes = [_dp, _dp, i64, i64, i64, _dp, _dp, _dp, C.c_double, _dp, _dp, _dp]
        _lib.dnbo_conv_forward.restype = None
        _lib.dnbo_conv_forward.argtypes = [_dp, _dp, i64, i64, i64, i64, i64, i64, _dp]
        _lib.dnbo_conv_dgrad.restype = None
        _lib.dnbo_conv_dgrad.argtypes = [_dp, _dp, i64, i64, i64, i64, i64, i64, _dp]
        _lib.dnbo_conv_wgrad.restype = None
        _lib.dnbo_conv_wgrad.argtypes = [_dp, _dp, i64, i64, i64, i64, i64, i64, _dp]
        _lib.dnbo_relu_inplace.restype = None
        _lib.dnbo_relu_inplace.argtypes = [_dp, i64]
        _lib.dnbo_relu_backward.restype = None
        _lib.dnbo_relu_backward.argtypes = [_dp, _dp, _dp, i64]
        _lib.dnbo_num_threads.restype = C.c_int
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a: np.ndarray):
    return a.ctypes.data_as(_dp)


@dataclass(frozen=True)
class BlockShape:
    n: int
    c0: int
    h: int
    w: int
    layers: int
    growth: int
    bottleneck: int
    eps: float = 1e-5

    def _c(self) -> _Desc:
        return _Desc(self.n, self.c0, self.h, self.w, self.layers, self.growth, self.bottleneck, self.eps)

    @property
    def c_out(self) -> int:
        return self.c0 + self.layers * self.growth

    def c_in(self, layer: int) -> int:
        return self.c0 + (layer - 1) * self.growth


def param_count(s: BlockShape) -> int:
    d = s._c()
    return int(lib().dnbo_param_count(C.byref(d)))


def param_slice(s: BlockShape, layer: int, which: int) -> slice:
    d = s._c()
    cnt = C.c_int64(0)
    off = lib().dnbo_param_offset(C.byref(d), layer, which, C.byref(cnt))
    if off < 0:
        raise KeyError((layer, which))
    return slice(int(off), int(off) + int(cnt.value))


def param_shape(s: BlockShape, layer: int, which: int):
    c, k, B = s.c_in(layer), s.growth, s.bottleneck
    if which in (G1, B1):
        return (c,)
    if which == W1:
        return (B, c)
    if which in (G2, B2):
        return (B,)
    return (k, B if B > 0 else c, 3, 3)


@dataclass
class BlockResult:
    y: np.ndarray
    dx0: np.ndarray | None
    dparams: np.ndarray | None
    peak_elems: int
    stored_elems: int


def block(s: BlockShape, x0, params, dy=None, schedule: str = "naive") -> BlockResult:
    """Forward (and, if ``dy`` is given, backward) of one dense block."""
    d = s._c()
    x0 = _f64(x0).reshape(s.n, s.c0, s.h, s.w)
    params = _f64(params).reshape(-1)
    assert params.size == param_count(s)
    y = np.zeros((s.n, s.c_out, s.h, s.w), dtype=np.float64)
    mem = _Mem()
    fn = {"naive": lib().dnbo_block_naive, "shared": lib().dnbo_block_shared,
          "naive_bf16": lib().dnbo_block_naive_bf16}[schedule]
    if dy is None:
        fn(C.byref(d), _p(x0), _p(params), None, _p(y), None, None, C.byref(mem))
        return BlockResult(y, None, None, int(mem.peak_elems), int(mem.stored_elems))
    dy = _f64(dy).reshape(y.shape)
    dx0 = np.zeros_like(x0)
    dparams = np.zeros_like(params)
    fn(C.byref(d), _p(x0), _p(params), _p(dy), _p(y), _p(dx0), _p(dparams), C.byref(mem))
    return BlockResult(y, dx0, dparams, int(mem.peak_elems), int(mem.stored_elems))


def round_bf16(v: float) -> float:
    """Nearest bfloat16 (ties to even) of a float64, as the storage-emulating block uses it."""
    return float(lib().dnbo_round_bf16(float(v)))


def probe_layer(s: BlockShape, x0, params, layer: int):
    d = s._c()
    x0 = _f64(x0)
    params = _f64(params).reshape(-1)
    c = s.c_in(layer)
    u = np.zeros((s.n, c, s.h, s.w))
    xhat = np.zeros_like(u)
    rc = lib().dnbo_block_probe_layer(C.byref(d), _p(x0), _p(params), layer, _p(u), _p(xhat))
    assert rc == 0
    return u, xhat


def bn_forward(u, gamma, beta, eps=1e-5):
    u = _f64(u)
    n, c = u.shape[:2]
    hw = int(np.prod(u.shape[2:]))
    gamma, beta = _f64(gamma), _f64(beta)
    z = np.zeros_like(u)
    mean = np.zeros(c)
    var = np.zeros(c)
    lib().dnbo_bn_forward(_p(u), n, c, hw, _p(gamma), _p(beta), eps, _p(z), _p(mean), _p(var))
    return z, mean, var


def bn_backward(u, dz, gamma, mean, var, eps=1e-5):
    u, dz = _f64(u), _f64(dz)
    n, c = u.shape[:2]
    hw = int(np.prod(u.shape[2:]))
    gamma, mean, var = _f64(gamma), _f64(mean), _f64(var)
    du = np.zeros_like(u)
    dg = np.zeros(c)
    db = np.zeros(c)
    lib().dnbo_bn_backward(_p(u), _p(dz), n, c, hw, _p(gamma), _p(mean), _p(var), eps, _p(du), _p(dg), _p(db))
    return du, dg, db


def conv_forward(x, wgt):
    x, wgt = _f64(x), _f64(wgt)
    n, ci, h, w = x.shape
    co, ci2, ks, ks2 = wgt.shape
    assert ci == ci2 and ks == ks2
    out = np.zeros((n, co, h, w))
    lib().dnbo_conv_forward(_p(x), _p(wgt), n, ci, co, h, w, ks, _p(out))
    return out


def conv_dgrad(dout, wgt):
    dout, wgt = _f64(dout), _f64(wgt)
    n, co, h, w = dout.shape
    co2, ci, ks, _ = wgt.shape
    assert co == co2
    din = np.zeros((n, ci, h, w))
    lib().dnbo_conv_dgrad(_p(dout), _p(wgt), n, ci, co, h, w, ks, _p(din))
    return din


def conv_wgrad(x, dout, ks):
    x, dout = _f64(x), _f64(dout)
    n, ci, h, w = x.shape
    co = dout.shape[1]
    dw = np.zeros((co, ci, ks, ks))
    lib().dnbo_conv_wgrad(_p(x), _p(dout), n, ci, co, h, w, ks, _p(dw))
    return dw


def relu(z):
    a = _f64(z).copy()
    lib().dnbo_relu_inplace(_p(a), a.size)
    return a


def relu_backward(a, da):
    a, da = _f64(a), _f64(da)
    dz = np.zeros_like(a)
    lib().dnbo_relu_backward(_p(a), _p(da), _p(dz), a.size)
    return dz


def num_threads() -> int:
    return int(lib().dnbo_num_threads())
