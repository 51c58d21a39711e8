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
_SRC_NET = os.path.join(_HERE, "dnb_net_oracle.c")
_SRC_INET = os.path.join(_HERE, "dnb_inet_oracle.c")
_LIB = os.path.join(_HERE, "libdnb_oracle.so")

G1, B1, W1, G2, B2, W3 = range(6)
PARAM_NAMES = ("g1", "b1", "W1", "g2", "b2", "W3")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, -O2).  Returns the library path."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_NET), os.path.getmtime(_SRC_INET))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", _LIB, _SRC, _SRC_NET, _SRC_INET, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("c0", C.c_int32), ("h", C.c_int32), ("w", C.c_int32),
                ("layers", C.c_int32), ("growth", C.c_int32), ("bottleneck", C.c_int32),
                ("eps", C.c_double)]


class _NetDesc(C.Structure):
    _fields_ = [("n", C.c_int32), ("image", C.c_int32), ("depth", C.c_int32), ("growth", C.c_int32),
                ("classes", C.c_int32), ("eps", C.c_double)]


class _InetDesc(C.Structure):
    _fields_ = [("n", C.c_int32), ("image", C.c_int32), ("growth", C.c_int32), ("layers", C.c_int32 * 4),
                ("classes", C.c_int32), ("eps", C.c_double)]


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
        _lib.dnbo_block_naive_masks.restype = C.c_int
        _lib.dnbo_block_naive_masks.argtypes = [C.POINTER(_Desc), _dp, _dp, _dp, _dp, _dp, _dp, C.POINTER(_Mem), C.c_int,
                                                C.c_void_p, C.c_void_p, _dp, C.c_int]
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
        # whole-network step (dnb_net_oracle.c)
        nd = C.POINTER(_NetDesc)
        _lib.dnbo_net_param_count.restype = C.c_int64
        _lib.dnbo_net_param_count.argtypes = [nd]
        _lib.dnbo_net_block_param_offset.restype = C.c_int64
        _lib.dnbo_net_block_param_offset.argtypes = [nd, C.c_int]
        _lib.dnbo_net_step.restype = C.c_double
        _lib.dnbo_net_step.argtypes = [nd, _dp, C.POINTER(C.c_int32), _dp, _dp, _dp]
        _lib.dnbo_net_decision_count.restype = C.c_int64
        _lib.dnbo_net_decision_count.argtypes = [nd]
        _lib.dnbo_net_step_masks.restype = C.c_double
        _lib.dnbo_net_step_masks.argtypes = [nd, _dp, C.POINTER(C.c_int32), _dp, _dp, _dp, C.c_int, C.c_void_p, _dp]
        idp = C.POINTER(_InetDesc)
        _lib.dnbo_inet_param_count.restype = C.c_int64
        _lib.dnbo_inet_param_count.argtypes = [idp]
        _lib.dnbo_inet_param_offset.restype = C.c_int64
        _lib.dnbo_inet_param_offset.argtypes = [idp, C.c_int, C.POINTER(C.c_int64)]
        _lib.dnbo_inet_decision_counts.restype = None
        _lib.dnbo_inet_decision_counts.argtypes = [idp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        _lib.dnbo_inet_step.restype = C.c_double
        _lib.dnbo_inet_step.argtypes = [idp, _dp, C.POINTER(C.c_int32), _dp, _dp, _dp, C.c_int, C.c_void_p, C.c_void_p, _dp,
                                        C.c_int]
        for nm in ("dnbo_conv_forward_strided", "dnbo_conv_wgrad_strided", "dnbo_conv_dgrad_strided"):
            getattr(_lib, nm).restype = None
            getattr(_lib, nm).argtypes = [_dp, _dp, i64, i64, i64, i64, i64, i64, i64, i64, _dp]
        _lib.dnbo_maxpool3s2.restype = None
        _lib.dnbo_maxpool3s2.argtypes = [_dp, i64, i64, i64, i64, _dp, C.c_void_p, C.c_int, _dp, _dp]
        _lib.dnbo_maxpool3s2_backward.restype = None
        _lib.dnbo_maxpool3s2_backward.argtypes = [_dp, C.c_void_p, i64, i64, i64, i64, _dp]
        _lib.dnbo_avgpool2.restype = None
        _lib.dnbo_avgpool2.argtypes = [_dp, i64, i64, i64, i64, _dp]
        _lib.dnbo_avgpool2_backward.restype = None
        _lib.dnbo_avgpool2_backward.argtypes = [_dp, i64, i64, i64, i64, _dp]
        _lib.dnbo_global_avgpool.restype = None
        _lib.dnbo_global_avgpool.argtypes = [_dp, i64, i64, i64, _dp]
        _lib.dnbo_global_avgpool_backward.restype = None
        _lib.dnbo_global_avgpool_backward.argtypes = [_dp, i64, i64, i64, _dp]
        _lib.dnbo_linear.restype = None
        _lib.dnbo_linear.argtypes = [_dp, _dp, _dp, i64, i64, i64, _dp]
        _lib.dnbo_linear_backward.restype = None
        _lib.dnbo_linear_backward.argtypes = [_dp, _dp, _dp, i64, i64, i64, _dp, _dp, _dp]
        _lib.dnbo_softmax_xent.restype = C.c_double
        _lib.dnbo_softmax_xent.argtypes = [_dp, C.POINTER(C.c_int32), i64, i64, _dp]
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


def relu_decision_counts(s: BlockShape):
    """Elements of the two ReLU-decision arrays of a block: the first BN of every layer (the layers'
    (n, C_l, h, w) arrays one after the other) and the second BN (layers x (n, B, h, w))."""
    P = s.n * s.h * s.w
    return sum(s.c_in(l) for l in range(1, s.layers + 1)) * P, s.layers * s.bottleneck * P


def block_with_decisions(s: BlockShape, x0, params, dy, decisions=None, bf16_storage: bool = False):
    """The store-everything block with its ReLU decisions (z > 0, one byte each) written out
    (decisions=None: returns (result, (m1, m2))) or taken from the caller (decisions=(m1, m2):
    returns (result, stats) with stats = dict(count1, margin1, count2, margin2): how many of the
    caller's decisions differ from the block's own and the largest margin |z| / sqrt(gamma^2 +
    beta^2) among those: the pre-activation in units of its channel's root mean square).
    bf16_storage: with the storage rounding of schedule "naive_bf16" on top."""
    d = s._c()
    x0 = _f64(x0).reshape(s.n, s.c0, s.h, s.w)
    params = _f64(params).reshape(-1)
    assert params.size == param_count(s)
    y = np.zeros((s.n, s.c_out, s.h, s.w), dtype=np.float64)
    dy = _f64(dy).reshape(y.shape)
    dx0 = np.zeros_like(x0)
    dparams = np.zeros_like(params)
    mem = _Mem()
    n1, n2 = relu_decision_counts(s)
    if decisions is None:
        m1, m2 = np.zeros(n1, dtype=np.uint8), np.zeros(max(n2, 1), dtype=np.uint8)
        mode = 0
    else:
        m1 = np.ascontiguousarray(np.asarray(decisions[0], dtype=np.uint8).reshape(-1))
        m2 = np.ascontiguousarray(np.asarray(decisions[1], dtype=np.uint8).reshape(-1)) if n2 else np.zeros(1, dtype=np.uint8)
        assert m1.size == n1 and (n2 == 0 or m2.size == n2)
        mode = 1
    stats = np.zeros(4)
    lib().dnbo_block_naive_masks(C.byref(d), _p(x0), _p(params), _p(dy), _p(y), _p(dx0), _p(dparams), C.byref(mem), mode,
                                 m1.ctypes.data_as(C.c_void_p), m2.ctypes.data_as(C.c_void_p), _p(stats),
                                 1 if bf16_storage else 0)
    res = BlockResult(y, dx0, dparams, int(mem.peak_elems), int(mem.stored_elems))
    if decisions is None:
        return res, (m1, m2[:n2])
    return res, dict(count1=int(stats[0]), margin1=float(stats[1]), count2=int(stats[2]), margin2=float(stats[3]))


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


# ---------------------------------------------------------------- whole network (dnb_net_oracle.c)

@dataclass(frozen=True)
class NetShape:
    """CIFAR-shaped DenseNet-BC: stem to 2k, three dense blocks of (depth-4)/6 bottleneck layers,
    transitions with compression 0.5, BN-ReLU-pool-linear tail."""
    n: int
    image: int
    depth: int
    growth: int
    classes: int
    eps: float = 1e-5

    def _c(self) -> _NetDesc:
        return _NetDesc(self.n, self.image, self.depth, self.growth, self.classes, self.eps)

    def block(self, b: int) -> BlockShape:
        per = (self.depth - 4) // 6
        c, s = 2 * self.growth, self.image
        for _ in range(b):
            c = (c + per * self.growth) // 2
            s //= 2
        return BlockShape(self.n, c, s, s, per, self.growth, 4 * self.growth, self.eps)


def net_param_count(s: NetShape) -> int:
    d = s._c()
    return int(lib().dnbo_net_param_count(C.byref(d)))


def net_param_slices(s: NetShape) -> dict:
    """Name -> slice of the network pack: 'stem', 'block0..2', 'trans0.g/b/W', 'trans1.*',
    'tail.g/b/Wl/bl'."""
    d = s._c()
    out = {"stem": slice(0, 2 * s.growth * 27)}
    for b in range(3):
        bs = s.block(b)
        o = int(lib().dnbo_net_block_param_offset(C.byref(d), b))
        n = param_count(bs)
        out[f"block{b}"] = slice(o, o + n)
        c = bs.c_out
        o += n
        pre = f"trans{b}" if b < 2 else "tail"
        out[pre + ".g"] = slice(o, o + c)
        out[pre + ".b"] = slice(o + c, o + 2 * c)
        if b < 2:
            out[pre + ".W"] = slice(o + 2 * c, o + 2 * c + (c // 2) * c)
        else:
            out[pre + ".Wl"] = slice(o + 2 * c, o + 2 * c + s.classes * c)
            out[pre + ".bl"] = slice(o + 2 * c + s.classes * c, o + 2 * c + s.classes * c + s.classes)
    return out


def net_step(s: NetShape, x, labels, params, backward: bool = True):
    """One training step: returns (loss, dparams or None, logits)."""
    d = s._c()
    x = _f64(x).reshape(s.n, 3, s.image, s.image)
    params = _f64(params).reshape(-1)
    assert params.size == net_param_count(s)
    lab = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    assert lab.shape == (s.n,) and lab.min() >= 0 and lab.max() < s.classes
    logits = np.zeros((s.n, s.classes))
    dparams = np.zeros_like(params) if backward else None
    loss = lib().dnbo_net_step(C.byref(d), _p(x), lab.ctypes.data_as(C.POINTER(C.c_int32)), _p(params),
                               _p(dparams) if backward else None, _p(logits))
    return float(loss), dparams, logits


def net_decision_count(s: NetShape) -> int:
    """Number of ReLU decisions of one step: per block its first-BN decisions (all layers), its
    second-BN decisions, then those of the BN+ReLU that follows the block."""
    d = s._c()
    return int(lib().dnbo_net_decision_count(C.byref(d)))


def net_step_with_decisions(s: NetShape, x, labels, params, decisions=None):
    """One training step with every ReLU decision written out (decisions=None: returns (loss,
    dparams, logits, decisions)) or imposed (returns (loss, dparams, logits, stats) with stats =
    dict(count, margin): decisions that differ from the step's own and their largest margin)."""
    d = s._c()
    x = _f64(x).reshape(s.n, 3, s.image, s.image)
    params = _f64(params).reshape(-1)
    assert params.size == net_param_count(s)
    lab = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    logits = np.zeros((s.n, s.classes))
    dparams = np.zeros_like(params)
    cnt = net_decision_count(s)
    if decisions is None:
        m, mode = np.zeros(cnt, dtype=np.uint8), 0
    else:
        m, mode = np.ascontiguousarray(np.asarray(decisions, dtype=np.uint8).reshape(-1)), 1
        assert m.size == cnt
    stats = np.zeros(2)
    loss = lib().dnbo_net_step_masks(C.byref(d), _p(x), lab.ctypes.data_as(C.POINTER(C.c_int32)), _p(params), _p(dparams),
                                     _p(logits), mode, m.ctypes.data_as(C.c_void_p), _p(stats))
    if decisions is None:
        return float(loss), dparams, logits, m
    return float(loss), dparams, logits, dict(count=int(stats[0]), margin=float(stats[1]))


def avgpool2(x):
    x = _f64(x)
    n, c, h, w = x.shape
    out = np.zeros((n, c, h // 2, w // 2))
    lib().dnbo_avgpool2(_p(x), n, c, h, w, _p(out))
    return out


def avgpool2_backward(dout, h, w):
    dout = _f64(dout)
    n, c = dout.shape[:2]
    din = np.zeros((n, c, h, w))
    lib().dnbo_avgpool2_backward(_p(dout), n, c, h, w, _p(din))
    return din


def global_avgpool(x):
    x = _f64(x)
    n, c, h, w = x.shape
    out = np.zeros((n, c))
    lib().dnbo_global_avgpool(_p(x), n, c, h * w, _p(out))
    return out


def global_avgpool_backward(dout, h, w):
    dout = _f64(dout)
    n, c = dout.shape
    din = np.zeros((n, c, h, w))
    lib().dnbo_global_avgpool_backward(_p(dout), n, c, h * w, _p(din))
    return din


def linear(f, wl, bl):
    f, wl, bl = _f64(f), _f64(wl), _f64(bl)
    n, c = f.shape
    out = np.zeros((n, wl.shape[0]))
    lib().dnbo_linear(_p(f), _p(wl), _p(bl), n, c, wl.shape[0], _p(out))
    return out


def linear_backward(f, wl, dlogits):
    f, wl, dlogits = _f64(f), _f64(wl), _f64(dlogits)
    n, c = f.shape
    df, dwl, dbl = np.zeros_like(f), np.zeros_like(wl), np.zeros(wl.shape[0])
    lib().dnbo_linear_backward(_p(f), _p(wl), _p(dlogits), n, c, wl.shape[0], _p(df), _p(dwl), _p(dbl))
    return df, dwl, dbl


def softmax_xent(logits, labels):
    logits = _f64(logits)
    n, classes = logits.shape
    lab = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    d = np.zeros_like(logits)
    loss = lib().dnbo_softmax_xent(_p(logits), lab.ctypes.data_as(C.POINTER(C.c_int32)), n, classes, _p(d))
    return float(loss), d


# ------------------------------------------------------------------ ImageNet-shaped network (four dense blocks)

def conv_forward_strided(x, wgt, stride, pad):
    x, wgt = _f64(x), _f64(wgt)
    n, ci, h, w = x.shape
    co, _, ks, _ = wgt.shape
    ho, wo = (h + 2 * pad - ks) // stride + 1, (w + 2 * pad - ks) // stride + 1
    out = np.zeros((n, co, ho, wo))
    lib().dnbo_conv_forward_strided(_p(x), _p(wgt), n, ci, co, h, w, ks, stride, pad, _p(out))
    return out


def conv_wgrad_strided(x, dout, ks, stride, pad):
    x, dout = _f64(x), _f64(dout)
    n, ci, h, w = x.shape
    co = dout.shape[1]
    dw = np.zeros((co, ci, ks, ks))
    lib().dnbo_conv_wgrad_strided(_p(x), _p(dout), n, ci, co, h, w, ks, stride, pad, _p(dw))
    return dw


def conv_dgrad_strided(dout, wgt, h, w, stride, pad):
    dout, wgt = _f64(dout), _f64(wgt)
    n, co = dout.shape[:2]
    ci, ks = wgt.shape[1], wgt.shape[2]
    din = np.zeros((n, ci, h, w))
    lib().dnbo_conv_dgrad_strided(_p(dout), _p(wgt), n, ci, co, h, w, ks, stride, pad, _p(din))
    return din


def maxpool3s2(x, positions=None, inv_rms=None):
    """3x3 max pooling, stride 2, pad 1.  Returns (out, positions) with positions the window index
    3*i + j of each maximum (first in scan order among equals); if `positions` is given they are
    imposed instead and (out, (count, margin)) of the differing ones is returned."""
    x = _f64(x)
    n, c, h, w = x.shape
    out = np.zeros((n, c, h // 2, w // 2))
    if positions is None:
        idx = np.zeros(out.shape, dtype=np.uint8)
        lib().dnbo_maxpool3s2(_p(x), n, c, h, w, _p(out), idx.ctypes.data_as(C.c_void_p), 0, None, None)
        return out, idx
    idx = np.ascontiguousarray(np.asarray(positions, dtype=np.uint8).reshape(out.shape))
    stat = np.zeros(2)
    ir = _f64(inv_rms) if inv_rms is not None else np.ones(c)
    lib().dnbo_maxpool3s2(_p(x), n, c, h, w, _p(out), idx.ctypes.data_as(C.c_void_p), 1, _p(ir), _p(stat))
    return out, (int(stat[0]), float(stat[1]))


def maxpool3s2_backward(dout, positions, h, w):
    dout = _f64(dout)
    n, c = dout.shape[:2]
    idx = np.ascontiguousarray(np.asarray(positions, dtype=np.uint8).reshape(dout.shape))
    din = np.zeros((n, c, h, w))
    lib().dnbo_maxpool3s2_backward(_p(dout), idx.ctypes.data_as(C.c_void_p), n, c, h, w, _p(din))
    return din


@dataclass(frozen=True)
class InetShape:
    n: int
    image: int
    growth: int
    layers: tuple
    classes: int
    eps: float = 1e-5

    def _c(self) -> _InetDesc:
        return _InetDesc(self.n, self.image, self.growth, (C.c_int32 * 4)(*self.layers), self.classes, self.eps)

    def block(self, b: int) -> BlockShape:
        c, s = 2 * self.growth, self.image // 4
        for i in range(b):
            c = (c + self.layers[i] * self.growth) // 2
            s //= 2
        return BlockShape(self.n, c, s, s, self.layers[b], self.growth, 4 * self.growth, self.eps)


def inet_param_count(s: InetShape) -> int:
    d = s._c()
    return int(lib().dnbo_inet_param_count(C.byref(d)))


def inet_param_slices(s: InetShape) -> dict:
    """Named slices of the network pack: stem.W, stem.g, stem.b, block0..3, trans0..2.{g,b,W}, tail.{g,b,Wl,bl}."""
    d = s._c()
    def sl(which):
        cnt = C.c_int64()
        off = int(lib().dnbo_inet_param_offset(C.byref(d), which, C.byref(cnt)))
        return slice(off, off + int(cnt.value))
    out = {"stem.W": sl(0), "stem.g": sl(1), "stem.b": sl(2)}
    for b in range(4):
        out[f"block{b}"] = sl(3 + 4 * b)
        pre = f"trans{b}" if b < 3 else "tail"
        out[f"{pre}.g"], out[f"{pre}.b"] = sl(4 + 4 * b), sl(5 + 4 * b)
        out[f"{pre}.W" if b < 3 else "tail.Wl"] = sl(6 + 4 * b)
    out["tail.bl"] = sl(19)
    return out


def inet_decision_counts(s: InetShape):
    d = s._c()
    a, b = C.c_int64(), C.c_int64()
    lib().dnbo_inet_decision_counts(C.byref(d), C.byref(a), C.byref(b))
    return int(a.value), int(b.value)


def inet_step(s: InetShape, x, labels, params, backward: bool = True, decisions=None, bf16_storage: bool = False):
    """One training step.  decisions=None: plain, returns (loss, dparams, logits).  decisions="write":
    returns (loss, dparams, logits, (relu, pool)) with the step's own ReLU decisions and pooling
    positions.  decisions=(relu, pool): they are imposed; returns (loss, dparams, logits, stats) with
    stats = dict(relu_count, relu_margin, pool_count, pool_margin) of the differing ones."""
    d = s._c()
    x = _f64(x).reshape(s.n, 3, s.image, s.image)
    params = _f64(params).reshape(-1)
    assert params.size == inet_param_count(s)
    lab = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    logits = np.zeros((s.n, s.classes))
    dparams = np.zeros_like(params) if backward else None
    nr, npool = inet_decision_counts(s)
    stats = np.zeros(4)
    if decisions is None:
        mode, m, pl = -1, None, None
    elif isinstance(decisions, str):
        mode, m, pl = 0, np.zeros(nr, dtype=np.uint8), np.zeros(npool, dtype=np.uint8)
    else:
        mode = 1
        m = np.ascontiguousarray(np.asarray(decisions[0], dtype=np.uint8).reshape(-1))
        pl = np.ascontiguousarray(np.asarray(decisions[1], dtype=np.uint8).reshape(-1))
        assert m.size == nr and pl.size == npool
    vp = lambda a: a.ctypes.data_as(C.c_void_p) if a is not None else None
    loss = lib().dnbo_inet_step(C.byref(d), _p(x), lab.ctypes.data_as(C.POINTER(C.c_int32)), _p(params),
                                _p(dparams) if backward else None, _p(logits), mode, vp(m), vp(pl), _p(stats),
                                1 if bf16_storage else 0)
    if decisions is None:
        return float(loss), dparams, logits
    if mode == 0:
        return float(loss), dparams, logits, (m, pl)
    return float(loss), dparams, logits, dict(relu_count=int(stats[0]), relu_margin=float(stats[1]),
                                               pool_count=int(stats[2]), pool_margin=float(stats[3]))
