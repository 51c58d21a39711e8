"""Thin ctypes binding of libdnb.so: same names as include/dnb.h, argument
marshalling only.  Device memory and streams come from PyTorch; every step of
the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing, importing this module raises."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdnb.so")

DNB_OK = 0
DNB_E_BADDESC, DNB_E_NULL, DNB_E_ALIGN, DNB_E_LAUNCH, DNB_E_UNSUPPORTED, DNB_E_RANGE, DNB_E_NOMEM = range(-1, -8, -1)
DNB_F32, DNB_BF16 = 0, 1
DNB_NCHW, DNB_NHWC = 0, 1
DNB_SCHED_SHARED, DNB_SCHED_STORE_ALL, DNB_SCHED_FUSED = 0, 1, 2
DNB_P_G1, DNB_P_B1, DNB_P_W1, DNB_P_G2, DNB_P_B2, DNB_P_W3 = range(6)
(DNB_NP_STEM, DNB_NP_BLOCK0, DNB_NP_BLOCK1, DNB_NP_BLOCK2, DNB_NP_TRANS0_G, DNB_NP_TRANS0_B, DNB_NP_TRANS0_W,
 DNB_NP_TRANS1_G, DNB_NP_TRANS1_B, DNB_NP_TRANS1_W, DNB_NP_TAIL_G, DNB_NP_TAIL_B, DNB_NP_TAIL_WL,
 DNB_NP_TAIL_BL) = range(14)


class dnb_block_desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("c0", C.c_int32), ("h", C.c_int32), ("w", C.c_int32),
                ("layers", C.c_int32), ("growth", C.c_int32), ("bottleneck", C.c_int32),
                ("dtype", C.c_int32), ("layout", C.c_int32), ("schedule", C.c_int32),
                ("eps", C.c_float)]


class dnb_net_desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("image", C.c_int32), ("depth", C.c_int32), ("growth", C.c_int32),
                ("classes", C.c_int32), ("schedule", C.c_int32), ("eps", C.c_float)]


class dnb_inet_desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("image", C.c_int32), ("growth", C.c_int32), ("layers", C.c_int32 * 4),
                ("classes", C.c_int32), ("schedule", C.c_int32), ("eps", C.c_float)]


class dnb_block_memory(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("stored_fwd_bytes", "shared_fwd_bytes", "grad_bytes", "peak_bytes",
                                           "stats_bytes", "scratch_bytes", "workspace_bytes")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not found: build it first (python -m paper_1707_06990_amd.build "
                      "or __graft_entry__.build()); there is no fallback path")

_lib = C.CDLL(LIB_PATH)
_vp, _i64, _sz = C.c_void_p, C.c_int64, C.c_size_t

_SIGS = {
    "dnb_block_create": (C.c_int, [C.POINTER(dnb_block_desc), C.POINTER(_vp)]),
    "dnb_block_destroy": (None, [_vp]),
    "dnb_block_peak_bytes": (_sz, [_vp]),
    "dnb_block_workspace_bytes": (_sz, [_vp]),
    "dnb_block_memory_breakdown": (C.c_int, [_vp, C.POINTER(dnb_block_memory)]),
    "dnb_block_param_count": (_sz, [_vp]),
    "dnb_block_param_bytes": (_sz, [_vp]),
    "dnb_block_relu_decision_bytes": (_sz, [_vp, C.c_int]),
    "dnb_block_relu_decisions": (C.c_int, [_vp] * 7),
    "dnb_block_param_offset": (C.c_int, [_vp, C.c_int, C.c_int, C.POINTER(_sz), C.POINTER(_sz)]),
    "dnb_block_forward": (C.c_int, [_vp] * 6),
    "dnb_block_backward": (C.c_int, [_vp] * 8),
    "dnb_block_set_concurrency": (C.c_int, [_vp, C.c_int]),
    "dnb_status_string": (C.c_char_p, [C.c_int]),
    "dnb_op_copy_slab": (C.c_int, [_vp, _i64, _vp, _i64, _i64, _i64, _vp]),
    "dnb_op_bn_scratch_bytes": (_sz, [_i64, _i64, _i64]),
    "dnb_op_bn_stats": (C.c_int, [_vp, _i64, _i64, _i64, _i64, C.c_float, _vp, _vp, _vp, _vp]),
    "dnb_op_bn_stats_static": (C.c_int, [_vp, _i64, _i64, _i64, _i64, C.c_float, _vp, _vp, _vp]),
    "dnb_op_bn_relu": (C.c_int, [_vp, _i64, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp]),
    "dnb_op_bn_relu_backward": (C.c_int, [_vp, _i64, _vp, _i64, _vp, _i64, C.c_int, _i64, _i64, _i64,
                                          _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "dnb_op_bn_relu_backward_apply": (C.c_int, [_vp, _i64, _vp, _i64, _vp, _i64, C.c_int, _i64, _i64, _i64,
                                                _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "dnb_op_conv_scratch_bytes": (_sz, [_i64, _i64, C.c_int]),
    "dnb_op_conv_forward": (C.c_int, [_vp, _i64, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i64, C.c_int, _vp, _vp]),
    "dnb_op_conv_stats_bytes": (_sz, [_i64, _i64, _i64, _i64]),
    "dnb_op_conv_bnrelu_forward": (C.c_int, [_vp, _i64, _vp, _vp, _vp, _i64, _vp, C.POINTER(C.c_int), _i64, _i64, _i64,
                                             _i64, _i64, C.c_int, _vp, C.c_int, _vp, _vp, _vp]),
    "dnb_op_conv_bnrelu_wgrad": (C.c_int, [_vp, _i64, _vp, _vp, _i64, _vp, _i64, _i64, _i64, _i64, _i64, C.c_int, _vp,
                                           _vp, _vp, _vp]),
    "dnb_op_layer_wgrads_scratch_bytes": (_sz, [_i64, _i64, _i64, _i64, _i64, _i64]),
    "dnb_op_layer_wgrads_bn_partials_offset": (_sz, [_i64, _i64, _i64, _i64, _i64, _i64]),
    "dnb_op_layer_wgrads": (C.c_int, [_vp, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _i64, _i64, _i64, _i64,
                                      _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "dnb_op_conv_dgrad": (C.c_int, [_vp, _i64, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i64, C.c_int, _vp, _vp]),
    "dnb_op_conv_wgrad_scratch_bytes": (_sz, [_i64, _i64, _i64, _i64, _i64, C.c_int]),
    "dnb_op_conv_wgrad": (C.c_int, [_vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _i64, _i64, C.c_int, _vp, _vp]),
    "dnb_op_nhwc_scratch_bytes": (_sz, [_i64, _i64, _i64, _i64, _i64, C.c_int]),
    "dnb_op_nhwc_conv_forward": (C.c_int, [_vp, _i64, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i64, C.c_int, _vp, _vp]),
    "dnb_op_nhwc_conv_dgrad": (C.c_int, [_vp, _i64, C.c_int, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i64, C.c_int, _vp, _vp]),
    "dnb_op_nhwc_conv_wgrad": (C.c_int, [_vp, _i64, _vp, _i64, C.c_int, _vp, _i64, _i64, _i64, _i64, _i64, C.c_int, _vp, _vp]),
    "dnb_op_nhwc_bn_relu_backward": (C.c_int, [_vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64,
                                               _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "dnb_net_create": (C.c_int, [C.POINTER(dnb_net_desc), C.POINTER(_vp)]),
    "dnb_net_destroy": (None, [_vp]),
    "dnb_net_param_count": (_sz, [_vp]),
    "dnb_net_param_offset": (C.c_int, [_vp, C.c_int, C.POINTER(_sz), C.POINTER(_sz)]),
    "dnb_net_workspace_bytes": (_sz, [_vp]),
    "dnb_net_workspace_piece": (C.c_int, [_vp, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_int), C.POINTER(_sz),
                                          C.POINTER(_sz)]),
    "dnb_net_peak_bytes": (_sz, [_vp]),
    "dnb_net_relu_decision_bytes": (_sz, [_vp]),
    "dnb_net_relu_decisions": (C.c_int, [_vp] * 5),
    "dnb_net_set_concurrency": (C.c_int, [_vp, C.c_int]),
    "dnb_net_forward": (C.c_int, [_vp] * 8),
    "dnb_net_backward": (C.c_int, [_vp] * 6),
    "dnb_inet_create": (C.c_int, [C.POINTER(dnb_inet_desc), C.POINTER(_vp)]),
    "dnb_inet_destroy": (None, [_vp]),
    "dnb_inet_param_count": (_sz, [_vp]),
    "dnb_inet_param_offset": (C.c_int, [_vp, C.c_int, C.POINTER(_sz), C.POINTER(_sz)]),
    "dnb_inet_workspace_bytes": (_sz, [_vp]),
    "dnb_inet_peak_bytes": (_sz, [_vp]),
    "dnb_inet_set_concurrency": (C.c_int, [_vp, C.c_int]),
    "dnb_inet_forward": (C.c_int, [_vp] * 8),
    "dnb_inet_backward": (C.c_int, [_vp] * 6),
    "dnb_inet_relu_decision_bytes": (_sz, [_vp]),
    "dnb_inet_pool_position_bytes": (_sz, [_vp]),
    "dnb_inet_decisions": (C.c_int, [_vp] * 6),
    "dnb_op_head_forward": (C.c_int, [_vp] * 8 + [_i64, _i64, _i64, _vp]),
    "dnb_op_head_backward": (C.c_int, [_vp] * 6 + [_i64, _i64, _i64, _vp]),
    "dnb_op_stem_scratch_bytes": (_sz, [_i64, _i64, _i64]),
    "dnb_op_stem_conv7": (C.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp]),
    "dnb_op_stem_wgrad7": (C.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp]),
    "dnb_op_maxpool3s2_bnrelu": (C.c_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp]),
    "dnb_op_maxpool3s2_backward": (C.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(_lib, _name)
    _f.restype = _res
    _f.argtypes = _args

EXPORTED = tuple(_SIGS)


class DnbError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"dnb status {status}: {dnb_status_string(status)}")


def _check(status: int) -> None:
    if status != DNB_OK:
        raise DnbError(status)


def _ptr(t):
    """Device address of a torch tensor (or a raw int / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def dnb_status_string(status: int) -> str:
    return _lib.dnb_status_string(status).decode()


def dnb_block_create(n, c0, h, w, layers, growth, bottleneck, dtype=DNB_F32, layout=DNB_NCHW,
                     schedule=DNB_SCHED_SHARED, eps=1e-5):
    desc = dnb_block_desc(n, c0, h, w, layers, growth, bottleneck, dtype, layout, schedule, eps)
    out = _vp()
    _check(_lib.dnb_block_create(C.byref(desc), C.byref(out)))
    return out


def dnb_block_destroy(b) -> None:
    _lib.dnb_block_destroy(b)


def dnb_block_peak_bytes(b) -> int:
    return int(_lib.dnb_block_peak_bytes(b))


def dnb_block_workspace_bytes(b) -> int:
    return int(_lib.dnb_block_workspace_bytes(b))


def dnb_block_memory_breakdown(b) -> dict:
    m = dnb_block_memory()
    _check(_lib.dnb_block_memory_breakdown(b, C.byref(m)))
    return m.as_dict()


def dnb_block_param_count(b) -> int:
    return int(_lib.dnb_block_param_count(b))


def dnb_block_param_bytes(b) -> int:
    return int(_lib.dnb_block_param_bytes(b))


def dnb_block_param_offset(b, layer: int, which: int):
    off, cnt = _sz(), _sz()
    _check(_lib.dnb_block_param_offset(b, layer, which, C.byref(off), C.byref(cnt)))
    return int(off.value), int(cnt.value)


def dnb_block_forward(b, x0, params, y, workspace, stream=None) -> None:
    _check(_lib.dnb_block_forward(b, _ptr(x0), _ptr(params), _ptr(y), _ptr(workspace), _stream(stream)))


def dnb_block_backward(b, params, y, dy, dx0, dparams, workspace, stream=None) -> None:
    _check(_lib.dnb_block_backward(b, _ptr(params), _ptr(y), _ptr(dy), _ptr(dx0), _ptr(dparams),
                                   _ptr(workspace), _stream(stream)))


def dnb_block_relu_decision_bytes(b, which: int) -> int:
    return int(_lib.dnb_block_relu_decision_bytes(b, which))


def dnb_block_relu_decisions(b, params, y, workspace, d1, d2, stream=None) -> None:
    _check(_lib.dnb_block_relu_decisions(b, _ptr(params), _ptr(y), _ptr(workspace), _ptr(d1), _ptr(d2), _stream(stream)))


def dnb_block_set_concurrency(b, enable: bool) -> None:
    _check(_lib.dnb_block_set_concurrency(b, int(bool(enable))))


def dnb_op_copy_slab(src, src_stride, dst, dst_stride, n, length, stream=None) -> None:
    _check(_lib.dnb_op_copy_slab(_ptr(src), src_stride, _ptr(dst), dst_stride, n, length, _stream(stream)))


def dnb_op_bn_scratch_bytes(n, c, hw) -> int:
    return int(_lib.dnb_op_bn_scratch_bytes(n, c, hw))


def dnb_op_bn_stats(x, stride, n, c, hw, eps, mean, istd, scratch, stream=None) -> None:
    _check(_lib.dnb_op_bn_stats(_ptr(x), stride, n, c, hw, eps, _ptr(mean), _ptr(istd), _ptr(scratch),
                                _stream(stream)))


def dnb_op_bn_stats_static(x, stride, n, c, hw, eps, mean, istd, stream=None) -> None:
    _check(_lib.dnb_op_bn_stats_static(_ptr(x), stride, n, c, hw, eps, _ptr(mean), _ptr(istd), _stream(stream)))


def dnb_op_bn_relu(x, x_stride, out, out_stride, n, c, hw, gamma, beta, mean, istd, stream=None) -> None:
    _check(_lib.dnb_op_bn_relu(_ptr(x), x_stride, _ptr(out), out_stride, n, c, hw, _ptr(gamma), _ptr(beta),
                               _ptr(mean), _ptr(istd), _stream(stream)))


def dnb_op_bn_relu_backward(x, x_stride, dact, dact_stride, du, du_stride, accumulate, n, c, hw, gamma, beta,
                            mean, istd, dgamma, dbeta, scratch, stream=None) -> None:
    _check(_lib.dnb_op_bn_relu_backward(_ptr(x), x_stride, _ptr(dact), dact_stride, _ptr(du), du_stride,
                                        int(accumulate), n, c, hw, _ptr(gamma), _ptr(beta), _ptr(mean),
                                        _ptr(istd), _ptr(dgamma), _ptr(dbeta), _ptr(scratch), _stream(stream)))


def dnb_op_bn_relu_backward_apply(x, x_stride, dact, dact_stride, du, du_stride, accumulate, n, c, hw, gamma,
                                  beta, mean, istd, dgamma, dbeta, scratch, ev_start=None, ev_stop=None,
                                  stream=None) -> None:
    """ev_start / ev_stop: torch.cuda.Event(enable_timing=True) that have been recorded once (so their
    handles exist), or None; they are stamped at the kernel's own start and end."""
    h0 = ev_start.cuda_event if ev_start is not None else None
    h1 = ev_stop.cuda_event if ev_stop is not None else None
    _check(_lib.dnb_op_bn_relu_backward_apply(_ptr(x), x_stride, _ptr(dact), dact_stride, _ptr(du), du_stride,
                                              int(accumulate), n, c, hw, _ptr(gamma), _ptr(beta), _ptr(mean),
                                              _ptr(istd), _ptr(dgamma), _ptr(dbeta), _ptr(scratch), h0, h1,
                                              _stream(stream)))


def dnb_op_conv_scratch_bytes(cin, cout, ks) -> int:
    return int(_lib.dnb_op_conv_scratch_bytes(cin, cout, ks))


def dnb_op_conv_forward(x, x_stride, wgt, out, out_stride, n, cin, cout, h, w, ks, scratch, stream=None) -> None:
    _check(_lib.dnb_op_conv_forward(_ptr(x), x_stride, _ptr(wgt), _ptr(out), out_stride, n, cin, cout, h, w,
                                    ks, _ptr(scratch), _stream(stream)))


def dnb_op_conv_stats_bytes(n, cout, h, w) -> int:
    return int(_lib.dnb_op_conv_stats_bytes(n, cout, h, w))


def dnb_op_conv_bnrelu_forward(x, x_stride, wgt, fold, out, out_stride, stats, n, cin, cout, h, w, ks, scratch,
                               prepacked=False, ev_start=None, ev_stop=None, stream=None) -> int:
    """Returns the number of statistics tiles per output channel.  Events as in
    dnb_op_bn_relu_backward_apply."""
    tiles = C.c_int(0)
    h0 = ev_start.cuda_event if ev_start is not None else None
    h1 = ev_stop.cuda_event if ev_stop is not None else None
    _check(_lib.dnb_op_conv_bnrelu_forward(_ptr(x), x_stride, _ptr(wgt), _ptr(fold), _ptr(out), out_stride,
                                           _ptr(stats), C.byref(tiles), n, cin, cout, h, w, ks, _ptr(scratch),
                                           int(prepacked), h0, h1, _stream(stream)))
    return int(tiles.value)


def dnb_op_conv_bnrelu_wgrad(x, x_stride, fold, dout, dout_stride, dwgt, n, cin, cout, h, w, ks, scratch,
                             ev_start=None, ev_stop=None, stream=None) -> None:
    h0 = ev_start.cuda_event if ev_start is not None else None
    h1 = ev_stop.cuda_event if ev_stop is not None else None
    _check(_lib.dnb_op_conv_bnrelu_wgrad(_ptr(x), x_stride, _ptr(fold), _ptr(dout), dout_stride, _ptr(dwgt), n, cin,
                                         cout, h, w, ks, _ptr(scratch), h0, h1, _stream(stream)))


def dnb_op_conv_dgrad(dout, dout_stride, wgt, din, din_stride, n, cin, cout, h, w, ks, scratch, stream=None) -> None:
    _check(_lib.dnb_op_conv_dgrad(_ptr(dout), dout_stride, _ptr(wgt), _ptr(din), din_stride, n, cin, cout, h,
                                  w, ks, _ptr(scratch), _stream(stream)))


def dnb_op_layer_wgrads_scratch_bytes(n, cin, bottleneck, growth, h, w) -> int:
    return int(_lib.dnb_op_layer_wgrads_scratch_bytes(n, cin, bottleneck, growth, h, w))


def dnb_op_layer_wgrads_bn_partials_offset(n, cin, bottleneck, growth, h, w) -> int:
    return int(_lib.dnb_op_layer_wgrads_bn_partials_offset(n, cin, bottleneck, growth, h, w))


def dnb_op_layer_wgrads(x1, x1_stride, fold1, db, dw1, cin, b, fold2, g, g_stride, dw3, n, bottleneck, growth, h, w,
                        scratch, bn_dact=None, bn_gamma=None, bn_beta=None, bn_mean=None, bn_istd=None,
                        ev_start=None, ev_stop=None, stream=None) -> None:
    h0 = ev_start.cuda_event if ev_start is not None else None
    h1 = ev_stop.cuda_event if ev_stop is not None else None
    opt = lambda t: _ptr(t) if t is not None else None
    _check(_lib.dnb_op_layer_wgrads(_ptr(x1), x1_stride, _ptr(fold1), _ptr(db), _ptr(dw1), cin, _ptr(b), _ptr(fold2),
                                    _ptr(g), g_stride, _ptr(dw3), n, bottleneck, growth, h, w, opt(bn_dact),
                                    opt(bn_gamma), opt(bn_beta), opt(bn_mean), opt(bn_istd), _ptr(scratch), h0, h1,
                                    _stream(stream)))


def dnb_op_conv_wgrad_scratch_bytes(n, cin, cout, h, w, ks) -> int:
    return int(_lib.dnb_op_conv_wgrad_scratch_bytes(n, cin, cout, h, w, ks))


def dnb_op_conv_wgrad(x, x_stride, dout, dout_stride, dwgt, n, cin, cout, h, w, ks, scratch, stream=None) -> None:
    _check(_lib.dnb_op_conv_wgrad(_ptr(x), x_stride, _ptr(dout), dout_stride, _ptr(dwgt), n, cin, cout, h, w,
                                  ks, _ptr(scratch), _stream(stream)))


def dnb_op_nhwc_scratch_bytes(n, cin, cout, h, w, ks) -> int:
    return int(_lib.dnb_op_nhwc_scratch_bytes(n, cin, cout, h, w, ks))


def dnb_op_nhwc_conv_forward(x, x_ld, wgt, out, out_ld, n, cin, cout, h, w, ks, scratch, stream=None) -> None:
    _check(_lib.dnb_op_nhwc_conv_forward(_ptr(x), x_ld, _ptr(wgt), _ptr(out), out_ld, n, cin, cout, h, w, ks,
                                         _ptr(scratch), _stream(stream)))


def dnb_op_nhwc_conv_dgrad(dout, dout_ld, dout_is_f32, wgt, din, din_ld, n, cin, cout, h, w, ks, scratch,
                           stream=None) -> None:
    _check(_lib.dnb_op_nhwc_conv_dgrad(_ptr(dout), dout_ld, int(dout_is_f32), _ptr(wgt), _ptr(din), din_ld, n, cin,
                                       cout, h, w, ks, _ptr(scratch), _stream(stream)))


def dnb_op_nhwc_conv_wgrad(x, x_ld, dout, dout_ld, dout_is_f32, dwgt, n, cin, cout, h, w, ks, scratch,
                           stream=None) -> None:
    _check(_lib.dnb_op_nhwc_conv_wgrad(_ptr(x), x_ld, _ptr(dout), dout_ld, int(dout_is_f32), _ptr(dwgt), n, cin, cout,
                                       h, w, ks, _ptr(scratch), _stream(stream)))


def dnb_op_nhwc_bn_relu_backward(x, x_ld, dact, dact_ld, du_bf16, du_ld, du_accum_f32, acc_ld, pixels, c, gamma, beta,
                                 mean, istd, dgamma, dbeta, scratch, stream=None) -> None:
    _check(_lib.dnb_op_nhwc_bn_relu_backward(_ptr(x), x_ld, _ptr(dact), dact_ld, _ptr(du_bf16), du_ld,
                                             _ptr(du_accum_f32), acc_ld, pixels, c, _ptr(gamma), _ptr(beta),
                                             _ptr(mean), _ptr(istd), _ptr(dgamma), _ptr(dbeta), _ptr(scratch),
                                             _stream(stream)))


# ---------------------------------------------------------------- whole network step

def dnb_net_create(n, image, depth, growth, classes, schedule=DNB_SCHED_FUSED, eps=1e-5):
    desc = dnb_net_desc(n, image, depth, growth, classes, schedule, eps)
    out = _vp()
    _check(_lib.dnb_net_create(C.byref(desc), C.byref(out)))
    return out


def dnb_net_destroy(net) -> None:
    _lib.dnb_net_destroy(net)


def dnb_net_param_count(net) -> int:
    return int(_lib.dnb_net_param_count(net))


def dnb_net_param_offset(net, part: int):
    off, cnt = _sz(), _sz()
    _check(_lib.dnb_net_param_offset(net, part, C.byref(off), C.byref(cnt)))
    return int(off.value), int(cnt.value)


def dnb_net_workspace_bytes(net) -> int:
    return int(_lib.dnb_net_workspace_bytes(net))


def dnb_net_workspace_piece(net, i: int):
    """(name, block index, byte offset, bytes) of the i-th carved piece, or None past the last."""
    name, idx, off, nb = C.c_char_p(), C.c_int(), _sz(), _sz()
    rc = _lib.dnb_net_workspace_piece(net, i, C.byref(name), C.byref(idx), C.byref(off), C.byref(nb))
    if rc == DNB_E_RANGE:
        return None
    _check(rc)
    return name.value.decode(), int(idx.value), int(off.value), int(nb.value)


def dnb_net_peak_bytes(net) -> int:
    return int(_lib.dnb_net_peak_bytes(net))


def dnb_net_relu_decision_bytes(net) -> int:
    return int(_lib.dnb_net_relu_decision_bytes(net))


def dnb_net_relu_decisions(net, params, workspace, out, stream=None) -> None:
    _check(_lib.dnb_net_relu_decisions(net, _ptr(params), _ptr(workspace), _ptr(out), _stream(stream)))


def dnb_net_set_concurrency(net, enable: bool) -> None:
    _check(_lib.dnb_net_set_concurrency(net, 1 if enable else 0))


def dnb_net_forward(net, x, labels, params, loss, logits, workspace, stream=None) -> None:
    _check(_lib.dnb_net_forward(net, _ptr(x), _ptr(labels), _ptr(params), _ptr(loss), _ptr(logits),
                                _ptr(workspace), _stream(stream)))


def dnb_net_backward(net, x, params, dparams, workspace, stream=None) -> None:
    _check(_lib.dnb_net_backward(net, _ptr(x), _ptr(params), _ptr(dparams), _ptr(workspace), _stream(stream)))


DNB_IP_STEM_W, DNB_IP_STEM_G, DNB_IP_STEM_B, DNB_IP_BLOCK0, DNB_IP_TAIL_BL = 0, 1, 2, 3, 19


def dnb_inet_create(n, image, growth, layers, classes, schedule=DNB_SCHED_FUSED, eps=1e-5):
    desc = dnb_inet_desc(n, image, growth, (C.c_int32 * 4)(*layers), classes, schedule, eps)
    out = _vp()
    _check(_lib.dnb_inet_create(C.byref(desc), C.byref(out)))
    return out


def dnb_inet_destroy(net) -> None:
    _lib.dnb_inet_destroy(net)


def dnb_inet_param_count(net) -> int:
    return int(_lib.dnb_inet_param_count(net))


def dnb_inet_param_offset(net, part: int):
    off, cnt = _sz(), _sz()
    _check(_lib.dnb_inet_param_offset(net, part, C.byref(off), C.byref(cnt)))
    return int(off.value), int(cnt.value)


def dnb_inet_workspace_bytes(net) -> int:
    return int(_lib.dnb_inet_workspace_bytes(net))


def dnb_inet_peak_bytes(net) -> int:
    return int(_lib.dnb_inet_peak_bytes(net))


def dnb_inet_set_concurrency(net, enable: bool) -> None:
    _check(_lib.dnb_inet_set_concurrency(net, 1 if enable else 0))


def dnb_inet_forward(net, x, labels, params, loss, logits, workspace, stream=None) -> None:
    _check(_lib.dnb_inet_forward(net, _ptr(x), _ptr(labels), _ptr(params), _ptr(loss), _ptr(logits), _ptr(workspace),
                                 _stream(stream)))


def dnb_inet_backward(net, x, params, dparams, workspace, stream=None) -> None:
    _check(_lib.dnb_inet_backward(net, _ptr(x), _ptr(params), _ptr(dparams), _ptr(workspace), _stream(stream)))


def dnb_inet_relu_decision_bytes(net) -> int:
    return int(_lib.dnb_inet_relu_decision_bytes(net))


def dnb_inet_pool_position_bytes(net) -> int:
    return int(_lib.dnb_inet_pool_position_bytes(net))


def dnb_inet_decisions(net, params, workspace, relu, pool, stream=None) -> None:
    _check(_lib.dnb_inet_decisions(net, _ptr(params), _ptr(workspace), _ptr(relu), _ptr(pool), _stream(stream)))


def dnb_op_head_forward(pooled, wl, bl, labels, logits, dlogits, terms, loss, n, c, classes, stream=None) -> None:
    _check(_lib.dnb_op_head_forward(_ptr(pooled), _ptr(wl), _ptr(bl), _ptr(labels), _ptr(logits), _ptr(dlogits),
                                    _ptr(terms), _ptr(loss), n, c, classes, _stream(stream)))


def dnb_op_head_backward(dlogits, pooled, wl, dpooled, dwl, dbl, n, c, classes, stream=None) -> None:
    _check(_lib.dnb_op_head_backward(_ptr(dlogits), _ptr(pooled), _ptr(wl), _ptr(dpooled), _ptr(dwl), _ptr(dbl),
                                     n, c, classes, _stream(stream)))


def dnb_op_stem_scratch_bytes(n, image, channels) -> int:
    return int(_lib.dnb_op_stem_scratch_bytes(n, image, channels))


def dnb_op_stem_conv7(x, w, out, n, image, channels, scratch, stream=None) -> None:
    _check(_lib.dnb_op_stem_conv7(_ptr(x), _ptr(w), _ptr(out), n, image, channels, _ptr(scratch), _stream(stream)))


def dnb_op_stem_wgrad7(x, g, dw, n, image, channels, scratch, stream=None) -> None:
    _check(_lib.dnb_op_stem_wgrad7(_ptr(x), _ptr(g), _ptr(dw), n, image, channels, _ptr(scratch), _stream(stream)))


def dnb_op_maxpool3s2_bnrelu(s, fold, out, pos, n, h, w, c, stream=None) -> None:
    _check(_lib.dnb_op_maxpool3s2_bnrelu(_ptr(s), _ptr(fold), _ptr(out), _ptr(pos), n, h, w, c, _stream(stream)))


def dnb_op_maxpool3s2_backward(dout, pos, din, n, h, w, c, stream=None) -> None:
    _check(_lib.dnb_op_maxpool3s2_backward(_ptr(dout), _ptr(pos), _ptr(din), n, h, w, c, _stream(stream)))
