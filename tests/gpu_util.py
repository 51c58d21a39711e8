"""Helpers for the GPU parity tests: marshal numpy inputs to device tensors, call the
C ABI through the binding, bring results back.  No arithmetic of the method here."""
import numpy as np
import torch

import workloads as wl

NAMES = wl.PARAM_NAMES


def rel_errors(a, r):
    """(L2 relative error, max-abs error relative to max |r|) of a against reference r."""
    a = np.asarray(a, dtype=np.float64).ravel()
    r = np.asarray(r, dtype=np.float64).ravel()
    den2 = np.linalg.norm(r)
    denm = np.max(np.abs(r)) if r.size else 0.0
    l2 = np.linalg.norm(a - r) / den2 if den2 > 0 else np.linalg.norm(a - r)
    mx = np.max(np.abs(a - r)) / denm if denm > 0 else (np.max(np.abs(a - r)) if r.size else 0.0)
    return float(l2), float(mx)


def assert_close(a, r, tol, what=""):
    l2, mx = rel_errors(a, r)
    assert l2 <= tol and mx <= tol, f"{what}: rel L2 {l2:.3e}, rel max {mx:.3e} > {tol:g}"


def dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device="cuda", dtype=dtype)


def pack_params_gpu(dnb, handle, layer_params):
    flat = np.zeros(dnb.dnb_block_param_count(handle), dtype=np.float32)
    for l, p in enumerate(layer_params, start=1):
        for name, arr in p.items():
            off, cnt = dnb.dnb_block_param_offset(handle, l, NAMES.index(name))
            assert cnt == arr.size
            flat[off:off + cnt] = arr.ravel()
    return flat


def pack_params_oracle(orc, shape, layer_params):
    flat = np.zeros(orc.param_count(shape))
    for l, p in enumerate(layer_params, start=1):
        for name, arr in p.items():
            flat[orc.param_slice(shape, l, NAMES.index(name))] = np.asarray(arr, dtype=np.float64).ravel()
    return flat


def run_block_gpu(dnb, cfg, x0, layer_params, dy, schedule=0, poison=True, concurrency=None):
    """Forward + backward of one block through the C ABI.  Returns dict of numpy arrays.
    concurrency=None keeps the library's default (what bench.py times)."""
    h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck,
                             schedule=schedule, eps=cfg.eps)
    try:
        if concurrency is not None:
            dnb.dnb_block_set_concurrency(h, concurrency)
        params = dev(pack_params_gpu(dnb, h, layer_params))
        ws_bytes = dnb.dnb_block_workspace_bytes(h)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        y = torch.empty((cfg.n, cfg.c_out, cfg.h, cfg.w), dtype=torch.float32, device="cuda")
        dx0 = torch.empty((cfg.n, cfg.c0, cfg.h, cfg.w), dtype=torch.float32, device="cuda")
        dparams = torch.empty_like(params)
        if poison:  # stale contents must never leak into results
            ws.fill_(0xFF)
            y.fill_(float("nan"))
            dx0.fill_(float("nan"))
            dparams.fill_(float("nan"))
        x0d, dyd = dev(x0), dev(dy)
        dnb.dnb_block_forward(h, x0d, params, y, ws)
        dnb.dnb_block_backward(h, params, y, dyd, dx0, dparams, ws)
        torch.cuda.synchronize()
        out = {"y": y.cpu().numpy(), "dx0": dx0.cpu().numpy(), "dparams": dparams.cpu().numpy(),
               "mem": dnb.dnb_block_memory_breakdown(h), "peak": dnb.dnb_block_peak_bytes(h)}
        out["slices"] = {(l, name): slice(*(lambda o, c: (o, o + c))(*dnb.dnb_block_param_offset(h, l, NAMES.index(name))))
                         for l in range(1, cfg.layers + 1) for name in NAMES if name in layer_params[0]}
        return out
    finally:
        dnb.dnb_block_destroy(h)


def run_block_oracle(orc, cfg, x0, layer_params, dy, schedule="naive"):
    s = orc.BlockShape(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck, cfg.eps)
    params = pack_params_oracle(orc, s, layer_params)
    res = orc.block(s, x0.astype(np.float64), params, dy.astype(np.float64), schedule=schedule)
    slices = {(l, name): orc.param_slice(s, l, NAMES.index(name))
              for l in range(1, cfg.layers + 1) for name in NAMES if name in layer_params[0]}
    return res, slices
