"""Harness helpers shared by the tests, bench.py and the smoke check: marshal numpy inputs to device
tensors, pack named parameter tensors into the flat packs of the library and of the oracle, call
the C ABI through the binding, bring results back, compare.  No arithmetic of the method here."""
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


def run_block_gpu(dnb, cfg, x0, layer_params, dy, schedule=0, poison=True, concurrency=None, decisions=False):
    """Forward + backward of one block through the C ABI.  Returns dict of numpy arrays.
    concurrency=None keeps the library's default (what bench.py times).  decisions=True also
    brings back the ReLU decisions the kernels took ("d1", "d2": bytes, the block's own layout)."""
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
        dec = None
        if decisions:   # between forward and backward, as a caller checking a step would take them
            dec = [torch.full((max(dnb.dnb_block_relu_decision_bytes(h, w), 1),), 7, dtype=torch.uint8, device="cuda")
                   for w in (1, 2)]
            dnb.dnb_block_relu_decisions(h, params, y, ws, dec[0], dec[1])
        dnb.dnb_block_backward(h, params, y, dyd, dx0, dparams, ws)
        torch.cuda.synchronize()
        out = {"y": y.cpu().numpy(), "dx0": dx0.cpu().numpy(), "dparams": dparams.cpu().numpy(),
               "mem": dnb.dnb_block_memory_breakdown(h), "peak": dnb.dnb_block_peak_bytes(h)}
        if decisions:
            out["d1"] = dec[0].cpu().numpy()[:dnb.dnb_block_relu_decision_bytes(h, 1)]
            out["d2"] = dec[1].cpu().numpy()[:dnb.dnb_block_relu_decision_bytes(h, 2)]
        out["slices"] = {(l, name): slice(*(lambda o, c: (o, o + c))(*dnb.dnb_block_param_offset(h, l, NAMES.index(name))))
                         for l in range(1, cfg.layers + 1) for name in NAMES if name in layer_params[0]}
        return out
    finally:
        dnb.dnb_block_destroy(h)


def run_block_oracle(orc, cfg, x0, layer_params, dy, schedule="naive", decisions=None, bf16_storage=False):
    """The oracle's block on the same inputs.  decisions=(d1, d2): the float64 block evaluated with
    these ReLU decisions instead of its own; returns (result, slices, stats) then."""
    s = orc.BlockShape(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck, cfg.eps)
    params = pack_params_oracle(orc, s, layer_params)
    if decisions is not None:
        res, stats = orc.block_with_decisions(s, x0.astype(np.float64), params, dy.astype(np.float64), decisions,
                                              bf16_storage=bf16_storage)
        slices = {(l, name): orc.param_slice(s, l, NAMES.index(name))
                  for l in range(1, cfg.layers + 1) for name in NAMES if name in layer_params[0]}
        return res, slices, stats
    res = orc.block(s, x0.astype(np.float64), params, dy.astype(np.float64), schedule=schedule)
    slices = {(l, name): orc.param_slice(s, l, NAMES.index(name))
              for l in range(1, cfg.layers + 1) for name in NAMES if name in layer_params[0]}
    return res, slices


def pack_net(orc, s, params):
    """Named tensors of workloads.make_net_inputs -> the oracle's flat network pack."""
    flat = np.zeros(orc.net_param_count(s))
    sl = orc.net_param_slices(s)
    flat[sl["stem"]] = params["stem"].ravel()
    for b in range(3):
        bs = s.block(b)
        blk = np.zeros(orc.param_count(bs))
        for l, p in enumerate(params[f"block{b}"], start=1):
            for name, arr in p.items():
                blk[orc.param_slice(bs, l, NAMES.index(name))] = arr.ravel()
        flat[sl[f"block{b}"]] = blk
        pre = f"trans{b}" if b < 2 else "tail"
        for name, arr in params[pre].items():
            flat[sl[f"{pre}.{name}"]] = arr.ravel()
    return flat


def run_net_gpu(dnb, oracle, cfg, x, labels, params, schedule, concurrency=None, decisions=False):
    s = oracle.NetShape(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, cfg.eps)
    flat = pack_net(oracle, s, params)   # the two packs have the same layout (checked by the host tests)
    net = dnb.dnb_net_create(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, schedule=schedule, eps=cfg.eps)
    try:
        if concurrency is not None:   # None: the library's default, what bench.py times
            dnb.dnb_net_set_concurrency(net, concurrency)
        p = dev(flat.astype(np.float32))
        dp = torch.full_like(p, float("nan"))
        guard = 1 << 20   # a band behind the workspace that must come back untouched
        nbytes = dnb.dnb_net_workspace_bytes(net)
        ws = torch.empty(nbytes + guard, dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        xd = dev(x)
        lab = torch.from_numpy(labels).to("cuda")
        loss = torch.full((1,), float("nan"), device="cuda")
        logits = torch.full((cfg.n, cfg.classes), float("nan"), device="cuda")
        dnb.dnb_net_forward(net, xd, lab, p, loss, logits, ws)
        dec = None
        if decisions:   # the ReLU decisions the kernels take, between forward and backward
            dec = torch.full((dnb.dnb_net_relu_decision_bytes(net),), 7, dtype=torch.uint8, device="cuda")
            dnb.dnb_net_relu_decisions(net, p, ws, dec)
        dnb.dnb_net_backward(net, xd, p, dp, ws)
        torch.cuda.synchronize()
        assert bool((ws[nbytes:] == 0xFF).all()), "the step wrote behind its workspace"
        if decisions:
            return s, flat, float(loss.item()), logits.cpu().numpy(), dp.cpu().numpy(), dec.cpu().numpy()
        return s, flat, float(loss.item()), logits.cpu().numpy(), dp.cpu().numpy()
    finally:
        dnb.dnb_net_destroy(net)


def pack_inet(orc, s, params):
    """Named tensors of workloads.make_inet_inputs -> the oracle's flat pack of the ImageNet-shaped network."""
    flat = np.zeros(orc.inet_param_count(s))
    sl = orc.inet_param_slices(s)
    for name in ("W", "g", "b"):
        flat[sl[f"stem.{name}"]] = params["stem"][name].ravel()
    for b in range(4):
        bs = s.block(b)
        blk = np.zeros(orc.param_count(bs))
        for l, p in enumerate(params[f"block{b}"], start=1):
            for name, arr in p.items():
                blk[orc.param_slice(bs, l, NAMES.index(name))] = arr.ravel()
        flat[sl[f"block{b}"]] = blk
        pre = f"trans{b}" if b < 3 else "tail"
        for name, arr in params[pre].items():
            flat[sl[f"{pre}.{name}"]] = arr.ravel()
    return flat


def run_inet_gpu(dnb, oracle, cfg, x, labels, params, schedule=2, decisions=False):
    """One training step of the ImageNet-shaped network through the C ABI (x: (n,3,S,S) float32 holding
    bf16 values).  Returns (shape, flat oracle pack, loss, logits, dparams[, (relu, pool)]); the
    decision bytes come back in the oracle's (n, c, h, w) order."""
    s = oracle.InetShape(cfg.n, cfg.image, cfg.growth, tuple(cfg.layers), cfg.classes, cfg.eps)
    flat = pack_inet(oracle, s, params)   # the two packs have the same layout (checked by the host tests)
    net = dnb.dnb_inet_create(cfg.n, cfg.image, cfg.growth, cfg.layers, cfg.classes, schedule=schedule, eps=cfg.eps)
    try:
        assert dnb.dnb_inet_param_count(net) == flat.size
        p = dev(flat.astype(np.float32))
        dp = torch.full_like(p, float("nan"))
        guard = 1 << 20
        nbytes = dnb.dnb_inet_workspace_bytes(net)
        ws = torch.empty(nbytes + guard, dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        xd = torch.from_numpy(np.ascontiguousarray(x)).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)
        lab = torch.from_numpy(labels).to("cuda")
        loss = torch.full((1,), float("nan"), device="cuda")
        logits = torch.full((cfg.n, cfg.classes), float("nan"), device="cuda")
        dnb.dnb_inet_forward(net, xd, lab, p, loss, logits, ws)
        dec = None
        if decisions:
            relu = torch.full((dnb.dnb_inet_relu_decision_bytes(net),), 7, dtype=torch.uint8, device="cuda")
            pool = torch.full((dnb.dnb_inet_pool_position_bytes(net),), 77, dtype=torch.uint8, device="cuda")
            dnb.dnb_inet_decisions(net, p, ws, relu, pool)
        dnb.dnb_inet_backward(net, xd, p, dp, ws)
        torch.cuda.synchronize()
        assert bool((ws[nbytes:] == 0xFF).all()), "the step wrote behind its workspace"
        out = [s, flat, float(loss.item()), logits.cpu().numpy(), dp.cpu().numpy()]
        if decisions:
            relu, pool = relu.cpu().numpy(), pool.cpu().numpy()
            # (n, h, w, c) per tensor -> (n, c, h, w), tensors in the same order
            pieces, o = [], 0
            def take(n_, h, w, c):
                nonlocal o
                cnt = n_ * h * w * c
                pieces.append(relu[o:o + cnt].reshape(n_, h, w, c).transpose(0, 3, 1, 2).ravel())
                o += cnt
            S2, S4, cs = cfg.image // 2, cfg.image // 4, 2 * cfg.growth
            take(cfg.n, S2, S2, cs)
            for bc in cfg.blocks():
                for l in range(1, bc.layers + 1):
                    take(bc.n, bc.h, bc.w, bc.c_in(l))
                for l in range(1, bc.layers + 1):
                    take(bc.n, bc.h, bc.w, bc.bottleneck)
                take(bc.n, bc.h, bc.w, bc.c_out)
            assert o == relu.size
            out.append((np.concatenate(pieces), pool.reshape(cfg.n, S4, S4, cs).transpose(0, 3, 1, 2).ravel()))
        return tuple(out)
    finally:
        dnb.dnb_inet_destroy(net)
