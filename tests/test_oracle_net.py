"""Pins for the CPU oracle's network glue (stem, transitions, pooling, linear head, softmax
cross-entropy) and whole training step, against things other than the oracle itself."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl

NAMES = wl.PARAM_NAMES
from harness import pack_net  # noqa: E402


def test_avgpool_and_global_pool_match_library_and_are_adjoint(oracle):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 3, 6, 4))
    got = oracle.avgpool2(x)
    assert np.allclose(got, F.avg_pool2d(torch.from_numpy(x), 2).numpy(), atol=1e-14)
    g = rng.standard_normal(got.shape)
    # <pool(x), g> = <x, pool^T(g)>
    assert np.isclose((got * g).sum(), (x * oracle.avgpool2_backward(g, 6, 4)).sum(), rtol=1e-12)
    gp = oracle.global_avgpool(x)
    assert np.allclose(gp, x.mean(axis=(2, 3)), atol=1e-14)
    h = rng.standard_normal(gp.shape)
    assert np.isclose((gp * h).sum(), (x * oracle.global_avgpool_backward(h, 6, 4)).sum(), rtol=1e-12)
    # hand case: one 2x2 window
    assert oracle.avgpool2(np.array([[[[1.0, 2.0], [3.0, 6.0]]]]))[0, 0, 0, 0] == 3.0


def test_linear_matches_matmul_and_its_gradients(oracle):
    rng = np.random.default_rng(1)
    f, w, b = rng.standard_normal((4, 7)), rng.standard_normal((3, 7)), rng.standard_normal(3)
    assert np.allclose(oracle.linear(f, w, b), f @ w.T + b, atol=1e-13)
    d = rng.standard_normal((4, 3))
    df, dw, db = oracle.linear_backward(f, w, d)
    assert np.allclose(df, d @ w, atol=1e-13) and np.allclose(dw, d.T @ f, atol=1e-13) and np.allclose(db, d.sum(0), atol=1e-13)


def test_softmax_cross_entropy_closed_forms(oracle):
    # uniform logits: loss = log(classes), gradient (1/classes - onehot)/n
    loss, d = oracle.softmax_xent(np.zeros((3, 5)), [0, 2, 4])
    assert np.isclose(loss, np.log(5.0), rtol=1e-14)
    ref = np.full((3, 5), 0.2 / 3)
    for i, l in enumerate([0, 2, 4]):
        ref[i, l] -= 1.0 / 3
    assert np.allclose(d, ref, atol=1e-15)
    # shift invariance, rows of the gradient sum to zero, large logits do not overflow
    rng = np.random.default_rng(2)
    z = rng.standard_normal((4, 6)) * 3
    lab = [1, 0, 5, 3]
    l1, d1 = oracle.softmax_xent(z, lab)
    l2, d2 = oracle.softmax_xent(z + 1000.0, lab)
    assert np.isclose(l1, l2, rtol=1e-10) and np.allclose(d1, d2, atol=1e-12)
    assert np.allclose(d1.sum(axis=1), 0.0, atol=1e-15)
    # library cross-check
    zt = torch.tensor(z, requires_grad=True)
    lt = F.cross_entropy(zt, torch.tensor(lab))
    lt.backward()
    assert np.isclose(l1, lt.item(), rtol=1e-12) and np.allclose(d1, zt.grad.numpy(), atol=1e-13)
    # a confident correct prediction costs almost nothing, a confident wrong one about the margin
    assert oracle.softmax_xent(np.array([[30.0, 0.0]]), [0])[0] < 1e-12
    assert np.isclose(oracle.softmax_xent(np.array([[30.0, 0.0]]), [1])[0], 30.0, rtol=1e-10)


def torch_net(cfg, x, labels, params, decisions=None):
    """The same network from library routines in float64 under autograd.  decisions: a flat byte
    array in the oracle's order (per block: first-BN decisions of all layers, second-BN decisions
    of all layers, decisions of the BN that follows the block); every ReLU then is a
    multiplication with its 0/1 tensor."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    P = {"stem": t(params["stem"])}
    for b in range(3):
        P[f"block{b}"] = [{k: t(v) for k, v in p.items()} for p in params[f"block{b}"]]
    for name in ("trans0", "trans1", "tail"):
        P[name] = {k: t(v) for k, v in params[name].items()}
    def bn(u, g, b, dec=None):
        z = F.batch_norm(u, None, None, g, b, True, 0.0, cfg.eps)
        return F.relu(z) if dec is None else z * torch.tensor(dec.reshape(z.shape).astype(np.float64))
    f = F.conv2d(torch.tensor(x, dtype=torch.float64), P["stem"], padding=1)
    B = 4 * cfg.growth
    pos = 0
    for b in range(3):
        feats = [f]
        n, _, hh, ww = f.shape
        px = n * hh * ww
        layers = P[f"block{b}"]
        widths = [f.shape[1] + l * cfg.growth for l in range(len(layers))]
        o1 = pos
        o2 = o1 + sum(widths) * px
        og = o2 + len(layers) * B * px
        for l, p in enumerate(layers):
            d1 = d2 = None
            if decisions is not None:
                d1 = decisions[o1:o1 + widths[l] * px]
                o1 += widths[l] * px
                d2 = decisions[o2 + l * B * px:o2 + (l + 1) * B * px]
            a = bn(torch.cat(feats, 1), p["g1"], p["b1"], d1)
            a2 = bn(F.conv2d(a, p["W1"].reshape(B, -1, 1, 1)), p["g2"], p["b2"], d2)
            feats.append(F.conv2d(a2, p["W3"], padding=1))
        y = torch.cat(feats, 1)
        dg = None if decisions is None else decisions[og:og + y.shape[1] * px]
        pos = og + y.shape[1] * px
        if b < 2:
            tr = P[f"trans{b}"]
            f = F.avg_pool2d(F.conv2d(bn(y, tr["g"], tr["b"], dg), tr["W"].reshape(tr["W"].shape[0], -1, 1, 1)), 2)
        else:
            tl = P["tail"]
            logits = F.linear(bn(y, tl["g"], tl["b"], dg).mean(dim=(2, 3)), tl["Wl"], tl["bl"])
    loss = F.cross_entropy(logits, torch.tensor(np.asarray(labels, dtype=np.int64)))
    loss.backward()
    return loss.item(), logits.detach().numpy(), P


@pytest.mark.parametrize("cfg", [wl.NetCfg(2, 8, 16, 4, 5), wl.NetCfg(3, 12, 10, 2, 3)], ids=["n2i8L16k4", "n3i12L10k2"])
def test_net_step_matches_library_autograd(oracle, cfg):
    """Loss, logits and the gradient of every parameter of the whole step against float64
    autograd over library conv / batch-norm / pooling / linear / cross-entropy routines."""
    x, labels, params = wl.make_net_inputs(cfg, affine="random")
    params["tail"]["bl"] = np.linspace(-0.3, 0.2, cfg.classes).astype(np.float32)
    s = oracle.NetShape(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, cfg.eps)
    flat = pack_net(oracle, s, params)
    loss, dflat, logits = oracle.net_step(s, x, labels, flat)
    tloss, tlogits, P = torch_net(cfg, x, labels, params)
    assert np.isclose(loss, tloss, rtol=1e-11)
    assert np.allclose(logits, tlogits, rtol=1e-9, atol=1e-11)
    sl = oracle.net_param_slices(s)
    close = lambda a, r, what: np.testing.assert_allclose(a, r.ravel(), rtol=1e-7, atol=1e-10, err_msg=what)
    close(dflat[sl["stem"]], P["stem"].grad.numpy(), "stem")
    for b in range(3):
        bs = s.block(b)
        blk = dflat[sl[f"block{b}"]]
        for l, p in enumerate(P[f"block{b}"], start=1):
            for name, tv in p.items():
                close(blk[oracle.param_slice(bs, l, NAMES.index(name))], tv.grad.numpy(), f"block{b} layer {l} {name}")
    for pre in ("trans0", "trans1", "tail"):
        for name, tv in P[pre].items():
            close(dflat[sl[f"{pre}.{name}"]], tv.grad.numpy(), f"{pre}.{name}")


@pytest.mark.parametrize("cfg", [wl.NetCfg(2, 8, 16, 4, 5), wl.NetCfg(3, 12, 10, 2, 3)], ids=["n2i8L16k4", "n3i12L10k2"])
def test_net_step_with_given_relu_decisions(oracle, cfg):
    """The step's own decisions fed back reproduce the plain step bit for bit with no disagreement;
    with a twentieth of all decisions inverted the step equals autograd of the network whose ReLUs
    are multiplications with the given 0/1 tensors."""
    x, labels, params = wl.make_net_inputs(cfg, affine="random")
    s = oracle.NetShape(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, cfg.eps)
    flat = pack_net(oracle, s, params)
    loss, dflat, logits = oracle.net_step(s, x, labels, flat)
    l0, d0, g0, dec = oracle.net_step_with_decisions(s, x, labels, flat)
    assert dec.size == oracle.net_decision_count(s)
    assert l0 == loss and np.array_equal(d0, dflat) and np.array_equal(g0, logits)
    l1, d1, g1, st = oracle.net_step_with_decisions(s, x, labels, flat, dec)
    assert st == dict(count=0, margin=0.0)
    assert l1 == loss and np.array_equal(d1, dflat) and np.array_equal(g1, logits)
    r = np.random.default_rng(8)
    forced = dec ^ (r.random(dec.size) < 0.05).astype(np.uint8)
    l2, d2, g2, st = oracle.net_step_with_decisions(s, x, labels, flat, forced)
    assert st["count"] > 0 and not np.allclose(d2, dflat, atol=1e-6)
    tloss, tlogits, P = torch_net(cfg, x, labels, params, forced)
    assert np.isclose(l2, tloss, rtol=1e-11)
    assert np.allclose(g2, tlogits, rtol=1e-9, atol=1e-11)
    sl = oracle.net_param_slices(s)
    close = lambda a, r_, what: np.testing.assert_allclose(a, r_.ravel(), rtol=1e-7, atol=1e-10, err_msg=what)
    close(d2[sl["stem"]], P["stem"].grad.numpy(), "stem")
    for b in range(3):
        bs = s.block(b)
        blk = d2[sl[f"block{b}"]]
        for l, p in enumerate(P[f"block{b}"], start=1):
            for name, tv in p.items():
                close(blk[oracle.param_slice(bs, l, NAMES.index(name))], tv.grad.numpy(), f"block{b} layer {l} {name}")
    for pre in ("trans0", "trans1", "tail"):
        for name, tv in P[pre].items():
            close(d2[sl[f"{pre}.{name}"]], tv.grad.numpy(), f"{pre}.{name}")


def test_net_loss_decreases_along_negative_gradient(oracle):
    """First-order check independent of any library: loss(p - h*g) = loss(p) - h*|g|^2 + O(h^2)."""
    cfg = wl.NetCfg(2, 8, 16, 4, 5)
    x, labels, params = wl.make_net_inputs(cfg, affine="random")
    s = oracle.NetShape(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, cfg.eps)
    flat = pack_net(oracle, s, params)
    loss, g, _ = oracle.net_step(s, x, labels, flat)
    h = 1e-6 / np.linalg.norm(g)
    lp, _, _ = oracle.net_step(s, x, labels, flat + h * g, backward=False)
    lm, _, _ = oracle.net_step(s, x, labels, flat - h * g, backward=False)
    assert np.isclose((lp - lm) / (2 * h), np.dot(g, g), rtol=1e-5)
