"""Pins for the CPU oracle's ImageNet-shaped network (7x7 stride-2 stem, 3x3 stride-2 max pool, four
dense blocks, transitions, head) against things other than the oracle itself: library routines in
float64, brute force, adjoint identities, hand cases, autograd of the whole step, the paper's
printed model sizes."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl
from harness import NAMES, pack_inet


def test_strided_conv_matches_library_brute_force_and_adjoints(oracle):
    r = np.random.default_rng(0)
    for (n, ci, co, h, w, ks, st, pad) in ((2, 3, 5, 12, 10, 7, 2, 3), (1, 2, 3, 7, 9, 3, 2, 1), (2, 4, 2, 6, 6, 1, 1, 0)):
        x = r.standard_normal((n, ci, h, w))
        wgt = r.standard_normal((co, ci, ks, ks))
        out = oracle.conv_forward_strided(x, wgt, st, pad)
        ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(wgt), stride=st, padding=pad).numpy()
        assert out.shape == ref.shape
        np.testing.assert_allclose(out, ref, atol=1e-12)
        # brute force on a padded copy, one output at a time
        xp = np.zeros((n, ci, h + 2 * pad, w + 2 * pad))
        xp[:, :, pad:pad + h, pad:pad + w] = x
        for (b, o, y, xx) in ((0, 0, 0, 0), (n - 1, co - 1, out.shape[2] - 1, out.shape[3] - 1), (0, co // 2, 1, 2)):
            v = sum(wgt[o, c, i, j] * xp[b, c, y * st + i, xx * st + j] for c in range(ci) for i in range(ks) for j in range(ks))
            assert abs(out[b, o, y, xx] - v) < 1e-12
        g = r.standard_normal(out.shape)
        dw = oracle.conv_wgrad_strided(x, g, ks, st, pad)
        dx = oracle.conv_dgrad_strided(g, wgt, h, w, st, pad)
        # <conv(x, W), g> = <x, dgrad(g, W)> = <W, wgrad(x, g)>
        lhs = float((out * g).sum())
        assert np.isclose(lhs, float((x * dx).sum()), rtol=1e-11)
        assert np.isclose(lhs, float((wgt * dw).sum()), rtol=1e-11)
    # a single non-zero tap shifts and subsamples the image: orientation, stride and padding at once
    x = r.standard_normal((1, 1, 8, 8))
    wgt = np.zeros((1, 1, 7, 7))
    wgt[0, 0, 1, 5] = 1.0
    out = oracle.conv_forward_strided(x, wgt, 2, 3)
    for y in range(4):
        for xx in range(4):
            yy, xc = 2 * y + 1 - 3, 2 * xx + 5 - 3
            want = x[0, 0, yy, xc] if 0 <= yy < 8 and 0 <= xc < 8 else 0.0
            assert out[0, 0, y, xx] == want


def test_max_pool_hand_case_ties_library_and_adjoint(oracle):
    # one 4x4 plane: windows of the 2x2 output (pad 1), hand-enumerated, with ties
    x = np.array([[1., 5., 5., 0.],
                  [2., 5., 3., 7.],
                  [0., 1., 7., 7.],
                  [4., 4., 2., 7.]]).reshape(1, 1, 4, 4)
    out, idx = oracle.maxpool3s2(x)
    # output (0,0): rows -1..1, cols -1..1 -> values {1,5,2,5}: first 5 at row 0 col 1 -> window position 3*1+2
    # output (0,1): rows -1..1, cols 1..3 -> {5,5,0,5,3,7}: 7 at row 1 col 3 -> position 3*2+2
    # output (1,0): rows 1..3, cols -1..1 -> {2,5,0,1,4,4}: 5 at row 1 col 1 -> position 3*0+2
    # output (1,1): rows 1..3, cols 1..3 -> {5,3,7,1,7,7,4,2,7}: first 7 at row 1 col 3 -> position 3*0+2
    assert out.reshape(-1).tolist() == [5.0, 7.0, 5.0, 7.0]
    assert idx.reshape(-1).tolist() == [5, 8, 2, 2]
    g = np.array([10., 20., 30., 40.]).reshape(1, 1, 2, 2)
    din = oracle.maxpool3s2_backward(g, idx, 4, 4)
    want = np.zeros((4, 4))
    want[0, 1] += 10.0
    want[1, 3] += 20.0 + 40.0
    want[1, 1] += 30.0
    assert np.array_equal(din[0, 0], want)
    # library routine on random data (no ties), forward and gradient
    r = np.random.default_rng(1)
    x = r.standard_normal((2, 3, 10, 12))
    out, idx = oracle.maxpool3s2(x)
    xt = torch.tensor(x, requires_grad=True)
    ref = F.max_pool2d(xt, 3, 2, 1)
    np.testing.assert_array_equal(out, ref.detach().numpy())
    g = r.standard_normal(out.shape)
    (ref * torch.tensor(g)).sum().backward()
    np.testing.assert_allclose(oracle.maxpool3s2_backward(g, idx, 10, 12), xt.grad.numpy(), atol=1e-15)
    # imposed positions: the pool's own give no difference; moved ones are counted with the right margin
    same, st = oracle.maxpool3s2(x, idx)
    assert np.array_equal(same, out) and st == (0, 0.0)
    forced = idx.copy()
    forced[0, 0, 2, 3] = (int(idx[0, 0, 2, 3]) + 1) % 9
    got, (cnt, margin) = oracle.maxpool3s2(x, forced, inv_rms=np.full(3, 0.5))
    p = int(forced[0, 0, 2, 3])
    v = x[0, 0, 2 * 2 + p // 3 - 1, 2 * 3 + p % 3 - 1]
    assert cnt == 1 and got[0, 0, 2, 3] == v and np.isclose(margin, (out[0, 0, 2, 3] - v) * 0.5)


def torch_inet(cfg, x, labels, params, decisions=None):
    """The same network from library routines in float64 under autograd.  decisions = (relu, pool):
    every ReLU is a multiplication with its 0/1 tensor and the max pool gathers the given window
    positions (the oracle's order: stem BN; per block first-BN decisions, second-BN decisions,
    decisions of the BN that follows the block)."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    P = {"stem": {k: t(v) for k, v in params["stem"].items()}}
    for b in range(4):
        P[f"block{b}"] = [{k: t(v) for k, v in p.items()} for p in params[f"block{b}"]]
    for name in ("trans0", "trans1", "trans2", "tail"):
        P[name] = {k: t(v) for k, v in params[name].items()}
    pos = [0]

    def bn(u, g, b):
        z = F.batch_norm(u, None, None, g, b, True, 0.0, cfg.eps)
        if decisions is None:
            return F.relu(z)
        cnt = z.numel()
        d = decisions[0][pos[0]:pos[0] + cnt].reshape(z.shape).astype(np.float64)
        pos[0] += cnt
        return z * torch.tensor(d)

    s = F.conv2d(torch.tensor(x, dtype=torch.float64), P["stem"]["W"], stride=2, padding=3)
    a0 = bn(s, P["stem"]["g"], P["stem"]["b"])
    if decisions is None:
        f = F.max_pool2d(a0, 3, 2, 1)
    else:
        n, c, h, w = a0.shape
        idx = torch.tensor(decisions[1].reshape(n, c, h // 2, w // 2).astype(np.int64))
        ap = F.pad(a0, (1, 1, 1, 1))
        yy = 2 * torch.arange(h // 2).view(1, 1, -1, 1) + idx // 3
        xx = 2 * torch.arange(w // 2).view(1, 1, 1, -1) + idx % 3
        f = ap.reshape(n, c, -1).gather(2, (yy * (w + 2) + xx).reshape(n, c, -1)).reshape(n, c, h // 2, w // 2)
    B = 4 * cfg.growth
    for b in range(4):
        feats = [f]
        layers = P[f"block{b}"]
        if decisions is not None:
            # first-BN decisions of all layers come first, then the second-BN ones: walk two cursors
            px = f.shape[0] * f.shape[2] * f.shape[3]
            widths = [f.shape[1] + l * cfg.growth for l in range(len(layers))]
            o1, o2 = pos[0], pos[0] + sum(widths) * px
        for l, p in enumerate(layers):
            u = torch.cat(feats, 1)
            if decisions is None:
                a = bn(u, p["g1"], p["b1"])
                a2 = bn(F.conv2d(a, p["W1"].reshape(B, -1, 1, 1)), p["g2"], p["b2"])
            else:
                pos[0] = o1
                a = bn(u, p["g1"], p["b1"])
                o1 = pos[0]
                pos[0] = o2
                a2 = bn(F.conv2d(a, p["W1"].reshape(B, -1, 1, 1)), p["g2"], p["b2"])
                o2 = pos[0]
            feats.append(F.conv2d(a2, p["W3"], padding=1))
        if decisions is not None:
            pos[0] = o2
        y = torch.cat(feats, 1)
        if b < 3:
            tr = P[f"trans{b}"]
            f = F.avg_pool2d(F.conv2d(bn(y, tr["g"], tr["b"]), tr["W"].reshape(tr["W"].shape[0], -1, 1, 1)), 2)
        else:
            tl = P["tail"]
            logits = F.linear(bn(y, tl["g"], tl["b"]).mean(dim=(2, 3)), tl["Wl"], tl["bl"])
    loss = F.cross_entropy(logits, torch.tensor(np.asarray(labels, dtype=np.int64)))
    loss.backward()
    return loss.item(), logits.detach().numpy(), P


def compare_with_autograd(oracle, s, dflat, P):
    sl = oracle.inet_param_slices(s)
    close = lambda a, r, what: np.testing.assert_allclose(a, r.ravel(), rtol=1e-7, atol=1e-10, err_msg=what)
    for name in ("W", "g", "b"):
        close(dflat[sl[f"stem.{name}"]], P["stem"][name].grad.numpy(), f"stem.{name}")
    for b in range(4):
        bs = s.block(b)
        blk = dflat[sl[f"block{b}"]]
        for l, p in enumerate(P[f"block{b}"], start=1):
            for name, tv in p.items():
                close(blk[oracle.param_slice(bs, l, NAMES.index(name))], tv.grad.numpy(), f"block{b} layer {l} {name}")
    for pre in ("trans0", "trans1", "trans2", "tail"):
        for name, tv in P[pre].items():
            close(dflat[sl[f"{pre}.{name}"]], tv.grad.numpy(), f"{pre}.{name}")


CFGS = [wl.InetCfg(2, 32, 4, (2, 1, 2, 1), 5), wl.InetCfg(3, 64, 2, (1, 2, 1, 2), 3)]


@pytest.mark.parametrize("cfg", CFGS, ids=["n2i32k4", "n3i64k2"])
def test_inet_step_matches_library_autograd(oracle, cfg):
    x, labels, params = wl.make_inet_inputs(cfg, affine="random")
    params["tail"]["bl"] = np.linspace(-0.3, 0.2, cfg.classes).astype(np.float32)
    s = oracle.InetShape(cfg.n, cfg.image, cfg.growth, cfg.layers, cfg.classes, cfg.eps)
    flat = pack_inet(oracle, s, params)
    loss, dflat, logits = oracle.inet_step(s, x, labels, flat)
    tloss, tlogits, P = torch_inet(cfg, x, labels, params)
    assert np.isclose(loss, tloss, rtol=1e-11)
    assert np.allclose(logits, tlogits, rtol=1e-9, atol=1e-11)
    compare_with_autograd(oracle, s, dflat, P)


@pytest.mark.parametrize("cfg", CFGS, ids=["n2i32k4", "n3i64k2"])
def test_inet_step_with_given_decisions(oracle, cfg):
    """The step's own ReLU decisions and pooling positions fed back reproduce the plain step bit for
    bit with nothing reported; with a twentieth of the ReLU decisions inverted and a twentieth of the
    pooling positions moved to another position inside the image the step equals autograd of the
    network that multiplies with the given 0/1 tensors and gathers the given positions."""
    x, labels, params = wl.make_inet_inputs(cfg, affine="random")
    s = oracle.InetShape(cfg.n, cfg.image, cfg.growth, cfg.layers, cfg.classes, cfg.eps)
    flat = pack_inet(oracle, s, params)
    loss, dflat, logits = oracle.inet_step(s, x, labels, flat)
    l0, d0, g0, (relu, pool) = oracle.inet_step(s, x, labels, flat, decisions="write")
    assert (relu.size, pool.size) == oracle.inet_decision_counts(s)
    assert l0 == loss and np.array_equal(d0, dflat) and np.array_equal(g0, logits)
    l1, d1, g1, st = oracle.inet_step(s, x, labels, flat, decisions=(relu, pool))
    assert st == dict(relu_count=0, relu_margin=0.0, pool_count=0, pool_margin=0.0)
    assert l1 == loss and np.array_equal(d1, dflat) and np.array_equal(g1, logits)
    r = np.random.default_rng(8)
    forced = relu ^ (r.random(relu.size) < 0.05).astype(np.uint8)
    moved = pool.copy()
    pick = r.random(pool.size) < 0.05
    moved[pick] = 4          # the window's centre is inside the image for every output
    l2, d2, g2, st = oracle.inet_step(s, x, labels, flat, decisions=(forced, moved))
    # (the counts are not those of the inversions: with decisions imposed upstream the step's own
    # decisions downstream are no longer the plain step's)
    assert st["relu_count"] > 0 and st["pool_count"] > 0 and st["pool_margin"] > 0
    tloss, tlogits, P = torch_inet(cfg, x, labels, params, (forced, moved))
    assert np.isclose(l2, tloss, rtol=1e-11)
    assert np.allclose(g2, tlogits, rtol=1e-9, atol=1e-11)
    compare_with_autograd(oracle, s, d2, P)


def test_inet_pack_sizes_match_the_papers_model_sizes(oracle):
    """The ImageNet models of Section 5: 161 layers k = 48 (6-12-36-24) 29 M parameters, 264 layers
    k = 32 (6-12-64-48) 33 M, k = 48 73 M -- reproduced by the network pack's own size."""
    for layers, k, printed, tol in (((6, 12, 36, 24), 48, 29e6, 0.6e6), ((6, 12, 64, 48), 32, 33e6, 0.6e6),
                                    ((6, 12, 64, 48), 48, 73e6, 0.8e6)):
        s = oracle.InetShape(1, 224, k, layers, 1000)
        assert abs(oracle.inet_param_count(s) - printed) <= tol
        sl = oracle.inet_param_slices(s)
        assert sl["tail.bl"].stop == oracle.inet_param_count(s)


def test_bf16_storage_step_stays_close_to_the_plain_step(oracle):
    """The storage-rounding variant of the step (what bf16 storage costs by itself) under the plain
    step's decisions is a different evaluation (it does round) that stays within a few per cent in
    loss, logits and gradients on a small network."""
    cfg = wl.InetCfg(8, 64, 8, (2, 2, 2, 2), 10)
    x, labels, params = wl.make_inet_inputs(cfg, affine="random")
    s = oracle.InetShape(cfg.n, cfg.image, cfg.growth, cfg.layers, cfg.classes, cfg.eps)
    flat = pack_inet(oracle, s, params)
    xq = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    loss, dflat, logits, dec = oracle.inet_step(s, xq, labels, flat, decisions="write")
    lq, dq, gq, st = oracle.inet_step(s, xq, labels, flat, decisions=dec, bf16_storage=True)
    assert 0 < abs(lq - loss) <= 5e-2 * abs(loss)
    assert np.linalg.norm(gq - logits) <= 5e-2 * np.linalg.norm(logits)
    assert 1e-4 < np.linalg.norm(dq - dflat) / np.linalg.norm(dflat) < 1e-1
