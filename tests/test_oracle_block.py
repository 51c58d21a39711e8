"""Pins for the CPU oracle's dense block (forward, backward, both schedules,
memory accounting) against things other than the oracle itself."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl

NAMES = wl.PARAM_NAMES


def pack(orc, shape, layer_params):
    """Pack per-layer tensors into the oracle's flat float64 parameter vector."""
    flat = np.zeros(orc.param_count(shape))
    for l, p in enumerate(layer_params, start=1):
        for name, arr in p.items():
            flat[orc.param_slice(shape, l, NAMES.index(name))] = np.asarray(arr, dtype=np.float64).ravel()
    return flat


def oshape(orc, cfg):
    return orc.BlockShape(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck, cfg.eps)


def setup(orc, cfg, affine="random", seeds=(0, 1, 2)):
    x0, lp, dy = wl.make_block_inputs(cfg, *seeds, affine=affine)
    s = oshape(orc, cfg)
    return s, x0.astype(np.float64), pack(orc, s, lp), dy.astype(np.float64), lp


# --------------------------------------------------- hand-enumerated tiny case

def tiny_block_by_hand(x0, lp, cfg):
    """Dense block written out with Python floats and explicit sums only
    (N=1, tiny H, W): an independent transcription of the definition
    x_l = conv3x3(relu(bn(conv1x1(relu(bn([x_0..x_{l-1}])))))."""
    H, W, eps = cfg.h, cfg.w, cfg.eps
    feats = [[[float(x0[0, c, y, x]) for x in range(W)] for y in range(H)] for c in range(cfg.c0)]

    def bn_relu(chans, gam, bet):
        out = []
        for c, ch in enumerate(chans):
            vals = [v for row in ch for v in row]
            mu = sum(vals) / len(vals)
            var = sum((v - mu) ** 2 for v in vals) / len(vals)
            out.append([[max(0.0, float(gam[c]) * (v - mu) / math.sqrt(var + eps) + float(bet[c])) for v in row]
                        for row in ch])
        return out

    for l in range(cfg.layers):
        p = lp[l]
        a = bn_relu(feats, p["g1"], p["b1"])
        if cfg.bottleneck:
            b = [[[sum(float(p["W1"][o, c]) * a[c][y][x] for c in range(len(a))) for x in range(W)]
                  for y in range(H)] for o in range(cfg.bottleneck)]
            a = bn_relu(b, p["g2"], p["b2"])
        new = []
        for o in range(cfg.growth):
            ch = [[0.0] * W for _ in range(H)]
            for y, x in itertools.product(range(H), range(W)):
                s = 0.0
                for c, i, j in itertools.product(range(len(a)), range(3), range(3)):
                    yy, xx = y + i - 1, x + j - 1
                    if 0 <= yy < H and 0 <= xx < W:
                        s += float(p["W3"][o, c, i, j]) * a[c][yy][xx]
                ch[y][x] = s
            new.append(ch)
        feats = feats + new
    return np.array(feats)[None]


@pytest.mark.parametrize("bott", [0, 2])
def test_tiny_block_by_hand(oracle, bott):
    cfg = wl.BlockCfg(n=1, c0=1, h=2, w=2, layers=2, growth=1, bottleneck=bott)
    s, x0, params, dy, lp = setup(oracle, cfg)
    y = oracle.block(s, x0, params).y
    np.testing.assert_allclose(y, tiny_block_by_hand(x0, lp, cfg), atol=1e-12)


# --------------------------------------------------- float64 library cross-check

def torch_block(x0, lp, cfg, dy):
    x0t = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    tp = [{k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in p.items()} for p in lp]
    feats = [x0t]
    for p in tp:
        u = torch.cat(feats, dim=1)
        a = F.relu(F.batch_norm(u, None, None, p["g1"], p["b1"], True, 0.0, cfg.eps))
        if cfg.bottleneck:
            b = F.conv2d(a, p["W1"][:, :, None, None])
            a = F.relu(F.batch_norm(b, None, None, p["g2"], p["b2"], True, 0.0, cfg.eps))
        feats.append(F.conv2d(a, p["W3"], padding=1))
    y = torch.cat(feats, dim=1)
    (y * torch.tensor(dy, dtype=torch.float64)).sum().backward()
    return y.detach().numpy(), x0t.grad.numpy(), tp


@pytest.mark.parametrize("cfg", [wl.config1(), wl.BlockCfg(3, 5, 5, 7, 3, 4, 0), wl.BlockCfg(2, 3, 6, 4, 3, 5, 7)])
def test_block_matches_float64_autograd(oracle, cfg):
    s, x0, params, dy, lp = setup(oracle, cfg)
    res = oracle.block(s, x0, params, dy)
    y, dx0, tp = torch_block(x0, lp, cfg, dy)
    np.testing.assert_allclose(res.y, y, atol=1e-11)
    np.testing.assert_allclose(res.dx0, dx0, atol=1e-10)
    for l, p in enumerate(tp, start=1):
        for name, t in p.items():
            got = res.dparams[oracle.param_slice(s, l, NAMES.index(name))]
            np.testing.assert_allclose(got, t.grad.numpy().ravel(), atol=1e-9, err_msg=f"layer {l} {name}")


# --------------------------------------------------- finite differences

def test_block_finite_differences_config1(oracle):
    """Central differences of L = sum(y * T) on the paper-shaped small block:
    random directions over (x0, params) jointly, plus single coordinates drawn from
    every parameter tensor of every layer and from x0."""
    cfg = wl.config1()
    s, x0, params, dy, lp = setup(oracle, cfg)
    res = oracle.block(s, x0, params, dy)

    def loss(xx, pp):
        return float(np.sum(oracle.block(s, xx, pp).y * dy))

    r = np.random.default_rng(99)
    h = 1e-6
    for _ in range(6):
        vx = r.standard_normal(x0.shape)
        vp = r.standard_normal(params.shape)
        nrm = math.sqrt(float(np.sum(vx * vx) + np.sum(vp * vp)))  # unit direction: few ReLU kinks crossed
        vx, vp = vx / nrm, vp / nrm
        fd = (loss(x0 + h * vx, params + h * vp) - loss(x0 - h * vx, params - h * vp)) / (2 * h)
        an = float(np.sum(res.dx0 * vx) + np.sum(res.dparams * vp))
        assert abs(fd - an) < 1e-5 * max(1.0, abs(an)), (fd, an)
    coords = []
    for l in range(1, cfg.layers + 1):
        for which in range(6):
            sl = oracle.param_slice(s, l, which)
            coords += list(r.choice(np.arange(sl.start, sl.stop), size=3, replace=False))
    for i in coords:
        pp, pm = params.copy(), params.copy()
        pp[i] += h
        pm[i] -= h
        fd = (loss(x0, pp) - loss(x0, pm)) / (2 * h)
        assert abs(fd - res.dparams[i]) < 1e-6 * max(1.0, abs(fd)) + 1e-7, (i, fd, res.dparams[i])
    for i in r.choice(x0.size, size=25, replace=False):
        xp, xm = x0.copy().ravel(), x0.copy().ravel()
        xp[i] += h
        xm[i] -= h
        fd = (loss(xp.reshape(x0.shape), params) - loss(xm.reshape(x0.shape), params)) / (2 * h)
        assert abs(fd - res.dx0.ravel()[i]) < 1e-6 * max(1.0, abs(fd)) + 1e-7


def test_block_finite_differences_all_coordinates_small(oracle):
    """Every coordinate of x0 and every parameter of a small bottleneck block."""
    cfg = wl.BlockCfg(n=2, c0=2, h=3, w=3, layers=2, growth=2, bottleneck=3, eps=1e-3)
    s, x0, params, dy, lp = setup(oracle, cfg)
    res = oracle.block(s, x0, params, dy)
    h = 1e-6

    def loss(xx, pp):
        return float(np.sum(oracle.block(s, xx, pp).y * dy))

    for i in range(params.size):
        pp, pm = params.copy(), params.copy()
        pp[i] += h
        pm[i] -= h
        fd = (loss(x0, pp) - loss(x0, pm)) / (2 * h)
        assert abs(fd - res.dparams[i]) < 1e-6 * max(1.0, abs(fd)), (i, fd, res.dparams[i])
    flat = x0.ravel()
    for i in range(flat.size):
        xp, xm = flat.copy(), flat.copy()
        xp[i] += h
        xm[i] -= h
        fd = (loss(xp.reshape(x0.shape), params) - loss(xm.reshape(x0.shape), params)) / (2 * h)
        assert abs(fd - res.dx0.ravel()[i]) < 1e-6 * max(1.0, abs(fd)), (i, fd)


# --------------------------------------------------- structure and special cases

def test_block_output_layout_oldest_first(oracle):
    cfg = wl.config1()
    s, x0, params, dy, lp = setup(oracle, cfg)
    y = oracle.block(s, x0, params).y
    assert y.shape == (cfg.n, cfg.c_out, cfg.h, cfg.w)
    np.testing.assert_array_equal(y[:, :cfg.c0], x0)
    # a one-layer-shorter block reproduces the same leading channels
    cfg3 = wl.BlockCfg(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers - 1, cfg.growth, cfg.bottleneck)
    s3 = oshape(oracle, cfg3)
    y3 = oracle.block(s3, x0, params[:oracle.param_count(s3)]).y
    np.testing.assert_array_equal(y[:, :cfg3.c_out], y3)


def test_first_bn_output_is_normalised(oracle):
    """Per channel of every layer's concatenated input: pre-affine mean 0,
    biased variance v/(v+eps)."""
    cfg = wl.config1()
    s, x0, params, dy, lp = setup(oracle, cfg)
    for l in range(1, cfg.layers + 1):
        u, xhat = oracle.probe_layer(s, x0, params, l)
        assert u.shape[1] == cfg.c_in(l)
        v = u.var(axis=(0, 2, 3))
        assert np.max(np.abs(xhat.mean(axis=(0, 2, 3)))) < 1e-12
        np.testing.assert_allclose(xhat.var(axis=(0, 2, 3)), v / (v + cfg.eps), rtol=1e-10)


def test_zero_W3_kills_the_layer(oracle):
    """W3_l = 0 => x_l = 0 and every gradient flowing up through layer l
    vanishes except dW3_l."""
    cfg = wl.config1()
    s, x0, params, dy, lp = setup(oracle, cfg)
    L = cfg.layers
    params = params.copy()
    params[oracle.param_slice(s, L, 5)] = 0.0
    res = oracle.block(s, x0, params, dy)
    assert np.all(res.y[:, cfg.c_in(L):] == 0.0)
    for which in range(5):
        assert np.all(res.dparams[oracle.param_slice(s, L, which)] == 0.0), which
    assert np.any(res.dparams[oracle.param_slice(s, L, 5)] != 0.0)
    # and the rest equals a block without that layer, fed dy's leading channels
    cfgm = wl.BlockCfg(cfg.n, cfg.c0, cfg.h, cfg.w, L - 1, cfg.growth, cfg.bottleneck)
    sm = oshape(oracle, cfgm)
    resm = oracle.block(sm, x0, params[:oracle.param_count(sm)], dy[:, :cfgm.c_out])
    np.testing.assert_allclose(res.dx0, resm.dx0, atol=1e-13)
    np.testing.assert_allclose(res.dparams[:oracle.param_count(sm)], resm.dparams, atol=1e-12)


def test_input_channel_scale_invariance(oracle):
    """BN removes a positive per-channel scale of the block input (eps -> 0):
    x_1..x_m do not change."""
    cfg = wl.BlockCfg(2, 3, 4, 4, 3, 2, 4, eps=1e-30)
    s, x0, params, dy, lp = setup(oracle, cfg)
    y = oracle.block(s, x0, params).y
    x0s = x0 * np.array([0.5, 3.0, 7.0])[None, :, None, None]
    ys = oracle.block(s, x0s, params).y
    np.testing.assert_allclose(ys[:, cfg.c0:], y[:, cfg.c0:], atol=1e-10)


def test_identity_bottleneck_reduces_to_two_bn(oracle):
    """m=1 with W1 = I (C_1 = B): layer equals BN-ReLU-BN-ReLU-conv3x3 built from primitives."""
    cfg = wl.BlockCfg(2, 4, 5, 5, 1, 3, 4)
    s, x0, params, dy, lp = setup(oracle, cfg)
    params = params.copy()
    params[oracle.param_slice(s, 1, 2)] = np.eye(4).ravel()
    y = oracle.block(s, x0, params).y
    p = lp[0]
    a = oracle.relu(oracle.bn_forward(x0, p["g1"], p["b1"], cfg.eps)[0])
    a2 = oracle.relu(oracle.bn_forward(a, p["g2"], p["b2"], cfg.eps)[0])
    np.testing.assert_allclose(y[:, 4:], oracle.conv_forward(a2, p["W3"]), atol=1e-13)


# --------------------------------------------------- the two schedules

CFGS = [wl.config1(), wl.BlockCfg(3, 5, 5, 7, 3, 4, 0), wl.BlockCfg(1, 7, 3, 3, 5, 3, 6)]


@pytest.mark.parametrize("cfg", CFGS)
def test_shared_schedule_equals_naive_bitwise(oracle, cfg):
    """Section 4: recomputation only re-populates buffers, so the efficient
    schedule returns exactly the naive schedule's numbers."""
    s, x0, params, dy, lp = setup(oracle, cfg)
    a = oracle.block(s, x0, params, dy, schedule="naive")
    b = oracle.block(s, x0, params, dy, schedule="shared")
    assert np.array_equal(a.y, b.y)
    assert np.array_equal(a.dx0, b.dx0)
    assert np.array_equal(a.dparams, b.dparams)


def sigma_c(cfg):
    return sum(cfg.c_in(l) for l in range(1, cfg.layers + 1))


@pytest.mark.parametrize("cfg", CFGS + [wl.BlockCfg(1, 4, 2, 2, 9, 2, 8)])
def test_feature_map_element_counts(oracle, cfg):
    """Live feature-map elements the two schedules allocate (counted by the oracle's
    allocator) against the closed forms: quadratic (through sum C_l) when every concat
    and BN output is kept, linear when they live in shared storage."""
    s, x0, params, dy, lp = setup(oracle, cfg)
    P, m, k, B = cfg.pixels, cfg.layers, cfg.growth, cfg.bottleneck
    cm, cout = cfg.c_in(m), cfg.c_out
    grads = cout + cm + B                       # accumulator slab + two scratch tensors
    naive_fwd = 2 * sigma_c(cfg) + m * (2 * B + k)
    shared_fwd = m * (B + k) + 2 * cm + B
    a = oracle.block(s, x0, params, dy, schedule="naive")
    b = oracle.block(s, x0, params, dy, schedule="shared")
    assert a.stored_elems == naive_fwd * P
    assert a.peak_elems == (naive_fwd + grads) * P
    assert b.stored_elems == shared_fwd * P
    assert b.peak_elems == (shared_fwd + grads) * P


def test_memory_growth_linear_vs_quadratic(oracle):
    """Second differences in depth: constant > 0 for the naive schedule, zero for the shared one."""
    peaks = {"naive": [], "shared": []}
    for m in (2, 3, 4, 5):
        cfg = wl.BlockCfg(1, 4, 2, 2, m, 2, 8)
        s, x0, params, dy, lp = setup(oracle, cfg)
        for sched in peaks:
            peaks[sched].append(oracle.block(s, x0, params, dy, schedule=sched).peak_elems)
    d2 = lambda v: [v[i + 2] - 2 * v[i + 1] + v[i] for i in range(len(v) - 2)]
    assert all(x == 0 for x in d2(peaks["shared"]))
    assert all(x == d2(peaks["naive"])[0] > 0 for x in d2(peaks["naive"]))


# --------------------------------------------------- values the paper prints

def read_golden():
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_param_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                parts = line.split()
                rows.append((parts[0], [int(v) for v in parts[1].split(",")], int(parts[2]), int(parts[3]),
                             float(parts[4]), float(parts[5])))
    return rows


@pytest.mark.parametrize("row", read_golden(), ids=lambda r: f"{r[0]}-{sum(r[1])}-k{r[2]}")
def test_parameter_counts_match_paper(oracle, row):
    """The oracle's parameter-pack size plus the glue layers reproduces the model
    sizes printed in the paper (Section 5), which pins C_l, B = 4k and the pack layout."""
    kind, blocks, k, classes, printed_m, tol_m = row
    if kind == "cifar":
        stem_c, stem_params, size = 2 * k, 2 * k * 3 * 9, 32
    else:
        stem_c, stem_params, size = 2 * k, 2 * k * 3 * 49 + 2 * (2 * k), 56
    total, c = stem_params, stem_c
    for bi, m in enumerate(blocks):
        s = oracle.BlockShape(1, c, 1, 1, m, k, 4 * k)
        total += oracle.param_count(s)
        c = c + m * k
        if bi + 1 < len(blocks):
            total += 2 * c + c * (c // 2)
            c //= 2
    total += 2 * c + c * classes + classes
    assert abs(total / 1e6 - printed_m) <= tol_m, total


# --------------------------------------------------- bf16 storage emulation

def test_round_bf16_matches_library_cast(oracle):
    """The oracle's rounding to bfloat16 against the tensor library's cast: random values over
    many binades, exact ties (round to even), signs, and values that are already representable."""
    rng = np.random.default_rng(7)
    vals = list((rng.standard_normal(2000) * np.exp(rng.uniform(-20, 20, 2000))).astype(np.float32))
    vals += [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -20, 0.0, -0.0, 1.5, 3.0e38 / 2]
    ref = torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.round_bf16(float(v)) for v in vals])
    assert np.array_equal(got, ref)


def _bf16_ste(t):
    """Value rounded to bf16, gradient passed through unchanged."""
    return t + (t.detach().to(torch.float32).to(torch.bfloat16).to(torch.float64) - t.detach())


def _round_grad(t):
    t.register_hook(lambda g: g.to(torch.float32).to(torch.bfloat16).to(torch.float64))
    return t


@pytest.mark.parametrize("cfg", [wl.BlockCfg(2, 4, 4, 4, 2, 4, 8), wl.BlockCfg(1, 8, 5, 3, 3, 2, 4)],
                         ids=["n2c4h4w4m2k4B8", "n1c8h5w3m3k2B4"])
def test_bf16_storage_block_matches_autograd_with_casts(oracle, cfg):
    """The storage-emulating block against an independent construction: library float64 batch
    norm and convolutions under autograd, with a cast to bfloat16 at every point where the bf16
    path stores a tensor (values: BN+ReLU outputs, conv weights, conv outputs; gradients: of each
    x_l before its convs use it, of each BN+ReLU output, of the bottleneck output, of x_0).  A
    rounding point that is missing, misplaced or applied to an accumulator shows up at the 1e-3
    level; agreement is asked to 1e-9."""
    s, x0, params, dy, lp = setup(oracle, cfg)
    r32 = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to(torch.bfloat16).to(torch.float64)
    x0q, dyq = r32(x0), r32(dy)
    res = oracle.block(s, x0q.numpy(), params, dyq.numpy(), schedule="naive_bf16")

    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    x0t = x0q.clone().requires_grad_(True)
    tp = [{k: t(v) for k, v in p.items()} for p in lp]
    feats = [x0t]
    for p in tp:
        u = torch.cat(feats, dim=1)
        a = _round_grad(_bf16_ste(F.relu(F.batch_norm(u, None, None, p["g1"], p["b1"], True, 0.0, cfg.eps))))
        b = _round_grad(_bf16_ste(F.conv2d(a, _bf16_ste(p["W1"]).reshape(cfg.bottleneck, -1, 1, 1))))
        a2 = _round_grad(_bf16_ste(F.relu(F.batch_norm(b, None, None, p["g2"], p["b2"], True, 0.0, cfg.eps))))
        x = _round_grad(_bf16_ste(F.conv2d(a2, _bf16_ste(p["W3"]), padding=1)))
        feats.append(x)
    y = torch.cat(feats, dim=1)
    y.backward(dyq)
    assert np.allclose(res.y, y.detach().numpy(), rtol=1e-9, atol=1e-12)
    dx0_ref = x0t.grad.to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.allclose(res.dx0, dx0_ref, rtol=1e-9, atol=1e-12)
    for l, p in enumerate(tp, start=1):
        for name in NAMES:
            got = res.dparams[oracle.param_slice(s, l, NAMES.index(name))]
            assert np.allclose(got, p[name].grad.numpy().ravel(), rtol=1e-8, atol=1e-11), (l, name)
    # and it is a small perturbation of the unrounded block
    plain = oracle.block(s, x0q.numpy(), params, dyq.numpy(), schedule="naive")
    assert np.linalg.norm(res.y - plain.y) / np.linalg.norm(plain.y) < 1e-2


# --------------------------------------------------- ReLU decisions written out / taken from the caller

def torch_block_with_decisions(x0, lp, cfg, dy, m1, m2):
    """The block under autograd with each ReLU replaced by a multiplication with a given 0/1
    tensor (forward a = z * decision, hence backward dz = da * decision)."""
    x0t = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    tp = [{k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in p.items()} for p in lp]
    feats = [x0t]
    o1 = 0
    P = cfg.n * cfg.h * cfg.w
    for l, p in enumerate(tp, start=1):
        u = torch.cat(feats, dim=1)
        c = u.shape[1]
        d1 = torch.tensor(m1[o1:o1 + c * P].reshape(cfg.n, c, cfg.h, cfg.w).astype(np.float64))
        o1 += c * P
        a = F.batch_norm(u, None, None, p["g1"], p["b1"], True, 0.0, cfg.eps) * d1
        if cfg.bottleneck:
            B = cfg.bottleneck
            b = F.conv2d(a, p["W1"][:, :, None, None])
            d2 = torch.tensor(m2[(l - 1) * B * P:l * B * P].reshape(cfg.n, B, cfg.h, cfg.w).astype(np.float64))
            a = F.batch_norm(b, None, None, p["g2"], p["b2"], True, 0.0, cfg.eps) * d2
        feats.append(F.conv2d(a, p["W3"], padding=1))
    y = torch.cat(feats, dim=1)
    (y * torch.tensor(dy, dtype=torch.float64)).sum().backward()
    return y.detach().numpy(), x0t.grad.numpy(), tp


@pytest.mark.parametrize("cfg", [wl.config1(), wl.BlockCfg(3, 5, 5, 7, 3, 4, 0), wl.BlockCfg(2, 3, 6, 4, 3, 5, 7)])
def test_block_with_given_relu_decisions(oracle, cfg):
    """(1) The decisions the block writes out are its own z > 0, and feeding them back reproduces
    the plain block bit for bit with no disagreement reported.  (2) With arbitrary decisions (a
    twentieth of them inverted) the block equals float64 autograd of the same network with every
    ReLU replaced by a multiplication with the given 0/1 tensor, and the number of disagreements
    reported is the number inverted.  (3) The reported margin |z| / sqrt(gamma^2 + beta^2) of the
    worst disagreement, recomputed here for the first layer's first BN from library batch norm."""
    s, x0, params, dy, lp = setup(oracle, cfg)
    plain = oracle.block(s, x0, params, dy)
    own, (m1, m2) = oracle.block_with_decisions(s, x0, params, dy)
    n1, n2 = oracle.relu_decision_counts(s)
    assert m1.size == n1 and m2.size == n2 and set(np.unique(m1)) <= {0, 1}
    for a, b in ((own.y, plain.y), (own.dx0, plain.dx0), (own.dparams, plain.dparams)):
        assert np.array_equal(a, b)
    # first layer's decisions against library batch norm
    z1 = F.batch_norm(torch.tensor(x0), None, None, torch.tensor(lp[0]["g1"].astype(np.float64)),
                      torch.tensor(lp[0]["b1"].astype(np.float64)), True, 0.0, cfg.eps).numpy()
    assert np.array_equal(m1[:x0.size].reshape(x0.shape), (z1 > 0).astype(np.uint8))
    back, st = oracle.block_with_decisions(s, x0, params, dy, (m1, m2))
    assert st == dict(count1=0, margin1=0.0, count2=0, margin2=0.0)
    for a, b in ((back.y, plain.y), (back.dx0, plain.dx0), (back.dparams, plain.dparams)):
        assert np.array_equal(a, b)

    r = np.random.default_rng(5)
    f1, f2 = r.random(n1) < 0.05, r.random(n2) < 0.05
    g1, g2 = m1 ^ f1.astype(np.uint8), m2 ^ f2.astype(np.uint8)
    res, st = oracle.block_with_decisions(s, x0, params, dy, (g1, g2))
    y, dx0, tp = torch_block_with_decisions(x0, lp, cfg, dy, g1, g2)
    np.testing.assert_allclose(res.y, y, atol=1e-11)
    np.testing.assert_allclose(res.dx0, dx0, atol=1e-10)
    for l, p in enumerate(tp, start=1):
        for name, t in p.items():
            got = res.dparams[oracle.param_slice(s, l, NAMES.index(name))]
            np.testing.assert_allclose(got, t.grad.numpy().ravel(), atol=1e-9, err_msg=f"layer {l} {name}")
    assert not np.allclose(res.dx0, plain.dx0, atol=1e-6)   # the inverted decisions do matter
    # With decisions imposed, every later pre-activation moves, so only a one-layer block's first BN
    # has a count known beforehand; its worst margin is recomputed here.
    cfg1 = wl.BlockCfg(cfg.n, cfg.c0, cfg.h, cfg.w, 1, cfg.growth, cfg.bottleneck, cfg.eps)
    s1, x0, params1, dy1, lp1 = setup(oracle, cfg1)
    _, (q1, q2) = oracle.block_with_decisions(s1, x0, params1, dy1)
    flip = r.random(q1.size) < 0.05
    _, st1 = oracle.block_with_decisions(s1, x0, params1, dy1, (q1 ^ flip.astype(np.uint8), q2))
    assert st1["count1"] == int(flip.sum())
    z1 = F.batch_norm(torch.tensor(x0), None, None, torch.tensor(lp1[0]["g1"].astype(np.float64)),
                      torch.tensor(lp1[0]["b1"].astype(np.float64)), True, 0.0, cfg.eps).numpy()
    rms = np.sqrt(lp1[0]["g1"].astype(np.float64) ** 2 + lp1[0]["b1"].astype(np.float64) ** 2)
    margin = (np.abs(z1) / rms[None, :, None, None])[flip.reshape(x0.shape)].max()
    assert abs(st1["margin1"] - margin) <= 1e-9 * margin
