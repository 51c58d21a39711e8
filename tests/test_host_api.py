"""CPU-side checks of the C-ABI library: it loads, exports everything include/dnb.h
declares, validates descriptors, and its byte accounting and parameter-pack offsets
agree with the oracle's independent counts.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))




def declared_functions():
    text = open(os.path.join(ROOT, "include", "dnb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dnb_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(dnb):
    names = declared_functions()
    assert "dnb_block_create" in names and "dnb_block_forward" in names
    assert "dnb_block_backward" in names and "dnb_block_peak_bytes" in names
    # the boundary's named calls
    for required in ("dnb_block_create", "dnb_block_destroy", "dnb_block_peak_bytes", "dnb_block_param_bytes",
                     "dnb_block_param_offset", "dnb_block_forward", "dnb_block_backward", "dnb_status_string"):
        assert required in names, required
    lib = ctypes.CDLL(dnb.binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(dnb.EXPORTED) == set(names)


def test_status_strings(dnb):
    assert dnb.dnb_status_string(0) == "ok"
    for code in range(-7, 0):
        assert dnb.dnb_status_string(code) not in ("ok", "unknown status")
    assert dnb.dnb_status_string(-99) == "unknown status"


@pytest.mark.parametrize("kw,code", [
    (dict(n=0), -1), (dict(c0=0), -1), (dict(layers=0), -1), (dict(growth=0), -1), (dict(bottleneck=-1), -1),
    (dict(h=-1), -1), (dict(eps=-1.0), -1), (dict(dtype=7), -1), (dict(layout=3), -1), (dict(schedule=9), -1),
    (dict(dtype=1), -5), (dict(layout=1), -5), (dict(n=4096, h=512, w=512), -6),
    (dict(schedule=2, h=7, w=7), -5), (dict(schedule=2, bottleneck=512), -5),
    (dict(bottleneck=0, schedule=2), -5), (dict(bottleneck=0, dtype=1, layout=1, schedule=2), -5)])
def test_descriptor_validation(dnb, kw, code):
    base = dict(n=2, c0=16, h=8, w=8, layers=4, growth=12, bottleneck=48)
    base.update(kw)
    with pytest.raises(dnb.binding.DnbError) as e:
        dnb.dnb_block_create(**base)
    assert e.value.status == code


def test_shapes_whose_tiles_do_not_fit_are_refused_at_create(dnb):
    """Kernels whose LDS tiles or launch plans do not fit a shape are found by dnb_block_create
    (DNB_E_UNSUPPORTED), not by a failing launch in the middle of a backward pass: the fp32 fused
    schedule's 3x3 weight gradient, and the any-shape 3x3 kernels of the materialised schedules, with
    rows of 256 pixels; the bf16 3x3 with rows of 80 pixels
    once the fused schedule's folded BN parameters share its LDS (the materialised schedules still
    take them), and rows of 84 pixels in any schedule."""
    def status(**kw):
        base = dict(n=2, c0=16, h=4, w=8, layers=2, growth=8, bottleneck=32)
        base.update(kw)
        try:
            dnb.dnb_block_destroy(dnb.dnb_block_create(**base))
            return 0
        except dnb.binding.DnbError as e:
            return e.status
    assert status(schedule=2, bottleneck=24, w=128) == 0
    assert status(schedule=2, bottleneck=24, w=256) == dnb.DNB_E_UNSUPPORTED
    assert status(schedule=0, bottleneck=24, w=128) == 0        # the materialised schedules have any-shape kernels,
    assert status(schedule=0, bottleneck=24, w=256) == dnb.DNB_E_UNSUPPORTED   # whose 3x3 tiles stop fitting LDS above ~136-pixel rows
    bf = dict(dtype=dnb.DNB_BF16, layout=dnb.DNB_NHWC, c0=96, growth=48, bottleneck=192)
    assert status(schedule=2, w=76, **bf) == 0
    assert status(schedule=2, w=80, **bf) == dnb.DNB_E_UNSUPPORTED
    assert status(schedule=0, w=80, **bf) == 0
    assert status(schedule=0, w=84, **bf) == dnb.DNB_E_UNSUPPORTED


def test_null_arguments_are_errors(dnb):
    lib = ctypes.CDLL(dnb.binding.LIB_PATH)
    assert lib.dnb_block_create(None, None) == -2
    h = dnb.dnb_block_create(2, 16, 8, 8, 4, 12, 48)
    lib.dnb_block_forward.argtypes = [ctypes.c_void_p] * 6
    assert lib.dnb_block_forward(h, None, None, None, None, None) == -2
    assert lib.dnb_block_forward(h, 256, 256, 264, 256, None) == -3  # misaligned y
    dnb.dnb_block_destroy(h)


def test_nhwc_ops_reject_misaligned_tensors_and_short_strides(dnb):
    """The bf16 / NHWC single operations move 16 bytes per lane: a feature-map pointer off a
    16-byte boundary is DNB_E_ALIGN (-3), a pixel stride shorter than the channel count or not a
    whole number of 16-byte vectors is DNB_E_RANGE (-6); both are found before anything is launched."""
    lib = ctypes.CDLL(dnb.binding.LIB_PATH)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    fwd = lib.dnb_op_nhwc_conv_forward
    fwd.argtypes = [vp, i64, vp, vp, i64, i64, i64, i64, i64, i64, ci, vp, vp]
    shape = (2, 16, 24, 6, 6, 1)   # n, cin, cout, h, w, ks
    assert fwd(4096 + 8, 16, 4096, 8192, 24, *shape, 12288, None) == -3       # x off by 8 bytes
    assert fwd(4096, 16, 4096, 8192 + 2, 24, *shape, 12288, None) == -3       # out off by 2 bytes
    assert fwd(4096, 16, 4096, 8192, 24, *shape, 12288 + 4, None) == -3       # scratch
    assert fwd(4096, 8, 4096, 8192, 24, *shape, 12288, None) == -6            # x stride < cin
    assert fwd(4096, 20, 4096, 8192, 24, *shape, 12288, None) == -6           # x stride not a multiple of 8
    assert fwd(4096, 16, 4096, 8192, 28, *shape, 12288, None) == -6           # out stride not a multiple of 8
    dgrad = lib.dnb_op_nhwc_conv_dgrad
    dgrad.argtypes = [vp, i64, ci, vp, vp, i64, i64, i64, i64, i64, i64, ci, vp, vp]
    assert dgrad(4096, 26, 1, 4096, 8192, 16, *shape, 12288, None) == -6      # fp32 dout stride not a multiple of 4
    assert dgrad(4096, 28, 0, 4096, 8192, 16, *shape, 12288, None) == -6      # the same stride for bf16 dout
    assert dgrad(4096, 24, 0, 4096, 8192 + 8, 16, *shape, 12288, None) == -3  # din
    bn = lib.dnb_op_nhwc_bn_relu_backward
    bn.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp]
    par = [256, 512, 768, 1024, 1280, 1536]
    assert bn(4096, 16, 8192, 16, None, 0, 12288 + 4, 16, 72, 16, *par, 16384, None) == -3   # fp32 accumulator
    assert bn(4096, 16, 8192, 16, None, 0, 12288, 18, 72, 16, *par, 16384, None) == -6       # its stride
    assert bn(4096, 16, 8192, 16, 8192, 12, None, 0, 72, 16, *par, 16384, None) == -6        # bf16 output stride


def sigma_c(cfg):
    return sum(cfg.c_in(l) for l in range(1, cfg.layers + 1))


CFGS = [wl.config1(), wl.BlockCfg(3, 5, 5, 7, 3, 4, 6), wl.BlockCfg(1, 7, 3, 3, 5, 3, 6)] + wl.config2() + wl.config3()
NOBOTTLE = [wl.BlockCfg(2, 8, 8, 8, 3, 4, 0), wl.BlockCfg(3, 5, 5, 7, 4, 3, 0)]   # BN-ReLU-3x3 layers (bottleneck = 0)


@pytest.mark.parametrize("cfg", CFGS + NOBOTTLE, ids=lambda c: f"{c.n}x{c.c0}x{c.h}x{c.w}-m{c.layers}k{c.growth}B{c.bottleneck}")
def test_peak_bytes_formula(dnb, cfg):
    """Linear-memory formula (shared) and quadratic one (store-all), in bytes."""
    Ps, m, k, B = cfg.pixels * 4, cfg.layers, cfg.growth, cfg.bottleneck
    cm, cout = cfg.c_in(m), cfg.c_out
    grad = (cout + cm + B) * Ps
    hs = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, m, k, B, schedule=0)
    ha = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, m, k, B, schedule=1)
    ms, ma = dnb.dnb_block_memory_breakdown(hs), dnb.dnb_block_memory_breakdown(ha)
    assert ms["stored_fwd_bytes"] == (m * B + m * k) * Ps
    assert ms["shared_fwd_bytes"] == (2 * cm + B) * Ps
    assert ms["grad_bytes"] == grad == ma["grad_bytes"]
    assert ma["stored_fwd_bytes"] == (2 * sigma_c(cfg) + m * (2 * B + k)) * Ps
    assert ma["shared_fwd_bytes"] == 0
    for h, mm in ((hs, ms), (ha, ma)):
        assert dnb.dnb_block_peak_bytes(h) == mm["peak_bytes"] == mm["stored_fwd_bytes"] + mm["shared_fwd_bytes"] + mm["grad_bytes"]
        # the workspace holds the feature maps (all but the x_l inside y), statistics, scratch, padding
        lo = mm["peak_bytes"] - m * k * Ps + mm["stats_bytes"] + mm["scratch_bytes"]
        assert lo <= mm["workspace_bytes"] == dnb.dnb_block_workspace_bytes(h) <= lo + 256 * (6 * m + 16)
        dnb.dnb_block_destroy(h)


@pytest.mark.parametrize("cfg", [c for c in CFGS if c.w % 4 == 0], ids=lambda c: f"{c.n}x{c.c0}x{c.h}x{c.w}-m{c.layers}k{c.growth}")
def test_fused_schedule_bytes(dnb, cfg):
    """No shared storage at all: stored conv outputs + gradient storage only, linear in m."""
    Ps, m, k, B = cfg.pixels * 4, cfg.layers, cfg.growth, cfg.bottleneck
    h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, m, k, B, schedule=2)
    mm = dnb.dnb_block_memory_breakdown(h)
    assert mm["shared_fwd_bytes"] == 0
    assert mm["stored_fwd_bytes"] == (m * B + m * k) * Ps
    assert mm["peak_bytes"] == (m * B + m * k + cfg.c_out + cfg.c_in(m) + B) * Ps == dnb.dnb_block_peak_bytes(h)
    dnb.dnb_block_destroy(h)


def test_config1_bytes_as_stated(dnb):
    h = dnb.dnb_block_create(2, 16, 8, 8, 4, 12, 48, schedule=0)
    assert dnb.dnb_block_peak_bytes(h) == 284672
    h1 = dnb.dnb_block_create(2, 16, 8, 8, 4, 12, 48, schedule=1)
    assert dnb.dnb_block_peak_bytes(h1) == 444416


@pytest.mark.parametrize("cfg", CFGS[:3] + NOBOTTLE)
def test_peak_bytes_match_oracle_allocation_count(dnb, oracle, cfg):
    """The library's formula against the elements the oracle's two schedules actually
    allocate (counted by its allocator), times the element size."""
    x0, lp, dy = wl.make_block_inputs(cfg)
    s = oracle.BlockShape(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck, cfg.eps)
    params = np.zeros(oracle.param_count(s))
    for sched, name in ((0, "shared"), (1, "naive")):
        h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck, schedule=sched)
        res = oracle.block(s, x0, params, dy, schedule=name)
        assert dnb.dnb_block_peak_bytes(h) == res.peak_elems * 4
        assert dnb.dnb_block_memory_breakdown(h)["stored_fwd_bytes"] + dnb.dnb_block_memory_breakdown(h)["shared_fwd_bytes"] == res.stored_elems * 4
        dnb.dnb_block_destroy(h)


@pytest.mark.parametrize("cfg", CFGS[:3] + NOBOTTLE)
def test_param_offsets_match_oracle(dnb, oracle, cfg):
    s = oracle.BlockShape(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck, cfg.eps)
    h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck)
    assert dnb.dnb_block_param_count(h) == oracle.param_count(s)
    assert dnb.dnb_block_param_bytes(h) == 4 * oracle.param_count(s)
    for l in range(1, cfg.layers + 1):
        for which in range(6):
            off, cnt = dnb.dnb_block_param_offset(h, l, which)
            if cfg.bottleneck == 0 and which in (2, 3, 4):   # W1, g2, b2 do not exist
                assert cnt == 0
                continue
            sl = oracle.param_slice(s, l, which)
            assert (off, off + cnt) == (sl.start, sl.stop)
    with pytest.raises(dnb.binding.DnbError):
        dnb.dnb_block_param_offset(h, cfg.layers + 1, 0)
    dnb.dnb_block_destroy(h)


def test_memory_is_linear_in_depth_for_shared_schedule(dnb):
    peaks = {0: [], 1: []}
    for m in (8, 16, 24, 32):
        for sched in (0, 1):
            h = dnb.dnb_block_create(64, 24, 32, 32, m, 12, 48, schedule=sched)
            peaks[sched].append(dnb.dnb_block_peak_bytes(h))
            dnb.dnb_block_destroy(h)
    d2 = lambda v: [v[i + 2] - 2 * v[i + 1] + v[i] for i in range(len(v) - 2)]
    assert all(x == 0 for x in d2(peaks[0]))
    assert all(x > 0 for x in d2(peaks[1]))


def test_depth_sweep_closed_form_matches_library(dnb):
    """The depth study's closed-form byte counts against the library's accounting, and the
    quadratic / linear growth they are meant to show."""
    import bench_depth_sweep as ds
    sched = {"shared": 0, "store_all": 1, "fused": 2}
    for L in (40, 100, 250):
        blocks = wl.densenet_bc_blocks(L, 12, 64)
        for name, code in sched.items():
            total = 0
            for c in blocks:
                h = dnb.dnb_block_create(c.n, c.c0, c.h, c.w, c.layers, c.growth, c.bottleneck, schedule=code)
                total += dnb.dnb_block_peak_bytes(h)
                dnb.dnb_block_destroy(h)
            assert total == ds.feature_map_bytes(blocks, name)
    f = lambda L, s: ds.feature_map_bytes(wl.densenet_bc_blocks(L, 12, 64), s)
    assert f(502, "store_all") / f(100, "store_all") > 15 > 6 > f(502, "shared") / f(100, "shared")
    assert ds.deepest_that_fits(wl, "store_all", 12, 64) < ds.deepest_that_fits(wl, "shared", 12, 64) < ds.deepest_that_fits(wl, "fused", 12, 64)


# ------------------------------------------------------------------ whole-network entry points

NET_PARTS = {"stem": 0, "block0": 1, "block1": 2, "block2": 3, "trans0.g": 4, "trans0.b": 5, "trans0.W": 6,
             "trans1.g": 7, "trans1.b": 8, "trans1.W": 9, "tail.g": 10, "tail.b": 11, "tail.Wl": 12, "tail.bl": 13}


@pytest.mark.parametrize("cfg", [wl.NetCfg(2, 8, 16, 4, 5), wl.net_config2(), wl.net_config3()],
                         ids=["tiny", "bc100", "bc250"])
def test_net_param_layout_matches_oracle(dnb, oracle, cfg):
    s = oracle.NetShape(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, cfg.eps)
    fusable = all(b.w % 4 == 0 for b in cfg.blocks())
    net = dnb.dnb_net_create(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, schedule=2 if fusable else 0)
    assert dnb.dnb_net_param_count(net) == oracle.net_param_count(s)
    for name, sl in oracle.net_param_slices(s).items():
        off, cnt = dnb.dnb_net_param_offset(net, NET_PARTS[name])
        assert (off, off + cnt) == (sl.start, sl.stop), name
    with pytest.raises(dnb.binding.DnbError):
        dnb.dnb_net_param_offset(net, 14)
    blocks = cfg.blocks()
    glue = sum((b.c0 + 2 * b.c_out) * b.pixels * 4 for b in blocks)           # block inputs, outputs, BN+ReLU of outputs
    glue += 2 * max((b.c_out // 2) * b.pixels for b in blocks[:2]) * 4        # transition conv output and its gradient
    glue += 2 * max(b.c_out * b.pixels for b in blocks) * 4 + max(b.c0 * b.pixels for b in blocks) * 4  # gradient buffers
    inner = sum((b.layers * b.bottleneck + b.c_out + b.c_in(b.layers) + b.bottleneck
                 + (0 if fusable else 2 * b.c_in(b.layers) + b.bottleneck)) * b.pixels * 4 for b in blocks)
    assert dnb.dnb_net_peak_bytes(net) == glue + inner <= dnb.dnb_net_workspace_bytes(net)
    dnb.dnb_net_destroy(net)


@pytest.mark.parametrize("kw", [dict(n=0), dict(depth=17), dict(depth=4), dict(image=10), dict(classes=0), dict(growth=0)])
def test_net_descriptor_validation(dnb, kw):
    base = dict(n=2, image=8, depth=16, growth=4, classes=5)
    base.update(kw)
    with pytest.raises(dnb.binding.DnbError) as e:
        dnb.dnb_net_create(**base)
    assert e.value.status == dnb.DNB_E_BADDESC


def net_pieces(dnb, net):
    out, i = [], 0
    while True:
        p = dnb.dnb_net_workspace_piece(net, i)
        if p is None:
            return out
        out.append(p)
        i += 1


@pytest.mark.parametrize("depth", [10, 16, 22, 88, 94, 100, 130, 190, 250])
@pytest.mark.parametrize("growth,n", [(12, 64), (24, 64), (4, 3)])
def test_net_workspace_pieces_hold_their_largest_writer(dnb, depth, growth, n):
    """Every piece of the network workspace against the largest tensor any step writes into it
    (with more than 14 layers per block the input of block 1 is larger than that of block 0), no
    two pieces overlap, and everything lies inside dnb_net_workspace_bytes."""
    cfg = wl.NetCfg(n, 32, depth, growth, 10)
    blocks = cfg.blocks()
    net = dnb.dnb_net_create(cfg.n, cfg.image, cfg.depth, cfg.growth, cfg.classes, schedule=2)
    pieces = net_pieces(dnb, net)
    total = dnb.dnb_net_workspace_bytes(net)
    spans = sorted((off, off + nb) for _, _, off, nb in pieces)
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert a1 <= b0
    assert spans[-1][1] <= total
    size = {(name, idx): nb for name, idx, _, nb in pieces}
    need = {}
    def want(key, nbytes):
        need[key] = max(need.get(key, 0), nbytes)
    for b, blk in enumerate(blocks):
        P, co = blk.pixels, blk.c_out
        want(("feat", b), blk.c0 * P * 4)        # stem / pooled transition output = block input
        want(("y", b), co * P * 4)
        want(("tz", b), co * P * 4)
        want(("mean", b), co * 4)
        want(("istd", b), co * 4)
        want(("gy", 0), co * P * 4)              # BN+ReLU backward of the block output
        want(("dfeat", 0), blk.c0 * P * 4)       # dnb_block_backward's dx0
        if b < 2:
            want(("tconv", 0), (co // 2) * P * 4)
            want(("dconv", 0), (co // 2) * P * 4)   # pooling backward of block b+1's input gradient
            want(("dtz", 0), co * P * 4)            # the transition conv's data gradient
            assert blocks[b + 1].c0 == co // 2 and blocks[b + 1].pixels * 4 == P
        else:
            want(("dtz", 0), co * P * 4)            # global pooling backward
            for key in ("pooled", "dpooled"):
                want((key, 0), n * co * 4)
    want(("logits", 0), n * cfg.classes * 4)
    want(("dlogits", 0), n * cfg.classes * 4)
    want(("terms", 0), n * 4)
    for key, nbytes in need.items():
        assert size[key] >= nbytes, (key, size[key], nbytes)
    dnb.dnb_net_destroy(net)


INET_PARTS = {"stem.W": 0, "stem.g": 1, "stem.b": 2, "tail.bl": 19}
for _b in range(4):
    INET_PARTS[f"block{_b}"] = 3 + 4 * _b
    _pre = f"trans{_b}" if _b < 3 else "tail"
    INET_PARTS[f"{_pre}.g"], INET_PARTS[f"{_pre}.b"] = 4 + 4 * _b, 5 + 4 * _b
    INET_PARTS[f"{_pre}.W" if _b < 3 else "tail.Wl"] = 6 + 4 * _b


@pytest.mark.parametrize("cfg", [wl.InetCfg(2, 64, 8, (2, 2, 2, 2), 5), wl.inet_config4(), wl.inet_config5()],
                         ids=["tiny", "densenet161", "densenet264"])
def test_inet_param_layout_matches_oracle_and_bytes(dnb, oracle, cfg):
    s = oracle.InetShape(cfg.n, cfg.image, cfg.growth, tuple(cfg.layers), cfg.classes, cfg.eps)
    net = dnb.dnb_inet_create(cfg.n, cfg.image, cfg.growth, cfg.layers, cfg.classes, schedule=2)
    assert dnb.dnb_inet_param_count(net) == oracle.inet_param_count(s)
    for name, sl in oracle.inet_param_slices(s).items():
        off, cnt = dnb.dnb_inet_param_offset(net, INET_PARTS[name])
        assert (off, off + cnt) == (sl.start, sl.stop), name
    with pytest.raises(dnb.binding.DnbError):
        dnb.dnb_inet_param_offset(net, 20)
    nr, npool = oracle.inet_decision_counts(s)
    assert dnb.dnb_inet_relu_decision_bytes(net) == nr and dnb.dnb_inet_pool_position_bytes(net) == npool
    blocks = cfg.blocks()
    cs, S2, S4 = 2 * cfg.growth, cfg.image // 2, cfg.image // 4
    glue = cfg.n * S2 * S2 * cs * 2 * 2 + cfg.n * S4 * S4 * cs                 # stem output and its gradient, pooling positions
    glue += sum((b.c0 + b.c_out) * b.pixels * 2 for b in blocks)              # block inputs and outputs
    glue += 2 * max((b.c_out // 2) * b.pixels for b in blocks[:3]) * 2        # transition conv output and its gradient
    glue += 2 * max(b.c_out * b.pixels for b in blocks) * 2 + max(b.c0 * b.pixels for b in blocks) * 2   # gradient buffers
    inner = sum((b.layers * b.bottleneck) * b.pixels * 2 + b.c_out * b.pixels * 4 + (b.c_in(b.layers) + b.bottleneck) * b.pixels * 2
                for b in blocks)
    assert dnb.dnb_inet_peak_bytes(net) == glue + inner <= dnb.dnb_inet_workspace_bytes(net)
    dnb.dnb_inet_destroy(net)


@pytest.mark.parametrize("kw,code", [(dict(n=0), -1), (dict(image=48), -1), (dict(layers=(2, 0, 2, 2)), -1), (dict(classes=0), -1),
                                     (dict(growth=12), -5), (dict(growth=8, layers=(1, 2, 2, 2)), -5)])
def test_inet_descriptor_validation(dnb, kw, code):
    base = dict(n=2, image=64, growth=8, layers=(2, 2, 2, 2), classes=5)
    base.update(kw)
    with pytest.raises(dnb.binding.DnbError) as e:
        dnb.dnb_inet_create(**base)
    assert e.value.status == code
