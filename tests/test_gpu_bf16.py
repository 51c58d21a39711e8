"""GPU parity of the bf16 / NHWC path (feature maps bf16, fp32 accumulation and statistics, fused
schedule) against the plain float64 oracle evaluated on the same bf16-rounded inputs, at the 2e-2
bound on both measures, for the output, dx0 and every parameter gradient (at full size with an
allowance, measured in the test, for what bf16 storage costs by itself).

A ReLU decision (pre-activation > 0) is an integer decided by floating point, and a feature map
stored in bf16 carries a relative error of 2^-9: about one decision in several hundred falls on the
other side of zero than in float64, and each such element changes a gradient element by its whole
size (tests/test_oracle_bf16_reading.py measures this on the CPU: several per cent in every
gradient tensor, whatever arithmetic computes the block).  Both sides therefore take the decisions
in the same precision, the kernel's: the library reports the decisions its kernels took
(dnb_block_relu_decisions) and the float64 oracle evaluates the block with them.  What is compared
is then unique, and the rest is checked to be valid: every decision that differs from the oracle's
own must be a tie within bf16 rounding (margin |z| / sqrt(gamma^2 + beta^2) <= MARGIN, at most
SHARE of all decisions)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import NAMES, assert_close, dev, pack_params_gpu, rel_errors, run_block_oracle

pytestmark = pytest.mark.gpu
TOL = 2e-2  # bf16 storage (the benchmark spec): relative error vs the float64 oracle, L2 and max-abs/max
# A stored conv output u carries half a bf16 ulp, 2^-9 |u|, and |u| reaches about six standard
# deviations of its channel: 0.012 of the channel's rms pre-activation from the store alone; the
# conv's bf16 operands (activations and weights, 2^-9 each) add as much again, and the features of
# earlier layers arrive with the error accumulated so far (the 2e-2 the output itself is allowed).
# Decisions with margin below m are a share of about 2 m pdf(0) <= m of all.
MARGIN = 0.1
SHARE = 0.02

CFGS = [
    wl.BlockCfg(2, 16, 8, 8, 3, 8, 32),        # small, one 64-pixel tile per image
    wl.BlockCfg(2, 32, 14, 14, 3, 16, 64),     # 196 pixels: three tiles and a ragged one
    wl.BlockCfg(1, 24, 7, 7, 2, 8, 32),        # 49 pixels: less than one tile, odd width
    wl.BlockCfg(2, 96, 28, 28, 2, 48, 192),    # DenseNet-161 widths (k = 48, B = 192)
    wl.BlockCfg(3, 64, 12, 20, 2, 32, 128),    # DenseNet-264 widths (k = 32, B = 128), non-square
    wl.BlockCfg(1, 96, 56, 56, 2, 48, 192),    # the first DenseNet-161 block's image size (row tiles of 5 rows, the last ragged)
]
IDS = [f"n{c.n}c{c.c0}h{c.h}w{c.w}m{c.layers}k{c.growth}B{c.bottleneck}" for c in CFGS]


def to_bf16_values(a):
    """fp32 array rounded to the nearest bf16 value (kept as fp32)."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).to(torch.float32).numpy()


def run_block_gpu_bf16(dnb, cfg, x0, layer_params, dy, concurrency=None, decisions=False, schedule=2):
    h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck,
                             dtype=dnb.DNB_BF16, layout=dnb.DNB_NHWC, schedule=schedule, eps=cfg.eps)
    try:
        if concurrency is not None:   # None: the library's default, what bench.py times
            dnb.dnb_block_set_concurrency(h, concurrency)
        params = dev(pack_params_gpu(dnb, h, layer_params))
        ws = torch.empty(dnb.dnb_block_workspace_bytes(h), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        nhwc = lambda a: torch.from_numpy(np.ascontiguousarray(a)).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)
        x0d, dyd = nhwc(x0), nhwc(dy)
        y = torch.full((cfg.n, cfg.h, cfg.w, cfg.c_out), float("nan"), dtype=torch.bfloat16, device="cuda")
        dx0 = torch.full((cfg.n, cfg.h, cfg.w, cfg.c0), float("nan"), dtype=torch.bfloat16, device="cuda")
        dparams = torch.full_like(params, float("nan"))
        dnb.dnb_block_forward(h, x0d, params, y, ws)
        dec = None
        if decisions:   # the ReLU decisions the kernels take, in the block's own (NHWC) layout
            dec = [torch.full((dnb.dnb_block_relu_decision_bytes(h, w),), 7, dtype=torch.uint8, device="cuda") for w in (1, 2)]
            dnb.dnb_block_relu_decisions(h, params, y, ws, dec[0], dec[1])
        dnb.dnb_block_backward(h, params, y, dyd, dx0, dparams, ws)
        torch.cuda.synchronize()
        back = lambda t: t.float().permute(0, 3, 1, 2).contiguous().cpu().numpy()
        out = {"y": back(y), "dx0": back(dx0), "dparams": dparams.cpu().numpy(),
               "mem": dnb.dnb_block_memory_breakdown(h)}
        if decisions:
            out["d1"], out["d2"] = dec[0].cpu().numpy(), dec[1].cpu().numpy()
        out["slices"] = {(l, name): slice(*(lambda o, c: (o, o + c))(*dnb.dnb_block_param_offset(h, l, NAMES.index(name))))
                         for l in range(1, cfg.layers + 1) for name in NAMES}
        return out
    finally:
        dnb.dnb_block_destroy(h)


def decisions_nchw(flat, cfg, widths):
    """The library's decision bytes ((n, h, w, c) per tensor, tensors one after the other) in the
    oracle's (n, c, h, w) order."""
    out, o = [], 0
    for c in widths:
        cnt = cfg.pixels * c
        out.append(flat[o:o + cnt].reshape(cfg.n, cfg.h, cfg.w, c).transpose(0, 3, 1, 2).ravel())
        o += cnt
    assert o == flat.size
    return np.concatenate(out)


def check_bf16_block(dnb, oracle, cfg, x0, lp, dy, storage_allowance=False):
    """GPU block against the plain float64 block evaluated with the kernels' ReLU decisions.
    storage_allowance=False: every tensor within TOL.  True (the full-size blocks: dozens of layers,
    10^5 pixels): bf16 storage by itself moves single gradient tensors by more than TOL even with
    identical decisions, so the oracle's storage-rounding variant, under the same decisions,
    measures that cost tensor by tensor (err_s = its distance from the plain block), and the GPU
    tensor must lie within err_s + TOL of the plain block on both measures, and within
    max(TOL, 1.5 err_s) in L2, max(TOL, 2.5 err_s) in the worst element: as close to the plain
    block as the storage format lets anything be.  The output y keeps TOL outright."""
    gpu = run_block_gpu_bf16(dnb, cfg, x0, lp, dy, decisions=True)
    assert set(np.unique(gpu["d1"])) <= {0, 1} and set(np.unique(gpu["d2"])) <= {0, 1}
    d1 = decisions_nchw(gpu["d1"], cfg, [cfg.c_in(l) for l in range(1, cfg.layers + 1)])
    d2 = decisions_nchw(gpu["d2"], cfg, [cfg.bottleneck] * cfg.layers)
    ores, osl, st = run_block_oracle(oracle, cfg, x0, lp, dy, decisions=(d1, d2))
    stor = run_block_oracle(oracle, cfg, x0, lp, dy, decisions=(d1, d2), bf16_storage=True)[0] if storage_allowance else None
    assert np.array_equal(gpu["y"][:, :cfg.c0], x0)
    assert_close(gpu["y"], ores.y, TOL, "y")

    def check(a, r, s_, what):
        if s_ is None:
            return assert_close(a, r, TOL, what)
        (l2, mx), (sl2, smx) = rel_errors(a, r), rel_errors(s_, r)
        ok = l2 <= sl2 + TOL and mx <= smx + TOL and l2 <= max(TOL, 1.5 * sl2) and mx <= max(TOL, 2.5 * smx)
        assert ok, f"{what}: rel L2 {l2:.3e} (storage alone {sl2:.3e}), rel max {mx:.3e} (storage alone {smx:.3e})"
    check(gpu["dx0"], ores.dx0, stor.dx0 if stor else None, "dx0")
    for l in range(1, cfg.layers + 1):
        for name in NAMES:
            sl = osl[(l, name)]
            check(gpu["dparams"][gpu["slices"][(l, name)]], ores.dparams[sl], stor.dparams[sl] if stor else None,
                  f"layer {l} d{name}")
    assert st["margin1"] <= MARGIN and st["margin2"] <= MARGIN, st
    assert st["count1"] <= SHARE * d1.size and st["count2"] <= SHARE * d2.size, st
    return gpu


@pytest.mark.parametrize("cfg", CFGS, ids=IDS)
def test_bf16_block_matches_oracle(dnb, oracle, cfg):
    x0, lp, dy = wl.make_block_inputs(cfg, affine="random")
    x0, dy = to_bf16_values(x0), to_bf16_values(dy)
    gpu = check_bf16_block(dnb, oracle, cfg, x0, lp, dy)
    plain, _ = run_block_oracle(oracle, cfg, x0, lp, dy)   # the output also with no decision imposed
    assert_close(gpu["y"], plain.y, TOL, "y vs the oracle's own decisions")


@pytest.mark.parametrize("cfg", CFGS, ids=IDS)
def test_bf16_schedules_bit_identical_and_their_bytes(dnb, cfg):
    """The shared-storage schedule (storage 1, 2, 3 re-populated in the backward pass), the
    store-everything schedule and the fused schedule (nothing materialised) compute the same
    numbers bit for bit; their feature-map bytes are the linear / quadratic / linear formulas."""
    x0, lp, dy = wl.make_block_inputs(cfg, affine="random")
    x0, dy = to_bf16_values(x0), to_bf16_values(dy)
    fused = run_block_gpu_bf16(dnb, cfg, x0, lp, dy, schedule=2)
    shared = run_block_gpu_bf16(dnb, cfg, x0, lp, dy, schedule=0)
    store = run_block_gpu_bf16(dnb, cfg, x0, lp, dy, schedule=1)
    for key in ("y", "dx0", "dparams"):
        assert np.array_equal(fused[key], shared[key]), key
        assert np.array_equal(fused[key], store[key]), key
    P, m, k, B = cfg.pixels, cfg.layers, cfg.growth, cfg.bottleneck
    cm, sigma = cfg.c_in(m), sum(cfg.c_in(l) for l in range(1, m + 1))
    grad = cfg.c_out * P * 4 + (cm + B) * P * 2
    assert fused["mem"]["peak_bytes"] == (m * B + m * k) * P * 2 + grad
    assert shared["mem"]["stored_fwd_bytes"] == (m * B + m * k) * P * 2 and shared["mem"]["shared_fwd_bytes"] == (2 * cm + B) * P * 2
    assert shared["mem"]["peak_bytes"] == (m * B + m * k + 2 * cm + B) * P * 2 + grad
    assert store["mem"]["peak_bytes"] == (2 * sigma + m * (2 * B + k)) * P * 2 + grad and store["mem"]["shared_fwd_bytes"] == 0


@pytest.mark.parametrize("cfg", [CFGS[1], CFGS[3]], ids=[IDS[1], IDS[3]])
def test_bf16_backward_chains_on_helper_streams_give_the_same_bits(dnb, cfg):
    """The weight gradients run on two helper streams beside the data-gradient chain; with
    concurrency off everything runs in program order on one stream.  Same kernels, same sums."""
    x0, lp, dy = wl.make_block_inputs(cfg, affine="random")
    x0, dy = to_bf16_values(x0), to_bf16_values(dy)
    a = run_block_gpu_bf16(dnb, cfg, x0, lp, dy, concurrency=True)
    b = run_block_gpu_bf16(dnb, cfg, x0, lp, dy, concurrency=False)
    for key in ("y", "dx0", "dparams"):
        assert np.array_equal(a[key], b[key]), key


def test_bf16_hip_graph_replays_match_eager(dnb):
    """The bf16 block's forward and backward captured in a HIP graph with the library's default
    stream order (the backward forks onto its helper stream and joins again), as bench.py times
    it: every replay, with eager work and synchronisation in between, reproduces the eager bits."""
    cfg = CFGS[3]
    x0, lp, dy = wl.make_block_inputs(cfg, affine="random")
    x0, dy = to_bf16_values(x0), to_bf16_values(dy)
    eager = run_block_gpu_bf16(dnb, cfg, x0, lp, dy)
    h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck,
                             dtype=dnb.DNB_BF16, layout=dnb.DNB_NHWC, schedule=dnb.DNB_SCHED_FUSED, eps=cfg.eps)
    params = dev(pack_params_gpu(dnb, h, lp))
    ws = torch.zeros(dnb.dnb_block_workspace_bytes(h), dtype=torch.uint8, device="cuda")
    nhwc = lambda a: torch.from_numpy(np.ascontiguousarray(a)).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)
    back = lambda t: t.float().permute(0, 3, 1, 2).contiguous().cpu().numpy()
    x0d, dyd = nhwc(x0), nhwc(dy)
    y = torch.zeros((cfg.n, cfg.h, cfg.w, cfg.c_out), dtype=torch.bfloat16, device="cuda")
    dx0 = torch.zeros((cfg.n, cfg.h, cfg.w, cfg.c0), dtype=torch.bfloat16, device="cuda")
    dparams = torch.zeros_like(params)

    def step():
        dnb.dnb_block_forward(h, x0d, params, y, ws)
        dnb.dnb_block_backward(h, params, y, dyd, dx0, dparams, ws)

    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(4):
        y.fill_(float("nan")); dx0.fill_(float("nan")); dparams.fill_(float("nan")); ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(back(y), eager["y"]), rep
        assert np.array_equal(back(dx0), eager["dx0"]), rep
        assert np.array_equal(dparams.cpu().numpy(), eager["dparams"]), rep
        _ = (torch.randn(1000, device="cuda") * 2).sum().item()  # unrelated eager work between replays
    dnb.dnb_block_destroy(h)


@pytest.mark.parametrize("which,i", [("config4", 0), ("config4", 2), ("config5", 1)])
def test_bf16_backward_is_exactly_linear_in_dy_at_full_size(dnb, which, i):
    """Doubling dy doubles dx0 and every parameter gradient bit for bit (each step of the backward
    pass is linear in dy, and a factor of 2 commutes with every rounding, bf16 included).  Needs no
    oracle, so it runs at the full size bench.py times: the 56x56 and 14x14 blocks of the
    DenseNet-161 shape and the 28x28 block of the DenseNet-264 shape, batch 32."""
    cfg = (wl.config4() if which == "config4" else wl.config5())[i]
    x0, lp, dy = wl.make_block_inputs(cfg, 80, 81, 82, affine="random")
    x0, dy = to_bf16_values(x0), to_bf16_values(dy)
    a = run_block_gpu_bf16(dnb, cfg, x0, lp, dy)
    b = run_block_gpu_bf16(dnb, cfg, x0, lp, 2.0 * dy)
    assert np.array_equal(a["y"], b["y"])
    assert np.isfinite(a["dx0"]).all() and np.isfinite(a["dparams"]).all()
    assert np.array_equal(2.0 * a["dx0"], b["dx0"])
    assert np.array_equal(2.0 * a["dparams"], b["dparams"])


@pytest.mark.parametrize("which,i", [("config4", 0), ("config4", 1), ("config4", 2), ("config4", 3),
                                     ("config5", 0), ("config5", 1), ("config5", 2), ("config5", 3)])
def test_bf16_full_size_blocks_match_oracle(dnb, oracle, which, i):
    """Every dense block of the DenseNet-161- and -264-shaped workloads exactly as bench.py times
    them (batch 32; 56x56, 28x28, 14x14 and 7x7 images; up to 64 layers, 2688 channels) against the
    plain float64 oracle, decisions as described at the top, with the allowance for what bf16
    storage costs by itself (see check_bf16_block)."""
    cfg = (wl.config4() if which == "config4" else wl.config5())[i]
    x0, lp, dy = wl.make_block_inputs(cfg, 90 + i, 91 + i, 92 + i, affine="random")
    x0, dy = to_bf16_values(x0), to_bf16_values(dy)
    check_bf16_block(dnb, oracle, cfg, x0, lp, dy, storage_allowance=True)


def test_bf16_bytes_and_unsupported_combinations(dnb):
    cfg = CFGS[3]
    h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck,
                             dtype=dnb.DNB_BF16, layout=dnb.DNB_NHWC, schedule=dnb.DNB_SCHED_FUSED)
    mm = dnb.dnb_block_memory_breakdown(h)
    P, m, k, B = cfg.pixels, cfg.layers, cfg.growth, cfg.bottleneck
    assert mm["stored_fwd_bytes"] == (m * B + m * k) * P * 2 and mm["shared_fwd_bytes"] == 0
    assert mm["grad_bytes"] == cfg.c_out * P * 4 + (cfg.c_in(m) + B) * P * 2
    assert mm["peak_bytes"] == mm["stored_fwd_bytes"] + mm["grad_bytes"]
    dnb.dnb_block_destroy(h)
    for kw in (dict(layout=dnb.DNB_NCHW), dict(bottleneck=0), dict(c0=20)):
        args = dict(n=2, c0=16, h=8, w=8, layers=2, growth=8, bottleneck=32, dtype=dnb.DNB_BF16,
                    layout=dnb.DNB_NHWC, schedule=dnb.DNB_SCHED_FUSED)
        args.update(kw)
        with pytest.raises(dnb.binding.DnbError) as e:
            dnb.dnb_block_create(**args)
        assert e.value.status == dnb.DNB_E_UNSUPPORTED


# ------------------------------------------------------------------ single operations

def nhwc_bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a)).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)


def nhwc_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a)).permute(0, 2, 3, 1).contiguous().to("cuda", torch.float32)


def back(t):
    return t.float().permute(0, 3, 1, 2).contiguous().cpu().numpy()


OP_SHAPES = [(2, 16, 8, 8, 8, 1), (2, 32, 8, 8, 8, 3), (2, 8, 32, 8, 8, 3), (1, 24, 16, 7, 7, 3), (2, 40, 64, 14, 14, 1),
             (1, 192, 48, 12, 20, 3), (2, 48, 192, 9, 11, 3), (1, 200, 192, 10, 10, 1),
             # 1x1 with nine input chunks, the last one 8 channels wide (forward takes the four-chunk ring);
             # weight gradient over 3 x 2 channel groups with a ragged last pixel tile
             (2, 520, 200, 9, 7, 1),
             # 1x1 whose data gradient reduces over nine chunks; output channels over three workgroup rows
             (1, 64, 576, 6, 6, 1),
             # 3x3 weight gradient: two row tiles per image and two channel groups; then more tiles than
             # splits (two tiles per workgroup)
             (5, 72, 16, 14, 14, 3), (130, 8, 8, 4, 4, 3),
             # 56-pixel rows as in the first ImageNet-shaped block: the 3x3's halo is 57 pixels a side, the weight
             # gradient's row tiles hold 5 rows and the last one 1
             (1, 64, 48, 56, 56, 3), (1, 32, 128, 56, 56, 3)]


@pytest.mark.parametrize("n,cin,cout,h,w,ks", OP_SHAPES)
@pytest.mark.parametrize("g_f32", [0, 1])
def test_nhwc_conv_ops(dnb, oracle, n, cin, cout, h, w, ks, g_f32):
    r = np.random.default_rng(5)
    x = to_bf16_values(r.standard_normal((n, cin, h, w)).astype(np.float32))
    wgt = to_bf16_values((r.standard_normal((cout, cin, ks, ks)) * np.sqrt(2.0 / (cin * ks * ks))).astype(np.float32))
    g = to_bf16_values(r.standard_normal((n, cout, h, w)).astype(np.float32))
    scratch = torch.empty(dnb.dnb_op_nhwc_scratch_bytes(n, cin, cout, h, w, ks), dtype=torch.uint8, device="cuda")
    d_w = dev(wgt)
    d_x = nhwc_bf16(x)
    d_g = nhwc_f32(g) if g_f32 else nhwc_bf16(g)
    out = torch.full((n, h, w, cout), float("nan"), dtype=torch.bfloat16, device="cuda")
    dnb.dnb_op_nhwc_conv_forward(d_x, cin, d_w, out, cout, n, cin, cout, h, w, ks, scratch)
    torch.cuda.synchronize()
    assert_close(back(out), oracle.conv_forward(x, wgt), 1e-2, "forward")
    din = torch.full((n, h, w, cin), float("nan"), dtype=torch.bfloat16, device="cuda")
    dnb.dnb_op_nhwc_conv_dgrad(d_g, cout, g_f32, d_w, din, cin, n, cin, cout, h, w, ks, scratch)
    torch.cuda.synchronize()
    assert_close(back(din), oracle.conv_dgrad(g, wgt), 1e-2, "dgrad")
    dw = torch.full(wgt.shape, float("nan"), device="cuda")
    dnb.dnb_op_nhwc_conv_wgrad(d_x, cin, d_g, cout, g_f32, dw, n, cin, cout, h, w, ks, scratch)
    torch.cuda.synchronize()
    assert_close(dw.cpu().numpy(), oracle.conv_wgrad(x, g, ks), 1e-2, "wgrad")


@pytest.mark.parametrize("n,cin,cout,h,w,ks", [(32, 336, 192, 56, 56, 1), (32, 192, 48, 56, 56, 3), (32, 720, 192, 28, 28, 1),
                                               (32, 192, 48, 28, 28, 3), (32, 224, 128, 56, 56, 1), (32, 128, 32, 56, 56, 3),
                                               (32, 480, 128, 28, 28, 1), (32, 2064, 192, 14, 14, 1)])
@pytest.mark.parametrize("g_f32", [0, 1])
def test_nhwc_conv_ops_at_benchmark_pixel_counts(dnb, oracle, n, cin, cout, h, w, ks, g_f32):
    """The convolutions of the DenseNet-161- and -264-shaped blocks (widest layer of the 56x56 and
    28x28 blocks, k = 48 / B = 192 and k = 32 / B = 128, and the widest 14x14 layer) at batch 32:
    forward, data gradient and weight gradient at the pixel counts bench.py runs them at."""
    test_nhwc_conv_ops(dnb, oracle, n, cin, cout, h, w, ks, g_f32)


@pytest.mark.parametrize("ks", [1, 3])
def test_nhwc_conv_ops_on_channel_slices_of_wider_slabs(dnb, oracle, ks):
    """Pixel strides wider than the channel ranges, as the block addresses its slabs in place: the
    input is channels 16..47 of a 64-channel tensor, the output channels 8..31 of a 40-channel one
    (an fp32 one for the data gradient's operand); everything outside the output range stays
    untouched."""
    n, cin, cout, h, w = 2, 32, 24, 9, 8
    r = np.random.default_rng(11)
    xs = to_bf16_values(r.standard_normal((n, 64, h, w)).astype(np.float32))
    gs = to_bf16_values(r.standard_normal((n, 40, h, w)).astype(np.float32))
    wgt = to_bf16_values((r.standard_normal((cout, cin, ks, ks)) * np.sqrt(2.0 / (cin * ks * ks))).astype(np.float32))
    x, g = xs[:, 16:48], gs[:, 8:32]
    scratch = torch.empty(dnb.dnb_op_nhwc_scratch_bytes(n, cin, cout, h, w, ks), dtype=torch.uint8, device="cuda")
    d_w, d_xs, d_gs, d_gs32 = dev(wgt), nhwc_bf16(xs), nhwc_bf16(gs), nhwc_f32(gs)
    sentinel = 7.0
    out = torch.full((n, h, w, 40), sentinel, dtype=torch.bfloat16, device="cuda")
    dnb.dnb_op_nhwc_conv_forward(d_xs.data_ptr() + 16 * 2, 64, d_w, out.data_ptr() + 8 * 2, 40, n, cin, cout, h, w, ks, scratch)
    torch.cuda.synchronize()
    o = back(out)
    assert_close(o[:, 8:32], oracle.conv_forward(x, wgt), 1e-2, "forward")
    assert np.all(o[:, :8] == sentinel) and np.all(o[:, 32:] == sentinel)
    for g_f32, d_g, esz in ((0, d_gs, 2), (1, d_gs32, 4)):
        din = torch.full((n, h, w, 64), sentinel, dtype=torch.bfloat16, device="cuda")
        dnb.dnb_op_nhwc_conv_dgrad(d_g.data_ptr() + 8 * esz, 40, g_f32, d_w, din.data_ptr() + 16 * 2, 64, n, cin, cout, h, w, ks,
                                   scratch)
        torch.cuda.synchronize()
        di = back(din)
        assert_close(di[:, 16:48], oracle.conv_dgrad(g, wgt), 1e-2, "dgrad")
        assert np.all(di[:, :16] == sentinel) and np.all(di[:, 48:] == sentinel)
        dw = torch.full(wgt.shape, float("nan"), device="cuda")
        dnb.dnb_op_nhwc_conv_wgrad(d_xs.data_ptr() + 16 * 2, 64, d_g.data_ptr() + 8 * esz, 40, g_f32, dw, n, cin, cout, h, w, ks,
                                   scratch)
        torch.cuda.synchronize()
        assert_close(dw.cpu().numpy(), oracle.conv_wgrad(x, g, ks), 1e-2, "wgrad")


@pytest.mark.parametrize("g_f32", [0, 1])
def test_nhwc_wgrad_rows_wider_than_the_row_tiled_kernel_takes(dnb, oracle, g_f32):
    """96-pixel rows: the 3x3 weight gradient falls back to the kernel that stages 64-pixel tiles
    once per tap (forward and data gradient do not take such rows at all)."""
    n, cin, cout, h, w = 1, 8, 8, 2, 96
    r = np.random.default_rng(9)
    x = to_bf16_values(r.standard_normal((n, cin, h, w)).astype(np.float32))
    g = to_bf16_values(r.standard_normal((n, cout, h, w)).astype(np.float32))
    scratch = torch.empty(dnb.dnb_op_nhwc_scratch_bytes(n, cin, cout, h, w, 3), dtype=torch.uint8, device="cuda")
    dw = torch.full((cout, cin, 3, 3), float("nan"), device="cuda")
    dnb.dnb_op_nhwc_conv_wgrad(nhwc_bf16(x), cin, nhwc_f32(g) if g_f32 else nhwc_bf16(g), cout, g_f32, dw, n, cin, cout, h, w, 3,
                               scratch)
    torch.cuda.synchronize()
    assert_close(dw.cpu().numpy(), oracle.conv_wgrad(x, g, 3), 1e-2, "wgrad")


@pytest.mark.parametrize("shape", [(2, 16, 8, 8), (3, 40, 7, 5), (2, 264, 6, 6), (4, 24, 40, 40), (2, 192, 28, 28),
                                   (32, 336, 56, 56), (32, 192, 56, 56), (32, 720, 28, 28)])
@pytest.mark.parametrize("accumulate", [0, 1])
def test_nhwc_bn_relu_backward(dnb, oracle, shape, accumulate):
    """(The last three shapes: the BN backward passes of the 56x56 and 28x28 blocks at batch 32.)"""
    r = np.random.default_rng(6)
    n, c, h, w = shape
    gamma = (1 + 0.3 * r.standard_normal(c)).astype(np.float32)
    beta = (0.3 * r.standard_normal(c)).astype(np.float32)
    x = to_bf16_values((r.standard_normal(shape) * 1.5 + 0.3).astype(np.float32))
    if n * c * h * w > 1e6:
        # tens of millions of elements: a few pre-activations lie within fp32 rounding of zero, where
        # the decision dz = dact * [z > 0] depends on the precision.  Move every element within 1e-3
        # of zero a bf16 step or two further out, so that the decision is the same in any precision.
        for _ in range(8):
            mu, var = x.mean(axis=(0, 2, 3), dtype=np.float64), x.var(axis=(0, 2, 3), dtype=np.float64)
            z = gamma[None, :, None, None] * (x - mu[None, :, None, None]) / np.sqrt(var + 1e-5)[None, :, None, None] \
                + beta[None, :, None, None]
            near = np.abs(z) < 1e-3
            if not near.any():
                break
            step = np.where(z >= 0, 1.0, -1.0) * (np.sign(gamma) * (0.03 + 0.003 / np.abs(gamma)))[None, :, None, None]
            x = np.where(near, to_bf16_values((x + step).astype(np.float32)), x).astype(np.float32)
        assert not near.any()
    dact = to_bf16_values(r.standard_normal(shape).astype(np.float32))
    base = r.standard_normal(shape).astype(np.float32)
    eps = 1e-5
    z, omean, ovar = oracle.bn_forward(x, gamma, beta, eps)
    mean, istd = dev(omean.astype(np.float32)), dev((1 / np.sqrt(ovar + eps)).astype(np.float32))
    scratch = torch.empty(dnb.dnb_op_nhwc_scratch_bytes(n, c, c, h, w, 1), dtype=torch.uint8, device="cuda")
    dg, db = torch.empty(c, device="cuda"), torch.empty(c, device="cuda")
    d_x, d_d = nhwc_bf16(x), nhwc_bf16(dact)
    P = n * h * w
    if accumulate:
        acc = nhwc_f32(base)
        dnb.dnb_op_nhwc_bn_relu_backward(d_x, c, d_d, c, None, 0, acc, c, P, c, dev(gamma), dev(beta), mean, istd, dg, db, scratch)
        got = back(acc)
    else:
        dnb.dnb_op_nhwc_bn_relu_backward(d_x, c, d_d, c, d_d, c, None, 0, P, c, dev(gamma), dev(beta), mean, istd, dg, db, scratch)
        got = back(d_d)
    torch.cuda.synchronize()
    # the mask is taken in fp32 from the same bf16 x: recompute z in fp32 like the kernel
    dz = oracle.relu_backward(oracle.relu(z), dact)
    odu, odg, odb = oracle.bn_backward(x, dz, gamma, omean, ovar, eps)
    if accumulate:
        odu = odu + base
    assert_close(got, odu, 1e-2, "du")
    assert_close(dg.cpu().numpy(), odg, 1e-2, "dgamma")
    assert_close(db.cpu().numpy(), odb, 1e-2, "dbeta")
