"""GPU parity of the whole ImageNet-shaped training step (7x7 stride-2 stem, BN-ReLU, 3x3 stride-2
max pool, four dense blocks, transitions, head, loss; bf16 feature maps, NHWC) through the C ABI
against the float64 oracle on the same seeded, bf16-rounded inputs.

Both kinds of integer that the step decides in floating point -- ReLU decisions and the position of
the maximum inside each pooling window -- are taken in the kernel's precision on both sides: the
library reports them (dnb_inet_decisions), the oracle evaluates the step with them, and the ones
that differ from the oracle's own are checked to be ties within bf16 rounding.  Tolerance: loss, logits
and every gradient tensor within 2e-2 plus what bf16 storage costs by itself (the oracle's
storage-rounding variant under the same decisions, measured in the test; on the small networks of
these tests, whose last block normalises over a few dozen samples, that alone is a few per cent)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import assert_close, rel_errors
from harness import run_inet_gpu

pytestmark = pytest.mark.gpu
TOL = 2e-2
MARGIN = 0.15   # ReLU ties: as in test_gpu_bf16.py, a little wider for the few-sample statistics of the tiny nets
SHARE = 0.02


def to_bf16_values(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).to(torch.float32).numpy()


def check_step(dnb, oracle, cfg, schedule=2):
    x, labels, params = wl.make_inet_inputs(cfg, affine="random")
    params["tail"]["bl"] = np.linspace(-0.3, 0.2, cfg.classes).astype(np.float32)
    x = to_bf16_values(x)
    s, flat, loss, logits, dp, dec = run_inet_gpu(dnb, oracle, cfg, x, labels, params, schedule, decisions=True)
    assert set(np.unique(dec[0])) <= {0, 1} and dec[1].max() <= 8
    oloss, odp, ologits, st = oracle.inet_step(s, x, labels, flat, decisions=dec)
    sloss, sdp, slogits, _ = oracle.inet_step(s, x, labels, flat, decisions=dec, bf16_storage=True)
    assert abs(loss - oloss) <= abs(sloss - oloss) + TOL * abs(oloss), (loss, oloss, sloss)

    def check(a, r, sv, what):
        (l2, mx), (sl2, smx) = rel_errors(a, r), rel_errors(sv, r)
        # within TOL of what storage alone costs where that is small; where storage alone already moves a
        # tensor by tens of per cent (sums with heavy cancellation, such as the stem's dbeta over mostly
        # inactive channels) two different roundings are as far from each other as from the truth: then
        # within half as much again (twice and a half for the worst element)
        assert l2 <= max(sl2 + TOL, 1.5 * sl2) and mx <= max(smx + TOL, 2.5 * smx), \
            f"{what}: rel L2 {l2:.3e} (storage alone {sl2:.3e}), rel max {mx:.3e} (storage alone {smx:.3e})"
    check(logits, ologits, slogits, "logits")
    for name, sl in oracle.inet_param_slices(s).items():
        check(dp[sl], odp[sl], sdp[sl], f"d{name}")
    # The decisions that differ from the oracle's own must be ties within bf16 rounding.  How wide such
    # ties are depends on the batch: at batch 2 the last blocks normalise over 98 samples and channels
    # with almost no batch variance amplify a rounding into a large move of the pre-activation.  The
    # measuring stick is again the oracle's storage-rounding variant: its own decisions, imposed on the
    # plain step, differ in count_s places with margin_s; the kernels' may differ half as much again.
    nr, npool = oracle.inet_decision_counts(s)
    _, _, _, sdec = oracle.inet_step(s, x, labels, flat, backward=False, decisions="write", bf16_storage=True)
    _, _, _, ss = oracle.inet_step(s, x, labels, flat, backward=False, decisions=sdec)
    assert st["relu_margin"] <= max(MARGIN, 1.5 * ss["relu_margin"]) and st["relu_count"] <= max(SHARE * nr, 1.5 * ss["relu_count"]), (st, ss)
    assert st["pool_margin"] <= max(MARGIN, 1.5 * ss["pool_margin"]) and st["pool_count"] <= max(SHARE * npool, 1.5 * ss["pool_count"]), (st, ss)
    return loss, logits, dp


CFGS = [wl.InetCfg(8, 64, 8, (2, 2, 2, 2), 10), wl.InetCfg(3, 96, 16, (2, 4, 2, 2), 7)]


@pytest.mark.parametrize("cfg", CFGS, ids=["n8i64k8", "n3i96k16"])
@pytest.mark.parametrize("schedule", [0, 1, 2])
def test_inet_step_matches_oracle(dnb, oracle, cfg, schedule):
    check_step(dnb, oracle, cfg, schedule)


def test_inet_schedules_agree_bitwise(dnb, oracle):
    cfg = CFGS[0]
    x, labels, params = wl.make_inet_inputs(cfg, affine="random")
    x = to_bf16_values(x)
    runs = [run_inet_gpu(dnb, oracle, cfg, x, labels, params, sch) for sch in (0, 1, 2)]
    for r in runs[1:]:
        assert r[2] == runs[0][2] and np.array_equal(r[3], runs[0][3]) and np.array_equal(r[4], runs[0][4])


@pytest.mark.parametrize("which", ["config4", "config5"])
def test_inet_full_widths_and_depths_at_batch_2(dnb, oracle, which):
    """The DenseNet-161- and DenseNet-264-shaped networks with every width, depth and image size of
    the benchmark workloads (224x224 inputs, blocks 6-12-36-24 at k = 48 and 6-12-64-48 at k = 32,
    1000 classes) at batch 2, which the oracle finishes in seconds."""
    cfg = wl.inet_config4(2) if which == "config4" else wl.inet_config5(2)
    check_step(dnb, oracle, cfg)


def test_inet_hip_graph_replays_match_eager(dnb, oracle):
    """The whole ImageNet-shaped step captured in a HIP graph with the library's default stream order
    (the blocks' backward passes fork onto their helper stream and join again), as bench.py times it:
    every replay, with eager work and synchronisation in between and the workspace poisoned before
    it, reproduces the eager bits of the loss, the logits and every parameter gradient."""
    from harness import dev, pack_inet
    cfg = CFGS[1]
    x, labels, params = wl.make_inet_inputs(cfg, affine="random")
    x = to_bf16_values(x)
    s, flat, loss0, logits0, dp0 = run_inet_gpu(dnb, oracle, cfg, x, labels, params, 2)
    net = dnb.dnb_inet_create(cfg.n, cfg.image, cfg.growth, cfg.layers, cfg.classes, schedule=2, eps=cfg.eps)
    p = dev(flat.astype(np.float32))
    dp = torch.zeros_like(p)
    ws = torch.zeros(dnb.dnb_inet_workspace_bytes(net), dtype=torch.uint8, device="cuda")
    xd = torch.from_numpy(np.ascontiguousarray(x)).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)
    lab = torch.from_numpy(labels).to("cuda")
    loss = torch.zeros((1,), device="cuda")
    logits = torch.zeros((cfg.n, cfg.classes), device="cuda")

    def step():
        dnb.dnb_inet_forward(net, xd, lab, p, loss, logits, ws)
        dnb.dnb_inet_backward(net, xd, p, dp, ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(4):
        dp.fill_(float("nan")); logits.fill_(float("nan")); loss.fill_(float("nan")); ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert float(loss.item()) == loss0, rep
        assert np.array_equal(logits.cpu().numpy(), logits0), rep
        assert np.array_equal(dp.cpu().numpy(), dp0), rep
        _ = (torch.randn(1000, device="cuda") * 2).sum().item()  # unrelated eager work between replays
    dnb.dnb_inet_destroy(net)
