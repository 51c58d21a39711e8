#!/usr/bin/env python3
"""Benchmark of the memory-efficient DenseNet training step on one MI355X.

A step = forward + backward of the workload through the C ABI, inputs resident in HBM.  Default
workload: DenseNet-BC L=100, k=12, batch 64, fp32 (benchmark configs[1]) as a whole network --
stem conv, three dense blocks of 16 bottleneck layers, two transitions, BN-ReLU-pool-linear head
and mean softmax cross-entropy (no optimiser update: the metric is forward + backward).  Prints
ONE JSON line with training images/s of the fastest linear-memory schedule (fused), the same
workload's dense blocks alone, the rates of the paper-literal shared-storage schedule and of the
store-everything schedule (recompute overhead), exact peak feature-map bytes, the roofline of the
dominant kernel measured live with events on the launch stream, and the CPU oracle timed on the
host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_F32_PEAK_TF = 157.3    # MI355X dense fp32 matrix


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2", "config3", "config4", "config5"],
                    help="config2 is the metric's workload; config4/5 are the bf16 NHWC ImageNet-shaped block sets (diagnostic)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--scope", default="auto", choices=["auto", "net", "blocks"],
                    help="net: the whole training step (stem, dense blocks, transitions, head, loss; configs 2-3); "
                         "blocks: the dense blocks alone; auto = net where it is built")
    ap.add_argument("--schedule", default="fused", choices=["shared", "store_all", "fused"],
                    help="fused: BN+ReLU recomputed inside the conv operand loads (default, fastest linear-memory schedule); "
                         "shared: storage 1/2/3 materialised as in the paper; store_all: every intermediate kept")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-compare", action="store_true", help="skip timing the other schedule")
    ap.add_argument("--only-block", type=int, default=-1, help="time a single dense block of the workload (diagnostic)")
    ap.add_argument("--serial", action="store_true", help="no helper streams in backward (the library's default for fp32)")
    ap.add_argument("--concurrent", action="store_true", help="weight gradients on helper streams in backward (the library's default for bf16)")
    ap.add_argument("--forward-only", action="store_true", help="time the forward pass alone (diagnostic, not the metric)")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the other workloads (config3: whole network; config4 / config5: dense-block sets) that the "
                         "default run times after the metric's workload and reports as objects of their own")
    return ap.parse_args()


def workload_blocks(wl, name, batch):
    if name == "config1":
        return [wl.config1()], "dense block n2 c16 8x8 m4 k12 B48 fp32 NCHW"
    if name == "config2":
        b = batch or 64
        return wl.config2(b), f"DenseNet-BC L=100 k=12 batch {b} fp32 NCHW, 3 dense blocks x 16 layers (fwd+bwd)"
    if name == "config3":
        b = batch or 64
        return wl.config3(b), f"DenseNet-BC L=250 k=24 batch {b} fp32 NCHW, 3 dense blocks x 41 layers (fwd+bwd)"
    if name == "config4":
        b = batch or 32
        return wl.config4(b), f"DenseNet-161-shaped k=48 batch {b} bf16 NHWC, dense blocks 6-12-36-24 (fwd+bwd)"
    b = batch or 32
    return wl.config5(b), f"DenseNet-264-shaped k=32 batch {b} bf16 NHWC, dense blocks 6-12-64-48 (fwd+bwd)"


class BlockRun:
    """Device buffers + handle of one dense block."""

    def __init__(self, dnb, torch, wl, cfg, schedule, seed, bf16=False):
        from harness import dev, pack_params_gpu
        self.cfg = cfg
        self.dnb = dnb
        kw = dict(dtype=dnb.DNB_BF16, layout=dnb.DNB_NHWC) if bf16 else {}
        self.h = dnb.dnb_block_create(cfg.n, cfg.c0, cfg.h, cfg.w, cfg.layers, cfg.growth, cfg.bottleneck,
                                      schedule=schedule, eps=cfg.eps, **kw)
        x0, lp, dy = wl.make_block_inputs(cfg, seed, seed + 1, seed + 2, affine="ones")
        if bf16:
            nhwc = lambda a: torch.from_numpy(a).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)
            self.x0, self.dy = nhwc(x0), nhwc(dy)
            self.y = torch.empty((cfg.n, cfg.h, cfg.w, cfg.c_out), dtype=torch.bfloat16, device="cuda")
        else:
            self.x0, self.dy = dev(x0), dev(dy)
            self.y = torch.empty((cfg.n, cfg.c_out, cfg.h, cfg.w), dtype=torch.float32, device="cuda")
        self.params = dev(pack_params_gpu(dnb, self.h, lp))
        self.dparams = torch.empty_like(self.params)
        self.dx0 = torch.empty_like(self.x0)
        self.ws = torch.empty(dnb.dnb_block_workspace_bytes(self.h), dtype=torch.uint8, device="cuda")
        self.mem = dnb.dnb_block_memory_breakdown(self.h)

    def close(self):
        if self.h is not None:
            self.dnb.dnb_block_destroy(self.h)
            self.h = None


class NetRun:
    """Device buffers + handle of one whole network."""

    def __init__(self, dnb, torch, wl, ncfg, schedule):
        import numpy as np
        from harness import dev
        self.cfg = ncfg
        self.h = dnb.dnb_net_create(ncfg.n, ncfg.image, ncfg.depth, ncfg.growth, ncfg.classes, schedule=schedule,
                                    eps=ncfg.eps)
        x, labels, params = wl.make_net_inputs(ncfg)
        flat = np.zeros(dnb.dnb_net_param_count(self.h), dtype=np.float32)

        def put(part, arr):
            off, cnt = dnb.dnb_net_param_offset(self.h, part)
            assert cnt == arr.size
            flat[off:off + cnt] = np.asarray(arr, dtype=np.float32).ravel()

        put(dnb.DNB_NP_STEM, params["stem"])
        for b, bc in enumerate(ncfg.blocks()):
            hb = dnb.dnb_block_create(bc.n, bc.c0, bc.h, bc.w, bc.layers, bc.growth, bc.bottleneck, eps=bc.eps)
            from harness import pack_params_gpu
            put(dnb.DNB_NP_BLOCK0 + b, pack_params_gpu(dnb, hb, params[f"block{b}"]))
            dnb.dnb_block_destroy(hb)
        for b in (0, 1):
            for i, name in enumerate(("g", "b", "W")):
                put(dnb.DNB_NP_TRANS0_G + 3 * b + i, params[f"trans{b}"][name])
        for i, name in enumerate(("g", "b", "Wl", "bl")):
            put(dnb.DNB_NP_TAIL_G + i, params["tail"][name])
        self.x, self.labels = dev(x), torch.from_numpy(labels).to("cuda")
        self.params = dev(flat)
        self.dparams = torch.empty_like(self.params)
        self.loss = torch.zeros(1, device="cuda")
        self.ws = torch.empty(dnb.dnb_net_workspace_bytes(self.h), dtype=torch.uint8, device="cuda")
        self.peak = dnb.dnb_net_peak_bytes(self.h)
        self.workspace = dnb.dnb_net_workspace_bytes(self.h)


class InetRun:
    """Device buffers + handle of one whole ImageNet-shaped network (bf16 NHWC)."""

    def __init__(self, dnb, torch, wl, icfg, schedule):
        import numpy as np
        from harness import dev, pack_params_gpu
        self.cfg = icfg
        self.dnb = dnb
        self.h = dnb.dnb_inet_create(icfg.n, icfg.image, icfg.growth, icfg.layers, icfg.classes, schedule=schedule, eps=icfg.eps)
        x, labels, params = wl.make_inet_inputs(icfg)
        flat = np.zeros(dnb.dnb_inet_param_count(self.h), dtype=np.float32)

        def put(part, arr):
            off, cnt = dnb.dnb_inet_param_offset(self.h, part)
            assert cnt == arr.size
            flat[off:off + cnt] = np.asarray(arr, dtype=np.float32).ravel()

        put(dnb.DNB_IP_STEM_W, params["stem"]["W"])
        put(dnb.DNB_IP_STEM_G, params["stem"]["g"])
        put(dnb.DNB_IP_STEM_B, params["stem"]["b"])
        for b, bc in enumerate(icfg.blocks()):
            hb = dnb.dnb_block_create(1, bc.c0, 8, 8, bc.layers, bc.growth, bc.bottleneck, eps=bc.eps)   # the pack layout only
            put(dnb.DNB_IP_BLOCK0 + 4 * b, pack_params_gpu(dnb, hb, params[f"block{b}"]))
            dnb.dnb_block_destroy(hb)
            pre = params[f"trans{b}"] if b < 3 else params["tail"]
            put(dnb.DNB_IP_BLOCK0 + 4 * b + 1, pre["g"])
            put(dnb.DNB_IP_BLOCK0 + 4 * b + 2, pre["b"])
            put(dnb.DNB_IP_BLOCK0 + 4 * b + 3, pre["W"] if b < 3 else pre["Wl"])
        put(dnb.DNB_IP_TAIL_BL, params["tail"]["bl"])
        self.x = torch.from_numpy(x).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)
        self.labels = torch.from_numpy(labels).to("cuda")
        self.params = dev(flat)
        self.dparams = torch.empty_like(self.params)
        self.loss = torch.zeros(1, device="cuda")
        self.ws = torch.empty(dnb.dnb_inet_workspace_bytes(self.h), dtype=torch.uint8, device="cuda")
        self.peak = dnb.dnb_inet_peak_bytes(self.h)
        self.workspace = dnb.dnb_inet_workspace_bytes(self.h)

    def close(self):
        if self.h is not None:
            self.dnb.dnb_inet_destroy(self.h)
            self.h = None


def make_inet_step(dnb, r, forward_only=False):
    def step():
        dnb.dnb_inet_forward(r.h, r.x, r.labels, r.params, r.loss, None, r.ws)
        if not forward_only:
            dnb.dnb_inet_backward(r.h, r.x, r.params, r.dparams, r.ws)
    return step


def make_net_step(dnb, r, forward_only=False):
    def step():
        dnb.dnb_net_forward(r.h, r.x, r.labels, r.params, r.loss, None, r.ws)
        if not forward_only:
            dnb.dnb_net_backward(r.h, r.x, r.params, r.dparams, r.ws)
    return step


def make_step(dnb, runs, forward_only=False):
    def step():
        for r in runs:
            dnb.dnb_block_forward(r.h, r.x0, r.params, r.y, r.ws)
        if forward_only:
            return
        for r in reversed(runs):
            dnb.dnb_block_backward(r.h, r.params, r.y, r.dy, r.dx0, r.dparams, r.ws)
    return step


def time_steps(torch, step, steps, warmup, use_graph):
    """Returns (seconds for `steps` steps, whether a graph was used)."""
    if use_graph:
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            step()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        run = g.replay
    else:
        run = step
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def event_time_ms(torch, fn, reps):
    """Average milliseconds of fn() (one or more launches on the current stream) over reps."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


# The kernel with the largest share of the step in the committed rocprofv3 summaries (profiles/), per
# workload, and the summary that holds its measured HBM bytes per launch (two rocprofv3 --pmc runs,
# FETCH_SIZE then WRITE_SIZE, each scaled by the copy kernel of known size): the figure is read from
# the line "traffic_bytes_per_launch: N" of that file, so it is whatever the committed profile says.
DOMINANT = {"config2:64": ("k_wgrad_pair<3, 4, 1, 3, true>", "bc100_b64_fp32_wgrad_pair_hbm_traffic.txt"),
            "config3:64": ("k_wgrad_pair<3, 4, 2, 2, true>", "bc250_b64_fp32_wgrad_pair_hbm_traffic.txt")}


def measured_traffic(key):
    import re
    if key not in DOMINANT:
        return None
    path = os.path.join(ROOT, "profiles", DOMINANT[key][1])
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", open(path).read(), flags=re.M)
    return int(m.group(1)) if m else None


def dominant_kernel_roofline(dnb, torch, runs, traffic_key):
    """Live measurement of the kernel with the largest share of the step in the committed
    rocprofv3 summary (profiles/): the launch that holds a bottleneck layer's two weight
    gradients (1x1 and 3x3, BN+ReLU of their activation operands recomputed in the operand
    loads, fp32 MFMA with pixels on the K axis) and the reduction pass of the layer's first BN
    backward.  Algorithmic work per launch: 2*P*C_l*B + 18*P*B*k flops; 4*(P*(C_l + B) + C_l*B)
    + 4*(P*(B + k) + 9*B*k) + 8*P*C_l bytes (the BN reduction reads the features and their
    gradient once more).  The roof whose time over the launches below is the larger is reported:
    at these widths HBM (8 TB/s).  The launches are the layers of the workload's largest dense
    block that take this instantiation (C_l >= 49), with the block's own slab strides, through
    the single-op entry point, each launch stamping its own pair of events at the kernel's start
    and end on the launch stream.  (Inside the step the launch also adds up the previous layer's
    weight-gradient partial sums: about 20 MB more.)"""
    import numpy as np
    cfg = runs[0].cfg
    n, B, k, h, w, m = cfg.n, cfg.bottleneck, cfg.growth, cfg.h, cfg.w, cfg.layers
    hw = h * w
    c_out = cfg.c0 + m * k
    dev = "cuda"
    y = torch.randn((n, c_out, h, w), device=dev)
    G = torch.randn((n, c_out, h, w), device=dev)
    db = torch.randn((n, B, h, w), device=dev)
    bact = torch.randn((n, B, h, w), device=dev)
    fold2 = torch.stack([torch.ones(B, device=dev), torch.zeros(B, device=dev)], dim=1).contiguous()
    dw3 = torch.empty((k, B, 3, 3), device=dev)
    cs = [cfg.c0 + (l - 1) * k for l in range(1, m + 1) if cfg.c0 + (l - 1) * k >= 49]
    reps = 3
    ms_sum, flops, nbytes, launches = 0.0, 0.0, 0.0, 0
    for c in cs:
        fold1 = torch.stack([torch.ones(c, device=dev), torch.zeros(c, device=dev)], dim=1).contiguous()
        dw1 = torch.empty((B, c, 1, 1), device=dev)
        dact = torch.randn((n, c, h, w), device=dev)
        ones, zeros = torch.ones(c, device=dev), torch.zeros(c, device=dev)
        scratch = torch.empty(dnb.dnb_op_layer_wgrads_scratch_bytes(n, c, B, k, h, w), dtype=torch.uint8, device=dev)
        g = G[:, c:c + k]     # the slab's slice of this layer, image stride c_out*hw
        args = (y, c_out * hw, fold1, db, dw1, c, bact, fold2, g, c_out * hw, dw3, n, B, k, h, w, scratch)
        kw = dict(bn_dact=dact, bn_gamma=ones, bn_beta=zeros, bn_mean=zeros, bn_istd=ones)
        dnb.dnb_op_layer_wgrads(*args, **kw)   # warm
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in evs:
            e0.record(); e1.record()   # creates the handles; the launch below re-stamps both
            dnb.dnb_op_layer_wgrads(*args, ev_start=e0, ev_stop=e1, **kw)
        torch.cuda.synchronize()
        ms_sum += float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs]))
        flops += 2.0 * n * hw * c * B + 18.0 * n * hw * B * k
        nbytes += 4.0 * (n * hw * (c + B) + c * B) + 4.0 * (n * hw * (B + k) + 9 * B * k) + 8.0 * n * hw * c
        launches += 1
    ms = ms_sum / launches
    t_hbm, t_mfma = nbytes / (HBM_PEAK_GBS * 1e9), flops / (MFMA_F32_PEAK_TF * 1e12)
    common = {"kernel": DOMINANT.get(traffic_key, ("k_wgrad_pair",))[0] +
              " (a layer's 1x1 and 3x3 weight gradients and its BN1 backward reduction in one launch)",
              "traffic": measured_traffic(traffic_key), "avg_launch_ms": round(ms, 5),
              "algorithmic_flops_per_launch": int(flops / launches),
              "algorithmic_bytes_per_launch": int(nbytes / launches), "launches_averaged": launches * reps,
              "shapes": "B = %d, k = %d over P = %d pixels, C_l = %d..%d (the %d layers of the first dense block with "
                        "C_l >= 49)" % (B, k, n * hw, cs[0], cs[-1], launches)}
    del y, G, db, bact
    if t_hbm >= t_mfma:
        achieved = nbytes / (ms_sum * 1e-3) / 1e9
        return dict({"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4)}, **common)
    achieved = flops / (ms_sum * 1e-3) / 1e12
    return dict({"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_F32_PEAK_TF, "unit": "TFLOP/s",
                 "frac": round(achieved / MFMA_F32_PEAK_TF, 4)}, **common)


def cpu_baseline(wl, blocks):
    """The oracle as it stands, on the host cores, same workload shapes (full batch when it
    finishes in tens of seconds, else a bounded number of images: cost per image is
    batch independent for its naive loops)."""
    from harness import run_block_oracle
    from oracle import oracle as orc
    batch = blocks[0].n
    flops_per_img = sum(6 * c.h * c.w * sum(c.c_in(l) * c.bottleneck + 9 * c.bottleneck * c.growth
                                            for l in range(1, c.layers + 1)) for c in blocks)
    sample = max(1, min(batch, int(400e9 // max(flops_per_img, 1))))
    t, passes = 0.0, 0
    inputs = []
    for c in blocks:
        cs = wl.BlockCfg(sample, c.c0, c.h, c.w, c.layers, c.growth, c.bottleneck, c.eps)
        inputs.append((cs,) + tuple(wl.make_block_inputs(cs)))
    while t < 10.0 and passes < 20:  # about 10-30 s of CPU work
        for cs, x0, lp, dy in inputs:
            t0 = time.perf_counter()
            run_block_oracle(orc, cs, x0, lp, dy)
            t += time.perf_counter() - t0
        passes += 1
    sample_total = sample * passes
    return {"value": round(sample_total / t, 3), "unit": "images/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{passes} pass(es) of {sample} of {batch} images through the same {len(blocks)} dense blocks "
                      f"(float64, store-everything schedule, fwd+bwd), {t:.1f} s"}


def cpu_baseline_net(wl, ncfg):
    """The oracle's whole training step on the host cores, on a bounded number of images of the
    same network (its cost per image does not depend on the batch)."""
    from oracle import oracle as orc
    from harness import pack_net
    sample = min(ncfg.n, 16)
    cs = wl.NetCfg(sample, ncfg.image, ncfg.depth, ncfg.growth, ncfg.classes, ncfg.eps)
    x, labels, params = wl.make_net_inputs(cs)
    s = orc.NetShape(cs.n, cs.image, cs.depth, cs.growth, cs.classes, cs.eps)
    flat = pack_net(orc, s, params)
    t, passes = 0.0, 0
    while t < 10.0 and passes < 20:
        t0 = time.perf_counter()
        orc.net_step(s, x, labels, flat)
        t += time.perf_counter() - t0
        passes += 1
    return {"value": round(sample * passes / t, 3), "unit": "images/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{passes} training step(s) of {sample} of {ncfg.n} images through the same network "
                      f"(float64, store-everything schedule, fwd+bwd), {t:.1f} s"}


def extra_fp32_net(dnb, torch, wl, name, steps, warmup):
    """Another CIFAR-shaped fp32 workload timed like the metric's: whole training step under the
    three schedules, exact peak bytes, recompute overhead, roofline of its dominant kernel."""
    sched = {"shared": dnb.DNB_SCHED_SHARED, "store_all": dnb.DNB_SCHED_STORE_ALL, "fused": dnb.DNB_SCHED_FUSED}
    blocks, wname = workload_blocks(wl, name, 0)
    batch = blocks[0].n
    ncfg = wl.net_config3(batch) if name == "config3" else wl.net_config2(batch)
    out = {"workload": wname.replace("3 dense blocks", "whole network: stem, 3 dense blocks").replace(
        "layers (fwd+bwd)", "layers, 2 transitions, head, softmax cross-entropy (fwd+bwd)"), "steps": steps, "warmup": warmup}
    t = {}
    for sname in ("fused", "shared", "store_all"):
        r = NetRun(dnb, torch, wl, ncfg, sched[sname])
        t[sname] = time_steps(torch, make_net_step(dnb, r), steps, warmup, True)
        out[sname] = {"images_per_s": round(batch * steps / t[sname], 2), "ms_per_step": round(1e3 * t[sname] / steps, 4),
                      "network_feature_map_bytes": r.peak}
        hs = [dnb.dnb_block_create(c.n, c.c0, c.h, c.w, c.layers, c.growth, c.bottleneck, schedule=sched[sname]) for c in blocks]
        out[sname]["dense_block_feature_map_bytes"] = sum(dnb.dnb_block_peak_bytes(h) for h in hs)
        for h in hs:
            dnb.dnb_block_destroy(h)
        dnb.dnb_net_destroy(r.h)
        del r
        torch.cuda.empty_cache()
    out["recompute_overhead"] = round(t["shared"] / t["store_all"] - 1.0, 4)
    out["fused_vs_store_all_time"] = round(t["fused"] / t["store_all"] - 1.0, 4)
    runs = [BlockRun(dnb, torch, wl, blocks[0], sched["fused"], 0)]
    out["roofline"] = dominant_kernel_roofline(dnb, torch, runs, f"{name}:{batch}")
    runs[0].close()
    del runs
    torch.cuda.empty_cache()
    return out


def extra_bf16_blocks(dnb, torch, wl, name, steps, warmup, use_graph=True, compare=True):
    """The dense-block set of an ImageNet-shaped bf16 / NHWC workload (batch 32): the fused schedule
    as the library runs it by default (weight gradients on a helper stream) and, for the recompute
    overhead, the three schedules in program order on one stream (the materialised ones only run
    that way), with their exact peak feature-map bytes."""
    sched = {"shared": dnb.DNB_SCHED_SHARED, "store_all": dnb.DNB_SCHED_STORE_ALL, "fused": dnb.DNB_SCHED_FUSED}
    blocks, wname = workload_blocks(wl, name, 0)
    batch = blocks[0].n
    out = {"workload": wname, "steps": steps, "warmup": warmup}
    t = {}
    for label, sname, serial in (("fused", "fused", False), ("fused_one_stream", "fused", True), ("shared", "shared", True),
                                 ("store_all", "store_all", True)):
        if not compare and label != "fused":
            continue
        runs = [BlockRun(dnb, torch, wl, c, sched[sname], 10 * i, True) for i, c in enumerate(blocks)]
        if serial:
            for r in runs:
                dnb.dnb_block_set_concurrency(r.h, False)
        t[label] = time_steps(torch, make_step(dnb, runs), steps, warmup, use_graph)
        out[label] = {"images_per_s": round(batch * steps / t[label], 2), "ms_per_step": round(1e3 * t[label] / steps, 4),
                      "feature_map_bytes": sum(r.mem["peak_bytes"] for r in runs)}
        for r in runs:
            r.close()
        del runs
        torch.cuda.empty_cache()
    if compare:
        out["recompute_overhead"] = round(t["shared"] / t["store_all"] - 1.0, 4)
        out["fused_vs_store_all_time"] = round(t["fused_one_stream"] / t["store_all"] - 1.0, 4)
    return out


def extra_bf16_net(dnb, torch, wl, name, steps, warmup, use_graph=True, compare=True):
    """The whole training step of an ImageNet-shaped bf16 / NHWC workload (batch 32, 224x224 inputs:
    stem, max pool, four dense blocks, transitions, head, loss): the fused schedule as the library
    runs it by default and the three schedules in program order on one stream, with the exact
    feature-map bytes of the whole network."""
    sched = {"shared": dnb.DNB_SCHED_SHARED, "store_all": dnb.DNB_SCHED_STORE_ALL, "fused": dnb.DNB_SCHED_FUSED}
    icfg = wl.inet_config4() if name == "config4" else wl.inet_config5()
    shape = "DenseNet-161-shaped k=48, blocks 6-12-36-24" if name == "config4" else "DenseNet-264-shaped k=32, blocks 6-12-64-48"
    out = {"workload": f"{shape}, batch {icfg.n}, 3x224x224 inputs, bf16 NHWC, whole network: 7x7 stride-2 stem, max pool, 4 dense "
                       "blocks, 3 transitions, head, softmax cross-entropy (fwd+bwd)", "steps": steps, "warmup": warmup}
    t = {}
    for label, sname, serial in (("fused", "fused", False), ("fused_one_stream", "fused", True), ("shared", "shared", True),
                                 ("store_all", "store_all", True)):
        if not compare and label != "fused":
            continue
        r = InetRun(dnb, torch, wl, icfg, sched[sname])
        if serial:
            dnb.dnb_inet_set_concurrency(r.h, False)
        t[label] = time_steps(torch, make_inet_step(dnb, r), steps, warmup, use_graph)
        out[label] = {"images_per_s": round(icfg.n * steps / t[label], 2), "ms_per_step": round(1e3 * t[label] / steps, 4),
                      "network_feature_map_bytes": r.peak, "workspace_bytes": r.workspace}
        r.close()
        del r
        torch.cuda.empty_cache()
    if compare:
        out["recompute_overhead"] = round(t["shared"] / t["store_all"] - 1.0, 4)
        out["fused_vs_store_all_time"] = round(t["fused_one_stream"] / t["store_all"] - 1.0, 4)
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1707_06990_amd as dnb
    import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    blocks, wname = workload_blocks(wl, a.workload, a.batch)
    if a.only_block >= 0:
        blocks = [blocks[a.only_block]]
        wname += f" [only dense block {a.only_block}]"
    if a.forward_only:
        wname += " [FORWARD ONLY]"
    batch = blocks[0].n
    sched = {"shared": dnb.DNB_SCHED_SHARED, "store_all": dnb.DNB_SCHED_STORE_ALL, "fused": dnb.DNB_SCHED_FUSED}
    use_graph = not a.no_graph

    bf16 = a.workload in ("config4", "config5")

    def measure(schedule):
        runs = [BlockRun(dnb, torch, wl, c, sched[schedule], 10 * i, bf16) for i, c in enumerate(blocks)]
        if a.serial or a.concurrent:
            for r in runs:
                dnb.dnb_block_set_concurrency(r.h, a.concurrent)
        secs = time_steps(torch, make_step(dnb, runs, a.forward_only), a.steps, a.warmup, use_graph)
        return runs, secs

    if bf16 and a.only_block < 0 and a.scope in ("auto", "net"):
        # the ImageNet-shaped workloads as whole training steps (diagnostic line of their own)
        res = extra_bf16_net(dnb, torch, wl, a.workload, a.steps, a.warmup, use_graph, not a.no_compare)
        res["dense_blocks_only"] = extra_bf16_blocks(dnb, torch, wl, a.workload, a.steps, a.warmup, use_graph, not a.no_compare)
        print(json.dumps({"metric": "train images/sec per MI355X (fwd+bwd) + peak feature-map bytes vs depth",
                          "value": res["fused"]["images_per_s"], "unit": "images/s", "n_gpus": 1, "steps": a.steps,
                          "warmup": a.warmup, "ms_per_step": res["fused"]["ms_per_step"], "higher_is_better": True,
                          "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": res["workload"], "schedule": "fused",
                                     "launch": "hip_graph" if use_graph else "eager", "global_batch": 32}, "detail": res}), flush=True)
        return
    net_scope = a.scope == "net" or (a.scope == "auto" and a.workload in ("config2", "config3") and a.only_block < 0)
    if net_scope and a.workload not in ("config2", "config3"):
        print("bench.py: --scope net with --only-block is not a combination", file=sys.stderr)
        sys.exit(2)
    ncfg = None
    if net_scope:
        ncfg = wl.net_config2(batch) if a.workload == "config2" else wl.net_config3(batch)
        wname = wname.replace("3 dense blocks", "whole network: stem, 3 dense blocks").replace(
            "layers (fwd+bwd)", "layers, 2 transitions, head, softmax cross-entropy (fwd+bwd)")

    def measure_net(schedule):
        r = NetRun(dnb, torch, wl, ncfg, sched[schedule])
        if a.serial or a.concurrent:
            dnb.dnb_net_set_concurrency(r.h, a.concurrent)
        secs = time_steps(torch, make_net_step(dnb, r, a.forward_only), a.steps, a.warmup, use_graph)
        return r, secs

    runs, secs = measure(a.schedule)   # dense blocks alone (also feeds the roofline measurement)
    block_secs = secs
    netrun = None
    if net_scope:
        netrun, secs = measure_net(a.schedule)
    value = batch * a.steps / secs
    out = {
        "metric": "train images/sec per MI355X (fwd+bwd) + peak feature-map bytes vs depth",
        "value": round(value, 2), "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(1e3 * secs / a.steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": wname, "schedule": a.schedule, "launch": "hip_graph" if use_graph else "eager",
                   "global_batch": batch},
        "peak_feature_map_bytes": {"per_block": [r.mem["peak_bytes"] for r in runs],
                                   "total": sum(r.mem["peak_bytes"] for r in runs),
                                   "workspace_total": sum(r.mem["workspace_bytes"] for r in runs)},
    }
    if net_scope:
        out["dense_blocks_only"] = {"images_per_s": round(batch * a.steps / block_secs, 2),
                                    "ms_per_step": round(1e3 * block_secs / a.steps, 4)}
        out["peak_feature_map_bytes"]["network_total"] = netrun.peak
        out["peak_feature_map_bytes"]["network_workspace"] = netrun.workspace
        dnb.dnb_net_destroy(netrun.h)
        del netrun
        torch.cuda.empty_cache()
    # the roofline entry is that of the fp32 path's dominant kernel; the bf16 block sets are diagnostic
    out["roofline"] = None if bf16 else dominant_kernel_roofline(dnb, torch, runs, f"{a.workload}:{batch}" if a.only_block < 0 else "")
    del runs
    torch.cuda.empty_cache()
    if not a.no_compare and not bf16:
        # the other schedules on the same workload: the paper-literal shared-storage schedule and
        # the store-everything schedule it is compared with (Section 5)
        t = {a.schedule: secs}
        for other in ("shared", "store_all", "fused"):
            if other in t:
                continue
            if net_scope:
                onet, osecs = measure_net(other)
                out["peak_feature_map_bytes"][other + "_network_total"] = onet.peak
                dnb.dnb_net_destroy(onet.h)
                del onet
                # the blocks' own exact accounting under this schedule
                hs = [dnb.dnb_block_create(c.n, c.c0, c.h, c.w, c.layers, c.growth, c.bottleneck, schedule=sched[other])
                      for c in blocks]
                out["peak_feature_map_bytes"][other + "_total"] = sum(dnb.dnb_block_peak_bytes(h) for h in hs)
                for h in hs:
                    dnb.dnb_block_destroy(h)
            else:
                oruns, osecs = measure(other)
                out["peak_feature_map_bytes"][other + "_total"] = sum(r.mem["peak_bytes"] for r in oruns)
                del oruns
            t[other] = osecs
            out[other + "_images_per_s"] = round(batch * a.steps / osecs, 2)
            torch.cuda.empty_cache()
        out["recompute_overhead"] = round(t["shared"] / t["store_all"] - 1.0, 4)
        out["fused_vs_store_all_time"] = round(t["fused"] / t["store_all"] - 1.0, 4)
    default_run = (a.workload == "config2" and net_scope and not a.batch and a.schedule == "fused" and use_graph
                   and not (a.serial or a.concurrent or a.forward_only or a.no_compare))
    if default_run and not a.no_extra:
        # the other workloads, so that one run of the default command measures them all: the largest
        # fp32 network as a whole training step, the two bf16 workloads as their dense-block sets
        out["config3"] = extra_fp32_net(dnb, torch, wl, "config3", 10, 3)
        out["config4"] = extra_bf16_net(dnb, torch, wl, "config4", 10, 3)
        out["config4"]["dense_blocks_only"] = extra_bf16_blocks(dnb, torch, wl, "config4", 10, 3)
        out["config5"] = extra_bf16_net(dnb, torch, wl, "config5", 10, 3)
        out["config5"]["dense_blocks_only"] = extra_bf16_blocks(dnb, torch, wl, "config5", 10, 3)
    if not a.no_cpu_baseline and not bf16:
        out["cpu_baseline"] = cpu_baseline_net(wl, ncfg) if net_scope else cpu_baseline(wl, blocks)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
