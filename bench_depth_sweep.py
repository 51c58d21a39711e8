#!/usr/bin/env python3
"""Memory and time against depth: the study of the paper's Section 5 (the memory-vs-depth and
time-vs-depth figures) on one MI355X.

DenseNet-BC, growth k = 12, batch 64, 32x32 inputs; for every depth L the three dense blocks of
(L-4)/6 bottleneck layers are run forward + backward under each schedule:
  store_all  every concatenation / BN output kept (Section 3, quadratic feature-map memory)
  shared     shared storage 1/2/3 + recomputation (Section 4, linear)
  fused      BN+ReLU recomputed inside the conv operand loads (nothing of storage 1/2/3 exists)
Reported per depth and schedule: exact feature-map bytes (the library's accounting, equal to the
closed-form formula), workspace bytes actually allocated, ms per step and images/s; then the
recomputation overhead shared/store_all - 1 and the deepest L whose feature maps fit 288 GB.
Synthetic inputs (N(0,1) features and loss weights, He-normal weights), as in bench.py.

    python bench_depth_sweep.py [--depths 40 100 160 250 340 502] [--batch 64] [--steps 5]
prints one JSON line per depth and a final summary line.
"""
import argparse
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)

HBM_BYTES = 288e9


def feature_map_bytes(blocks, schedule, esz=4):
    """Closed form (units: bytes) of the library's peak feature-map accounting, per schedule."""
    total = 0
    for c in blocks:
        m, k, B, P = c.layers, c.growth, c.bottleneck, c.pixels
        cm, cout = c.c_in(m), c.c_out
        sigma = sum(c.c_in(l) for l in range(1, m + 1))
        grad = cout + cm + B
        if schedule == "store_all":
            fwd = 2 * sigma + m * (2 * B + k)
        elif schedule == "shared":
            fwd = m * B + m * k + 2 * cm + B
        else:
            fwd = m * B + m * k
        total += (fwd + grad) * P * esz
    return total


def deepest_that_fits(wl, schedule, growth, batch, limit=HBM_BYTES):
    """Largest depth L = 6n + 4 whose feature maps fit `limit` bytes (bytes grow with n: bisection)."""
    fits = lambda n: feature_map_bytes(wl.densenet_bc_blocks(6 * n + 4, growth, batch), schedule) <= limit
    lo, hi = 1, 2
    while fits(hi):
        lo, hi = hi, hi * 2
    while hi - lo > 1:
        mid = (lo + hi) // 2
        lo, hi = (mid, hi) if fits(mid) else (lo, mid)
    return 6 * lo + 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--depths", type=int, nargs="+", default=[40, 100, 160, 250, 340, 502])
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--growth", type=int, default=12)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    a = ap.parse_args()
    import torch
    import paper_1707_06990_amd as dnb
    import workloads as wl
    import bench
    assert torch.cuda.is_available(), "bench_depth_sweep.py needs a GPU"
    torch.cuda.set_device(0)
    sched = {"shared": dnb.DNB_SCHED_SHARED, "store_all": dnb.DNB_SCHED_STORE_ALL, "fused": dnb.DNB_SCHED_FUSED}
    rows = []
    for L in a.depths:
        assert (L - 4) % 6 == 0, "DenseNet-BC depths are 6n + 4"
        blocks = wl.densenet_bc_blocks(L, a.growth, a.batch)
        row = {"depth": L, "layers_per_block": blocks[0].layers, "batch": a.batch, "growth": a.growth}
        for name in ("store_all", "shared", "fused"):
            runs = [bench.BlockRun(dnb, torch, wl, c, sched[name], 10 * i) for i, c in enumerate(blocks)]
            fm = sum(r.mem["peak_bytes"] for r in runs)
            assert fm == feature_map_bytes(blocks, name), (L, name)
            secs = bench.time_steps(torch, bench.make_step(dnb, runs), a.steps, a.warmup, True)
            row[name] = {"feature_map_bytes": fm, "workspace_bytes": sum(r.mem["workspace_bytes"] for r in runs),
                         "ms_per_step": round(1e3 * secs / a.steps, 3),
                         "images_per_s": round(a.batch * a.steps / secs, 1)}
            for r in runs:
                dnb.dnb_block_destroy(r.h)
            del runs
            torch.cuda.empty_cache()
        row["recompute_overhead"] = round(row["shared"]["ms_per_step"] / row["store_all"]["ms_per_step"] - 1, 4)
        row["fused_vs_store_all_time"] = round(row["fused"]["ms_per_step"] / row["store_all"]["ms_per_step"] - 1, 4)
        row["memory_ratio_shared"] = round(row["shared"]["feature_map_bytes"] / row["store_all"]["feature_map_bytes"], 4)
        rows.append(row)
        print(json.dumps(row), flush=True)
    print(json.dumps({"deepest_L_fitting_288GB_feature_maps": {
        s: deepest_that_fits(wl, s, a.growth, a.batch) for s in ("store_all", "shared", "fused")},
        "batch": a.batch, "growth": a.growth}), flush=True)


if __name__ == "__main__":
    main()
