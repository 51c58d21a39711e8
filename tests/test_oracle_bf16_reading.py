"""Evidence, on the CPU, for the reading that bf16 gradient parity cannot be judged against the
plain float64 block at the 2e-2 bar.

A feature map stored in bf16 carries a relative rounding error of up to 2^-9.  Where the
pre-activation of the BN that consumes it lies within that error of zero, the ReLU mask decided on
the stored value differs from the unrounded one, and the gradient element behind a differing mask
changes by its whole size.  With a fraction f of masks differing and gradients that are
independent of the masks (N(0,1) loss weights), the relative L2 change of the gradient is
sqrt(f / share of elements passed): above two per cent already for f of three in ten thousand --
whatever arithmetic computes the block.
The tests measure f and that change with the oracle's own BN / ReLU routines, and then the
distance between the oracle's storage-rounding block and its plain block.  The GPU tests therefore
let both sides take the ReLU decisions in the kernel's precision (the float64 block is evaluated
with the decisions the kernels took, and the decisions that differ from its own must be ties within
rounding); with that, the bf16 path meets 2e-2 against the plain float64 block."""
import numpy as np
import torch

import workloads as wl
from harness import NAMES, rel_errors, run_block_oracle


def to_bf16_values(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def test_masks_decided_on_bf16_stored_features_move_the_gradient_by_the_root_of_their_share(oracle):
    r = np.random.default_rng(3)
    shape = (2, 96, 28, 28)
    b = r.standard_normal(shape) * r.uniform(0.5, 2.0, (1, shape[1], 1, 1)) + r.uniform(-1, 1, (1, shape[1], 1, 1))
    gamma, beta = 1 + 0.3 * r.standard_normal(shape[1]), 0.3 * r.standard_normal(shape[1])
    dact = r.standard_normal(shape)
    z, _, _ = oracle.bn_forward(b, gamma, beta, 1e-5)
    zq, _, _ = oracle.bn_forward(to_bf16_values(b), gamma, beta, 1e-5)   # the same features as stored in bf16
    flipped = (z > 0) != (zq > 0)
    f = float(flipped.mean())
    assert 1 / 10000 < f < 1 / 1000, f        # one rounding point: a few masks in ten thousand differ
    dz = oracle.relu_backward(oracle.relu(z), dact)
    dzq = oracle.relu_backward(oracle.relu(zq), dact)
    l2, mx = rel_errors(dzq, dz)
    # dz is non-zero on the share of elements with decision 1; a differing decision adds or removes one whole element
    expect = np.sqrt(f / float((z > 0).mean()))
    assert abs(l2 - expect) <= 0.2 * expect, (l2, expect)
    assert l2 > 2e-2      # beyond the 2e-2 bar from ONE rounding point; a layer has about ten
    assert mx > 0.5       # a changed element changes by its whole size
    # the forward values themselves stay well inside the bar
    assert rel_errors(oracle.relu(zq), oracle.relu(z))[0] < 5e-3


def test_storage_rounding_block_lies_several_per_cent_from_the_plain_block_in_its_gradients(oracle):
    """The block output of the storage-rounding variant stays within 2e-2 of the plain float64
    block; its gradients do not: 3-7 % in dx0, up to 12 % in single parameter tensors, on blocks
    of only two or three layers (DenseNet-161 widths included), more with depth."""
    for cfg, lo, hi in ((wl.BlockCfg(2, 32, 14, 14, 3, 16, 64), 0.03, 0.09), (wl.BlockCfg(2, 96, 28, 28, 2, 48, 192), 0.03, 0.07)):
        x0, lp, dy = wl.make_block_inputs(cfg, affine="random")
        x0, dy = to_bf16_values(x0), to_bf16_values(dy)
        plain, osl = run_block_oracle(oracle, cfg, x0, lp, dy)
        emul, _ = run_block_oracle(oracle, cfg, x0, lp, dy, schedule="naive_bf16")
        ly, my = rel_errors(emul.y, plain.y)
        assert ly < 2e-2 and my < 2e-2
        l2, mx = rel_errors(emul.dx0, plain.dx0)
        assert lo < l2 < hi and mx > 0.1, (l2, mx)
        worst = max(rel_errors(emul.dparams[osl[(l, nm)]], plain.dparams[osl[(l, nm)]])[0]
                    for l in range(1, cfg.layers + 1) for nm in NAMES)
        assert 0.05 < worst < 0.15, worst
