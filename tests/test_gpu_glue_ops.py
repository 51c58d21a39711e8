"""GPU parity of the network glue's kernels as single operations, through the C ABI, against the
float64 oracle's primitives on the same seeded inputs: the classifier head (linear layer, mean softmax
cross-entropy and their gradients; fp32, 1e-4) at the benchmark networks' shapes, and the stem of the
ImageNet-shaped step (7x7 stride-2 conv and its weight gradient, BN+ReLU fused into the 3x3 stride-2
max pool with its positions, the pooling's adjoint; bf16 tensors with fp32 accumulation: 1e-2 for
what is stored in bf16, 1e-4 for the fp32 weight gradient)."""
import numpy as np
import pytest
import torch

from gpu_util import assert_close, dev

pytestmark = pytest.mark.gpu


def bf16_values(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def nhwc_bf16(a):   # (n, c, h, w) float -> device (n, h, w, c) bf16
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).permute(0, 2, 3, 1).contiguous().to("cuda", torch.bfloat16)


def back(t):        # device (n, h, w, c) -> numpy (n, c, h, w) float32
    return t.float().permute(0, 3, 1, 2).contiguous().cpu().numpy()


@pytest.mark.parametrize("n,c,classes", [(64, 342, 10), (64, 1734, 100), (32, 2208, 1000), (5, 70, 3), (3, 64, 17)],
                         ids=["bc100", "bc250", "dn161", "ragged", "classes17"])
def test_classifier_head(dnb, oracle, n, c, classes):
    """Logits, loss, the loss's gradient and the head's backward pass at the head shapes of the four
    benchmark networks (the last: 2208 features, 1000 classes, batch 32) and two ragged ones; one
    label is out of range and must add nothing."""
    rng = np.random.default_rng(1000 + n + c + classes)
    pooled = np.abs(rng.standard_normal((n, c))).astype(np.float32)
    wl = (rng.standard_normal((classes, c)) / np.sqrt(c)).astype(np.float32)
    bl = rng.uniform(-0.3, 0.3, classes).astype(np.float32)
    labels = rng.integers(0, classes, n).astype(np.int32)
    ologits = oracle.linear(pooled, wl, bl)
    oloss, odl = oracle.softmax_xent(ologits, labels)
    odf, odwl, odbl = oracle.linear_backward(pooled, wl, odl)
    p, w, b, lab = dev(pooled), dev(wl), dev(bl), torch.from_numpy(labels).to("cuda")
    logits = torch.full((n, classes), float("nan"), device="cuda")
    dlogits = torch.full((n, classes), float("nan"), device="cuda")
    terms = torch.empty(n, device="cuda")
    loss = torch.full((1,), float("nan"), device="cuda")
    dnb.dnb_op_head_forward(p, w, b, lab, logits, dlogits, terms, loss, n, c, classes)
    dpooled = torch.full((n, c), float("nan"), device="cuda")
    dwl = torch.full((classes, c), float("nan"), device="cuda")
    dbl = torch.full((classes,), float("nan"), device="cuda")
    dnb.dnb_op_head_backward(dlogits, p, w, dpooled, dwl, dbl, n, c, classes)
    torch.cuda.synchronize()
    assert_close(logits.cpu().numpy(), ologits, 1e-4, "logits")
    assert abs(float(loss.item()) - oloss) <= 1e-4 * abs(oloss)
    assert_close(dlogits.cpu().numpy(), odl, 1e-4, "dlogits")
    assert_close(dpooled.cpu().numpy(), odf, 1e-4, "dpooled")
    assert_close(dwl.cpu().numpy(), odwl, 1e-4, "dWl")
    assert_close(dbl.cpu().numpy(), odbl, 1e-4, "dbl")
    # a label outside [0, classes): that sample adds nothing to the loss or to any gradient
    bad = labels.copy(); bad[0] = classes
    dnb.dnb_op_head_forward(p, w, b, torch.from_numpy(bad).to("cuda"), logits, dlogits, terms, loss, n, c, classes)
    torch.cuda.synchronize()
    assert np.all(dlogits[0].cpu().numpy() == 0.0)
    t = np.array([np.log(np.exp(ologits[i] - ologits[i].max()).sum()) + ologits[i].max() - ologits[i, labels[i]] for i in range(1, n)])
    assert abs(float(loss.item()) - t.sum() / n) <= 1e-4 * abs(t.sum() / n) + 1e-7


@pytest.mark.parametrize("n,image,channels", [(2, 64, 16), (3, 96, 32), (2, 64, 64), (2, 224, 96), (1, 32, 96)],
                         ids=["c16", "c32", "c64", "c96_full_image", "one_tile_row"])
def test_stem_conv_and_weight_gradient(dnb, oracle, n, image, channels):
    """7x7 stride-2 pad-3 conv of a 3-channel image (every built channel count; 224x224 at the width
    of the DenseNet-161-shaped network) and its weight gradient against the oracle's strided conv."""
    rng = np.random.default_rng(2000 + image + channels)
    x = bf16_values(rng.standard_normal((n, 3, image, image)))
    w = (rng.standard_normal((channels, 3, 7, 7)) * np.sqrt(2.0 / 147)).astype(np.float32)
    wq = bf16_values(w)   # the conv reads its weights rounded to bf16
    oout = oracle.conv_forward_strided(x, wq, 2, 3)
    scratch = torch.empty(dnb.dnb_op_stem_scratch_bytes(n, image, channels), dtype=torch.uint8, device="cuda")
    xd = nhwc_bf16(x)
    out = torch.full((n, image // 2, image // 2, channels), float("nan"), dtype=torch.bfloat16, device="cuda")
    dnb.dnb_op_stem_conv7(xd, dev(w), out, n, image, channels, scratch)
    torch.cuda.synchronize()
    assert_close(back(out), oout, 1e-2, "stem conv")   # bf16 output: 2^-9 per element
    g = bf16_values(rng.standard_normal((n, channels, image // 2, image // 2)))
    odw = oracle.conv_wgrad_strided(x, g, 7, 2, 3)
    dw = torch.full((channels, 3, 7, 7), float("nan"), device="cuda")
    dnb.dnb_op_stem_wgrad7(xd, nhwc_bf16(g), dw, n, image, channels, scratch)
    torch.cuda.synchronize()
    assert_close(dw.cpu().numpy(), odw, 1e-4, "stem dW")   # exact bf16 products, fp32 sums


@pytest.mark.parametrize("n,h,w,c", [(2, 32, 32, 16), (3, 16, 48, 64), (2, 112, 112, 96), (1, 2, 2, 8)],
                         ids=["small", "wide", "dn161_stem", "one_window"])
def test_max_pool_with_bn_relu_and_its_adjoint(dnb, oracle, n, h, w, c):
    """BN+ReLU (given scale and shift per channel) fused into the 3x3 stride-2 pad-1 max pool: values
    and positions against the oracle's pooling of the float64 BN+ReLU output.  About half of the
    inputs are cut to zero by the ReLU, so windows with several equal maxima (all zero) are frequent
    and the first-in-scan-order rule is exercised; a position may differ from the oracle's only where
    the window's two largest values are closer than fp32 rounding.  Then the adjoint with the kernel's
    own positions against the oracle's with the same positions."""
    rng = np.random.default_rng(3000 + h + w + c)
    s = bf16_values(rng.standard_normal((n, c, h, w)))
    scale = rng.uniform(0.5, 1.5, c).astype(np.float32) * np.where(rng.random(c) < 0.2, -1.0, 1.0).astype(np.float32)
    shift = rng.uniform(-0.5, 0.5, c).astype(np.float32)
    a = np.maximum(s.astype(np.float64) * scale.astype(np.float64)[None, :, None, None] + shift.astype(np.float64)[None, :, None, None], 0.0)
    oout, opos = oracle.maxpool3s2(a)
    fold = dev(np.stack([scale, shift], axis=1).astype(np.float32))
    out = torch.full((n, h // 2, w // 2, c), float("nan"), dtype=torch.bfloat16, device="cuda")
    pos = torch.full((n, h // 2, w // 2, c), 99, dtype=torch.uint8, device="cuda")
    dnb.dnb_op_maxpool3s2_bnrelu(nhwc_bf16(s), fold, out, pos, n, h, w, c)
    torch.cuda.synchronize()
    assert_close(back(out), oout, 1e-2, "pooled")
    kpos = pos.permute(0, 3, 1, 2).contiguous().cpu().numpy()
    assert kpos.max() <= 8
    diff = kpos != opos
    # imposing the kernel's positions on the oracle: where they differ, the value there must equal the maximum to fp32 rounding
    _, (count, margin) = oracle.maxpool3s2(a, positions=kpos)
    assert count == int(diff.sum())
    assert count <= 1e-4 * kpos.size + 2 and margin <= 1e-5, (count, margin)
    g = bf16_values(rng.standard_normal((n, c, h // 2, w // 2)))
    odin = oracle.maxpool3s2_backward(g, kpos, h, w)
    din = torch.full((n, h, w, c), float("nan"), dtype=torch.bfloat16, device="cuda")
    dnb.dnb_op_maxpool3s2_backward(nhwc_bf16(g), pos, din, n, h, w, c)
    torch.cuda.synchronize()
    assert_close(back(din), odin, 1e-2, "pool adjoint")


def test_glue_ops_reject_what_is_not_built(dnb):
    z = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(dnb.DnbError):
        dnb.dnb_op_stem_conv7(z, z, z, 1, 64, 48, z)          # 48 channels: not a built width
    with pytest.raises(dnb.DnbError):
        dnb.dnb_op_stem_conv7(z, z, z, 1, 50, 32, z)          # image not a multiple of 32
    with pytest.raises(dnb.DnbError):
        dnb.dnb_op_maxpool3s2_bnrelu(z, z, z, z, 1, 7, 8, 8)  # odd height
    assert dnb.dnb_op_stem_scratch_bytes(1, 64, 48) == 0
