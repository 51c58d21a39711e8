"""GPU parity of the single operations (through the C ABI) against the CPU oracle,
element by element, on seeded inputs whose shapes span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from gpu_util import assert_close, dev

pytestmark = pytest.mark.gpu
TOL = 1e-4  # fp32 path vs float64 oracle, relative (L2 and max-abs/max)


def rng(seed):
    return np.random.default_rng(seed)


def f32(a):
    return np.asarray(a, dtype=np.float32)


@pytest.mark.parametrize("n,len_,sstride,dstride", [(3, 40, 40, 72), (2, 37, 50, 37), (5, 4096, 8192, 4096), (1, 1, 1, 1)])
def test_copy_slab(dnb, n, len_, sstride, dstride):
    src = f32(rng(1).standard_normal((n, sstride)))
    d_src = dev(src)
    d_dst = torch.full((n, dstride), -7.0, device="cuda")
    dnb.dnb_op_copy_slab(d_src, sstride, d_dst, dstride, n, len_)
    torch.cuda.synchronize()
    out = d_dst.cpu().numpy()
    np.testing.assert_array_equal(out[:, :len_], src[:, :len_])
    assert np.all(out[:, len_:] == -7.0)


BN_SHAPES = [(2, 16, 8, 8), (3, 5, 7, 9), (64, 12, 4, 4), (2, 70, 16, 16), (1, 3, 1, 1), (5, 9, 3, 2)]


def bn_stats_gpu(dnb, x, eps):
    n, c, h, w = x.shape
    d_x = dev(x)
    mean = torch.empty(c, device="cuda")
    istd = torch.empty(c, device="cuda")
    scratch = torch.empty(dnb.dnb_op_bn_scratch_bytes(n, c, h * w), dtype=torch.uint8, device="cuda")
    dnb.dnb_op_bn_stats(d_x, c * h * w, n, c, h * w, eps, mean, istd, scratch)
    torch.cuda.synchronize()
    return d_x, mean, istd, scratch


@pytest.mark.parametrize("shape", BN_SHAPES)
def test_bn_stats_and_apply(dnb, oracle, shape):
    r = rng(2)
    n, c, h, w = shape
    x = f32(r.standard_normal(shape) * r.uniform(0.2, 4, (1, c, 1, 1)) + r.uniform(-2, 2, (1, c, 1, 1)))
    gamma, beta = f32(1 + 0.3 * r.standard_normal(c)), f32(0.3 * r.standard_normal(c))
    eps = 1e-5
    d_x, mean, istd, _ = bn_stats_gpu(dnb, x, eps)
    z, omean, ovar = oracle.bn_forward(x, gamma, beta, eps)
    assert_close(mean.cpu().numpy(), omean, TOL, "mean")
    assert_close(istd.cpu().numpy(), 1 / np.sqrt(ovar + eps), TOL, "istd")
    out = torch.full(shape, float("nan"), device="cuda")
    dnb.dnb_op_bn_relu(d_x, c * h * w, out, c * h * w, n, c, h * w, dev(gamma), dev(beta), mean, istd)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), oracle.relu(z), TOL, "bn+relu")


def test_bn_stats_large_offset_channel(dnb, oracle):
    """|mean| >> std: a one-pass E[x^2]-E[x]^2 in fp32 would lose the variance."""
    r = rng(3)
    x = f32(1000.0 + 0.5 * r.standard_normal((8, 4, 16, 16)))
    _, mean, istd, _ = bn_stats_gpu(dnb, x, 1e-5)
    _, omean, ovar = oracle.bn_forward(x, np.ones(4), np.zeros(4), 1e-5)
    assert_close(istd.cpu().numpy(), 1 / np.sqrt(ovar + 1e-5), 1e-3, "istd")


@pytest.mark.parametrize("shape", BN_SHAPES)
@pytest.mark.parametrize("accumulate", [0, 1])
def test_bn_relu_backward(dnb, oracle, shape, accumulate):
    r = rng(4)
    n, c, h, w = shape
    x = f32(r.standard_normal(shape) * 1.5 + 0.3)
    gamma, beta = f32(1 + 0.3 * r.standard_normal(c)), f32(0.3 * r.standard_normal(c))
    dact = f32(r.standard_normal(shape))
    base = f32(r.standard_normal(shape))
    eps = 1e-5
    d_x, mean, istd, scratch = bn_stats_gpu(dnb, x, eps)
    du = dev(base.copy())
    dg = torch.empty(c, device="cuda")
    db = torch.empty(c, device="cuda")
    hw = h * w
    dnb.dnb_op_bn_relu_backward(d_x, c * hw, dev(dact), c * hw, du, c * hw, accumulate, n, c, hw, dev(gamma),
                                dev(beta), mean, istd, dg, db, scratch)
    torch.cuda.synchronize()
    z, omean, ovar = oracle.bn_forward(x, gamma, beta, eps)
    dz = oracle.relu_backward(oracle.relu(z), dact)
    odu, odg, odb = oracle.bn_backward(x, dz, gamma, omean, ovar, eps)
    if accumulate:
        odu = odu + base
    if n * hw > 1:
        assert_close(du.cpu().numpy(), odu, TOL, "du")
        assert_close(dg.cpu().numpy(), odg, TOL, "dgamma")
    assert_close(db.cpu().numpy(), odb, TOL, "dbeta")


def test_bn_relu_backward_in_place(dnb, oracle):
    """du may alias dact (the block overwrites the gradient of storage 3 with that of b_l)."""
    r = rng(5)
    shape = (4, 48, 8, 8)
    n, c, h, w = shape
    x, dact = f32(r.standard_normal(shape)), f32(r.standard_normal(shape))
    gamma, beta = f32(1 + 0.3 * r.standard_normal(c)), f32(0.3 * r.standard_normal(c))
    d_x, mean, istd, scratch = bn_stats_gpu(dnb, x, 1e-5)
    buf = dev(dact.copy())
    dg, db = torch.empty(c, device="cuda"), torch.empty(c, device="cuda")
    dnb.dnb_op_bn_relu_backward(d_x, c * 64, buf, c * 64, buf, c * 64, 0, n, c, 64, dev(gamma), dev(beta), mean,
                                istd, dg, db, scratch)
    torch.cuda.synchronize()
    z, omean, ovar = oracle.bn_forward(x, gamma, beta, 1e-5)
    odu, _, _ = oracle.bn_backward(x, oracle.relu_backward(oracle.relu(z), dact), gamma, omean, ovar, 1e-5)
    assert_close(buf.cpu().numpy(), odu, TOL, "du in place")


CONV_SHAPES = [
    # n, cin, cout, h, w, ks
    (2, 16, 48, 8, 8, 1), (2, 48, 12, 8, 8, 3),      # the small block's two convs
    (3, 20, 12, 9, 7, 3), (1, 5, 3, 1, 1, 3), (2, 7, 5, 2, 3, 3), (1, 17, 33, 5, 5, 1),
    (2, 52, 48, 32, 32, 1), (2, 48, 12, 32, 32, 3), (2, 96, 24, 16, 16, 3),
    (1, 70, 100, 6, 6, 1), (2, 9, 200, 5, 4, 1), (1, 12, 48, 11, 13, 3), (4, 30, 64, 7, 7, 3),
    # aligned shapes (16-byte fast kernels): wide K, many M tiles, tiny and ragged images, channel tails
    (2, 330, 48, 8, 8, 1), (1, 200, 48, 16, 16, 1), (3, 36, 48, 4, 4, 1), (2, 16, 8, 4, 4, 3),
    (1, 32, 16, 8, 56, 3), (2, 28, 20, 12, 12, 3), (2, 100, 36, 8, 8, 3), (5, 60, 64, 8, 8, 3), (1, 24, 48, 20, 20, 1),
    (1, 16, 16, 4, 64, 3),   # rows too wide for the 3x3 weight gradient's one-batch first chunk
]


@pytest.mark.parametrize("n,cin,cout,h,w,ks", CONV_SHAPES)
def test_conv_forward_dgrad_wgrad(dnb, oracle, n, cin, cout, h, w, ks):
    r = rng(6)
    x = f32(r.standard_normal((n, cin, h, w)))
    wgt = f32(r.standard_normal((cout, cin, ks, ks)) * np.sqrt(2.0 / (cin * ks * ks)))
    g = f32(r.standard_normal((n, cout, h, w)))
    hw = h * w
    d_x, d_w, d_g = dev(x), dev(wgt), dev(g)
    out = torch.full((n, cout, h, w), float("nan"), device="cuda")
    pk = torch.full((dnb.dnb_op_conv_scratch_bytes(cin, cout, ks) // 4,), float("nan"), device="cuda")
    dnb.dnb_op_conv_forward(d_x, cin * hw, d_w, out, cout * hw, n, cin, cout, h, w, ks, pk)
    din = torch.full((n, cin, h, w), float("nan"), device="cuda")
    pk2 = torch.full_like(pk, float("nan"))
    dnb.dnb_op_conv_dgrad(d_g, cout * hw, d_w, din, cin * hw, n, cin, cout, h, w, ks, pk2)
    dw = torch.full(wgt.shape, float("nan"), device="cuda")
    scratch = torch.empty(max(16, dnb.dnb_op_conv_wgrad_scratch_bytes(n, cin, cout, h, w, ks)), dtype=torch.uint8, device="cuda")
    dnb.dnb_op_conv_wgrad(d_x, cin * hw, d_g, cout * hw, dw, n, cin, cout, h, w, ks, scratch)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), oracle.conv_forward(x, wgt), TOL, "forward")
    assert_close(din.cpu().numpy(), oracle.conv_dgrad(g, wgt), TOL, "dgrad")
    assert_close(dw.cpu().numpy(), oracle.conv_wgrad(x, g, ks), TOL, "wgrad")


def test_conv_on_channel_slices_of_wider_slabs(dnb, oracle):
    """Input and output addressed in place inside wider tensors (explicit image strides),
    as the block does with the output slab y and the gradient slab."""
    r = rng(7)
    n, cin, cout, h, w = 3, 24, 12, 8, 8
    hw = h * w
    wide_in = f32(r.standard_normal((n, cin + 10, h, w)))
    wgt = f32(r.standard_normal((cout, cin, 3, 3)) * 0.1)
    d_in = dev(wide_in)
    wide_out = torch.full((n, 40, h, w), -3.0, device="cuda")
    x_view = d_in.data_ptr() + 4 * 4 * hw          # channels 4..4+cin
    o_view = wide_out.data_ptr() + 4 * 20 * hw     # channels 20..32
    pk = torch.empty(dnb.dnb_op_conv_scratch_bytes(cin, cout, 3), dtype=torch.uint8, device="cuda")
    dnb.dnb_op_conv_forward(x_view, (cin + 10) * hw, dev(wgt), o_view, 40 * hw, n, cin, cout, h, w, 3, pk)
    torch.cuda.synchronize()
    res = wide_out.cpu().numpy()
    assert_close(res[:, 20:32], oracle.conv_forward(wide_in[:, 4:4 + cin], wgt), TOL, "slice conv")
    assert np.all(res[:, :20] == -3.0) and np.all(res[:, 32:] == -3.0)


@pytest.mark.parametrize("n,cin,cout,h,w,ks", [(2, 48, 12, 32, 32, 3), (3, 40, 48, 16, 16, 1), (2, 204, 48, 8, 8, 1),
                                               (2, 24, 12, 8, 12, 3)])
def test_fused_conv_bnrelu_forward_and_statistics(dnb, oracle, n, cin, cout, h, w, ks):
    """BN+ReLU applied in the operand load, statistics of the output from the epilogue: against
    relu(x*scale+shift) -> conv of the oracle, and the merged tile statistics against the output's
    mean and biased variance."""
    r = rng(21)
    x = f32(r.standard_normal((n, cin, h, w)))
    wgt = f32(r.standard_normal((cout, cin, ks, ks)) * np.sqrt(2.0 / (cin * ks * ks)))
    fold = f32(np.stack([1.0 + 0.3 * r.standard_normal(cin), 0.3 * r.standard_normal(cin)], axis=1))
    hw = h * w
    out = torch.full((n, cout, h, w), float("nan"), device="cuda")
    pk = torch.empty(dnb.dnb_op_conv_scratch_bytes(cin, cout, ks), dtype=torch.uint8, device="cuda")
    stats = torch.full((dnb.dnb_op_conv_stats_bytes(n, cout, h, w) // 4,), float("nan"), device="cuda")
    T = dnb.dnb_op_conv_bnrelu_forward(dev(x), cin * hw, dev(wgt), dev(fold), out, cout * hw, stats, n, cin, cout, h, w, ks, pk)
    torch.cuda.synchronize()
    a = np.maximum(x.astype(np.float64) * fold[:, 0].astype(np.float64)[None, :, None, None]
                   + fold[:, 1].astype(np.float64)[None, :, None, None], 0.0)
    ref = oracle.conv_forward(a, wgt)
    assert_close(out.cpu().numpy(), ref, TOL, "fused conv")
    st = stats.cpu().numpy()[:cout * T * 3].reshape(cout, T, 3).astype(np.float64)
    assert np.all(st[:, :, 0].sum(axis=1) == n * hw)
    mean = (st[:, :, 0] * st[:, :, 1]).sum(axis=1) / (n * hw)
    m2 = (st[:, :, 2] + st[:, :, 0] * (st[:, :, 1] - mean[:, None]) ** 2).sum(axis=1)
    assert_close(mean, ref.mean(axis=(0, 2, 3)), 1e-4 * max(1.0, float(np.abs(ref).max() / np.abs(ref.mean(axis=(0, 2, 3))).max())), "mean")
    assert_close(m2 / (n * hw), ref.var(axis=(0, 2, 3)), TOL, "variance")


@pytest.mark.parametrize("n,cin,cout,h,w,ks", [(2, 48, 12, 32, 32, 3), (3, 40, 48, 16, 16, 1), (2, 204, 48, 8, 8, 1),
                                               (2, 24, 12, 8, 12, 3), (1, 16, 12, 4, 64, 3)])
def test_fused_conv_bnrelu_wgrad(dnb, oracle, n, cin, cout, h, w, ks):
    """Weight gradient with BN+ReLU of the activation recomputed in the operand load."""
    r = rng(22)
    x = f32(r.standard_normal((n, cin, h, w)))
    g = f32(r.standard_normal((n, cout, h, w)))
    fold = f32(np.stack([1.0 + 0.3 * r.standard_normal(cin), 0.3 * r.standard_normal(cin)], axis=1))
    hw = h * w
    dw = torch.full((cout, cin, ks, ks), float("nan"), device="cuda")
    scratch = torch.empty(max(16, dnb.dnb_op_conv_wgrad_scratch_bytes(n, cin, cout, h, w, ks)), dtype=torch.uint8, device="cuda")
    dnb.dnb_op_conv_bnrelu_wgrad(dev(x), cin * hw, dev(fold), dev(g), cout * hw, dw, n, cin, cout, h, w, ks, scratch)
    torch.cuda.synchronize()
    a = np.maximum(x.astype(np.float64) * fold[:, 0].astype(np.float64)[None, :, None, None]
                   + fold[:, 1].astype(np.float64)[None, :, None, None], 0.0)
    assert_close(dw.cpu().numpy(), oracle.conv_wgrad(a, g, ks), TOL, "fused wgrad")


def away_from_zero(x, scale, shift, margin=1e-3):
    """x (n, c, h, w) with every element whose pre-activation x*scale_c + shift_c lies within
    `margin` of zero moved so that it lies 2*margin away: the ReLU decisions of such inputs are the
    same in any precision, so an element-wise comparison needs no allowance for ties."""
    x = x.astype(np.float64)
    sc, sh = scale.astype(np.float64)[None, :, None, None], shift.astype(np.float64)[None, :, None, None]
    z = x * sc + sh
    near = np.abs(z) < margin
    target = np.where(z >= 0, 2 * margin, -2 * margin)
    x = np.where(near, (target - sh) / sc, x)
    return x.astype(np.float32)


def layer_wgrads_case(dnb, oracle, n, cin, B, k, h, w, with_bn, seed=31):
    r = rng(seed)
    c_tot = cin + 8                                  # the slab is wider than the layer's input
    hw = h * w
    fold1 = f32(np.stack([1.0 + 0.3 * r.standard_normal(cin), 0.3 * r.standard_normal(cin)], axis=1))
    fold2 = f32(np.stack([1.0 + 0.3 * r.standard_normal(B), 0.3 * r.standard_normal(B)], axis=1))
    gamma, beta = f32(1.0 + 0.1 * r.standard_normal(cin)), f32(0.1 * r.standard_normal(cin))
    mean, istd = f32(0.1 * r.standard_normal(cin)), f32(1.0 + 0.1 * r.random(cin))
    y = f32(r.standard_normal((n, c_tot, h, w)))
    if with_bn:   # the BN reduction decides dz = dact * [z > 0] per element: keep every z away from zero
        scale = gamma.astype(np.float64) * istd
        y[:, :cin] = away_from_zero(y[:, :cin], scale, beta - mean * scale)
    db = f32(r.standard_normal((n, B, h, w)))
    b = f32(r.standard_normal((n, B, h, w)))
    g_slab = f32(r.standard_normal((n, k + 4, h, w)))  # g is a channel slice of a wider slab
    dw1 = torch.full((B, cin, 1, 1), float("nan"), device="cuda")
    dw3 = torch.full((k, B, 3, 3), float("nan"), device="cuda")
    scratch = torch.empty(dnb.dnb_op_layer_wgrads_scratch_bytes(n, cin, B, k, h, w), dtype=torch.uint8, device="cuda")
    scratch.fill_(0xFF)
    d_g, d_y = dev(g_slab), dev(y)
    g_view = d_g[:, 4:]                              # channels 4.., image stride (k + 4) * hw
    bn = {}
    if with_bn:
        dact = f32(r.standard_normal((n, cin, h, w)))
        bn = dict(bn_dact=dev(dact), bn_gamma=dev(gamma), bn_beta=dev(beta), bn_mean=dev(mean), bn_istd=dev(istd))
    dnb.dnb_op_layer_wgrads(d_y, c_tot * hw, dev(fold1), dev(db), dw1, cin, dev(b), dev(fold2), g_view, (k + 4) * hw,
                            dw3, n, B, k, h, w, scratch, **bn)
    torch.cuda.synchronize()
    act = lambda x, f: np.maximum(x.astype(np.float64) * f[:, 0].astype(np.float64)[None, :, None, None]
                                  + f[:, 1].astype(np.float64)[None, :, None, None], 0.0)
    assert_close(dw1.cpu().numpy(), oracle.conv_wgrad(act(y[:, :cin], fold1), db, 1), TOL, "1x1 weight gradient")
    assert_close(dw3.cpu().numpy(), oracle.conv_wgrad(act(b, fold2), g_slab[:, 4:], 3), TOL, "3x3 weight gradient")
    if with_bn:
        # the third output of the launch: the partial sums of the BN backward reduction, finished by
        # the element-wise pass (which reads them where the launch left them)
        off = dnb.dnb_op_layer_wgrads_bn_partials_offset(n, cin, B, k, h, w)
        du = torch.full((n, cin, h, w), float("nan"), device="cuda")
        dg, dbt = torch.full((cin,), float("nan"), device="cuda"), torch.full((cin,), float("nan"), device="cuda")
        dnb.dnb_op_bn_relu_backward_apply(d_y, c_tot * hw, bn["bn_dact"], cin * hw, du, cin * hw, 0, n, cin, hw, bn["bn_gamma"],
                                          bn["bn_beta"], bn["bn_mean"], bn["bn_istd"], dg, dbt, scratch.data_ptr() + off)
        torch.cuda.synchronize()
        # the oracle's BN backward takes (mean, var): the given 1/sqrt(var + eps) with eps = 0
        var = 1.0 / istd.astype(np.float64) ** 2
        x1 = y[:, :cin].astype(np.float64)
        z = gamma.astype(np.float64)[None, :, None, None] * (x1 - mean.astype(np.float64)[None, :, None, None]) \
            * istd.astype(np.float64)[None, :, None, None] + beta.astype(np.float64)[None, :, None, None]
        dz = oracle.relu_backward(oracle.relu(z), dact)
        odu, odg, odb = oracle.bn_backward(x1, dz, gamma, mean, var, 0.0)
        assert_close(dg.cpu().numpy(), odg, TOL, "BN dgamma from the launch's partial sums")
        assert_close(dbt.cpu().numpy(), odb, TOL, "BN dbeta from the launch's partial sums")
        assert_close(du.cpu().numpy(), odu, TOL, "BN du")


@pytest.mark.parametrize("n,cin,B,k,h,w,with_bn", [(4, 72, 48, 12, 16, 16, True), (2, 40, 96, 24, 8, 8, False),
                                                   (3, 24, 48, 12, 8, 12, True)])
def test_layer_weight_gradients_in_one_launch(dnb, oracle, n, cin, B, k, h, w, with_bn):
    """All outputs of the launch the one-stream backward pass uses for a bottleneck layer: both
    weight gradients (BN+ReLU of their activation operands recomputed in the operand loads) against
    the oracle's weight gradient, and, when the BN backward reduction rides along, its partial
    sums -- finished by the element-wise pass -- against the oracle's BN backward (dgamma, dbeta, du)."""
    layer_wgrads_case(dnb, oracle, n, cin, B, k, h, w, with_bn)


@pytest.mark.parametrize("cin,B,k", [(60, 48, 12), (204, 48, 12), (264, 96, 24), (1008, 96, 24)])
def test_layer_weight_gradients_at_benchmark_pixel_counts(dnb, oracle, cin, B, k):
    """The same launch at the pixel count the benchmarks run it at (batch 64, 32x32 images: the
    first dense block of DenseNet-BC-100 and -250, narrowest and widest layers): long pixel ranges
    per workgroup, all its roles, strict bound on every output."""
    layer_wgrads_case(dnb, oracle, 64, cin, B, k, 32, 32, True, seed=41)


@pytest.mark.parametrize("n,cin,cout,h,w,ks", [(64, 60, 48, 32, 32, 1), (64, 204, 48, 32, 32, 1), (64, 264, 96, 32, 32, 1),
                                               (64, 1008, 96, 32, 32, 1), (64, 48, 12, 32, 32, 3), (64, 96, 24, 32, 32, 3),
                                               (64, 1476, 96, 16, 16, 1), (64, 516, 1032, 16, 16, 1)])
def test_conv_ops_at_benchmark_pixel_counts(dnb, oracle, n, cin, cout, h, w, ks):
    """Forward, data gradient and weight gradient of the block's convolutions (and the widest
    transition conv) at the benchmarks' full pixel counts, strict bound."""
    test_conv_forward_dgrad_wgrad(dnb, oracle, n, cin, cout, h, w, ks)


def test_layer_weight_gradients_reports_unbuilt_pairs(dnb):
    n, cin, B, k, h, w = 2, 16, 32, 8, 8, 8          # B = 32: two 16-channel tiles, not a built pair
    z = lambda *s: torch.zeros(s, device="cuda")
    scratch = torch.empty(dnb.dnb_op_layer_wgrads_scratch_bytes(n, cin, B, k, h, w), dtype=torch.uint8, device="cuda")
    with pytest.raises(dnb.binding.DnbError) as e:
        dnb.dnb_op_layer_wgrads(z(n, cin, h, w), cin * h * w, z(cin, 2), z(n, B, h, w), z(B, cin, 1, 1), cin, z(n, B, h, w),
                                z(B, 2), z(n, k, h, w), k * h * w, z(k, B, 3, 3), n, B, k, h, w, scratch)
    assert e.value.status == dnb.DNB_E_UNSUPPORTED

