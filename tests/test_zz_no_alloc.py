"""The entry point that allocates nothing (dnb_op_bn_stats_static: BN batch statistics with the
split-reduction partials in a device array inside the library) against the existing entry point
that takes the caller's scratch buffer (dnb_op_bn_stats), through the C ABI: two calls in a row,
the second on a smaller input, so stale partials of the first call would show.  Both run the same
kernels, so the results must agree bit for bit; the existing entry point is itself checked against
the oracle in test_gpu_ops.py, and the oracle is compared here once more."""
import numpy as np
import pytest
import torch

from gpu_util import assert_close, dev

pytestmark = pytest.mark.gpu


def stats_both(dnb, x, eps):
    n, c, h, w = x.shape
    d_x = dev(x)
    out = []
    for static in (False, True):
        mean = torch.full((c,), float("nan"), device="cuda")
        istd = torch.full((c,), float("nan"), device="cuda")
        if static:
            dnb.dnb_op_bn_stats_static(d_x, c * h * w, n, c, h * w, eps, mean, istd)
        else:
            scratch = torch.empty(dnb.dnb_op_bn_scratch_bytes(n, c, h * w), dtype=torch.uint8, device="cuda")
            dnb.dnb_op_bn_stats(d_x, c * h * w, n, c, h * w, eps, mean, istd, scratch)
        torch.cuda.synchronize()
        out.append((mean.cpu().numpy(), istd.cpu().numpy()))
    return out


def test_static_scratch_entry_point_matches_the_one_with_a_caller_buffer(dnb, oracle):
    r = np.random.default_rng(11)
    eps = 1e-5
    # a large input first (64 splits x 204 channels of partials), then a smaller one
    for shape in ((64, 204, 16, 16), (3, 20, 7, 9)):
        n, c, h, w = shape
        x = (r.standard_normal(shape) * r.uniform(0.2, 4, (1, c, 1, 1)) + r.uniform(-2, 2, (1, c, 1, 1))).astype(np.float32)
        (m0, i0), (m1, i1) = stats_both(dnb, x, eps)
        assert np.array_equal(m0, m1) and np.array_equal(i0, i1), shape
        _, omean, ovar = oracle.bn_forward(x, np.ones(c), np.zeros(c), eps)
        assert_close(m1, omean, 1e-4, "mean")
        assert_close(i1, 1 / np.sqrt(ovar + eps), 1e-4, "istd")


def test_static_scratch_entry_point_rejects_what_does_not_fit(dnb):
    # 40000 channels x 12 bytes of partials is beyond the 256 KiB array: refused before any launch
    with pytest.raises(dnb.binding.DnbError) as e:
        dnb.dnb_op_bn_stats_static(4096, 40000 * 4, 2, 40000, 4, 1e-5, 4096, 4096, 0)
    assert e.value.status == dnb.DNB_E_RANGE
