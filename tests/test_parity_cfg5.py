"""Configuration 5 at full size ([256, 128, 16384], 2 GiB of input), in the launch shape the
bench times: sliding add / max with w in {16, 64, 255} and the 31-tap depthwise convolution.
Every one of the 32768 rows is compared with the oracle, output by output, for every operator
(all 128 tap sets of the depthwise layer included): the oracle runs over slabs of 8192 rows on
the host cores, its values are uploaded and the element-wise acceptance rule is evaluated on the
device (the rule itself is the one of parity_util, restated on tensors).  Rows are not
interchangeable in these kernels (tile origins and border tiles depend on the row), hence no
sampling."""
import numpy as np
import pytest

import oracle
from paper_2305_16513_amd import workloads
from parity_util import TOL, assert_bit_exact, assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu

ROWS, LEN, CH = 256 * 128, 16384, 128
SLAB = 8192


@pytest.fixture(scope="module")
def data():
    import torch
    from paper_2305_16513_amd import binding
    binding.lib()
    x, taps = workloads.make(5)
    workloads.check_clean(x)
    xg = to_gpu(x)
    yield binding, x.reshape(ROWS, LEN), taps, xg
    del xg
    torch.cuda.empty_cache()


def _slabs():
    return [(r0, min(r0 + SLAB, ROWS)) for r0 in range(0, ROWS, SLAB)]


def _check_bits_on_device(yg_rows, ref, what):
    """yg_rows: device fp32 [n, lo]; ref: host fp64 [n, lo].  Bit equality of every output."""
    import torch
    want = torch.from_numpy(ref.astype(np.float32)).cuda()
    same = yg_rows.view(torch.int32) == want.view(torch.int32)
    if not bool(same.all()):
        assert_bit_exact(to_host(yg_rows), ref, what)           # names the first mismatch
        raise AssertionError(what + ": device and host comparisons disagree")


def _check_tol_on_device(yg_rows, ref, mag, what):
    """|y - ref| <= TOL * sum|terms| for every output; returns the worst ratio."""
    import torch
    r = torch.from_numpy(ref).cuda()
    m = torch.from_numpy(mag).cuda()
    err = (yg_rows.double() - r).abs_()
    del r
    ok = bool((err <= TOL * m).all()) and bool(torch.isfinite(yg_rows).all())
    if not ok:
        assert_within_tol(to_host(yg_rows), ref, mag, what)     # names the first offender
        raise AssertionError(what + ": device and host comparisons disagree")
    ratio = torch.where(m > 0, err / m, torch.zeros_like(err))
    return float(ratio.max())


@pytest.mark.parametrize("w", [16, 64, 255])
def test_cfg5_slide_max_every_row(data, w):
    B, x, _, xg = data
    yg = B.sws_slide1d(1, xg, w).reshape(ROWS, LEN - w + 1)
    for r0, r1 in _slabs():
        ref, _ = oracle.slide1d(oracle.OP_MAX, x[r0:r1], w)
        _check_bits_on_device(yg[r0:r1], ref, "cfg5 max w=%d rows %d..%d" % (w, r0, r1))
        del ref
    del yg


@pytest.mark.parametrize("w", [16, 64, 255])
def test_cfg5_slide_add_every_row(data, w):
    import torch
    B, x, _, xg = data
    yg = B.sws_slide1d(0, xg, w).reshape(ROWS, LEN - w + 1)
    worst = 0.0
    for r0, r1 in _slabs():
        ref, mag = oracle.slide1d(oracle.OP_ADD, x[r0:r1], w)
        worst = max(worst, _check_tol_on_device(yg[r0:r1], ref, mag, "cfg5 add w=%d rows %d..%d" % (w, r0, r1)))
        del ref, mag
    assert worst < 2e-6            # the bound the arithmetic gives (about 2.3e-6), with measured margin
    del yg
    torch.cuda.empty_cache()


def test_cfg5_depthwise_conv_every_row(data):
    """All 256 x 128 rows, each against its own channel's 31 taps."""
    import torch
    B, x, taps, xg = data
    lo = LEN - 30
    yg = B.sws_conv1d(xg, to_gpu(taps), groups=CH).reshape(ROWS, lo)
    worst = 0.0
    for r0, r1 in _slabs():
        n = r1 - r0
        ref, mag = oracle.conv1d(x[r0:r1].reshape(n // CH, CH, LEN), taps, groups=CH)
        worst = max(worst, _check_tol_on_device(yg[r0:r1], ref.reshape(n, lo), mag.reshape(n, lo),
                                                "cfg5 dwconv rows %d..%d" % (r0, r1)))
        del ref, mag
    assert worst < 2e-6
    del yg
    torch.cuda.empty_cache()
