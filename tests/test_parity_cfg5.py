"""Configuration 5 at full size ([256, 128, 16384], 2 GiB of input), in the launch shape the
bench times: sliding add / max with w in {16, 64, 255} and the 31-tap depthwise convolution.
The oracle checks a seeded sample of whole rows (first and last included); properties that
hold at any size cover every output."""
import numpy as np
import pytest

import oracle
from paper_2305_16513_amd import workloads
from parity_util import assert_bit_exact, assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu

ROWS, LEN = 256 * 128, 16384


@pytest.fixture(scope="module")
def data():
    import torch
    from paper_2305_16513_amd import binding
    binding.lib()
    x, taps = workloads.make(5)
    rng = np.random.Generator(np.random.PCG64(55))
    rows = sorted(set([0, 1, ROWS - 1] + rng.integers(0, ROWS, size=21).tolist()))
    xg = to_gpu(x)
    yield binding, x.reshape(ROWS, LEN), taps, xg, rows
    del xg
    torch.cuda.empty_cache()


@pytest.mark.parametrize("w", [16, 64, 255])
def test_cfg5_slide_max(data, w):
    B, x, _, xg, rows = data
    yg = B.sws_slide1d(1, xg, w)
    lo = LEN - w + 1
    y = to_host(yg.reshape(ROWS, lo)[rows])
    ref, _ = oracle.slide1d(1, x[rows], w)
    assert_bit_exact(y, ref, "cfg5 max w=%d" % w)
    # every output is >= the first, the middle and the last element of its window
    for off in (0, w // 2, w - 1):
        assert bool((yg >= xg[..., off:off + lo]).all())
    del yg


@pytest.mark.parametrize("w", [16, 64, 255])
def test_cfg5_slide_add(data, w):
    import torch
    B, x, _, xg, rows = data
    yg = B.sws_slide1d(0, xg, w)
    lo = LEN - w + 1
    y = to_host(yg.reshape(ROWS, lo)[rows])
    ref, mag = oracle.slide1d(0, x[rows], w)
    worst = assert_within_tol(y, ref, mag, "cfg5 add w=%d" % w)
    assert worst < 2e-6
    # recurrence y[i+1] - y[i] = x[i+w] - x[i], up to the rounding of sums of magnitude <= w
    d = (yg[..., 1:] - yg[..., :-1]) - (xg[..., w:] - xg[..., :lo - 1])
    assert float(d.abs().max()) < 1e-5 * w
    del yg, d
    torch.cuda.empty_cache()


def test_cfg5_depthwise_conv(data):
    B, x, taps, xg, rows = data
    yg = B.sws_conv1d(xg, to_gpu(taps), groups=128)
    y = to_host(yg.reshape(ROWS, LEN - 30)[rows])
    for n, r in enumerate(rows):
        ref, mag = oracle.conv1d(x[r].reshape(1, 1, LEN), taps[r % 128].reshape(1, 1, 31))
        assert_within_tol(y[n], ref[0, 0], mag[0, 0], "cfg5 dwconv row %d" % r)
    assert bool(yg.isfinite().all())
