"""The shapes of the paper's two experiments (Experiments section) at full size, in the launch
shape the bench times: single-channel 1-D convolution over the filter sizes of the first
figure, and the 51-tap dilation-8 kernel of the second at its output sizes.  The oracle checks
seeded samples (whole short sequences; stretches of the long ones, first and last included)."""
import numpy as np
import pytest

import oracle
from paper_2305_16513_amd import workloads
from parity_util import assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    return binding


def test_filter_sweep_full_size(B):
    import torch
    x, _ = workloads.make(6)
    rows, _, length = x.shape
    xg = to_gpu(x)
    rng = np.random.Generator(np.random.PCG64(66))
    for k in workloads.FILTER_SIZES:
        taps = workloads.make(6, x_shape=(1,), wgt_shape=(1, 1, k))[1]
        yg = B.sws_conv1d(xg, to_gpu(taps))
        lo = length - k + 1
        assert yg.shape == (rows, 1, lo)
        n = 3000                                   # outputs per sampled stretch: spans tile seams
        starts = [0, lo - n] + rng.integers(0, lo - n, size=4).tolist()
        for r in (0, rows - 1, int(rng.integers(0, rows))):
            for s in starts:
                ref, mag = oracle.conv1d(x[r:r + 1, :, s:s + n + k - 1], taps)
                assert_within_tol(to_host(yg[r, 0, s:s + n]), ref[0, 0], mag[0, 0], "k=%d row %d at %d" % (k, r, s))
        assert bool(yg.isfinite().all())
        del yg
    del xg
    torch.cuda.empty_cache()


@pytest.mark.parametrize("q", workloads.DILATED_OUTPUT_SIZES)
def test_dilated_single_sequence(B, q):
    k, d = workloads.DILATED_K, workloads.DILATED_D
    x, taps = workloads.make(7, x_shape=(1, 1, q + (k - 1) * d), wgt_shape=(1, 1, k))
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(taps), 1, 0, d, 1))
    ref, mag = oracle.conv1d(x, taps, 1, 0, d, 1)
    assert y.shape == (1, 1, q)
    assert_within_tol(y, ref, mag, "dilated q=%d" % q)


def test_dilated_batched_full_size(B):
    import torch
    k, d = workloads.DILATED_K, workloads.DILATED_D
    x, taps = workloads.make(7)
    ch, length = x.shape[1], x.shape[2]
    yg = B.sws_conv1d(to_gpu(x), to_gpu(taps), 1, 0, d, ch)
    rng = np.random.Generator(np.random.PCG64(77))
    for c in sorted(set([0, 1, ch - 1] + rng.integers(0, ch, size=13).tolist())):
        ref, mag = oracle.conv1d(x[:, c:c + 1], taps[c:c + 1], 1, 0, d, 1)
        assert_within_tol(to_host(yg[0, c]), ref[0, 0], mag[0, 0], "dilated depthwise channel %d" % c)
    assert bool(yg.isfinite().all())
    del yg
    torch.cuda.empty_cache()
