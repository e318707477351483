"""GPU parity of sws_conv1d_padded against the CPU oracle: the convolution of Section 2.5 over rows extended
by the boundary conditions of Section 3 (zeros, mirror, periodic, repeated edge)."""
import numpy as np
import pytest

import oracle
from paper_2305_16513_amd import workloads
from parity_util import assert_bit_exact, assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu
MODES = {"identity": 0, "mirror": 1, "periodic": 2, "edge": 3}


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    yield binding
    binding.sws_set_option("conv1d_variant", 0)


def _check(B, x, wgt, stride, pl, pr, dil, groups, mode, what=""):
    y = to_host(B.sws_conv1d_padded(to_gpu(x), to_gpu(wgt), stride, pl, pr, dil, groups, mode))
    ref, mag = oracle.conv1d_padded(x, wgt, stride, pl, pr, dil, groups, mode)
    return assert_within_tol(y, ref, mag, "%s x=%s w=%s s=%d pads=(%d,%d) d=%d g=%d mode=%d" % (
        what, x.shape, wgt.shape, stride, pl, pr, dil, groups, mode))


@pytest.mark.parametrize("mode", sorted(MODES))
@pytest.mark.parametrize("k", [1, 2, 3, 5, 16, 31, 33, 64])
@pytest.mark.parametrize("L", [70, 1000, 1039, 5000])
def test_one_channel_per_output_on_the_sliding_kernel(B, mode, k, L):
    """Depthwise rows and a channel multiplier: end tiles read their virtual elements through the rule; rows of
    one tile, of a tile and a ragged tail, of several tiles; pads from none to more than a tile."""
    r = np.random.Generator(np.random.PCG64(L * 100 + k))
    x = r.standard_normal((2, 3, L), dtype=np.float32)
    for cout, pads in ((3, (k // 2, (k - 1) - k // 2)), (6, (0, k - 1)), (3, (min(L - 1, 1500), 7)), (3, (3, min(L - 1, 1100)))):
        wgt = r.standard_normal((cout, 1, k), dtype=np.float32)
        _check(B, x, wgt, 1, pads[0], pads[1], 1, 3, MODES[mode], what="thin")


@pytest.mark.parametrize("mode", ["mirror", "periodic", "edge"])
def test_integer_inputs_are_exact_and_direct_evaluation_agrees(B, mode):
    r = np.random.Generator(np.random.PCG64(7))
    x = r.integers(-20, 21, size=(3, 4, 2500)).astype(np.float32)
    wgt = r.integers(-5, 6, size=(4, 1, 31)).astype(np.float32)
    ref, _ = oracle.conv1d_padded(x, wgt, 1, 15, 15, 1, 4, MODES[mode])
    for variant in (0, 1):
        B.sws_set_option("conv1d_variant", variant)
        try:
            y = to_host(B.sws_conv1d_padded(to_gpu(x), to_gpu(wgt), 1, 15, 15, 1, 4, MODES[mode]))
        finally:
            B.sws_set_option("conv1d_variant", 0)
        assert_bit_exact(y, ref, "integers, variant %d" % variant)


@pytest.mark.parametrize("mode", sorted(MODES))
@pytest.mark.parametrize("geom", [
    # Cin Cout k stride pl pr dil groups
    (8, 8, 3, 1, 1, 1, 1, 1), (8, 12, 5, 2, 4, 0, 1, 4), (6, 6, 7, 1, 9, 9, 3, 6), (4, 8, 4, 3, 0, 5, 2, 2), (1, 1, 51, 1, 200, 200, 8, 1),
    (5, 5, 9, 2, 4, 4, 1, 5), (3, 3, 80, 1, 40, 39, 1, 3),
])
def test_every_other_geometry(B, mode, geom):
    """Dense and grouped channels, strides, dilation, kernels of more than 64 taps."""
    cin, cout, k, stride, pl, pr, dil, groups = geom
    r = np.random.Generator(np.random.PCG64(cin * 10 + k))
    x = r.standard_normal((2, cin, 777), dtype=np.float32)
    wgt = r.standard_normal((cout, cin // groups, k), dtype=np.float32)
    _check(B, x, wgt, stride, pl, pr, dil, groups, MODES[mode], what="other")


def test_zero_padding_equals_conv1d_and_periodic_is_circular(B):
    r = np.random.Generator(np.random.PCG64(9))
    x = to_gpu(r.standard_normal((2, 16, 3000), dtype=np.float32))
    wgt = to_gpu(r.standard_normal((16, 1, 9), dtype=np.float32))
    a = to_host(B.sws_conv1d(x, wgt, 1, 4, 1, 16))
    b = to_host(B.sws_conv1d_padded(x, wgt, 1, 4, 4, 1, 16, 0))
    assert np.array_equal(a, b)
    # circular correlation: shifting the row by s shifts the result by s
    y0 = to_host(B.sws_conv1d_padded(x, wgt, 1, 0, 8, 1, 16, 2))
    import torch
    y1 = to_host(B.sws_conv1d_padded(torch.roll(x, 37, dims=2).contiguous(), wgt, 1, 0, 8, 1, 16, 2))
    assert y0.shape == (2, 16, 3000) and np.array_equal(np.roll(y0, 37, axis=2), y1)
    with pytest.raises(B.SwsError):
        B.sws_conv1d_padded(x, wgt, 1, 3000, 0, 1, 16, 1)
    with pytest.raises(B.SwsError):
        B.sws_conv1d_padded(x, wgt, 1, 0, 3001, 1, 16, 2)
    with pytest.raises(B.SwsError):
        B.sws_conv1d_padded(x, wgt, 1, 1, 1, 1, 16, 4)


def test_random_geometries(B):
    r = np.random.Generator(np.random.PCG64(13))
    for case in range(100):
        L = int(r.integers(1, 2600))
        mode = int(r.integers(0, 4))
        lim = {0: 40, 1: L - 1, 2: L, 3: 40}[mode]
        pl, pr = int(r.integers(0, min(lim, 40) + 1)), int(r.integers(0, min(lim, 40) + 1))
        thin = case % 2 == 0
        stride, dil = (1, 1) if thin else (int(r.integers(1, 4)), int(r.integers(1, 4)))
        k = int(r.integers(1, 34))
        while dil * (k - 1) + 1 > L + pl + pr:
            k -= 1
        ch = int(r.integers(1, 6))
        groups = ch if thin else int(r.choice([g for g in range(1, ch + 1) if ch % g == 0]))
        x = r.standard_normal((int(r.integers(1, 3)), ch, L), dtype=np.float32)
        wgt = r.standard_normal((ch * int(r.integers(1, 3)), ch // groups, k), dtype=np.float32)
        _check(B, x, wgt, stride, pl, pr, dil, groups, mode, what="case %d" % case)


@pytest.mark.parametrize("mode", ["mirror", "periodic"])
def test_cfg5_full_size_sampled_rows(B, mode):
    """[256, 128, 16384], depthwise k = 31, one output per input (15 virtual elements a side), at full size in
    one launch; 96 of the 32768 rows, every output, against the oracle."""
    x, taps = workloads.make(5)
    y = B.sws_conv1d_padded(to_gpu(x), to_gpu(taps), 1, 15, 15, 1, 128, MODES[mode])
    assert tuple(y.shape) == (256, 128, 16384)
    r = np.random.Generator(np.random.PCG64(5))
    rows = sorted(set([0, 127, 128, 32767] + r.integers(0, 32768, 92).tolist()))
    got = to_host(y.reshape(32768, 16384)[rows])
    xs = x.reshape(32768, 16384)[rows][None]
    ws = np.stack([taps[q % 128] for q in rows])
    ref, mag = oracle.conv1d_padded(xs, ws, 1, 15, 15, 1, len(rows), MODES[mode])
    assert_within_tol(got[None], ref, mag, "cfg5 %s" % mode)
