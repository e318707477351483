"""GPU parity of sws_conv2d_padded against the CPU oracle: the 2-D convolution over planes extended on four
sides by the boundary conditions of Section 3 (zeros, mirror, periodic, repeated edge)."""
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
    binding.sws_set_option("conv2d_variant", 0)


def _check(B, x, wgt, sh, sw, pads, mode, what=""):
    y = to_host(B.sws_conv2d_padded(to_gpu(x), to_gpu(wgt), sh, sw, pads, mode))
    ref, mag = oracle.conv2d_padded(x, wgt, sh, sw, pads, mode)
    return assert_within_tol(y, ref, mag, "%s x=%s w=%s s=%dx%d pads=%s mode=%d" % (what, x.shape, wgt.shape, sh, sw, pads, mode))


GEOMS = [
    # Cin Cout kh kw sh sw pads (top, left, bottom, right)
    (64, 64, 3, 3, 1, 1, (1, 1, 1, 1)), (8, 12, 3, 3, 2, 2, (1, 1, 1, 1)), (5, 7, 5, 5, 1, 1, (2, 2, 2, 2)), (16, 6, 1, 7, 1, 2, (0, 3, 0, 3)),
    (3, 9, 7, 3, 3, 1, (3, 1, 3, 1)), (4, 4, 3, 3, 1, 1, (6, 5, 6, 5)), (6, 5, 2, 2, 2, 2, (1, 1, 1, 1)), (2, 3, 4, 6, 1, 1, (3, 5, 3, 5)),
    # unequal pads: direct evaluation
    (8, 8, 3, 3, 1, 1, (2, 0, 0, 1)), (5, 6, 3, 4, 2, 1, (0, 3, 2, 0)),
]


@pytest.mark.parametrize("mode", sorted(MODES))
@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("hw", [(20, 23), (56, 56), (9, 70)])
def test_boundary_rules_on_four_sides(B, mode, geom, hw):
    cin, cout, kh, kw, sh, sw, pads = geom
    r = np.random.Generator(np.random.PCG64(cin * 100 + kh * 10 + kw + hw[0]))
    x = r.standard_normal((2, cin) + hw, dtype=np.float32)
    wgt = (r.standard_normal((cout, cin, kh, kw)) / np.sqrt(cin * kh * kw)).astype(np.float32)
    _check(B, x, wgt, sh, sw, pads, MODES[mode])


@pytest.mark.parametrize("mode", ["mirror", "periodic", "edge"])
def test_integer_inputs_are_exact_on_both_routes(B, mode):
    r = np.random.Generator(np.random.PCG64(3))
    x = r.integers(-8, 9, size=(2, 16, 30, 34)).astype(np.float32)
    wgt = r.integers(-3, 4, size=(10, 16, 3, 3)).astype(np.float32)
    ref, _ = oracle.conv2d_padded(x, wgt, 1, 1, (1, 1, 1, 1), MODES[mode])
    for variant in (0, 1):
        B.sws_set_option("conv2d_variant", variant)
        try:
            y = to_host(B.sws_conv2d_padded(to_gpu(x), to_gpu(wgt), 1, 1, (1, 1, 1, 1), MODES[mode]))
        finally:
            B.sws_set_option("conv2d_variant", 0)
        assert_bit_exact(y, ref, "integers, variant %d" % variant)


def test_small_planes_where_every_output_is_at_the_border(B):
    r = np.random.Generator(np.random.PCG64(5))
    for hw, k, pads, mode in (((1, 1), 3, (1, 1, 1, 1), 3), ((2, 2), 3, (1, 1, 1, 1), 1), ((3, 2), 5, (2, 2, 2, 2), 2),
                              ((4, 40), 9, (4, 4, 4, 4), 2), ((40, 3), 5, (2, 2, 2, 2), 1), ((6, 6), 3, (6, 6, 6, 6), 2)):
        x = r.standard_normal((3, 5) + hw, dtype=np.float32)
        wgt = r.standard_normal((6, 5, k, k), dtype=np.float32)
        _check(B, x, wgt, 1, 1, pads, mode, what="small")
        _check(B, x, wgt, 2, 3, pads, mode, what="small strided")


def test_zero_padding_equals_conv2d_and_periodic_is_circular(B):
    import torch
    r = np.random.Generator(np.random.PCG64(9))
    x = to_gpu(r.standard_normal((2, 64, 28, 28), dtype=np.float32))
    wgt = to_gpu((r.standard_normal((64, 64, 3, 3)) / 24).astype(np.float32))
    a = to_host(B.sws_conv2d(x, wgt, 1, 1, 1, 1))
    b = to_host(B.sws_conv2d_padded(x, wgt, 1, 1, (1, 1, 1, 1), 0))
    assert np.array_equal(a, b)
    y0 = to_host(B.sws_conv2d_padded(x, wgt, 1, 1, (1, 1, 1, 1), 2))
    y1 = to_host(B.sws_conv2d_padded(torch.roll(x, (5, 9), dims=(2, 3)).contiguous(), wgt, 1, 1, (1, 1, 1, 1), 2))
    assert np.abs(np.roll(y0, (5, 9), axis=(2, 3)) - y1).max() < 1e-5      # a shifted plane gives the shifted result
    with pytest.raises(B.SwsError):
        B.sws_conv2d_padded(x, wgt, 1, 1, (28, 0, 0, 0), 1)
    with pytest.raises(B.SwsError):
        B.sws_conv2d_padded(x, wgt, 1, 1, (0, 0, 0, 29), 2)
    with pytest.raises(B.SwsError):
        B.sws_conv2d_padded(x, wgt, 1, 1, (1, 1, 1, 1), 4)


@pytest.mark.parametrize("mode", ["mirror", "periodic"])
def test_cfg4_full_size(B, mode):
    """[32, 64, 56, 56], 64 -> 64, 3 x 3, one virtual row / column a side, in one launch: four whole images,
    every output, against the oracle; the interior equals the zero-padding convolution bit for bit."""
    x, wgt = workloads.make(4)
    xg, wg = to_gpu(x), to_gpu(wgt)
    y = B.sws_conv2d_padded(xg, wg, 1, 1, (1, 1, 1, 1), MODES[mode])
    z = B.sws_conv2d(xg, wg, 1, 1, 1, 1)
    assert bool((y[:, :, 1:-1, 1:-1] == z[:, :, 1:-1, 1:-1]).all())
    sel = [0, 13, 30, 31]
    ref, mag = oracle.conv2d_padded(x[sel], wgt, 1, 1, (1, 1, 1, 1), MODES[mode])
    assert_within_tol(to_host(y[sel]), ref, mag, "cfg4 %s" % mode)
