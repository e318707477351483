"""GPU parity of sws_pool2d_padded against the CPU oracle: pooling over planes extended on four sides by
the boundary conditions of Section 3 (identity, mirror, periodic, repeated edge, shrinking windows)."""
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
    binding.sws_set_option("pool2d_variant", 0)


def _check(B, op, x, kh, kw, sh, sw, pads, mode, scale=None, what=""):
    scale = 1.0 / (kh * kw) if scale is None else scale
    y = to_host(B.sws_pool2d_padded(op, to_gpu(x), kh, kw, sh, sw, pads, mode, scale))
    ref, mag = oracle.pool2d_padded(op, x, kh, kw, sh, sw, pads, mode, scale)
    what = "%s op=%d k=%dx%d s=%dx%d pads=%s mode=%d shape=%s" % (what, op, kh, kw, sh, sw, pads, mode, x.shape)
    if op == 0:
        return assert_within_tol(y, ref, mag, what)
    assert_bit_exact(y, ref, what)
    return 0.0


GEOMS = [
    # kh kw sh sw (top, left, bottom, right)
    (3, 3, 1, 1, (1, 1, 1, 1)), (3, 3, 2, 2, (1, 1, 1, 1)), (2, 2, 2, 2, (0, 1, 1, 0)), (5, 5, 1, 1, (2, 2, 2, 2)),
    (3, 5, 1, 2, (0, 4, 2, 1)), (7, 2, 3, 1, (6, 0, 0, 1)), (1, 1, 1, 1, (2, 3, 1, 0)), (1, 9, 1, 1, (0, 4, 0, 4)),
    (9, 1, 2, 1, (4, 0, 4, 0)), (13, 13, 1, 1, (6, 6, 6, 6)), (4, 4, 4, 4, (3, 3, 3, 3)), (16, 3, 5, 2, (7, 1, 7, 2)),
    (3, 3, 1, 1, (7, 6, 5, 7)), (2, 31, 1, 4, (1, 7, 0, 7)),
]


@pytest.mark.parametrize("mode", sorted(MODES))
@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("shape", [(3, 5, 37, 41), (2, 3, 112, 112), (1, 2, 8, 300)])
def test_boundary_rules_on_four_sides(B, mode, op, geom, shape):
    kh, kw, sh, sw, pads = geom
    r = np.random.Generator(np.random.PCG64(kh * 100 + kw * 10 + sh + sum(pads) + shape[2] + MODES[mode]))
    x = r.standard_normal(shape, dtype=np.float32)
    _check(B, op, x, kh, kw, sh, sw, pads, MODES[mode])


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("mode", sorted(MODES))
def test_integer_inputs_are_exact_on_every_kernel(B, variant, mode):
    """Small integers: every partial sum is an integer below 2^24, so + must be bit-exact whatever the
    order; variant 1 is direct evaluation, 2 the narrowest column tiles."""
    r = np.random.Generator(np.random.PCG64(5 + variant))
    x = r.integers(-40, 41, size=(2, 3, 45, 83)).astype(np.float32)
    B.sws_set_option("pool2d_variant", variant)
    try:
        for kh, kw, sh, sw, pads in GEOMS:
            y = to_host(B.sws_pool2d_padded(0, to_gpu(x), kh, kw, sh, sw, pads, MODES[mode], 1.0))
            ref, _ = oracle.pool2d_padded(0, x, kh, kw, sh, sw, pads, MODES[mode], 1.0)
            assert_bit_exact(y, ref, "integers variant %d %s %s" % (variant, mode, (kh, kw, sh, sw, pads)))
            _check(B, 1, x, kh, kw, sh, sw, pads, MODES[mode], what="variant %d" % variant)
    finally:
        B.sws_set_option("pool2d_variant", 0)


@pytest.mark.parametrize("mode", sorted(MODES))
@pytest.mark.parametrize("op", [0, 1])
@pytest.mark.parametrize("geom,shape", [((3, 3, 1, 1, (1, 1, 1, 1)), (1, 2, 7, 5000)), ((5, 5, 2, 2, (2, 2, 2, 2)), (1, 1, 30, 4001)),
                                        ((2, 16, 2, 16, (0, 9, 0, 9)), (1, 2, 6, 3200)), ((7, 7, 1, 3, (3, 3, 3, 3)), (1, 1, 12, 9000)),
                                        ((1, 255, 1, 1, (0, 127, 0, 127)), (1, 3, 1, 6000))])
def test_planes_wider_than_a_slice_are_cut_into_column_tiles(B, mode, op, geom, shape):
    x = np.random.Generator(np.random.PCG64(shape[3] + geom[1])).standard_normal(shape, dtype=np.float32)
    _check(B, op, x, *geom, MODES[mode], what="wide")


@pytest.mark.parametrize("mode", ["mirror", "periodic", "edge"])
@pytest.mark.parametrize("W", [4, 8, 28, 60, 112, 200, 256, 260, 480, 484, 512, 1000])
def test_row_streaming_kernel_shapes(B, mode, W):
    """3 x 3 (one virtual column a side), 5 x 5 (two), 7 x 7 (three), 9 x 9 to 13 x 13 (four to six: the strip form on
    rows of 64 and more) and 2 x 2 stride 2 on rows of 4 .. 256 elements:
    several groups per wavefront, bands that end inside a group, unequal virtual rows above and below.  Wider rows:
    strips of 256 columns whose outside lanes hold what the rule puts there (planes that end inside a strip, exactly
    on a strip boundary, four columns past one)."""
    r = np.random.Generator(np.random.PCG64(W))
    for H in ((5, 33, 57) if W <= 256 else (5, 21)):
        x = r.standard_normal((2, 5, H, W), dtype=np.float32)
        xi = r.integers(-9, 10, size=(1, 9, H, W)).astype(np.float32)
        for kh, s, pads in ((3, 1, (1, 1, 1, 1)), (3, 1, (4, 1, 0, 1)), (3, 2, (1, 1, 1, 1)), (3, 2, (0, 1, 3, 0)),
                            (2, 2, (0, 0, 0, 0)), (2, 2, (1, 0, 2, 1)), (2, 2, (3, 0, 0, 0)),
                            (5, 1, (2, 2, 2, 2)), (5, 1, (0, 2, 4, 2)), (7, 1, (3, 3, 3, 3)), (7, 1, (4, 3, 2, 3)),
                            (9, 1, (4, 4, 4, 4)), (9, 1, (0, 4, 8, 4)), (11, 1, (5, 5, 5, 5)), (13, 1, (6, 6, 6, 6)),
                            (13, 1, (9, 6, 3, 6))):
            if max(pads[0], pads[2]) > H - 1 or max(pads[1], pads[3]) > W - 1:
                continue                                 # (a mirrored or periodic pad cannot exceed the plane)
            for op in (0, 1, 2):
                _check(B, op, x, kh, kh, s, s, pads, MODES[mode], what="rows")
            y = to_host(B.sws_pool2d_padded(0, to_gpu(xi), kh, kh, s, s, pads, MODES[mode], 1.0))
            ref, _ = oracle.pool2d_padded(0, xi, kh, kh, s, s, pads, MODES[mode], 1.0)
            assert_bit_exact(y, ref, "rows, integers %s" % (pads,))


def test_largest_pads_and_smallest_planes(B):
    r = np.random.Generator(np.random.PCG64(19))
    x = r.standard_normal((2, 3, 9, 13), dtype=np.float32)
    for op in (0, 1, 2):
        _check(B, op, x, 4, 5, 1, 1, (8, 12, 8, 12), MODES["mirror"])          # pads = extent - 1
        _check(B, op, x, 4, 5, 2, 3, (9, 13, 9, 13), MODES["periodic"])        # pads = extent: the plane three times
        _check(B, op, x, 6, 6, 1, 1, (20, 17, 30, 25), MODES["edge"])
        _check(B, op, x, 3, 3, 1, 1, (5, 4, 6, 7), MODES["identity"])          # windows wholly inside the padding
    one = r.standard_normal((3, 2, 1, 1), dtype=np.float32)
    for op in (0, 1, 2):
        _check(B, op, one, 1, 1, 1, 1, (0, 0, 0, 0), MODES["mirror"])
        _check(B, op, one, 2, 2, 1, 1, (1, 1, 1, 1), MODES["periodic"])
        _check(B, op, one, 3, 2, 1, 1, (2, 2, 2, 2), MODES["edge"])
        _check(B, op, one, 2, 2, 1, 1, (1, 1, 1, 1), MODES["identity"])
    col = r.standard_normal((1, 2, 40, 1), dtype=np.float32)
    _check(B, 0, col, 5, 3, 1, 1, (2, 1, 2, 1), MODES["periodic"])
    _check(B, 1, col, 5, 3, 2, 1, (2, 2, 2, 2), MODES["edge"])


def test_windows_too_large_for_a_slice_fall_back_to_direct_evaluation(B):
    r = np.random.Generator(np.random.PCG64(23))
    x = r.standard_normal((1, 2, 90, 120), dtype=np.float32)
    for mode in MODES.values():
        _check(B, 0, x, 70, 50, 1, 1, (35, 25, 34, 24), mode)
        _check(B, 1, x, 80, 64, 3, 2, (10, 10, 10, 10), mode)


def test_identity_and_shrinking_windows_equal_the_other_entry_points(B):
    r = np.random.Generator(np.random.PCG64(29))
    xh = r.standard_normal((2, 4, 56, 60), dtype=np.float32)
    x = to_gpu(xh)
    pads = (1, 2, 0, 1)
    a = to_host(B.sws_pool2d_ex(0, x, 3, 3, 2, 2, pads, B.SWS_DIV_SCALE, 1 / 9))
    b = to_host(B.sws_pool2d_padded(0, x, 3, 3, 2, 2, pads, 0, 1 / 9))
    assert np.array_equal(a, b)
    a = to_host(B.sws_pool2d_ex(0, x, 3, 3, 2, 2, pads, B.SWS_DIV_REAL_CELLS, 1.0))
    b = to_host(B.sws_pool2d_padded(0, x, 3, 3, 2, 2, pads, 4, 1.0))
    assert np.array_equal(a, b)
    ref, mag = oracle.pool2d_ex(0, xh, 3, 3, 2, 2, pads, True, 1.0)
    assert_within_tol(b, ref, mag, "shrinking windows")
    for op in (1, 2):                                                          # max / min ignore the divisor
        b = to_host(B.sws_pool2d_padded(op, x, 3, 3, 2, 2, pads, 4, 1.0))
        ref, _ = oracle.pool2d_padded(op, xh, 3, 3, 2, 2, pads, 0, 1.0)
        assert_bit_exact(b, ref, "shrinking windows op %d" % op)
    with pytest.raises(B.SwsError):
        B.sws_pool2d_padded(0, x, 3, 3, 1, 1, (56, 0, 0, 0), 1)
    with pytest.raises(B.SwsError):
        B.sws_pool2d_padded(0, x, 3, 3, 1, 1, (0, 0, 0, 61), 2)
    with pytest.raises(B.SwsError):
        B.sws_pool2d_padded(0, x, 3, 3, 1, 1, (0, 0, 0, 0), 7)


def test_random_geometries(B):
    r = np.random.Generator(np.random.PCG64(31))
    for case in range(120):
        H, W = int(r.integers(1, 70)), int(r.integers(1, 200))
        mode = int(r.integers(0, 4))
        lim_h = {0: 12, 1: H - 1, 2: H, 3: 12}[mode]
        lim_w = {0: 12, 1: W - 1, 2: W, 3: 12}[mode]
        pads = (int(r.integers(0, min(lim_h, 12) + 1)), int(r.integers(0, min(lim_w, 12) + 1)),
                int(r.integers(0, min(lim_h, 12) + 1)), int(r.integers(0, min(lim_w, 12) + 1)))
        kh = int(r.integers(1, min(H + pads[0] + pads[2], 17) + 1))
        kw = int(r.integers(1, min(W + pads[1] + pads[3], 17) + 1))
        sh, sw = int(r.integers(1, 4)), int(r.integers(1, 4))
        x = r.standard_normal((int(r.integers(1, 4)), int(r.integers(1, 6)), H, W), dtype=np.float32)
        _check(B, int(r.integers(0, 3)), x, kh, kw, sh, sw, pads, mode, what="case %d" % case)


@pytest.mark.parametrize("mode", ["mirror", "periodic"])
def test_cfg3_full_size_every_plane(B, mode):
    """[32, 64, 112, 112], 3 x 3, one virtual row / column on every side, stride 1 and 2, at full size in
    one launch: every output of all 2048 planes against the oracle."""
    x, _ = workloads.make(3)
    xg = to_gpu(x)
    for stride, op in ((1, 0), (2, 1)):
        y = to_host(B.sws_pool2d_padded(op, xg, 3, 3, stride, stride, (1, 1, 1, 1), MODES[mode], 1 / 9))
        ref, mag = oracle.pool2d_padded(op, x, 3, 3, stride, stride, (1, 1, 1, 1), MODES[mode], 1 / 9)
        if op == 0:
            assert_within_tol(y, ref, mag, "cfg3 %s stride %d" % (mode, stride))
        else:
            assert_bit_exact(y, ref, "cfg3 %s stride %d" % (mode, stride))
