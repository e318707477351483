"""GPU parity of sws_pool2d against the CPU oracle (Section 2.3 in two dimensions)."""
import numpy as np
import pytest

import oracle
from paper_2305_16513_amd import workloads
from parity_util import assert_bit_exact, assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu
OPS = {"add": 0, "max": 1, "min": 2}


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    yield binding
    binding.sws_set_option("pool2d_variant", 0)


def _check(B, op, x, kh, kw, sh, sw, ph, pw, what=""):
    scale = 1.0 / (kh * kw)
    y = to_host(B.sws_pool2d(OPS[op], to_gpu(x), kh, kw, sh, sw, ph, pw, scale))
    ref, mag = oracle.pool2d(OPS[op], x, kh, kw, sh, sw, ph, pw, scale)
    if op == "add":
        return assert_within_tol(y, ref, mag, what)
    assert_bit_exact(y, ref, what)
    return 0.0


GEOMS = [
    # kh kw sh sw ph pw
    (3, 3, 1, 1, 1, 1), (3, 3, 2, 2, 1, 1), (3, 3, 1, 1, 0, 0), (2, 2, 2, 2, 0, 0), (5, 5, 1, 1, 2, 2),
    (3, 5, 1, 2, 1, 2), (7, 2, 3, 1, 3, 0), (1, 1, 1, 1, 0, 0), (1, 4, 1, 1, 0, 3), (4, 1, 2, 1, 3, 0),
    (13, 13, 1, 1, 6, 6), (3, 3, 3, 3, 0, 0), (9, 9, 1, 1, 4, 4), (7, 7, 1, 1, 3, 3), (2, 2, 1, 1, 0, 0),
    # no specialised kernel: the run-time separable kernel
    (11, 11, 1, 1, 5, 5), (4, 4, 4, 4, 0, 0), (6, 6, 2, 2, 2, 2), (15, 15, 1, 1, 7, 7), (1, 7, 1, 1, 0, 3), (16, 3, 5, 2, 8, 1),
    (3, 31, 1, 4, 2, 15),
]


@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("shape", [(2, 3, 37, 53), (1, 5, 112, 112), (3, 2, 16, 200), (2, 2, 129, 19)])
def test_geometries(B, op, geom, shape):
    kh, kw, sh, sw, ph, pw = geom
    if kh > shape[2] + 2 * ph or kw > shape[3] + 2 * pw:
        pytest.skip("window larger than plane")
    rng = np.random.Generator(np.random.PCG64(hash((geom, shape)) % (2 ** 31)))
    x = rng.standard_normal(shape, dtype=np.float32)
    _check(B, op, x, *geom, what="%s %s %s" % (op, geom, shape))


def test_all_negative_plane_max_ignores_padding(B):
    x = -np.abs(np.random.Generator(np.random.PCG64(3)).standard_normal((2, 2, 20, 24), dtype=np.float32)) - 1
    _check(B, "max", x, 3, 3, 1, 1, 1, 1)
    _check(B, "min", -x, 3, 3, 2, 2, 1, 1)


def test_add_bit_exact_on_integer_valued_input(B):
    x = workloads.integer_valued((2, 3, 57, 61), -32, 32, seed=9)
    y = to_host(B.sws_pool2d(0, to_gpu(x), 3, 3, 1, 1, 1, 1, 1.0))
    ref, _ = oracle.pool2d(0, x, 3, 3, 1, 1, 1, 1, 1.0)
    assert np.array_equal(y.astype(np.float64), ref)


@pytest.mark.parametrize("flags", [128, 128 | 2, 128 | 512])
def test_band_kernel_knobs(B, flags):
    """The band kernel where the row-streaming kernel would be taken (128), with the XCD-contiguous
    placement (2) or four-wavefront workgroups in launch order (512): measurement knobs, not semantics."""
    x = np.random.Generator(np.random.PCG64(flags)).standard_normal((3, 5, 60, 112), dtype=np.float32)
    B.sws_set_option("pool2d_variant", flags)
    try:
        _check(B, "max", x, 3, 3, 1, 1, 1, 1)
        _check(B, "add", x, 3, 3, 2, 2, 1, 1)
    finally:
        B.sws_set_option("pool2d_variant", 0)


ROW_SHAPES = [(1, 1, 1, 4), (2, 3, 5, 8), (3, 2, 9, 28), (2, 9, 56, 56), (1, 11, 112, 112), (2, 2, 31, 224), (1, 3, 7, 256),
              (1, 17, 3, 36), (19, 1, 2, 100)]


@pytest.mark.parametrize("band_kernel", [False, True])
@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("geom", [(3, 1, 1), (3, 2, 1), (2, 2, 0), (5, 1, 2), (7, 1, 3), (9, 1, 4), (11, 1, 5), (13, 1, 6)])
@pytest.mark.parametrize("shape", ROW_SHAPES)
def test_row_streaming_kernel(B, band_kernel, op, geom, shape):
    """3 x 3 pad 1 at stride 1 and 2 and 2 x 2 stride 2 on rows of 4 .. 256 elements (multiples of 4) run on the
    kernel without LDS: one to sixteen lane groups per wavefront, planes that end inside the last round of
    eight, odd heights, x off the 16-byte boundary.  Option pool2d_variant 128 puts the same calls on the band
    kernel; both must agree with the oracle."""
    import torch
    k, s, p = geom
    n, c, h, w = shape
    if s == 2 and w % 2:
        pytest.skip("odd width")
    rng = np.random.Generator(np.random.PCG64(1000 * k + 100 * s + h * w + n))
    x = rng.standard_normal(shape, dtype=np.float32)
    flat = torch.empty(x.size + 1, device="cuda")
    xg = flat[1:].view(shape)                         # 4-byte aligned only
    xg.copy_(to_gpu(x))
    scale = 1.0 / (k * k)
    B.sws_set_option("pool2d_variant", 128 if band_kernel else 0)
    try:
        for ph in sorted({p, 0, k - 1}):
            if h + 2 * ph < k:
                continue
            y = to_host(B.sws_pool2d(OPS[op], xg, k, k, s, s, ph, p, scale))
            ref, mag = oracle.pool2d(OPS[op], x, k, k, s, s, ph, p, scale)
            what = "rows kernel %s %s ph=%d %s" % (op, geom, ph, shape)
            if op == "add":
                assert_within_tol(y, ref, mag, what)
            else:
                assert_bit_exact(y, ref, what)
    finally:
        B.sws_set_option("pool2d_variant", 0)


def test_row_streaming_kernel_guard_band(B):
    """Nothing is written outside y: guard elements around the output keep their value."""
    import torch
    x = np.random.Generator(np.random.PCG64(77)).standard_normal((5, 3, 21, 44), dtype=np.float32)
    for k, s, p in ((3, 1, 1), (3, 2, 1), (2, 2, 0)):
        ho, wo = (21 + 2 * p - k) // s + 1, (44 + 2 * p - k) // s + 1
        buf = torch.full((15 * ho * wo + 64,), 12345.0, device="cuda")
        y = buf[32:32 + 15 * ho * wo].view(5, 3, ho, wo)
        B.sws_pool2d(1, to_gpu(x), k, k, s, s, p, p, 1.0, y=y)
        ref, _ = oracle.pool2d(1, x, k, k, s, s, p, p, 1.0)
        assert_bit_exact(to_host(y), ref, "guarded %s" % ((k, s, p),))
        assert bool((buf[:32] == 12345.0).all()) and bool((buf[32 + 15 * ho * wo:] == 12345.0).all())


@pytest.mark.parametrize("op", ["add", "max"])
@pytest.mark.parametrize("geom,shape", [((1, 3, 1, 2, 0, 1), (2, 3, 1, 20001)), ((1, 9, 1, 1, 0, 4), (1, 2, 1, 50000)),
                                        ((3, 3, 1, 1, 1, 1), (1, 2, 7, 5000)), ((5, 5, 2, 2, 2, 2), (1, 1, 30, 4001)),
                                        ((2, 16, 2, 16, 0, 0), (1, 2, 6, 3200)), ((7, 7, 1, 3, 3, 3), (1, 1, 12, 9000))])
def test_planes_wider_than_a_slice_are_cut_into_column_tiles(B, op, geom, shape):
    """Rows too wide for a wavefront's LDS slice (and 1-D pooling with a stride, as planes of one row)."""
    x = np.random.Generator(np.random.PCG64(shape[3] + geom[1])).standard_normal(shape, dtype=np.float32)
    _check(B, op, x, *geom, what="wide %s %s %s" % (op, geom, shape))
    y = to_host(B.sws_pool2d_ex(0, to_gpu(x), geom[0], geom[1], geom[2], geom[3], (geom[4], geom[5], 0, geom[1] - 1),
                                B.SWS_DIV_REAL_CELLS, 1.0))
    ref, mag = oracle.pool2d_ex(oracle.OP_ADD, x, geom[0], geom[1], geom[2], geom[3], (geom[4], geom[5], 0, geom[1] - 1), True, 1.0)
    assert_within_tol(y, ref, mag, "wide pool2d_ex %s %s" % (geom, shape))


def test_wide_plane_falls_back(B):
    """Wide rows with the specialised geometries (these used to run on the direct-evaluation kernel)."""
    x = np.random.Generator(np.random.PCG64(8)).standard_normal((1, 2, 9, 3000), dtype=np.float32)
    _check(B, "max", x, 3, 3, 1, 1, 1, 1)
    _check(B, "add", x, 3, 3, 2, 2, 1, 1)


def test_tiny_planes(B):
    for shape in [(1, 1, 1, 1), (3, 1, 2, 2), (1, 2, 3, 1), (2, 2, 1, 9)]:
        x = np.random.Generator(np.random.PCG64(11)).standard_normal(shape, dtype=np.float32)
        _check(B, "add", x, 1, 1, 1, 1, 0, 0)
        if shape[2] >= 2 and shape[3] >= 2:
            _check(B, "max", x, 2, 2, 1, 1, 1, 1)


@pytest.mark.parametrize("stride", [1, 2])
def test_cfg3_full_size_every_plane(B, stride):
    """[32, 64, 112, 112], 3x3, pad 1, stride 1 and 2, at full size in one launch: all 2048
    planes against the oracle, every output; and the stride-2 result is the stride-1 result
    subsampled."""
    import torch
    x, _ = workloads.make(3)
    xg = to_gpu(x)
    for op in ("max", "add"):
        yg = B.sws_pool2d(OPS[op], xg, 3, 3, stride, stride, 1, 1, 1.0 / 9)
        y = to_host(yg)
        ref, mag = oracle.pool2d(OPS[op], x, 3, 3, stride, stride, 1, 1, 1.0 / 9)
        if op == "max":
            assert_bit_exact(y, ref, "cfg3 max s%d" % stride)
        else:
            assert_within_tol(y, ref, mag, "cfg3 avg s%d" % stride)
        if stride == 2:
            y1 = B.sws_pool2d(OPS[op], xg, 3, 3, 1, 1, 1, 1, 1.0 / 9)
            assert torch.equal(yg, y1[:, :, ::2, ::2])


EX_GEOMS = [  # kh, kw, sh, sw, (top, left, bottom, right)
    (3, 3, 1, 1, (1, 1, 1, 1)), (3, 3, 2, 2, (1, 1, 0, 0)), (3, 3, 2, 2, (0, 0, 1, 1)), (2, 2, 2, 2, (0, 0, 1, 1)),
    (3, 3, 1, 1, (2, 1, 0, 2)), (5, 5, 1, 1, (4, 2, 1, 3)), (7, 7, 1, 1, (0, 3, 6, 3)), (3, 3, 2, 2, (2, 1, 2, 2)),
    (4, 3, 2, 1, (1, 2, 3, 0)), (2, 5, 1, 3, (1, 4, 0, 2))]


@pytest.mark.parametrize("divisor", [0, 1])
@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("geom", EX_GEOMS)
@pytest.mark.parametrize("shape", [(3, 5, 37, 41), (2, 3, 112, 112), (1, 2, 8, 300)])
def test_four_sided_padding_and_real_cell_average(B, divisor, op, geom, shape):
    """sws_pool2d_ex: separate padding per side; ADD divided by the window's real cells."""
    kh, kw, sh, sw, pads = geom
    if divisor and op:
        pytest.skip("the divisor only applies to add")
    r = np.random.Generator(np.random.PCG64(kh * 100 + kw * 10 + sh + sum(pads) + shape[2]))
    x = r.standard_normal(shape, dtype=np.float32)
    scale = 1.0 if divisor else 1.0 / (kh * kw)
    y = to_host(B.sws_pool2d_ex(op, to_gpu(x), kh, kw, sh, sw, pads, divisor, scale))
    ref, mag = oracle.pool2d_ex(op, x, kh, kw, sh, sw, pads, bool(divisor), scale)
    if op == 0:
        assert_within_tol(y, ref, mag, "pool2d_ex %s div=%d" % (geom, divisor))
    else:
        assert_bit_exact(y, ref, "pool2d_ex %s op=%d" % (geom, op))


def test_pool2d_ex_equal_pads_match_pool2d_and_argument_checks(B):
    r = np.random.Generator(np.random.PCG64(77))
    x = to_gpu(r.standard_normal((2, 4, 56, 56), dtype=np.float32))
    a = to_host(B.sws_pool2d(0, x, 3, 3, 2, 2, 1, 1, 1 / 9))
    b = to_host(B.sws_pool2d_ex(0, x, 3, 3, 2, 2, (1, 1, 1, 1), B.SWS_DIV_SCALE, 1 / 9))
    assert np.array_equal(a, b)
    with pytest.raises(B.SwsError):
        B.sws_pool2d_ex(0, x, 3, 3, 1, 1, (3, 0, 0, 0))
    with pytest.raises(B.SwsError):
        B.sws_pool2d_ex(0, x, 3, 3, 1, 1, (0, 0, 0, 0), 5)


def test_more_than_2_to_the_32_elements(B):
    """349 952 planes of 112 x 112 (4.4e9 elements): plane offsets beyond 2^32 elements, for the
    specialised band kernel, the run-time separable kernel and the two pooling adjoints."""
    import torch
    planes = 349952                                                       # 5468 x 64
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * planes * 112 * 112 * 3.3:
        pytest.skip("not enough device memory")
    g = torch.Generator(device="cuda")
    g.manual_seed(41)
    x = torch.randn(planes // 64, 64, 112, 112, device="cuda", generator=g)
    flat = x.view(planes, 112, 112)
    sample = [0, 171195, 171196, 342392, 342393, planes - 1]              # around the 2^31- and 2^32-element marks
    xs = to_host(flat[sample]).reshape(1, len(sample), 112, 112)
    for kh, kw, sh, sw, ph, pw in ((3, 3, 2, 2, 1, 1), (4, 4, 4, 4, 0, 0)):
        y = B.sws_pool2d(1, x, kh, kw, sh, sw, ph, pw, 1.0)
        ref, _ = oracle.pool2d(oracle.OP_MAX, xs, kh, kw, sh, sw, ph, pw)
        got = to_host(y.view(planes, y.shape[2], y.shape[3])[sample])
        assert_bit_exact(got.reshape(ref.shape), ref, "big max pool %dx%d" % (kh, kw))
        del y
    gy = torch.randn(planes // 64, 64, 56, 56, device="cuda", generator=g)
    gx = B.sws_maxpool2d_grad(x, gy, 3, 3, 2, 2, 1, 1)
    gys = to_host(gy.view(planes, 56, 56)[sample]).reshape(1, len(sample), 56, 56)
    ref = oracle.maxpool2d_grad(xs, gys, 3, 3, 2, 2, 1, 1)
    mag = oracle.maxpool2d_grad(xs, np.abs(gys), 3, 3, 2, 2, 1, 1)
    assert_within_tol(to_host(gx.view(planes, 112, 112)[sample]).reshape(ref.shape), ref, mag, "big max pool adjoint")
    B.sws_avgpool2d_grad(gy, 112, 112, 3, 3, 2, 2, 1, 1, B.SWS_DIV_REAL_CELLS, 1.0, gx=gx)
    ref, mag = oracle.avgpool2d_grad(gys, 112, 112, 3, 3, 2, 2, 1, 1, True, 1.0)
    assert_within_tol(to_host(gx.view(planes, 112, 112)[sample]).reshape(ref.shape), ref, mag, "big average pool adjoint")
    del x, gy, gx
    torch.cuda.empty_cache()


SMALL_GEOMS = [(3, 3, 1, 1, 1, 1), (3, 3, 2, 2, 1, 1), (2, 2, 2, 2, 0, 0), (7, 7, 1, 1, 0, 0), (7, 7, 1, 1, 3, 3), (5, 3, 1, 2, 2, 0),
               (1, 1, 1, 1, 0, 0), (4, 4, 4, 4, 0, 0), (2, 5, 1, 3, 1, 4)]


@pytest.mark.parametrize("variant", [0, 32, 64])
@pytest.mark.parametrize("geom", SMALL_GEOMS)
@pytest.mark.parametrize("shape", [(3, 700, 7, 7), (2, 333, 14, 14), (5, 41, 5, 9), (1, 67, 16, 16), (2, 9, 1, 1), (1, 13, 3, 300),
                                   (1, 5, 32, 32), (1, 3, 33, 31)])
def test_small_planes(B, variant, geom, shape):
    """Planes of a few hundred elements, thousands of them: the small-plane kernel (several planes
    per workgroup), as the library chooses it, forced (option pool2d_variant 32, planes up to 1024
    elements) and switched off (64); a last workgroup with fewer planes; x off the 16-byte boundary."""
    import torch
    kh, kw, sh, sw, ph, pw = geom
    n, c, h, w = shape
    if h + 2 * ph < kh or w + 2 * pw < kw or ph >= kh or pw >= kw:
        pytest.skip("window does not fit")
    r = np.random.Generator(np.random.PCG64(kh * 100 + kw * 10 + h * 7 + w))
    x = r.standard_normal(shape, dtype=np.float32)
    B.sws_set_option("pool2d_variant", variant)
    try:
        for shift in (0, 1):
            xbuf = torch.zeros(x.size + 4, device="cuda")
            xs = xbuf[shift:shift + x.size].view(shape)
            xs.copy_(torch.from_numpy(x))
            for op in ("add", "max", "min"):
                scale = 1.0 / (kh * kw)
                y = to_host(B.sws_pool2d(OPS[op], xs, kh, kw, sh, sw, ph, pw, scale))
                ref, mag = oracle.pool2d(OPS[op], x, kh, kw, sh, sw, ph, pw, scale)
                what = "small planes %s %s %s variant %d shift %d" % (shape, geom, op, variant, shift)
                if op == "add":
                    assert_within_tol(y, ref, mag, what)
                else:
                    assert_bit_exact(y, ref, what)
    finally:
        B.sws_set_option("pool2d_variant", 0)


@pytest.mark.parametrize("divisor", [0, 1])
@pytest.mark.parametrize("geom", EX_GEOMS)
@pytest.mark.parametrize("shape", [(3, 500, 7, 7), (2, 99, 14, 14), (1, 30, 9, 20)])
def test_small_planes_four_sided_padding_and_real_cell_average(B, divisor, geom, shape):
    kh, kw, sh, sw, pads = geom
    r = np.random.Generator(np.random.PCG64(kh * 100 + kw * 10 + sh + sum(pads) + shape[2]))
    x = r.standard_normal(shape, dtype=np.float32)
    scale = 1.0 if divisor else 1.0 / (kh * kw)
    for op in ((0,) if divisor else (0, 1, 2)):
        y = to_host(B.sws_pool2d_ex(op, to_gpu(x), kh, kw, sh, sw, pads, divisor, scale))
        ref, mag = oracle.pool2d_ex(op, x, kh, kw, sh, sw, pads, bool(divisor), scale)
        if op == 0:
            assert_within_tol(y, ref, mag, "small pool2d_ex %s %s div=%d" % (shape, geom, divisor))
        else:
            assert_bit_exact(y, ref, "small pool2d_ex %s %s op=%d" % (shape, geom, op))



@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("geom", [(3, 1, 1), (3, 2, 1), (2, 2, 0), (5, 1, 2), (7, 1, 3), (9, 1, 4), (11, 1, 5), (13, 1, 6)])
@pytest.mark.parametrize("shape", [(2, 3, 37, 260), (1, 2, 20, 512), (1, 1, 9, 1000), (9, 1, 6, 480), (1, 2, 11, 244 + 240)])
def test_row_streaming_kernel_on_strips_of_wide_planes(B, op, geom, shape):
    """The same windows on planes wider than 256 columns: strips of 256 input columns whose end lanes only serve
    their neighbours (strip boundaries at multiples of 240, planes that end inside a strip or exactly on one, nine
    planes = a second round of eight).  Against the oracle and against the band kernel (option pool2d_variant 128);
    guard elements around y keep their value."""
    import torch
    k, s, p = geom
    n, c, h, w = shape
    rng = np.random.Generator(np.random.PCG64(2000 * k + 100 * s + h * w + n))
    x = rng.standard_normal(shape, dtype=np.float32)
    scale = 1.0 / (k * k)
    for ph in sorted({p, 0, k - 1}):
        if h + 2 * ph < k:
            continue
        ho, wo = (h + 2 * ph - k) // s + 1, (w + 2 * p - k) // s + 1
        buf = torch.full((n * c * ho * wo + 64,), 4321.0, device="cuda")
        yv = buf[32:32 + n * c * ho * wo].view(n, c, ho, wo)
        B.sws_pool2d(OPS[op], to_gpu(x), k, k, s, s, ph, p, scale, y=yv)
        y = to_host(yv)
        ref, mag = oracle.pool2d(OPS[op], x, k, k, s, s, ph, p, scale)
        what = "wide rows kernel %s %s ph=%d %s" % (op, geom, ph, shape)
        if op == "add":
            assert_within_tol(y, ref, mag, what)
        else:
            assert_bit_exact(y, ref, what)
        assert bool((buf[:32] == 4321.0).all()) and bool((buf[32 + n * c * ho * wo:] == 4321.0).all()), what
        B.sws_set_option("pool2d_variant", 128)
        try:
            other = to_host(B.sws_pool2d(OPS[op], to_gpu(x), k, k, s, s, ph, p, scale))
        finally:
            B.sws_set_option("pool2d_variant", 0)
        if op == "add":
            assert_within_tol(other, ref, mag, what + " (band kernel)")
        else:
            assert np.array_equal(y, other), what


@pytest.mark.parametrize("k,s", [(3, 1), (3, 2), (2, 2), (5, 1), (7, 1), (9, 1), (13, 1)])
@pytest.mark.parametrize("shape", [(2, 3, 30, 64), (1, 2, 17, 112), (3, 1, 9, 256), (1, 2, 21, 260), (1, 1, 15, 512), (2, 2, 56, 56)])
def test_real_cell_average_on_the_row_streaming_kernels(B, k, s, shape):
    """The average over the cells inside the plane (sws_pool2d_ex, SWS_DIV_REAL_CELLS) for the geometries of the
    row-streaming kernels, narrow planes and strips, with more and fewer rows of padding below than above; against
    the oracle and against the band kernel (option pool2d_variant 128)."""
    p = 0 if k == 2 else k // 2
    h = shape[2]
    r = np.random.Generator(np.random.PCG64(k * 10 + s + shape[3]))
    x = r.standard_normal(shape, dtype=np.float32)
    for pads in ((p, p, p, p), (p, p, 0, p), (0, p, p, p)):
        if h + pads[0] + pads[2] < k:
            continue
        if k == 2 and pads != (0, 0, 0, 0):
            continue
        y = to_host(B.sws_pool2d_ex(0, to_gpu(x), k, k, s, s, pads, B.SWS_DIV_REAL_CELLS, 1.0))
        ref, mag = oracle.pool2d_ex(0, x, k, k, s, s, pads, True, 1.0)
        assert_within_tol(y, ref, mag, "real-cell average k=%d s=%d pads=%s %s" % (k, s, pads, shape))
        B.sws_set_option("pool2d_variant", 128)
        try:
            other = to_host(B.sws_pool2d_ex(0, to_gpu(x), k, k, s, s, pads, B.SWS_DIV_REAL_CELLS, 1.0))
        finally:
            B.sws_set_option("pool2d_variant", 0)
        assert_within_tol(other, ref, mag, "band kernel, real-cell average k=%d s=%d pads=%s %s" % (k, s, pads, shape))


@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("k", [3, 5, 7, 9, 11, 13])
@pytest.mark.parametrize("shape", [(2, 3, 19, 65), (1, 2, 30, 111), (1, 9, 9, 149), (1, 1, 12, 255), (2, 1, 7, 257), (1, 2, 10, 301),
                                   (1, 1, 6, 483), (1, 1, 5, 242)])
def test_row_streaming_kernel_on_rows_not_a_multiple_of_4_long(B, op, k, shape):
    """Stride-1 windows on rows of 65 .. 483 elements with every remainder mod 4: the lane that straddles the end of a
    row takes the row's last four elements and keeps its own; rows start off the 16-byte boundaries.  Against the
    oracle (also the real-cell average) and against the band kernel; guard elements around y."""
    import torch
    p = k // 2
    n, c, h, w = shape
    rng = np.random.Generator(np.random.PCG64(3000 * k + h * w + n))
    x = rng.standard_normal(shape, dtype=np.float32)
    scale = 1.0 / (k * k)
    for ph in sorted({p, 0}):
        if h + 2 * ph < k:
            continue
        ho = h + 2 * ph - k + 1
        buf = torch.full((n * c * ho * w + 64,), 4321.0, device="cuda")
        yv = buf[32:32 + n * c * ho * w].view(n, c, ho, w)
        B.sws_pool2d(OPS[op], to_gpu(x), k, k, 1, 1, ph, p, scale, y=yv)
        y = to_host(yv)
        ref, mag = oracle.pool2d(OPS[op], x, k, k, 1, 1, ph, p, scale)
        what = "ragged rows %s k=%d ph=%d %s" % (op, k, ph, shape)
        if op == "add":
            assert_within_tol(y, ref, mag, what)
        else:
            assert_bit_exact(y, ref, what)
        assert bool((buf[:32] == 4321.0).all()) and bool((buf[32 + n * c * ho * w:] == 4321.0).all()), what
        B.sws_set_option("pool2d_variant", 128)
        try:
            other = to_host(B.sws_pool2d(OPS[op], to_gpu(x), k, k, 1, 1, ph, p, scale))
        finally:
            B.sws_set_option("pool2d_variant", 0)
        if op != "add":
            assert np.array_equal(y, other), what
    if op == "add":
        yr = to_host(B.sws_pool2d_ex(0, to_gpu(x), k, k, 1, 1, (p, p, p, p), B.SWS_DIV_REAL_CELLS, 1.0))
        ref, mag = oracle.pool2d_ex(0, x, k, k, 1, 1, (p, p, p, p), True, 1.0)
        assert_within_tol(yr, ref, mag, "ragged rows, real-cell average k=%d %s" % (k, shape))


@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("geom", [(3, 2, 1), (3, 2, 0), (2, 2, 0)])
@pytest.mark.parametrize("shape", [(2, 3, 19, 65), (1, 2, 30, 111), (1, 9, 9, 149), (1, 1, 12, 255), (2, 1, 7, 257), (1, 2, 10, 301),
                                   (1, 1, 6, 483), (1, 2, 21, 112), (1, 1, 9, 64), (1, 1, 8, 512), (3, 1, 5, 242)])
def test_row_streaming_kernel_stride_2_on_ragged_rows_and_without_padding(B, op, geom, shape):
    """Stride 2 on the strip form: rows with every remainder mod 4, and 3 x 3 without padding (the classic 3 x 3 / 2
    "valid" pooling), where the last lane of a row has one output or a window that ends on the row's last element.
    Against the oracle and the band kernel, guard elements around y."""
    import torch
    k, s, p = geom
    n, c, h, w = shape
    if w % 4 == 0 and geom != (3, 2, 0):
        pytest.skip("covered by the tests of the aligned rows")
    rng = np.random.Generator(np.random.PCG64(4000 * k + 10 * p + h * w + n))
    x = rng.standard_normal(shape, dtype=np.float32)
    scale = 1.0 / (k * k)
    for ph in sorted({p, 0, k - 1}):
        if h + 2 * ph < k:
            continue
        ho, wo = (h + 2 * ph - k) // s + 1, (w + 2 * p - k) // s + 1
        buf = torch.full((n * c * ho * wo + 64,), 4321.0, device="cuda")
        yv = buf[32:32 + n * c * ho * wo].view(n, c, ho, wo)
        B.sws_pool2d(OPS[op], to_gpu(x), k, k, s, s, ph, p, scale, y=yv)
        y = to_host(yv)
        ref, mag = oracle.pool2d(OPS[op], x, k, k, s, s, ph, p, scale)
        what = "stride 2 %s %s ph=%d %s" % (op, geom, ph, shape)
        if op == "add":
            assert_within_tol(y, ref, mag, what)
        else:
            assert_bit_exact(y, ref, what)
        assert bool((buf[:32] == 4321.0).all()) and bool((buf[32 + n * c * ho * wo:] == 4321.0).all()), what
        B.sws_set_option("pool2d_variant", 128)
        try:
            other = to_host(B.sws_pool2d(OPS[op], to_gpu(x), k, k, s, s, ph, p, scale))
        finally:
            B.sws_set_option("pool2d_variant", 0)
        if op != "add":
            assert np.array_equal(y, other), what
