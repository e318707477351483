"""GPU parity of sws_conv1d / sws_conv2d against the CPU oracle (Section 2.5: convolution
as a sliding dot product, no column matrix)."""
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
    yield binding
    binding.sws_set_option("conv1d_variant", 0)
    binding.sws_set_option("conv2d_variant", 0)


def _c1(B, x, w, stride=1, pad=0, dilation=1, groups=1, what=""):
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w), stride, pad, dilation, groups))
    ref, mag = oracle.conv1d(x, w, stride, pad, dilation, groups)
    return assert_within_tol(y, ref, mag, what)


def _c2(B, x, w, sh=1, sw=1, ph=0, pw=0, what=""):
    y = to_host(B.sws_conv2d(to_gpu(x), to_gpu(w), sh, sw, ph, pw))
    ref, mag = oracle.conv2d(x, w, sh, sw, ph, pw)
    return assert_within_tol(y, ref, mag, what)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("k", [1, 2, 3, 5, 11, 31, 51])
@pytest.mark.parametrize("length", [64, 1000, 4099])
def test_conv1d_single_channel(B, k, length):
    r = _rng(k * 1000 + length)
    x = (r.random((2, 1, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = r.standard_normal((1, 1, k), dtype=np.float32)
    _c1(B, x, w, what="k=%d L=%d" % (k, length))


@pytest.mark.parametrize("k", [1, 3, 5, 31, 33])
@pytest.mark.parametrize("channels,length", [(5, 700), (128, 300), (3, 4100)])
def test_conv1d_depthwise(B, k, channels, length):
    r = _rng(k * 77 + channels)
    x = (r.random((3, channels, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (r.standard_normal((channels, 1, k), dtype=np.float32) / np.sqrt(k)).astype(np.float32)
    _c1(B, x, w, groups=channels, what="dw k=%d C=%d" % (k, channels))


@pytest.mark.parametrize("cin,cout,k", [(64, 64, 3), (64, 64, 1), (32, 48, 5), (7, 5, 3), (64, 128, 3), (96, 64, 7),
                                         (32, 40, 3), (96, 64, 3), (40, 64, 3), (128, 64, 3)])
@pytest.mark.parametrize("length", [130, 1027])
def test_conv1d_dense(B, cin, cout, k, length):
    r = _rng(cin * 31 + cout + k)
    x = r.standard_normal((2, cin, length), dtype=np.float32)
    w = (r.standard_normal((cout, cin, k), dtype=np.float32) * np.sqrt(2.0 / (cin * k))).astype(np.float32)
    _c1(B, x, w, what="dense %d->%d k=%d" % (cin, cout, k))


@pytest.mark.parametrize("stride,pad,dilation,groups", [(2, 0, 1, 1), (1, 2, 1, 1), (1, 0, 3, 1), (3, 4, 2, 2),
                                                       (1, 1, 1, 4), (2, 5, 4, 8)])
def test_conv1d_stride_pad_dilation_groups(B, stride, pad, dilation, groups):
    r = _rng(stride * 1000 + pad * 100 + dilation * 10 + groups)
    x = r.standard_normal((2, 8, 333), dtype=np.float32)
    w = r.standard_normal((16, 8 // groups, 5), dtype=np.float32)
    _c1(B, x, w, stride, pad, dilation, groups, what=str((stride, pad, dilation, groups)))


@pytest.mark.parametrize("dilation", [2, 3, 4, 5, 8, 16, 33, 64])
@pytest.mark.parametrize("k", [2, 3, 17, 51])
def test_conv1d_dilated_single_channel(B, dilation, k):
    """Taps spaced `dilation` apart on one long sequence (the shape of the dilated-kernel
    experiment of the Experiments section); several tiles and a ragged tail."""
    length = (k - 1) * dilation + 2500
    r = _rng(dilation * 100 + k)
    x = (r.random((2, 1, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (r.standard_normal((1, 1, k), dtype=np.float32) / np.sqrt(k)).astype(np.float32)
    _c1(B, x, w, dilation=dilation, what="dil=%d k=%d" % (dilation, k))


@pytest.mark.parametrize("dilation,k,pad", [(2, 5, 4), (8, 51, 200), (7, 9, 3), (64, 4, 100), (16, 33, 256)])
def test_conv1d_dilated_depthwise_padded(B, dilation, k, pad):
    r = _rng(dilation * 7 + k)
    x = r.standard_normal((2, 6, 1500), dtype=np.float32)
    w = (r.standard_normal((12, 1, k), dtype=np.float32) / np.sqrt(k)).astype(np.float32)   # two outputs per input channel
    _c1(B, x, w, pad=pad, dilation=dilation, groups=6, what="dw dil=%d k=%d pad=%d" % (dilation, k, pad))


def test_conv1d_dilated_short_rows_and_fallbacks(B):
    r = _rng(99)
    # rows shorter than one tile, span equal to the row, and a dilation beyond the tuned kernel's range
    for length, k, dil in [(9, 3, 4), (101, 51, 2), (40, 2, 39), (700, 3, 100), (5000, 64, 64)]:
        x = r.standard_normal((3, 2, length), dtype=np.float32)
        w = r.standard_normal((2, 1, k), dtype=np.float32)
        _c1(B, x, w, dilation=dil, groups=2, what="L=%d k=%d dil=%d" % (length, k, dil))


def test_conv1d_dilated_integer_valued_bit_exact_and_variants_agree(B):
    x = workloads.integer_valued((2, 3, 3000), -8, 8, seed=5)
    w = workloads.integer_valued((3, 1, 21), -4, 4, seed=6)
    ref, _ = oracle.conv1d(x, w, 1, 80, 8, 3)
    for variant in (0, 4, 1):
        B.sws_set_option("conv1d_variant", variant)
        y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w), 1, 80, 8, 3))
        assert np.array_equal(y.astype(np.float64), ref), "variant %d" % variant
    B.sws_set_option("conv1d_variant", 0)


def test_conv1d_integer_valued_bit_exact(B):
    x = workloads.integer_valued((2, 6, 500), -8, 8, seed=1)
    w = workloads.integer_valued((4, 6, 5), -4, 4, seed=2)
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w)))
    ref, _ = oracle.conv1d(x, w)
    assert np.array_equal(y.astype(np.float64), ref)
    wd = workloads.integer_valued((6, 1, 31), -4, 4, seed=3)
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(wd), groups=6))
    ref, _ = oracle.conv1d(x, wd, groups=6)
    assert np.array_equal(y.astype(np.float64), ref)


@pytest.mark.parametrize("cin,cout,kh,kw", [(64, 64, 3, 3), (16, 32, 3, 3), (3, 8, 5, 5), (64, 64, 1, 1), (8, 8, 3, 1), (5, 7, 2, 4)])
@pytest.mark.parametrize("h,w_,geom", [(56, 56, (1, 1, 1, 1)), (19, 33, (1, 1, 0, 0)), (30, 17, (2, 2, 1, 1)), (14, 14, (1, 2, 2, 0))])
def test_conv2d(B, cin, cout, kh, kw, h, w_, geom):
    sh, sw, ph, pw = geom
    if kh > h + 2 * ph or kw > w_ + 2 * pw:
        pytest.skip("kernel larger than image")
    r = _rng(cin + cout * 3 + kh * 5 + kw * 7 + h)
    x = np.maximum(r.standard_normal((2, cin, h, w_), dtype=np.float32), 0).astype(np.float32)
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.sqrt(2.0 / (cin * kh * kw))).astype(np.float32)
    _c2(B, x, w, sh, sw, ph, pw, what=str((cin, cout, kh, kw, h, w_, geom)))


@pytest.mark.parametrize("cin,cout,kh,kw,h,w_,ph,pw", [
    (12, 20, 3, 3, 21, 25, 1, 1),      # Cin % 8 != 0, % 4 == 0: scalar-read matrix kernel, 4-channel blocks
    (16, 70, 5, 5, 30, 31, 2, 2),      # 25 taps: scalar-read matrix kernel; Cout not a multiple of 64
    (32, 64, 1, 7, 9, 300, 0, 3),      # wide rows: column tiles; 7 taps through the generic tap loop
    (8, 8, 3, 3, 5, 5, 1, 1),          # a single small tile
    (24, 33, 2, 2, 17, 40, 0, 1),      # even tap count, Cout not a multiple of 32
    (64, 64, 6, 6, 20, 20, 2, 2),      # 36 taps
    (64, 64, 7, 7, 20, 20, 3, 3),      # 49 taps: beyond the matrix kernels, direct evaluation
    (32, 32, 5, 5, 28, 28, 2, 2),      # 25 taps, Cin % 8 == 0: five chunks of one kernel row each
    (8, 16, 4, 2, 19, 23, 1, 0),       # 8 taps in one launch; (16, 16, 4, 4): rows in chunks of two
    (16, 16, 4, 4, 19, 23, 1, 2),
    (64, 48, 1, 3, 11, 40, 0, 1),      # 1 x 3 taps, Cin % 32 == 0: four channel blocks per barrier pair
    (32, 64, 1, 3, 3, 500, 0, 1),      # the same on wide rows (column tiles)
])
def test_conv2d_kernel_selection_paths(B, cin, cout, kh, kw, h, w_, ph, pw):
    r = _rng(cin * 7 + cout + kh * 3 + kw)
    x = r.standard_normal((3, cin, h, w_), dtype=np.float32)
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.sqrt(2.0 / (cin * kh * kw))).astype(np.float32)
    _c2(B, x, w, 1, 1, ph, pw, what=str((cin, cout, kh, kw, h, w_)))


@pytest.mark.parametrize("cin,cout,kh,kw,h,w_,sh,sw,ph,pw", [
    (64, 64, 3, 3, 56, 56, 2, 2, 1, 1),     # ResNet-style downsampling: tall input tiles (128-segment staging plan)
    (64, 128, 1, 1, 56, 56, 2, 2, 0, 0),    # 1 x 1 projection with stride 2
    (32, 64, 3, 3, 33, 47, 2, 1, 1, 0),     # stride along H only, ragged sizes
    (16, 16, 3, 3, 20, 300, 1, 3, 1, 1),    # wide rows (column tiles), stride 3 along W
    (8, 24, 2, 2, 64, 64, 2, 2, 0, 0),      # non-overlapping 2 x 2 patches
    (64, 64, 3, 3, 112, 112, 2, 2, 1, 1),   # input tile too tall for the staging plan: direct evaluation
])
def test_conv2d_strided(B, cin, cout, kh, kw, h, w_, sh, sw, ph, pw):
    r = _rng(cin + cout + kh * 11 + h + sh * 3 + sw)
    x = r.standard_normal((2, cin, h, w_), dtype=np.float32)
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.sqrt(2.0 / (cin * kh * kw))).astype(np.float32)
    _c2(B, x, w, sh, sw, ph, pw, what=str((cin, cout, kh, kw, h, w_, sh, sw, ph, pw)))


@pytest.mark.parametrize("cin,cout,k,dilation,pad,stride,length", [
    (16, 16, 51, 8, 200, 1, 3000),     # a very long dilated kernel on few channels: six chunks of taps
    (16, 16, 51, 8, 0, 1, 1000),
    (32, 40, 11, 1, 5, 1, 1500),       # 11 taps: two chunks
    (8, 8, 10, 3, 13, 2, 700),         # chunks + dilation + stride
    (64, 64, 3, 4, 4, 1, 2000),        # three dilated taps in one launch
    (24, 16, 31, 2, 30, 1, 900),
])
def test_conv1d_dense_dilated_and_long_kernels(B, cin, cout, k, dilation, pad, stride, length):
    r = _rng(cin + cout + k * 3 + dilation)
    x = r.standard_normal((2, cin, length), dtype=np.float32)
    w = (r.standard_normal((cout, cin, k), dtype=np.float32) * np.sqrt(2.0 / (cin * k))).astype(np.float32)
    _c1(B, x, w, stride=stride, pad=pad, dilation=dilation, what="dense k=%d d=%d" % (k, dilation))


@pytest.mark.parametrize("cin,cout,groups,k,dilation,pad", [
    (15, 15, 1, 51, 8, 200),      # odd channel counts, long dilated kernel: the vector-ALU kernel sums over input channels
    (3, 5, 1, 7, 1, 3),
    (12, 8, 4, 9, 2, 5),          # grouped: three input channels per output channel
    (16, 16, 1, 31, 1, 15),       # few dense channels, many taps
    (6, 6, 2, 64, 1, 0),
    (10, 4, 2, 2, 64, 10),
])
def test_conv1d_few_channels_on_the_vector_alu(B, cin, cout, groups, k, dilation, pad):
    r = _rng(cin * 3 + cout + groups + k)
    x = r.standard_normal((3, cin, 2600), dtype=np.float32)
    w = (r.standard_normal((cout, cin // groups, k), dtype=np.float32) * np.sqrt(2.0 / (cin // groups * k))).astype(np.float32)
    for variant in (0, 6, 1):
        B.sws_set_option("conv1d_variant", variant)
        try:
            _c1(B, x, w, pad=pad, dilation=dilation, groups=groups, what="few %d->%d g%d k%d d%d variant %d" % (cin, cout, groups, k, dilation, variant))
        finally:
            B.sws_set_option("conv1d_variant", 0)


@pytest.mark.parametrize("cin,cout,groups,k,dilation,pad", [
    (4, 4, 4, 65, 1, 0), (4, 8, 4, 127, 1, 63), (2, 2, 2, 200, 1, 10), (3, 3, 3, 70, 3, 100), (6, 4, 2, 80, 1, 7),
    (5, 3, 1, 129, 2, 128),
])
def test_conv1d_kernels_longer_than_64_taps_run_as_chunks(B, cin, cout, groups, k, dilation, pad):
    r = _rng(cin + cout * 5 + k)
    x = r.standard_normal((2, cin, 3500), dtype=np.float32)
    w = (r.standard_normal((cout, cin // groups, k), dtype=np.float32) / np.sqrt(cin // groups * k)).astype(np.float32)
    _c1(B, x, w, pad=pad, dilation=dilation, groups=groups, what="long k=%d d=%d g=%d" % (k, dilation, groups))


@pytest.mark.parametrize("cin,cout,groups,k,stride,pad", [
    (1, 64, 1, 10, 5, 0),         # one input channel fanned out to many, stride 5 (a raw-waveform front end)
    (6, 6, 6, 3, 2, 1),           # depthwise, stride 2
    (4, 8, 4, 7, 3, 3),
    (12, 8, 4, 9, 2, 4),          # grouped, three input channels per output channel
    (5, 7, 1, 64, 7, 10),         # odd dense channels, long kernel, stride 7
    (3, 3, 3, 2, 64, 0),          # stride larger than the kernel
    (2, 2, 2, 5, 17, 2),
])
def test_conv1d_strided_thin_and_grouped(B, cin, cout, groups, k, stride, pad):
    r = _rng(cin * 7 + cout + k * 3 + stride)
    x = r.standard_normal((3, cin, 5000), dtype=np.float32)
    w = (r.standard_normal((cout, cin // groups, k), dtype=np.float32) / np.sqrt(cin // groups * k)).astype(np.float32)
    for variant in (0, 7, 1):
        B.sws_set_option("conv1d_variant", variant)
        try:
            _c1(B, x, w, stride=stride, pad=pad, groups=groups, what="strided %d->%d g%d k%d s%d variant %d" % (cin, cout, groups, k, stride, variant))
        finally:
            B.sws_set_option("conv1d_variant", 0)


@pytest.mark.parametrize("stride,k,pad", [(2, 3, 1), (3, 5, 2), (2, 1, 0), (4, 9, 4)])
def test_conv1d_dense_strided(B, stride, k, pad):
    r = _rng(stride * 10 + k)
    x = r.standard_normal((3, 32, 1500), dtype=np.float32)
    w = (r.standard_normal((48, 32, k), dtype=np.float32) * np.sqrt(2.0 / (32 * k))).astype(np.float32)
    _c1(B, x, w, stride=stride, pad=pad, what="dense stride=%d k=%d" % (stride, k))


@pytest.mark.parametrize("cin,cout,kh,kw,ph,pw", [(32, 32, 5, 5, 2, 2), (16, 16, 4, 4, 1, 2), (8, 8, 6, 3, 0, 1), (64, 64, 7, 7, 3, 3)])
def test_conv2d_chunks_of_kernel_rows(B, cin, cout, kh, kw, ph, pw):
    """Kernels of more than 9 taps as a chain of launches over whole kernel rows, each adding to y
    (forced here also where the one-pass kernel would be chosen)."""
    r = _rng(cin + kh * 13 + kw)
    x = r.standard_normal((2, cin, 30, 41), dtype=np.float32)
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.sqrt(2.0 / (cin * kh * kw))).astype(np.float32)
    B.sws_set_option("conv2d_variant", 6)
    try:
        _c2(B, x, w, 1, 1, ph, pw, what="row chunks %dx%d" % (kh, kw))
    finally:
        B.sws_set_option("conv2d_variant", 0)


@pytest.mark.parametrize("cin,cout,kh,kw,h,w_,sh,sw,ph,pw", [
    (3, 64, 7, 7, 64, 64, 2, 2, 3, 3),       # a ResNet stem: three input channels (a zero-padded channel block), seven row chunks
    (3, 24, 11, 11, 67, 67, 4, 4, 2, 2),     # an AlexNet stem: rows wider than 9 taps -> runs of taps of each row
    (16, 16, 2, 12, 20, 50, 1, 1, 1, 6),     # two rows of twelve taps
    (5, 7, 3, 3, 19, 23, 1, 1, 1, 1),        # odd channel counts on both sides
    (13, 9, 1, 1, 10, 10, 1, 1, 0, 0),
    (12, 8, 3, 10, 15, 40, 2, 1, 1, 0),      # 12 channels with strides: no block-of-4 kernel
])
def test_conv2d_any_channel_count_and_wide_kernels(B, cin, cout, kh, kw, h, w_, sh, sw, ph, pw):
    r = _rng(cin * 3 + cout + kh * 11 + kw)
    x = r.standard_normal((2, cin, h, w_), dtype=np.float32)
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.sqrt(2.0 / (cin * kh * kw))).astype(np.float32)
    _c2(B, x, w, sh, sw, ph, pw, what=str((cin, cout, kh, kw, h, w_, sh, sw, ph, pw)))
    xi = workloads.integer_valued((1, cin, h, w_), -3, 3, cin + kh)
    wi = workloads.integer_valued((cout, cin, kh, kw), -2, 2, cout + kw)
    y = to_host(B.sws_conv2d(to_gpu(xi), to_gpu(wi), sh, sw, ph, pw))
    ref, _ = oracle.conv2d(xi, wi, sh, sw, ph, pw)
    assert np.array_equal(y.astype(np.float64), ref)


@pytest.mark.parametrize("variant", [1, 3, 8, 10, 12, 14])
def test_conv2d_variants_agree_with_oracle(B, variant):
    """The direct-evaluation kernel (1), the 4-wavefront scalar-read matrix kernel (3), and the
    channel-fastest matrix kernel forced to 8 / 10 / 12 / 14 wavefronts per workgroup."""
    r = _rng(variant)
    x = r.standard_normal((2, 32, 24, 24), dtype=np.float32)
    w = (r.standard_normal((64, 32, 3, 3), dtype=np.float32) * 0.06).astype(np.float32)
    B.sws_set_option("conv2d_variant", variant)
    try:
        _c2(B, x, w, 1, 1, 1, 1, what="variant %d" % variant)
    finally:
        B.sws_set_option("conv2d_variant", 0)


def test_conv1d_dense_long_kernel_and_padding(B):
    """Dense channels with k = 9 (largest single-pass tap count) and padding, ragged length."""
    r = _rng(99)
    x = r.standard_normal((3, 16, 2051), dtype=np.float32)
    w = (r.standard_normal((24, 16, 9), dtype=np.float32) * 0.1).astype(np.float32)
    _c1(B, x, w, pad=4, what="dense k=9 pad=4")
    w = (r.standard_normal((24, 16, 11), dtype=np.float32) * 0.1).astype(np.float32)
    _c1(B, x, w, pad=5, what="dense k=11 pad=5")


def test_conv2d_integer_valued_bit_exact(B):
    x = workloads.integer_valued((2, 5, 20, 23), -8, 8, seed=4)
    w = workloads.integer_valued((6, 5, 3, 3), -4, 4, seed=5)
    y = to_host(B.sws_conv2d(to_gpu(x), to_gpu(w), 1, 1, 1, 1))
    ref, _ = oracle.conv2d(x, w, 1, 1, 1, 1)
    assert np.array_equal(y.astype(np.float64), ref)


STREAM_2D = [  # N, Cout, H, W, ph, pw
    (2, 64, 20, 20, 1, 1), (1, 64, 56, 56, 1, 1), (3, 64, 7, 9, 1, 1), (2, 64, 33, 62, 1, 1), (1, 128, 12, 40, 0, 0),
    (2, 64, 5, 30, 2, 2), (1, 64, 3, 3, 1, 1), (5, 128, 14, 14, 1, 0), (1, 64, 1, 60, 1, 1), (4, 64, 9, 31, 0, 1),
    (1, 64, 40, 5, 2, 0), (37, 64, 6, 6, 1, 1)]


@pytest.mark.parametrize("geom", STREAM_2D)
def test_streaming_kernel_3x3(B, geom):
    """The weight-stationary streaming kernel (64 input channels, 3 x 3, stride 1), forced on small problems
    (option conv2d_variant 17): images narrower and wider than a position block, blocks that span several
    rows, several images and output-channel tiles per run, every padding below the kernel size, runs that
    are empty.  Integer-valued data in the same call: every fp32 partial sum is exact, so the result must
    equal the oracle's bit for bit whatever the order of the four partial sums."""
    n, cout, h, w, ph, pw = geom
    r = _rng(sum(geom) * 7 + h)
    x = r.standard_normal((n, 64, h, w), dtype=np.float32)
    wt = (r.standard_normal((cout, 64, 3, 3), dtype=np.float32) * 0.06).astype(np.float32)
    xi = workloads.integer_valued((n, 64, h, w), -4, 4, seed=h * w)
    wi = workloads.integer_valued((cout, 64, 3, 3), -3, 3, seed=cout)
    for variant in (17, 18):                          # fp32 matrix instructions; bf16 ones with split operands
        B.sws_set_option("conv2d_variant", variant)
        try:
            _c2(B, x, wt, 1, 1, ph, pw, what="stream 3x3 %s variant %d" % (geom, variant))
            y = to_host(B.sws_conv2d(to_gpu(xi), to_gpu(wi), 1, 1, ph, pw))
        finally:
            B.sws_set_option("conv2d_variant", 0)
        ref, _ = oracle.conv2d(xi, wi, 1, 1, ph, pw)
        assert np.array_equal(y.astype(np.float64), ref), "stream 3x3 integer-valued %s variant %d" % (geom, variant)


@pytest.mark.parametrize("geom", [(2, 64, 34, 0), (1, 64, 500, 1), (3, 128, 1000, 2), (16, 64, 4096, 0), (5, 64, 3, 1),
                                  (1, 64, 66, 1), (2, 64, 32, 1), (7, 64, 95, 2)])
def test_streaming_kernel_1d(B, geom):
    """The same kernel on 1-D rows (1 x 3): lines are 32-column chunks of the padded row."""
    n, cout, length, pad = geom
    r = _rng(sum(geom) + 3)
    x = r.standard_normal((n, 64, length), dtype=np.float32)
    wt = (r.standard_normal((cout, 64, 3), dtype=np.float32) * 0.1).astype(np.float32)
    xi = workloads.integer_valued((n, 64, length), -4, 4, seed=length)
    wi = workloads.integer_valued((cout, 64, 3), -3, 3, seed=cout + 1)
    B.sws_set_option("conv2d_variant", 17)
    try:
        _c1(B, x, wt, pad=pad, what="stream 1x3 %s" % (geom,))
        y = to_host(B.sws_conv1d(to_gpu(xi), to_gpu(wi), 1, pad))
    finally:
        B.sws_set_option("conv2d_variant", 0)
    ref, _ = oracle.conv1d(xi, wi, 1, pad)
    assert np.array_equal(y.astype(np.float64), ref), "stream 1x3 integer-valued %s" % (geom,)


def test_streaming_kernel_against_tile_kernel_full_size(B):
    """cfg 4 on all three matrix-core kernels (option 2 switches the streaming one off and leaves the tile
    kernel with 128-bit operand reads; 16 also switches that one off, leaving the scalar-read kernel): each
    within tolerance of the oracle."""
    x, w = workloads.make(4)
    ref, mag = oracle.conv2d(x, w, 1, 1, 1, 1)
    xg, wg = to_gpu(x), to_gpu(w)
    assert_within_tol(to_host(B.sws_conv2d(xg, wg, 1, 1, 1, 1)), ref, mag, "cfg4 streaming kernel")
    for variant, name in ((2, "tile kernel"), (16, "scalar-read kernel"), (18, "streaming kernel, split bf16 operands")):
        B.sws_set_option("conv2d_variant", variant)
        try:
            yt = to_host(B.sws_conv2d(xg, wg, 1, 1, 1, 1))
        finally:
            B.sws_set_option("conv2d_variant", 0)
        worst = assert_within_tol(yt, ref, mag, "cfg4 " + name)
        assert worst < 2e-6, "cfg4 %s: worst error ratio %g" % (name, worst)


def test_split_operand_kernel_carries_every_bit(B):
    """Inputs and weights whose magnitudes spread over six decades and whose mantissas use all 24 bits:
    the bf16 x 3 evaluation must stay at fp32 accuracy (each operand is the exact sum of its three pieces;
    only products below 2^-24 of a term are dropped)."""
    r = _rng(4242)
    x = (r.standard_normal((2, 64, 24, 30)) * 10.0 ** r.uniform(-3, 3, (2, 64, 24, 30))).astype(np.float32)
    w = (r.standard_normal((64, 64, 3, 3)) * 10.0 ** r.uniform(-3, 3, (64, 64, 3, 3))).astype(np.float32)
    ref, mag = oracle.conv2d(x, w, 1, 1, 1, 1)
    worst = {}
    for variant in (17, 18):
        B.sws_set_option("conv2d_variant", variant)
        try:
            y = to_host(B.sws_conv2d(to_gpu(x), to_gpu(w), 1, 1, 1, 1))
        finally:
            B.sws_set_option("conv2d_variant", 0)
        worst[variant] = assert_within_tol(y, ref, mag, "wide-range data, variant %d" % variant)
    assert worst[18] < 1e-6 and worst[18] < 4 * worst[17] + 1e-7, worst


def test_cfg1_correlation_full_size(B):
    """N = 1,048,576, 5-tap correlation."""
    x, w = workloads.make(1)
    worst = _c1(B, x, w, what="cfg1 corr")
    assert worst < 1e-6


def test_cfg2_conv1d_full_size(B):
    """[16, 64, 4096] x [64, 64, 3], every output checked."""
    x, w = workloads.make(2)
    _c1(B, x, w, what="cfg2 conv1d")


def test_cfg4_conv2d_full_size(B):
    """[32, 64, 56, 56] x [64, 64, 3, 3], pad 1: one launch, all 32 images against the oracle,
    every one of the 6,422,528 outputs (576 terms each)."""
    x, w = workloads.make(4)
    workloads.check_clean(x)
    y = to_host(B.sws_conv2d(to_gpu(x), to_gpu(w), 1, 1, 1, 1))
    ref, mag = oracle.conv2d(x, w, 1, 1, 1, 1)
    worst = assert_within_tol(y, ref, mag, "cfg4 conv2d")
    assert worst < 2e-6


def test_conv2d_more_than_2_to_the_32_elements(B):
    """22 000 images of [64, 56, 56] (4.4e9 elements): image offsets beyond 2^32 elements in the matrix kernel
    and in both adjoints."""
    import torch
    n = 22000
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * n * 64 * 56 * 56 * 3.3:
        pytest.skip("not enough device memory")
    g = torch.Generator(device="cuda")
    g.manual_seed(43)
    x = torch.randn(n, 64, 56, 56, device="cuda", generator=g)
    w = (_rng(44).standard_normal((64, 64, 3, 3), dtype=np.float32) * np.float32(0.06)).astype(np.float32)
    y = B.sws_conv2d(x, to_gpu(w), 1, 1, 1, 1)
    sample = [0, 10699, 10700, 21399, 21400, n - 1]                       # around the 2^31- and 2^32-element marks
    for i in sample:
        ref, mag = oracle.conv2d(to_host(x[i:i + 1]), w, 1, 1, 1, 1)
        assert_within_tol(to_host(y[i:i + 1]), ref, mag, "big conv2d image %d" % i)
    gx = B.sws_conv2d_grad_input(y, to_gpu(w), 56, 56, 1, 1, 1, 1)
    for i in (0, 21400, n - 1):
        ref, mag = oracle.conv2d_grad_input(to_host(y[i:i + 1]), w, 56, 56, 1, 1, 1, 1)
        assert_within_tol(to_host(gx[i:i + 1]), ref, mag, "big conv2d grad-input image %d" % i)
    del gx
    # grad-weight sums over every image: compare with the sum over the same three images given alone
    idx = torch.tensor([0, 21400, n - 1], device="cuda")
    xs, ys = x[idx].contiguous(), y[idx].contiguous()
    y.zero_()
    y[idx] = ys                                                           # gradients only at the three images
    gw = to_host(B.sws_conv2d_grad_weight(x, y, 3, 3, 1, 1, 1, 1))
    ref, mag = oracle.conv2d_grad_weight(to_host(xs), to_host(ys), 3, 3, 1, 1, 1, 1)
    assert_within_tol(gw, ref, mag, "big conv2d grad-weight")
    del x, y
    torch.cuda.empty_cache()


# Dense 1-D layers of 32 / 64 input channels: the split-operand kernel that streams the input from memory
# (bf16 matrix cores, fp32 accuracy).  B, Cin, L, Cout, k, pad
SPLIT_1D = [(2, 64, 500, 64, 3, 0), (3, 64, 1000, 96, 3, 1), (1, 32, 77, 32, 3, 2), (2, 32, 300, 160, 5, 2), (4, 64, 33, 32, 1, 0),
            (1, 64, 5, 64, 3, 1), (16, 64, 4096, 64, 3, 0), (5, 64, 31, 64, 3, 40), (2, 32, 2000, 32, 5, 0), (300, 64, 40, 64, 3, 1)]


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("case", SPLIT_1D)
def test_conv1d_dense_split_operands(B, case, integer):
    b, cin, length, cout, k, pad = case
    if integer:
        x = workloads.integer_valued((b, cin, length), -6, 6, 1)
        w = workloads.integer_valued((cout, cin, k), -4, 4, 2)
    else:
        r = _rng(700 + cin + length + k)
        x = r.standard_normal((b, cin, length), dtype=np.float32)
        w = (r.standard_normal((cout, cin, k)) / np.sqrt(cin * k)).astype(np.float32)
    ref, mag = oracle.conv1d(x, w, 1, pad, 1, 1)
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w), 1, pad, 1, 1))
    B.sws_set_option("conv1d_variant", 3)                        # the fp32-instruction tile kernel
    try:
        z = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w), 1, pad, 1, 1))
    finally:
        B.sws_set_option("conv1d_variant", 0)
    if integer:
        assert np.array_equal(y.astype(np.float64), ref) and np.array_equal(z.astype(np.float64), ref), str(case)
    else:
        worst = assert_within_tol(y, ref, mag, "split conv1d %s" % (case,))
        assert worst < 2e-6, (case, worst)                       # fp32 accuracy, not bf16's
        assert_within_tol(z, ref, mag, "tile conv1d %s" % (case,))


def test_conv1d_dense_split_operands_carry_every_bit(B):
    """x = 1 + k 2^-23 against weights of +-1 that cancel the ones: what is left lives in the third bf16 piece."""
    r = _rng(71)
    x = (1.0 + r.integers(0, 128, size=(2, 64, 300)) * 2.0 ** -23).astype(np.float32)
    w = np.where(r.integers(0, 2, size=(64, 64, 3)) > 0, 1.0, -1.0).astype(np.float32)
    ref, mag = oracle.conv1d(x, w, 1, 1, 1, 1)
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w), 1, 1, 1, 1))
    assert_within_tol(y, ref, mag, "low bits", tol=2e-7)
