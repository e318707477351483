"""Seeded random sweeps of shapes against the oracle: row lengths around tile seams, row counts
that move the output alignment, windows, pads, strides, dilations and channel counts drawn at
random (fixed seeds, so every run sees the same cases)."""
import numpy as np
import pytest

import oracle
from parity_util import assert_bit_exact, assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    return binding


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _near_seams(r, w, lo_max=6000):
    """An output length that sits on, just before or just after a multiple of the tile's outputs."""
    tout = max(16, (1024 - (w - 1)) & ~15)
    base = int(r.integers(1, max(2, lo_max // tout))) * tout
    return max(1, base + int(r.integers(-20, 21)))


@pytest.mark.parametrize("seed", range(40))
def test_slide1d_random(B, seed):
    r = _rng(7000 + seed)
    w = int(r.choice([1, 2, 3, 4, 5, 7, 9, 15, 16, 17, 33, 64, 100, 255, 256, 511, 700, 850, 851, 961, 1100]))
    lo = _near_seams(r, min(w, 961))
    rows = int(r.integers(1, 9))
    x = (r.random((rows, lo + w - 1), dtype=np.float32) * 2 - 1).astype(np.float32)
    op = int(r.integers(0, 3))
    scale = float(r.choice([1.0, 1.0 / w, 0.37]))
    y = to_host(B.sws_slide1d(op, to_gpu(x), w, scale))
    ref, mag = oracle.slide1d(op, x, w, scale)
    what = "seed %d: op %d w %d rows %d lo %d" % (seed, op, w, rows, lo)
    if op == 0:
        assert_within_tol(y, ref, mag, what)
    else:
        assert_bit_exact(y, ref, what)


@pytest.mark.parametrize("seed", range(30))
def test_slide1d_padded_random(B, seed):
    r = _rng(7100 + seed)
    w = int(r.choice([1, 2, 3, 5, 8, 16, 31, 64, 255, 600, 961]))
    length = int(r.integers(max(2, w // 2), 5000))
    mode = int(r.integers(0, 4))
    cap = length - 1 if mode == 1 else (length if mode == 2 else 2 * w)
    pl, pr = int(r.integers(0, min(cap, 2 * w) + 1)), int(r.integers(0, min(cap, 2 * w) + 1))
    if length + pl + pr < w:
        pl = min(cap, w)
        pr = min(cap, w)
    if length + pl + pr < w:
        pytest.skip("window longer than the extended row")
    rows = int(r.integers(1, 6))
    x = r.standard_normal((rows, length), dtype=np.float32)
    op = int(r.integers(0, 3))
    y = to_host(B.sws_slide1d_padded(op, to_gpu(x), w, pl, pr, mode, 0.5))
    ref, mag = oracle.slide1d_padded(op, x, w, pl, pr, mode, 0.5)
    what = "seed %d: op %d w %d len %d pads (%d,%d) mode %d" % (seed, op, w, length, pl, pr, mode)
    if op == 0:
        assert_within_tol(y, ref, mag, what)
    else:
        assert_bit_exact(y, ref, what)


@pytest.mark.parametrize("seed", range(40))
def test_conv1d_random(B, seed):
    r = _rng(7200 + seed)
    kind = seed % 4
    if kind == 0:                                   # depthwise / single channel, taps adjacent
        c, mult, k, dil, stride = int(r.integers(1, 9)), int(r.integers(1, 3)), int(r.integers(1, 200)), 1, 1
        cin, cout, groups = c, c * mult, c
    elif kind == 1:                                 # depthwise, dilated
        c, k, dil, stride = int(r.integers(1, 6)), int(r.integers(2, 40)), int(r.integers(2, 65)), 1
        cin, cout, groups = c, c, c
    elif kind == 2:                                 # dense on the matrix cores: strides, dilation, long kernels
        cin, cout = 8 * int(r.integers(1, 9)), int(r.integers(1, 100))
        k, dil, stride, groups = int(r.integers(1, 30)), int(r.integers(1, 5)), int(r.integers(1, 4)), 1
    else:                                           # anything: grouped, odd channel counts, strides
        groups = int(r.choice([1, 2, 3]))
        cin, cout = groups * int(r.integers(1, 7)), groups * int(r.integers(1, 7))
        k, dil, stride = int(r.integers(1, 12)), int(r.integers(1, 4)), int(r.integers(1, 4))
    span = (k - 1) * dil + 1
    pad = int(r.integers(0, span))
    length = max(span - 2 * pad, 1) + int(r.integers(0, 3000))
    x = r.standard_normal((int(r.integers(1, 4)), cin, length), dtype=np.float32)
    w = (r.standard_normal((cout, cin // groups, k), dtype=np.float32) / np.sqrt(k * cin / groups)).astype(np.float32)
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w), stride, pad, dil, groups))
    ref, mag = oracle.conv1d(x, w, stride, pad, dil, groups)
    assert_within_tol(y, ref, mag, "seed %d: %d->%d g%d k%d d%d s%d p%d L%d" % (seed, cin, cout, groups, k, dil, stride, pad, length))


@pytest.mark.parametrize("seed", range(30))
def test_pool2d_random(B, seed):
    r = _rng(7300 + seed)
    geoms = [(3, 3, 1, 1, 1, 1), (3, 3, 2, 2, 1, 1), (3, 3, 1, 1, 0, 0), (3, 3, 2, 2, 0, 0), (2, 2, 2, 2, 0, 0),
             (2, 2, 1, 1, 0, 0), (5, 5, 1, 1, 2, 2), (5, 5, 1, 1, 0, 0), (7, 7, 1, 1, 3, 3), (9, 9, 1, 1, 4, 4),
             (13, 13, 1, 1, 6, 6), (4, 3, 2, 1, 1, 2), (1, 7, 1, 3, 0, 3)]
    kh, kw, sh, sw, ph, pw = geoms[int(r.integers(0, len(geoms)))]
    h, w_ = int(r.integers(kh, 150)), int(r.integers(kw, 260))
    x = r.standard_normal((int(r.integers(1, 3)), int(r.integers(1, 5)), h, w_), dtype=np.float32)
    op = int(r.integers(0, 3))
    y = to_host(B.sws_pool2d(op, to_gpu(x), kh, kw, sh, sw, ph, pw, 1.0 / (kh * kw)))
    ref, mag = oracle.pool2d(op, x, kh, kw, sh, sw, ph, pw, 1.0 / (kh * kw))
    what = "seed %d: op %d %dx%d s(%d,%d) p(%d,%d) on %dx%d" % (seed, op, kh, kw, sh, sw, ph, pw, h, w_)
    if op == 0:
        assert_within_tol(y, ref, mag, what)
    else:
        assert_bit_exact(y, ref, what)


@pytest.mark.parametrize("seed", range(30))
def test_conv2d_random(B, seed):
    r = _rng(7400 + seed)
    cin = int(r.choice([3, 4, 8, 12, 16, 24, 32, 64]))
    cout = int(r.integers(1, 130))
    kh, kw = int(r.integers(1, 8)), int(r.integers(1, 8))
    sh, sw = int(r.integers(1, 4)), int(r.integers(1, 4))
    ph, pw = int(r.integers(0, kh)), int(r.integers(0, kw))
    h, w_ = int(r.integers(kh, 70)), int(r.integers(kw, 260))
    x = r.standard_normal((int(r.integers(1, 4)), cin, h, w_), dtype=np.float32)
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) / np.sqrt(cin * kh * kw)).astype(np.float32)
    y = to_host(B.sws_conv2d(to_gpu(x), to_gpu(w), sh, sw, ph, pw))
    ref, mag = oracle.conv2d(x, w, sh, sw, ph, pw)
    assert_within_tol(y, ref, mag, "seed %d: %d->%d %dx%d s(%d,%d) p(%d,%d) on %dx%d" % (seed, cin, cout, kh, kw, sh, sw, ph, pw, h, w_))


@pytest.mark.parametrize("seed", range(20))
def test_slide1d_pair_random(B, seed):
    r = _rng(7500 + seed)
    w = int(r.choice([1, 2, 3, 5, 16, 64, 255, 309, 310, 500, 961, 1000]))
    length = w - 1 + int(r.integers(1, 4000))
    rows = int(r.integers(1, 5))
    u = ((1.0 + 0.03 * (2.0 * r.random((rows, length)) - 1.0)) * np.where(r.random((rows, length)) < 0.2, -1.0, 1.0)).astype(np.float32)
    v = r.standard_normal((rows, length)).astype(np.float32)
    yu, yv = B.sws_slide1d_pair(to_gpu(u), to_gpu(v), w)
    ru, rv, mu, mv = oracle.slide1d_pair(u, v, w)
    tol = (w + 24) * 2.0 ** -24
    assert_within_tol(to_host(yu), ru, mu, "seed %d pair u w %d" % (seed, w), tol=tol)
    assert_within_tol(to_host(yv), rv, mv, "seed %d pair v w %d" % (seed, w), tol=tol)


@pytest.mark.parametrize("seed", range(30))
def test_slide1d_16_random(B, seed):
    import torch
    r = _rng(7500 + seed)
    w = int(r.choice([1, 2, 3, 5, 9, 16, 17, 33, 64, 100, 255, 256, 511, 850, 961, 1100]))
    tout = max(32, (1024 - (min(w, 961) - 1)) & ~31)
    lo = max(1, int(r.integers(1, 8)) * tout + int(r.integers(-40, 41)))
    rows = int(r.integers(1, 9))
    x = (r.random((rows, lo + w - 1), dtype=np.float32) * 2 - 1).astype(np.float32)
    op = int(r.integers(0, 3))
    tdt, odt, half = ((torch.bfloat16, oracle.DTYPE_BF16, 2.0 ** -8), (torch.float16, oracle.DTYPE_F16, 2.0 ** -11))[seed % 2]
    xq = torch.from_numpy(x).to(tdt)
    scale = float(r.choice([1.0, 1.0 / w]))
    got = B.sws_slide1d_16(op, xq.cuda(), w, scale).cpu().to(torch.float64).numpy()
    ref, mag = oracle.slide1d(op, xq.to(torch.float32).numpy(), w, scale)
    what = "seed %d: op %d w %d rows %d lo %d %s" % (seed, op, w, rows, lo, tdt)
    if op:
        assert np.array_equal(got, ref), what
    else:
        allowed = 1e-5 * mag + (np.abs(ref) + 1e-5 * mag) * half + 2.0 ** -25
        assert (np.abs(got - ref) <= allowed).all(), what


@pytest.mark.parametrize("seed", range(40))
def test_conv1d_adjoints_random(B, seed):
    r = _rng(7600 + seed)
    kind = seed % 4
    if kind == 0:                                   # thin channels
        c, mult = int(r.integers(1, 7)), int(r.integers(1, 3))
        cin, cout, groups, k, dil, stride = c, c * mult, c, int(r.integers(1, 70)), int(r.choice([1, 1, 2, 5])), 1
    elif kind == 1:                                 # dense channels
        cin, cout, groups = int(r.choice([8, 16, 24, 40, 64, 72])), int(r.integers(1, 80)), 1
        k, dil, stride = int(r.integers(1, 12)), int(r.choice([1, 1, 2, 3])), 1
    elif kind == 2:                                 # grouped
        groups = int(r.integers(2, 5))
        cin, cout = groups * int(r.integers(2, 6)), groups * int(r.integers(1, 5))
        k, dil, stride = int(r.integers(1, 20)), int(r.choice([1, 2])), 1
    else:                                           # strided: direct evaluation
        groups = int(r.choice([1, 2]))
        cin, cout = groups * int(r.integers(1, 9)), groups * int(r.integers(1, 9))
        k, dil, stride = int(r.integers(1, 9)), int(r.choice([1, 2])), int(r.integers(2, 5))
    span = dil * (k - 1) + 1
    length = span + int(r.integers(0, 2500))
    pad = int(r.integers(0, span + 2))
    b = int(r.integers(1, 4))
    lo = (length + 2 * pad - span) // stride + 1
    x = r.standard_normal((b, cin, length), dtype=np.float32)
    w = (r.standard_normal((cout, cin // groups, k), dtype=np.float32) * np.float32(0.3)).astype(np.float32)
    g = r.standard_normal((b, cout, lo), dtype=np.float32)
    what = "seed %d: B %d Cin %d L %d Cout %d k %d stride %d pad %d dil %d groups %d" % (
        seed, b, cin, length, cout, k, stride, pad, dil, groups)
    gx = to_host(B.sws_conv1d_grad_input(to_gpu(g), to_gpu(w), length, stride, pad, dil, groups))
    rx, mx = oracle.conv1d_grad_input(g, w, length, stride, pad, dil, groups)
    assert_within_tol(gx, rx, mx, "grad_input " + what)
    gw = to_host(B.sws_conv1d_grad_weight(to_gpu(x), to_gpu(g), k, stride, pad, dil, groups))
    rw, mw = oracle.conv1d_grad_weight(x, g, k, stride, pad, dil, groups)
    assert_within_tol(gw, rw, mw, "grad_weight " + what)


@pytest.mark.parametrize("seed", range(20))
def test_conv2d_adjoints_random(B, seed):
    r = _rng(7700 + seed)
    cin, cout = int(r.choice([3, 8, 16, 24, 40])), int(r.integers(1, 50))
    kh, kw = int(r.integers(1, 6)), int(r.integers(1, 6))
    sh, sw = (1, 1) if seed % 3 else (int(r.integers(1, 3)), int(r.integers(1, 3)))
    ph, pw = int(r.integers(0, kh + 1)), int(r.integers(0, kw + 1))
    h, wd = kh + int(r.integers(0, 40)), kw + int(r.integers(0, 90))
    n = int(r.integers(1, 3))
    ho, wo = (h + 2 * ph - kh) // sh + 1, (wd + 2 * pw - kw) // sw + 1
    x = r.standard_normal((n, cin, h, wd), dtype=np.float32)
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.float32(0.2)).astype(np.float32)
    g = r.standard_normal((n, cout, ho, wo), dtype=np.float32)
    what = "seed %d: N %d Cin %d H %d W %d Cout %d k %dx%d s %dx%d p %dx%d" % (seed, n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw)
    gx = to_host(B.sws_conv2d_grad_input(to_gpu(g), to_gpu(w), h, wd, sh, sw, ph, pw))
    rx, mx = oracle.conv2d_grad_input(g, w, h, wd, sh, sw, ph, pw)
    assert_within_tol(gx, rx, mx, "grad_input " + what)
    gw = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, sw, ph, pw))
    rw, mw = oracle.conv2d_grad_weight(x, g, kh, kw, sh, sw, ph, pw)
    assert_within_tol(gw, rw, mw, "grad_weight " + what)


@pytest.mark.parametrize("seed", range(30))
def test_pool2d_ex_random(B, seed):
    r = _rng(7800 + seed)
    kh, kw, sh, sw = [(3, 3, 1, 1), (3, 3, 2, 2), (2, 2, 2, 2), (5, 5, 1, 1), (7, 7, 1, 1), (4, 2, 3, 1)][seed % 6]
    pads = tuple(int(r.integers(0, lim)) for lim in (kh, kw, kh, kw))
    h, wd = kh + int(r.integers(0, 120)), kw + int(r.integers(0, 150))
    x = r.standard_normal((int(r.integers(1, 3)), int(r.integers(1, 6)), h, wd), dtype=np.float32)
    op, div = int(r.integers(0, 3)), int(r.integers(0, 2))
    y = to_host(B.sws_pool2d_ex(op, to_gpu(x), kh, kw, sh, sw, pads, div if op == 0 else 0, 0.25))
    ref, mag = oracle.pool2d_ex(op, x, kh, kw, sh, sw, pads, bool(div) and op == 0, 0.25)
    what = "seed %d: %dx%d s%dx%d pads %s plane %dx%d op %d div %d" % (seed, kh, kw, sh, sw, pads, h, wd, op, div)
    if op == 0:
        assert_within_tol(y, ref, mag, what)
    else:
        assert_bit_exact(y, ref, what)


@pytest.mark.parametrize("seed", range(40))
def test_maxpool2d_grad_random(B, seed):
    """Windows, strides and paddings drawn at random (strides above the window included: cells no
    window covers get zero), planes from a few cells to several bands, few distinct values (ties)."""
    r = _rng(7900 + seed)
    kh, kw = int(r.integers(1, 7)), int(r.integers(1, 7))
    sh, sw = int(r.integers(1, 5)), int(r.integers(1, 5))
    ph, pw = int(r.integers(0, kh)), int(r.integers(0, kw))
    h = max(1, kh - 2 * ph) + int(r.integers(0, 130))
    wd = max(1, kw - 2 * pw) + int(r.integers(0, 300 if seed % 4 else 1500))
    n, c = int(r.integers(1, 3)), int(r.integers(1, 4))
    ho, wo = (h + 2 * ph - kh) // sh + 1, (wd + 2 * pw - kw) // sw + 1
    x = r.integers(0, 6 if seed % 2 else 1000, (n, c, h, wd)).astype(np.float32)
    gy = r.standard_normal((n, c, ho, wo), dtype=np.float32)
    gx = to_host(B.sws_maxpool2d_grad(to_gpu(x), to_gpu(gy), kh, kw, sh, sw, ph, pw))
    ref = oracle.maxpool2d_grad(x, gy, kh, kw, sh, sw, ph, pw)
    mag = oracle.maxpool2d_grad(x, np.abs(gy), kh, kw, sh, sw, ph, pw)
    assert_within_tol(gx, ref, mag, "seed %d: %dx%d s%dx%d p%dx%d plane %dx%d" % (seed, kh, kw, sh, sw, ph, pw, h, wd))


@pytest.mark.parametrize("seed", range(30))
def test_conv2d_grad_weight_short_rows_random(B, seed):
    """Planes narrow enough that the dense kernel packs several output rows into one slab."""
    r = _rng(8000 + seed)
    cin, cout = int(r.integers(2, 70)), int(r.integers(1, 70))
    kh, kw = int(r.integers(1, 6)), int(r.integers(1, 6))
    sh = int(r.integers(1, 3))
    ph, pw = int(r.integers(0, kh)), int(r.integers(0, kw))
    h = max(1, kh - 2 * ph) + int(r.integers(0, 20))
    wd = max(1, kw - 2 * pw) + int(r.integers(0, 30))
    n = int(r.integers(1, 12))
    ho, wo = (h + 2 * ph - kh) // sh + 1, (wd + 2 * pw - kw) + 1
    x = r.standard_normal((n, cin, h, wd), dtype=np.float32)
    g = r.standard_normal((n, cout, ho, wo), dtype=np.float32)
    gw = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, 1, ph, pw))
    rw, mw = oracle.conv2d_grad_weight(x, g, kh, kw, sh, 1, ph, pw)
    assert_within_tol(gw, rw, mw, "seed %d: N %d Cin %d H %d W %d Cout %d k %dx%d sh %d p %dx%d" % (seed, n, cin, h, wd, cout, kh, kw, sh, ph, pw))


@pytest.mark.parametrize("seed", range(40))
def test_conv2d_grad_input_strided_random(B, seed):
    """Strides up to 4 (also above the kernel size: cells no tap reaches must come out zero), kernels
    up to 7 x 7 (phases of more than 9 taps run as chains), paddings up to k - 1."""
    r = _rng(8100 + seed)
    cin, cout = int(r.integers(1, 40)), int(r.integers(1, 40))
    kh, kw = int(r.integers(1, 8)), int(r.integers(1, 8))
    sh, sw = int(r.integers(1, 5)), int(r.integers(1, 5))
    ph, pw = int(r.integers(0, kh)), int(r.integers(0, kw))
    h = max(1, kh - 2 * ph) + int(r.integers(0, 40))
    wd = max(1, kw - 2 * pw) + int(r.integers(0, 60 if seed % 5 else 260))
    n = int(r.integers(1, 4))
    ho, wo = (h + 2 * ph - kh) // sh + 1, (wd + 2 * pw - kw) // sw + 1
    w = (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.float32(0.2)).astype(np.float32)
    g = r.standard_normal((n, cout, ho, wo), dtype=np.float32)
    gx = to_host(B.sws_conv2d_grad_input(to_gpu(g), to_gpu(w), h, wd, sh, sw, ph, pw))
    rx, mx = oracle.conv2d_grad_input(g, w, h, wd, sh, sw, ph, pw)
    assert_within_tol(gx, rx, mx, "seed %d: N %d Cin %d H %d W %d Cout %d k %dx%d s %dx%d p %dx%d" % (seed, n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw))


@pytest.mark.parametrize("seed", range(30))
def test_conv2d_1x1_random(B, seed):
    """1 x 1 kernels (planes taken as one long row, four channel blocks per barrier pair where the
    channel count allows), forward and both adjoints, strides 1 and 2."""
    r = _rng(8200 + seed)
    cin = int(r.choice([32, 64, 96, 128, 8, 24, 40, 33]))
    cout = int(r.integers(1, 130))
    h, wd = int(r.integers(1, 40)), int(r.integers(1, 70))
    n = int(r.integers(1, 4))
    s = 1 if seed % 3 else 2
    ho, wo = (h - 1) // s + 1, (wd - 1) // s + 1
    x = r.standard_normal((n, cin, h, wd), dtype=np.float32)
    w = (r.standard_normal((cout, cin, 1, 1), dtype=np.float32) * np.float32(0.2)).astype(np.float32)
    g = r.standard_normal((n, cout, ho, wo), dtype=np.float32)
    what = "seed %d: N %d Cin %d Cout %d plane %dx%d stride %d" % (seed, n, cin, cout, h, wd, s)
    ry, my = oracle.conv2d(x, w, s, s, 0, 0)
    assert_within_tol(to_host(B.sws_conv2d(to_gpu(x), to_gpu(w), s, s, 0, 0)), ry, my, "forward " + what)
    rx, mx = oracle.conv2d_grad_input(g, w, h, wd, s, s, 0, 0)
    assert_within_tol(to_host(B.sws_conv2d_grad_input(to_gpu(g), to_gpu(w), h, wd, s, s, 0, 0)), rx, mx, "grad_input " + what)
    rw, mw = oracle.conv2d_grad_weight(x, g, 1, 1, s, s, 0, 0)
    assert_within_tol(to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), 1, 1, s, s, 0, 0)), rw, mw, "grad_weight " + what)
