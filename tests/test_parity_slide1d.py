"""GPU parity of sws_slide1d against the CPU oracle (Section 2.2, Eq. 3), through the C ABI.

Sizes are chosen so that every kernel sees several tiles and a ragged tail; max / min must
be bit-exact, add must satisfy |err| <= 1e-5 * sum|terms| per output."""
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
    binding.sws_set_option("slide_variant", 0)


def _check(B, op, x, w, scale=1.0, what=""):
    y = to_host(B.sws_slide1d(OPS[op], to_gpu(x), w, scale))
    ref, mag = oracle.slide1d(OPS[op], x.reshape(-1, x.shape[-1]), w, scale)
    ref, mag = ref.reshape(y.shape), mag.reshape(y.shape)
    if op == "add":
        return assert_within_tol(y, ref, mag, what)
    assert_bit_exact(y, ref, what)
    return 0.0


WINDOWS = [1, 2, 3, 4, 5, 7, 8, 9, 10, 15, 16, 17, 31, 33, 64, 65, 100, 255, 256, 257, 500, 770, 961]


@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("w", WINDOWS)
def test_several_tiles_and_ragged_tail(B, op, w):
    """3 rows of 5003 (not a multiple of 4: every row after the first is misaligned)."""
    rng = np.random.Generator(np.random.PCG64(1000 + w))
    x = (rng.random((3, 5003), dtype=np.float32) * 2 - 1).astype(np.float32)
    _check(B, op, x, w, scale=1.0 / w, what="%s w=%d" % (op, w))


@pytest.mark.parametrize("op", ["add", "max"])
@pytest.mark.parametrize("length,w", [(1, 1), (2, 2), (5, 5), (17, 16), (64, 9), (255, 255), (256, 255),
                                      (1023, 300), (1024, 64), (1025, 2), (2047, 1000), (4097, 1025)])
def test_degenerate_and_short_rows(B, op, length, w):
    """Single-output rows, rows shorter than a tile, windows beyond the scan kernel's reach."""
    rng = np.random.Generator(np.random.PCG64(length * 7 + w))
    x = rng.standard_normal((5, length), dtype=np.float32)
    _check(B, op, x, w, what="%s len=%d w=%d" % (op, length, w))


@pytest.mark.parametrize("w", [3, 8, 9, 16, 64, 255])
def test_add_is_bit_exact_on_integer_valued_input(B, w):
    """Every fp32 partial sum is exact, so any association order must give the same bits."""
    x = workloads.integer_valued((4, 3001), -64, 64, seed=w)
    y = to_host(B.sws_slide1d(0, to_gpu(x), w))
    ref, _ = oracle.slide1d(0, x, w)
    assert np.array_equal(y.astype(np.float64), ref)


@pytest.mark.parametrize("variant", [1, 2, 3])
@pytest.mark.parametrize("w", [2, 5, 9])
def test_every_kernel_variant(B, variant, w):
    rng = np.random.Generator(np.random.PCG64(variant * 100 + w))
    x = rng.standard_normal((7, 2500), dtype=np.float32)
    B.sws_set_option("slide_variant", variant)
    try:
        for op in ("add", "max", "min"):
            _check(B, op, x, w, scale=0.25, what="variant %d %s w=%d" % (variant, op, w))
    finally:
        B.sws_set_option("slide_variant", 0)


@pytest.mark.parametrize("bits", [1, 2, 4, 8, 1 | 8, 2 | 4])
@pytest.mark.parametrize("group", [0, 4, 12, 64])
def test_scan_kernel_tiling_knobs(B, bits, group):
    """Unaligned / aligned tiles, plain / non-temporal stores, both workgroup placements and
    several tiles-per-workgroup counts must all give the same answer."""
    rng = np.random.Generator(np.random.PCG64(bits * 10 + group))
    x = rng.standard_normal((9, 4099), dtype=np.float32)
    B.sws_set_option("slide_chunk", bits)
    B.sws_set_option("slide_group", group)
    try:
        for w in (2, 17, 100, 255, 700):
            _check(B, "add", x, w, scale=0.5, what="bits %d group %d w %d" % (bits, group, w))
            _check(B, "max", x, w, what="bits %d group %d w %d" % (bits, group, w))
    finally:
        B.sws_set_option("slide_chunk", 0)
        B.sws_set_option("slide_group", 0)


def test_many_short_rows(B):
    """More rows than any grid dimension trick would hide: 40000 rows of 37."""
    rng = np.random.Generator(np.random.PCG64(77))
    x = rng.standard_normal((40000, 37), dtype=np.float32)
    _check(B, "add", x, 5)
    _check(B, "max", x, 12)


def test_leading_dimensions_are_rows(B):
    x, _ = workloads.make(2, x_shape=(2, 3, 300))
    y = to_host(B.sws_slide1d(1, to_gpu(x), 3))
    ref, _ = oracle.slide1d(1, x.reshape(6, 300), 3)
    assert y.shape == (2, 3, 298)
    assert_bit_exact(y.reshape(6, 298), ref)


def test_scale_ignored_for_max(B):
    x, _ = workloads.make(1, x_shape=(1, 1, 999))
    a = to_host(B.sws_slide1d(1, to_gpu(x), 16, 123.0))
    b = to_host(B.sws_slide1d(1, to_gpu(x), 16, 1.0))
    assert np.array_equal(a, b)


def test_poisoned_surroundings(B):
    """x and y sit in the middle of larger device buffers filled with huge sentinels: a
    read that strays outside x shows up in the result, a write outside y in the guard."""
    import torch
    rng = np.random.Generator(np.random.PCG64(5))
    rows, length, guard = 6, 1501, 4099
    x = rng.standard_normal((rows, length), dtype=np.float32)
    for w in (1, 5, 64, 255, 1100):
        lo = length - w + 1
        for op in ("add", "max"):
            xbuf = torch.full((guard + rows * length + guard,), 1e30, device="cuda")
            ybuf = torch.full((guard + rows * lo + guard,), -7e29, device="cuda")
            xin = xbuf[guard:guard + rows * length].view(rows, length)
            xin.copy_(torch.from_numpy(x))
            yout = ybuf[guard:guard + rows * lo].view(rows, lo)
            B.sws_slide1d(OPS[op], xin, w, 1.0, y=yout)
            ref, mag = oracle.slide1d(OPS[op], x, w)
            if op == "add":
                assert_within_tol(to_host(yout), ref, mag, "guarded add w=%d" % w)
            else:
                assert_bit_exact(to_host(yout), ref, "guarded max w=%d" % w)
            assert bool((ybuf[:guard] == -7e29).all()) and bool((ybuf[guard + rows * lo:] == -7e29).all())


def test_cfg1_full_size(B):
    """1-D single sequence, N = 1,048,576, w = 5: sliding add and max at full size."""
    x, _ = workloads.make(1)
    workloads.check_clean(x)
    worst = _check(B, "add", x.reshape(1, -1), 5, what="cfg1 add")
    _check(B, "max", x.reshape(1, -1), 5, what="cfg1 max")
    assert worst < 1e-6


def test_cfg2_pooling_full_size(B):
    """[16, 64, 4096] avg and max pool, w = 3, stride 1."""
    x, _ = workloads.make(2)
    _check(B, "add", x.reshape(-1, 4096), 3, scale=1.0 / 3, what="cfg2 avg")
    _check(B, "max", x.reshape(-1, 4096), 3, what="cfg2 max")


def test_graph_replay_matches_eager(B):
    """The entry points only enqueue kernels on the caller's stream, so a launch-bound sequence can
    be captured in a HIP graph.  Several replays, with eager work and synchronisation between them
    and fresh inputs each time, must reproduce the eager results bit for bit."""
    import torch
    r = np.random.Generator(np.random.PCG64(2024))
    x = to_gpu((r.random((1, 1, 100000), dtype=np.float32) * 2 - 1).astype(np.float32))
    taps = to_gpu(r.standard_normal((1, 1, 5), dtype=np.float32))
    ya, ym, yc = (torch.empty(1, 1, 99996, device="cuda") for _ in range(3))
    yp = torch.empty(1, 1, 100000, device="cuda")

    def launch_all():
        B.sws_slide1d(0, x, 5, 0.2, y=ya)
        B.sws_slide1d(1, x, 5, 1.0, y=ym)
        B.sws_conv1d(x, taps, y=yc)
        B.sws_slide1d_padded(1, x, 5, 2, 2, B.SWS_PAD_MIRROR, 1.0, y=yp)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch_all()                                           # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        launch_all()
    for rep in range(4):
        x.copy_(to_gpu((r.random((1, 1, 100000), dtype=np.float32) * 2 - 1).astype(np.float32)))   # eager work between replays
        for t in (ya, ym, yc, yp):
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (ya, ym, yc, yp)]
        launch_all()                                           # eager, same inputs
        torch.cuda.synchronize()
        for a, b in zip(got, (ya, ym, yc, yp)):
            assert torch.equal(a, b), "replay %d differs from the eager result" % rep
        ref, mag = oracle.slide1d(0, to_host(x).reshape(1, -1), 5, 0.2)
        assert_within_tol(to_host(got[0]).reshape(1, -1), ref, mag, "graph replay %d" % rep)


@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("w,length", [(851, 2000), (962, 2000), (1500, 1500), (1537, 7000), (2048, 20000), (5000, 20011),
                                      (16384, 16385)])
def test_windows_longer_than_a_tile(B, op, w, length):
    """w > 850 on the default route: the one-pass long-window kernel up to 8192, beyond it the window split into
    links within the scan kernel's reach, each link combined with the earlier ones in y."""
    r = np.random.Generator(np.random.PCG64(op * 100000 + w))
    x = (r.random((3, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    y = to_host(B.sws_slide1d(op, to_gpu(x), w, 1.0 / w))
    ref, mag = oracle.slide1d(op, x, w, 1.0 / w)
    if op == 0:
        assert_within_tol(y, ref, mag, "chain add w=%d" % w)
    else:
        assert_bit_exact(y, ref, "chain op %d w=%d" % (op, w))
    B.sws_set_option("slide_variant", 1)                        # and the direct-evaluation kernel agrees
    try:
        y1 = to_host(B.sws_slide1d(op, to_gpu(x), w, 1.0 / w))
    finally:
        B.sws_set_option("slide_variant", 0)
    if op == 0:
        assert_within_tol(y1, ref, mag, "direct add w=%d" % w)
    else:
        assert_bit_exact(y1, ref, "direct op %d w=%d" % (op, w))


@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("w,length", [(513, 513), (600, 3000), (1024, 5000), (1025, 1025), (1025, 1026), (1026, 9000), (2047, 4100),
                                      (2048, 16384), (4097, 13000), (8192, 16384), (8192, 8200)])
def test_long_window_kernel_and_chain_agree_with_the_oracle(B, op, w, length):
    """Windows longer than a wave tile: the one-pass kernel (slide_variant 8: suffix sums of the tile, one shared
    middle reduction, prefix sums where the windows end) and the chain of shorter windows (slide_variant 5)."""
    r = np.random.Generator(np.random.PCG64(op * 7 + w + length))
    x = (r.random((5, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    ref, mag = oracle.slide1d(op, x, w, 1.0 / w)
    for variant in (8, 5):
        B.sws_set_option("slide_variant", variant)
        try:
            y = to_host(B.sws_slide1d(op, to_gpu(x), w, 1.0 / w))
        finally:
            B.sws_set_option("slide_variant", 0)
        if op == 0:
            assert_within_tol(y, ref, mag, "variant %d add w=%d" % (variant, w))
        else:
            assert_bit_exact(y, ref, "variant %d op %d w=%d" % (variant, op, w))


def test_long_window_kernel_on_integer_valued_input_is_exact(B):
    x = workloads.integer_valued((3, 20000), -8, 8, seed=13)
    for w in (700, 1500, 3001, 8000):
        B.sws_set_option("slide_variant", 8)
        try:
            y = to_host(B.sws_slide1d(0, to_gpu(x), w, 1.0))
        finally:
            B.sws_set_option("slide_variant", 0)
        ref, _ = oracle.slide1d(0, x, w, 1.0)
        assert np.array_equal(y.astype(np.float64), ref), w


def test_chain_on_integer_valued_input_is_exact(B):
    x = workloads.integer_valued((2, 9000), -8, 8, seed=12)
    y = to_host(B.sws_slide1d(0, to_gpu(x), 3001, 1.0))
    ref, _ = oracle.slide1d(0, x, 3001, 1.0)
    assert np.array_equal(y.astype(np.float64), ref)


def test_longest_supported_row(B):
    """One row of the largest length the ABI accepts (2^31 - 1 - 65536 elements, 8.6 GB): 32-bit
    tile arithmetic at its limit.  The oracle checks stretches at the start, the end and seeded
    places in between; one element more is an argument error (checked before anything is touched)."""
    import torch
    length = 2 ** 31 - 1 - 65536
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * length * 2.2:
        pytest.skip("not enough device memory for the longest row")
    g = torch.Generator(device="cuda")
    g.manual_seed(31)
    x = torch.rand(1, length, device="cuda", generator=g) * 2 - 1
    r = np.random.Generator(np.random.PCG64(31))
    n = 3000
    for op, w in ((0, 16), (1, 255), (0, 900)):
        lo = length - w + 1
        y = B.sws_slide1d(op, x, w, 1.0)
        assert y.shape == (1, lo)
        starts = [0, lo - n] + [int(v) for v in r.integers(0, lo - n, size=5)] + [2 ** 30 - 1500, 2 ** 31 - 70000 - n]
        for s0 in starts:
            s0 = min(max(s0, 0), lo - n)
            ref, mag = oracle.slide1d(op, to_host(x[:, s0:s0 + n + w - 1]), w, 1.0)
            got = to_host(y[:, s0:s0 + n])
            if op == 0:
                assert_within_tol(got, ref, mag, "longest row add w=%d at %d" % (w, s0))
            else:
                assert_bit_exact(got, ref, "longest row max w=%d at %d" % (w, s0))
        del y
    del x
    torch.cuda.empty_cache()
    assert B.lib().sws_slide1d(0, 16, 16, 1, length + 1, 16, 1.0, None) == B.SWS_ERR_INVALID_ARG


def test_more_than_2_to_the_32_elements(B):
    """70 000 rows of 65 536 (4.6e9 elements, 18 GB in): every row offset beyond 2^31 and 2^32 elements
    must be computed in 64 bits.  The oracle checks the first and last rows and those around the
    2^31- and 2^32-element marks, for the scan kernel (fp32 and bf16), the shifted-load kernel and the
    thin convolution."""
    import torch
    rows, length = 70000, 65536
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * rows * length * 2.3:
        pytest.skip("not enough device memory")
    g = torch.Generator(device="cuda")
    g.manual_seed(32)
    x = torch.rand(rows, length, device="cuda", generator=g) * 2 - 1
    sample = [0, 1, 32767, 32768, 32769, 65535, 65536, 65537, rows - 2, rows - 1]
    xs = to_host(x[sample])
    for op, w in ((0, 64), (1, 5), (0, 900)):
        y = B.sws_slide1d(op, x, w, 1.0)
        ref, mag = oracle.slide1d(op, xs, w, 1.0)
        got = to_host(y[sample])
        del y
        if op == 0:
            assert_within_tol(got, ref, mag, "big add w=%d" % w)
        else:
            assert_bit_exact(got, ref, "big max w=%d" % w)
    xc = x.view(rows // 2, 2, length)                                     # [35000, 2, 65536], depthwise, two channels
    t2 = np.random.Generator(np.random.PCG64(34)).standard_normal((2, 1, 9), dtype=np.float32)
    y = B.sws_conv1d(xc, to_gpu(t2), groups=2)
    for b in (0, 16384, 32768, rows // 2 - 1):
        ref, mag = oracle.conv1d(to_host(xc[b:b + 1]), t2, groups=2)
        assert_within_tol(to_host(y[b:b + 1]), ref, mag, "big depthwise conv image %d" % b)
    del y
    xb = x.to(torch.bfloat16)
    del x
    y = B.sws_slide1d_16(1, xb, 33, 1.0)
    ref, _ = oracle.slide1d(1, xb[sample].float().cpu().numpy(), 33, 1.0)
    assert np.array_equal(y[sample].float().cpu().numpy().astype(np.float64), ref)
    del y, xb
    torch.cuda.empty_cache()


@pytest.mark.parametrize("variant", [0, 1, 3, 4])
def test_copy_is_bit_exact_for_every_variant_and_ragged_sizes(B, variant):
    """sws_copy (the calibration copy behind the bandwidth ceilings): whole tiles, a ragged tail, sizes below one tile."""
    import torch
    B.sws_set_option("copy_variant", variant)
    try:
        for n in (1, 255, 256, 257, 4095, 4096, 4097, 3 * 4096 + 1000, (1 << 20) + 3):
            src = torch.arange(n, device="cuda", dtype=torch.float32) * 0.5 - 7.0
            dst = torch.full((n + 8,), -1.0, device="cuda")
            B.sws_copy(src, dst[:n])
            assert torch.equal(dst[:n], src) and bool((dst[n:] == -1.0).all()), "variant %d n %d" % (variant, n)
    finally:
        B.sws_set_option("copy_variant", 0)


@pytest.mark.parametrize("chunk", [16, 32])
@pytest.mark.parametrize("w", [1, 2, 3, 4, 5, 7, 9, 10, 11])
def test_shifted_load_kernel_in_both_shapes(B, w, chunk):
    """The small-window kernel as 1024-output tiles (option slide_chunk bit 16) and as 256-output strips, one
    per single-wavefront workgroup (bit 32): rows that move the output alignment, ragged tails, rows
    shorter than a strip."""
    B.sws_set_option("slide_variant", 2)
    B.sws_set_option("slide_chunk", chunk)
    try:
        for rows, lo in ((3, 1000), (5, 255), (2, 256), (7, 257), (4, 4099), (1, 70001), (9, 3), (6, 1)):
            r = np.random.Generator(np.random.PCG64(w * 1000 + lo + chunk))
            x = (r.random((rows, lo + w - 1), dtype=np.float32) * 2 - 1).astype(np.float32)
            for op in (0, 1, 2):
                y = to_host(B.sws_slide1d(op, to_gpu(x), w, 0.5))
                ref, mag = oracle.slide1d(op, x, w, 0.5)
                what = "w %d rows %d lo %d op %d chunk %d" % (w, rows, lo, op, chunk)
                if op == 0:
                    assert_within_tol(y, ref, mag, what)
                else:
                    assert_bit_exact(y, ref, what)
    finally:
        B.sws_set_option("slide_variant", 0)
        B.sws_set_option("slide_chunk", 0)


@pytest.mark.parametrize("variant", [0, 7])
@pytest.mark.parametrize("w", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 13, 16, 17, 21, 25, 29, 32, 33, 34])
def test_short_row_kernel(B, w, variant):
    """Windows up to 33 on short rows: four outputs per lane, several rows per wavefront.  Forced
    (option slide_variant 7, also on rows longer than it is chosen for) and as the library chooses;
    x and y start off the 16-byte boundaries, and the elements around y must stay untouched."""
    import torch
    B.sws_set_option("slide_variant", variant)
    try:
        for rows, length in ((7, 56), (300, 57), (1000, 9), (40, 260), (2, 4), (5, 1031), (3, 5003), (130, 224),
                             (65, 1), (64, 64), (9, 255 + w), (9, 256 + w)):
            if w > length:
                continue
            lo = length - w + 1
            r = np.random.Generator(np.random.PCG64(w * 977 + length))
            x = (r.random((rows, length), dtype=np.float32) * 2 - 1).astype(np.float32)
            xbuf = torch.zeros(rows * length + 8, device="cuda")
            xs = xbuf[1:1 + rows * length].view(rows, length)
            xs.copy_(torch.from_numpy(x))
            for op in (0, 1, 2):
                ybuf = torch.full((rows * lo + 8,), 7.0, device="cuda")
                ys = ybuf[3:3 + rows * lo].view(rows, lo)
                B.sws_slide1d(op, xs, w, 0.5, y=ys)
                y = to_host(ys)
                ref, mag = oracle.slide1d(op, x, w, 0.5)
                what = "w %d rows %d len %d op %d variant %d" % (w, rows, length, op, variant)
                if op == 0:
                    assert_within_tol(y, ref, mag, what)
                else:
                    assert_bit_exact(y, ref, what)
                guard = ybuf.cpu()
                assert (guard[:3] == 7.0).all() and (guard[3 + rows * lo:] == 7.0).all(), what
    finally:
        B.sws_set_option("slide_variant", 0)



@pytest.mark.parametrize("w", [5, 6, 7, 8, 9, 12, 13, 15, 16, 17, 18, 20, 31, 32, 33, 34, 35, 48, 49, 62, 63, 64, 65])
def test_strips_in_registers_kernel(B, w):
    """Windows 5 .. 65 on one 256-element strip per wavefront, whole lanes summed across the wavefront (option
    slide_variant 9 forces the kernel on every shape): several strips per row and ragged ends, rows shorter than a
    strip, x and y off the 16-byte boundaries, the elements around y untouched."""
    import torch
    B.sws_set_option("slide_variant", 9)
    try:
        for rows, length in ((3, 5003), (7, 700), (40, 260), (9, 255 + w), (9, 256 + w), (300, 65), (5, 1031), (2, w),
                             (130, 224), (1, 4099)):
            if w > length:
                continue
            lo = length - w + 1
            r = np.random.Generator(np.random.PCG64(w * 991 + length))
            x = (r.random((rows, length), dtype=np.float32) * 2 - 1).astype(np.float32)
            xbuf = torch.zeros(rows * length + 8, device="cuda")
            xs = xbuf[1:1 + rows * length].view(rows, length)
            xs.copy_(torch.from_numpy(x))
            for op in (0, 1, 2):
                ybuf = torch.full((rows * lo + 8,), 7.0, device="cuda")
                ys = ybuf[3:3 + rows * lo].view(rows, lo)
                B.sws_slide1d(op, xs, w, 0.5, y=ys)
                y = to_host(ys)
                ref, mag = oracle.slide1d(op, x, w, 0.5)
                what = "w %d rows %d len %d op %d" % (w, rows, length, op)
                if op == 0:
                    assert_within_tol(y, ref, mag, what)
                else:
                    assert_bit_exact(y, ref, what)
                guard = ybuf.cpu()
                assert (guard[:3] == 7.0).all() and (guard[3 + rows * lo:] == 7.0).all(), what
    finally:
        B.sws_set_option("slide_variant", 0)


def test_strips_in_registers_kernel_is_exact_on_integers(B):
    """Small integers: every order of summation gives the same fp32 result, so + must agree bit for bit too."""
    B.sws_set_option("slide_variant", 9)
    try:
        for w in (16, 23, 64):
            x = workloads.integer_valued((33, 3000), -8, 8, 5 + w)
            y = to_host(B.sws_slide1d(0, to_gpu(x), w, 1.0))
            ref, _ = oracle.slide1d(0, x, w, 1.0)
            assert_bit_exact(y, ref, "w %d" % w)
    finally:
        B.sws_set_option("slide_variant", 0)
