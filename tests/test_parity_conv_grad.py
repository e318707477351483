"""GPU parity of the adjoints of sws_conv1d (sws_conv1d_grad_input, sws_conv1d_grad_weight) against the
CPU oracle's scatter-form definitions, through the C ABI: |err| <= 1e-5 * sum|terms| per element, and
bit-exact on small-integer data (every fp32 partial sum is exact, whatever the order of the atomic adds)."""
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


def _lo(length, k, stride, pad, dil):
    return (length + 2 * pad - dil * (k - 1) - 1) // stride + 1


def _data(case, seed, integer=False):
    b, cin, length, cout, k, stride, pad, dil, groups = case
    lo = _lo(length, k, stride, pad, dil)
    if integer:
        x = workloads.integer_valued((b, cin, length), -3, 3, seed)
        w = workloads.integer_valued((cout, cin // groups, k), -3, 3, seed + 1)
        g = workloads.integer_valued((b, cout, lo), -3, 3, seed + 2)
    else:
        r = np.random.Generator(np.random.PCG64(seed))
        x = r.standard_normal((b, cin, length), dtype=np.float32)
        w = (r.standard_normal((cout, cin // groups, k), dtype=np.float32) * np.float32(0.3)).astype(np.float32)
        g = r.standard_normal((b, cout, lo), dtype=np.float32)
    return x, w, g


def _check_gx(B, case, seed=0, integer=False):
    b, cin, length, cout, k, stride, pad, dil, groups = case
    x, w, g = _data(case, seed, integer)
    gx = to_host(B.sws_conv1d_grad_input(to_gpu(g), to_gpu(w), length, stride, pad, dil, groups))
    ref, mag = oracle.conv1d_grad_input(g, w, length, stride, pad, dil, groups)
    if integer:
        assert np.array_equal(gx.astype(np.float64), ref), str(case)
    else:
        assert_within_tol(gx, ref, mag, "grad_input %s" % (case,))


def _check_gw(B, case, seed=0, integer=False):
    b, cin, length, cout, k, stride, pad, dil, groups = case
    x, w, g = _data(case, seed, integer)
    gw = to_host(B.sws_conv1d_grad_weight(to_gpu(x), to_gpu(g), k, stride, pad, dil, groups))
    ref, mag = oracle.conv1d_grad_weight(x, g, k, stride, pad, dil, groups)
    if integer:
        assert np.array_equal(gw.astype(np.float64), ref), str(case)
    else:
        assert_within_tol(gw, ref, mag, "grad_weight %s" % (case,))


# B, Cin, L, Cout, k, stride, pad, dilation, groups
THIN = [(3, 8, 5003, 8, 31, 1, 15, 1, 8), (2, 4, 3000, 4, 5, 1, 0, 1, 4), (2, 3, 2500, 3, 64, 1, 7, 1, 3),
        (2, 2, 1500, 2, 1, 1, 0, 1, 2), (5, 3, 1024, 3, 3, 1, 1, 1, 3), (2, 2, 4100, 6, 7, 1, 3, 1, 2),
        (1, 1, 100000, 1, 51, 1, 25, 1, 1)]
THIN_DILATED = [(2, 4, 3000, 4, 5, 1, 6, 3, 4), (1, 2, 9000, 2, 51, 1, 0, 8, 2), (2, 3, 2000, 3, 100, 1, 50, 1, 3)]
GROUPED = [(2, 4, 3001, 6, 5, 1, 2, 1, 2), (2, 6, 2000, 3, 9, 1, 4, 1, 3), (2, 15, 1500, 15, 11, 1, 0, 2, 1),
           (2, 12, 1200, 20, 3, 1, 1, 1, 1)]
DENSE = [(3, 64, 1000, 64, 3, 1, 1, 1, 1), (2, 16, 700, 24, 5, 1, 2, 1, 1), (2, 72, 333, 136, 3, 1, 0, 1, 1),
         (2, 32, 900, 32, 4, 1, 3, 2, 1), (1, 8, 2000, 16, 11, 1, 5, 1, 1), (2, 64, 260, 64, 1, 1, 0, 1, 1),
         (2, 24, 500, 8, 2, 1, 0, 7, 1)]
DIRECT = [(2, 4, 500, 4, 5, 2, 2, 1, 4), (2, 8, 301, 16, 3, 2, 1, 1, 1), (2, 6, 400, 4, 4, 3, 0, 2, 2),
          (1, 2, 50, 2, 3, 1, 5, 1, 2)]


@pytest.mark.parametrize("case", THIN + THIN_DILATED + GROUPED + DENSE + DIRECT)
def test_grad_input(B, case):
    _check_gx(B, case, seed=hash(case) % 1000)


@pytest.mark.parametrize("case", THIN + THIN_DILATED + GROUPED + DENSE + DIRECT)
def test_grad_weight(B, case):
    _check_gw(B, case, seed=hash(case) % 1000 + 7)


@pytest.mark.parametrize("case", [THIN[0], THIN[5], GROUPED[0], DENSE[0], DENSE[1], DENSE[3], DIRECT[1]])
def test_exact_on_small_integers(B, case):
    _check_gx(B, case, seed=11, integer=True)
    _check_gw(B, case, seed=12, integer=True)


@pytest.mark.parametrize("case", [THIN[0], DENSE[0], GROUPED[1]])
def test_tuned_kernels_agree_with_direct_evaluation_on_the_gpu(B, case):
    """conv1d_variant = 1 forces the direct-evaluation kernels: both must pass against the oracle."""
    B.sws_set_option("conv1d_variant", 1)
    try:
        _check_gx(B, case, seed=21)
        _check_gw(B, case, seed=22)
    finally:
        B.sws_set_option("conv1d_variant", 0)


def test_layer_shaped_depthwise(B):
    """A slice of configuration 5: 128 channels, 16384-long rows, k = 31 (4 images)."""
    case = (4, 128, 16384, 128, 31, 1, 0, 1, 128)
    _check_gx(B, case, seed=31)
    _check_gw(B, case, seed=32)


def test_layer_shaped_dense(B):
    """Configuration 2: x[16,64,4096], 64 -> 64 channels, k = 3."""
    case = (16, 64, 4096, 64, 3, 1, 0, 1, 1)
    _check_gx(B, case, seed=33)
    _check_gw(B, case, seed=34)


def test_inner_product_identities_on_the_gpu(B):
    """<conv(x; W), g> = <x, gx> = <W, gw> with all three computed on the GPU."""
    case = (2, 32, 1500, 48, 5, 1, 2, 1, 1)
    x, w, g = _data(case, 40)
    y = to_host(B.sws_conv1d(to_gpu(x), to_gpu(w), 1, 2, 1, 1)).astype(np.float64)
    gx = to_host(B.sws_conv1d_grad_input(to_gpu(g), to_gpu(w), 1500, 1, 2, 1, 1)).astype(np.float64)
    gw = to_host(B.sws_conv1d_grad_weight(to_gpu(x), to_gpu(g), 5, 1, 2, 1, 1)).astype(np.float64)
    loss = float((y * g).sum())
    scale = float(np.abs(y * g).sum())
    assert abs(loss - float((x * gx).sum())) < 1e-5 * scale
    assert abs(loss - float((w * gw).sum())) < 1e-5 * scale


def test_argument_checks(B):
    import torch
    g = torch.zeros((2, 4, 98), device="cuda")
    w = torch.zeros((4, 1, 3), device="cuda")
    with pytest.raises(B.SwsError):
        B.sws_conv1d_grad_input(g, w, 101, 1, 0, 1, 4)          # gy is not the forward output's shape
    L = B.lib()
    assert L.sws_conv1d_grad_input(g.data_ptr(), w.data_ptr(), None, 2, 4, 100, 4, 3, 1, 0, 1, 4, None) == B.SWS_ERR_INVALID_ARG
    assert L.sws_conv1d_grad_weight(g.data_ptr(), g.data_ptr(), w.data_ptr(), 2, 4, 100, 4, 3, 0, 0, 1, 4, None) == B.SWS_ERR_INVALID_ARG
    gw = torch.ones((4, 1, 3), device="cuda")
    assert L.sws_conv1d_grad_weight(None, None, gw.data_ptr(), 0, 4, 100, 4, 3, 1, 0, 1, 4, None) == B.SWS_OK
    torch.cuda.synchronize()
    assert float(gw.abs().sum()) == 0.0


# ------------------------------------------------------------------------------ 2-D
# N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw
CASES_2D = [(2, 64, 20, 20, 64, 3, 3, 1, 1, 1, 1), (2, 16, 13, 17, 24, 3, 3, 1, 1, 0, 0), (1, 8, 30, 9, 40, 5, 5, 1, 1, 2, 2),
            (2, 32, 14, 14, 32, 1, 1, 1, 1, 0, 0), (1, 24, 12, 70, 8, 2, 4, 1, 1, 1, 3), (2, 8, 15, 15, 8, 3, 3, 2, 2, 1, 1),
            (1, 6, 11, 12, 10, 3, 3, 1, 1, 1, 1), (2, 16, 16, 16, 16, 3, 3, 2, 1, 1, 1), (1, 40, 9, 140, 72, 3, 7, 1, 1, 1, 3)]


def _data2d(case, seed, integer=False):
    n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
    ho, wo = (h + 2 * ph - kh) // sh + 1, (wd + 2 * pw - kw) // sw + 1
    if integer:
        return (workloads.integer_valued((n, cin, h, wd), -3, 3, seed), workloads.integer_valued((cout, cin, kh, kw), -3, 3, seed + 1),
                workloads.integer_valued((n, cout, ho, wo), -3, 3, seed + 2))
    r = np.random.Generator(np.random.PCG64(seed))
    return (r.standard_normal((n, cin, h, wd), dtype=np.float32),
            (r.standard_normal((cout, cin, kh, kw), dtype=np.float32) * np.float32(0.2)).astype(np.float32),
            r.standard_normal((n, cout, ho, wo), dtype=np.float32))


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("case", CASES_2D)
def test_conv2d_adjoints(B, case, integer):
    n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
    x, w, g = _data2d(case, 300 + kh * 7 + cin, integer)
    gx = to_host(B.sws_conv2d_grad_input(to_gpu(g), to_gpu(w), h, wd, sh, sw, ph, pw))
    gw = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, sw, ph, pw))
    rx, mx = oracle.conv2d_grad_input(g, w, h, wd, sh, sw, ph, pw)
    rw, mw = oracle.conv2d_grad_weight(x, g, kh, kw, sh, sw, ph, pw)
    if integer:
        assert np.array_equal(gx.astype(np.float64), rx) and np.array_equal(gw.astype(np.float64), rw), str(case)
    else:
        assert_within_tol(gx, rx, mx, "conv2d grad_input %s" % (case,))
        assert_within_tol(gw, rw, mw, "conv2d grad_weight %s" % (case,))


# short rows: several (image, output row) pairs share one 64-position slab of the dense grad-weight
# kernel; in the third case a slab holds more rows than an image has, in the last the rows are images
SHORT_ROWS_2D = [(3, 40, 7, 7, 33, 3, 3, 1, 1, 1, 1), (5, 16, 14, 14, 16, 3, 3, 1, 1, 1, 1), (33, 8, 5, 6, 8, 3, 3, 1, 1, 1, 1),
                 (2, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1), (7, 12, 3, 30, 20, 1, 5, 1, 1, 0, 2), (4, 8, 9, 4, 8, 3, 3, 1, 1, 1, 1)]
SHORT_ROWS_1D = [(37, 16, 12, 24, 3, 1, 1, 1, 1), (40, 8, 9, 8, 2, 1, 0, 3, 1), (9, 32, 31, 32, 1, 1, 0, 1, 1), (70, 8, 6, 8, 4, 1, 2, 1, 1)]


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("case", SHORT_ROWS_2D)
def test_conv2d_adjoints_short_rows(B, case, integer):
    test_conv2d_adjoints(B, case, integer)


@pytest.mark.parametrize("case", SHORT_ROWS_1D)
def test_conv1d_adjoints_short_rows(B, case):
    test_grad_weight(B, case)
    test_grad_input(B, case)
    test_exact_on_small_integers(B, case)


# stride 2 along the row on the matrix-core grad-weight kernel (plain and packed slabs)
STRIDE2_2D = [(2, 16, 28, 28, 24, 3, 3, 2, 2, 1, 1), (2, 32, 30, 30, 16, 1, 1, 2, 2, 0, 0), (2, 3, 40, 40, 16, 7, 7, 2, 2, 3, 3),
              (6, 8, 9, 13, 8, 3, 3, 2, 2, 1, 1), (1, 8, 12, 300, 8, 3, 3, 1, 2, 1, 1), (3, 8, 20, 33, 12, 2, 4, 3, 2, 0, 1)]
STRIDE2_1D = [(2, 16, 700, 24, 5, 2, 2, 3, 1), (3, 8, 1001, 8, 3, 2, 1, 1, 1), (20, 8, 25, 8, 3, 2, 1, 1, 1), (2, 40, 300, 33, 1, 2, 0, 1, 1)]


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("case", STRIDE2_2D)
def test_conv2d_adjoints_row_stride_2(B, case, integer):
    test_conv2d_adjoints(B, case, integer)


@pytest.mark.parametrize("case", STRIDE2_1D)
def test_conv1d_adjoints_stride_2(B, case):
    test_grad_weight(B, case)
    test_grad_input(B, case)
    test_exact_on_small_integers(B, case)


def test_strided_grad_input_by_phases_agrees_with_direct_evaluation(B):
    """Small-integer data: the phase-wise matrix-core route and the direct kernel must give the same bits."""
    for case in (STRIDE2_2D[0], STRIDE2_2D[2], STRIDE2_2D[5], (2, 8, 21, 22, 8, 2, 2, 3, 4, 1, 0)):
        n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
        x, w, g = _data2d(case, 91, integer=True)
        fast = to_host(B.sws_conv2d_grad_input(to_gpu(g), to_gpu(w), h, wd, sh, sw, ph, pw))
        B.sws_set_option("conv2d_variant", 1)
        try:
            direct = to_host(B.sws_conv2d_grad_input(to_gpu(g), to_gpu(w), h, wd, sh, sw, ph, pw))
        finally:
            B.sws_set_option("conv2d_variant", 0)
        assert np.array_equal(fast, direct), str(case)
        assert np.array_equal(fast.astype(np.float64), oracle.conv2d_grad_input(g, w, h, wd, sh, sw, ph, pw)[0]), str(case)


def test_packed_and_unpacked_slabs_agree(B):
    """The dense grad-weight kernel with and without row packing (option conv2d_variant = 3 turns it off)."""
    case = SHORT_ROWS_2D[1]
    n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
    x, w, g = _data2d(case, 77, integer=True)
    packed = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, sw, ph, pw))
    B.sws_set_option("conv2d_variant", 3)
    try:
        plain = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, sw, ph, pw))
    finally:
        B.sws_set_option("conv2d_variant", 0)
    assert np.array_equal(packed, plain)


def test_conv2d_adjoints_direct_evaluation_kernels(B):
    B.sws_set_option("conv2d_variant", 1)
    try:
        test_conv2d_adjoints(B, CASES_2D[0], False)
        test_conv2d_adjoints(B, CASES_2D[4], True)
    finally:
        B.sws_set_option("conv2d_variant", 0)


def test_conv2d_adjoints_resnet_layer_slice(B):
    """Configuration 4's layer (64 -> 64 channels, 3 x 3, pad 1, 56 x 56 planes) on 2 images."""
    test_conv2d_adjoints(B, (2, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1), False)


def test_graph_replay_of_the_adjoints_and_the_16_bit_sums(B):
    """The newer entry points also only enqueue kernels (gw is cleared by a fill kernel, not a
    memset): captured in a HIP graph and replayed with eager work between the replays they must give
    the eager results — bit for bit except gw, whose atomic adds land in no fixed order (small-integer
    data makes that exact too)."""
    import torch
    case = (2, 16, 1500, 24, 3, 1, 1, 1, 1)
    x, w, g = _data(case, 5, integer=True)
    xd, wd, gd = to_gpu(x), to_gpu(w), to_gpu(g)
    x16 = xd.to(torch.bfloat16)
    gx = torch.empty_like(xd)
    gw = torch.empty_like(wd)
    y16 = torch.empty(2, 16, 1500 - 63, device="cuda", dtype=torch.bfloat16)
    pe = torch.empty(2, 16, 750, 1, device="cuda")

    def launch_all():
        B.sws_conv1d_grad_input(gd, wd, 1500, 1, 1, 1, 1, gx=gx)
        B.sws_conv1d_grad_weight(xd, gd, 3, 1, 1, 1, 1, gw=gw)
        B.sws_slide1d_16(1, x16, 64, 1.0, y=y16)
        B.sws_pool2d_ex(0, xd.view(2, 16, 1500, 1), 3, 1, 2, 1, (1, 0, 1, 0), B.SWS_DIV_REAL_CELLS, 1.0, y=pe)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch_all()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        launch_all()
    for rep in range(3):
        gd.copy_(to_gpu(workloads.integer_valued(g.shape, -3, 3, 50 + rep)))      # eager work between replays
        for t in (gx, gw, pe):
            t.fill_(7.0)
        y16.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (gx, gw, y16, pe)]
        launch_all()
        torch.cuda.synchronize()
        for a, b in zip(got, (gx, gw, y16, pe)):
            assert torch.equal(a, b), "replay %d differs from the eager result" % rep
        ref, _ = oracle.conv1d_grad_weight(x, to_host(gd), 3, 1, 1, 1, 1)
        assert np.array_equal(to_host(got[1]).astype(np.float64), ref)


@pytest.mark.parametrize("variant", [17, 18])
@pytest.mark.parametrize("case", [(2, 64, 20, 20, 64, 3, 3, 1, 1, 1, 1), (3, 64, 9, 31, 128, 3, 3, 1, 1, 0, 1),
                                  (1, 64, 33, 62, 64, 3, 3, 1, 1, 2, 2), (5, 64, 6, 6, 64, 3, 3, 1, 1, 1, 0)])
def test_conv2d_grad_input_on_the_streaming_kernels(B, case, variant):
    """grad-input of 64-channel 3 x 3 layers through the adjoint weight view of the weight-stationary
    streaming kernels, forced on small problems: 17 = fp32 matrix instructions, 18 = bf16 ones with
    split operands.  Random data within tolerance, integer data bit for bit."""
    n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
    _, w, g = _data2d(case, 900 + h, False)
    _, wi, gi = _data2d(case, 901 + h, True)
    B.sws_set_option("conv2d_variant", variant)
    try:
        gx = to_host(B.sws_conv2d_grad_input(to_gpu(g), to_gpu(w), h, wd, sh, sw, ph, pw))
        gxi = to_host(B.sws_conv2d_grad_input(to_gpu(gi), to_gpu(wi), h, wd, sh, sw, ph, pw))
    finally:
        B.sws_set_option("conv2d_variant", 0)
    rx, mx = oracle.conv2d_grad_input(g, w, h, wd, sh, sw, ph, pw)
    assert_within_tol(gx, rx, mx, "streaming grad_input %s variant %d" % (case, variant))
    rxi, _ = oracle.conv2d_grad_input(gi, wi, h, wd, sh, sw, ph, pw)
    assert np.array_equal(gxi.astype(np.float64), rxi), "streaming grad_input, integers %s variant %d" % (case, variant)


# 3 x 3, horizontal stride 1, channel counts in multiples of 32: the grad-weight kernel on the bf16 matrix cores
# with split fp32 operands.  Rows that are not whole groups of 8 positions, blocks of 64 x 64 channels with an idle
# half, vertical strides, no padding, images whose groups split unevenly over the workgroups.
SPLIT_GW = [(2, 32, 20, 20, 32, 3, 3, 1, 1, 1, 1), (3, 96, 13, 13, 32, 3, 3, 1, 1, 1, 1), (1, 32, 9, 7, 160, 3, 3, 1, 1, 1, 1),
            (5, 64, 11, 30, 64, 3, 3, 2, 1, 1, 1), (2, 128, 10, 19, 64, 3, 3, 1, 1, 0, 0), (7, 32, 3, 3, 32, 3, 3, 1, 1, 1, 1),
            (2, 64, 17, 9, 96, 3, 3, 3, 1, 0, 2), (1, 32, 3, 5, 32, 3, 3, 1, 1, 0, 0),
            # rows in multiples of 4: the kernel's own shapes, stride 1 (pad 0 and 1) and stride 2
            (2, 32, 12, 16, 32, 3, 3, 1, 1, 0, 0), (3, 64, 9, 24, 32, 3, 3, 1, 1, 1, 1), (1, 32, 40, 8, 64, 3, 3, 1, 1, 1, 1),
            (2, 32, 28, 28, 32, 3, 3, 2, 2, 1, 1), (3, 64, 16, 24, 96, 3, 3, 2, 2, 1, 1), (1, 32, 8, 8, 32, 3, 3, 2, 2, 1, 1),
            (2, 32, 13, 16, 64, 3, 3, 2, 2, 1, 1), (5, 32, 56, 56, 32, 3, 3, 2, 2, 1, 1),
            # rows of any length: every element loaded on its own
            (2, 32, 14, 14, 32, 3, 3, 1, 1, 1, 1), (3, 64, 7, 7, 32, 3, 3, 1, 1, 1, 1), (2, 32, 14, 14, 32, 3, 3, 2, 2, 1, 1),
            (1, 32, 9, 13, 32, 3, 3, 1, 1, 0, 0), (2, 32, 15, 10, 64, 3, 3, 2, 2, 1, 1), (40, 32, 3, 3, 32, 3, 3, 1, 1, 1, 1)]


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("case", SPLIT_GW)
def test_split_operand_grad_weight(B, case, integer):
    n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
    x, _, g = _data2d(case, 500 + cin + wd, integer)
    gw = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, sw, ph, pw))
    rw, mw = oracle.conv2d_grad_weight(x, g, kh, kw, sh, sw, ph, pw)
    if integer:
        assert np.array_equal(gw.astype(np.float64), rw), str(case)
    else:
        worst = assert_within_tol(gw, rw, mw, "split grad_weight %s" % (case,))
        assert worst < 2e-6, (case, worst)                       # fp32 accuracy, not bf16's
    B.sws_set_option("conv2d_variant", 3)                        # the fp32-instruction kernel
    try:
        other = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, sw, ph, pw))
    finally:
        B.sws_set_option("conv2d_variant", 0)
    if integer:
        assert np.array_equal(gw, other), str(case)
    else:
        assert_within_tol(other, rw, mw, "fp32-instruction grad_weight %s" % (case,))


def test_split_operand_grad_weight_carries_every_bit(B):
    """Inputs whose low mantissa bits matter: x = 1 + k * 2^-23 against gradients of +-1 that cancel the ones —
    what is left lives entirely in the third bf16 piece."""
    r = np.random.Generator(np.random.PCG64(61))
    kx = r.integers(0, 128, size=(2, 32, 10, 16))
    x = (1.0 + kx * 2.0 ** -23).astype(np.float32)
    g = np.where(r.integers(0, 2, size=(2, 32, 10, 16)) > 0, 1.0, -1.0).astype(np.float32)
    gw = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), 3, 3, 1, 1, 1, 1))
    rw, mw = oracle.conv2d_grad_weight(x, g, 3, 3, 1, 1, 1, 1)
    assert_within_tol(gw, rw, mw, "low bits", tol=2e-7)


# ---- kernels one row high on the split-operand matrix-core kernel that walks along the row
# B, Cin, L, Cout, k, stride, pad, dilation, groups
SPLIT_GW_1D = [(3, 64, 1000, 64, 3, 1, 1, 1, 1), (2, 32, 333, 96, 3, 1, 0, 1, 1), (5, 96, 47, 32, 5, 1, 2, 1, 1),
               (2, 32, 16, 32, 1, 1, 0, 1, 1), (9, 160, 31, 32, 1, 1, 0, 1, 1), (40, 32, 5, 32, 3, 1, 1, 1, 1),
               (1, 32, 2049, 64, 5, 1, 4, 1, 1), (2, 64, 100, 32, 3, 1, 5, 1, 1), (1, 32, 3, 32, 3, 1, 0, 1, 1),
               # even row lengths: pairs of positions as one 64-bit load, staged from an even position (odd and even pads)
               (2, 32, 200, 32, 3, 1, 0, 1, 1), (2, 32, 130, 64, 5, 1, 2, 1, 1), (3, 32, 66, 32, 5, 1, 1, 1, 1),
               (2, 64, 64, 32, 1, 1, 0, 1, 1), (2, 32, 500, 32, 3, 1, 2, 1, 1), (1, 32, 2, 32, 1, 1, 0, 1, 1),
               (5, 32, 192, 32, 3, 1, 1, 1, 1), (1, 96, 4100, 32, 3, 1, 1, 1, 1), (2, 32, 70, 32, 5, 1, 3, 1, 1)]
# N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw: 1 x 1 layers (the plane as one row) and 1 x k layers (each image row a row)
SPLIT_GW_ROWS_2D = [(2, 64, 14, 14, 32, 1, 1, 1, 1, 0, 0), (3, 32, 7, 9, 96, 1, 1, 1, 1, 0, 0), (2, 32, 12, 21, 64, 1, 3, 1, 1, 0, 1),
                    (1, 64, 5, 40, 32, 1, 5, 1, 1, 0, 0), (4, 32, 6, 6, 32, 1, 3, 1, 1, 0, 2), (2, 32, 12, 20, 64, 1, 3, 1, 1, 0, 1),
                    (3, 32, 8, 8, 32, 1, 1, 1, 1, 0, 0)]


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("case", SPLIT_GW_1D)
def test_split_operand_grad_weight_rows_1d(B, case, integer):
    b, cin, length, cout, k, stride, pad, dil, groups = case
    x, _, g = _data(case, 700 + cin + length, integer)
    gw = to_host(B.sws_conv1d_grad_weight(to_gpu(x), to_gpu(g), k, stride, pad, dil, groups))
    ref, mag = oracle.conv1d_grad_weight(x, g, k, stride, pad, dil, groups)
    if integer:
        assert np.array_equal(gw.astype(np.float64), ref), str(case)
    else:
        worst = assert_within_tol(gw, ref, mag, "split grad_weight %s" % (case,))
        assert worst < 2e-6, (case, worst)                       # fp32 accuracy, not bf16's
    B.sws_set_option("conv1d_variant", 3)                        # keeps the split-operand kernel out
    try:
        other = to_host(B.sws_conv1d_grad_weight(to_gpu(x), to_gpu(g), k, stride, pad, dil, groups))
    finally:
        B.sws_set_option("conv1d_variant", 0)
    if integer:
        assert np.array_equal(gw, other), str(case)
    else:
        assert_within_tol(other, ref, mag, "fp32-instruction grad_weight %s" % (case,))


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("case", SPLIT_GW_ROWS_2D)
def test_split_operand_grad_weight_rows_2d(B, case, integer):
    n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
    x, _, g = _data2d(case, 800 + cin + wd, integer)
    gw = to_host(B.sws_conv2d_grad_weight(to_gpu(x), to_gpu(g), kh, kw, sh, sw, ph, pw))
    rw, mw = oracle.conv2d_grad_weight(x, g, kh, kw, sh, sw, ph, pw)
    if integer:
        assert np.array_equal(gw.astype(np.float64), rw), str(case)
    else:
        worst = assert_within_tol(gw, rw, mw, "split grad_weight %s" % (case,))
        assert worst < 2e-6, (case, worst)


def test_split_operand_grad_weight_rows_carry_every_bit(B):
    """x = 1 + k * 2^-23 against gradients of +-1: what survives the cancellation lives in the third bf16 piece."""
    r = np.random.Generator(np.random.PCG64(62))
    kx = r.integers(0, 128, size=(3, 32, 200))
    x = (1.0 + kx * 2.0 ** -23).astype(np.float32)
    g = np.where(r.integers(0, 2, size=(3, 32, 200)) > 0, 1.0, -1.0).astype(np.float32)
    gw = to_host(B.sws_conv1d_grad_weight(to_gpu(x), to_gpu(g), 3, 1, 1, 1, 1))
    ref, mag = oracle.conv1d_grad_weight(x, g, 3, 1, 1, 1, 1)
    assert_within_tol(gw, ref, mag, "low bits", tol=2e-7)


def test_split_operand_grad_weight_rows_at_full_size_on_sampled_channels(B):
    """The layers bench.py times on this kernel, whole: the 256 -> 256 channel 1-D layer on [32,256,3136] (k = 3, pad 1)
    and a 1 x 1 layer, 64 -> 256 channels on [32,64,56,56].  gw[co, ci, :] depends on channels co of gy and ci of x only,
    so the oracle evaluates the sampled channel pairs from those channels' slices."""
    r = np.random.Generator(np.random.PCG64(77))
    x = r.standard_normal((32, 256, 3136), dtype=np.float32)
    g = r.standard_normal((32, 256, 3136), dtype=np.float32)
    gw = to_host(B.sws_conv1d_grad_weight(to_gpu(x), to_gpu(g), 3, 1, 1, 1, 1))
    assert gw.shape == (256, 256, 3)
    cos, cis = np.array([0, 31, 32, 63, 64, 130, 200, 255]), np.array([0, 1, 33, 62, 65, 127, 192, 255])
    ref, mag = oracle.conv1d_grad_weight(np.ascontiguousarray(x[:, cis]), np.ascontiguousarray(g[:, cos]), 3, 1, 1, 1, 1)
    worst = assert_within_tol(gw[np.ix_(cos, cis)], ref, mag, "256 -> 256 layer, sampled channel pairs")
    assert worst < 2e-6, worst
    del x, g
    x2 = r.standard_normal((32, 64, 56, 56), dtype=np.float32)
    g2 = r.standard_normal((32, 256, 56, 56), dtype=np.float32)
    gw2 = to_host(B.sws_conv2d_grad_weight(to_gpu(x2), to_gpu(g2), 1, 1, 1, 1, 0, 0))
    cis2 = np.array([0, 5, 31, 32, 40, 63])
    ref2, mag2 = oracle.conv2d_grad_weight(np.ascontiguousarray(x2[:, cis2]), np.ascontiguousarray(g2[:, cos]), 1, 1, 1, 1, 0, 0)
    worst = assert_within_tol(gw2[np.ix_(cos, cis2)], ref2, mag2, "1 x 1 layer, sampled channel pairs")
    assert worst < 2e-6, worst
