"""GPU parity of sws_slide1d_padded (Eq. 3 over rows extended by identity / mirror / periodic /
edge padding, the boundary conditions Section 3 names) against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2305_16513_amd import workloads
from parity_util import assert_bit_exact, assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    yield binding
    binding.sws_set_option("slide_variant", 0)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _check(B, op, x, w, pl, pr, mode, what):
    scale = 1.0 / w if op == 0 else 1.0
    y = to_host(B.sws_slide1d_padded(op, to_gpu(x), w, pl, pr, mode, scale))
    ref, mag = oracle.slide1d_padded(op, x, w, pl, pr, mode, scale)
    if op == 0:
        assert_within_tol(y, ref, mag, what)
    else:
        assert_bit_exact(y, ref, what)


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("w,pl,pr", [(1, 3, 2), (2, 1, 0), (3, 1, 1), (5, 2, 2), (16, 15, 0), (31, 15, 15), (64, 0, 63),
                                     (255, 127, 127), (961, 480, 480), (1200, 600, 599)])
@pytest.mark.parametrize("length", [700, 3001])
def test_padded_modes_ops_windows(B, mode, op, w, pl, pr, length):
    r = _rng(mode * 1000 + op * 100 + w + length)
    x = (r.random((3, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    _check(B, op, x, w, pl, pr, mode, "mode=%d op=%d w=%d pads=(%d,%d) len=%d" % (mode, op, w, pl, pr, length))


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_padded_short_rows_and_extreme_pads(B, mode):
    r = _rng(40 + mode)
    for length, w, pl, pr in [(1, 1, 0, 0), (2, 2, 1, 1), (5, 3, 4, 4), (9, 17, 8, 8), (40, 9, 0, 39), (33, 64, 32, 32)]:
        if mode == 1 and (pl > length - 1 or pr > length - 1):
            continue
        if length + pl + pr < w:
            continue
        x = r.standard_normal((4, length), dtype=np.float32)
        for op in (0, 1, 2):
            _check(B, op, x, w, pl, pr, mode, "short len=%d w=%d pads=(%d,%d) mode=%d op=%d" % (length, w, pl, pr, mode, op))


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("w,pl,pr,length", [(962, 481, 480, 3000), (2000, 999, 1000, 5003), (2049, 0, 2048, 2100), (5000, 4000, 999, 6001),
                                            (1500, 1499, 0, 1600)])
def test_padded_windows_longer_than_a_tile(B, mode, op, w, pl, pr, length):
    """The default route (one pass of the long-window kernel, its loads through the boundary rule), the chain over the
    extended row (slide_variant 6) and the long-window kernel forced (8)."""
    r = _rng(mode * 7 + op * 3 + w)
    x = (r.random((3, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    _check(B, op, x, w, pl, pr, mode, "long mode=%d op=%d w=%d pads=(%d,%d) len=%d" % (mode, op, w, pl, pr, length))
    for variant in (6, 8):
        B.sws_set_option("slide_variant", variant)
        try:
            _check(B, op, x, w, pl, pr, mode, "variant %d mode=%d op=%d w=%d pads=(%d,%d) len=%d" % (variant, mode, op, w, pl, pr, length))
        finally:
            B.sws_set_option("slide_variant", 0)


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_same_size_pooling_with_long_windows(B, mode):
    r = _rng(90 + mode)
    x = (r.random((4, 9000), dtype=np.float32) * 2 - 1).astype(np.float32)
    for w in (513, 1025, 2049, 8191):
        for op in (0, 1):
            _check(B, op, x, w, w // 2, w // 2, mode, "same-size w=%d" % w)


def test_padded_zero_pads_match_the_unpadded_entry_point(B):
    r = _rng(44)
    x = r.standard_normal((5, 2500), dtype=np.float32)
    xg = to_gpu(x)
    for op in (0, 1, 2):
        for w in (1, 7, 200):
            a = to_host(B.sws_slide1d(op, xg, w, 0.5))
            for mode in range(4):
                b = to_host(B.sws_slide1d_padded(op, xg, w, 0, 0, mode, 0.5))
                assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_padded_integer_valued_add_is_exact(B):
    x = workloads.integer_valued((3, 4000), -8, 8, seed=9)
    for mode in range(4):
        y = to_host(B.sws_slide1d_padded(0, to_gpu(x), 33, 16, 16, mode, 1.0))
        ref, _ = oracle.slide1d_padded(0, x, 33, 16, 16, mode, 1.0)
        assert y.shape == x.shape and np.array_equal(y.astype(np.float64), ref)


def test_same_size_pooling_on_cfg2_shape(B):
    """'Same' average and max pooling of configuration 2's tensor (w = 3, one output per input)."""
    x, _ = workloads.make(2)
    xg = to_gpu(x)
    for op, mode in ((0, 0), (1, 0), (0, 1), (1, 3)):
        y = B.sws_slide1d_padded(op, xg, 3, 1, 1, mode, 1 / 3)
        assert y.shape == xg.shape
        ref, mag = oracle.slide1d_padded(op, x.reshape(-1, x.shape[-1]), 3, 1, 1, mode, 1 / 3)
        if op == 0:
            assert_within_tol(to_host(y).reshape(ref.shape), ref, mag, "cfg2 same avg mode %d" % mode)
        else:
            assert_bit_exact(to_host(y).reshape(ref.shape), ref, "cfg2 same max mode %d" % mode)


@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("w,pl,pr", [(1, 0, 0), (2, 1, 0), (3, 1, 1), (5, 4, 2), (16, 15, 0), (31, 15, 15), (64, 0, 63),
                                     (255, 127, 127), (961, 480, 480), (1200, 600, 599)])
@pytest.mark.parametrize("length", [700, 3001])
def test_shrinking_window_mode(B, op, w, pl, pr, length):
    """SWS_PAD_SHRINK: average over the real elements of a window that hangs over an end of the row."""
    r = _rng(5000 + op * 100 + w + length)
    x = (r.random((3, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    _check(B, op, x, w, pl, pr, 4, "shrink op=%d w=%d pads=(%d,%d) len=%d" % (op, w, pl, pr, length))


def test_shrinking_window_constant_row_and_argument_checks(B):
    x = np.full((2, 500), 3.0, np.float32)
    y = to_host(B.sws_slide1d_padded(0, to_gpu(x), 9, 4, 4, B.SWS_PAD_SHRINK, 1.0 / 9))
    assert np.abs(y - 3.0).max() < 1e-5
    with pytest.raises(B.SwsError):
        B.sws_slide1d_padded(0, to_gpu(x), 9, 9, 0, B.SWS_PAD_SHRINK, 1.0)


@pytest.mark.parametrize("variant", [0, 7])
@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("w,pl,pr", [(1, 2, 1), (2, 1, 0), (3, 1, 1), (4, 0, 3), (5, 2, 2), (8, 7, 0), (9, 4, 4), (16, 8, 7),
                                     (17, 0, 16), (25, 12, 12), (33, 16, 16), (33, 32, 0)])
def test_padded_short_row_kernel(B, variant, mode, w, pl, pr):
    """Rows of a few dozen to a few hundred elements with a boundary rule: the short-row kernel, as
    the library chooses it and forced (option slide_variant 7, also on longer rows)."""
    if mode == 4 and (pl >= w or pr >= w):
        pytest.skip("a shrinking window keeps at least one real element")
    B.sws_set_option("slide_variant", variant)
    try:
        for rows, length in ((7, 56), (300, 57), (40, 260), (130, 224), (5, 1031), (3, 5003), (64, 33), (9, 255)):
            if mode == 1 and (pl > length - 1 or pr > length - 1):
                continue
            if mode == 2 and (pl > length or pr > length):
                continue
            r = _rng(mode * 131 + w * 7 + length)
            x = (r.random((rows, length), dtype=np.float32) * 2 - 1).astype(np.float32)
            for op in (0, 1, 2):
                _check(B, op, x, w, pl, pr, mode, "short rows %dx%d w=%d pads=(%d,%d) mode=%d op=%d variant=%d" % (
                    rows, length, w, pl, pr, mode, op, variant))
    finally:
        B.sws_set_option("slide_variant", 0)

