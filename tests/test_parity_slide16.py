"""GPU parity of sws_slide1d_16 (sliding window sums on bf16 / fp16 storage, fp32 arithmetic, one
rounding per output) against the CPU oracle: round16(slide1d(x widened)).

max / min of representable values is representable: bit-exact.  add: the fp32 sum is within
1e-5 * sum|terms| of the exact one and is then rounded once, so
    |gpu - exact| <= 1e-5 * sum|terms| + half a step of the storage type at the fp32 value
(half a step: 2^-8 relative for bf16, 2^-11 for fp16, 2^-25 absolute for fp16 subnormals); and
the result must be the correctly rounded exact value for all but the rare outputs where the fp32
error straddles a rounding boundary."""
import numpy as np
import pytest
import torch

import oracle
from paper_2305_16513_amd import workloads
from parity_util import TOL

pytestmark = pytest.mark.gpu

OPS = {"add": 0, "max": 1, "min": 2}
TYPES = {"bf16": (torch.bfloat16, oracle.DTYPE_BF16, 2.0 ** -8), "f16": (torch.float16, oracle.DTYPE_F16, 2.0 ** -11)}


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    yield binding
    binding.sws_set_option("slide_variant", 0)


def _check(B, op, kind, x32, w, scale=1.0, what=""):
    """x32: float32 host array; it is rounded to the storage type here (input preparation)."""
    tdt, odt, half_step = TYPES[kind]
    xq = torch.from_numpy(np.ascontiguousarray(x32)).to(tdt)              # the data both sides read
    y = B.sws_slide1d_16(OPS[op], xq.cuda(), w, scale)
    assert y.dtype == tdt
    got = y.cpu().to(torch.float64).numpy()
    xw = xq.to(torch.float32).numpy()                                      # exact widening
    ref, mag = oracle.slide1d(OPS[op], xw.reshape(-1, xw.shape[-1]), w, scale)
    ref, mag = ref.reshape(got.shape), mag.reshape(got.shape)
    if op != "add":
        assert np.array_equal(got, ref), "%s: %d outputs differ" % (what, int((got != ref).sum()))
        return
    assert np.isfinite(got).all(), what
    allowed = TOL * mag + (np.abs(ref) + TOL * mag) * half_step + (2.0 ** -25 if kind == "f16" else 0.0)
    err = np.abs(got - ref)
    assert (err <= allowed).all(), "%s: %d outputs out of tolerance, worst %g of allowed" % (
        what, int((err > allowed).sum()), float((err / np.maximum(allowed, 1e-300)).max()))
    exact = oracle.round16(ref, odt)
    assert (got == exact).mean() > 0.99, "%s: only %.4f of the outputs are the correctly rounded sum" % (
        what, float((got == exact).mean()))


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("w", [1, 2, 3, 5, 16, 17, 64, 100, 255, 256, 500, 961, 962, 1500])
def test_several_tiles_and_ragged_tail(B, kind, op, w):
    """3 rows of 5003 elements (odd: every row after the first starts on an odd 2-byte boundary)."""
    rng = np.random.Generator(np.random.PCG64(2000 + w))
    x = (rng.random((3, 5003), dtype=np.float32) * 2 - 1).astype(np.float32)
    _check(B, op, kind, x, w, scale=1.0 / w, what="%s %s w=%d" % (kind, op, w))


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("op", ["add", "max"])
@pytest.mark.parametrize("length,w", [(1, 1), (2, 2), (5, 5), (17, 16), (33, 2), (255, 255), (256, 255), (1023, 300),
                                      (1024, 64), (1025, 2), (2047, 1000), (1056, 33)])
def test_degenerate_and_short_rows(B, kind, op, length, w):
    rng = np.random.Generator(np.random.PCG64(length * 11 + w))
    x = rng.standard_normal((5, length), dtype=np.float32)
    _check(B, op, kind, x, w, what="%s %s len=%d w=%d" % (kind, op, length, w))


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("rows,length,w", [(64, 16384, 16), (64, 16384, 64), (64, 16384, 255), (257, 4096, 31),
                                           (7, 65536 + 13, 850)])
def test_layer_shaped_rows(B, kind, rows, length, w):
    """Rows of the headline workload's length (and a short-row and a long-row relative)."""
    x, _ = workloads.make(5, x_shape=(rows, length), wgt_shape=(1, 1, 1), seed_offset=w)
    for op in ("add", "max"):
        _check(B, op, kind, x, w, scale=1.0 / w, what="%s %s %dx%d w=%d" % (kind, op, rows, length, w))


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_add_is_exact_on_small_integers(B, kind):
    """Sums of small integers are exact in fp32 and representable in the storage type: any
    association order must give exactly the oracle's value."""
    x = workloads.integer_valued((4, 3001), -4, 4, seed=5)
    for w in (3, 16, 64):
        tdt = TYPES[kind][0]
        y = B.sws_slide1d_16(0, torch.from_numpy(x).to(tdt).cuda(), w, 1.0).cpu().to(torch.float64).numpy()
        ref, _ = oracle.slide1d(0, x, w, 1.0)
        assert np.array_equal(y, ref)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("w", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 15, 16, 17, 18, 24, 25, 26, 31, 32, 33, 34])
@pytest.mark.parametrize("rows,length", [(3, 5003), (300, 56), (1000, 9), (5, 520), (2, 1031), (40, 512 + 8), (17, 24)])
def test_small_windows_on_both_kernels(B, kind, w, rows, length):
    """Windows up to 33 have two kernels (shifted loads; the scan).  Both are forced in turn, with x
    and y starting 2 bytes past a 16-byte boundary as well, so that the strips' alignment to y is
    exercised for every phase; memory around y must stay untouched."""
    if w > length:
        pytest.skip("window longer than the row")
    tdt, odt, half_step = TYPES[kind]
    rng = np.random.Generator(np.random.PCG64(77 * w + length))
    x32 = (rng.random((rows, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    xq = torch.from_numpy(x32).to(tdt)
    xw = xq.to(torch.float32).numpy()
    lo = length - w + 1
    try:
        for variant in (2, 3):
            B.sws_set_option("slide_variant", variant)
            for shift in (0, 1, 5):
                xbuf = torch.zeros(rows * length + 8, dtype=tdt, device="cuda")
                xs = xbuf[shift:shift + rows * length].view(rows, length)
                xs.copy_(xq)
                ybuf = torch.full((rows * lo + 16,), 7.0, dtype=tdt, device="cuda")
                ys = ybuf[shift:shift + rows * lo].view(rows, lo)
                for op in ("add", "max", "min"):
                    B.sws_slide1d_16(OPS[op], xs, w, 1.0, y=ys)
                    got = ys.cpu().to(torch.float64).numpy()
                    ref, mag = oracle.slide1d(OPS[op], xw, w, 1.0)
                    what = "%s %s w=%d %dx%d variant %d shift %d" % (kind, op, w, rows, length, variant, shift)
                    if op != "add":
                        assert np.array_equal(got, ref), what
                    else:
                        allowed = TOL * mag + (np.abs(ref) + TOL * mag) * half_step + (2.0 ** -25 if kind == "f16" else 0.0)
                        assert (np.abs(got - ref) <= allowed).all(), what
                    guard = ybuf.cpu().to(torch.float32)
                    assert (guard[:shift] == 7.0).all() and (guard[shift + rows * lo:] == 7.0).all(), what
    finally:
        B.sws_set_option("slide_variant", 0)


def test_argument_checks(B):
    x = torch.zeros((2, 100), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.SwsError):
        B.sws_slide1d_16(0, x, 101)
    with pytest.raises(TypeError):
        B.sws_slide1d_16(0, x.float(), 3)
    assert B.lib().sws_slide1d_16(0, 7, x.data_ptr(), x.data_ptr(), 2, 100, 3, 1.0, None) == B.SWS_ERR_INVALID_ARG
    assert B.lib().sws_slide1d_16(5, 1, x.data_ptr(), x.data_ptr(), 2, 100, 3, 1.0, None) == B.SWS_ERR_INVALID_ARG


# ------------------------------------------------------------------------------ 2-D pooling on 16-bit storage
POOL_GEOMS = [(3, 3, 1, 1, 1, 1), (3, 3, 2, 2, 1, 1), (2, 2, 2, 2, 0, 0), (5, 5, 1, 1, 2, 2), (7, 7, 1, 1, 3, 3),
              (4, 4, 4, 4, 0, 0), (11, 11, 1, 1, 5, 5), (1, 7, 1, 1, 0, 3), (6, 3, 2, 1, 2, 1)]


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("geom", POOL_GEOMS)
@pytest.mark.parametrize("shape", [(2, 3, 37, 53), (1, 4, 112, 112), (2, 2, 9, 3000)])
def test_pool2d_16(B, kind, op, geom, shape):
    """sws_pool2d_16 against round16(pool2d(x widened)): specialised band kernels, the run-time
    separable kernel, and (the 3000-wide planes) direct evaluation."""
    kh, kw, sh, sw, ph, pw = geom
    tdt, odt, half_step = TYPES[kind]
    rng = np.random.Generator(np.random.PCG64(kh * 97 + kw * 13 + shape[3]))
    xq = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(tdt)
    scale = 1.0 / (kh * kw)
    y = B.sws_pool2d_16(OPS[op], xq.cuda(), kh, kw, sh, sw, ph, pw, scale)
    assert y.dtype == tdt
    got = y.cpu().to(torch.float64).numpy()
    ref, mag = oracle.pool2d(OPS[op], xq.to(torch.float32).numpy(), kh, kw, sh, sw, ph, pw, scale)
    what = "%s %s %s %s" % (kind, op, geom, shape)
    if op != "add":
        assert np.array_equal(got, ref), what
        return
    allowed = TOL * mag + (np.abs(ref) + TOL * mag) * half_step + (2.0 ** -25 if kind == "f16" else 0.0)
    assert (np.abs(got - ref) <= allowed).all(), what
    # (sums of normal data cancel: the fp32 error is a larger share of a 16-bit step than for the sliding sums above)
    assert (got == oracle.round16(ref, odt)).mean() > 0.97, what


def test_pool2d_16_argument_checks(B):
    x = torch.zeros((1, 2, 8, 8), dtype=torch.float16, device="cuda")
    with pytest.raises(TypeError):
        B.sws_pool2d_16(0, x.float(), 3, 3)
    assert B.lib().sws_pool2d_16(0, 0, x.data_ptr(), x.data_ptr(), 1, 2, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, None) == B.SWS_ERR_INVALID_ARG
    assert B.lib().sws_pool2d_16(0, 2, x.data_ptr(), x.data_ptr(), 1, 2, 8, 8, 3, 3, 1, 1, 3, 1, 1.0, None) == B.SWS_ERR_INVALID_ARG


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("op", ["add", "max", "min"])
@pytest.mark.parametrize("w,length", [(257, 300), (512, 2000), (513, 5003), (962, 5003), (1024, 4097), (1025, 1025), (2048, 9001), (5000, 16384)])
def test_windows_longer_than_a_tile_in_one_pass(B, kind, op, w, length):
    """The long-window kernel on 16-bit storage (forced from w = 257 by slide_variant 8; the default from w = 962),
    and direct evaluation (slide_variant 1) beside it."""
    rng = np.random.Generator(np.random.PCG64(3000 + w + length))
    x = (rng.random((3, length), dtype=np.float32) * 2 - 1).astype(np.float32)
    for variant in (8, 0, 1):
        B.sws_set_option("slide_variant", variant)
        try:
            _check(B, op, kind, x, w, scale=1.0 / w, what="%s %s w=%d variant %d" % (kind, op, w, variant))
        finally:
            B.sws_set_option("slide_variant", 0)
