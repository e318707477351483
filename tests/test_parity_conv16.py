"""GPU parity of sws_conv1d_16 (the sliding dot product of Section 2.5 on bf16 / fp16 storage, fp32
taps and arithmetic, one rounding per output) against the CPU oracle: round16(conv1d(x widened)).

The fp32 sum is within 1e-5 * sum|terms| of the exact one and is then rounded once, so
    |gpu - exact| <= 1e-5 * sum|terms| + half a step of the storage type at the fp32 value
(half a step: 2^-8 relative for bf16, 2^-11 for fp16, 2^-25 absolute for fp16 subnormals); and the
result must be the correctly rounded exact value for all but the rare outputs where the fp32 error
straddles a rounding boundary.  Integer-valued data (every partial sum exact and representable)
must match bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2305_16513_amd import workloads
from parity_util import TOL

pytestmark = pytest.mark.gpu

TYPES = {"bf16": (torch.bfloat16, oracle.DTYPE_BF16, 2.0 ** -8), "f16": (torch.float16, oracle.DTYPE_F16, 2.0 ** -11)}


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    yield binding
    binding.sws_set_option("conv1d_variant", 0)
    binding.sws_set_option("slide_group", 0)
    binding.sws_set_option("slide_chunk", 0)


def _check(B, kind, x32, wgt, what, min_exact=0.99, variant=0, **geom):
    """x32 [B, Cin, L] float32 host array, rounded to the storage type here (input preparation).
    variant: 0 the library's choice (matrix-core kernel for depthwise layers), 1 direct evaluation,
    2 the vector-ALU depthwise kernel."""
    tdt, odt, half_step = TYPES[kind]
    xq = torch.from_numpy(np.ascontiguousarray(x32)).to(tdt)               # the data both sides read
    B.sws_set_option("conv1d_variant", variant)
    try:
        y = B.sws_conv1d_16(xq.cuda(), torch.from_numpy(wgt).cuda(), **geom)
    finally:
        B.sws_set_option("conv1d_variant", 0)
    assert y.dtype == tdt
    got = y.cpu().to(torch.float64).numpy()
    ref, mag = oracle.conv1d(xq.to(torch.float32).numpy(), wgt, **geom)    # exact widening
    assert got.shape == ref.shape, what
    assert np.isfinite(got).all(), what
    allowed = TOL * mag + (np.abs(ref) + TOL * mag) * half_step + (2.0 ** -25 if kind == "f16" else 0.0)
    err = np.abs(got - ref)
    assert (err <= allowed).all(), "%s: %d outputs out of tolerance, worst %g of allowed" % (
        what, int((err > allowed).sum()), float((err / np.maximum(allowed, 1e-300)).max()))
    exact = oracle.round16(ref, odt)
    assert (got == exact).mean() > min_exact, "%s: only %.4f of the outputs are the correctly rounded sum" % (
        what, float((got == exact).mean()))


def _data(shape_x, shape_w, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal(shape_x, dtype=np.float32)
    w = rng.standard_normal(shape_w, dtype=np.float32) * np.float32(1.0 / np.sqrt(shape_w[1] * shape_w[2]))
    return x, w


@pytest.mark.parametrize("variant", [0, 2])
@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 18, 31, 32, 33, 34, 47, 48, 49, 50, 63, 64])
def test_depthwise_every_tap_count(B, kind, k, variant):
    """Depthwise rows of odd length (every row after the first starts on an odd 2-byte boundary, so
    no strip load is aligned) spanning several 1024-output tiles and a ragged tail."""
    x, w = _data((2, 3, 5003), (3, 1, k), 300 + k)
    _check(B, kind, x, w, "%s depthwise k=%d variant %d" % (kind, k, variant), variant=variant, groups=3)


@pytest.mark.parametrize("variant", [0, 2])
@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("length,k,pad", [(1, 1, 0), (2, 2, 0), (5, 5, 2), (9, 3, 1), (17, 16, 15), (31, 31, 0),
                                          (64, 64, 63), (255, 7, 3), (1023, 31, 15), (1024, 31, 15), (1025, 2, 1),
                                          (1054, 31, 0), (1055, 31, 0), (2047, 64, 0), (2048, 5, 4), (3000, 33, 32)])
def test_depthwise_short_rows_and_padding(B, kind, length, k, pad, variant):
    """Rows shorter than a tile, rows that end right at a tile edge, zero padding up to k-1."""
    x, w = _data((3, 5, length), (5, 1, k), 11 * length + k)
    _check(B, kind, x, w, "%s len=%d k=%d pad=%d variant %d" % (kind, length, k, pad, variant), min_exact=0.97,
           variant=variant, groups=5, pad=pad)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_channel_multiplier(B, kind):
    """groups = Cin with two output channels per input channel: still one input row per output row."""
    x, w = _data((2, 4, 2500), (8, 1, 9), 77)
    _check(B, kind, x, w, kind + " multiplier 2", groups=4, pad=4)


@pytest.mark.parametrize("variant", [0, 2])
@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("group", [1, 3, 4, 9])
def test_chunking_of_a_row(B, kind, group, variant):
    """The row is cut into runs of `group` tiles per work unit: every split must give the same outputs.
    (7 rows: the last workgroup of the matrix-core kernel has idle wavefronts.)"""
    B.sws_set_option("slide_group", group)
    try:
        x, w = _data((1, 7, 20011), (7, 1, 31), 5 + group)
        _check(B, kind, x, w, "%s group=%d variant %d" % (kind, group, variant), variant=variant, groups=7, pad=7)
    finally:
        B.sws_set_option("slide_group", 0)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("k", [3, 31, 40, 64])
def test_one_tile_in_flight(B, kind, k):
    """The matrix-core kernel with a single tile of loads ahead of the arithmetic (A/B knob)."""
    B.sws_set_option("slide_chunk", 1)
    try:
        x, w = _data((2, 3, 7001), (3, 1, k), 60 + k)
        _check(B, kind, x, w, "%s k=%d one tile ahead" % (kind, k), groups=3, pad=k // 2)
    finally:
        B.sws_set_option("slide_chunk", 0)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("geom", [
    dict(shape=(2, 6, 301), cout=4, k=5, stride=1, pad=2, dilation=1, groups=1),
    dict(shape=(2, 6, 301), cout=4, k=3, stride=2, pad=1, dilation=1, groups=2),
    dict(shape=(1, 4, 500), cout=4, k=7, stride=1, pad=0, dilation=3, groups=4),
    dict(shape=(3, 8, 130), cout=16, k=4, stride=3, pad=5, dilation=2, groups=4),
    dict(shape=(1, 3, 2000), cout=3, k=80, stride=1, pad=0, dilation=1, groups=3),      # more taps than the tuned path takes
])
def test_general_geometries(B, kind, geom):
    """Dense, grouped, strided and dilated layers (direct evaluation)."""
    g = dict(geom)
    shape, cout, k = g.pop("shape"), g.pop("cout"), g.pop("k")
    x, w = _data(shape, (cout, shape[1] // g["groups"], k), 900 + k)
    _check(B, kind, x, w, "%s %r" % (kind, geom), min_exact=0.97, **g)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_all_kernels_agree_with_the_oracle_on_the_same_layer(B, kind):
    x, w = _data((2, 3, 4100), (3, 1, 31), 41)
    for variant in (0, 1, 2):
        _check(B, kind, x, w, "%s variant %d" % (kind, variant), variant=variant, groups=3, pad=15)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_exact_on_small_integers(B, kind):
    """Integer taps and data: every product and partial sum is exact in fp32 and the results are
    representable in the storage type, so any summation order must reproduce the oracle's bits."""
    tdt = TYPES[kind][0]
    for variant in (0, 2):
        for k, pad in ((3, 1), (8, 0), (31, 15), (64, 0)):
            x = workloads.integer_valued((2, 4, 3001), -2, 2, seed=k)
            w = workloads.integer_valued((4, 1, k), -1, 1, seed=100 + k)
            B.sws_set_option("conv1d_variant", variant)
            try:
                y = B.sws_conv1d_16(torch.from_numpy(x).to(tdt).cuda(), torch.from_numpy(w).cuda(), pad=pad, groups=4)
            finally:
                B.sws_set_option("conv1d_variant", 0)
            ref, _ = oracle.conv1d(x, w, pad=pad, groups=4)
            assert np.abs(ref).max() <= 256
            assert np.array_equal(y.cpu().to(torch.float64).numpy(), ref), "variant %d k=%d" % (variant, k)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("variant", [0, 2])
def test_layer_shaped_rows(B, kind, variant):
    """A slab of the headline depthwise layer: 128 channels of 16384 elements, 31 taps, 2 images."""
    x, w = workloads.make(5, x_shape=(2, 128, 16384))
    _check(B, kind, x, w, "%s cfg5 slab variant %d" % (kind, variant), variant=variant, groups=128)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_taps_that_need_all_three_pieces(B, kind):
    """Taps with 24 significant bits and a wide spread of magnitudes (1e-6 .. 10) on data of mixed
    magnitude: the matrix-core kernel must carry every bit of every tap."""
    rng = np.random.Generator(np.random.PCG64(77))
    w = (rng.standard_normal((6, 1, 31)) * 10.0 ** rng.uniform(-6, 1, (6, 1, 31))).astype(np.float32)
    x = (rng.standard_normal((2, 6, 3000)) * 10.0 ** rng.uniform(-3, 1, (2, 6, 3000))).astype(np.float32)
    _check(B, kind, x, w, kind + " wide taps", min_exact=0.985, groups=6)


def test_output_guard_band(B):
    """Nothing is written outside y (ragged tails store element by element)."""
    x, w = _data((2, 3, 1500), (3, 1, 31), 9)
    xq = torch.from_numpy(x).to(torch.bfloat16).cuda()
    lo = 1500 - 30
    buf = torch.full((2 * 3 * lo + 128,), 7.0, dtype=torch.bfloat16, device="cuda")
    y = buf[64:64 + 2 * 3 * lo].view(2, 3, lo)
    B.sws_conv1d_16(xq, torch.from_numpy(w).cuda(), groups=3, y=y)
    torch.cuda.synchronize()
    assert bool((buf[:64] == 7.0).all()) and bool((buf[64 + 2 * 3 * lo:] == 7.0).all())
    want = B.sws_conv1d_16(xq, torch.from_numpy(w).cuda(), groups=3)
    assert torch.equal(y, want)


def test_argument_checks(B):
    x = torch.zeros(1, 4, 100, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(4, 1, 3, device="cuda")
    with pytest.raises(TypeError):
        B.sws_conv1d_16(x.float(), w, groups=4)
    with pytest.raises(B.SwsError):
        B.sws_conv1d_16(x, w, groups=2)
    with pytest.raises(B.SwsError):
        B.sws_conv1d_16(x, torch.zeros(4, 1, 101, device="cuda"), groups=4)
    assert B.lib().sws_conv1d_16(0, x.data_ptr(), w.data_ptr(), x.data_ptr(), 1, 4, 100, 4, 3, 1, 0, 1, 4, None) \
        == B.SWS_ERR_INVALID_ARG
