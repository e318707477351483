"""GPU parity of sws_slide1d_pair (sliding window sum under the non-commutative pair operator
of Section 2.4, Eq. 8) and of the generic-operator kernel run with +, max, min, against the
CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2305_16513_amd import workloads
from parity_util import assert_bit_exact, assert_within_tol, to_gpu, to_host

pytestmark = pytest.mark.gpu


def pair_tol(w):
    """A fold of w pairs puts at most w - 1 product roundings and (tree depth <= 24) fma roundings
    on any term: |err| <= (w + 24) * 2^-24 * (sum of |terms|) to first order."""
    return (w + 24) * 2.0 ** -24


@pytest.fixture(scope="module")
def B():
    from paper_2305_16513_amd import binding
    binding.lib()
    yield binding
    binding.sws_set_option("slide_variant", 0)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _pairs(r, shape):
    u = (1.0 + 0.03 * (2.0 * r.random(shape) - 1.0)) * np.where(r.random(shape) < 0.2, -1.0, 1.0)
    v = r.standard_normal(shape)
    return u.astype(np.float32), v.astype(np.float32)


def _check(B, u, v, w, what):
    yu, yv = B.sws_slide1d_pair(to_gpu(u), to_gpu(v), w)
    ru, rv, mu, mv = oracle.slide1d_pair(u, v, w)
    a = assert_within_tol(to_host(yu), ru, mu, what + " u", tol=pair_tol(w))
    b = assert_within_tol(to_host(yv), rv, mv, what + " v", tol=pair_tol(w))
    return max(a, b)


@pytest.mark.parametrize("w", [1, 2, 3, 4, 5, 8, 16, 17, 64, 255, 309, 310, 449, 600, 961, 962, 1500, 2500])
@pytest.mark.parametrize("length", [64, 700, 1500, 4099])
def test_pair_windows_and_ragged_lengths(B, w, length):
    if w > length:
        pytest.skip("window longer than the row")
    r = _rng(w * 10000 + length)
    u, v = _pairs(r, (3, length))
    _check(B, u, v, w, "w=%d len=%d" % (w, length))


@pytest.mark.parametrize("w", [2, 7, 64, 255, 700, 2000])
def test_pair_exact_on_signs_and_small_integers(B, w):
    """u in {-1, +1}, v small integers: every partial result is exact in fp32, so the GPU must
    agree bit for bit whatever its association order — and the order of operands must be right."""
    r = _rng(500 + w)
    u = np.where(r.random((4, 3001)) < 0.5, -1.0, 1.0).astype(np.float32)
    v = r.integers(-8, 9, size=(4, 3001)).astype(np.float32)
    yu, yv = B.sws_slide1d_pair(to_gpu(u), to_gpu(v), w)
    ru, rv, _, _ = oracle.slide1d_pair(u, v, w)
    assert np.array_equal(to_host(yu).astype(np.float64), ru)
    assert np.array_equal(to_host(yv).astype(np.float64), rv)


def test_pair_reduces_to_sliding_add_and_sliding_product(B):
    r = _rng(77)
    v = r.standard_normal((5, 2000)).astype(np.float32)
    yu, yv = B.sws_slide1d_pair(to_gpu(np.ones_like(v)), to_gpu(v), 31)
    ref, mag = oracle.slide1d(oracle.OP_ADD, v, 31)
    assert np.array_equal(to_host(yu), np.ones((5, 1970), np.float32))
    assert_within_tol(to_host(yv), ref, mag, "u = 1")
    u = np.exp2(r.integers(-1, 2, size=(5, 2000))).astype(np.float32)       # powers of two: exact products
    yu, yv = B.sws_slide1d_pair(to_gpu(u), to_gpu(np.zeros_like(u)), 20)
    ru, _, _, _ = oracle.slide1d_pair(u, np.zeros_like(u), 20)
    assert np.array_equal(to_host(yu).astype(np.float64), ru) and not to_host(yv).any()


def test_pair_dot_product_as_one_window(B):
    """Eq. 5, 7, 9 on the GPU: the pairs built from (taps, x), folded over one window of M + 1
    pairs, carry the dot product; compared with the convolution oracle (Eq. 4)."""
    r = _rng(78)
    M = 31
    taps = r.standard_normal(M).astype(np.float32)
    taps[[3, 17]] = 0.0
    x = r.standard_normal((64, M)).astype(np.float32)
    al = np.where(taps == 0, 1.0, taps).astype(np.float64)
    u = np.concatenate([[1.0], al[:-1] / al[1:], [al[-1]]]).astype(np.float32)
    v = np.concatenate([np.where(taps == 0, 0.0, 1.0) * x, np.zeros((64, 1))], axis=1).astype(np.float32)
    _, yv = B.sws_slide1d_pair(to_gpu(np.broadcast_to(u, v.shape).copy()), to_gpu(v), M + 1)
    ref, mag = oracle.conv1d(x.reshape(64, 1, M), taps.reshape(1, 1, M))
    # the ratios alpha_{i-1} / alpha_i are rounded to fp32 once more than in the direct sum
    _, _, _, mv = oracle.slide1d_pair(np.broadcast_to(u, v.shape).copy(), v, M + 1)
    assert np.all(np.abs(to_host(yv)[:, 0] - ref[:, 0, 0]) <= 2 * pair_tol(M + 1) * mv[:, 0])


@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("w", [2, 5, 16, 64, 255, 309, 310, 961])
def test_generic_kernel_with_scalar_operators(B, op, w):
    """The generic-operator kernel instantiated for +, max, min, selected instead of the tuned one."""
    r = _rng(900 + op * 10 + w)
    x = (r.random((3, 5000), dtype=np.float32) * 2 - 1).astype(np.float32)
    B.sws_set_option("slide_variant", 4)
    try:
        y = to_host(B.sws_slide1d(op, to_gpu(x), w, 1.0 / w))
    finally:
        B.sws_set_option("slide_variant", 0)
    ref, mag = oracle.slide1d(op, x, w, 1.0 / w)
    if op == 0:
        assert_within_tol(y, ref, mag, "generic add w=%d" % w)
    else:
        assert_bit_exact(y, ref, "generic op %d w=%d" % (op, w))


def test_pair_full_size(B):
    """[8192, 16384] pairs (1 GiB in, 1 GiB out) in the launch shape the bench times; the oracle
    checks a seeded sample of whole rows, first and last included."""
    import torch
    rows, length = 8192, 16384
    r = _rng(79)
    u, v = workloads.make_pairs((rows, length))
    ug, vg = to_gpu(u), to_gpu(v)
    sample = sorted(set([0, rows - 1] + r.integers(0, rows, size=6).tolist()))
    for w in (16, 255):
        yu, yv = B.sws_slide1d_pair(ug, vg, w)
        ru, rv, mu, mv = oracle.slide1d_pair(u[sample], v[sample], w)
        assert_within_tol(to_host(yu[sample]), ru, mu, "full size u w=%d" % w, tol=pair_tol(w))
        assert_within_tol(to_host(yv[sample]), rv, mv, "full size v w=%d" % w, tol=pair_tol(w))
        assert bool(yu.isfinite().all()) and bool(yv.isfinite().all())
        del yu, yv
    del ug, vg
    torch.cuda.empty_cache()
