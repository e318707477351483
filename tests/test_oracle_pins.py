"""Pins for the CPU oracle: everything here checks oracle/ against something other
than itself — hand-enumerated values, closed forms, invariants, the paper's own
algorithms emulated step by step, and library routines as a third opinion.

The paper prints no worked numeric example, so there are no paper-printed values
to match; Fig. 1 / Fig. 2 speedups are "parity unpinned" (they need the authors'
CPU and baseline library).
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import OP_ADD, OP_MAX, OP_MIN

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "slide_hand_cases.txt")
OPS = {"add": OP_ADD, "max": OP_MAX, "min": OP_MIN}


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ----------------------------------------------------------------------------- P1
def _hand_cases():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            op, w, xs, ys = [p.strip() for p in line.split(";")]
            out.append((op, int(w), [float(v) for v in xs.split()], [float(v) for v in ys.split()]))
    return out


@pytest.mark.parametrize("op,w,xs,ys", _hand_cases())
def test_hand_enumerated(op, w, xs, ys):
    """Section 2.2 Eq. 3 on tiny inputs worked out by hand (tests/golden)."""
    y, _ = oracle.slide1d(OPS[op], np.array(xs, np.float32), w)
    assert y.shape == (1, len(xs) - w + 1)
    assert y[0].tolist() == ys


def test_output_count_and_w_equals_len():
    """Exactly w addends per output => len-w+1 outputs; w = len is the full reduction (Eq. 1 last element)."""
    x = _rng(1).integers(-9, 10, size=(3, 17)).astype(np.float32)
    for w in (1, 2, 16, 17):
        y, _ = oracle.slide1d(OP_ADD, x, w)
        assert y.shape == (3, 17 - w + 1)
    y, _ = oracle.slide1d(OP_ADD, x, 17)
    assert y[:, 0].tolist() == x.astype(np.float64).sum(axis=1).tolist()
    with pytest.raises(ValueError):
        oracle.slide1d(OP_ADD, x, 18)
    with pytest.raises(ValueError):
        oracle.slide1d(OP_ADD, x, 0)


def test_rows_do_not_bleed():
    """Each row is its own sequence: a window never crosses from one row into the next."""
    x = np.array([[1, 2, 3, 4], [100, 200, 300, 400]], np.float32)
    y, _ = oracle.slide1d(OP_ADD, x, 3)
    assert y.tolist() == [[6, 9], [600, 900]]
    y, _ = oracle.slide1d(OP_MAX, x, 2)
    assert y.tolist() == [[2, 3, 4], [200, 300, 400]]


# ----------------------------------------------------------------------------- P2
@pytest.mark.parametrize("w", [1, 2, 5, 16, 255])
def test_constant_closed_form(w):
    c = 3.0
    x = np.full((2, 300), c, np.float32)
    y, s = oracle.slide1d(OP_ADD, x, w)
    assert np.all(y == w * c) and np.all(s == w * c)
    y, _ = oracle.slide1d(OP_MAX, x, w)
    assert np.all(y == c)
    y, _ = oracle.slide1d(OP_MIN, x, w)
    assert np.all(y == c)
    y, _ = oracle.slide1d(OP_ADD, x, w, scale=0.5)
    assert np.all(y == 0.5 * w * c)


def test_pool2d_constant_border_counts():
    """3x3, pad 1 on a constant plane: interior sees 9 cells, an edge 6, a corner 4."""
    c = 2.0
    x = np.full((1, 2, 6, 7), c, np.float32)
    y, _ = oracle.pool2d(OP_ADD, x, 3, 3, 1, 1, 1, 1, scale=1.0)
    assert y.shape == (1, 2, 6, 7)
    assert y[0, 0, 0, 0] == 4 * c and y[0, 1, 5, 6] == 4 * c and y[0, 0, 0, 6] == 4 * c
    assert y[0, 0, 0, 3] == 6 * c and y[0, 0, 2, 0] == 6 * c and y[0, 0, 5, 2] == 6 * c
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * c)
    y, _ = oracle.pool2d(OP_ADD, x, 3, 3, 1, 1, 1, 1, scale=1.0 / 8.0)
    assert y[0, 0, 0, 0] == 4 * c / 8 and y[0, 0, 2, 2] == 9 * c / 8
    # max with identity padding: padding never wins, even on an all-negative plane
    y, _ = oracle.pool2d(OP_MAX, -x, 3, 3, 1, 1, 1, 1)
    assert np.all(y == -c)
    y, _ = oracle.pool2d(OP_MIN, x, 3, 3, 1, 1, 1, 1)
    assert np.all(y == c)


def test_conv_constant_closed_form():
    """Constant input c: every valid output equals c * sum of taps."""
    taps = np.array([[[1, -2, 4, 8, -16]]], np.float32)
    x = np.full((1, 1, 40), 3.0, np.float32)
    y, s = oracle.conv1d(x, taps)
    assert np.all(y == 3.0 * taps.sum()) and np.all(s == 3.0 * np.abs(taps).sum())
    w2 = np.arange(1, 19, dtype=np.float32).reshape(1, 2, 3, 3)
    x2 = np.full((1, 2, 5, 5), 2.0, np.float32)
    y, _ = oracle.conv2d(x2, w2)
    assert y.shape == (1, 1, 3, 3) and np.all(y == 2.0 * w2.sum())


# ----------------------------------------------------------------------------- P3
@pytest.mark.parametrize("w", [2, 5, 31])
@pytest.mark.parametrize("b", [3, -2])
def test_ramp_closed_form(w, b):
    a, n = 7, 200
    j = np.arange(n, dtype=np.float64)
    x = (a + b * j).astype(np.float32)
    i = np.arange(n - w + 1, dtype=np.float64)
    y, _ = oracle.slide1d(OP_ADD, x, w)
    assert np.all(y[0] == w * a + b * (w * i + w * (w - 1) / 2))
    y, _ = oracle.slide1d(OP_MAX, x, w)
    assert np.all(y[0] == (a + b * (i + w - 1) if b > 0 else a + b * i))
    y, _ = oracle.slide1d(OP_MIN, x, w)
    assert np.all(y[0] == (a + b * i if b > 0 else a + b * (i + w - 1)))


# ----------------------------------------------------------------------------- P4
@pytest.mark.parametrize("w", [1, 3, 16, 64, 255])
def test_add_equals_prefix_sum_difference_exact(w):
    """Integer-valued data: y_i = S_{i+w} - S_i exactly, and y_{i+1} = y_i - x_i + x_{i+w}."""
    x = _rng(w).integers(-50, 51, size=(4, 700)).astype(np.float32)
    y, s = oracle.slide1d(OP_ADD, x, w)
    S = np.concatenate([np.zeros((4, 1)), np.cumsum(x.astype(np.float64), axis=1)], axis=1)
    assert np.array_equal(y, S[:, w:] - S[:, :-w])
    assert np.array_equal(y[:, 1:], y[:, :-1] - x[:, :-w] + x[:, w:])
    A = np.concatenate([np.zeros((4, 1)), np.cumsum(np.abs(x).astype(np.float64), axis=1)], axis=1)
    assert np.array_equal(s, A[:, w:] - A[:, :-w])


@pytest.mark.parametrize("w", [3, 16, 255])
def test_add_prefix_difference_real_valued(w):
    x = (_rng(10 + w).random((2, 1000), dtype=np.float32) * 2 - 1).astype(np.float32)
    y, s = oracle.slide1d(OP_ADD, x, w, scale=1.0 / w)
    S = np.concatenate([np.zeros((2, 1)), np.cumsum(x.astype(np.float64), axis=1)], axis=1)
    assert np.allclose(y * w, S[:, w:] - S[:, :-w], rtol=0, atol=1e-11)
    assert np.all(s > 0)


@pytest.mark.parametrize("w", [2, 5, 64])
@pytest.mark.parametrize("op", [OP_MAX, OP_MIN])
def test_extremum_membership_and_bound(op, w):
    """max: y_i >= every element of its window and is one of them (min mirrored)."""
    x = _rng(100 + w).standard_normal((3, 400), dtype=np.float32)
    y, _ = oracle.slide1d(op, x, w)
    win = np.lib.stride_tricks.sliding_window_view(x.astype(np.float64), w, axis=1)
    if op == OP_MAX:
        assert np.all(y[..., None] >= win)
    else:
        assert np.all(y[..., None] <= win)
    assert np.all((y[..., None] == win).any(axis=-1))
    # exact in fp32 too: converting back loses nothing
    assert np.array_equal(y.astype(np.float32).astype(np.float64), y)


# ----------------------------------------------------------------------------- P5
def test_conv_all_ones_taps_is_sliding_add():
    x = _rng(5).integers(-20, 21, size=(2, 3, 90)).astype(np.float32)
    for k in (1, 3, 8):
        taps = np.ones((3, 1, k), np.float32)
        yc, _ = oracle.conv1d(x, taps, groups=3)
        ys, _ = oracle.slide1d(OP_ADD, x.reshape(6, 90), k)
        assert np.array_equal(yc.reshape(6, -1), ys)


def test_conv_one_hot_tap_is_shift_no_flip():
    """A one-hot tap e_t picks x[i+t]: cross-correlation, taps are NOT reversed."""
    x = _rng(6).integers(-20, 21, size=(1, 1, 50)).astype(np.float32)
    k = 5
    for t in range(k):
        taps = np.zeros((1, 1, k), np.float32)
        taps[0, 0, t] = 1
        y, _ = oracle.conv1d(x, taps)
        assert np.array_equal(y[0, 0], x[0, 0, t:t + 50 - k + 1].astype(np.float64))


def test_conv_linearity():
    r = _rng(7)
    x1 = r.integers(-9, 10, size=(2, 3, 40)).astype(np.float32)
    x2 = r.integers(-9, 10, size=(2, 3, 40)).astype(np.float32)
    w1 = r.integers(-4, 5, size=(4, 3, 3)).astype(np.float32)
    w2 = r.integers(-4, 5, size=(4, 3, 3)).astype(np.float32)
    f = lambda x, w: oracle.conv1d(x, w, stride=2, pad=1)[0]
    assert np.array_equal(f(x1 + x2, w1), f(x1, w1) + f(x2, w1))
    assert np.array_equal(f(x1, w1 + w2), f(x1, w1) + f(x1, w2))


def test_conv1d_channels_sum_and_groups():
    """groups=1 sums over input channels; depthwise equals each channel convolved alone."""
    r = _rng(8)
    x = r.integers(-9, 10, size=(2, 4, 30)).astype(np.float32)
    w = r.integers(-4, 5, size=(3, 4, 5)).astype(np.float32)
    y, _ = oracle.conv1d(x, w)
    acc = np.zeros_like(y)
    for ci in range(4):
        acc += oracle.conv1d(x[:, ci:ci + 1], w[:, ci:ci + 1])[0]
    assert np.array_equal(y, acc)
    wd = r.integers(-4, 5, size=(4, 1, 5)).astype(np.float32)
    yd, _ = oracle.conv1d(x, wd, groups=4)
    for c in range(4):
        assert np.array_equal(yd[:, c:c + 1], oracle.conv1d(x[:, c:c + 1], wd[c:c + 1])[0])


def test_conv1d_padding_stride_dilation_by_hand():
    x = np.array([[[1, 2, 3, 4, 5, 6]]], np.float32)
    w = np.array([[[1, 10, 100]]], np.float32)
    assert oracle.conv1d(x, w)[0][0, 0].tolist() == [321, 432, 543, 654]
    assert oracle.conv1d(x, w, pad=1)[0][0, 0].tolist() == [210, 321, 432, 543, 654, 65]
    assert oracle.conv1d(x, w, stride=2)[0][0, 0].tolist() == [321, 543]
    assert oracle.conv1d(x, w, dilation=2)[0][0, 0].tolist() == [531, 642]
    assert oracle.conv1d(x, w, stride=2, pad=2, dilation=2)[0][0, 0].tolist() == [310, 531, 53]


def test_conv2d_rank1_taps_separate():
    """Taps u v^T: 2-D correlation = 1-D along W with v, then 1-D along H with u."""
    r = _rng(9)
    x = r.integers(-9, 10, size=(1, 1, 9, 11)).astype(np.float32)
    u = np.array([1, -2, 3], np.float32)
    v = np.array([2, 0, -1, 4], np.float32)
    w2 = np.outer(u, v).reshape(1, 1, 3, 4).astype(np.float32)
    y2, _ = oracle.conv2d(x, w2)
    rows = oracle.conv1d(x.reshape(9, 1, 11), v.reshape(1, 1, 4))[0].reshape(9, 8)
    cols = oracle.conv1d(np.ascontiguousarray(rows.T.astype(np.float32)).reshape(8, 1, 9), u.reshape(1, 1, 3))[0]
    assert np.array_equal(y2[0, 0], cols.reshape(8, 7).T)


def test_conv2d_asymmetric_by_hand():
    """kh != kw, H != W, distinct strides/pads: catches swapped H/W indices."""
    x = np.arange(1, 13, dtype=np.float32).reshape(1, 1, 3, 4)
    w = np.array([[[[1, 10]]]], np.float32)          # kh=1, kw=2
    y, _ = oracle.conv2d(x, w)
    assert y[0, 0].tolist() == [[21, 32, 43], [65, 76, 87], [109, 120, 131]]
    y, _ = oracle.conv2d(x, w, sh=2, sw=1, ph=0, pw=1)
    assert y[0, 0].tolist() == [[10, 21, 32, 43, 4], [90, 109, 120, 131, 12]]
    wt = np.array([[[[1], [10]]]], np.float32)       # kh=2, kw=1
    y, _ = oracle.conv2d(x, wt)
    assert y[0, 0].tolist() == [[51, 62, 73, 84], [95, 106, 117, 128]]


@pytest.mark.parametrize("op", [OP_ADD, OP_MAX, OP_MIN])
def test_pool2d_is_separable_sliding_sums(op):
    """pool2d (no padding) = slide1d down H then along W."""
    x = _rng(11).integers(-30, 31, size=(2, 2, 10, 13)).astype(np.float32)
    kh, kw = 3, 4
    y, _ = oracle.pool2d(op, x, kh, kw)
    cols = np.ascontiguousarray(x.transpose(0, 1, 3, 2)).reshape(-1, 10)       # rows of H
    v = oracle.slide1d(op, cols, kh)[0].reshape(2, 2, 13, 8).transpose(0, 1, 3, 2)
    h = oracle.slide1d(op, np.ascontiguousarray(v).astype(np.float32).reshape(-1, 13), kw)[0]
    assert np.array_equal(y, h.reshape(2, 2, 8, 10))


@pytest.mark.parametrize("op", [OP_ADD, OP_MAX])
def test_pool2d_stride2_is_subsampled_stride1(op):
    x = _rng(12).integers(-30, 31, size=(1, 3, 12, 14)).astype(np.float32)
    y1, _ = oracle.pool2d(op, x, 3, 3, 1, 1, 1, 1)
    y2, _ = oracle.pool2d(op, x, 3, 3, 2, 2, 1, 1)
    assert y2.shape == (1, 3, 6, 7)
    assert np.array_equal(y2, y1[:, :, ::2, ::2])


def test_pool2d_padding_matches_explicit_identity_padding():
    x = _rng(13).integers(-30, 31, size=(1, 2, 7, 9)).astype(np.float32)
    for op, ident in ((OP_ADD, 0.0), (OP_MAX, -1e30), (OP_MIN, 1e30)):
        xp = np.full((1, 2, 7 + 4, 9 + 2), ident, np.float32)
        xp[:, :, 2:-2, 1:-1] = x
        a, _ = oracle.pool2d(op, x, 4, 3, 2, 1, 2, 1)
        b, _ = oracle.pool2d(op, xp, 4, 3, 2, 1, 0, 0)
        assert np.array_equal(a, b)


# ----------------------------------------------------------------------------- P6
def _brute(op2, x, w):
    """Eq. 3 written out in pure Python for an arbitrary binary operator."""
    out = []
    for i in range(len(x) - w + 1):
        acc = x[i]
        for j in range(1, w):
            acc = op2(acc, x[i + j])
        out.append(acc)
    return out


def _vector_input(op2, ident, x, w, P):
    """Section 3, Algorithm 2 (Vector Input) with vectors of width P > w.

    Reading used: the carry Y holds, in lanes 0..w-2, the suffix sums of the last
    w-1 inputs seen (w-1, w-2, ..., 1 terms, each ending at the newest input);
    X1[t] is the prefix sum of the new vector ending at lane t with at most w
    terms; the outputs are Y (+) X1, and lanes whose window is entirely inside
    the new vector take X1 alone (Y holds the identity there).
    """
    N = len(x)
    assert P > w and N >= w

    def suffixes(vals):            # suffix sums of the last w-1 values, longest first
        out = []
        for s in range(len(vals) - (w - 1), len(vals)):
            acc = vals[s]
            for v in vals[s + 1:]:
                acc = op2(acc, v)
            out.append(acc)
        return out

    y = []
    Y = suffixes(x[:w - 1]) if w > 1 else []
    i = w - 1
    while i < N:
        X = x[i:i + P]
        X1 = []
        for t in range(len(X)):
            lo = max(0, t - (w - 1))
            acc = X[lo]
            for v in X[lo + 1:t + 1]:
                acc = op2(acc, v)
            X1.append(acc)
        for t in range(len(X)):
            y.append(op2(Y[t], X1[t]) if t < len(Y) else X1[t])
        if w > 1:
            tail = (x[max(0, i - (w - 1)):i] + X)[-(w - 1):]
            Y = suffixes(tail)
        i += P
    return y


def _segment_scheme(op2, x, w):
    """Block form of the same idea: segments of length S = w-1 from the origin,
    Pre = in-segment prefix sums, Suf = in-segment suffix sums, and
    y_i = Suf[i] (+) Pre[i+w-1] — one combination per output, older operand left."""
    N, S = len(x), w - 1
    if S == 0:
        return list(x)
    pre, suf = list(x), list(x)
    for j in range(N):
        if j % S:
            pre[j] = op2(pre[j - 1], x[j])
    for j in range(N - 1, -1, -1):
        if (j + 1) % S and j + 1 < N:
            suf[j] = op2(x[j], suf[j + 1])
    return [op2(suf[i], pre[i + S]) for i in range(N - w + 1)]


def test_paper_algorithms_noncommutative():
    """Vector Input (Alg. 2) and the segment prefix/suffix scheme reproduce Eq. 3 for
    string concatenation, which is associative but not commutative — so operand
    order and every index of the reading are pinned."""
    cat = lambda a, b: a + b
    for N, w in itertools.product((7, 16, 33, 64), range(1, 9)):
        if w > N:
            continue
        x = [chr(ord("a") + (i * 7 + 3) % 26) + str(i % 10) for i in range(N)]
        want = _brute(cat, x, w)
        assert _segment_scheme(cat, x, w) == want
        for P in (w + 1, 9, 16):
            if P > w:
                assert _vector_input(cat, "", x, w, P) == want


@pytest.mark.parametrize("w", [2, 3, 7, 12])
def test_paper_algorithms_agree_with_c_oracle(w):
    """The emulated algorithms, run on integer-valued floats, equal the C oracle exactly."""
    x = _rng(20 + w).integers(-40, 41, size=61).astype(np.float32)
    xs = [float(v) for v in x]
    for op, f in ((OP_ADD, lambda a, b: a + b), (OP_MAX, max), (OP_MIN, min)):
        y, _ = oracle.slide1d(op, x, w)
        assert _vector_input(f, None, xs, w, 16) == y[0].tolist()
        assert _segment_scheme(f, xs, w) == y[0].tolist()


# ----------------------------------------------------------------------------- P7
def _gamma_dot(a, b):
    """Section 2.4: dot product as a prefix sum.  Mask (Eq. 5), build the M+1 pairs
    (u_i, v_i) of Eq. 7, fold them with the operator of Eq. 8 (Eq. 9); the bottom
    element of the last sum is the dot product."""
    M = len(a)
    al = [1.0 if ai == 0 else float(ai) for ai in a]
    be = [0.0 if ai == 0 else float(bi) for ai, bi in zip(a, b)]
    g = []
    for i in range(M + 1):
        if i == 0:
            u = 1.0
        elif i < M:
            u = al[i - 1] / al[i]
        else:
            u = al[M - 1]
        v = be[i] if i < M else 0.0
        g.append((u, v))
    comb = lambda p, q: (p[0] * q[0], q[0] * p[1] + q[1])
    left = g[0]
    for q in g[1:]:
        left = comb(left, q)
    # associativity: a balanced bracketing gives the same bottom element
    def tree(lo, hi):
        if hi - lo == 1:
            return g[lo]
        mid = (lo + hi) // 2
        return comb(tree(lo, mid), tree(mid, hi))
    return left[1], tree(0, M + 1)[1]


@pytest.mark.parametrize("k", [1, 2, 5, 31])
def test_dot_product_as_prefix_sum_matches_conv_oracle(k):
    r = _rng(30 + k)
    taps = r.standard_normal(k).astype(np.float32)
    if k >= 5:
        taps[[1, 3]] = 0.0                          # exercise the masking of Eq. 5
    x = r.standard_normal(k).astype(np.float32)
    y, s = oracle.conv1d(x.reshape(1, 1, k), taps.reshape(1, 1, k))
    seq, tr = _gamma_dot(taps, x)
    assert abs(seq - y[0, 0, 0]) <= 1e-11 * max(1.0, s[0, 0, 0])
    assert abs(tr - y[0, 0, 0]) <= 1e-11 * max(1.0, s[0, 0, 0])


# ----------------------------------------------------------------------------- P8
def test_third_opinion_library_routines():
    """fp64 library routines on small shapes — a third opinion, never the oracle."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    r = _rng(40)
    x = r.standard_normal((2, 6, 37), dtype=np.float32)
    w = r.standard_normal((4, 3, 5), dtype=np.float32)
    for stride, pad, dil in ((1, 0, 1), (2, 3, 1), (1, 2, 3), (3, 1, 2)):
        y, _ = oracle.conv1d(x, w, stride=stride, pad=pad, dilation=dil, groups=2)
        t = F.conv1d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), None, stride, pad, dil, 2)
        assert np.allclose(y, t.numpy(), rtol=0, atol=1e-12)
    x2 = r.standard_normal((2, 3, 11, 9), dtype=np.float32)
    w2 = r.standard_normal((5, 3, 3, 2), dtype=np.float32)
    for sh, sw, ph, pw in ((1, 1, 0, 0), (2, 1, 1, 1), (1, 3, 2, 0)):
        y, _ = oracle.conv2d(x2, w2, sh, sw, ph, pw)
        t = F.conv2d(torch.from_numpy(x2).double(), torch.from_numpy(w2).double(), None, (sh, sw), (ph, pw))
        assert np.allclose(y, t.numpy(), rtol=0, atol=1e-12)
    for kh, kw, sh, sw, ph, pw in ((3, 3, 1, 1, 1, 1), (3, 3, 2, 2, 1, 1), (2, 4, 1, 2, 1, 2), (5, 1, 2, 1, 2, 0)):
        y, _ = oracle.pool2d(OP_ADD, x2, kh, kw, sh, sw, ph, pw, scale=1.0 / (kh * kw))
        t = F.avg_pool2d(torch.from_numpy(x2).double(), (kh, kw), (sh, sw), (ph, pw), count_include_pad=True)
        assert np.allclose(y, t.numpy(), rtol=0, atol=1e-12)
        y, _ = oracle.pool2d(OP_MAX, x2, kh, kw, sh, sw, ph, pw)
        t = F.max_pool2d(torch.from_numpy(x2).double(), (kh, kw), (sh, sw), (ph, pw))
        assert np.array_equal(y, t.numpy())
    y, _ = oracle.slide1d(OP_ADD, x.reshape(12, 37), 7, scale=1.0 / 7)
    t = F.avg_pool1d(torch.from_numpy(x).double(), 7, 1)
    assert np.allclose(y, t.numpy().reshape(12, -1), rtol=0, atol=1e-12)


def test_abs_sum_is_sum_of_magnitudes():
    r = _rng(50)
    x = r.standard_normal((1, 3, 20), dtype=np.float32)
    w = r.standard_normal((2, 3, 4), dtype=np.float32)
    _, s = oracle.conv1d(x, w, pad=1)
    y_abs, _ = oracle.conv1d(np.abs(x), np.abs(w), pad=1)
    assert np.allclose(s, y_abs, rtol=1e-14, atol=0)
    x2 = r.standard_normal((1, 2, 6, 6), dtype=np.float32)
    w2 = r.standard_normal((2, 2, 3, 3), dtype=np.float32)
    _, s = oracle.conv2d(x2, w2, 1, 1, 1, 1)
    y_abs, _ = oracle.conv2d(np.abs(x2), np.abs(w2), 1, 1, 1, 1)
    assert np.allclose(s, y_abs, rtol=1e-14, atol=0)
    _, s = oracle.pool2d(OP_ADD, x2, 3, 3, 1, 1, 1, 1, scale=-0.25)
    y_abs, _ = oracle.pool2d(OP_ADD, np.abs(x2), 3, 3, 1, 1, 1, 1, scale=0.25)
    assert np.allclose(s, y_abs, rtol=1e-14, atol=0)


# ----------------------------------------------------------------------------- P9
# The pair operator of Section 2.4 (Eq. 8) as a sliding window sum (Eq. 3).
PAIR_GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pair_hand_cases.txt")


def _pair_cases():
    out = []
    with open(PAIR_GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w, us, vs, yus, yvs = [[float(t) for t in p.split()] for p in line.split(";")]
            out.append((int(w[0]), us, vs, yus, yvs))
    return out


@pytest.mark.parametrize("w,us,vs,yus,yvs", _pair_cases())
def test_pair_hand_enumerated(w, us, vs, yus, yvs):
    yu, yv, _, _ = oracle.slide1d_pair(np.array(us, np.float32), np.array(vs, np.float32), w)
    assert yu[0].tolist() == yus and yv[0].tolist() == yvs


@pytest.mark.parametrize("w", [1, 2, 7, 40])
def test_pair_unit_u_is_sliding_add_and_zero_v_is_sliding_product(w):
    r = _rng(90 + w)
    v = r.standard_normal((3, 97), dtype=np.float32)
    one = np.ones_like(v)
    yu, yv, mu, mv = oracle.slide1d_pair(one, v, w)
    add, mag = oracle.slide1d(OP_ADD, v, w)
    assert np.array_equal(yu, np.ones_like(yu)) and np.allclose(yv, add, rtol=0, atol=1e-13 * mag.max())
    assert np.allclose(mv, mag, rtol=1e-14)
    u = (1.0 + 0.25 * r.standard_normal((3, 97))).astype(np.float32)
    yu, yv, mu, _ = oracle.slide1d_pair(u, np.zeros_like(u), w)
    prod = np.ones((3, 97 - w + 1))
    for t in range(w):
        prod = prod * u[:, t:97 - w + 1 + t].astype(np.float64)
    assert np.array_equal(yv, np.zeros_like(yv)) and np.allclose(yu, prod, rtol=1e-13) and np.allclose(mu, np.abs(prod), rtol=1e-13)
    c = np.full((1, 50), 1.5, np.float32)                      # closed form: constant u, constant v
    yu, yv, _, _ = oracle.slide1d_pair(c, np.full_like(c, 2.0), w)
    assert np.allclose(yu, 1.5 ** w, rtol=1e-14) and np.allclose(yv, 2.0 * (1.5 ** w - 1) / 0.5, rtol=1e-13)


def test_pair_exact_rationals_and_map_composition():
    """Small integers: the fold equals exact rational arithmetic, and applying the folded map to a
    point equals applying the w maps z -> u z + v one after the other (oldest first)."""
    from fractions import Fraction
    r = _rng(91)
    u = r.integers(-3, 4, size=(2, 23)).astype(np.float32)
    v = r.integers(-5, 6, size=(2, 23)).astype(np.float32)
    for w in (1, 2, 5, 9):
        yu, yv, _, _ = oracle.slide1d_pair(u, v, w)
        for row in range(2):
            for i in range(23 - w + 1):
                U, V, z = Fraction(1), Fraction(0), Fraction(7, 3)
                for t in range(w):
                    uj, vj = Fraction(int(u[row, i + t])), Fraction(int(v[row, i + t]))
                    U, V = U * uj, uj * V + vj
                    z = uj * z + vj
                assert Fraction(yu[row, i]) == U and Fraction(yv[row, i]) == V
                assert U * Fraction(7, 3) + V == z


def test_pair_operator_is_order_sensitive_and_associative():
    r = _rng(92)
    u = r.integers(2, 5, size=(1, 12)).astype(np.float32)
    v = r.integers(1, 9, size=(1, 12)).astype(np.float32)
    yu, yv, _, _ = oracle.slide1d_pair(u, v, 4)
    ru, rv, _, _ = oracle.slide1d_pair(u[:, ::-1].copy(), v[:, ::-1].copy(), 4)
    assert np.array_equal(yu, ru[:, ::-1])                       # products commute ...
    assert not np.array_equal(yv, rv[:, ::-1])                   # ... the pair operator does not
    # a window of 4 = (first two) (+) (last two), by associativity
    au, av, _, _ = oracle.slide1d_pair(u, v, 2)
    cu = au[:, :-2] * au[:, 2:]
    cv = au[:, 2:] * av[:, :-2] + av[:, 2:]
    assert np.array_equal(cu, yu) and np.array_equal(cv, yv)


@pytest.mark.parametrize("k", [1, 2, 5, 31])
def test_pair_full_window_of_gamma_sequence_is_the_dot_product(k):
    """Eq. 5, 7, 9: the M + 1 pairs built from the masked vectors, folded over one window of
    length M + 1, carry the dot product in the second component."""
    r = _rng(93 + k)
    a = r.integers(-4, 5, size=k).astype(np.float64)
    a[a == 3] = 0.0                                              # masked entries (Eq. 5)
    b = r.integers(-6, 7, size=k).astype(np.float64)
    al = np.where(a == 0, 1.0, a)
    be = np.where(a == 0, 0.0, b)
    al = np.where(np.abs(al) == 3, 1.0, al)                      # keep the ratios exactly representable: |alpha| in {1, 2, 4}
    u = np.array([1.0] + [al[i - 1] / al[i] for i in range(1, k)] + [al[k - 1]], np.float32)
    v = np.array(list(be) + [0.0], np.float32)
    _, yv, _, _ = oracle.slide1d_pair(u, v, k + 1)
    assert yv.shape == (1, 1) and yv[0, 0] == float(np.dot(al, be))


# ----------------------------------------------------------------------------- P10
# Boundary conditions (Section 3 names padding, mirroring and periodicity).
def test_padded_hand_enumerated():
    x = np.array([1, 2, 3], np.float32)
    # extended rows by hand: mirror 3 2 | 1 2 3 | 2 1 ; periodic 2 3 | 1 2 3 | 1 2 ; edge 1 1 | 1 2 3 | 3 3
    want = {oracle.PAD_MIRROR: [3, 2, 1, 2, 3, 2, 1], oracle.PAD_PERIODIC: [2, 3, 1, 2, 3, 1, 2],
            oracle.PAD_EDGE: [1, 1, 1, 2, 3, 3, 3]}
    for mode, ext in want.items():
        y, _ = oracle.slide1d_padded(OP_ADD, x, 1, 2, 2, mode)
        assert y[0].tolist() == ext
        y, _ = oracle.slide1d_padded(OP_ADD, x, 3, 2, 2, mode)
        assert y[0].tolist() == [sum(ext[i:i + 3]) for i in range(5)]
        y, _ = oracle.slide1d_padded(OP_MAX, x, 2, 2, 2, mode)
        assert y[0].tolist() == [max(ext[i:i + 2]) for i in range(6)]
    y, m = oracle.slide1d_padded(OP_ADD, x, 3, 2, 1, oracle.PAD_IDENTITY, 0.5)      # 0 0 | 1 2 3 | 0
    assert y[0].tolist() == [0.5, 1.5, 3.0, 2.5] and m[0].tolist() == [0.5, 1.5, 3.0, 2.5]
    y, _ = oracle.slide1d_padded(OP_MAX, -x, 2, 2, 0, oracle.PAD_IDENTITY)          # -inf -inf | -1 -2 -3
    assert y[0].tolist() == [-np.inf, -1.0, -1.0, -2.0]
    y, _ = oracle.slide1d_padded(OP_MIN, x, 2, 0, 2, oracle.PAD_IDENTITY)           # 1 2 3 | +inf +inf
    assert y[0].tolist() == [1.0, 2.0, 3.0, np.inf]


@pytest.mark.parametrize("mode,np_mode", [(1, "reflect"), (2, "wrap"), (3, "edge"), (0, "constant")])
@pytest.mark.parametrize("w,pl,pr", [(1, 0, 0), (3, 1, 1), (5, 4, 0), (8, 0, 7), (16, 15, 15), (31, 20, 9)])
def test_padded_equals_plain_definition_on_an_explicitly_extended_row(mode, np_mode, w, pl, pr):
    """numpy.pad writes the extended row out (a library routine as a second opinion on the index
    rules); the unpadded oracle then runs over it."""
    r = _rng(100 + w + pl)
    x = r.standard_normal((3, 33), dtype=np.float32)
    for op in (OP_ADD, OP_MAX, OP_MIN):
        fill = {OP_ADD: 0.0, OP_MAX: -np.inf, OP_MIN: np.inf}[op]
        kw = {"constant_values": fill} if mode == 0 else {}
        ext = np.pad(x, ((0, 0), (pl, pr)), mode=np_mode, **kw).astype(np.float32)
        y, m = oracle.slide1d_padded(op, x, w, pl, pr, mode, 0.25)
        with np.errstate(invalid="ignore"):
            ref, _ = oracle.slide1d(op, ext, w, 0.25)
        assert np.array_equal(y, ref)


def test_padded_without_padding_is_the_plain_sliding_sum_and_periodic_wraps():
    r = _rng(101)
    x = r.standard_normal((2, 50), dtype=np.float32)
    for mode in range(4):
        y, m = oracle.slide1d_padded(OP_ADD, x, 7, 0, 0, mode)
        ref, mag = oracle.slide1d(OP_ADD, x, 7)
        assert np.array_equal(y, ref) and np.array_equal(m, mag)
    # periodic with pad_right = w - 1: one output per input, and their total is w times the row total
    y, _ = oracle.slide1d_padded(OP_ADD, x, 7, 0, 6, oracle.PAD_PERIODIC)
    assert y.shape == (2, 50) and np.allclose(y.sum(axis=1), 7 * x.astype(np.float64).sum(axis=1), atol=1e-12)
    with pytest.raises(ValueError):
        oracle.slide1d_padded(OP_ADD, x, 3, 50, 0, oracle.PAD_MIRROR)           # mirror reaches past the row
    with pytest.raises(ValueError):
        oracle.slide1d_padded(OP_ADD, x, 3, 0, 51, oracle.PAD_PERIODIC)


# ----------------------------------------------------------------------------- P11
# Adjoint identities: <A x, g> = <x, A^T g> ties the plain, padded and convolution functions
# together (the backward pass of pooling / convolution is again a sliding sum).
@pytest.mark.parametrize("w", [1, 2, 5, 16])
def test_adjoint_of_sliding_add_is_identity_padded_sliding_add(w):
    r = _rng(110 + w)
    x = r.standard_normal((2, 61), dtype=np.float32)
    y, _ = oracle.slide1d(OP_ADD, x, w)
    g = r.standard_normal(y.shape).astype(np.float32)
    gx, _ = oracle.slide1d_padded(OP_ADD, g, w, w - 1, w - 1, oracle.PAD_IDENTITY)      # A^T g
    assert gx.shape == x.shape
    assert abs(float((y * g).sum()) - float((x.astype(np.float64) * gx).sum())) < 1e-10


@pytest.mark.parametrize("k,dilation,pad", [(1, 1, 0), (3, 1, 0), (5, 2, 3), (4, 3, 0)])
def test_adjoint_of_depthwise_convolution_is_convolution_with_flipped_taps(k, dilation, pad):
    r = _rng(120 + k)
    x = r.standard_normal((2, 3, 47), dtype=np.float32)
    w = r.standard_normal((3, 1, k), dtype=np.float32)
    y, _ = oracle.conv1d(x, w, 1, pad, dilation, 3)
    g = r.standard_normal(y.shape).astype(np.float32)
    span = (k - 1) * dilation
    gx, _ = oracle.conv1d(g, w[:, :, ::-1].copy(), 1, span - pad, dilation, 3)           # A^T g
    assert gx.shape == x.shape
    assert abs(float((y * g).sum()) - float((x.astype(np.float64) * gx).sum())) < 1e-10


def test_adjoint_of_dense_convolution_swaps_channels_and_flips_taps():
    r = _rng(130)
    x = r.standard_normal((2, 4, 29), dtype=np.float32)
    w = r.standard_normal((5, 4, 3), dtype=np.float32)
    y, _ = oracle.conv1d(x, w, 1, 1, 1, 1)
    g = r.standard_normal(y.shape).astype(np.float32)
    wt = np.ascontiguousarray(w.transpose(1, 0, 2)[:, :, ::-1])                          # [Cin, Cout, k], flipped
    gx, _ = oracle.conv1d(g, wt, 1, 1, 1, 1)
    assert abs(float((y * g).sum()) - float((x.astype(np.float64) * gx).sum())) < 1e-10
    x2 = r.standard_normal((1, 3, 9, 8), dtype=np.float32)
    w2 = r.standard_normal((2, 3, 3, 3), dtype=np.float32)
    y2, _ = oracle.conv2d(x2, w2, 1, 1, 1, 1)
    g2 = r.standard_normal(y2.shape).astype(np.float32)
    wt2 = np.ascontiguousarray(w2.transpose(1, 0, 2, 3)[:, :, ::-1, ::-1])
    gx2, _ = oracle.conv2d(g2, wt2, 1, 1, 1, 1)
    assert abs(float((y2 * g2).sum()) - float((x2.astype(np.float64) * gx2).sum())) < 1e-10


# ----------------------------------------------------------------------------- P12
# round16: the nearest bf16 / fp16 value, ties to even — how a result on 16-bit storage is written.
def test_round16_hand_written_ties_subnormals_and_overflow():
    bf = oracle.round16(np.array([1 + 2.0**-8, 1 + 2.0**-7 + 2.0**-8, 1 + 2.0**-8 + 2.0**-40, -(1 + 2.0**-8),
                                  0.0, 3.0, 2.0**-133 * 1.5, 2.0**-134, 3.39e38, 3.4e38]), oracle.DTYPE_BF16)
    want = [1.0, 1 + 2.0**-6, 1 + 2.0**-7, -1.0, 0.0, 3.0, 2.0**-132, 0.0, (2 - 2.0**-7) * 2.0**127, np.inf]
    assert bf.tolist() == want
    h = oracle.round16(np.array([1 + 2.0**-11, 1 + 2.0**-10 + 2.0**-11, 2049.0, 2051.0, 65504.0, 65519.99, 65520.0,
                                 2.0**-25, 2.0**-25 * 1.01, 2.0**-24 * 2.5, -2.0**-24 * 3.5]), oracle.DTYPE_F16)
    want = [1.0, 1 + 2.0**-9, 2048.0, 2052.0, 65504.0, 65504.0, np.inf, 0.0, 2.0**-24, 2.0**-23, -2.0**-22]
    assert h.tolist() == want


def test_round16_matches_the_library_casts():
    """fp16 against numpy's double -> float16 cast; bf16 against torch's float32 -> bfloat16 cast (on values
    that are float32 already, so that cast rounds once)."""
    import torch
    r = _rng(140)
    v = np.concatenate([r.standard_normal(20000) * 10.0 ** r.integers(-9, 5, 20000),
                        np.ldexp(r.integers(0, 4096, 4000) + 0.5, r.integers(-30, 4, 4000)),      # exact ties
                        np.array([0.0, -0.0, 65504.0, 65519.0, 65521.0, 1e6])])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).astype(np.float64)
    got = oracle.round16(v, oracle.DTYPE_F16)
    assert np.array_equal(got, want)
    v32 = np.concatenate([v.astype(np.float32), np.ldexp(r.integers(128, 256, 4000) + 0.5, r.integers(-140, 120, 4000))
                          .astype(np.float32)])
    want_bf = torch.from_numpy(v32).to(torch.bfloat16).to(torch.float64).numpy()
    got_bf = oracle.round16(v32.astype(np.float64), oracle.DTYPE_BF16)
    assert np.array_equal(got_bf, want_bf)


def test_round16_is_idempotent_monotone_and_within_half_a_step():
    r = _rng(141)
    v = np.sort(r.standard_normal(5000) * 100)
    for dt, frac in ((oracle.DTYPE_BF16, 7), (oracle.DTYPE_F16, 10)):
        q = oracle.round16(v, dt)
        assert np.array_equal(oracle.round16(q, dt), q)
        assert (np.diff(q) >= 0).all()
        assert (np.abs(q - v) <= np.abs(v) * 2.0 ** -(frac + 1)).all()


# ----------------------------------------------------------------------------- P13
# The adjoints of the sliding dot product (scatter form) against the pinned forward function.
GRAD_CASES = [  # B, Cin, L, Cout, k, stride, pad, dilation, groups
    (2, 3, 41, 3, 5, 1, 2, 1, 3), (2, 4, 37, 6, 3, 1, 1, 1, 1), (1, 4, 50, 8, 4, 2, 3, 1, 2),
    (3, 2, 33, 2, 3, 1, 0, 4, 2), (2, 6, 29, 4, 2, 3, 1, 2, 2), (1, 1, 20, 1, 20, 1, 0, 1, 1)]


@pytest.mark.parametrize("case", GRAD_CASES)
def test_conv1d_adjoints_satisfy_the_inner_product_identities(case):
    b, cin, length, cout, k, stride, pad, dil, groups = case
    r = _rng(150 + k + cin)
    x = r.standard_normal((b, cin, length), dtype=np.float32)
    w = r.standard_normal((cout, cin // groups, k), dtype=np.float32)
    y, _ = oracle.conv1d(x, w, stride, pad, dil, groups)
    g = r.standard_normal(y.shape).astype(np.float32)
    gx, _ = oracle.conv1d_grad_input(g, w, length, stride, pad, dil, groups)
    gw, _ = oracle.conv1d_grad_weight(x, g, k, stride, pad, dil, groups)
    loss = float((y * g).sum())
    assert gx.shape == x.shape and gw.shape == w.shape
    assert abs(loss - float((x.astype(np.float64) * gx).sum())) < 1e-9 * max(1.0, abs(loss))
    assert abs(loss - float((w.astype(np.float64) * gw).sum())) < 1e-9 * max(1.0, abs(loss))


def test_conv1d_adjoints_are_the_derivatives_of_the_bilinear_loss():
    """loss(x, W) = <conv(x; W), g> is linear in x and in W: a central difference is its exact
    partial derivative (up to fp64 rounding), element by element."""
    b, cin, length, cout, k, stride, pad, dil, groups = 1, 4, 19, 4, 3, 2, 2, 2, 2
    r = _rng(160)
    x = r.integers(-3, 4, (b, cin, length)).astype(np.float32)
    w = r.integers(-3, 4, (cout, cin // groups, k)).astype(np.float32)
    y, _ = oracle.conv1d(x, w, stride, pad, dil, groups)
    g = r.integers(-3, 4, y.shape).astype(np.float32)
    gx, _ = oracle.conv1d_grad_input(g, w, length, stride, pad, dil, groups)
    gw, _ = oracle.conv1d_grad_weight(x, g, k, stride, pad, dil, groups)
    loss = lambda xx, ww: float((oracle.conv1d(xx, ww, stride, pad, dil, groups)[0] * g).sum())
    for idx in np.ndindex(x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += 1
        xm[idx] -= 1
        assert (loss(xp, w) - loss(xm, w)) / 2 == gx[idx]
    for idx in np.ndindex(w.shape):
        wp, wm = w.copy(), w.copy()
        wp[idx] += 1
        wm[idx] -= 1
        assert (loss(x, wp) - loss(x, wm)) / 2 == gw[idx]


def test_conv1d_adjoints_hand_written_one_hot_cases():
    """One output gradient at i = 2 (k = 3, pad 1, stride 1): it returns the taps to x[1..3] and
    x[1..3] to the taps; at i = 0 the first tap fell into the padding and gets nothing."""
    x = np.array([[[1, 2, 3, 4, 5]]], np.float32)
    w = np.array([[[10, 20, 30]]], np.float32)
    g = np.zeros((1, 1, 5), np.float32)
    g[0, 0, 2] = 2
    gx, mag = oracle.conv1d_grad_input(g, w, 5, 1, 1, 1, 1)
    assert gx.ravel().tolist() == [0, 20, 40, 60, 0] and mag.ravel().tolist() == [0, 20, 40, 60, 0]
    gw, _ = oracle.conv1d_grad_weight(x, g, 3, 1, 1, 1, 1)
    assert gw.ravel().tolist() == [4, 6, 8]
    g[:] = 0
    g[0, 0, 0] = 1
    gw, _ = oracle.conv1d_grad_weight(x, g, 3, 1, 1, 1, 1)
    assert gw.ravel().tolist() == [0, 1, 2]
    gx, _ = oracle.conv1d_grad_input(g, w, 5, 1, 1, 1, 1)
    assert gx.ravel().tolist() == [20, 30, 0, 0, 0]
    # stride 2, dilation 2, no padding: output 1 reads x[2], x[4], x[6]
    g2 = np.array([[[0, 1]]], np.float32)
    gx, _ = oracle.conv1d_grad_input(g2, w, 7, 2, 0, 2, 1)
    assert gx.ravel().tolist() == [0, 0, 10, 0, 20, 0, 30]


def test_conv1d_grad_input_is_the_forward_function_on_flipped_taps_at_stride_one():
    """The gather form the GPU uses: taps flipped, channels swapped inside each group, padding span - pad."""
    b, cin, length, cout, k, pad, dil, groups = 2, 4, 31, 6, 4, 2, 3, 2
    r = _rng(170)
    w = r.standard_normal((cout, cin // groups, k), dtype=np.float32)
    lo = length + 2 * pad - dil * (k - 1)
    g = r.standard_normal((b, cout, lo), dtype=np.float32)
    gx, _ = oracle.conv1d_grad_input(g, w, length, 1, pad, dil, groups)
    cig, cog = cin // groups, cout // groups
    wt = np.ascontiguousarray(w.reshape(groups, cog, cig, k).transpose(0, 2, 1, 3)[..., ::-1]).reshape(cin, cog, k)
    via, _ = oracle.conv1d(g, wt, 1, dil * (k - 1) - pad, dil, groups)
    assert np.abs(via - gx).max() < 1e-12


# ----------------------------------------------------------------------------- P14
# pool2d_ex: four-sided padding and the divide-by-real-cells average.
def test_pool2d_ex_hand_written_case():
    """3 x 3 plane, 2 x 2 window, stride 1, padding top 1, left 1, bottom 0, right 1."""
    x = np.array([[[[1, 2, 3], [4, 5, 6], [7, 8, 9]]]], np.float32)
    y, _ = oracle.pool2d_ex(oracle.OP_ADD, x, 2, 2, 1, 1, (1, 1, 0, 1))
    assert y[0, 0].tolist() == [[1, 3, 5, 3], [5, 12, 16, 9], [11, 24, 28, 15]]
    y, _ = oracle.pool2d_ex(oracle.OP_ADD, x, 2, 2, 1, 1, (1, 1, 0, 1), div_valid=True)
    assert y[0, 0].tolist() == [[1, 1.5, 2.5, 3], [2.5, 3, 4, 4.5], [5.5, 6, 7, 7.5]]
    y, _ = oracle.pool2d_ex(oracle.OP_MAX, x, 2, 2, 1, 1, (1, 1, 0, 1))
    assert y[0, 0].tolist() == [[1, 2, 3, 3], [4, 5, 6, 6], [7, 8, 9, 9]]
    y, _ = oracle.pool2d_ex(oracle.OP_MIN, x, 2, 2, 2, 2, (0, 0, 1, 1))
    assert y[0, 0].tolist() == [[1, 3], [7, 9]]


@pytest.mark.parametrize("kh,kw,sh,sw,pads", [(3, 3, 1, 1, (1, 1, 1, 1)), (3, 3, 2, 2, (0, 1, 2, 0)), (2, 4, 1, 3, (1, 3, 0, 2)),
                                              (5, 2, 2, 1, (4, 0, 3, 1))])
def test_pool2d_ex_against_explicit_padding_and_closed_forms(kh, kw, sh, sw, pads):
    r = _rng(180 + kh + kw)
    x = r.standard_normal((2, 3, 9, 11), dtype=np.float32)
    pt, pl, pb, pr = pads
    for op, fill in ((oracle.OP_ADD, 0.0), (oracle.OP_MAX, -np.inf), (oracle.OP_MIN, np.inf)):
        y, _ = oracle.pool2d_ex(op, x, kh, kw, sh, sw, pads)
        xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (pt, pb), (pl, pr)), constant_values=fill)
        red = {oracle.OP_ADD: np.sum, oracle.OP_MAX: np.max, oracle.OP_MIN: np.min}[op]
        for ho in range(y.shape[2]):
            for wo in range(y.shape[3]):
                want = red(xp[:, :, ho * sh:ho * sh + kh, wo * sw:wo * sw + kw], axis=(2, 3))
                assert np.allclose(y[:, :, ho, wo], want, rtol=0, atol=1e-12)
    # the number of real cells per window: the plain sum of an all-ones plane; and the mean of a
    # constant plane over real cells is that constant
    ones = np.ones((1, 1, 9, 11), np.float32)
    cnt, _ = oracle.pool2d_ex(oracle.OP_ADD, ones, kh, kw, sh, sw, pads)
    rows = np.array([min(h * sh - pt + kh, 9) - max(h * sh - pt, 0) for h in range(cnt.shape[2])])
    cols = np.array([min(w * sw - pl + kw, 11) - max(w * sw - pl, 0) for w in range(cnt.shape[3])])
    assert np.array_equal(cnt[0, 0], np.outer(rows, cols))
    mean, _ = oracle.pool2d_ex(oracle.OP_ADD, 3 * ones, kh, kw, sh, sw, pads, div_valid=True)
    assert np.array_equal(mean, np.full_like(mean, 3.0))
    ys, _ = oracle.pool2d_ex(oracle.OP_ADD, x, kh, kw, sh, sw, pads)
    ym, _ = oracle.pool2d_ex(oracle.OP_ADD, x, kh, kw, sh, sw, pads, div_valid=True, scale=2.0)
    assert np.allclose(ym, 2.0 * ys / cnt, rtol=1e-14, atol=0)


def test_pool2d_ex_with_equal_pads_is_pool2d():
    r = _rng(190)
    x = r.standard_normal((1, 2, 12, 10), dtype=np.float32)
    for op in (oracle.OP_ADD, oracle.OP_MAX):
        a, ma = oracle.pool2d(op, x, 3, 3, 2, 2, 1, 1, 1 / 9)
        b, mb = oracle.pool2d_ex(op, x, 3, 3, 2, 2, (1, 1, 1, 1), scale=1 / 9)
        assert np.array_equal(a, b) and np.array_equal(ma, mb)


def test_padded_shrinking_window_hand_written_and_closed_forms():
    """PAD_SHRINK: virtual elements are skipped and add is rescaled by w / (real elements)."""
    x = np.array([[1, 2, 3, 4, 5]], np.float32)
    y, _ = oracle.slide1d_padded(oracle.OP_ADD, x, 3, 1, 2, oracle.PAD_SHRINK, 1 / 3)
    assert np.allclose(y[0], [1.5, 2, 3, 4, 4.5, 5], rtol=1e-15)        # means over 2,3,3,3,2,1 real elements
    y, _ = oracle.slide1d_padded(oracle.OP_MAX, x, 3, 1, 2, oracle.PAD_SHRINK)
    assert y[0].tolist() == [2, 3, 4, 5, 5, 5]
    r = _rng(200)
    z = r.standard_normal((3, 40), dtype=np.float32)
    for w, pl, pr in ((5, 2, 2), (7, 6, 0), (4, 0, 3)):
        a, _ = oracle.slide1d_padded(oracle.OP_ADD, z, w, pl, pr, oracle.PAD_IDENTITY, 1.0)
        ones, _ = oracle.slide1d_padded(oracle.OP_ADD, np.ones_like(z), w, pl, pr, oracle.PAD_IDENTITY, 1.0)
        b, _ = oracle.slide1d_padded(oracle.OP_ADD, z, w, pl, pr, oracle.PAD_SHRINK, 1.0 / w)
        assert np.allclose(b, a / ones, rtol=1e-14, atol=0)
        c, _ = oracle.slide1d_padded(oracle.OP_ADD, 2 * np.ones_like(z), w, pl, pr, oracle.PAD_SHRINK, 1.0 / w)
        assert np.allclose(c, 2.0, rtol=1e-15)
        m0, _ = oracle.slide1d_padded(oracle.OP_MIN, z, w, pl, pr, oracle.PAD_IDENTITY)
        m4, _ = oracle.slide1d_padded(oracle.OP_MIN, z, w, pl, pr, oracle.PAD_SHRINK)
        assert np.array_equal(m0, m4)
    with pytest.raises(ValueError):
        oracle.slide1d_padded(oracle.OP_ADD, z, 3, 3, 0, oracle.PAD_SHRINK)


# ----------------------------------------------------------------------------- P15
# The adjoints of the 2-D sliding dot product (scatter form).
@pytest.mark.parametrize("case", [(2, 3, 9, 8, 4, 3, 3, 1, 1, 1, 1), (1, 2, 10, 7, 3, 2, 4, 2, 1, 0, 2), (2, 4, 6, 6, 2, 1, 1, 1, 1, 0, 0),
                                  (1, 3, 11, 9, 2, 5, 3, 2, 3, 2, 1)])
def test_conv2d_adjoints_inner_product_identities_and_central_differences(case):
    n, cin, h, wd, cout, kh, kw, sh, sw, ph, pw = case
    r = _rng(210 + kh + kw)
    x = r.integers(-3, 4, (n, cin, h, wd)).astype(np.float32)
    w = r.integers(-3, 4, (cout, cin, kh, kw)).astype(np.float32)
    y, _ = oracle.conv2d(x, w, sh, sw, ph, pw)
    g = r.integers(-3, 4, y.shape).astype(np.float32)
    gx, _ = oracle.conv2d_grad_input(g, w, h, wd, sh, sw, ph, pw)
    gw, _ = oracle.conv2d_grad_weight(x, g, kh, kw, sh, sw, ph, pw)
    loss = float((y * g).sum())
    assert loss == float((x.astype(np.float64) * gx).sum()) == float((w.astype(np.float64) * gw).sum())
    f = lambda xx, ww: float((oracle.conv2d(xx, ww, sh, sw, ph, pw)[0] * g).sum())
    for idx in list(np.ndindex(x.shape))[::7]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += 1
        xm[idx] -= 1
        assert (f(xp, w) - f(xm, w)) / 2 == gx[idx]
    for idx in list(np.ndindex(w.shape))[::3]:
        wp, wm = w.copy(), w.copy()
        wp[idx] += 1
        wm[idx] -= 1
        assert (f(x, wp) - f(x, wm)) / 2 == gw[idx]


def test_conv2d_adjoints_on_one_row_planes_are_the_1d_adjoints_and_a_hand_case():
    r = _rng(220)
    x = r.standard_normal((2, 3, 1, 23), dtype=np.float32)
    w = r.standard_normal((4, 3, 1, 5), dtype=np.float32)
    g = r.standard_normal((2, 4, 1, 23), dtype=np.float32)
    gx2, _ = oracle.conv2d_grad_input(g, w, 1, 23, 1, 1, 0, 2)
    gw2, _ = oracle.conv2d_grad_weight(x, g, 1, 5, 1, 1, 0, 2)
    gx1, _ = oracle.conv1d_grad_input(g[:, :, 0], w[:, :, 0], 23, 1, 2, 1, 1)
    gw1, _ = oracle.conv1d_grad_weight(x[:, :, 0], g[:, :, 0], 5, 1, 2, 1, 1)
    assert np.abs(gx2[:, :, 0] - gx1).max() < 1e-12 and np.abs(gw2[:, :, 0] - gw1).max() < 1e-12
    # one gradient at output (1, 0) of a 3 x 3 plane, 2 x 2 taps, no padding: it reads x[1:3, 0:2]
    xh = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 3, 3)
    wh = np.array([[[[10, 20], [30, 40]]]], np.float32)
    gh = np.zeros((1, 1, 2, 2), np.float32)
    gh[0, 0, 1, 0] = 2
    gx, _ = oracle.conv2d_grad_input(gh, wh, 3, 3)
    assert gx[0, 0].tolist() == [[0, 0, 0], [20, 40, 0], [60, 80, 0]]
    gw, _ = oracle.conv2d_grad_weight(xh, gh, 2, 2)
    assert gw[0, 0].tolist() == [[8, 10], [14, 16]]


# ----------------------------------------------------------------------------- P16
# The adjoint of max pooling: gradients routed to the (first) maximum of every window.
def test_maxpool2d_grad_hand_written_case_and_tie_rule():
    x = np.array([[[[1, 5, 2], [7, 3, 7], [0, 4, 6]]]], np.float32)
    gy = np.array([[[[1, 10], [100, 1000]]]], np.float32)                  # 2 x 2 windows, stride 1
    gx = oracle.maxpool2d_grad(x, gy, 2, 2)
    # windows: [[1,5],[7,3]] -> 7 at (1,0); [[5,2],[3,7]] -> 7 at (1,2); [[7,3],[0,4]] -> 7 at (1,0); [[3,7],[4,6]] -> 7 at (1,2)
    assert gx[0, 0].tolist() == [[0, 0, 0], [101, 0, 1010], [0, 0, 0]]
    flat = np.full((1, 1, 3, 3), 2.0, np.float32)                          # all equal: the first cell of each window
    gx = oracle.maxpool2d_grad(flat, gy, 2, 2)
    assert gx[0, 0].tolist() == [[1, 10, 0], [100, 1000, 0], [0, 0, 0]]
    gx = oracle.maxpool2d_grad(flat, np.ones((1, 1, 3, 3), np.float32), 3, 3, 1, 1, 1, 1)     # padded: first cell inside the plane
    assert gx[0, 0].tolist() == [[4, 2, 0], [2, 1, 0], [0, 0, 0]]


@pytest.mark.parametrize("geom", [(3, 3, 1, 1, 1, 1), (3, 3, 2, 2, 1, 1), (2, 2, 2, 2, 0, 0), (4, 2, 3, 1, 2, 0), (1, 5, 1, 2, 0, 4)])
def test_maxpool2d_grad_is_the_derivative_of_the_pooled_loss(geom):
    """On distinct values max pooling is linear near x: central differences of sum(gy * maxpool(x)) with a step
    that keeps the order are its exact partial derivatives; and gradients are conserved."""
    kh, kw, sh, sw, ph, pw = geom
    r = _rng(230 + kh * 7 + kw)
    x = r.permutation(2 * 3 * 9 * 11).reshape(2, 3, 9, 11).astype(np.float32)      # distinct integers
    y, _ = oracle.pool2d(oracle.OP_MAX, x, kh, kw, sh, sw, ph, pw)
    gy = r.integers(-3, 4, y.shape).astype(np.float32)
    gx = oracle.maxpool2d_grad(x, gy, kh, kw, sh, sw, ph, pw)
    loss = lambda xx: float((oracle.pool2d(oracle.OP_MAX, xx, kh, kw, sh, sw, ph, pw)[0] * gy).sum())
    for idx in list(np.ndindex(x.shape))[::5]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += 0.25
        xm[idx] -= 0.25
        assert (loss(xp) - loss(xm)) / 0.5 == gx[idx]
    assert gx.sum() == float(gy.astype(np.float64).sum())
    assert np.array_equal(gx.sum(axis=(2, 3)), gy.astype(np.float64).sum(axis=(2, 3)))


# ----------------------------------------------------------------------------- P17
# The adjoint of average pooling: every window spreads f * gy over its cells inside the plane.
def test_avgpool2d_grad_hand_written_cases():
    gy = np.array([[[[1, 10], [100, 1000]]]], np.float32)                  # 2 x 2 windows, stride 1, on a 3 x 3 plane
    gx, mag = oracle.avgpool2d_grad(gy, 3, 3, 2, 2, scale=0.25)
    # cell (h, c) collects the windows (ho, wo) with ho in {h-1, h}, wo in {c-1, c} that exist
    want = np.array([[1, 11, 10], [101, 1111, 1010], [100, 1100, 1000]], np.float64) * 0.25
    assert np.array_equal(gx[0, 0], want) and np.array_equal(mag[0, 0], want)
    # stride 2 with padding 1 on a 3 x 3 plane, 3 x 3 windows: windows at rows / cols {-1..1} and {1..3};
    # window (0,0) holds the 4 real cells (0..1, 0..1), (0,1) the cells (0..1, 1..2), and so on
    gx, _ = oracle.avgpool2d_grad(gy, 3, 3, 3, 3, 2, 2, 1, 1, div_valid=True, scale=1.0)
    q = np.array([[1, 11, 10], [101, 1111, 1010], [100, 1100, 1000]], np.float64) / 4.0
    assert np.array_equal(gx[0, 0], q)
    gx, _ = oracle.avgpool2d_grad(gy, 3, 3, 3, 3, 2, 2, 1, 1, div_valid=False, scale=1.0)
    assert np.array_equal(gx[0, 0], q * 4.0)
    # a stride above the window: cells between the windows get nothing
    gx, _ = oracle.avgpool2d_grad(np.array([[[[2, 3]]]], np.float32), 1, 5, 1, 2, 1, 3)
    assert gx[0, 0].tolist() == [[2, 2, 0, 3, 3]]


@pytest.mark.parametrize("geom", [(3, 3, 1, 1, 1, 1), (3, 3, 2, 2, 1, 1), (2, 2, 2, 2, 0, 0), (4, 2, 3, 1, 2, 0), (1, 5, 1, 2, 0, 4),
                                  (5, 5, 3, 2, 2, 1), (2, 3, 4, 5, 1, 2)])
@pytest.mark.parametrize("div_valid", [False, True])
def test_avgpool2d_grad_is_the_adjoint_of_the_pinned_forward_pooling(geom, div_valid):
    """<pool2d_ex(x), gy> = <x, avgpool2d_grad(gy)> exactly on small integers with a power-of-two scale (the
    divide-by-real-cells factors are rationals, so that case is held to 1e-12); at stride 1 without the
    real-cell divisor the adjoint is itself a sliding add of gy over a plane padded by k - 1 - p; and the
    gradient every window hands out adds up to gy times its number of real cells times f."""
    kh, kw, sh, sw, ph, pw = geom
    r = _rng(240 + kh * 11 + kw + sh)
    x = r.integers(-4, 5, (2, 3, 11, 13)).astype(np.float32)
    y, _ = oracle.pool2d_ex(oracle.OP_ADD, x, kh, kw, sh, sw, (ph, pw, ph, pw), div_valid, 0.5)
    gy = r.integers(-3, 4, y.shape).astype(np.float32)
    gx, mag = oracle.avgpool2d_grad(gy, 11, 13, kh, kw, sh, sw, ph, pw, div_valid, 0.5)
    lhs, rhs = float((y * gy).sum()), float((gx * x).sum())
    assert lhs == rhs if not div_valid else abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    assert (mag >= np.abs(gx) - 1e-15).all()
    if not div_valid:
        ones, _ = oracle.pool2d_ex(oracle.OP_ADD, np.ones_like(x), kh, kw, sh, sw, (ph, pw, ph, pw), False, 1.0)   # real cells per window
        assert gx.sum() == float((gy.astype(np.float64) * ones * 0.5).sum())
    else:
        assert abs(gx.sum() - 0.5 * float(gy.astype(np.float64).sum())) <= 1e-12 * np.abs(gy).sum()
    if sh == 1 and sw == 1 and not div_valid:
        slid, _ = oracle.pool2d_ex(oracle.OP_ADD, gy, kh, kw, 1, 1, (kh - 1 - ph, kw - 1 - pw, kh - 1 - ph, kw - 1 - pw), False, 0.5)
        assert np.array_equal(slid, gx)


# ----------------------------------------------------------------------------- P18
# The boundary conditions of Section 3 in two dimensions (sws_ref_pool2d_padded).
def test_pool2d_padded_hand_enumerated():
    x = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    # one row above and one column in front, 2 x 2 windows; extended planes written out by hand:
    #   mirror   5 4 5 6     periodic 6 4 5 6     edge 1 1 2 3     identity . . . .
    #            2 1 2 3              3 1 2 3          1 1 2 3              . 1 2 3
    #            5 4 5 6              6 4 5 6          4 4 5 6              . 4 5 6
    want_add = {oracle.PAD_MIRROR: [[12, 12, 16], [12, 12, 16]], oracle.PAD_PERIODIC: [[14, 12, 16], [14, 12, 16]],
                oracle.PAD_EDGE: [[4, 6, 10], [10, 12, 16]], oracle.PAD_IDENTITY: [[1, 3, 5], [5, 12, 16]]}
    want_max = {oracle.PAD_MIRROR: [[5, 5, 6], [5, 5, 6]], oracle.PAD_PERIODIC: [[6, 5, 6], [6, 5, 6]],
                oracle.PAD_EDGE: [[1, 2, 3], [4, 5, 6]], oracle.PAD_IDENTITY: [[1, 2, 3], [4, 5, 6]]}
    for mode in want_add:
        y, m = oracle.pool2d_padded(OP_ADD, x, 2, 2, 1, 1, (1, 1, 0, 0), mode)
        assert y.tolist() == want_add[mode] and m.tolist() == want_add[mode]
        y, _ = oracle.pool2d_padded(OP_MAX, x, 2, 2, 1, 1, (1, 1, 0, 0), mode)
        assert y.tolist() == want_max[mode]
    y, _ = oracle.pool2d_padded(OP_MIN, -x, 2, 2, 2, 2, (0, 0, 2, 1), oracle.PAD_EDGE, 1.0)
    # -x with two rows below and one column behind (edge): rows -1 -2 -3 -3 / -4 -5 -6 -6 / -4.. / -4..; stride 2
    assert y.tolist() == [[-5.0, -6.0], [-5.0, -6.0]]


@pytest.mark.parametrize("mode,np_mode", [(1, "reflect"), (2, "wrap"), (3, "edge"), (0, "constant")])
@pytest.mark.parametrize("geom", [(3, 3, 1, 1, (1, 1, 1, 1)), (2, 4, 2, 1, (0, 3, 1, 0)), (5, 1, 1, 2, (4, 0, 0, 0)),
                                  (1, 6, 3, 3, (0, 2, 0, 5)), (4, 4, 4, 4, (2, 2, 2, 2)), (7, 7, 1, 1, (6, 6, 6, 6))])
def test_pool2d_padded_equals_pooling_of_an_explicitly_extended_plane(mode, np_mode, geom):
    """numpy.pad writes the extended planes out (a library routine as a second opinion on the index rules
    in both dimensions); the pinned unpadded pooling then runs over them."""
    kh, kw, sh, sw, pads = geom
    pt, pl, pb, pr = pads
    r = _rng(180 + kh * 10 + kw + mode)
    x = r.standard_normal((2, 3, 9, 11), dtype=np.float32)
    for op in (OP_ADD, OP_MAX, OP_MIN):
        fill = {OP_ADD: 0.0, OP_MAX: -np.inf, OP_MIN: np.inf}[op]
        kwargs = {"constant_values": fill} if mode == 0 else {}
        ext = np.pad(x, ((0, 0), (0, 0), (pt, pb), (pl, pr)), mode=np_mode, **kwargs).astype(np.float32)
        y, m = oracle.pool2d_padded(op, x, kh, kw, sh, sw, pads, mode, 0.5)
        with np.errstate(invalid="ignore"):
            ref, _ = oracle.pool2d(op, ext, kh, kw, sh, sw, 0, 0, 0.5)
        assert np.array_equal(y, ref)


def test_pool2d_padded_reduces_to_the_other_pooling_functions_and_to_rows():
    r = _rng(181)
    x = r.standard_normal((1, 3, 12, 14), dtype=np.float32)
    for op in (OP_ADD, OP_MAX):
        y, m = oracle.pool2d_padded(op, x, 3, 3, 2, 2, (1, 1, 1, 1), oracle.PAD_IDENTITY, 1 / 9)
        ref, mag = oracle.pool2d(op, x, 3, 3, 2, 2, 1, 1, 1 / 9)
        assert np.array_equal(y, ref) and np.array_equal(m, mag)
        # windows of one row: the rows of a plane under the 1-D boundary rule
        for mode in range(4):
            y, _ = oracle.pool2d_padded(op, x, 1, 5, 1, 1, (0, 3, 0, 2), mode, 0.2)
            rows, _ = oracle.slide1d_padded(op, x.reshape(36, 14), 5, 3, 2, mode, 0.2)
            assert np.array_equal(y.reshape(36, -1), rows)
    # periodic with pads k - 1 behind: one output per cell and every cell counted kh * kw times
    y, _ = oracle.pool2d_padded(OP_ADD, x, 3, 4, 1, 1, (0, 0, 2, 3), oracle.PAD_PERIODIC)
    assert y.shape == x.shape and np.allclose(y.sum(axis=(2, 3)), 12 * x.astype(np.float64).sum(axis=(2, 3)), atol=1e-10)
    with pytest.raises(ValueError):
        oracle.pool2d_padded(OP_ADD, x, 3, 3, 1, 1, (12, 0, 0, 0), oracle.PAD_MIRROR)      # mirror reaches past the plane
    with pytest.raises(ValueError):
        oracle.pool2d_padded(OP_ADD, x, 3, 3, 1, 1, (0, 0, 0, 15), oracle.PAD_PERIODIC)


# ----------------------------------------------------------------------------- P19
# The convolution of Section 2.5 over rows extended by the boundary conditions of Section 3 (sws_ref_conv1d_padded).
def test_conv1d_padded_hand_enumerated():
    x = np.array([[[1, 2, 3, 4]]], np.float32)
    taps = np.array([[[1, 10, 100]]], np.float32)
    # extended rows, one element a side:  mirror 2 1 2 3 4 3 | periodic 4 1 2 3 4 1 | edge 1 1 2 3 4 4 | zero 0 1 2 3 4 0
    want = {oracle.PAD_MIRROR: [212, 321, 432, 343], oracle.PAD_PERIODIC: [214, 321, 432, 143],
            oracle.PAD_EDGE: [211, 321, 432, 443], oracle.PAD_IDENTITY: [210, 321, 432, 43]}
    for mode, w in want.items():
        y, m = oracle.conv1d_padded(x, taps, 1, 1, 1, 1, 1, mode)
        assert y[0, 0].tolist() == w and m[0, 0].tolist() == w
    # two in front, none behind, taps two apart, every second output: mirror row 3 2 1 2 3 4
    y, _ = oracle.conv1d_padded(x, taps[:, :, :2], 2, 2, 0, 2, 1, oracle.PAD_MIRROR)
    assert y[0, 0].tolist() == [3 + 10, 1 + 30]


@pytest.mark.parametrize("mode,np_mode", [(1, "reflect"), (2, "wrap"), (3, "edge"), (0, "constant")])
@pytest.mark.parametrize("geom", [(3, 1, 1, 1, 1, 1), (5, 2, 4, 0, 1, 1), (4, 1, 0, 7, 3, 1), (7, 3, 6, 6, 2, 2), (1, 1, 2, 3, 1, 4),
                                  (9, 1, 8, 8, 1, 4)])
def test_conv1d_padded_equals_convolution_of_an_explicitly_extended_row(mode, np_mode, geom):
    k, stride, pl, pr, dil, groups = geom
    r = _rng(190 + k + mode)
    x = r.standard_normal((2, 4, 23), dtype=np.float32)
    wgt = r.standard_normal((8, 4 // groups, k), dtype=np.float32)
    ext = np.pad(x, ((0, 0), (0, 0), (pl, pr)), mode=np_mode)
    y, m = oracle.conv1d_padded(x, wgt, stride, pl, pr, dil, groups, mode)
    ref, mag = oracle.conv1d(ext, wgt, stride, 0, dil, groups)
    assert np.array_equal(y, ref) and np.array_equal(m, mag)


def test_conv1d_padded_periodic_is_circular_correlation_and_other_reductions():
    r = _rng(191)
    L, k = 64, 9
    x = r.standard_normal((1, 1, L), dtype=np.float32)
    taps = r.standard_normal((1, 1, k), dtype=np.float32)
    y, _ = oracle.conv1d_padded(x, taps, 1, 0, k - 1, 1, 1, oracle.PAD_PERIODIC)
    wl = np.zeros(L)
    wl[:k] = taps[0, 0]
    circ = np.fft.irfft(np.fft.rfft(x[0, 0].astype(np.float64)) * np.conj(np.fft.rfft(wl)), L)   # correlation theorem
    assert y.shape == (1, 1, L) and np.allclose(y[0, 0], circ, atol=1e-12)
    # zero padding, the same on both sides: the plain convolution
    xs = r.standard_normal((2, 6, 40), dtype=np.float32)
    ws = r.standard_normal((6, 2, 5), dtype=np.float32)
    a, am = oracle.conv1d_padded(xs, ws, 2, 3, 3, 2, 3, oracle.PAD_IDENTITY)
    b, bm = oracle.conv1d(xs, ws, 2, 3, 2, 3)
    assert np.array_equal(a, b) and np.array_equal(am, bm)
    # taps all one, one channel: the sliding sum over the padded row
    ones = np.ones((1, 1, 7), np.float32)
    for mode in range(4):
        c, _ = oracle.conv1d_padded(xs[:1, :1], ones, 1, 3, 3, 1, 1, mode)
        s, _ = oracle.slide1d_padded(OP_ADD, xs[0, :1], 7, 3, 3, mode)
        assert np.allclose(c[0], s, atol=1e-12)
    with pytest.raises(ValueError):
        oracle.conv1d_padded(xs, ws, 1, 40, 0, 1, 3, oracle.PAD_MIRROR)
    with pytest.raises(ValueError):
        oracle.conv1d_padded(xs, ws, 1, 0, 41, 1, 3, oracle.PAD_PERIODIC)


# ----------------------------------------------------------------------------- P20
# The 2-D convolution over planes extended by the boundary conditions of Section 3 (sws_ref_conv2d_padded).
def test_conv2d_padded_hand_enumerated():
    x = np.array([[[[1, 2, 3], [4, 5, 6]]]], np.float32)
    taps = np.array([[[[1, 10], [100, 1000]]]], np.float32)
    # one row above, one column in front (the extended planes of test_pool2d_padded_hand_enumerated):
    #   mirror 5 4 5 6 / 2 1 2 3 / 5 4 5 6   periodic 6 4 5 6 / 3 1 2 3 / 6 4 5 6   edge 1 1 2 3 / 1 1 2 3 / 4 4 5 6
    want = {oracle.PAD_MIRROR: [[5 + 40 + 200 + 1000, 4 + 50 + 100 + 2000, 5 + 60 + 200 + 3000],
                                [2 + 10 + 500 + 4000, 1 + 20 + 400 + 5000, 2 + 30 + 500 + 6000]],
            oracle.PAD_PERIODIC: [[6 + 40 + 300 + 1000, 4 + 50 + 100 + 2000, 5 + 60 + 200 + 3000],
                                  [3 + 10 + 600 + 4000, 1 + 20 + 400 + 5000, 2 + 30 + 500 + 6000]],
            oracle.PAD_EDGE: [[1 + 10 + 100 + 1000, 1 + 20 + 100 + 2000, 2 + 30 + 200 + 3000],
                              [1 + 10 + 400 + 4000, 1 + 20 + 400 + 5000, 2 + 30 + 500 + 6000]],
            oracle.PAD_IDENTITY: [[1000, 100 + 2000, 200 + 3000], [10 + 4000, 1 + 20 + 400 + 5000, 2 + 30 + 500 + 6000]]}
    for mode, w in want.items():
        y, m = oracle.conv2d_padded(x, taps, 1, 1, (1, 1, 0, 0), mode)
        assert y[0, 0].tolist() == w and m[0, 0].tolist() == w


@pytest.mark.parametrize("mode,np_mode", [(1, "reflect"), (2, "wrap"), (3, "edge"), (0, "constant")])
@pytest.mark.parametrize("geom", [(3, 3, 1, 1, (1, 1, 1, 1)), (2, 4, 2, 1, (0, 3, 1, 0)), (5, 1, 1, 2, (4, 0, 0, 0)),
                                  (1, 6, 3, 3, (0, 2, 0, 5)), (7, 7, 1, 1, (6, 6, 6, 6))])
def test_conv2d_padded_equals_convolution_of_an_explicitly_extended_plane(mode, np_mode, geom):
    kh, kw, sh, sw, pads = geom
    pt, pl, pb, pr = pads
    r = _rng(200 + kh * 10 + kw + mode)
    x = r.standard_normal((2, 3, 9, 11), dtype=np.float32)
    wgt = r.standard_normal((4, 3, kh, kw), dtype=np.float32)
    ext = np.pad(x, ((0, 0), (0, 0), (pt, pb), (pl, pr)), mode=np_mode)
    y, m = oracle.conv2d_padded(x, wgt, sh, sw, pads, mode)
    ref, mag = oracle.conv2d(ext, wgt, sh, sw, 0, 0)
    assert np.array_equal(y, ref) and np.array_equal(m, mag)


def test_conv2d_padded_periodic_is_circular_correlation_and_other_reductions():
    r = _rng(201)
    H, W, kh, kw = 12, 16, 3, 5
    x = r.standard_normal((1, 1, H, W), dtype=np.float32)
    taps = r.standard_normal((1, 1, kh, kw), dtype=np.float32)
    y, _ = oracle.conv2d_padded(x, taps, 1, 1, (0, 0, kh - 1, kw - 1), oracle.PAD_PERIODIC)
    wl = np.zeros((H, W))
    wl[:kh, :kw] = taps[0, 0]
    circ = np.fft.irfft2(np.fft.rfft2(x[0, 0].astype(np.float64)) * np.conj(np.fft.rfft2(wl)), (H, W))
    assert y.shape == (1, 1, H, W) and np.allclose(y[0, 0], circ, atol=1e-12)
    xs = r.standard_normal((2, 3, 10, 9), dtype=np.float32)
    ws = r.standard_normal((5, 3, 3, 4), dtype=np.float32)
    a, am = oracle.conv2d_padded(xs, ws, 2, 1, (1, 2, 1, 2), oracle.PAD_IDENTITY)
    b, bm = oracle.conv2d(xs, ws, 2, 1, 1, 2)
    assert np.array_equal(a, b) and np.array_equal(am, bm)
    # one-row planes and taps: the 1-D convolution of the rows
    for mode in range(4):
        c, _ = oracle.conv2d_padded(xs[:, :, :1], ws[:, :, :1], 1, 2, (0, 3, 0, 1), mode)
        d, _ = oracle.conv1d_padded(xs[:, :, 0], ws[:, :, 0], 2, 3, 1, 1, 1, mode)
        assert np.array_equal(c[:, :, 0], d)
    # all taps one, one channel: the pooling sum over the extended plane
    ones = np.ones((1, 1, 3, 2), np.float32)
    for mode in range(4):
        c, _ = oracle.conv2d_padded(xs[:, :1], ones, 1, 1, (2, 1, 0, 1), mode)
        p, _ = oracle.pool2d_padded(OP_ADD, xs[:, :1], 3, 2, 1, 1, (2, 1, 0, 1), mode)
        assert np.allclose(c, p, atol=1e-12)
    with pytest.raises(ValueError):
        oracle.conv2d_padded(xs, ws, 1, 1, (10, 0, 0, 0), oracle.PAD_MIRROR)
    with pytest.raises(ValueError):
        oracle.conv2d_padded(xs, ws, 1, 1, (0, 0, 0, 10), oracle.PAD_PERIODIC)
