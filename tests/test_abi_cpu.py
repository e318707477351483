"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in ("sws.h", "sws_dev.h")]


@pytest.fixture(scope="module")
def L():
    from paper_2305_16513_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2305_16513_amd import build
        build.build()
    return binding.lib()


def _declared():
    names = set()
    for h in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(sws_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(L):
    from paper_2305_16513_amd import binding
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_out_len(L):
    assert L.sws_out_len(1048576, 5, 1, 0, 1) == 1048572
    assert L.sws_out_len(4096, 3, 1, 0, 1) == 4094
    assert L.sws_out_len(112, 3, 2, 1, 1) == 56
    assert L.sws_out_len(112, 3, 1, 1, 1) == 112
    assert L.sws_out_len(16384, 255, 1, 0, 1) == 16130
    assert L.sws_out_len(10, 3, 1, 0, 4) == 2
    assert L.sws_out_len(4, 5, 1, 0, 1) == -1
    assert L.sws_out_len(4, 0, 1, 0, 1) == -1
    assert L.sws_out_len(4, 2, 0, 0, 1) == -1
    assert L.sws_out_len(-1, 2, 1, 0, 1) == -1


def test_status_strings(L):
    seen = {L.sws_status_string(i) for i in range(4)}
    assert len(seen) == 4 and all(s for s in seen)
    assert L.sws_status_string(99)


def test_slide1d_argument_checks(L):
    one = ctypes.c_void_p(16)      # never dereferenced: every call below fails or is empty
    nul = ctypes.c_void_p(0)
    assert L.sws_slide1d(0, one, one, 0, 100, 3, 1.0, nul) == 0            # no rows: nothing to do
    assert L.sws_slide1d(7, one, one, 1, 100, 3, 1.0, nul) == 1            # unknown op
    assert L.sws_slide1d(0, one, one, 1, 100, 0, 1.0, nul) == 1            # w < 1
    assert L.sws_slide1d(0, one, one, 1, 100, 101, 1.0, nul) == 1          # w > len
    assert L.sws_slide1d(0, one, one, -1, 100, 3, 1.0, nul) == 1
    assert L.sws_slide1d(0, one, one, 1, -5, 3, 1.0, nul) == 1
    assert L.sws_slide1d(0, nul, one, 1, 100, 3, 1.0, nul) == 1            # NULL with output
    assert L.sws_slide1d(0, one, nul, 1, 100, 3, 1.0, nul) == 1
    assert L.sws_slide1d(0, one, one, 1, 2 ** 31, 3, 1.0, nul) == 1        # row too long for int32
    assert L.sws_slide1d(0, one, one, 2 ** 40, 2 ** 30, 3, 1.0, nul) == 1  # size overflow


def test_slide1d_padded_argument_checks(L):
    one = ctypes.c_void_p(16)
    nul = ctypes.c_void_p(0)
    f = L.sws_slide1d_padded
    assert f(0, one, one, 0, 100, 3, 1, 1, 0, 1.0, nul) == 0               # no rows: nothing to do
    assert f(0, one, one, 1, 100, 3, -1, 1, 0, 1.0, nul) == 1              # negative pad
    assert f(0, one, one, 1, 100, 3, 1, 1, 5, 1.0, nul) == 1               # unknown mode
    assert f(0, one, one, 1, 100, 3, 3, 1, 4, 1.0, nul) == 1               # shrinking window: pad not below w
    assert f(0, one, one, 1, 100, 103, 1, 1, 0, 1.0, nul) == 1             # w longer than the extended row
    assert f(0, one, one, 1, 100, 3, 100, 0, 1, 1.0, nul) == 1             # mirror pad reaches past the row
    assert f(0, one, one, 1, 100, 3, 0, 101, 2, 1.0, nul) == 1             # periodic pad longer than the row
    assert f(0, one, one, 1, 0, 1, 1, 1, 0, 1.0, nul) == 1                 # empty rows cannot be extended
    assert f(5, one, one, 1, 100, 3, 1, 1, 0, 1.0, nul) == 1               # unknown op
    assert f(0, nul, one, 1, 100, 3, 1, 1, 0, 1.0, nul) == 1               # NULL with output
    assert f(0, one, one, 1, 2 ** 31 - 10, 3, 100000, 0, 3, 1.0, nul) == 1  # extended row too long for int32


def test_slide1d_pair_argument_checks(L):
    one = ctypes.c_void_p(16)
    nul = ctypes.c_void_p(0)
    assert L.sws_slide1d_pair(one, one, one, one, 0, 100, 3, nul) == 0        # no rows: nothing to do
    assert L.sws_slide1d_pair(one, one, one, one, 1, 100, 0, nul) == 1        # w < 1
    assert L.sws_slide1d_pair(one, one, one, one, 1, 100, 101, nul) == 1      # w > len
    assert L.sws_slide1d_pair(one, one, one, one, -1, 100, 3, nul) == 1
    assert L.sws_slide1d_pair(one, one, one, one, 1, 2 ** 31, 3, nul) == 1    # row too long for int32
    for k in range(4):                                                       # any NULL plane with output
        args = [one, one, one, one]
        args[k] = nul
        assert L.sws_slide1d_pair(*args, 1, 100, 3, nul) == 1


def test_pool2d_argument_checks(L):
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    ok = (0, one, one, 0, 3, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, nul)
    assert L.sws_pool2d(*ok) == 0                                          # N = 0
    bad = lambda **kw: L.sws_pool2d(*[kw.get(n, v) for n, v in zip(
        ("op", "x", "y", "N", "C", "H", "W", "kh", "kw", "sh", "sw", "ph", "pw", "scale", "s"),
        (0, one, one, 1, 3, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, nul))])
    assert bad(op=5) == 1
    assert bad(kh=0) == 1
    assert bad(sw=0) == 1
    assert bad(ph=3) == 1                                                  # window wholly in padding
    assert bad(pw=-1) == 1
    assert bad(kh=11) == 1                                                 # window larger than padded input
    assert bad(x=nul) == 1
    assert bad(N=-1) == 1


def test_conv_argument_checks(L):
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    c1 = lambda **kw: L.sws_conv1d(*[kw.get(n, v) for n, v in zip(
        ("x", "w", "y", "B", "Cin", "L", "Cout", "k", "stride", "pad", "dil", "groups", "s"),
        (one, one, one, 1, 4, 32, 6, 3, 1, 0, 1, 1, nul))])
    assert c1(B=0) == 0
    assert c1(groups=3) == 1                                               # Cin % groups
    assert c1(groups=4) == 1                                               # Cout % groups
    assert c1(k=0) == 1 and c1(stride=0) == 1 and c1(dil=0) == 1 and c1(pad=-1) == 1
    assert c1(k=33) == 1                                                   # taps span more than the row
    assert c1(k=9, dil=4) == 1
    assert c1(w=nul) == 1 and c1(x=nul) == 1 and c1(y=nul) == 1
    c2 = lambda **kw: L.sws_conv2d(*[kw.get(n, v) for n, v in zip(
        ("x", "w", "y", "N", "Cin", "H", "W", "Cout", "kh", "kw", "sh", "sw", "ph", "pw", "s"),
        (one, one, one, 1, 4, 8, 8, 6, 3, 3, 1, 1, 1, 1, nul))])
    assert c2(N=0) == 0
    assert c2(kh=0) == 1 and c2(sw=0) == 1 and c2(ph=-1) == 1 and c2(Cin=0) == 1
    assert c2(kw=11) == 1
    assert c2(w=nul) == 1


def test_options_and_copy_checks(L):
    assert L.sws_set_option(b"slide_variant", 0) == 0
    assert L.sws_set_option(b"no_such_knob", 1) == 1
    assert L.sws_set_option(None, 1) == 1
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    assert L.sws_copy(one, one, 0, nul) == 0
    assert L.sws_copy(one, one, -1, nul) == 1
    assert L.sws_copy(nul, one, 8, nul) == 1


def test_binding_refuses_cpu_tensors():
    """The product path never computes on the CPU: host tensors are an error."""
    import torch
    from paper_2305_16513_amd import binding
    with pytest.raises(TypeError):
        binding.sws_slide1d(0, torch.zeros(8), 3)


def test_new_entry_points_argument_checks(L):
    """sws_slide1d_16, sws_pool2d_ex and the conv1d adjoints reject bad arguments before any launch."""
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    i64, i32, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    L.sws_slide1d_16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, i64, i64, i32, f32, ctypes.c_void_p]
    assert L.sws_slide1d_16(0, 1, one, one, 0, 100, 3, 1.0, nul) == 0      # no rows
    assert L.sws_slide1d_16(0, 0, one, one, 1, 100, 3, 1.0, nul) == 1      # fp32 is not a 16-bit type
    assert L.sws_slide1d_16(0, 2, one, one, 1, 100, 101, 1.0, nul) == 1    # window longer than the row
    assert L.sws_slide1d_16(0, 2, nul, one, 1, 100, 3, 1.0, nul) == 1
    L.sws_pool2d_ex.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, i64, i64, i64, i64, i32, i32, i32, i32,
                                i32, i32, i32, i32, ctypes.c_int, f32, ctypes.c_void_p]
    pe = lambda **kw: L.sws_pool2d_ex(*[kw.get(n, v) for n, v in zip(
        ("op", "x", "y", "N", "C", "H", "W", "kh", "kw", "sh", "sw", "pt", "pl", "pb", "pr", "div", "scale", "s"),
        (0, one, one, 1, 3, 8, 8, 3, 3, 1, 1, 1, 0, 2, 1, 0, 1.0, nul))])
    assert pe(N=0) == 0
    assert pe(pt=3) == 1 and pe(pb=3) == 1 and pe(pl=3) == 1 and pe(pr=-1) == 1
    assert pe(div=2) == 1 and pe(op=4) == 1 and pe(y=nul) == 1 and pe(H=0) == 1
    for f in (L.sws_conv1d_grad_input, L.sws_conv1d_grad_weight):
        f.argtypes = [ctypes.c_void_p] * 3 + [i64, i64, i64, i64, i32, i32, i32, i32, i32, ctypes.c_void_p]
        g = lambda **kw: f(*[kw.get(n, v) for n, v in zip(
            ("a", "b", "c", "B", "Cin", "L", "Cout", "k", "stride", "pad", "dil", "groups", "s"),
            (one, one, one, 1, 4, 32, 6, 3, 1, 0, 1, 1, nul))])
        assert g(groups=3) == 1 and g(k=0) == 1 and g(k=40) == 1 and g(stride=0) == 1 and g(c=nul) == 1
    assert L.sws_conv1d_grad_input(one, one, one, 0, 4, 32, 6, 3, 1, 0, 1, 1, nul) == 0
    for f in (L.sws_conv2d_grad_input, L.sws_conv2d_grad_weight):
        f.argtypes = [ctypes.c_void_p] * 3 + [i64] * 5 + [i32] * 6 + [ctypes.c_void_p]
        g2 = lambda **kw: f(*[kw.get(n, v) for n, v in zip(
            ("a", "b", "c", "N", "Cin", "H", "W", "Cout", "kh", "kw", "sh", "sw", "ph", "pw", "s"),
            (one, one, one, 1, 4, 8, 8, 6, 3, 3, 1, 1, 1, 1, nul))])
        assert g2(kh=0) == 1 and g2(sw=0) == 1 and g2(kh=11) == 1 and g2(c=nul) == 1 and g2(Cin=0) == 1
    L.sws_maxpool2d_grad.argtypes = [ctypes.c_void_p] * 3 + [i64] * 4 + [i32] * 6 + [ctypes.c_void_p]
    mp = lambda **kw: L.sws_maxpool2d_grad(*[kw.get(n, v) for n, v in zip(
        ("x", "gy", "gx", "N", "C", "H", "W", "kh", "kw", "sh", "sw", "ph", "pw", "s"),
        (one, one, one, 1, 3, 8, 8, 3, 3, 1, 1, 1, 1, nul))])
    assert mp(N=0) == 0 and mp(ph=3) == 1 and mp(kw=0) == 1 and mp(gx=nul) == 1 and mp(kh=12) == 1
    L.sws_avgpool2d_grad.argtypes = [ctypes.c_void_p] * 2 + [i64] * 4 + [i32] * 6 + [ctypes.c_int, f32, ctypes.c_void_p]
    ap = lambda **kw: L.sws_avgpool2d_grad(*[kw.get(n, v) for n, v in zip(
        ("gy", "gx", "N", "C", "H", "W", "kh", "kw", "sh", "sw", "ph", "pw", "div", "scale", "s"),
        (one, one, 1, 3, 8, 8, 3, 3, 2, 2, 1, 1, 0, 1.0, nul))])
    assert ap(N=0) == 0 and ap(ph=3) == 1 and ap(sh=0) == 1 and ap(gx=nul) == 1 and ap(kh=12) == 1 and ap(div=2) == 1
    L.sws_pool2d_16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, i64, i64, i64, i64,
                                i32, i32, i32, i32, i32, i32, f32, ctypes.c_void_p]
    assert L.sws_pool2d_16(0, 1, one, one, 0, 3, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, nul) == 0
    assert L.sws_pool2d_16(0, 3, one, one, 1, 3, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, nul) == 1
    assert L.sws_pool2d_16(0, 1, one, nul, 1, 3, 8, 8, 3, 3, 1, 1, 1, 1, 1.0, nul) == 1


def test_conv1d_16_argument_checks(L):
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    i64, i32 = ctypes.c_int64, ctypes.c_int32
    L.sws_conv1d_16.argtypes = [ctypes.c_int] + [ctypes.c_void_p] * 3 + [i64] * 4 + [i32] * 5 + [ctypes.c_void_p]
    c = lambda **kw: L.sws_conv1d_16(*[kw.get(n, v) for n, v in zip(
        ("dtype", "x", "w", "y", "B", "Cin", "L", "Cout", "k", "stride", "pad", "dil", "groups", "s"),
        (1, one, one, one, 1, 4, 32, 4, 3, 1, 0, 1, 4, nul))])
    assert c(B=0) == 0
    assert c(dtype=0) == 1 and c(dtype=3) == 1                             # fp32 / unknown storage type
    assert c(groups=3) == 1 and c(k=0) == 1 and c(k=33) == 1 and c(stride=0) == 1 and c(dil=0) == 1 and c(pad=-1) == 1
    assert c(x=nul) == 1 and c(w=nul) == 1 and c(y=nul) == 1
    assert c(L=2 ** 31) == 1


def test_headers_compile_as_plain_c(tmp_path):
    """The boundary is a C ABI: both headers must be valid C99 with no HIP include."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use.c"
    src.write_text('#include "sws.h"\n#include "sws_dev.h"\n'
                   'int f(sws_stream_t s) { return (int)sws_slide1d(SWS_OP_ADD, 0, 0, 0, 8, 3, 1.0f, s); }\n')
    subprocess.run([cc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)


def test_pool2d_padded_argument_checks(L):
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    i64, i32, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    L.sws_pool2d_padded.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, i64, i64, i64, i64, i32, i32, i32, i32,
                                    i32, i32, i32, i32, ctypes.c_int, f32, ctypes.c_void_p]
    pp = lambda **kw: L.sws_pool2d_padded(*[kw.get(n, v) for n, v in zip(
        ("op", "x", "y", "N", "C", "H", "W", "kh", "kw", "sh", "sw", "pt", "pl", "pb", "pr", "mode", "scale", "s"),
        (0, one, one, 1, 3, 8, 6, 3, 3, 1, 1, 1, 0, 2, 1, 1, 1.0, nul))])
    assert pp(N=0) == 0 and pp(C=0, mode=2) == 0
    assert pp(mode=5) == 1 and pp(mode=-1) == 1 and pp(op=3) == 1 and pp(H=0) == 1 and pp(pr=-1) == 1
    assert pp(pt=8) == 1 and pp(pb=8) == 1 and pp(pl=6) == 1 and pp(pr=6) == 1            # mirror: at most extent - 1
    assert pp(mode=2, pt=9) == 1 and pp(mode=2, pr=7) == 1                                # periodic: at most the extent
    assert pp(mode=4, pt=3) == 1 and pp(mode=4, pr=3) == 1                                # shrinking: below the window
    assert pp(kh=12) == 1 and pp(kw=8) == 1 and pp(sh=0) == 1 and pp(x=nul) == 1 and pp(y=nul) == 1


def test_conv1d_padded_argument_checks(L):
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    i64, i32 = ctypes.c_int64, ctypes.c_int32
    L.sws_conv1d_padded.argtypes = [ctypes.c_void_p] * 3 + [i64] * 4 + [i32] * 6 + [ctypes.c_int, ctypes.c_void_p]
    c = lambda **kw: L.sws_conv1d_padded(*[kw.get(n, v) for n, v in zip(
        ("x", "w", "y", "B", "Cin", "L", "Cout", "k", "stride", "pl", "pr", "dil", "groups", "mode", "s"),
        (one, one, one, 1, 4, 32, 4, 3, 1, 1, 1, 1, 4, 1, nul))])
    assert c(B=0) == 0
    assert c(mode=4) == 1 and c(mode=-1) == 1 and c(L=0) == 1 and c(pl=-1) == 1 and c(pr=-1) == 1
    assert c(pl=32) == 1 and c(pr=32) == 1 and c(mode=2, pl=33) == 1 and c(mode=2, pr=33) == 1
    assert c(groups=3) == 1 and c(k=0) == 1 and c(k=40) == 1 and c(stride=0) == 1 and c(dil=0) == 1 and c(y=nul) == 1


def test_conv2d_padded_argument_checks(L):
    one, nul = ctypes.c_void_p(16), ctypes.c_void_p(0)
    i64, i32 = ctypes.c_int64, ctypes.c_int32
    L.sws_conv2d_padded.argtypes = [ctypes.c_void_p] * 3 + [i64] * 5 + [i32] * 8 + [ctypes.c_int, ctypes.c_void_p]
    c = lambda **kw: L.sws_conv2d_padded(*[kw.get(n, v) for n, v in zip(
        ("x", "w", "y", "N", "Cin", "H", "W", "Cout", "kh", "kw", "sh", "sw", "pt", "pl", "pb", "pr", "mode", "s"),
        (one, one, one, 1, 4, 8, 6, 6, 3, 3, 1, 1, 1, 1, 1, 1, 1, nul))])
    assert c(N=0) == 0
    assert c(mode=4) == 1 and c(mode=-1) == 1 and c(H=0) == 1 and c(pt=-1) == 1 and c(Cin=0) == 1
    assert c(pt=8) == 1 and c(pr=6) == 1 and c(mode=2, pb=9) == 1 and c(mode=2, pl=7) == 1
    assert c(kh=11) == 1 and c(kw=9) == 1 and c(sh=0) == 1 and c(y=nul) == 1 and c(w=nul) == 1
