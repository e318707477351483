"""ctypes wrapper around oracle/sws_ref.c.  TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays to the C oracle and returns (y, abs_sum) as float64
arrays.  No arithmetic of the method happens in this file.
"""
import ctypes
import os
import subprocess

import numpy as np

OP_ADD, OP_MAX, OP_MIN = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sws_ref.c")
_LIB = os.path.join(_HERE, "libsws_ref.so")
_lib = None


def build(force=True):
    """Compile sws_ref.c into libsws_ref.so with gcc (OpenMP over rows only)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_i64, _i32, _f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_double
_fp = ctypes.POINTER(ctypes.c_float)
_dp = ctypes.POINTER(ctypes.c_double)


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.sws_ref_threads.restype = ctypes.c_int
        lib.sws_ref_set_threads.restype = None
        lib.sws_ref_set_threads.argtypes = [ctypes.c_int]
        lib.sws_ref_slide1d.restype = ctypes.c_int
        lib.sws_ref_slide1d.argtypes = [ctypes.c_int, _fp, _dp, _dp, _i64, _i64, _i32, _f64]
        lib.sws_ref_pool2d.restype = ctypes.c_int
        lib.sws_ref_pool2d.argtypes = [ctypes.c_int, _fp, _dp, _dp, _i64, _i64, _i64, _i64,
                                       _i32, _i32, _i32, _i32, _i32, _i32, _f64]
        lib.sws_ref_pool2d_ex.restype = ctypes.c_int
        lib.sws_ref_pool2d_ex.argtypes = [ctypes.c_int, _fp, _dp, _dp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32,
                                          _i32, _i32, _i32, _i32, ctypes.c_int, _f64]
        lib.sws_ref_conv2d_padded.restype = ctypes.c_int
        lib.sws_ref_conv2d_padded.argtypes = [_fp, _fp, _dp, _dp, _i64, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32,
                                              _i32, _i32, _i32, _i32, ctypes.c_int]
        lib.sws_ref_conv1d_padded.restype = ctypes.c_int
        lib.sws_ref_conv1d_padded.argtypes = [_fp, _fp, _dp, _dp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32,
                                              ctypes.c_int]
        lib.sws_ref_pool2d_padded.restype = ctypes.c_int
        lib.sws_ref_pool2d_padded.argtypes = [ctypes.c_int, _fp, _dp, _dp, _i64, _i64, _i64, _i32, _i32, _i32, _i32,
                                              _i32, _i32, _i32, _i32, ctypes.c_int, _f64]
        lib.sws_ref_slide1d_padded.restype = ctypes.c_int
        lib.sws_ref_slide1d_padded.argtypes = [ctypes.c_int, _fp, _dp, _dp, _i64, _i64, _i32, _i32, _i32,
                                               ctypes.c_int, _f64]
        lib.sws_ref_slide1d_pair.restype = ctypes.c_int
        lib.sws_ref_slide1d_pair.argtypes = [_fp, _fp, _dp, _dp, _dp, _dp, _i64, _i64, _i32]
        for f in (lib.sws_ref_conv1d_grad_input, lib.sws_ref_conv1d_grad_weight):
            f.restype = ctypes.c_int
            f.argtypes = [_fp, _fp, _dp, _dp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32]
        for f in (lib.sws_ref_conv2d_grad_input, lib.sws_ref_conv2d_grad_weight):
            f.restype = ctypes.c_int
            f.argtypes = [_fp, _fp, _dp, _dp, _i64, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32]
        lib.sws_ref_avgpool2d_grad.restype = ctypes.c_int
        lib.sws_ref_avgpool2d_grad.argtypes = [_fp, _dp, _dp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32,
                                               ctypes.c_int, ctypes.c_double]
        lib.sws_ref_maxpool2d_grad.restype = ctypes.c_int
        lib.sws_ref_maxpool2d_grad.argtypes = [_fp, _fp, _dp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32]
        lib.sws_ref_round16.restype = ctypes.c_int
        lib.sws_ref_round16.argtypes = [_dp, _dp, _i64, ctypes.c_int]
        lib.sws_ref_conv1d.restype = ctypes.c_int
        lib.sws_ref_conv1d.argtypes = [_fp, _fp, _dp, _dp, _i64, _i64, _i64, _i64,
                                       _i32, _i32, _i32, _i32, _i32]
        lib.sws_ref_conv2d.restype = ctypes.c_int
        lib.sws_ref_conv2d.argtypes = [_fp, _fp, _dp, _dp, _i64, _i64, _i64, _i64, _i64,
                                       _i32, _i32, _i32, _i32, _i32, _i32]
        _lib = lib
    return _lib


def set_threads(n):
    """Threads the oracle's row loops use from now on (for a per-core timing)."""
    _load().sws_ref_set_threads(int(n))


def threads():
    """Number of OpenMP threads the oracle will use."""
    return int(_load().sws_ref_threads())


def _f32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs must be float32 (the data the GPU path reads)")
    return a


def _ptr_f(a):
    return a.ctypes.data_as(_fp)


def _ptr_d(a):
    return a.ctypes.data_as(_dp)


def slide1d(op, x, w, scale=1.0):
    """x: [rows, len] float32 -> (y, abs_sum), each [rows, len-w+1] float64 (Eq. 3)."""
    x = _f32(x)
    if x.ndim == 1:
        x = x[None, :]
    rows, length = x.shape
    lo = length - w + 1
    if lo < 1:
        raise ValueError("w must satisfy 1 <= w <= len")
    y = np.empty((rows, lo), np.float64)
    s = np.empty((rows, lo), np.float64)
    rc = _load().sws_ref_slide1d(op, _ptr_f(x), _ptr_d(y), _ptr_d(s), rows, length, w, float(scale))
    if rc:
        raise ValueError("sws_ref_slide1d rejected its arguments")
    return y, s


DTYPE_BF16, DTYPE_F16 = 1, 2


def round16(y, dtype):
    """float64 array -> float64 array holding the nearest bf16 / fp16 values (ties to even)."""
    y = np.ascontiguousarray(y, dtype=np.float64)
    out = np.empty_like(y)
    if _load().sws_ref_round16(_ptr_d(y), _ptr_d(out), y.size, dtype):
        raise ValueError("sws_ref_round16 rejected its arguments")
    return out


PAD_IDENTITY, PAD_MIRROR, PAD_PERIODIC, PAD_EDGE, PAD_SHRINK = 0, 1, 2, 3, 4


def pool2d_padded(op, x, kh, kw, sh=1, sw=1, pads=(0, 0, 0, 0), mode=PAD_IDENTITY, scale=1.0):
    """x: [..., H, W] float32, pads = (top, left, bottom, right) -> (y, abs_sum) [..., Ho, Wo] float64:
    pooling over planes extended on their four sides by the rule of `mode` (identity, mirror,
    periodic or edge)."""
    x = _f32(x)
    h, w = x.shape[-2:]
    lead = x.shape[:-2]
    planes = int(np.prod(lead)) if lead else 1
    pt, pl, pb, pr = pads
    he, we = h + pt + pb, w + pl + pr
    if kh > he or kw > we:
        raise ValueError("window larger than the extended plane")
    ho, wo = (he - kh) // sh + 1, (we - kw) // sw + 1
    y = np.empty(lead + (ho, wo), np.float64)
    s = np.empty(lead + (ho, wo), np.float64)
    rc = _load().sws_ref_pool2d_padded(op, _ptr_f(x), _ptr_d(y), _ptr_d(s), planes, h, w, kh, kw, sh, sw, pt, pl, pb, pr,
                                       mode, float(scale))
    if rc:
        raise ValueError("sws_ref_pool2d_padded rejected its arguments")
    return y, s


def slide1d_padded(op, x, w, pad_left, pad_right, mode, scale=1.0):
    """x: [rows, len] float32 -> (y, abs_sum), each [rows, len+pad_left+pad_right-w+1] float64:
    Eq. 3 over rows extended at both ends by the rule of `mode`."""
    x = _f32(x)
    if x.ndim == 1:
        x = x[None, :]
    rows, length = x.shape
    lo = length + pad_left + pad_right - w + 1
    if lo < 1:
        raise ValueError("window longer than the extended row")
    y = np.empty((rows, lo), np.float64)
    s = np.empty((rows, lo), np.float64)
    rc = _load().sws_ref_slide1d_padded(op, _ptr_f(x), _ptr_d(y), _ptr_d(s), rows, length, w, pad_left, pad_right,
                                        mode, float(scale))
    if rc:
        raise ValueError("sws_ref_slide1d_padded rejected its arguments")
    return y, s


def slide1d_pair(u, v, w):
    """u, v: [rows, len] float32 -> (yu, yv, mag_u, mag_v), each [rows, len-w+1] float64:
    the sliding window sum of the pairs (u_i, v_i) under the operator of Eq. 8."""
    u, v = _f32(u), _f32(v)
    if u.ndim == 1:
        u, v = u[None, :], v[None, :]
    if u.shape != v.shape:
        raise ValueError("u and v must have the same shape")
    rows, length = u.shape
    lo = length - w + 1
    if lo < 1:
        raise ValueError("w must satisfy 1 <= w <= len")
    out = [np.empty((rows, lo), np.float64) for _ in range(4)]
    rc = _load().sws_ref_slide1d_pair(_ptr_f(u), _ptr_f(v), *[_ptr_d(a) for a in out], rows, length, w)
    if rc:
        raise ValueError("sws_ref_slide1d_pair rejected its arguments")
    return tuple(out)


def pool2d(op, x, kh, kw, sh=1, sw=1, ph=0, pw=0, scale=1.0):
    """x: [N, C, H, W] float32 -> (y, abs_sum) [N, C, Ho, Wo] float64."""
    x = _f32(x)
    n, c, h, wd = x.shape
    ho = (h + 2 * ph - kh) // sh + 1
    wo = (wd + 2 * pw - kw) // sw + 1
    y = np.empty((n, c, ho, wo), np.float64)
    s = np.empty((n, c, ho, wo), np.float64)
    rc = _load().sws_ref_pool2d(op, _ptr_f(x), _ptr_d(y), _ptr_d(s), n, c, h, wd,
                                kh, kw, sh, sw, ph, pw, float(scale))
    if rc:
        raise ValueError("sws_ref_pool2d rejected its arguments")
    return y, s


def conv1d(x, wgt, stride=1, pad=0, dilation=1, groups=1):
    """x: [B, Cin, L], wgt: [Cout, Cin/groups, k] float32 -> (y, abs_sum) [B, Cout, Lo] float64."""
    x = _f32(x)
    wgt = _f32(wgt)
    b, cin, length = x.shape
    cout, cig, k = wgt.shape
    if cig * groups != cin:
        raise ValueError("wgt.shape[1] * groups must equal Cin")
    lo = (length + 2 * pad - dilation * (k - 1) - 1) // stride + 1
    y = np.empty((b, cout, lo), np.float64)
    s = np.empty((b, cout, lo), np.float64)
    rc = _load().sws_ref_conv1d(_ptr_f(x), _ptr_f(wgt), _ptr_d(y), _ptr_d(s), b, cin, length, cout,
                                k, stride, pad, dilation, groups)
    if rc:
        raise ValueError("sws_ref_conv1d rejected its arguments")
    return y, s


def conv1d_padded(x, wgt, stride=1, pad_left=0, pad_right=0, dilation=1, groups=1, mode=PAD_IDENTITY):
    """x: [B, Cin, L], wgt: [Cout, Cin/groups, k] float32 -> (y, abs_sum) [B, Cout, Lo] float64: the convolution
    over rows extended at both ends by the rule of `mode` (PAD_IDENTITY = zero padding)."""
    x = _f32(x)
    wgt = _f32(wgt)
    b, cin, length = x.shape
    cout, cig, k = wgt.shape
    if cig * groups != cin:
        raise ValueError("wgt.shape[1] * groups must equal Cin")
    lo = (length + pad_left + pad_right - dilation * (k - 1) - 1) // stride + 1
    if lo < 1:
        raise ValueError("kernel longer than the extended row")
    y = np.empty((b, cout, lo), np.float64)
    s = np.empty((b, cout, lo), np.float64)
    rc = _load().sws_ref_conv1d_padded(_ptr_f(x), _ptr_f(wgt), _ptr_d(y), _ptr_d(s), b, cin, length, cout, k, stride,
                                       pad_left, pad_right, dilation, groups, mode)
    if rc:
        raise ValueError("sws_ref_conv1d_padded rejected its arguments")
    return y, s


def conv2d(x, wgt, sh=1, sw=1, ph=0, pw=0):
    """x: [N, Cin, H, W], wgt: [Cout, Cin, kh, kw] float32 -> (y, abs_sum) [N, Cout, Ho, Wo] float64."""
    x = _f32(x)
    wgt = _f32(wgt)
    n, cin, h, wd = x.shape
    cout, cin2, kh, kw = wgt.shape
    if cin2 != cin:
        raise ValueError("wgt.shape[1] must equal Cin")
    ho = (h + 2 * ph - kh) // sh + 1
    wo = (wd + 2 * pw - kw) // sw + 1
    y = np.empty((n, cout, ho, wo), np.float64)
    s = np.empty((n, cout, ho, wo), np.float64)
    rc = _load().sws_ref_conv2d(_ptr_f(x), _ptr_f(wgt), _ptr_d(y), _ptr_d(s), n, cin, h, wd, cout,
                                kh, kw, sh, sw, ph, pw)
    if rc:
        raise ValueError("sws_ref_conv2d rejected its arguments")
    return y, s


def conv1d_grad_input(gy, wgt, length, stride=1, pad=0, dilation=1, groups=1):
    """gy: [B, Cout, Lo], wgt: [Cout, Cin/groups, k] float32, length = L of the forward input
    -> (gx, abs_sum) [B, Cin, L] float64: the adjoint of conv1d with respect to x."""
    gy = _f32(gy)
    wgt = _f32(wgt)
    b, cout, lo = gy.shape
    cout2, cig, k = wgt.shape
    cin = cig * groups
    if cout2 != cout or lo != (length + 2 * pad - dilation * (k - 1) - 1) // stride + 1:
        raise ValueError("gy does not have the forward output's shape")
    gx = np.empty((b, cin, length), np.float64)
    s = np.empty((b, cin, length), np.float64)
    rc = _load().sws_ref_conv1d_grad_input(_ptr_f(gy), _ptr_f(wgt), _ptr_d(gx), _ptr_d(s), b, cin, length, cout,
                                           k, stride, pad, dilation, groups)
    if rc:
        raise ValueError("sws_ref_conv1d_grad_input rejected its arguments")
    return gx, s


def conv1d_grad_weight(x, gy, k, stride=1, pad=0, dilation=1, groups=1):
    """x: [B, Cin, L], gy: [B, Cout, Lo] float32 -> (gw, abs_sum) [Cout, Cin/groups, k] float64:
    the adjoint of conv1d with respect to wgt."""
    x = _f32(x)
    gy = _f32(gy)
    b, cin, length = x.shape
    b2, cout, lo = gy.shape
    if b2 != b or lo != (length + 2 * pad - dilation * (k - 1) - 1) // stride + 1:
        raise ValueError("gy does not have the forward output's shape")
    gw = np.empty((cout, cin // groups, k), np.float64)
    s = np.empty((cout, cin // groups, k), np.float64)
    rc = _load().sws_ref_conv1d_grad_weight(_ptr_f(x), _ptr_f(gy), _ptr_d(gw), _ptr_d(s), b, cin, length, cout,
                                            k, stride, pad, dilation, groups)
    if rc:
        raise ValueError("sws_ref_conv1d_grad_weight rejected its arguments")
    return gw, s


def pool2d_ex(op, x, kh, kw, sh=1, sw=1, pads=(0, 0, 0, 0), div_valid=False, scale=1.0):
    """x: [N, C, H, W] float32, pads = (top, left, bottom, right) -> (y, abs_sum) [N, C, Ho, Wo] float64.
    div_valid: ADD results are divided by the number of window cells inside the plane."""
    x = _f32(x)
    n, c, h, wd = x.shape
    pt, pl, pb, pr = pads
    ho = (h + pt + pb - kh) // sh + 1
    wo = (wd + pl + pr - kw) // sw + 1
    if ho < 1 or wo < 1:
        raise ValueError("window larger than the padded plane")
    y = np.empty((n, c, ho, wo), np.float64)
    s = np.empty((n, c, ho, wo), np.float64)
    rc = _load().sws_ref_pool2d_ex(op, _ptr_f(x), _ptr_d(y), _ptr_d(s), n, c, h, wd, kh, kw, sh, sw, pt, pl, pb, pr,
                                   1 if div_valid else 0, float(scale))
    if rc:
        raise ValueError("sws_ref_pool2d_ex rejected its arguments")
    return y, s


def conv2d_padded(x, wgt, sh=1, sw=1, pads=(0, 0, 0, 0), mode=PAD_IDENTITY):
    """x: [N, Cin, H, W], wgt: [Cout, Cin, kh, kw] float32, pads = (top, left, bottom, right) ->
    (y, abs_sum) [N, Cout, Ho, Wo] float64: planes extended on four sides by the rule of `mode`."""
    x = _f32(x)
    wgt = _f32(wgt)
    n, cin, h, wd = x.shape
    cout, cin2, kh, kw = wgt.shape
    if cin2 != cin:
        raise ValueError("wgt.shape[1] must equal Cin")
    pt, pl, pb, pr = pads
    ho, wo = (h + pt + pb - kh) // sh + 1, (wd + pl + pr - kw) // sw + 1
    if ho < 1 or wo < 1:
        raise ValueError("kernel larger than the extended plane")
    y = np.empty((n, cout, ho, wo), np.float64)
    s = np.empty((n, cout, ho, wo), np.float64)
    rc = _load().sws_ref_conv2d_padded(_ptr_f(x), _ptr_f(wgt), _ptr_d(y), _ptr_d(s), n, cin, h, wd, cout, kh, kw, sh, sw,
                                       pt, pl, pb, pr, mode)
    if rc:
        raise ValueError("sws_ref_conv2d_padded rejected its arguments")
    return y, s


def conv2d_grad_input(gy, wgt, h, wd, sh=1, sw=1, ph=0, pw=0):
    """gy: [N, Cout, Ho, Wo], wgt: [Cout, Cin, kh, kw] float32, (h, wd) = the forward input's plane
    -> (gx, abs_sum) [N, Cin, H, W] float64 (serial: small cases only)."""
    gy = _f32(gy)
    wgt = _f32(wgt)
    n, cout, ho, wo = gy.shape
    cout2, cin, kh, kw = wgt.shape
    if cout2 != cout or ho != (h + 2 * ph - kh) // sh + 1 or wo != (wd + 2 * pw - kw) // sw + 1:
        raise ValueError("gy does not have the forward output's shape")
    gx = np.empty((n, cin, h, wd), np.float64)
    s = np.empty((n, cin, h, wd), np.float64)
    rc = _load().sws_ref_conv2d_grad_input(_ptr_f(gy), _ptr_f(wgt), _ptr_d(gx), _ptr_d(s), n, cin, h, wd, cout,
                                           kh, kw, sh, sw, ph, pw)
    if rc:
        raise ValueError("sws_ref_conv2d_grad_input rejected its arguments")
    return gx, s


def conv2d_grad_weight(x, gy, kh, kw, sh=1, sw=1, ph=0, pw=0):
    """x: [N, Cin, H, W], gy: [N, Cout, Ho, Wo] float32 -> (gw, abs_sum) [Cout, Cin, kh, kw] float64."""
    x = _f32(x)
    gy = _f32(gy)
    n, cin, h, wd = x.shape
    n2, cout, ho, wo = gy.shape
    if n2 != n or ho != (h + 2 * ph - kh) // sh + 1 or wo != (wd + 2 * pw - kw) // sw + 1:
        raise ValueError("gy does not have the forward output's shape")
    gw = np.empty((cout, cin, kh, kw), np.float64)
    s = np.empty((cout, cin, kh, kw), np.float64)
    rc = _load().sws_ref_conv2d_grad_weight(_ptr_f(x), _ptr_f(gy), _ptr_d(gw), _ptr_d(s), n, cin, h, wd, cout,
                                            kh, kw, sh, sw, ph, pw)
    if rc:
        raise ValueError("sws_ref_conv2d_grad_weight rejected its arguments")
    return gw, s


def avgpool2d_grad(gy, h, wd, kh, kw, sh=1, sw=1, ph=0, pw=0, div_valid=False, scale=1.0):
    """gy: [N, C, Ho, Wo] float32, (h, wd) = the pooled plane -> (gx, abs_sum) [N, C, H, W] float64: the
    adjoint of pool2d_ex(ADD, pads = (ph, pw, ph, pw), div_valid, scale)."""
    gy = _f32(gy)
    n, c, ho, wo = gy.shape
    if ho != (h + 2 * ph - kh) // sh + 1 or wo != (wd + 2 * pw - kw) // sw + 1:
        raise ValueError("gy does not have the pooled shape")
    gx = np.empty((n, c, h, wd), np.float64)
    s = np.empty((n, c, h, wd), np.float64)
    rc = _load().sws_ref_avgpool2d_grad(_ptr_f(gy), _ptr_d(gx), _ptr_d(s), n, c, h, wd, kh, kw, sh, sw, ph, pw,
                                        1 if div_valid else 0, float(scale))
    if rc:
        raise ValueError("sws_ref_avgpool2d_grad rejected its arguments")
    return gx, s


def maxpool2d_grad(x, gy, kh, kw, sh=1, sw=1, ph=0, pw=0):
    """x: [N, C, H, W], gy: [N, C, Ho, Wo] float32 -> gx [N, C, H, W] float64: every window's gradient
    goes to the first cell (row-major) holding its maximum."""
    x = _f32(x)
    gy = _f32(gy)
    n, c, h, wd = x.shape
    ho, wo = (h + 2 * ph - kh) // sh + 1, (wd + 2 * pw - kw) // sw + 1
    if tuple(gy.shape) != (n, c, ho, wo):
        raise ValueError("gy does not have the pooled shape")
    gx = np.empty((n, c, h, wd), np.float64)
    rc = _load().sws_ref_maxpool2d_grad(_ptr_f(x), _ptr_f(gy), _ptr_d(gx), n, c, h, wd, kh, kw, sh, sw, ph, pw)
    if rc:
        raise ValueError("sws_ref_maxpool2d_grad rejected its arguments")
    return gx
