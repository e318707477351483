"""ctypes binding of libsws.so — argument marshalling only.

Every function mirrors one entry point of include/sws.h, takes torch tensors that live
on the GPU (PyTorch is used for device memory and streams, nothing else), checks
dtype / device / contiguity, and passes raw device pointers plus the current HIP stream
to the C ABI.  There is no fallback: a missing library or a non-zero status raises.
"""
import ctypes
import os

import torch

OP_ADD, OP_MAX, OP_MIN = 0, 1, 2
SWS_OK, SWS_ERR_INVALID_ARG, SWS_ERR_UNSUPPORTED, SWS_ERR_HIP = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsws.so")
_lib = None

_i64, _i32, _f32, _vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p

EXPORTS = ("sws_slide1d", "sws_slide1d_16", "sws_slide1d_padded", "sws_slide1d_pair", "sws_pool2d", "sws_maxpool2d_grad", "sws_avgpool2d_grad", "sws_pool2d_16", "sws_pool2d_ex", "sws_pool2d_padded", "sws_conv1d", "sws_conv1d_padded", "sws_conv1d_16", "sws_conv1d_grad_input", "sws_conv1d_grad_weight", "sws_conv2d", "sws_conv2d_padded", "sws_conv2d_grad_input", "sws_conv2d_grad_weight", "sws_copy", "sws_out_len",
           "sws_status_string", "sws_set_option", "sws_version")


class SwsError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, status_string(status), status))


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2305_16513_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        L.sws_slide1d.restype = ctypes.c_int
        L.sws_slide1d.argtypes = [ctypes.c_int, _vp, _vp, _i64, _i64, _i32, _f32, _vp]
        L.sws_slide1d_16.restype = ctypes.c_int
        L.sws_slide1d_16.argtypes = [ctypes.c_int, ctypes.c_int, _vp, _vp, _i64, _i64, _i32, _f32, _vp]
        L.sws_slide1d_padded.restype = ctypes.c_int
        L.sws_slide1d_padded.argtypes = [ctypes.c_int, _vp, _vp, _i64, _i64, _i32, _i32, _i32, ctypes.c_int, _f32, _vp]
        L.sws_slide1d_pair.restype = ctypes.c_int
        L.sws_slide1d_pair.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i32, _vp]
        L.sws_pool2d.restype = ctypes.c_int
        L.sws_pool2d.argtypes = [ctypes.c_int, _vp, _vp, _i64, _i64, _i64, _i64,
                                 _i32, _i32, _i32, _i32, _i32, _i32, _f32, _vp]
        L.sws_avgpool2d_grad.restype = ctypes.c_int
        L.sws_avgpool2d_grad.argtypes = [_vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32, ctypes.c_int,
                                         ctypes.c_float, _vp]
        L.sws_maxpool2d_grad.restype = ctypes.c_int
        L.sws_maxpool2d_grad.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32, _vp]
        L.sws_pool2d_16.restype = ctypes.c_int
        L.sws_pool2d_16.argtypes = [ctypes.c_int, ctypes.c_int, _vp, _vp, _i64, _i64, _i64, _i64,
                                    _i32, _i32, _i32, _i32, _i32, _i32, _f32, _vp]
        L.sws_pool2d_ex.restype = ctypes.c_int
        L.sws_pool2d_ex.argtypes = [ctypes.c_int, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32,
                                    _i32, _i32, _i32, _i32, ctypes.c_int, _f32, _vp]
        L.sws_pool2d_padded.restype = ctypes.c_int
        L.sws_pool2d_padded.argtypes = [ctypes.c_int, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32,
                                        _i32, _i32, _i32, _i32, ctypes.c_int, _f32, _vp]
        L.sws_conv1d.restype = ctypes.c_int
        L.sws_conv1d.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _vp]
        L.sws_conv2d_padded.restype = ctypes.c_int
        L.sws_conv2d_padded.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32, _i32,
                                        _i32, ctypes.c_int, _vp]
        L.sws_conv1d_padded.restype = ctypes.c_int
        L.sws_conv1d_padded.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32,
                                        ctypes.c_int, _vp]
        L.sws_conv1d_16.restype = ctypes.c_int
        L.sws_conv1d_16.argtypes = [ctypes.c_int, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _vp]
        for f in (L.sws_conv1d_grad_input, L.sws_conv1d_grad_weight):
            f.restype = ctypes.c_int
            f.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _vp]
        L.sws_conv2d.restype = ctypes.c_int
        L.sws_conv2d.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64,
                                 _i32, _i32, _i32, _i32, _i32, _i32, _vp]
        for f in (L.sws_conv2d_grad_input, L.sws_conv2d_grad_weight):
            f.restype = ctypes.c_int
            f.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _i64, _i32, _i32, _i32, _i32, _i32, _i32, _vp]
        L.sws_copy.restype = ctypes.c_int
        L.sws_copy.argtypes = [_vp, _vp, _i64, _vp]
        L.sws_out_len.restype = _i64
        L.sws_out_len.argtypes = [_i64, _i32, _i32, _i32, _i32]
        L.sws_status_string.restype = ctypes.c_char_p
        L.sws_status_string.argtypes = [ctypes.c_int]
        L.sws_set_option.restype = ctypes.c_int
        L.sws_set_option.argtypes = [ctypes.c_char_p, _i64]
        L.sws_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status):
    return lib().sws_status_string(int(status)).decode()


def sws_version():
    return lib().sws_version().decode()


def sws_out_len(length, w, stride=1, pad=0, dilation=1):
    return int(lib().sws_out_len(length, w, stride, pad, dilation))


def sws_set_option(key, value):
    rc = lib().sws_set_option(key.encode(), int(value))
    if rc:
        raise SwsError(rc, "sws_set_option(%r)" % key)


def _dev(t, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a GPU tensor" % name)
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError("%s must be contiguous float32" % name)
    return t


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _out(y, shape, like, name="y"):
    if y is None:
        return torch.empty(shape, dtype=torch.float32, device=like.device)
    _dev(y, name)
    if tuple(y.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(y.shape), tuple(shape)))
    return y


def _check(rc, what):
    if rc != SWS_OK:
        raise SwsError(rc, what)


def sws_slide1d(op, x, w, scale=1.0, y=None, stream=None):
    """x [..., len] -> y [..., len-w+1]; all leading dimensions are independent rows."""
    _dev(x, "x")
    length = x.shape[-1]
    rows = x.numel() // length if length else 0
    lo = length - w + 1
    if lo < 1 or w < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_slide1d")
    y = _out(y, tuple(x.shape[:-1]) + (lo,), x)
    _check(lib().sws_slide1d(op, x.data_ptr(), y.data_ptr(), rows, length, w, scale, _stream(stream)),
           "sws_slide1d")
    return y


SWS_DTYPE_BF16, SWS_DTYPE_F16 = 1, 2
_DTYPE_16 = {torch.bfloat16: SWS_DTYPE_BF16, torch.float16: SWS_DTYPE_F16}


def sws_slide1d_16(op, x, w, scale=1.0, y=None, stream=None):
    """x [..., len] of bfloat16 or float16 -> y [..., len-w+1] of the same type (fp32 arithmetic)."""
    if not isinstance(x, torch.Tensor) or not x.is_cuda:
        raise TypeError("x must be a GPU tensor")
    if x.dtype not in _DTYPE_16 or not x.is_contiguous():
        raise TypeError("x must be contiguous bfloat16 or float16")
    length = x.shape[-1]
    rows = x.numel() // length if length else 0
    lo = length - w + 1
    if lo < 1 or w < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_slide1d_16")
    shape = tuple(x.shape[:-1]) + (lo,)
    if y is None:
        y = torch.empty(shape, dtype=x.dtype, device=x.device)
    elif (not isinstance(y, torch.Tensor) or not y.is_cuda or y.dtype != x.dtype or not y.is_contiguous()
          or tuple(y.shape) != shape):
        raise TypeError("y must be a contiguous GPU tensor of x's type and shape %s" % (shape,))
    _check(lib().sws_slide1d_16(op, _DTYPE_16[x.dtype], x.data_ptr(), y.data_ptr(), rows, length, w, scale,
                                _stream(stream)), "sws_slide1d_16")
    return y


SWS_PAD_IDENTITY, SWS_PAD_MIRROR, SWS_PAD_PERIODIC, SWS_PAD_EDGE, SWS_PAD_SHRINK = 0, 1, 2, 3, 4


def sws_slide1d_padded(op, x, w, pad_left, pad_right, mode, scale=1.0, y=None, stream=None):
    """x [..., len] -> y [..., len+pad_left+pad_right-w+1]: the rows are extended by the boundary rule `mode`."""
    _dev(x, "x")
    length = x.shape[-1]
    rows = x.numel() // length if length else 0
    lo = length + pad_left + pad_right - w + 1
    if lo < 1 or w < 1 or pad_left < 0 or pad_right < 0:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_slide1d_padded")
    y = _out(y, tuple(x.shape[:-1]) + (lo,), x)
    _check(lib().sws_slide1d_padded(op, x.data_ptr(), y.data_ptr(), rows, length, w, pad_left, pad_right, mode,
                                    scale, _stream(stream)), "sws_slide1d_padded")
    return y


def sws_slide1d_pair(u, v, w, yu=None, yv=None, stream=None):
    """u, v [..., len] -> (yu, yv) [..., len-w+1]: sliding window sum under the pair operator."""
    _dev(u, "u")
    _dev(v, "v")
    if u.shape != v.shape:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_slide1d_pair")
    length = u.shape[-1]
    rows = u.numel() // length if length else 0
    lo = length - w + 1
    if lo < 1 or w < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_slide1d_pair")
    yu = _out(yu, tuple(u.shape[:-1]) + (lo,), u)
    yv = _out(yv, tuple(u.shape[:-1]) + (lo,), u)
    _check(lib().sws_slide1d_pair(u.data_ptr(), v.data_ptr(), yu.data_ptr(), yv.data_ptr(), rows, length, w,
                                  _stream(stream)), "sws_slide1d_pair")
    return yu, yv


def sws_pool2d(op, x, kh, kw, sh=1, sw=1, ph=0, pw=0, scale=1.0, y=None, stream=None):
    """x [N, C, H, W] -> y [N, C, Ho, Wo]."""
    _dev(x, "x")
    n, c, h, wd = x.shape
    ho, wo = sws_out_len(h, kh, sh, ph), sws_out_len(wd, kw, sw, pw)
    if ho < 1 or wo < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_pool2d")
    y = _out(y, (n, c, ho, wo), x)
    _check(lib().sws_pool2d(op, x.data_ptr(), y.data_ptr(), n, c, h, wd, kh, kw, sh, sw, ph, pw, scale,
                            _stream(stream)), "sws_pool2d")
    return y


def sws_maxpool2d_grad(x, gy, kh, kw, sh=1, sw=1, ph=0, pw=0, gx=None, stream=None):
    """x [N, C, H, W], gy [N, C, Ho, Wo] -> gx [N, C, H, W]: gradients routed to the windows' maxima."""
    _dev(x, "x")
    _dev(gy, "gy")
    n, c, h, wd = x.shape
    if tuple(gy.shape) != (n, c, sws_out_len(h, kh, sh, ph), sws_out_len(wd, kw, sw, pw)):
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_maxpool2d_grad")
    gx = _out(gx, (n, c, h, wd), x, "gx")
    _check(lib().sws_maxpool2d_grad(x.data_ptr(), gy.data_ptr(), gx.data_ptr(), n, c, h, wd, kh, kw, sh, sw, ph, pw,
                                    _stream(stream)), "sws_maxpool2d_grad")
    return gx


def sws_avgpool2d_grad(gy, h, wd, kh, kw, sh=1, sw=1, ph=0, pw=0, divisor=0, scale=1.0, gx=None, stream=None):
    """gy [N, C, Ho, Wo], (h, wd) = the pooled plane -> gx [N, C, H, W]: the adjoint of average pooling
    (sws_pool2d_ex with SWS_OP_ADD, pads (ph, pw, ph, pw), the same divisor (0 = SWS_DIV_SCALE) and scale)."""
    _dev(gy, "gy")
    n, c, ho, wo = gy.shape
    if (ho, wo) != (sws_out_len(h, kh, sh, ph), sws_out_len(wd, kw, sw, pw)):
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_avgpool2d_grad")
    gx = _out(gx, (n, c, h, wd), gy, "gx")
    _check(lib().sws_avgpool2d_grad(gy.data_ptr(), gx.data_ptr(), n, c, h, wd, kh, kw, sh, sw, ph, pw, int(divisor),
                                    float(scale), _stream(stream)), "sws_avgpool2d_grad")
    return gx


def sws_pool2d_16(op, x, kh, kw, sh=1, sw=1, ph=0, pw=0, scale=1.0, y=None, stream=None):
    """x [N, C, H, W] of bfloat16 or float16 -> y [N, C, Ho, Wo] of the same type (fp32 arithmetic)."""
    if not isinstance(x, torch.Tensor) or not x.is_cuda:
        raise TypeError("x must be a GPU tensor")
    if x.dtype not in _DTYPE_16 or not x.is_contiguous():
        raise TypeError("x must be contiguous bfloat16 or float16")
    n, c, h, wd = x.shape
    ho, wo = sws_out_len(h, kh, sh, ph), sws_out_len(wd, kw, sw, pw)
    if ho < 1 or wo < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_pool2d_16")
    shape = (n, c, ho, wo)
    if y is None:
        y = torch.empty(shape, dtype=x.dtype, device=x.device)
    elif (not isinstance(y, torch.Tensor) or not y.is_cuda or y.dtype != x.dtype or not y.is_contiguous()
          or tuple(y.shape) != shape):
        raise TypeError("y must be a contiguous GPU tensor of x's type and shape %s" % (shape,))
    _check(lib().sws_pool2d_16(op, _DTYPE_16[x.dtype], x.data_ptr(), y.data_ptr(), n, c, h, wd, kh, kw, sh, sw, ph, pw,
                               scale, _stream(stream)), "sws_pool2d_16")
    return y


SWS_DIV_SCALE, SWS_DIV_REAL_CELLS = 0, 1


def sws_pool2d_ex(op, x, kh, kw, sh=1, sw=1, pads=(0, 0, 0, 0), divisor=SWS_DIV_SCALE, scale=1.0, y=None, stream=None):
    """x [N, C, H, W], pads = (top, left, bottom, right) -> y [N, C, Ho, Wo]."""
    _dev(x, "x")
    n, c, h, wd = x.shape
    pt, pl, pb, pr = pads
    ho, wo = (h + pt + pb - kh) // sh + 1, (wd + pl + pr - kw) // sw + 1
    if ho < 1 or wo < 1 or min(pads) < 0:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_pool2d_ex")
    y = _out(y, (n, c, ho, wo), x)
    _check(lib().sws_pool2d_ex(op, x.data_ptr(), y.data_ptr(), n, c, h, wd, kh, kw, sh, sw, pt, pl, pb, pr, divisor,
                               scale, _stream(stream)), "sws_pool2d_ex")
    return y


def sws_pool2d_padded(op, x, kh, kw, sh=1, sw=1, pads=(0, 0, 0, 0), mode=0, scale=1.0, y=None, stream=None):
    """x [N, C, H, W], pads = (top, left, bottom, right), mode = SWS_PAD_* -> y [N, C, Ho, Wo]: pooling over
    planes extended on four sides by the boundary rule `mode`."""
    _dev(x, "x")
    n, c, h, wd = x.shape
    pt, pl, pb, pr = pads
    ho, wo = (h + pt + pb - kh) // sh + 1, (wd + pl + pr - kw) // sw + 1
    if ho < 1 or wo < 1 or min(pads) < 0:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_pool2d_padded")
    y = _out(y, (n, c, ho, wo), x)
    _check(lib().sws_pool2d_padded(op, x.data_ptr(), y.data_ptr(), n, c, h, wd, kh, kw, sh, sw, pt, pl, pb, pr, mode,
                                   scale, _stream(stream)), "sws_pool2d_padded")
    return y


def sws_conv1d_padded(x, wgt, stride=1, pad_left=0, pad_right=0, dilation=1, groups=1, mode=0, y=None, stream=None):
    """x [B, Cin, L], wgt [Cout, Cin/groups, k] -> y [B, Cout, Lo]: rows extended at both ends by the boundary
    rule `mode` (SWS_PAD_IDENTITY = zeros, SWS_PAD_MIRROR, SWS_PAD_PERIODIC, SWS_PAD_EDGE)."""
    _dev(x, "x")
    _dev(wgt, "wgt")
    b, cin, length = x.shape
    cout, cig, k = wgt.shape
    lo = (length + pad_left + pad_right - dilation * (k - 1) - 1) // stride + 1
    if lo < 1 or cig * groups != cin or pad_left < 0 or pad_right < 0:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv1d_padded")
    y = _out(y, (b, cout, lo), x)
    _check(lib().sws_conv1d_padded(x.data_ptr(), wgt.data_ptr(), y.data_ptr(), b, cin, length, cout, k, stride, pad_left,
                                   pad_right, dilation, groups, mode, _stream(stream)), "sws_conv1d_padded")
    return y


def sws_conv1d(x, wgt, stride=1, pad=0, dilation=1, groups=1, y=None, stream=None):
    """x [B, Cin, L], wgt [Cout, Cin/groups, k] -> y [B, Cout, Lo]."""
    _dev(x, "x")
    _dev(wgt, "wgt")
    b, cin, length = x.shape
    cout, cig, k = wgt.shape
    if cig * groups != cin:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv1d")
    lo = sws_out_len(length, k, stride, pad, dilation)
    if lo < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv1d")
    y = _out(y, (b, cout, lo), x)
    _check(lib().sws_conv1d(x.data_ptr(), wgt.data_ptr(), y.data_ptr(), b, cin, length, cout, k, stride,
                            pad, dilation, groups, _stream(stream)), "sws_conv1d")
    return y


def sws_conv1d_16(x, wgt, stride=1, pad=0, dilation=1, groups=1, y=None, stream=None):
    """x [B, Cin, L] of bfloat16 or float16, wgt [Cout, Cin/groups, k] fp32 -> y [B, Cout, Lo] of x's type."""
    if not isinstance(x, torch.Tensor) or not x.is_cuda:
        raise TypeError("x must be a GPU tensor")
    if x.dtype not in _DTYPE_16 or not x.is_contiguous() or x.dim() != 3:
        raise TypeError("x must be contiguous bfloat16 or float16 of shape [B, Cin, L]")
    _dev(wgt, "wgt")
    b, cin, length = x.shape
    cout, cig, k = wgt.shape
    if cig * groups != cin:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv1d_16")
    lo = sws_out_len(length, k, stride, pad, dilation)
    if lo < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv1d_16")
    shape = (b, cout, lo)
    if y is None:
        y = torch.empty(shape, dtype=x.dtype, device=x.device)
    elif (not isinstance(y, torch.Tensor) or not y.is_cuda or y.dtype != x.dtype or not y.is_contiguous()
          or tuple(y.shape) != shape):
        raise TypeError("y must be a contiguous GPU tensor of x's type and shape %s" % (shape,))
    _check(lib().sws_conv1d_16(_DTYPE_16[x.dtype], x.data_ptr(), wgt.data_ptr(), y.data_ptr(), b, cin, length, cout,
                               k, stride, pad, dilation, groups, _stream(stream)), "sws_conv1d_16")
    return y


def sws_conv1d_grad_input(gy, wgt, length, stride=1, pad=0, dilation=1, groups=1, gx=None, stream=None):
    """gy [B, Cout, Lo], wgt [Cout, Cin/groups, k], length = L of the forward input -> gx [B, Cin, L]."""
    _dev(gy, "gy")
    _dev(wgt, "wgt")
    b, cout, lo = gy.shape
    cout2, cig, k = wgt.shape
    if cout2 != cout or lo != sws_out_len(length, k, stride, pad, dilation):
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv1d_grad_input")
    cin = cig * groups
    gx = _out(gx, (b, cin, length), gy, "gx")
    _check(lib().sws_conv1d_grad_input(gy.data_ptr(), wgt.data_ptr(), gx.data_ptr(), b, cin, length, cout, k, stride,
                                       pad, dilation, groups, _stream(stream)), "sws_conv1d_grad_input")
    return gx


def sws_conv1d_grad_weight(x, gy, k, stride=1, pad=0, dilation=1, groups=1, gw=None, stream=None):
    """x [B, Cin, L], gy [B, Cout, Lo] -> gw [Cout, Cin/groups, k]."""
    _dev(x, "x")
    _dev(gy, "gy")
    b, cin, length = x.shape
    b2, cout, lo = gy.shape
    if b2 != b or cin % groups or lo != sws_out_len(length, k, stride, pad, dilation):
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv1d_grad_weight")
    gw = _out(gw, (cout, cin // groups, k), x, "gw")
    _check(lib().sws_conv1d_grad_weight(x.data_ptr(), gy.data_ptr(), gw.data_ptr(), b, cin, length, cout, k, stride,
                                        pad, dilation, groups, _stream(stream)), "sws_conv1d_grad_weight")
    return gw


def sws_conv2d_padded(x, wgt, sh=1, sw=1, pads=(0, 0, 0, 0), mode=0, y=None, stream=None):
    """x [N, Cin, H, W], wgt [Cout, Cin, kh, kw], pads = (top, left, bottom, right) -> y [N, Cout, Ho, Wo]:
    planes extended on four sides by the boundary rule `mode` (SWS_PAD_IDENTITY = zeros, MIRROR, PERIODIC, EDGE)."""
    _dev(x, "x")
    _dev(wgt, "wgt")
    n, cin, h, wd = x.shape
    cout, cin2, kh, kw = wgt.shape
    pt, pl, pb, pr = pads
    ho, wo = (h + pt + pb - kh) // sh + 1, (wd + pl + pr - kw) // sw + 1
    if cin2 != cin or ho < 1 or wo < 1 or min(pads) < 0:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv2d_padded")
    y = _out(y, (n, cout, ho, wo), x)
    _check(lib().sws_conv2d_padded(x.data_ptr(), wgt.data_ptr(), y.data_ptr(), n, cin, h, wd, cout, kh, kw, sh, sw,
                                   pt, pl, pb, pr, mode, _stream(stream)), "sws_conv2d_padded")
    return y


def sws_conv2d(x, wgt, sh=1, sw=1, ph=0, pw=0, y=None, stream=None):
    """x [N, Cin, H, W], wgt [Cout, Cin, kh, kw] -> y [N, Cout, Ho, Wo]."""
    _dev(x, "x")
    _dev(wgt, "wgt")
    n, cin, h, wd = x.shape
    cout, cin2, kh, kw = wgt.shape
    if cin2 != cin:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv2d")
    ho, wo = sws_out_len(h, kh, sh, ph), sws_out_len(wd, kw, sw, pw)
    if ho < 1 or wo < 1:
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv2d")
    y = _out(y, (n, cout, ho, wo), x)
    _check(lib().sws_conv2d(x.data_ptr(), wgt.data_ptr(), y.data_ptr(), n, cin, h, wd, cout, kh, kw,
                            sh, sw, ph, pw, _stream(stream)), "sws_conv2d")
    return y


def sws_conv2d_grad_input(gy, wgt, h, wd, sh=1, sw=1, ph=0, pw=0, gx=None, stream=None):
    """gy [N, Cout, Ho, Wo], wgt [Cout, Cin, kh, kw], (h, wd) = the forward input's plane -> gx [N, Cin, H, W]."""
    _dev(gy, "gy")
    _dev(wgt, "wgt")
    n, cout, ho, wo = gy.shape
    cout2, cin, kh, kw = wgt.shape
    if cout2 != cout or ho != sws_out_len(h, kh, sh, ph) or wo != sws_out_len(wd, kw, sw, pw):
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv2d_grad_input")
    gx = _out(gx, (n, cin, h, wd), gy, "gx")
    _check(lib().sws_conv2d_grad_input(gy.data_ptr(), wgt.data_ptr(), gx.data_ptr(), n, cin, h, wd, cout, kh, kw,
                                       sh, sw, ph, pw, _stream(stream)), "sws_conv2d_grad_input")
    return gx


def sws_conv2d_grad_weight(x, gy, kh, kw, sh=1, sw=1, ph=0, pw=0, gw=None, stream=None):
    """x [N, Cin, H, W], gy [N, Cout, Ho, Wo] -> gw [Cout, Cin, kh, kw]."""
    _dev(x, "x")
    _dev(gy, "gy")
    n, cin, h, wd = x.shape
    n2, cout, ho, wo = gy.shape
    if n2 != n or ho != sws_out_len(h, kh, sh, ph) or wo != sws_out_len(wd, kw, sw, pw):
        raise SwsError(SWS_ERR_INVALID_ARG, "sws_conv2d_grad_weight")
    gw = _out(gw, (cout, cin, kh, kw), x, "gw")
    _check(lib().sws_conv2d_grad_weight(x.data_ptr(), gy.data_ptr(), gw.data_ptr(), n, cin, h, wd, cout, kh, kw,
                                        sh, sw, ph, pw, _stream(stream)), "sws_conv2d_grad_weight")
    return gw


def sws_copy(src, dst=None, stream=None):
    _dev(src, "src")
    dst = _out(dst, tuple(src.shape), src, "dst")
    _check(lib().sws_copy(src.data_ptr(), dst.data_ptr(), src.numel(), _stream(stream)), "sws_copy")
    return dst
