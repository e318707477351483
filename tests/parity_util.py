"""Shared helpers for the parity tests: acceptance rules and host<->device plumbing."""
import numpy as np

TOL = 1e-5          # |err| <= TOL * sum|terms| per output, fp32 add / avg / convolution


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t):
    return t.detach().cpu().numpy()


def assert_bit_exact(y_gpu, y_ref, what=""):
    """max / min: the fp32 result must carry exactly the bits of the oracle's value."""
    y_gpu = np.ascontiguousarray(y_gpu, dtype=np.float32)
    want = np.ascontiguousarray(y_ref.astype(np.float32))
    assert y_gpu.shape == want.shape, (what, y_gpu.shape, want.shape)
    same = y_gpu.view(np.uint32) == want.view(np.uint32)
    if not same.all():
        bad = np.argwhere(~same)
        first = tuple(bad[0])
        raise AssertionError("%s: %d of %d outputs differ in bits; first at %s: gpu=%r ref=%r" % (
            what, len(bad), same.size, first, y_gpu[first], want[first]))


def assert_within_tol(y_gpu, y_ref, abs_sum, what="", tol=TOL):
    """add / avg / conv: |y_gpu - y_ref| <= tol * sum|terms| for every output (an output
    whose terms are all zero must be exactly zero).  Returns the worst ratio seen."""
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    assert y_gpu.shape == y_ref.shape, (what, y_gpu.shape, y_ref.shape)
    assert np.isfinite(y_gpu).all(), what + ": non-finite output"
    err = np.abs(y_gpu - y_ref)
    ok = err <= tol * abs_sum
    if not ok.all():
        bad = np.argwhere(~ok)
        first = tuple(bad[0])
        raise AssertionError("%s: %d of %d outputs out of tolerance; first at %s: gpu=%r ref=%r err=%g allowed=%g" % (
            what, len(bad), ok.size, first, y_gpu[first], y_ref[first], err[first], tol * abs_sum[first]))
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(abs_sum > 0, err / abs_sum, 0.0)
    return float(ratio.max()) if ratio.size else 0.0
