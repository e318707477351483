"""Seeded synthetic inputs shaped like the paper's DNN-layer workloads.

This module holds input generation only — none of the method's arithmetic —
so that the GPU path and the CPU oracle can both be fed identical bits.  The
paper measures on no public dataset (an unspecified "large 1-D input" and a
scenario from a cited work); these five configurations stand in for them, and
configurations 6 and 7 give the two experiments of the Experiments section their shapes
(a filter-size sweep on a large 1-D input; one very long dilated kernel at growing
output sizes).

All tensors are float32, finite, and never contain -0.0 (so that max/min have
a unique bit pattern).  Generation is on the host with numpy's PCG64 so the
same seed gives the same bits everywhere.
"""
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 2305165130  # + config number 1..8


@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    x_shape: tuple
    x_dist: str                 # "uniform" (U[-1,1]), "normal" (N(0,1)), "relu" (max(N(0,1),0))
    wgt_shape: tuple = ()
    wgt_std: float = 0.0
    ops: tuple = field(default_factory=tuple)


CONFIGS = {
    1: Config(1, "cfg1_1d_single", (1, 1, 1048576), "uniform", (1, 1, 5), 1.0,
              ("slide_add_w5", "slide_max_w5", "corr_k5")),
    2: Config(2, "cfg2_1d_multichannel", (16, 64, 4096), "normal", (64, 64, 3), (2.0 / (64 * 3)) ** 0.5,
              ("avgpool_w3", "maxpool_w3", "conv1d_k3")),
    3: Config(3, "cfg3_pool2d", (32, 64, 112, 112), "normal", (), 0.0,
              ("maxpool3x3_s1", "avgpool3x3_s1", "maxpool3x3_s2", "avgpool3x3_s2")),
    4: Config(4, "cfg4_conv2d_resnet", (32, 64, 56, 56), "relu", (64, 64, 3, 3), (2.0 / (64 * 9)) ** 0.5,
              ("conv2d_3x3_p1",)),
    5: Config(5, "cfg5_large_window_1d", (256, 128, 16384), "uniform", (128, 1, 31), (1.0 / 31.0) ** 0.5,
              ("slide_add_w16", "slide_max_w16", "slide_add_w64", "slide_max_w64",
               "slide_add_w255", "slide_max_w255", "dwconv_k31")),
    # Experiments section, first figure: single-channel sequences, filter sizes FILTER_SIZES.
    6: Config(6, "exp_filter_sweep_1d", (64, 1, 4194304), "uniform", (1, 1, 51), 0.2, ("conv1d_k*",)),
    # Experiments section, second figure: a 51-tap kernel with dilation 8; one sequence whose
    # output size runs over DILATED_OUTPUT_SIZES, and a batched depthwise form that fills the device.
    7: Config(7, "exp_dilated_1d", (1, 4096, 65536), "uniform", (4096, 1, 51), 0.2, ("dwconv_k51_d8",)),

    # Section 2.4: pairs (u, v) for the sliding window sum under the pair operator of Eq. 8.
    8: Config(8, "pair_operator_1d", (16384, 16384), "pairs", (), 0.0, ("slide_pair_w16", "slide_pair_w255")),
}

FILTER_SIZES = (3, 5, 11, 17, 21, 29, 37, 49, 51)
DILATED_K, DILATED_D = 51, 8
DILATED_OUTPUT_SIZES = (1000, 5000, 10000, 50000, 100000)


def _draw(rng, shape, dist):
    if dist == "uniform":
        a = rng.random(shape, dtype=np.float32)
        a *= np.float32(2.0)
        a -= np.float32(1.0)
    elif dist in ("normal", "relu"):
        a = rng.standard_normal(shape, dtype=np.float32)
        if dist == "relu":
            np.maximum(a, np.float32(0.0), out=a)
    else:
        raise ValueError(dist)
    a += np.float32(0.0)          # turns any -0.0 into +0.0
    return a


def make_pairs(shape=None, seed_offset=0):
    """(u, v) planes for configuration 8: u = +-(1 + 0.03 U[-1,1]) with one sign in five negative,
    so that products of a few hundred factors stay in range; v ~ N(0,1)."""
    shape = tuple(shape or CONFIGS[8].x_shape)
    ss = np.random.SeedSequence(SEED_BASE + 8 + 1000 * seed_offset)
    su, sg, sv = ss.spawn(3)
    u = np.random.Generator(np.random.PCG64(su)).random(shape, dtype=np.float32)
    u *= np.float32(0.06)
    u += np.float32(0.97)
    neg = np.random.Generator(np.random.PCG64(sg)).random(shape, dtype=np.float32) < np.float32(0.2)
    np.negative(u, out=u, where=neg)
    v = np.random.Generator(np.random.PCG64(sv)).standard_normal(shape, dtype=np.float32)
    v += np.float32(0.0)
    return u, v


def check_clean(a):
    """Raise if `a` holds NaN/inf or a negative zero."""
    if not np.isfinite(a).all():
        raise ValueError("non-finite synthetic input")
    if np.any((a == 0) & np.signbit(a)):
        raise ValueError("-0.0 in synthetic input")


def make(cfg, x_shape=None, wgt_shape=None, seed_offset=0):
    """Return (x, wgt) for configuration `cfg` (wgt is None where the config has none).

    `x_shape` / `wgt_shape` override the full-size shapes with the same
    distributions, for reduced parity cases.  Sub-streams are spawned in the
    fixed order x, weights.
    """
    c = CONFIGS[cfg]
    ss = np.random.SeedSequence(SEED_BASE + cfg + 1000 * seed_offset)
    sx, sw = ss.spawn(2)
    x = _draw(np.random.Generator(np.random.PCG64(sx)), tuple(x_shape or c.x_shape), c.x_dist)
    wgt = None
    shape_w = tuple(wgt_shape or c.wgt_shape)
    if shape_w:
        wgt = np.random.Generator(np.random.PCG64(sw)).standard_normal(shape_w, dtype=np.float32)
        wgt *= np.float32(c.wgt_std)
        wgt += np.float32(0.0)
    return x, wgt


def integer_valued(shape, lo, hi, seed):
    """Small-integer-valued float32 tensor: every fp32 partial sum is exact, so
    add/conv results can be compared bit for bit."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)
