"""CPU oracle for sliding window sums (fp64, naive).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It holds the plain definitions (Section 2.2 Eq. 3, Section 2.3,
Section 2.4 Eq. 8, Section 2.5 of the paper) written out as loops in C (sws_ref.c) behind a ctypes
wrapper that does argument marshalling only.  It imports nothing from the GPU
package and the GPU package imports nothing from here.
"""
from .ref import (  # noqa: F401
    DTYPE_BF16,
    DTYPE_F16,
    OP_ADD,
    OP_MAX,
    OP_MIN,
    build,
    conv1d,
    conv1d_grad_input,
    conv1d_grad_weight,
    conv2d,
    conv2d_grad_input,
    conv2d_grad_weight,
    avgpool2d_grad,
    maxpool2d_grad,
    pool2d,
    pool2d_ex,
    round16,
    set_threads,
    PAD_EDGE,
    PAD_IDENTITY,
    PAD_MIRROR,
    PAD_PERIODIC,
    PAD_SHRINK,
    slide1d,
    pool2d_padded,
    conv1d_padded,
    conv2d_padded,
    slide1d_padded,
    slide1d_pair,
    threads,
)
