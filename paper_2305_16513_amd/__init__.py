"""MI355X-native sliding window sums (arXiv 2305.16513): pooling and im2col-free
convolution as hand-written HIP kernels behind the C ABI of include/sws.h.

`paper_2305_16513_amd.binding` holds the ctypes binding (argument marshalling only);
`paper_2305_16513_amd.workloads` the seeded synthetic inputs; `paper_2305_16513_amd.build`
compiles csrc/ into libsws.so.  Importing this package loads nothing heavy: the shared
library is opened on first use and its absence is an error, never a fallback.
"""
__all__ = ["binding", "workloads", "build"]
