// Kernel selection for 2-D convolution.
#include "sws_internal.h"

namespace sws {

hipError_t launch_conv2d(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                         int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh,
                         int32_t sw, int32_t ph, int32_t pw, hipStream_t s)
{
    if (g_opt.conv2d_variant != 1) {
        bool taken = false;
        const hipError_t e = launch_conv2d_mfma(x, wgt, y, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, ph, pw, 1, 1, s, &taken);
        if (taken) return e;
    }
    return launch_conv2d_naive(x, wgt, y, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, ph, pw, s);
}

}  // namespace sws
