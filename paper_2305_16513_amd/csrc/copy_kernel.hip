// Calibration copy: the one-read-one-write pattern of the sliding kernels with no
// arithmetic, used to measure the bandwidth ceiling and to scale byte counters.
#include "sws_internal.h"

namespace sws {

namespace {

// Each workgroup moves 4096 consecutive floats as four fully coalesced 128-bit
// accesses per lane (lane l touches 16 bytes at 16*l within each 4 KB strip).
template <int NT>
__global__ __launch_bounds__(256) void copy_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                   int64_t n)
{
    const int64_t base = (int64_t)blockIdx.x * 4096;
    if (base + 4096 <= n) {
        v4f r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const v4f_u *p = (const v4f_u *)(src + base + j * 1024 + 4 * threadIdx.x);
            r[j] = NT ? __builtin_nontemporal_load(p) : *p;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v4f_u *p = (v4f_u *)(dst + base + j * 1024 + 4 * threadIdx.x);
            if (NT) __builtin_nontemporal_store(r[j], p);
            else *p = r[j];
        }
    } else {
        for (int64_t o = base + threadIdx.x; o < n; o += 256) dst[o] = src[o];
    }
}

}  // namespace

hipError_t launch_copy(const float *src, float *dst, int64_t n, hipStream_t s)
{
    const int64_t grid = (n + 4095) / 4096;
    if (grid > 2147483647LL) return hipErrorInvalidValue;
    if (g_opt.copy_variant == 1)
        hipLaunchKernelGGL(copy_kernel<0>, dim3((unsigned)grid), dim3(256), 0, s, src, dst, n);
    else
        hipLaunchKernelGGL(copy_kernel<1>, dim3((unsigned)grid), dim3(256), 0, s, src, dst, n);
    return hipGetLastError();
}

}  // namespace sws
