// Calibration copy: the one-read-one-write pattern of the sliding kernels with no
// arithmetic, used to measure the bandwidth ceiling and to scale byte counters.
#include "sws_internal.h"

namespace sws {

namespace {

// Each workgroup moves 4096 consecutive floats, each wavefront a tile of 1024 of them as four
// fully coalesced 128-bit strips (lane l touches 16 bytes at 16*l within each 1 KB strip) — the
// tile shape and workgroup size of the sliding kernels.
template <int NT>
__global__ __launch_bounds__(256) void copy_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                   int64_t n)
{
    const int64_t base = (int64_t)blockIdx.x * 4096;
    if (base + 4096 <= n) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int64_t tile = base + wave * 1024;
        v4f r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const v4f_u *p = (const v4f_u *)(src + tile + j * 256 + 4 * lane);
            r[j] = NT == 2 ? __builtin_nontemporal_load(p) : *p;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v4f_u *p = (v4f_u *)(dst + tile + j * 256 + 4 * lane);
            if (NT) __builtin_nontemporal_store(r[j], p);
            else *p = r[j];
        }
    } else {
        for (int64_t o = base + threadIdx.x; o < n; o += 256) dst[o] = src[o];
    }
}

// The finest-grained copy: a workgroup is one wavefront and moves one 1 KB strip (one 128-bit
// access per lane).  Measured faster than the tile-shaped copy above (6.6-6.8 against 6.1 TB/s on
// 2 GiB): what HBM gives a kernel whose wavefronts need no more than 1 KB each, which the sliding
// kernels' 4 KB tiles (16 elements per lane for the scans) are not.
__global__ __launch_bounds__(64) void copy_fine_kernel(const float *__restrict__ src, float *__restrict__ dst, int64_t n)
{
    const int64_t base = (int64_t)blockIdx.x * 256;
    if (base + 256 <= n) {
        const v4f v = __builtin_nontemporal_load((const v4f_u *)(src + base + 4 * threadIdx.x));
        __builtin_nontemporal_store(v, (v4f_u *)(dst + base + 4 * threadIdx.x));
    } else {
        for (int64_t o = base + threadIdx.x; o < n; o += 64) dst[o] = src[o];
    }
}

}  // namespace

hipError_t launch_copy(const float *src, float *dst, int64_t n, hipStream_t s)
{
    if (g_opt.copy_variant == 4) {                   // one 1 KB strip per single-wavefront workgroup
        const int64_t fine = (n + 255) / 256;
        if (fine > 2147483647LL) return kNotTaken;
        if (fine > 0) hipLaunchKernelGGL(copy_fine_kernel, dim3((unsigned)fine), dim3(64), 0, s, src, dst, n);
        return hipGetLastError();
    }
    const int64_t grid = (n + 4095) / 4096;
    if (grid > 2147483647LL) return kNotTaken;
    // copy_variant: 0 non-temporal loads and stores (the fastest copy measured: 6.07 TB/s on 2 GiB),
    // 1 plain both (5.73), 3 plain loads + non-temporal stores, as the sliding kernels do (5.75),
    // 4 the fine-grained copy above
    if (g_opt.copy_variant == 1)
        hipLaunchKernelGGL(copy_kernel<0>, dim3((unsigned)grid), dim3(256), 0, s, src, dst, n);
    else if (g_opt.copy_variant == 3)
        hipLaunchKernelGGL(copy_kernel<1>, dim3((unsigned)grid), dim3(256), 0, s, src, dst, n);
    else
        hipLaunchKernelGGL(copy_kernel<2>, dim3((unsigned)grid), dim3(256), 0, s, src, dst, n);
    return hipGetLastError();
}

}  // namespace sws
