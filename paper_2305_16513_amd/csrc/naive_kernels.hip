// Direct-evaluation kernels: one thread per output, the definition written out on the
// device.  They cover every legal argument combination and serve as the fallback for
// shapes the tuned kernels do not take (and as an A/B reference on the GPU itself).
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;

// Section 2.2, Eq. 3: y[r,i] = x[r,i] (+) ... (+) x[r,i+w-1], left to right, over the row
// extended by pad_left elements in front (boundary rule `pad_mode`); lo outputs per row.
template <int OP>
__global__ __launch_bounds__(kThreads) void slide_naive_kernel(const float *__restrict__ x,
                                                               float *__restrict__ y, int64_t rows,
                                                               int len, int lo, int w, int pad_left,
                                                               int pad_mode, float scale)
{
    using O = Op<OP>;
    const int64_t total = rows * (int64_t)lo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * kThreads) {
        const int64_t r = o / lo;
        const int i = (int)(o - r * lo);
        const float *xr = x + r * (int64_t)len;
        float acc = O::id();
        int real = 0;                                // elements that are not identity padding
        for (int j = 0; j < w; ++j) {
            const int src = pad_src(i + j, len, pad_left, pad_mode);
            acc = O::f(acc, src >= 0 ? xr[src] : O::id());
            real += src >= 0;
        }
        if (OP == SWS_OP_ADD) acc *= (pad_mode == SWS_PAD_SHRINK && real > 0) ? scale * (float)w / (float)real : scale;
        y[o] = acc;
    }
}

// Section 2.3 in two dimensions, separable order H then W evaluated per output.
template <int OP>
__global__ __launch_bounds__(kThreads) void pool2d_naive_kernel(const float *__restrict__ x,
                                                                float *__restrict__ y, int64_t planes,
                                                                int H, int W, int Ho, int Wo, int kh,
                                                                int kw, int sh, int sw, int ph, int pw,
                                                                float scale, int div_valid)
{
    using O = Op<OP>;
    const int64_t total = planes * (int64_t)Ho * Wo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * kThreads) {
        const int wo = (int)(o % Wo);
        const int ho = (int)((o / Wo) % Ho);
        const int64_t p = o / ((int64_t)Wo * Ho);
        const float *xp = x + p * (int64_t)H * W;
        float acc = O::id();
        int cells = 0;                               // window cells inside the plane
        for (int b = 0; b < kw; ++b) {
            const int c = wo * sw - pw + b;
            if (c < 0 || c >= W) continue;
            float col = O::id();
            for (int a = 0; a < kh; ++a) {
                const int h = ho * sh - ph + a;
                if (h < 0 || h >= H) continue;
                col = O::f(col, xp[(int64_t)h * W + c]);
                ++cells;
            }
            acc = O::f(acc, col);
        }
        if (OP == SWS_OP_ADD) acc *= div_valid ? scale / (float)cells : scale;
        y[o] = acc;
    }
}

// Section 2.5: sliding dot product, taps applied in index order (no flip); the row is extended by `pad`
// elements in front under the boundary rule `mode` (SWS_PAD_IDENTITY: zero padding).
__global__ __launch_bounds__(kThreads) void conv1d_naive_kernel(const float *__restrict__ x,
                                                                const float *__restrict__ wgt,
                                                                float *__restrict__ y, int64_t B, int Cin,
                                                                int L, int Cout, int Lo, int k, int stride,
                                                                int pad, int dilation, int groups, int mode)
{
    const int cig = Cin / groups, cog = Cout / groups;
    const int64_t total = B * (int64_t)Cout * Lo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * kThreads) {
        const int i = (int)(o % Lo);
        const int co = (int)((o / Lo) % Cout);
        const int64_t b = o / ((int64_t)Lo * Cout);
        const int g = co / cog;
        float acc = 0.0f;
        for (int ci = 0; ci < cig; ++ci) {
            const float *xr = x + (b * Cin + (int64_t)g * cig + ci) * L;
            const float *wr = wgt + ((int64_t)co * cig + ci) * k;
            for (int t = 0; t < k; ++t) {
                const int j = pad_src(i * stride + t * dilation, L, pad, mode);   // -1: zero padding
                if (j >= 0) acc = fmaf(wr[t], xr[j], acc);
            }
        }
        y[o] = acc;
    }
}

__global__ __launch_bounds__(kThreads) void conv2d_naive_kernel(const float *__restrict__ x,
                                                                const float *__restrict__ wgt,
                                                                float *__restrict__ y, int64_t N, int Cin,
                                                                int H, int W, int Cout, int Ho, int Wo,
                                                                int kh, int kw, int sh, int sw, int ph,
                                                                int pw)
{
    const int64_t total = N * (int64_t)Cout * Ho * Wo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * kThreads) {
        const int wo = (int)(o % Wo);
        const int ho = (int)((o / Wo) % Ho);
        const int co = (int)((o / ((int64_t)Wo * Ho)) % Cout);
        const int64_t n = o / ((int64_t)Wo * Ho * Cout);
        float acc = 0.0f;
        for (int ci = 0; ci < Cin; ++ci) {
            const float *xp = x + (n * Cin + ci) * (int64_t)H * W;
            const float *wp = wgt + ((int64_t)co * Cin + ci) * kh * kw;
            for (int a = 0; a < kh; ++a) {
                const int h = ho * sh - ph + a;
                if (h < 0 || h >= H) continue;
                for (int b = 0; b < kw; ++b) {
                    const int c = wo * sw - pw + b;
                    if (c >= 0 && c < W) acc = fmaf(wp[a * kw + b], xp[(int64_t)h * W + c], acc);
                }
            }
        }
        y[o] = acc;
    }
}

int grid_for(int64_t total)
{
    const int64_t want = (total + kThreads - 1) / kThreads;
    const int64_t cap = 256LL * 64;          // 64 workgroups per CU, grid-stride beyond
    return (int)(want < cap ? want : cap);
}

}  // namespace

hipError_t launch_slide1d_naive(int op, const float *x, float *y, int64_t rows, int64_t len, int32_t w,
                                int32_t pad_left, int32_t pad_right, int pad_mode, float scale, hipStream_t s)
{
    const int lo = (int)(len + pad_left + pad_right - w + 1);
    const int grid = grid_for(rows * lo);
    switch (op) {
    case SWS_OP_ADD:
        hipLaunchKernelGGL(slide_naive_kernel<SWS_OP_ADD>, dim3(grid), dim3(kThreads), 0, s, x, y, rows,
                           (int)len, lo, w, pad_left, pad_mode, scale);
        break;
    case SWS_OP_MAX:
        hipLaunchKernelGGL(slide_naive_kernel<SWS_OP_MAX>, dim3(grid), dim3(kThreads), 0, s, x, y, rows,
                           (int)len, lo, w, pad_left, pad_mode, scale);
        break;
    default:
        hipLaunchKernelGGL(slide_naive_kernel<SWS_OP_MIN>, dim3(grid), dim3(kThreads), 0, s, x, y, rows,
                           (int)len, lo, w, pad_left, pad_mode, scale);
        break;
    }
    return hipGetLastError();
}

hipError_t launch_pool2d_naive(int op, const float *x, float *y, int64_t planes, int64_t H, int64_t W,
                               int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                               int32_t ph, int32_t pw, float scale, int div_valid, hipStream_t s)
{
    const int grid = grid_for(planes * Ho * Wo);
#define SWS_LAUNCH_POOL(OPV)                                                                             \
    hipLaunchKernelGGL(pool2d_naive_kernel<OPV>, dim3(grid), dim3(kThreads), 0, s, x, y, planes, (int)H, \
                       (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw, scale, div_valid)
    switch (op) {
    case SWS_OP_ADD: SWS_LAUNCH_POOL(SWS_OP_ADD); break;
    case SWS_OP_MAX: SWS_LAUNCH_POOL(SWS_OP_MAX); break;
    default: SWS_LAUNCH_POOL(SWS_OP_MIN); break;
    }
#undef SWS_LAUNCH_POOL
    return hipGetLastError();
}

hipError_t launch_conv1d_naive(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin,
                               int64_t L, int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad,
                               int32_t dilation, int32_t groups, hipStream_t s, int mode)
{
    const int grid = grid_for(B * Cout * Lo);
    hipLaunchKernelGGL(conv1d_naive_kernel, dim3(grid), dim3(kThreads), 0, s, x, wgt, y, B, (int)Cin,
                       (int)L, (int)Cout, (int)Lo, k, stride, pad, dilation, groups, mode);
    return hipGetLastError();
}

hipError_t launch_conv2d_naive(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin,
                               int64_t H, int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh,
                               int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, hipStream_t s)
{
    const int grid = grid_for(N * Cout * Ho * Wo);
    hipLaunchKernelGGL(conv2d_naive_kernel, dim3(grid), dim3(kThreads), 0, s, x, wgt, y, N, (int)Cin,
                       (int)H, (int)W, (int)Cout, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw);
    return hipGetLastError();
}

}  // namespace sws
