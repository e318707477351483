// sws_pool2d on small planes — 2-D pooling (Section 2.3) when a plane is a few hundred elements
// (the 7 x 7 and 14 x 14 planes of a network's last stages, with thousands of channels).
//
// The band kernel gives a wavefront to a band of one plane; on a 49-element plane that leaves most
// lanes idle.  Here a workgroup takes G whole planes: they are contiguous in memory, so they are
// staged into LDS as one range of 128-bit loads, and the G * Ho * Wo outputs — contiguous as well —
// are dealt to the threads one by one, each combining its window from LDS (down H, then across W,
// as the direct evaluation does) and stored coalesced.  Window cells outside the plane are skipped
// by clamping the loop bounds, so padding and real-cell averages cost nothing extra.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kStage = 4096;                         // floats of LDS per workgroup (16 KB)

typedef float v4f __attribute__((ext_vector_type(4)));

template <int OP>
__global__ __launch_bounds__(kThreads) void pool2d_small_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                int64_t planes, int H, int W, int Ho, int Wo, int kh,
                                                                int kw, int sh, int sw, int ph, int pw, float scale,
                                                                int div_valid, int G, unsigned rcp_q, unsigned rcp_wo)
{
    using O = Op<OP>;
    __shared__ __attribute__((aligned(16))) float lds[kStage];
    const int tid = threadIdx.x;
    const int P = H * W, Q = Ho * Wo;
    const int64_t p0 = (int64_t)blockIdx.x * G;
    const int g = planes - p0 < G ? (int)(planes - p0) : G;
    const float *src = x + p0 * P;
    const int n = g * P;
    if (((uintptr_t)src & 15) == 0) {
        const int n4 = n >> 2;
        for (int i = tid; i < n4; i += kThreads) *(v4f *)(lds + 4 * i) = *(const v4f *)(src + 4 * i);
        for (int i = 4 * n4 + tid; i < n; i += kThreads) lds[i] = src[i];
    } else {
        for (int i = tid; i < n; i += kThreads) lds[i] = src[i];
    }
    __syncthreads();
    float *dst = y + p0 * Q;
    const int m = g * Q;
    for (int o = tid; o < m; o += kThreads) {
        // o = (plane, ho, wo); the quotients by multiplication with 2^32 / d + 1 (exact: o < 2^16, d < 2^12)
        const int pl = Q == 1 ? o : (int)__umulhi((unsigned)o, rcp_q);
        const int cell = o - pl * Q;
        const int ho = Wo == 1 ? cell : (int)__umulhi((unsigned)cell, rcp_wo);
        const int wo = cell - ho * Wo;
        const float *xp = lds + pl * P;
        const int h0 = ho * sh - ph, c0 = wo * sw - pw;
        const int a_lo = h0 < 0 ? -h0 : 0, a_hi = kh < H - h0 ? kh : H - h0;
        const int b_lo = c0 < 0 ? -c0 : 0, b_hi = kw < W - c0 ? kw : W - c0;
        float acc = O::id();
        for (int b = b_lo; b < b_hi; ++b) {
            float col = O::id();
            for (int a = a_lo; a < a_hi; ++a) col = O::f(col, xp[(h0 + a) * W + c0 + b]);
            acc = O::f(acc, col);
        }
        if (OP == SWS_OP_ADD) {
            const int cells = (a_hi > a_lo ? a_hi - a_lo : 0) * (b_hi > b_lo ? b_hi - b_lo : 0);
            acc *= div_valid ? scale / (float)cells : scale;
        }
        dst[o] = acc;
    }
}

}  // namespace

// Planes of at most kStage / 4 elements.  *taken = false: not this kernel's case.
hipError_t launch_pool2d_small(int op, const float *x, float *y, int64_t planes, int H, int W, int Ho, int Wo, int kh,
                               int kw, int sh, int sw, int ph, int pw, float scale, int div_valid, hipStream_t s,
                               bool *taken)
{
    *taken = false;
    const int64_t P = (int64_t)H * W, Q = (int64_t)Ho * Wo;
    if (P < 1 || P > kStage / 4 || Q < 1 || Q > 4095 || Wo > 4095) return hipSuccess;
    // whole planes per workgroup, a multiple of four so that every workgroup's range starts on a
    // 16-byte boundary when x does
    const int G = (int)(kStage / P) & ~3;
    if ((int64_t)G * Q >= 65536) return hipSuccess;
    const int64_t grid = (planes + G - 1) / G;
    if (grid > 2147483647LL) return hipSuccess;
    *taken = true;
    const unsigned rcp_q = (unsigned)(4294967296ULL / (uint64_t)Q + 1), rcp_wo = (unsigned)(4294967296ULL / (uint64_t)Wo + 1);
#define SWS_PS(OPV)                                                                                                \
    hipLaunchKernelGGL((pool2d_small_kernel<OPV>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, planes, H, W, Ho, Wo, \
                       kh, kw, sh, sw, ph, pw, scale, div_valid, G, rcp_q, rcp_wo)
    switch (op) {
    case SWS_OP_ADD: SWS_PS(SWS_OP_ADD); break;
    case SWS_OP_MAX: SWS_PS(SWS_OP_MAX); break;
    default: SWS_PS(SWS_OP_MIN); break;
    }
#undef SWS_PS
    return hipGetLastError();
}

}  // namespace sws
