// sws_maxpool2d_grad — the adjoint of 2-D max pooling (Section 2.3's max operator, training side):
// every window sends its output gradient to the cell holding its maximum, the first such cell in
// row-major order when several tie.
//
// Gather form, no atomics, every gx element written exactly once and summed in a fixed order.  A
// wavefront owns a band of input rows of one plane.  It stages in its LDS slice the input rows every
// window touching the band can see (with -inf rows and columns where the plane ends, so that window
// scans need no bounds tests) and the gy rows of those windows; then
//   1. one lane per window scans its kh x kw cells in row-major order with a strict ">" and leaves
//      the LDS position of the maximum in an index row;
//   2. one lane per input cell walks the ceil(kh/sh) * ceil(kw/sw) windows that can cover it and
//      adds the gradients of those whose index is its own position.
// (Routing with LDS atomic adds instead of step 2 measured 2.5 x slower: an LDS atomic instruction
// costs about 150 cycles.)  Windows that straddle two bands are scanned by both.  HBM sees one read
// of x, one of gy and one write of gx (halo rows are re-read through L2).
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kSlice = 12 * 1024;                    // bytes of LDS per wavefront

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__host__ __device__ inline int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }
__host__ __device__ inline int ceil_div(int a, int b) { return -floor_div(-a, b); }

struct PgGeom {
    int H, W, Ho, Wo, kh, kw, sh, sw, ph, pw;
    int TH, bands;                                   // input rows per band, bands per plane
    int PX, pwl, PO;                                 // pitch of a staged x row, -inf columns in front of it, pitch of a window row
    int x_rows, w_rows;                              // most x rows / window rows a band needs
    int slice;                                       // floats per wavefront
};

// KH > 0: window extents and strides at compile time (scans unrolled, divisions by constants);
// KH = 0: everything taken from g.
template <int KH, int KW, int SH, int SW>
__global__ __launch_bounds__(kThreads) void maxpool2d_grad_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                  float *__restrict__ gx, PgGeom g, int64_t n_units)
{
    const int kh = KH > 0 ? KH : g.kh, kw = KH > 0 ? KW : g.kw, sh = KH > 0 ? SH : g.sh, sw = KH > 0 ? SW : g.sw;
    extern __shared__ __attribute__((aligned(16))) float lds_all[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t unit = (int64_t)blockIdx.x * kWaves + wave;
    if (unit >= n_units) return;
    float *X = lds_all + wave * g.slice;             // [x_rows][PX]
    float *G = X + g.x_rows * g.PX;                  // [w_rows][PO]  gy of the windows touching the band
    int *IDX = (int *)(G + g.w_rows * g.PO);         // [w_rows][PO]  where each window's maximum sits in X
    const int64_t plane = unit / g.bands;
    const int band = (int)(unit - plane * g.bands);
    const float *xp = x + plane * (int64_t)g.H * g.W;
    const float *gp = gy + plane * (int64_t)g.Ho * g.Wo;
    float *op = gx + plane * (int64_t)g.H * g.W;
    const int h0 = band * g.TH;
    const int h1 = h0 + g.TH < g.H ? h0 + g.TH : g.H;
    // windows (rows ho_lo .. ho_hi) that contain at least one row of the band
    int ho_lo = ceil_div(h0 + g.ph - kh + 1, sh), ho_hi = floor_div(h1 - 1 + g.ph, sh);
    if (ho_lo < 0) ho_lo = 0;
    if (ho_hi > g.Ho - 1) ho_hi = g.Ho - 1;
    const int nwr = ho_hi - ho_lo + 1;               // may be <= 0: no window reaches the band
    const int xr_lo = ho_lo * sh - g.ph;             // first (possibly virtual) x row they see
    const int nxr = nwr > 0 ? (nwr - 1) * sh + kh : 0;
    const float ninf = -__builtin_huge_valf();

    // ---- stage x rows xr_lo .. xr_lo + nxr - 1 (columns -pwl .. PX - pwl - 1), -inf outside the plane,
    //      and the gy rows; eight loads per lane are issued before the first LDS write
    {
        constexpr int U = 8;
        const float inv_px = 1.0f / (float)g.PX;
        for (int i0 = 0; i0 < nxr * g.PX; i0 += kWave * U) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                const int r = (int)(((float)i + 0.5f) * inv_px), c = i - r * g.PX - g.pwl;
                const int h = xr_lo + r;
                const bool ok = i < nxr * g.PX && h >= 0 && h < g.H && c >= 0 && c < g.W;
                v[u] = xp[ok ? (int64_t)h * g.W + c : 0];
                v[u] = ok ? v[u] : ninf;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                if (i < nxr * g.PX) X[i] = v[u];
            }
        }
        const float inv_po = 1.0f / (float)g.PO;
        for (int i0 = 0; i0 < nwr * g.PO; i0 += kWave * U) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                const int r = (int)(((float)i + 0.5f) * inv_po), c = i - r * g.PO;
                const bool ok = i < nwr * g.PO && c < g.Wo;
                v[u] = gp[ok ? (int64_t)(ho_lo + r) * g.Wo + c : 0];
                v[u] = ok ? v[u] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                if (i < nwr * g.PO) G[i] = v[u];
            }
        }
    }
    wave_lds_sync();
    // ---- 1. the position of every window's maximum
    {
        const float inv_wo = 1.0f / (float)g.Wo;
        for (int i = lane; i < nwr * g.Wo; i += kWave) {
            const int r = (int)(((float)i + 0.5f) * inv_wo), wo = i - r * g.Wo;
            const int base = r * sh * g.PX + g.pwl - g.pw + wo * sw;       // the window's first cell
            float best = ninf;
            int at = base;
            if (KH > 0) {
                float v[(KH > 0 ? KH : 1) * (KW > 0 ? KW : 1)];
#pragma unroll
                for (int a = 0; a < KH; ++a)
#pragma unroll
                    for (int b = 0; b < KW; ++b) v[a * KW + b] = X[base + a * g.PX + b];     // all reads before the first compare
#pragma unroll
                for (int a = 0; a < KH; ++a)
#pragma unroll
                    for (int b = 0; b < KW; ++b) {
                        const bool gt = v[a * KW + b] > best;
                        best = gt ? v[a * KW + b] : best;
                        at = gt ? base + a * g.PX + b : at;
                    }
            } else {
                for (int a = 0; a < kh; ++a) {
                    const int ra = base + a * g.PX;
                    for (int b = 0; b < kw; ++b) {
                        const float v = X[ra + b];
                        const bool gt = v > best;
                        best = gt ? v : best;
                        at = gt ? ra + b : at;
                    }
                }
            }
            IDX[r * g.PO + wo] = at;
        }
    }
    wave_lds_sync();
    // ---- 2. every cell of the band collects the windows that chose it: rows a_hi, a_hi - 1, ... and
    //      columns b_hi, b_hi - 1, ... of windows, NA x NB candidates (those outside the ranges are masked)
    {
        const float inv_w = 1.0f / (float)g.W;
        const int nrows = h1 - h0;
        const int NA = (kh + sh - 1) / sh, NB = (kw + sw - 1) / sw;
        for (int i = lane; i < nrows * g.W; i += kWave) {
            const int r = (int)(((float)i + 0.5f) * inv_w), c = i - r * g.W;
            const int h = h0 + r;
            const int me = (h - xr_lo) * g.PX + g.pwl + c;
            // h + ph and c + pw are >= 0: plain division is the floor
            int a_hi = (h + g.ph) / sh, b_hi = (c + g.pw) / sw;
            int a_lo = (h + g.ph - kh + sh) / sh, b_lo = (c + g.pw - kw + sw) / sw;   // ceil((.. - k + 1) / s), numerator + s - 1
            if (h + g.ph - kh + 1 <= 0) a_lo = 0;
            if (c + g.pw - kw + 1 <= 0) b_lo = 0;
            if (a_lo < ho_lo) a_lo = ho_lo;
            if (a_hi > ho_hi) a_hi = ho_hi;
            if (b_hi > g.Wo - 1) b_hi = g.Wo - 1;
            float acc = 0.0f;
            auto candidate = [&](int da, int db) {
                const int ho = a_hi - da, wo = b_hi - db;
                const bool ok = ho >= a_lo && wo >= b_lo;
                const int at = ok ? (ho - ho_lo) * g.PO + wo : 0;
                const int idx = IDX[at];
                const float gv = G[at];
                acc += (ok && idx == me) ? gv : 0.0f;
            };
            if (KH > 0) {
                constexpr int CA = KH > 0 ? (KH + SH - 1) / SH : 1, CB = KH > 0 ? (KW + SW - 1) / SW : 1;
#pragma unroll
                for (int da = CA - 1; da >= 0; --da)
#pragma unroll
                    for (int db = CB - 1; db >= 0; --db) candidate(da, db);
            } else {
                for (int da = NA - 1; da >= 0; --da)
                    for (int db = NB - 1; db >= 0; --db) candidate(da, db);
            }
            __builtin_nontemporal_store(acc, op + (int64_t)h * g.W + c);
        }
    }
}

// Direct evaluation for planes whose rows do not fit the slice: one thread per input cell, window
// maxima recomputed from global memory.
__global__ __launch_bounds__(kThreads) void maxpool2d_grad_naive_kernel(const float *__restrict__ x,
                                                                        const float *__restrict__ gy,
                                                                        float *__restrict__ gx, int64_t planes, int H, int W,
                                                                        int Ho, int Wo, int kh, int kw, int sh, int sw,
                                                                        int ph, int pw)
{
    const int64_t total = planes * (int64_t)H * W;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int c = (int)(o % W);
        const int h = (int)((o / W) % H);
        const int64_t p = o / ((int64_t)W * H);
        const float *xp = x + p * (int64_t)H * W;
        int a_lo = ceil_div(h + ph - kh + 1, sh), a_hi = floor_div(h + ph, sh);
        int b_lo = ceil_div(c + pw - kw + 1, sw), b_hi = floor_div(c + pw, sw);
        if (a_lo < 0) a_lo = 0;
        if (a_hi > Ho - 1) a_hi = Ho - 1;
        if (b_lo < 0) b_lo = 0;
        if (b_hi > Wo - 1) b_hi = Wo - 1;
        float acc = 0.0f;
        for (int ho = a_lo; ho <= a_hi; ++ho)
            for (int wo = b_lo; wo <= b_hi; ++wo) {
                int best_h = -1, best_c = -1;
                float best = -__builtin_huge_valf();
                for (int a = 0; a < kh; ++a) {
                    const int hh = ho * sh - ph + a;
                    if (hh < 0 || hh >= H) continue;
                    for (int b = 0; b < kw; ++b) {
                        const int cc = wo * sw - pw + b;
                        if (cc < 0 || cc >= W) continue;
                        const float v = xp[(int64_t)hh * W + cc];
                        if (v > best) { best = v; best_h = hh; best_c = cc; }
                    }
                }
                if (best_h == h && best_c == c) acc += gy[(p * Ho + ho) * (int64_t)Wo + wo];
            }
        gx[o] = acc;
    }
}

}  // namespace

hipError_t launch_maxpool2d_grad(const float *x, const float *gy, float *gx, int64_t planes, int64_t H, int64_t W,
                                 int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph,
                                 int32_t pw, hipStream_t s)
{
    PgGeom g;
    g.H = (int)H; g.W = (int)W; g.Ho = (int)Ho; g.Wo = (int)Wo; g.kh = kh; g.kw = kw; g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.pwl = pw;
    int right = (int)((Wo - 1) * sw - pw + kw - W);   // columns a window reaches beyond the plane
    if (right < 0) right = 0;
    g.PX = (int)W + pw + right;
    g.PO = (int)Wo;
    // rows per band: the most that fit the slice (a band of TH rows is touched by up to
    // (TH + kh - 2) / sh + 2 window rows, which see up to (that - 1) * sh + kh input rows)
    int TH = H < 64 ? (int)H : 64;
    for (; TH >= 1; --TH) {
        g.w_rows = (TH + kh - 2) / sh + 2;
        g.x_rows = (g.w_rows - 1) * sh + kh;
        g.slice = (g.x_rows * g.PX + 2 * g.w_rows * g.PO + 3) / 4 * 4;
        if ((size_t)g.slice * 4 <= (size_t)kSlice) break;
    }
    const bool fits = TH >= 1 && g_opt.pool2d_variant != 1 && (int64_t)g.x_rows * g.PX < (1 << 20) && H * W < (1 << 20);
    if (fits) {
        g.TH = TH;
        g.bands = (int)((H + TH - 1) / TH);
        const int64_t n_units = planes * g.bands;
        const int64_t grid = (n_units + kWaves - 1) / kWaves;
        if (grid <= 2147483647LL) {
#define SWS_PG(KH, KW, SH, SW)                                                                                   \
    hipLaunchKernelGGL((maxpool2d_grad_kernel<KH, KW, SH, SW>), dim3((unsigned)grid), dim3(kThreads),                \
                       (size_t)g.slice * 4 * kWaves, s, x, gy, gx, g, n_units)
            if (kh == 3 && kw == 3 && sh == 1 && sw == 1) SWS_PG(3, 3, 1, 1);
            else if (kh == 3 && kw == 3 && sh == 2 && sw == 2) SWS_PG(3, 3, 2, 2);
            else if (kh == 2 && kw == 2 && sh == 2 && sw == 2) SWS_PG(2, 2, 2, 2);
            else SWS_PG(0, 0, 1, 1);
#undef SWS_PG
            return hipGetLastError();
        }
    }
    int64_t grid = (planes * H * W + kThreads - 1) / kThreads;
    if (grid > 1048576) grid = 1048576;
    hipLaunchKernelGGL(maxpool2d_grad_naive_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, x, gy, gx, planes, (int)H,
                       (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw);
    return hipGetLastError();
}

}  // namespace sws
