// sws_pool2d — 2-D pooling as separable sliding sums (Section 2.3 carried to two
// dimensions): first the sliding sum down H, then the sliding sum along W, both on a
// tile that stays on chip, so HBM sees one read of x and one write of y.
//
// A wavefront stages a band of input rows of one plane in its own LDS slice with coalesced
// 128-bit loads (the band is one contiguous range of the plane); there is no workgroup
// barrier, the four wavefronts of a workgroup work on four consecutive bands.  A lane then
// owns four adjacent output columns and R consecutive output rows: it reads the
// (R-1)*SH+KH input rows of its column window once, combines them down H (each input row is
// shared by up to KH output rows), then slides the KW-window along W in registers.  Cells
// outside the plane hold the identity of the operator.  Bands are small (a few KB in, a few KB
// out per wavefront) so that the tiles in flight form a compact window sweeping through memory.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kLdsBudget = 8 * 1024;                 // bytes of LDS per wavefront

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// R = consecutive output rows per lane: 4 at stride 1 (each staged row feeds up to KH of them);
// 1 at larger strides, where rows overlap little and consecutive lanes then store one
// contiguous run of y.
template <int SH> struct RowsPerItem { static constexpr int value = (SH == 1) ? 4 : 1; };

template <int OP, int KH, int KW, int SH, int SW, int PW>
__global__ __launch_bounds__(kThreads) void pool2d_band_kernel(
    const float *__restrict__ x, float *__restrict__ y, int H, int W, int Ho, int Wo, int ph, int P, int TH,
    int bands, float scale, int64_t n_units, int lds_floats, int flags)
{
    using O = Op<OP>;
    constexpr int R = RowsPerItem<SH>::value;
    constexpr int NR = (R - 1) * SH + KH;            // input rows per item
    constexpr int LPAD = (PW + 3) / 4 * 4;           // aligned columns read left of the window
    constexpr int OFF = LPAD - PW;                   // window start inside the aligned read
    constexpr int NC = 3 * SW + KW;                  // input columns per item
    constexpr int NG = (OFF + NC + 3) / 4;           // aligned 4-column groups per input row
    extern __shared__ __attribute__((aligned(16))) float lds_all[];

    // flag bits: 2 = XCD-contiguous placement of workgroups (default: launch order), 4 = plain stores,
    // 8 = ADD results are divided by the number of window cells inside the plane
    const int64_t wg = (flags & 2) ? xcd_unit((n_units + kWaves - 1) / kWaves) : (int64_t)blockIdx.x;
    if (wg < 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t unit = wg * kWaves + wave;          // one band per wavefront
    if (unit >= n_units) return;
    float *lds = lds_all + wave * lds_floats;
    const int64_t plane = unit / bands;
    const int band = (int)(unit - plane * bands);
    const float *xp = x + plane * (int64_t)H * W;
    float *yp = y + plane * (int64_t)Ho * Wo;
    const int ho0 = band * TH;                       // first output row of the band
    int ho1 = ho0 + TH;
    if (ho1 > Ho) ho1 = Ho;
    int row_lo = ho0 * SH - ph;                      // input rows [row_lo, row_hi) feed the band
    int row_hi = (ho1 - 1) * SH - ph + KH;
    if (row_lo < 0) row_lo = 0;
    if (row_hi > H) row_hi = H;

    // ---- stage the band
    if (P == W) {
        // the band is one contiguous range: all its 128-bit loads are issued before the first
        // LDS write (lanes past the end re-read element 0 and drop it)
        const float *src = xp + (int64_t)row_lo * W;
        const int n = (row_hi - row_lo) * W;         // multiple of 4, at most kLdsBudget / 4
        constexpr int NL = kLdsBudget / 16 / kWave;
        v4f g[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int i = 4 * (lane + kWave * j);
            g[j] = *(const v4f_u *)(src + (i < n ? i : 0));
        }
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int i = 4 * (lane + kWave * j);
            if (i < n) *(v4f *)(lds + i) = g[j];
        }
    } else {
        const int n = (row_hi - row_lo) * P;
        for (int i = lane; i < n; i += kWave) {
            const int r = i / P, c = i - r * P;
            lds[i] = (c < W) ? xp[(int64_t)(row_lo + r) * W + c] : O::id();
        }
    }
    wave_lds_sync();

    // ---- items: (row block, column group), column group fastest
    const int CG = (Wo + 3) / 4;
    const int RB = (ho1 - ho0 + R - 1) / R;
    for (int item = lane; item < CG * RB; item += kWave) {
        const int rb = item / CG, cg = item - rb * CG;
        const int ho = ho0 + rb * R;
        const int hin0 = ho * SH - ph;               // first input row of the item
        const int a0 = 4 * cg * SW - LPAD;           // first aligned column read
        float in[NR][4 * NG];
#pragma unroll
        for (int rr = 0; rr < NR; ++rr) {
            const int row = hin0 + rr;
            const bool row_ok = (row >= row_lo) && (row < row_hi);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int col = a0 + 4 * g;
                v4f v = {O::id(), O::id(), O::id(), O::id()};
                if (row_ok && col >= 0 && col < P) v = *(const v4f *)(lds + (row - row_lo) * P + col);
                in[rr][4 * g] = v.x; in[rr][4 * g + 1] = v.y; in[rr][4 * g + 2] = v.z; in[rr][4 * g + 3] = v.w;
            }
        }
#pragma unroll
        for (int ro = 0; ro < R; ++ro) {
            if (ho + ro >= ho1) break;
            // sliding sum down H ...
            float v[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                float acc = in[ro * SH][OFF + c];
#pragma unroll
                for (int a = 1; a < KH; ++a) acc = O::f(acc, in[ro * SH + a][OFF + c]);
                v[c] = acc;
            }
            // ... then along W
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float acc = v[e * SW];
#pragma unroll
                for (int b = 1; b < KW; ++b) acc = O::f(acc, v[e * SW + b]);
                if (OP == SWS_OP_ADD) {
                    float sc = scale;
                    if (flags & 8) {                 // real cells of this window: rows x columns inside the plane
                        const int h0 = hin0 + ro * SH, c0 = (4 * cg + e) * SW - PW;
                        const int nr = (h0 + KH < H ? h0 + KH : H) - (h0 > 0 ? h0 : 0);
                        const int nc = (c0 + KW < W ? c0 + KW : W) - (c0 > 0 ? c0 : 0);
                        sc = scale / (float)(nr * nc);
                    }
                    acc *= sc;
                }
                o[e] = acc;
            }
            float *dst = yp + (int64_t)(ho + ro) * Wo + 4 * cg;
            if (4 * cg + 4 <= Wo) {
                if (flags & 4) *(v4f_u *)dst = (v4f){o[0], o[1], o[2], o[3]};
                else __builtin_nontemporal_store((v4f){o[0], o[1], o[2], o[3]}, (v4f_u *)dst);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * cg + e < Wo) dst[e] = o[e];
            }
        }
    }
}

struct BandPlan {
    int P, TH, bands, threads;
    size_t lds_bytes;
    bool ok;
};

BandPlan plan_bands(int W, int Ho, int Wo, int KH, int SH, int R)
{
    BandPlan p;
    p.P = (W + 3) / 4 * 4;
    // Aim for about 4.5 KB of staged input per wavefront (measured best on 112x112 planes: 10
    // input rows, i.e. 8 output rows at stride 1 and 4 at stride 2), never more than the slice.
    const int want_rows = 4608 / (4 * p.P);
    int th = (want_rows - KH) / SH + 1;
    if (g_opt.slide_group > 0) th = g_opt.slide_group;
    th = th / R * R;
    if (th < R) th = R;
    if (th > (Ho + R - 1) / R * R) th = (Ho + R - 1) / R * R;
    p.TH = th;
    p.bands = (Ho + th - 1) / th;
    p.lds_bytes = (size_t)((th - 1) * SH + KH) * p.P * 4;
    p.ok = p.lds_bytes <= (size_t)kLdsBudget;
    p.threads = kThreads;
    return p;
}

template <int OP, int KH, int KW, int SH, int SW, int PW>
hipError_t launch_band(const float *x, float *y, int64_t planes, int H, int W, int Ho, int Wo, int ph, float scale,
                       int div_valid, hipStream_t s, bool *taken)
{
    const BandPlan p = plan_bands(W, Ho, Wo, KH, SH, RowsPerItem<SH>::value);
    *taken = p.ok;
    if (!p.ok) return hipSuccess;
    const int64_t n_units = planes * p.bands;
    const int flags = (g_opt.pool2d_variant & 6) | (div_valid ? 8 : 0);
    const int64_t n_wg = (n_units + kWaves - 1) / kWaves;
    const int64_t grid = (flags & 2) ? xcd_grid(n_wg) : n_wg;
    if (grid > 2147483647LL) { *taken = false; return hipSuccess; }
    hipLaunchKernelGGL((pool2d_band_kernel<OP, KH, KW, SH, SW, PW>), dim3((unsigned)grid), dim3(kThreads),
                       p.lds_bytes * kWaves, s, x, y, H, W, Ho, Wo, ph, p.P, p.TH, p.bands, scale, n_units,
                       (int)(p.lds_bytes / 4), flags);
    return hipGetLastError();
}

template <int OP>
hipError_t dispatch_band(const float *x, float *y, int64_t planes, int H, int W, int Ho, int Wo, int kh, int kw,
                         int sh, int sw, int ph, int pw, float scale, int div_valid, hipStream_t s, bool *taken)
{
#define SWS_BAND(KH, KW, SH, SW, PW)                                                                  \
    if (kh == KH && kw == KW && sh == SH && sw == SW && pw == PW)                                      \
        return launch_band<OP, KH, KW, SH, SW, PW>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken)
    SWS_BAND(3, 3, 1, 1, 1);
    SWS_BAND(3, 3, 2, 2, 1);
    SWS_BAND(3, 3, 1, 1, 0);
    SWS_BAND(3, 3, 2, 2, 0);
    SWS_BAND(2, 2, 2, 2, 0);
    SWS_BAND(2, 2, 1, 1, 0);
    SWS_BAND(5, 5, 1, 1, 2);
    SWS_BAND(5, 5, 1, 1, 0);
    SWS_BAND(7, 7, 1, 1, 3);
    SWS_BAND(9, 9, 1, 1, 4);
    SWS_BAND(13, 13, 1, 1, 6);
#undef SWS_BAND
    *taken = false;
    return hipSuccess;
}

}  // namespace

hipError_t launch_pool2d(int op, const float *x, float *y, int64_t planes, int64_t H, int64_t W, int64_t Ho,
                         int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                         float scale, int div_valid, hipStream_t s)
{
    // ph / pw are the top / left padding; the bottom / right padding is implied by Ho / Wo (cells
    // beyond the plane hold the identity whichever side they are on).
    if (g_opt.pool2d_variant != 1) {
        bool taken = false;
        hipError_t e;
        switch (op) {
        case SWS_OP_ADD:
            e = dispatch_band<SWS_OP_ADD>(x, y, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw,
                                          scale, div_valid, s, &taken);
            break;
        case SWS_OP_MAX:
            e = dispatch_band<SWS_OP_MAX>(x, y, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw,
                                          scale, div_valid, s, &taken);
            break;
        default:
            e = dispatch_band<SWS_OP_MIN>(x, y, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw,
                                          scale, div_valid, s, &taken);
            break;
        }
        if (taken) return e;
    }
    return launch_pool2d_naive(op, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s);
}

}  // namespace sws
