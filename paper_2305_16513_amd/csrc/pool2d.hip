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

// Element types in memory: fp32, or bf16 / fp16 widened exactly on the way in and rounded to nearest
// even once on the way out (all arithmetic is fp32).
template <typename T> struct Io;
template <> struct Io<float> {
    static __device__ __forceinline__ v4f load4(const float *p) { return *(const v4f_u *)p; }
    static __device__ __forceinline__ float load1(const float *p) { return *p; }
    static __device__ __forceinline__ void store1(float *p, float v) { *p = v; }
    static __device__ __forceinline__ void store1_nt(float *p, float v) { __builtin_nontemporal_store(v, p); }
    static __device__ __forceinline__ void store4(float *p, v4f o, bool plain)
    {
        if (plain) *(v4f_u *)p = o;
        else __builtin_nontemporal_store(o, (v4f_u *)p);
    }
    typedef v2f v2f_u __attribute__((aligned(4)));
    static __device__ __forceinline__ void store2_nt(float *p, v2f o) { __builtin_nontemporal_store(o.x, p); __builtin_nontemporal_store(o.y, p + 1); }
};
template <typename T> struct Io16 {
    typedef T v4 __attribute__((ext_vector_type(4)));
    typedef v4 v4_u __attribute__((aligned(2)));
    static __device__ __forceinline__ v4f load4(const T *p) { return __builtin_convertvector(*(const v4_u *)p, v4f); }
    static __device__ __forceinline__ float load1(const T *p) { return (float)*p; }
    static __device__ __forceinline__ void store1(T *p, float v) { *p = (T)v; }
    static __device__ __forceinline__ void store1_nt(T *p, float v) { *p = (T)v; }
    static __device__ __forceinline__ void store4(T *p, v4f o, bool plain)
    {
        const v4 h = __builtin_convertvector(o, v4);
        if (plain) *(v4_u *)p = h;
        else __builtin_nontemporal_store(h, (v4_u *)p);
    }
    typedef T v2 __attribute__((ext_vector_type(2)));
    typedef v2 v2_u __attribute__((aligned(2)));
    static __device__ __forceinline__ void store2_nt(T *p, v2f o) { __builtin_nontemporal_store(__builtin_convertvector(o, v2), (v2_u *)p); }
};
template <> struct Io<__bf16> : Io16<__bf16> {};
template <> struct Io<_Float16> : Io16<_Float16> {};

// R = consecutive output rows per lane: 4 at stride 1 (each staged row feeds up to KH of them);
// 1 at larger strides, where rows overlap little and consecutive lanes then store one
// contiguous run of y.
template <int SH> struct RowsPerItem { static constexpr int value = (SH == 1) ? 4 : 1; };

template <int OP, int KH, int KW, int SH, int SW, int PW, typename T>
__global__ __launch_bounds__(kThreads) void pool2d_band_kernel(
    const T *__restrict__ x, T *__restrict__ y, int H, int W, int Ho, int Wo, int ph, int P, int TH,
    int bands, float scale, int64_t n_units, int lds_floats, int flags)
{
    using O = Op<OP>;
    using IO = Io<T>;
    constexpr int R = RowsPerItem<SH>::value;
    constexpr int NR = (R - 1) * SH + KH;            // input rows per item
    constexpr int LPAD = (PW + 3) / 4 * 4;           // aligned columns read left of the window
    constexpr int OFF = LPAD - PW;                   // window start inside the aligned read
    constexpr int NC = 3 * SW + KW;                  // input columns per item
    constexpr int NG = (OFF + NC + 3) / 4;           // aligned 4-column groups per input row
    extern __shared__ __attribute__((aligned(16))) float lds_all[];

    // flag bits: 2 = XCD-contiguous placement of workgroups (default: launch order),
    // 8 = ADD results are divided by the number of window cells inside the plane
    const int wpb = blockDim.x >> 6;                 // wavefronts per workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t plane;
    int band;
    if (flags & 16) {
        // workgroup b runs on XCD b mod 8: XCD x takes the planes 8q + x, band by band, so that the
        // eight L2s work on eight adjacent planes and a band's halo rows are in the L2 that fetched them
        const int64_t k = ((int64_t)blockIdx.x >> 3) * wpb + wave;
        const int64_t q = k / bands;
        band = (int)(k - q * bands);
        plane = q * kXcd + (blockIdx.x & 7);
        if (plane * bands + band >= n_units) return;
    } else {
        const int64_t wg = (flags & 2) ? xcd_unit((n_units + wpb - 1) / wpb) : (int64_t)blockIdx.x;
        if (wg < 0) return;
        const int64_t unit = wg * wpb + wave;         // one band per wavefront
        if (unit >= n_units) return;
        plane = unit / bands;
        band = (int)(unit - plane * bands);
    }
    float *lds = lds_all + wave * lds_floats;
    const T *xp = x + plane * (int64_t)H * W;
    T *yp = y + plane * (int64_t)Ho * Wo;
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
        const T *src = xp + (int64_t)row_lo * W;
        const int n = (row_hi - row_lo) * W;         // multiple of 4, at most kLdsBudget / 4
        constexpr int NL = kLdsBudget / 16 / kWave;
        // Loads go in four chunks, the third and fourth only if the band reaches them (wave-uniform
        // tests), so that a short band does not issue loads it drops.  (Streaming loads for the rows no
        // other band stages were measured: no difference.)
        constexpr int NQ = NL / 4;
        v4f g[NL];
        auto load = [&](int j0, int j1) {
#pragma unroll
            for (int j = j0; j < j1; ++j) {
                const int i = 4 * (lane + kWave * j);
                g[j] = IO::load4(src + (i < n ? i : 0));
            }
        };
        auto keep = [&](int j0, int j1) {
#pragma unroll
            for (int j = j0; j < j1; ++j) {
                const int i = 4 * (lane + kWave * j);
                if (i < n) *(v4f *)(lds + i) = g[j];
            }
        };
        load(0, 2 * NQ);
        if (n > 4 * kWave * 2 * NQ) {
            load(2 * NQ, 3 * NQ);
            if (n > 4 * kWave * 3 * NQ) {
                load(3 * NQ, NL);
                keep(3 * NQ, NL);
            }
            keep(2 * NQ, 3 * NQ);
        }
        keep(0, 2 * NQ);
    } else {
        const int n = (row_hi - row_lo) * P;
        for (int i = lane; i < n; i += kWave) {
            const int r = i / P, c = i - r * P;
            lds[i] = (c < W) ? IO::load1(xp + (int64_t)(row_lo + r) * W + c) : O::id();
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
            T *dst = yp + (int64_t)(ho + ro) * Wo + 4 * cg;
            if (4 * cg + 4 <= Wo) {
                // always non-temporal: a run-time choice between a plain and a non-temporal store of the
                // same value makes the compiler merge the two into one plain store
                IO::store4(dst, (v4f){o[0], o[1], o[2], o[3]}, false);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * cg + e < Wo) IO::store1(dst + e, o[e]);
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

template <int OP, int KH, int KW, int SH, int SW, int PW, typename T>
hipError_t launch_band(const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int ph, float scale,
                       int div_valid, hipStream_t s, bool *taken)
{
    const BandPlan p = plan_bands(W, Ho, Wo, KH, SH, RowsPerItem<SH>::value);
    *taken = p.ok;
    if (!p.ok) return hipSuccess;
    const int64_t n_units = planes * p.bands;
    // default: single-wavefront workgroups, planes dealt cyclically to the XCDs (measured on [2048,112,112]
    // under rotating buffers: 36.0 / 22.7 us at stride 1 / 2 against 37.0 / 23.2 us for four-wavefront
    // workgroups in launch order, which option bit 512 brings back; bit 2: the XCD-contiguous placement)
    const bool old_shape = (g_opt.pool2d_variant & (512 | 2)) != 0;
    const int flags = (g_opt.pool2d_variant & 2) | (old_shape ? 0 : 16) | (div_valid ? 8 : 0);
    const int wpb = old_shape ? kWaves : 1;
    const int64_t n_wg = (n_units + wpb - 1) / wpb;
    int64_t grid = (flags & 2) ? xcd_grid(n_wg) : n_wg;
    if (flags & 16) grid = (((planes + kXcd - 1) / kXcd * p.bands + wpb - 1) / wpb) * kXcd;
    if (grid > 2147483647LL) { *taken = false; return hipSuccess; }
    hipLaunchKernelGGL((pool2d_band_kernel<OP, KH, KW, SH, SW, PW, T>), dim3((unsigned)grid), dim3(wpb * kWave),
                       p.lds_bytes * wpb, s, x, y, H, W, Ho, Wo, ph, p.P, p.TH, p.bands, scale, n_units,
                       (int)(p.lds_bytes / 4), flags);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Any window, stride and padding: the same separable evaluation with the geometry at run time.
// A wavefront stages the input rows of a band of TH output rows, reduces them down H into a
// second LDS array (one row per output row, kh combines per column), then reduces along W from
// there (kw combines per output): kh + kw combines per output where direct evaluation does kh*kw,
// and HBM still sees one read of x and one write of y.
// ------------------------------------------------------------------------------------------------
constexpr int kSepLds = 12 * 1024;                   // bytes of LDS per wavefront

template <int OP, typename T>
__global__ __launch_bounds__(kThreads) void pool2d_sep_kernel(const T *__restrict__ x, T *__restrict__ y, int H,
                                                              int W, int Ho, int Wo, int kh, int kw, int sh, int sw,
                                                              int ph, int pw, int P, int PC, int pwl, int TH, int bands,
                                                              float scale, int64_t n_units, int lds_floats,
                                                              int in_rows, int div_valid, int ctiles, int TWO)
{
    using O = Op<OP>;
    using IO = Io<T>;
    extern __shared__ __attribute__((aligned(16))) float lds_all[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t unit = (int64_t)blockIdx.x * kWaves + wave;
    if (unit >= n_units) return;
    // Planes whose rows do not fit the slice are cut into ctiles column tiles of TWO outputs each
    // (ctiles = 1: the whole width).  A column tile stages the input columns its windows see,
    // identity where they leave the plane, and needs no margins in `col` (pwl = 0, PC = P).
    // in:  [in_rows][P]  the input rows hv0 .. hv0 + in_rows - 1 of the band, rows outside the plane
    //                    (and columns W .. P-1) holding the identity, so that the loop over kh needs no bounds
    // col: [TH][PC]      those rows reduced down H, with pwl identity columns in front and enough
    //                    behind that the loop over kw needs none either
    float *in = lds_all + wave * lds_floats;
    float *col = in + in_rows * P;
    const bool tiled = ctiles > 1;
    const int ct = (int)(unit % ctiles);
    const int64_t pb = unit / ctiles;
    const int64_t plane = pb / bands;
    const int band = (int)(pb - plane * bands);
    const T *xp = x + plane * (int64_t)H * W;
    T *yp = y + plane * (int64_t)Ho * Wo;
    const int ho0 = band * TH;
    int ho1 = ho0 + TH;
    if (ho1 > Ho) ho1 = Ho;
    const int nr = ho1 - ho0;
    const int wo0 = ct * TWO;                        // my outputs: columns wo0 .. wo1 - 1
    const int wo1 = wo0 + TWO < Wo ? wo0 + TWO : Wo;
    const int nwo = wo1 - wo0;
    const int c_first = tiled ? wo0 * sw - pw : 0;   // plane column of staged column 0
    const int hv0 = ho0 * sh - ph;                   // first (possibly virtual) input row of the band
    const int rows_need = (nr - 1) * sh + kh;
    int row_lo = hv0 < 0 ? 0 : hv0, row_hi = hv0 + rows_need > H ? H : hv0 + rows_need;
    const int P4 = P >> 2;
    const float inv_p4 = 1.0f / (float)P4;
    const v4f id4 = {O::id(), O::id(), O::id(), O::id()};
    // ---- stage: identity rows above and below the plane, then the real rows
    for (int i = lane; i < (row_lo - hv0) * P4; i += kWave) *(v4f *)(in + 4 * i) = id4;
    for (int i = (row_hi - hv0) * P4 + lane; i < rows_need * P4; i += kWave) *(v4f *)(in + 4 * i) = id4;
    float *in_real = in + (row_lo - hv0) * P;
    if (P == W && !tiled) {
        // the real rows are one contiguous range: all its 128-bit loads are issued before the first
        // LDS write (lanes past the end re-read element 0 and drop it)
        const T *src = xp + (int64_t)row_lo * W;
        const int n4 = (row_hi - row_lo) * P4;
        constexpr int NL = kSepLds / 16 / kWave;
        v4f g4[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int i = lane + kWave * j;
            g4[j] = IO::load4(src + (i < n4 ? 4 * i : 0));
        }
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int i = lane + kWave * j;
            if (i < n4) *(v4f *)(in_real + 4 * i) = g4[j];
        }
    } else {
        const int n = (row_hi - row_lo) * P;
        const float inv_p = 1.0f / (float)P;
        constexpr int U = 8;                         // eight loads per lane in flight
        for (int i0 = 0; i0 < n; i0 += kWave * U) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                const int r = (int)(((float)i + 0.5f) * inv_p), c = c_first + i - r * P;
                const bool ok = i < n && c >= 0 && c < W;
                v[u] = IO::load1(xp + (ok ? (int64_t)(row_lo + r) * W + c : 0));
                v[u] = ok ? v[u] : O::id();
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                if (i < n) in_real[i] = v[u];
            }
        }
    }
    // identity margins of col: pwl columns in front, PC - pwl - P behind
    const int mr = PC - pwl - P;
    for (int i = lane; i < nr * (pwl + mr); i += kWave) {
        const int r = i / (pwl + mr), c = i - r * (pwl + mr);
        col[r * PC + (c < pwl ? c : P + c)] = O::id();
    }
    wave_lds_sync();
    // ---- down H: col[r][pwl + c] = (+)_{a < kh} in[r*sh + a][c], four columns per item
    for (int item = lane; item < nr * P4; item += kWave) {
        const int r = (int)(((float)item + 0.5f) * inv_p4), g = item - r * P4;
        const float *p = in + r * sh * P + 4 * g;
        v4f acc = *(const v4f *)p;
        int a = 1;
#define SWS_ACC4(v) acc.x = O::f(acc.x, v.x); acc.y = O::f(acc.y, v.y); acc.z = O::f(acc.z, v.z); acc.w = O::f(acc.w, v.w)
        for (; a + 4 <= kh; a += 4) {                // four reads in flight per wait
            const v4f v0 = *(const v4f *)(p + a * P), v1 = *(const v4f *)(p + (a + 1) * P);
            const v4f v2 = *(const v4f *)(p + (a + 2) * P), v3 = *(const v4f *)(p + (a + 3) * P);
            SWS_ACC4(v0); SWS_ACC4(v1); SWS_ACC4(v2); SWS_ACC4(v3);
        }
        for (; a < kh; ++a) {
            const v4f v = *(const v4f *)(p + a * P);
            SWS_ACC4(v);
        }
#undef SWS_ACC4
        *(v4f *)(col + r * PC + pwl + 4 * g) = acc;
    }
    wave_lds_sync();
    // ---- along W: one output per lane, consecutive lanes on consecutive outputs (their LDS reads
    //      fall on consecutive banks, their stores on one contiguous run of y)
    const float inv_wo = 1.0f / (float)nwo;
    for (int item = lane; item < nr * nwo; item += kWave) {
        const int r = (int)(((float)item + 0.5f) * inv_wo), wq = item - r * nwo, wo = wo0 + wq;
        const float *cr = col + r * PC + (tiled ? wq * sw : pwl - pw + wo * sw);
        float acc = cr[0];
        int b = 1;
        for (; b + 4 <= kw; b += 4) {                // four reads in flight per wait
            const float v0 = cr[b], v1 = cr[b + 1], v2 = cr[b + 2], v3 = cr[b + 3];
            acc = O::f(O::f(O::f(O::f(acc, v0), v1), v2), v3);
        }
        for (; b < kw; ++b) acc = O::f(acc, cr[b]);
        const int ho = ho0 + r;
        if (OP == SWS_OP_ADD) {
            float sc = scale;
            if (div_valid) {                         // real cells of this window
                const int h0 = ho * sh - ph, c0 = wo * sw - pw;
                const int rows_in = (h0 + kh < H ? h0 + kh : H) - (h0 > 0 ? h0 : 0);
                const int cols_in = (c0 + kw < W ? c0 + kw : W) - (c0 > 0 ? c0 : 0);
                sc = scale / (float)(rows_in * cols_in);
            }
            acc *= sc;
        }
        IO::store1_nt(yp + (int64_t)ho * Wo + wo, acc);
    }
}

template <int OP, typename T>
hipError_t launch_sep(const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int kh, int kw, int sh,
                      int sw, int ph, int pw, float scale, int div_valid, hipStream_t s, bool *taken)
{
    const int budget = kSepLds / 4;
    int P = (W + 3) / 4 * 4;
    int pwl = (pw + 3) / 4 * 4;                      // identity columns in front of a reduced row (kept 16-byte aligned)
    int right = (Wo - 1) * sw - pw + kw - P;         // columns a window reaches beyond the staged pitch
    if (right < 0) right = 0;
    int PC = pwl + P + (right + 3) / 4 * 4;
    // output rows per band: as many as the slice holds — (TH-1)*sh + kh staged rows of P floats plus
    // TH reduced rows of PC floats
    int TH = (budget - (kh - sh) * P) / (sh * P + PC);
    if (TH > Ho) TH = Ho;
    int ctiles = 1, TWO = Wo;
    if (TH < 1) {
        // the rows do not fit: column tiles.  A few output rows per band, the widest staged pitch the
        // slice then allows, and as many outputs per tile as that pitch covers.
        for (TH = Ho < 4 ? Ho : 4; TH >= 1; --TH) {
            P = budget / ((TH - 1) * sh + kh + TH) / 4 * 4;
            if (P >= kw + 15 * sw) break;            // at least 16 outputs per tile
        }
        if (TH >= 1) {
            TWO = (P - kw) / sw + 1;
            ctiles = (Wo + TWO - 1) / TWO;
            pwl = 0;
            PC = P;
        }
    }
    *taken = TH >= 1 && (int64_t)Ho * Wo < (1LL << 40) && (int64_t)TH * (ctiles > 1 ? TWO : Wo) < (1 << 20);
    if (!*taken) return hipSuccess;
    const int in_rows = (TH - 1) * sh + kh;
    const int lds_floats = in_rows * P + TH * PC;
    const int bands = (Ho + TH - 1) / TH;
    const int64_t n_units = planes * bands * ctiles;
    const int64_t grid = (n_units + kWaves - 1) / kWaves;
    if (grid > 2147483647LL) { *taken = false; return hipSuccess; }
    hipLaunchKernelGGL((pool2d_sep_kernel<OP, T>), dim3((unsigned)grid), dim3(kThreads), (size_t)lds_floats * 4 * kWaves, s,
                       x, y, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, P, PC, pwl, TH, bands, scale, n_units, lds_floats,
                       in_rows, div_valid, ctiles, TWO);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Row-streaming kernel for the small windows of pooling layers on planes whose rows fit a wavefront
// (W a multiple of 4, W <= 256), without LDS.  A lane owns four adjacent columns; the W/4 lanes of a
// group load one input row as one contiguous run of 128-bit accesses, and the G = 64 / (W/4) groups of
// a wavefront take G consecutive bands of TH output rows.  A lane keeps the (TH-1)*S + K rows of its
// band in registers, forms the sliding sum down H on them, and gets the few columns its windows need
// from the neighbouring lanes by DPP lane shifts (the Slide of Section 3 between registers) for the
// sliding sum along W.  A wavefront is short-lived (a few loads, a few stores) and is a workgroup of
// its own: the shape in which this GPU's memory system streams fastest.  Workgroup b runs on XCD
// b mod 8; XCD x takes the planes 8q + x band by band, so the rows two bands share are in the L2 that
// fetched them and the eight L2s sweep eight adjacent planes.
// Stride 1 needs Wo = W (window centred: 2 PW = K - 1), stride 2 needs Wo = W / 2.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float lane_before(float v)       // the value held by lane - 1 (0 for lane 0)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_after(float v)        // the value held by lane + 1 (0 for lane 63)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130, 0xf, 0xf, false));
}

template <int OP, int K, int S, int PW, int TH, typename T>
__global__ __launch_bounds__(kWave) void pool2d_rows_kernel(const T *__restrict__ x, T *__restrict__ y, int H, int W,
                                                            int Ho, int Wo, int ph, int LPR, int G, int lpr_rcp,
                                                            int64_t planes, float scale, int div_valid)
{
    using O = Op<OP>;
    using IO = Io<T>;
    constexpr int NL = PW;                                           // columns wanted from the lane before
    constexpr int NRT = (S == 1) ? K - 1 - PW : (K - 2 - PW > 0 ? K - 2 - PW : 0);   // ... from the lane after
    constexpr int NOUT = (S == 1) ? 4 : 2;                           // outputs per lane and row
    constexpr int NR = (TH - 1) * S + K;                             // input rows of a band
    static_assert(NL <= 4 && NRT <= 4, "windows reach the immediate neighbour lanes only");
    const int lane = threadIdx.x;
    const int grp = (lane * lpr_rcp) >> 16, l = lane - grp * LPR;    // lane / LPR (exact for lane < 64)
    if (grp >= G) return;
    // grid: x = 8 * (wavefront of the plane) + XCD, y = round of eight planes.  Workgroups are dealt to
    // the XCDs by their linear index, and gridDim.x is a multiple of 8.
    const int sl = (int)(blockIdx.x >> 3);
    const int64_t plane = (int64_t)blockIdx.y * kXcd + (blockIdx.x & 7);
    if (plane >= planes) return;
    const int ho0 = (sl * G + grp) * TH;                             // first output row of my band
    if (ho0 >= Ho) return;
    const T *xp = x + plane * (int64_t)H * W + 4 * l;
    T *yp = y + plane * (int64_t)Ho * Wo + NOUT * l;
    const v4f id4 = {O::id(), O::id(), O::id(), O::id()};
    v4f r[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) {                                   // all loads in flight together
        const int row = ho0 * S - ph + j;
        const bool ok = row >= 0 && row < H;
        const v4f v = IO::load4(xp + (int64_t)(ok ? row : 0) * W);
        r[j] = ok ? v : id4;                                         // rows outside the plane hold the identity
    }
    const bool first = l == 0, last = l == LPR - 1;
    // the sums down the columns of all TH output rows at once where they share rows (stride 1)
    v4f vs[TH];
    if constexpr (S == 1) {
        windows_shared<K, TH>(r, vs, [](v4f a, v4f b) {
            return (v4f){O::f(a.x, b.x), O::f(a.y, b.y), O::f(a.z, b.z), O::f(a.w, b.w)};
        });
    }
#pragma unroll
    for (int i = 0; i < TH; ++i) {
        // sliding sum down H on the lane's four columns ...
        float e[NL + 4 + NRT];
        v4f v = r[i * S];
        if constexpr (S == 1) {
            v = vs[i];
        } else {
#pragma unroll
            for (int a = 1; a < K; ++a) {
                v.x = O::f(v.x, r[i * S + a].x); v.y = O::f(v.y, r[i * S + a].y);
                v.z = O::f(v.z, r[i * S + a].z); v.w = O::f(v.w, r[i * S + a].w);
            }
        }
        e[NL] = v.x; e[NL + 1] = v.y; e[NL + 2] = v.z; e[NL + 3] = v.w;
        // ... the columns beside them from the neighbouring lanes (identity beyond the plane's edges) ...
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            const float nb = lane_before(e[NL + 3 - t]);
            e[NL - 1 - t] = first ? O::id() : nb;
        }
#pragma unroll
        for (int t = 0; t < NRT; ++t) {
            const float nb = lane_after(e[NL + t]);
            e[NL + 4 + t] = last ? O::id() : nb;
        }
        // ... then along W, operands in column order
        float o[NOUT];
        if constexpr (S == 1) {
            windows_shared<K, NOUT>(e, o, [](float a, float b) { return O::f(a, b); });
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) o[cc] = (OP == SWS_OP_ADD) ? o[cc] * scale : o[cc];
        } else {
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) {
                float acc = e[cc * S];
#pragma unroll
                for (int b = 1; b < K; ++b) acc = O::f(acc, e[cc * S + b]);
                o[cc] = (OP == SWS_OP_ADD) ? acc * scale : acc;
            }
        }
        const int ho = ho0 + i;
        if (OP == SWS_OP_ADD && div_valid) {                         // the average over the cells inside the plane
            const int h0 = ho * S - ph;
            const int rows_in = (h0 + K < H ? h0 + K : H) - (h0 > 0 ? h0 : 0);
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) {
                const int c0 = (NOUT * l + cc) * S - PW;
                const int cols_in = (c0 + K < W ? c0 + K : W) - (c0 > 0 ? c0 : 0);
                o[cc] = o[cc] / (float)(rows_in * cols_in);
            }
        }
        if (ho < Ho) {
            if constexpr (NOUT == 4) IO::store4(yp + (int64_t)ho * Wo, (v4f){o[0], o[1], o[2], o[3]}, false);
            else IO::store2_nt(yp + (int64_t)ho * Wo, (v2f){o[0], o[1]});
        }
    }
}

template <int OP, int K, int S, int PW, int TH, typename T>
hipError_t launch_rows(const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int ph, float scale,
                       int div_valid, hipStream_t s, bool *taken)
{
    const int LPR = W / 4, G = kWave / LPR;
    const int bands = (Ho + TH - 1) / TH;
    const int spp = (bands + G - 1) / G;                             // wavefronts per plane
    const int64_t rounds = (planes + kXcd - 1) / kXcd;
    *taken = rounds <= 65535;
    if (!*taken) return hipSuccess;
    hipLaunchKernelGGL((pool2d_rows_kernel<OP, K, S, PW, TH, T>), dim3((unsigned)(spp * kXcd), (unsigned)rounds), dim3(kWave),
                       0, s, x, y, H, W, Ho, Wo, ph, LPR, G, (65536 + LPR - 1) / LPR, planes, scale, div_valid);
    return hipGetLastError();
}

// The same kernel for planes wider than a wavefront's 256 columns: a wavefront takes a strip of 256 input columns
// of its band, of which the two lanes at either end only serve their neighbours — strips overlap by 16 columns,
// a strip yields 240 columns of outputs (stride 2: 120) and its stores are whole 64-byte lines (32-bit elements).
// Columns outside the plane hold the identity, like rows outside it.  The strips of a band are neighbours in
// launch order and run on one XCD, so the overlap is read from the L2 that fetched it.
constexpr int kStripCols = 240, kStripHalo = 8;

// RAG: rows whose length is not a multiple of 4.  The lane whose four columns straddle the end of the row
// loads the row's last four elements instead and moves the ones that are its own to the front (once per output row,
// after the sums down the columns); its outputs leave one by one.  Rows then start off the 16-byte boundaries.
template <int OP, int K, int S, int PW, int TH, typename T, bool RAG = false>
__global__ __launch_bounds__(kWave) void pool2d_rows_wide_kernel(const T *__restrict__ x, T *__restrict__ y, int H, int W,
                                                                 int Ho, int Wo, int ph, int nstrips, int64_t planes,
                                                                 float scale, int div_valid)
{
    using O = Op<OP>;
    using IO = Io<T>;
    constexpr int NL = PW;
    constexpr int NRT = (S == 1) ? K - 1 - PW : (K - 2 - PW > 0 ? K - 2 - PW : 0);
    constexpr int NOUT = (S == 1) ? 4 : 2;
    constexpr int NR = (TH - 1) * S + K;
    static_assert(NL <= kStripHalo && NRT <= kStripHalo, "windows reach no further than the lanes a strip gives away");
    const int lane = threadIdx.x;
    const int sl = (int)(blockIdx.x >> 3);                          // (band, strip) of the plane
    const int64_t plane = (int64_t)blockIdx.y * kXcd + (blockIdx.x & 7);
    if (plane >= planes) return;
    const int band = sl / nstrips, strip = sl - band * nstrips;
    const int ho0 = band * TH;
    if (ho0 >= Ho) return;
    const int c = strip * kStripCols - kStripHalo + 4 * lane;       // my four columns (a multiple of 4: wholly in or out)
    const bool in_cols = c >= 0 && c < W;
    const int nv = RAG ? W - c : 4;                                  // my columns inside the row: 1 .. 3 for the straddling lane
    const bool part = RAG && in_cols && nv < 4;
    const T *xp = x + plane * (int64_t)H * W + (in_cols ? (part ? W - 4 : c) : 0);
    const v4f id4 = {O::id(), O::id(), O::id(), O::id()};
    v4f r[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) {                                   // all loads in flight together
        const int row = ho0 * S - ph + j;
        const bool ok = row >= 0 && row < H;
        const v4f v = IO::load4(xp + (int64_t)(ok ? row : 0) * W);
        r[j] = (ok && in_cols) ? v : id4;
    }
    const bool mine = lane >= kStripHalo / 4 && lane < kWave - kStripHalo / 4 && in_cols;
    T *yp = y + plane * (int64_t)Ho * Wo + (S == 1 ? c : c / 2);
    // the sums down the columns of all TH output rows at once where they share rows (stride 1)
    v4f vs[TH];
    if constexpr (S == 1) {
        windows_shared<K, TH>(r, vs, [](v4f a, v4f b) {
            return (v4f){O::f(a.x, b.x), O::f(a.y, b.y), O::f(a.z, b.z), O::f(a.w, b.w)};
        });
    }
#pragma unroll
    for (int i = 0; i < TH; ++i) {
        float e[NL + 4 + NRT];
        v4f v = r[i * S];
        if constexpr (S == 1) {
            v = vs[i];
        } else {
#pragma unroll
            for (int a = 1; a < K; ++a) {
                v.x = O::f(v.x, r[i * S + a].x); v.y = O::f(v.y, r[i * S + a].y);
                v.z = O::f(v.z, r[i * S + a].z); v.w = O::f(v.w, r[i * S + a].w);
            }
        }
        if constexpr (RAG) {                                         // the straddling lane: its nv elements to the front
            const float idv = O::id();
            const v4f m1 = {v.y, v.z, v.w, idv}, m2 = {v.z, v.w, idv, idv}, m3 = {v.w, idv, idv, idv};
            v = !part ? v : (nv == 3 ? m1 : (nv == 2 ? m2 : m3));
        }
        e[NL] = v.x; e[NL + 1] = v.y; e[NL + 2] = v.z; e[NL + 3] = v.w;
        // (the lanes that store have both neighbours inside the wavefront, holding real columns or the identity)
        // column -(t + 1) of my four is element 3 - t % 4 of the lane t / 4 + 1 before me: one or two lane shifts
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            const float one = lane_before(e[NL + 3 - (t & 3)]);
            e[NL - 1 - t] = t < 4 ? one : lane_before(one);
        }
#pragma unroll
        for (int t = 0; t < NRT; ++t) {
            const float one = lane_after(e[NL + (t & 3)]);
            e[NL + 4 + t] = t < 4 ? one : lane_after(one);
        }
        float o[NOUT];
        if constexpr (S == 1) {
            windows_shared<K, NOUT>(e, o, [](float a, float b) { return O::f(a, b); });
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) o[cc] = (OP == SWS_OP_ADD) ? o[cc] * scale : o[cc];
        } else {
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) {
                float acc = e[cc * S];
#pragma unroll
                for (int b = 1; b < K; ++b) acc = O::f(acc, e[cc * S + b]);
                o[cc] = (OP == SWS_OP_ADD) ? acc * scale : acc;
            }
        }
        const int ho = ho0 + i;
        if (OP == SWS_OP_ADD && div_valid) {                         // the average over the cells inside the plane
            const int h0 = ho * S - ph;
            const int rows_in = (h0 + K < H ? h0 + K : H) - (h0 > 0 ? h0 : 0);
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) {
                const int c0 = (S == 1 ? c + cc : c + 2 * cc) - PW;
                const int cols_in = (c0 + K < W ? c0 + K : W) - (c0 > 0 ? c0 : 0);
                o[cc] = o[cc] / (float)(rows_in * (cols_in > 0 ? cols_in : 1));
            }
        }
        if (mine && ho < Ho) {
            // the outputs of mine that exist: all of them except at the end of a row (a straddling lane; at stride 2 a
            // last window that would pass the end of the plane)
            const int n_ok = Wo - (S == 1 ? c : c / 2);
            if (n_ok < NOUT) {
#pragma unroll
                for (int cc = 0; cc < NOUT; ++cc)
                    if (cc < n_ok) IO::store1_nt(yp + (int64_t)ho * Wo + cc, o[cc]);
            } else if constexpr (NOUT == 4) IO::store4(yp + (int64_t)ho * Wo, (v4f){o[0], o[1], o[2], o[3]}, false);
            else IO::store2_nt(yp + (int64_t)ho * Wo, (v2f){o[0], o[1]});
        }
    }
}

template <int OP, int K, int S, int PW, int TH, typename T>
hipError_t launch_rows_wide(const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int ph, float scale,
                            int div_valid, hipStream_t s, bool *taken)
{
    {
        if (W & 3) {                                                 // ragged rows
            const int nstrips = (W + kStripCols - 1) / kStripCols;
            const int bands = (Ho + TH - 1) / TH;
            const int64_t spp = (int64_t)bands * nstrips;
            const int64_t rounds = (planes + kXcd - 1) / kXcd;
            *taken = rounds <= 65535 && spp * kXcd <= 2147483647LL;
            if (!*taken) return hipSuccess;
            hipLaunchKernelGGL((pool2d_rows_wide_kernel<OP, K, S, PW, TH, T, true>), dim3((unsigned)(spp * kXcd), (unsigned)rounds),
                               dim3(kWave), 0, s, x, y, H, W, Ho, Wo, ph, nstrips, planes, scale, div_valid);
            return hipGetLastError();
        }
    }
    const int nstrips = (W + kStripCols - 1) / kStripCols;
    const int bands = (Ho + TH - 1) / TH;
    const int64_t spp = (int64_t)bands * nstrips;                    // wavefronts per plane
    const int64_t rounds = (planes + kXcd - 1) / kXcd;
    *taken = rounds <= 65535 && spp * kXcd <= 2147483647LL;
    if (!*taken) return hipSuccess;
    hipLaunchKernelGGL((pool2d_rows_wide_kernel<OP, K, S, PW, TH, T>), dim3((unsigned)(spp * kXcd), (unsigned)rounds), dim3(kWave),
                       0, s, x, y, H, W, Ho, Wo, ph, nstrips, planes, scale, div_valid);
    return hipGetLastError();
}

// The geometries the row-streaming kernel is built for: 3 x 3 with one column of padding at stride 1
// and 2, 2 x 2 stride 2 without padding; rows of 4 .. 256 elements in multiples of 4; every output
// divided by the same number.  Band heights as measured on [2048, 112, 112] under rotating buffers:
// two output rows per lane at stride 1 (35.0 us against 36.5 with one and 35.2 with four), one at stride 2
// (21.8 us against 23.9 with two).
template <int OP, typename T>
hipError_t dispatch_rows(const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int kh, int kw, int sh,
                         int sw, int ph, int pw, float scale, int div_valid, hipStream_t s, bool *taken)
{
    *taken = false;
    if (kh != kw || sh != sw || W < 4 || ph < 0 || ph >= kh || (g_opt.pool2d_variant & 128)) return hipSuccess;
    if (W & 3) {
        // rows that are not a multiple of 4 long: the strip form, from 64 columns on (narrower planes: too many lanes on
        // partial groups).  Stride 2 with and without padding (3 x 3 without: the classic "valid" pooling).  Cold,
        // strips / band kernel: [2048,111,111] 3 x 3 stride 2 29.8 / 50.0 us, [1024,149,149] 21.7 / 48.1 us; on rows that
        // are a multiple of 4 long the band kernel's own 3 x 3 stride-2 instances are level or ahead (28.8 / 24.1 us).
        if (W < 64) return hipSuccess;
        if (sh == 2) {
            if (Wo != (W + 2 * pw - kh) / 2 + 1) return hipSuccess;
            if (kh == 3 && pw <= 1) {
                if (pw == 1) return launch_rows_wide<OP, 3, 2, 1, 1, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
                return launch_rows_wide<OP, 3, 2, 0, 1, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
            }
            if (kh == 2 && pw == 0) return launch_rows_wide<OP, 2, 2, 0, 1, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
            return hipSuccess;
        }
        if (sh != 1 || Wo != W) return hipSuccess;
        if (kh == 3 && pw == 1) return launch_rows_wide<OP, 3, 1, 1, 2, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 5 && pw == 2) return launch_rows_wide<OP, 5, 1, 2, 2, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 7 && pw == 3) return launch_rows_wide<OP, 7, 1, 3, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 9 && pw == 4) return launch_rows_wide<OP, 9, 1, 4, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 11 && pw == 5) return launch_rows_wide<OP, 11, 1, 5, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 13 && pw == 6) return launch_rows_wide<OP, 13, 1, 6, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        return hipSuccess;
    }
    if (W > 256) {                                   // strips of 256 columns
        if (kh == 3 && sh == 1 && pw == 1 && Wo == W)
            return launch_rows_wide<OP, 3, 1, 1, 2, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        // (measured on [128, 512, 512], cold, strips / band kernel: 3 x 3 stride 1 50 / 95 us, 2 x 2 stride 2 27.8 / 29.2 us,
        // 3 x 3 stride 2 29.5 / 28.8 us — the last stays on the band kernel)
        if (kh == 2 && sh == 2 && pw == 0 && Wo == W / 2)
            return launch_rows_wide<OP, 2, 2, 0, 1, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 5 && sh == 1 && pw == 2 && Wo == W)
            return launch_rows_wide<OP, 5, 1, 2, 2, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 7 && sh == 1 && pw == 3 && Wo == W)
            return launch_rows_wide<OP, 7, 1, 3, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 9 && sh == 1 && pw == 4 && Wo == W)
            return launch_rows_wide<OP, 9, 1, 4, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 11 && sh == 1 && pw == 5 && Wo == W)
            return launch_rows_wide<OP, 11, 1, 5, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        if (kh == 13 && sh == 1 && pw == 6 && Wo == W)
            return launch_rows_wide<OP, 13, 1, 6, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
        return hipSuccess;
    }
    if (kh == 3 && sh == 1 && pw == 1 && Wo == W)
        return launch_rows<OP, 3, 1, 1, 2, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    if (kh == 3 && sh == 2 && pw == 1 && Wo == W / 2)
        return launch_rows<OP, 3, 2, 1, 1, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    if (kh == 2 && sh == 2 && pw == 0 && Wo == W / 2)
        return launch_rows<OP, 2, 2, 0, 1, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    // 5 x 5 and 7 x 7 at stride 1: a band of two output rows loads six or eight rows, which pays on wide rows only.
    // Measured cold, this kernel / the band kernel: [2048,112,112] 5 x 5 38.0 / 54.8 us, 7 x 7 43.7 / 69.0 us;
    // [8192,56,56] 5 x 5 39.9 / 40.6 us; [32768,28,28] 5 x 5 57.9 / 40.4 us.
    const bool wide_enough = W >= 64;
    if (kh == 5 && sh == 1 && pw == 2 && Wo == W && wide_enough)
        return launch_rows<OP, 5, 1, 2, 2, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    if (kh == 7 && sh == 1 && pw == 3 && Wo == W && wide_enough)
        return launch_rows<OP, 7, 1, 3, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    if (kh == 9 && sh == 1 && pw == 4 && Wo == W && wide_enough)
        return launch_rows<OP, 9, 1, 4, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    // windows that reach two lanes away: the strip form (one strip), whose outside lanes stand in for the edges
    if (kh == 11 && sh == 1 && pw == 5 && Wo == W && wide_enough)
        return launch_rows_wide<OP, 11, 1, 5, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    if (kh == 13 && sh == 1 && pw == 6 && Wo == W && wide_enough)
        return launch_rows_wide<OP, 13, 1, 6, 4, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken);
    return hipSuccess;
}

template <int OP, typename T>
hipError_t dispatch_band(const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int kh, int kw,
                         int sh, int sw, int ph, int pw, float scale, int div_valid, hipStream_t s, bool *taken)
{
#define SWS_BAND(KH, KW, SH, SW, PW)                                                                  \
    if (kh == KH && kw == KW && sh == SH && sw == SW && pw == PW)                                      \
        return launch_band<OP, KH, KW, SH, SW, PW, T>(x, y, planes, H, W, Ho, Wo, ph, scale, div_valid, s, taken)
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

// The tuned kernels for one element type: a specialised band kernel if the geometry has one, else
// the run-time separable kernel.  *taken = false: neither covers the shape, nothing was launched.
template <typename T>
hipError_t pool2d_tuned(int op, const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int kh, int kw, int sh,
                        int sw, int ph, int pw, float scale, int div_valid, hipStream_t s, bool *taken)
{
    hipError_t e;
    switch (op) {
    case SWS_OP_ADD: e = dispatch_rows<SWS_OP_ADD, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken); break;
    case SWS_OP_MAX: e = dispatch_rows<SWS_OP_MAX, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken); break;
    default: e = dispatch_rows<SWS_OP_MIN, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken); break;
    }
    if (*taken) return e;
    switch (op) {
    case SWS_OP_ADD: e = dispatch_band<SWS_OP_ADD, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken); break;
    case SWS_OP_MAX: e = dispatch_band<SWS_OP_MAX, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken); break;
    default: e = dispatch_band<SWS_OP_MIN, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken); break;
    }
    if (*taken) return e;
    switch (op) {
    case SWS_OP_ADD: return launch_sep<SWS_OP_ADD, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken);
    case SWS_OP_MAX: return launch_sep<SWS_OP_MAX, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken);
    default: return launch_sep<SWS_OP_MIN, T>(x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s, taken);
    }
}

// Direct evaluation on 16-bit elements (planes too wide for the LDS slices): one thread per output.
template <int OP, typename T>
__global__ __launch_bounds__(kThreads) void pool2d16_naive_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                                  int64_t planes, int H, int W, int Ho, int Wo, int kh,
                                                                  int kw, int sh, int sw, int ph, int pw, float scale)
{
    using O = Op<OP>;
    const int64_t total = planes * (int64_t)Ho * Wo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int wo = (int)(o % Wo);
        const int ho = (int)((o / Wo) % Ho);
        const T *xp = x + (o / ((int64_t)Wo * Ho)) * (int64_t)H * W;
        float acc = O::id();
        for (int b = 0; b < kw; ++b) {
            const int c = wo * sw - pw + b;
            if (c < 0 || c >= W) continue;
            float colv = O::id();
            for (int a = 0; a < kh; ++a) {
                const int h = ho * sh - ph + a;
                if (h >= 0 && h < H) colv = O::f(colv, (float)xp[(int64_t)h * W + c]);
            }
            acc = O::f(acc, colv);
        }
        if (OP == SWS_OP_ADD) acc *= scale;
        y[o] = (T)acc;
    }
}

template <typename T>
hipError_t pool2d_16(int op, const T *x, T *y, int64_t planes, int H, int W, int Ho, int Wo, int kh, int kw, int sh,
                     int sw, int ph, int pw, float scale, hipStream_t s)
{
    if (g_opt.pool2d_variant != 1) {
        bool taken = false;
        const hipError_t e = pool2d_tuned<T>(op, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, 0, s, &taken);
        if (taken) return e;
    }
    int64_t grid = (planes * (int64_t)Ho * Wo + kThreads - 1) / kThreads;
    if (grid > 1048576) grid = 1048576;
#define SWS_P16(OPV)                                                                                            \
    hipLaunchKernelGGL((pool2d16_naive_kernel<OPV, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, planes, H, W, \
                       Ho, Wo, kh, kw, sh, sw, ph, pw, scale)
    switch (op) {
    case SWS_OP_ADD: SWS_P16(SWS_OP_ADD); break;
    case SWS_OP_MAX: SWS_P16(SWS_OP_MAX); break;
    default: SWS_P16(SWS_OP_MIN); break;
    }
#undef SWS_P16
    return hipGetLastError();
}

}  // namespace

constexpr int kSmallPlane = 256;                     // plane elements up to which the small-plane kernel is taken

hipError_t launch_pool2d(int op, const float *x, float *y, int64_t planes, int64_t H, int64_t W, int64_t Ho,
                         int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                         float scale, int div_valid, hipStream_t s)
{
    // ph / pw are the top / left padding; the bottom / right padding is implied by Ho / Wo (cells
    // beyond the plane hold the identity whichever side they are on).
    // option pool2d_variant 32 forces the small-plane kernel wherever it applies, 64 switches it off
    // Its time goes with outputs x window cells, the band kernel's with planes.  Measured, max, us, small /
    // band: 65536 planes of 7 x 7: 3 x 3 20 / 36, 7 x 7 -> 1 x 1 10 / 43, 2 x 2 s2 10 / 22; 10 x 10: 3 x 3
    // 30 / 38; 32768 planes of 14 x 14: 3 x 3 s1 31 / 26, 3 x 3 s2 10 / 18, 2 x 2 s2 10 / 18; 16 x 16:
    // 3 x 3 s1 35 / 19, 2 x 2 s2 10 / 12; 20 x 20: slower throughout.
    const int64_t P = H * W, work = Ho * Wo * (int64_t)kh * kw;
    const bool small = g_opt.pool2d_variant == 32 ||
                       (g_opt.pool2d_variant != 64 && (P <= 100 || (P <= kSmallPlane && work <= 4 * P)));
    if (g_opt.pool2d_variant != 1 && small) {
        bool taken = false;
        const hipError_t e = launch_pool2d_small(op, x, y, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw,
                                                 scale, div_valid, s, &taken);
        if (taken) return e;
    }
    if (g_opt.pool2d_variant != 1) {
        bool taken = false;
        const hipError_t e = pool2d_tuned<float>(op, x, y, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw,
                                                 scale, div_valid, s, &taken);
        if (taken) return e;
    }
    return launch_pool2d_naive(op, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, div_valid, s);
}

// 16-bit storage (dtype SWS_DTYPE_BF16 / SWS_DTYPE_F16), fp32 arithmetic, one rounding per output.
hipError_t launch_pool2d_16(int op, int dtype, const void *x, void *y, int64_t planes, int64_t H, int64_t W, int64_t Ho,
                            int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                            float scale, hipStream_t s)
{
    if (dtype == SWS_DTYPE_BF16)
        return pool2d_16<__bf16>(op, (const __bf16 *)x, (__bf16 *)y, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh,
                                 sw, ph, pw, scale, s);
    return pool2d_16<_Float16>(op, (const _Float16 *)x, (_Float16 *)y, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw,
                               sh, sw, ph, pw, scale, s);
}

}  // namespace sws
