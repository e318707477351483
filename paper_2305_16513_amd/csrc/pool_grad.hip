// sws_maxpool2d_grad — the adjoint of 2-D max pooling (Section 2.3's max operator, training side):
// every window sends its output gradient to the cell holding its maximum, the first such cell in
// row-major order when several tie.
//
// Gather form, no atomics, every gx element written exactly once and summed in a fixed order.  A
// workgroup owns a band of input rows of one plane.  It stages in LDS the input rows every
// window touching the band can see (with -inf rows and columns where the plane ends, so that window
// scans need no bounds tests) and the gy rows of those windows; then
//   1. one lane per window scans its kh x kw cells in row-major order with a strict ">" and leaves
//      the LDS position of the maximum in an index row;
//   2. one lane per input cell looks at the ceil(kh/sh) x ceil(kw/sw) windows that can cover it and
//      adds the gradients of those whose index is its own position.
// The index and gradient rows carry a border of windows that do not exist (index 0xFFFF, which is
// no cell's position), so that step 2 reads a fixed rectangle of windows per cell with no range
// tests: the kernel is bound by vector-instruction issue, not by memory.
// (Routing with LDS atomic adds instead of step 2 measured 2.5 x slower: an LDS atomic instruction
// costs about 150 cycles.)  Windows that straddle two bands are scanned by both.  HBM sees one read
// of x, one of gy and one write of gx (halo rows are re-read through L2).
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kSlice = 28 * 1024;                    // bytes of LDS per workgroup (one band); 16 .. 40 KB measured alike
constexpr int kRegsX = 20, kRegsG = 16, kRegGroup = 4;   // staging registers per thread: a band's x rows <= kRegsX * kThreads floats, its window rows <= kRegsG * kThreads

__host__ __device__ inline int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }
__host__ __device__ inline int ceil_div(int a, int b) { return -floor_div(-a, b); }

struct PgGeom {
    int H, W, Ho, Wo, kh, kw, sh, sw, ph, pw;
    int TH, bands;                                   // input rows per band, bands per plane
    int PX, pwl;                                     // pitch of a staged x row, -inf columns in front of it
    int CA, CB;                                      // ceil(kh / sh), ceil(kw / sw): window rows / columns that can cover one cell
    int PO, colpad;                                  // pitch of a window row in LDS; window column wo sits at colpad + wo
    int x_rows, w_rows;                              // most x rows / window rows (with border) a band needs
    int cwx, kmx, cwg, kmg;                          // staging: log2 of the column chunk and chunks per row, for x rows and for gy rows
    int slice;                                       // floats of LDS
};

// KH > 0: window extents and strides at compile time (scans unrolled, divisions by constants);
// KH = 0: everything taken from g.
//
// A workgroup takes `upb` consecutive bands.  While it works on one band out of LDS, the loads of
// the next band are already in flight into registers.
template <int KH, int KW, int SH, int SW>
__global__ __launch_bounds__(kThreads) void maxpool2d_grad_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                  float *__restrict__ gx, PgGeom g, int64_t n_units, int upb)
{
    const int kh = KH > 0 ? KH : g.kh, kw = KH > 0 ? KW : g.kw, sh = KH > 0 ? SH : g.sh, sw = KH > 0 ? SW : g.sw;
    const int CA = KH > 0 ? (KH + SH - 1) / (SH > 0 ? SH : 1) : g.CA, CB = KH > 0 ? (KW + SW - 1) / (SW > 0 ? SW : 1) : g.CB;
    extern __shared__ __attribute__((aligned(16))) float lds_all[];
    const int lane = threadIdx.x;                    // the whole workgroup works on one band
    const int n_x = g.x_rows * g.PX, n_g = g.w_rows * g.PO;
    float *X = lds_all;                              // [x_rows][PX]
    float *G = X + n_x;                              // [w_rows][PO]  gy of the windows around the band, 0 where there is no window
    unsigned short *IDX = (unsigned short *)(G + n_g);   // [w_rows][PO]  where each window's maximum sits in X, 0xFFFF where there is no window
    const float ninf = -__builtin_huge_valf();
    const float inv_po = 1.0f / (float)g.PO, inv_w = 1.0f / (float)g.W;

    struct Band {
        int64_t plane;
        int h0, h1;                                  // the band's rows
        int wr0, nrw;                                // first window row of the LDS rectangle (may be < 0) and its rows
        int ho_lo, nwr;                              // the window rows among them that exist (nwr may be <= 0)
        int xr_lo, nxr;                              // first (possibly virtual) x row those windows see, and how many
    };
    auto band_of = [&](int64_t unit) {
        Band b;
        b.plane = unit / g.bands;
        const int band = (int)(unit - b.plane * g.bands);
        b.h0 = band * g.TH;
        b.h1 = b.h0 + g.TH < g.H ? b.h0 + g.TH : g.H;
        b.wr0 = (b.h0 + g.ph) / sh - (CA - 1);       // the rows step 2 reads for the band's first row start here
        const int wr1 = (b.h1 - 1 + g.ph) / sh;      // and those for its last row end here
        b.nrw = wr1 - b.wr0 + 1;
        b.ho_lo = b.wr0 > 0 ? b.wr0 : 0;
        const int ho_hi = wr1 < g.Ho - 1 ? wr1 : g.Ho - 1;
        b.nwr = ho_hi - b.ho_lo + 1;
        b.xr_lo = b.ho_lo * sh - g.ph;
        b.nxr = b.nwr > 0 ? (b.nwr - 1) * sh + kh : 0;
        return b;
    };

    // Staging.  The threads form a grid of (kThreads >> cwx) rows by (1 << cwx) columns over the x
    // rows (cwx: the power of two that covers a row, at most 64 columns wide; wider rows take several
    // column chunks), and likewise with cwg over the gy rows, so that rows and columns come from
    // shifts and adds.  Register sx[q] holds row ry + (q / kmx) * rows_per_pass, column
    // lc + ((q % kmx) << cwx): x rows xr_lo .. xr_lo + nxr - 1 at columns -pwl .. PX - pwl - 1 with -inf
    // outside the plane.  sg[q] the same for the gy rows wr0 .. at columns -colpad .. (what lies outside
    // gy is never used: the index there is 0xFFFF).  request() only issues the loads; the values are
    // first touched in commit().
    float sx[kRegsX], sg[kRegsG];
    unsigned ok_x = 0, ok_g = 0;
    auto request = [&](const Band &b) {
        const char *xp = (const char *)(x + b.plane * (int64_t)g.H * g.W);
        const char *gp = (const char *)(gy + b.plane * (int64_t)g.Ho * g.Wo);
        ok_x = ok_g = 0;
        int me = lane, zero = 0;
        asm volatile("" : "+v"(me), "+s"(zero));     // row / column arithmetic is redone per band instead of being kept in registers across bands
        {
            const int ry = me >> g.cwx, lc = me & ((1 << g.cwx) - 1), rpp = kThreads >> g.cwx;
            int k = zero, m = zero;
#pragma unroll
            for (int u0 = 0; u0 < kRegsX; u0 += kRegGroup) {
                if (k * rpp >= g.x_rows) break;
#pragma unroll
                for (int u = u0; u < u0 + kRegGroup; ++u) {
                    const int r = ry + k * rpp, c = lc + (m << g.cwx) - g.pwl;
                    const int row = b.xr_lo + r;
                    const bool ok = r < b.nxr && (unsigned)row < (unsigned)g.H && (unsigned)c < (unsigned)g.W;
                    sx[u] = *(const float *)(xp + (ok ? (unsigned)(__mul24(row, g.W) + c) * 4u : 0u));     // a plane has < 2^20 cells
                    ok_x |= ok ? 1u << u : 0u;
                    if (++m == g.kmx) { m = 0; ++k; }
                }
                __builtin_amdgcn_sched_barrier(0);   // keeps the address arithmetic of later groups from piling up in registers
            }
        }
        {
            const int ry = me >> g.cwg, lc = me & ((1 << g.cwg) - 1), rpp = kThreads >> g.cwg;
            int k = zero, m = zero;
#pragma unroll
            for (int u0 = 0; u0 < kRegsG; u0 += kRegGroup) {
                if (k * rpp >= g.w_rows) break;
#pragma unroll
                for (int u = u0; u < u0 + kRegGroup; ++u) {
                    const int r = ry + k * rpp, wo = lc + (m << g.cwg) - g.colpad;
                    const int ho = b.wr0 + r;
                    const bool ok = (unsigned)ho < (unsigned)g.Ho && (unsigned)wo < (unsigned)g.Wo;
                    sg[u] = *(const float *)(gp + (ok ? (unsigned)(__mul24(ho, g.Wo) + wo) * 4u : 0u));
                    ok_g |= ok ? 1u << u : 0u;
                    if (++m == g.kmg) { m = 0; ++k; }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    auto commit = [&]() {
        int me = lane, zero = 0;
        asm volatile("" : "+v"(me), "+s"(zero));
        {
            const int ry = me >> g.cwx, lc = me & ((1 << g.cwx) - 1), rpp = kThreads >> g.cwx;
            float *mine = X + __mul24(ry, g.PX) + lc;
            int k = zero, m = zero;
#pragma unroll
            for (int u0 = 0; u0 < kRegsX; u0 += kRegGroup) {
                if (k * rpp >= g.x_rows) break;
#pragma unroll
                for (int u = u0; u < u0 + kRegGroup; ++u) {
                    if (ry < g.x_rows - k * rpp && lc < g.PX - (m << g.cwx))
                        mine[k * rpp * g.PX + (m << g.cwx)] = (ok_x >> u & 1u) ? sx[u] : ninf;
                    if (++m == g.kmx) { m = 0; ++k; }
                }
            }
        }
        {
            const int ry = me >> g.cwg, lc = me & ((1 << g.cwg) - 1), rpp = kThreads >> g.cwg;
            float *mine = G + __mul24(ry, g.PO) + lc;
            int k = zero, m = zero;
#pragma unroll
            for (int u0 = 0; u0 < kRegsG; u0 += kRegGroup) {
                if (k * rpp >= g.w_rows) break;
#pragma unroll
                for (int u = u0; u < u0 + kRegGroup; ++u) {
                    if (ry < g.w_rows - k * rpp && lc < g.PO - (m << g.cwg))
                        mine[k * rpp * g.PO + (m << g.cwg)] = (ok_g >> u & 1u) ? sg[u] : 0.0f;
                    if (++m == g.kmg) { m = 0; ++k; }
                }
            }
        }
    };

    const int64_t unit0 = (int64_t)blockIdx.x * upb;
    const int64_t unit1 = unit0 + upb < n_units ? unit0 + upb : n_units;
    Band nb = band_of(unit0);
    request(nb);
    for (int64_t unit = unit0; unit < unit1; ++unit) {
        const Band b = nb;
        float *op = gx + b.plane * (int64_t)g.H * g.W;
        __syncthreads();                             // the previous band's step 2 has left LDS
        commit();
        __syncthreads();
        if (unit + 1 < unit1) {
            nb = band_of(unit + 1);
            request(nb);
        }
        // ---- 1. the position of every window's maximum (0xFFFF in the border)
        for (int i = lane; i < b.nrw * g.PO; i += kThreads) {
            const int r = (int)(((float)i + 0.5f) * inv_po), wo = i - __mul24(r, g.PO) - g.colpad;
            const int ho = b.wr0 + r;
            const bool valid = ho >= 0 && ho < g.Ho && wo >= 0 && wo < g.Wo;
            const int base = valid ? __mul24((ho - b.ho_lo) * sh, g.PX) + g.pwl - g.pw + wo * sw : 0;   // the window's first cell
            float best = ninf;
            int at = base;
            if (KH > 0) {
                float v[(KH > 0 ? KH : 1) * (KW > 0 ? KW : 1)];
#pragma unroll
                for (int a = 0; a < KH; ++a)
#pragma unroll
                    for (int c = 0; c < KW; ++c) v[a * KW + c] = X[base + a * g.PX + c];     // all reads before the first compare
#pragma unroll
                for (int a = 0; a < KH; ++a)
#pragma unroll
                    for (int c = 0; c < KW; ++c) {
                        const bool gt = v[a * KW + c] > best;
                        best = gt ? v[a * KW + c] : best;
                        at = gt ? base + a * g.PX + c : at;
                    }
            } else {
                for (int a = 0; a < kh; ++a) {
                    const int ra = base + a * g.PX;
                    for (int c = 0; c < kw; ++c) {
                        const float v = X[ra + c];
                        const bool gt = v > best;
                        best = gt ? v : best;
                        at = gt ? ra + c : at;
                    }
                }
            }
            IDX[i] = (unsigned short)(valid ? at : 0xFFFF);
        }
        __syncthreads();
        // ---- 2. every cell of the band collects the windows that chose it, oldest window first: the
        //      CA x CB rectangle of windows ending at row (h + ph) / sh, column (c + pw) / sw
        const int nrows = b.h1 - b.h0;
        for (int i = lane; i < nrows * g.W; i += kThreads) {
            const int r = (int)(((float)i + 0.5f) * inv_w), c = i - __mul24(r, g.W);
            const int h = b.h0 + r;
            const int me = __mul24(h - b.xr_lo, g.PX) + g.pwl + c;
            const int top = __mul24((h + g.ph) / sh - b.wr0 - CA + 1, g.PO) + (c + g.pw) / sw;   // column + colpad - (CB - 1)
            float acc = 0.0f;
            if (KH > 0) {
                constexpr int NA = KH > 0 ? (KH + SH - 1) / SH : 1, NB = KH > 0 ? (KW + SW - 1) / SW : 1;
                int idx[NA * NB];
                float gv[NA * NB];
#pragma unroll
                for (int da = 0; da < NA; ++da)
#pragma unroll
                    for (int db = 0; db < NB; ++db) {
                        idx[da * NB + db] = (int)IDX[top + da * g.PO + db];
                        gv[da * NB + db] = G[top + da * g.PO + db];
                    }
#pragma unroll
                for (int q = 0; q < NA * NB; ++q) acc += idx[q] == me ? gv[q] : 0.0f;
            } else {
                for (int da = 0; da < CA; ++da)
                    for (int db = 0; db < CB; ++db) {
                        const int t = top + da * g.PO + db;
                        acc += (int)IDX[t] == me ? G[t] : 0.0f;
                    }
            }
            __builtin_nontemporal_store(acc, op + (__mul24(h, g.W) + c));   // a plane has < 2^20 cells
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

// ---------------------------------------------------------------------------------------------
// The adjoint of average pooling: gx[h, c] = sum over the windows that hold (h, c) of f * gy, with
// f = scale, or scale / (cells of that window inside the plane).  The same band scheme without the
// maxima: a workgroup stages the rows of f * gy its band's cells can ask for (zero where there is
// no window) and every cell adds a fixed CA x CB rectangle of them, oldest window first.  Only the
// rectangle's first row and first column can hold windows that end before the cell (when the
// stride does not divide the window); they are masked.
// ---------------------------------------------------------------------------------------------
template <int KH, int KW, int SH, int SW>
__global__ __launch_bounds__(kThreads) void avgpool2d_grad_kernel(const float *__restrict__ gy, float *__restrict__ gx, PgGeom g,
                                                                  int64_t n_units, float scale, int div_real)
{
    const int kh = KH > 0 ? KH : g.kh, kw = KH > 0 ? KW : g.kw, sh = KH > 0 ? SH : g.sh, sw = KH > 0 ? SW : g.sw;
    const int CA = KH > 0 ? (KH + SH - 1) / (SH > 0 ? SH : 1) : g.CA, CB = KH > 0 ? (KW + SW - 1) / (SW > 0 ? SW : 1) : g.CB;
    extern __shared__ __attribute__((aligned(16))) float G[];     // [w_rows][PO]
    const int64_t unit = blockIdx.x;
    if (unit >= n_units) return;
    const int64_t plane = unit / g.bands;
    const int band = (int)(unit - plane * g.bands);
    const int h0 = band * g.TH, h1 = h0 + g.TH < g.H ? h0 + g.TH : g.H;
    const int wr0 = (h0 + g.ph) / sh - (CA - 1);     // the rows the band's first row reads start here
    const int nrw = (h1 - 1 + g.ph) / sh - wr0 + 1;  // and those of its last row end here
    const float *gp = gy + plane * (int64_t)g.Ho * g.Wo;
    float *op = gx + plane * (int64_t)g.H * g.W;
    const float inv_po = 1.0f / (float)g.PO, inv_w = 1.0f / (float)g.W;
    {
        constexpr int U = 4;
        for (int j0 = threadIdx.x; j0 < nrw * g.PO; j0 += kThreads * U) {
            float v[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u * kThreads;
                const int r = (int)(((float)j + 0.5f) * inv_po), wo = j - __mul24(r, g.PO) - g.colpad;
                const int ho = wr0 + r;
                ok[u] = j < nrw * g.PO && (unsigned)ho < (unsigned)g.Ho && (unsigned)wo < (unsigned)g.Wo;
                v[u] = gp[ok[u] ? __mul24(ho, g.Wo) + wo : 0];
                if (div_real) {                      // cells of window (ho, wo) inside the plane
                    const int r0 = ho * sh - g.ph, c0 = wo * sw - g.pw;
                    const int nr = (r0 + kh < g.H ? r0 + kh : g.H) - (r0 > 0 ? r0 : 0);
                    const int nc = (c0 + kw < g.W ? c0 + kw : g.W) - (c0 > 0 ? c0 : 0);
                    v[u] = ok[u] ? v[u] * (scale / (float)(nr * nc)) : 0.0f;
                } else {
                    v[u] = ok[u] ? v[u] * scale : 0.0f;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u * kThreads;
                if (j < nrw * g.PO) G[j] = v[u];
            }
        }
    }
    __syncthreads();
    const int nrows = h1 - h0;
    for (int i = threadIdx.x; i < nrows * g.W; i += kThreads) {
        const int r = (int)(((float)i + 0.5f) * inv_w), c = i - __mul24(r, g.W);
        const int h = h0 + r;
        const int a_hi = (h + g.ph) / sh, b_hi = (c + g.pw) / sw;
        const int top = __mul24(a_hi - wr0 - CA + 1, g.PO) + b_hi;        // column + colpad - (CB - 1)
        // the oldest candidate row / column ends before the cell unless the cell's offset in it is below kh / kw
        constexpr bool kExact = KH > 0 && KH % (SH > 0 ? SH : 1) == 0 && KW % (SW > 0 ? SW : 1) == 0;   // every candidate covers the cell
        const bool row0 = kExact || (h + g.ph) - (a_hi - CA + 1) * sh < kh, col0 = kExact || (c + g.pw) - (b_hi - CB + 1) * sw < kw;
        float acc = 0.0f;
        if (KH > 0) {
            constexpr int NA = KH > 0 ? (KH + SH - 1) / SH : 1, NB = KH > 0 ? (KW + SW - 1) / SW : 1;
            float gv[NA * NB];
#pragma unroll
            for (int da = 0; da < NA; ++da)
#pragma unroll
                for (int db = 0; db < NB; ++db) gv[da * NB + db] = G[top + da * g.PO + db];
#pragma unroll
            for (int da = 0; da < NA; ++da)
#pragma unroll
                for (int db = 0; db < NB; ++db) acc += ((da > 0 || row0) && (db > 0 || col0)) ? gv[da * NB + db] : 0.0f;
        } else {
            for (int da = 0; da < CA; ++da)
                for (int db = 0; db < CB; ++db) acc += ((da > 0 || row0) && (db > 0 || col0)) ? G[top + da * g.PO + db] : 0.0f;
        }
        __builtin_nontemporal_store(acc, op + (__mul24(h, g.W) + c));      // a plane has < 2^20 cells
    }
}

// Direct evaluation for planes whose window rows do not fit LDS.
__global__ __launch_bounds__(kThreads) void avgpool2d_grad_naive_kernel(const float *__restrict__ gy, float *__restrict__ gx,
                                                                        int64_t planes, int H, int W, int Ho, int Wo, int kh,
                                                                        int kw, int sh, int sw, int ph, int pw, float scale,
                                                                        int div_real)
{
    const int64_t total = planes * (int64_t)H * W;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int c = (int)(o % W);
        const int h = (int)((o / W) % H);
        const int64_t p = o / ((int64_t)W * H);
        int a_lo = ceil_div(h + ph - kh + 1, sh), a_hi = floor_div(h + ph, sh);
        int b_lo = ceil_div(c + pw - kw + 1, sw), b_hi = floor_div(c + pw, sw);
        if (a_lo < 0) a_lo = 0;
        if (b_lo < 0) b_lo = 0;
        if (a_hi > Ho - 1) a_hi = Ho - 1;
        if (b_hi > Wo - 1) b_hi = Wo - 1;
        float acc = 0.0f;
        for (int ho = a_lo; ho <= a_hi; ++ho)
            for (int wo = b_lo; wo <= b_hi; ++wo) {
                float f = scale;
                if (div_real) {
                    const int r0 = ho * sh - ph, c0 = wo * sw - pw;
                    const int nr = (r0 + kh < H ? r0 + kh : H) - (r0 > 0 ? r0 : 0);
                    const int nc = (c0 + kw < W ? c0 + kw : W) - (c0 > 0 ? c0 : 0);
                    f = scale / (float)(nr * nc);
                }
                acc += gy[(p * Ho + ho) * (int64_t)Wo + wo] * f;
            }
        gx[o] = acc;
    }
}

}  // namespace

hipError_t launch_maxpool2d_grad(const float *x, const float *gy, float *gx, int64_t planes, int64_t H, int64_t W,
                                 int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph,
                                 int32_t pw, hipStream_t s)
{
    // 3 x 3 windows on rows that fit a wavefront: the row-streaming kernel (pool2d_variant bit 128 switches it off)
    if (g_opt.pool2d_variant != 1 && !(g_opt.pool2d_variant & 128)) {
        bool taken = false;
        const hipError_t e = launch_maxpool2d_grad_rows(x, gy, gx, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw,
                                                        ph, pw, s, &taken);
        if (taken) return e;
    }
    PgGeom g;
    g.H = (int)H; g.W = (int)W; g.Ho = (int)Ho; g.Wo = (int)Wo; g.kh = kh; g.kw = kw; g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.pwl = pw;
    int right = (int)((Wo - 1) * sw - pw + kw - W);   // columns a window reaches beyond the plane
    if (right < 0) right = 0;
    g.PX = (int)W + pw + right;
    g.CA = (kh + sh - 1) / sh;
    g.CB = (kw + sw - 1) / sw;
    g.colpad = g.CB - 1;
    const int last_col = (int)((W - 1 + pw) / sw);   // the last window column a cell can ask for
    g.PO = g.colpad + (last_col + 1 > (int)Wo ? last_col + 1 : (int)Wo);
    auto chunk = [](int pitch, int &cw, int &km) {   // the power of two that covers a row, at most 64 columns
        cw = 0;
        while ((1 << cw) < pitch && cw < 6) ++cw;
        km = (pitch + (1 << cw) - 1) >> cw;
    };
    chunk(g.PX, g.cwx, g.kmx);
    chunk(g.PO, g.cwg, g.kmg);
    // rows per band: the most that fit LDS and the staging registers.  The cells of a band of th rows
    // ask for at most ceil((th - 1) / sh) + CA window rows, which see (that - 1) * sh + kh input rows.
    auto plan = [&](int th) {
        g.w_rows = (th - 1 + sh - 1) / sh + g.CA;
        g.x_rows = (g.w_rows - 1) * sh + kh;
        const int n_x = g.x_rows * g.PX, n_g = g.w_rows * g.PO;
        g.slice = (n_x + n_g + (n_g + 1) / 2 + 3) / 4 * 4;              // x rows, gy rows, 16-bit index rows
        const int regs_x = (g.x_rows + (kThreads >> g.cwx) - 1) / (kThreads >> g.cwx) * g.kmx;
        const int regs_g = (g.w_rows + (kThreads >> g.cwg) - 1) / (kThreads >> g.cwg) * g.kmg;
        return (size_t)g.slice * 4 <= (size_t)kSlice && regs_x <= kRegsX && regs_g <= kRegsG && n_x < 65535;
    };
    int TH = H < 64 ? (int)H : 64;
    while (TH >= 1 && !plan(TH)) --TH;
    if (TH >= 1) {                                   // bands of equal height
        const int nb = (int)((H + TH - 1) / TH);
        TH = (int)((H + nb - 1) / nb);
        plan(TH);
    }
    const bool fits = TH >= 1 && g_opt.pool2d_variant != 1 && H * W < (1 << 20) && Ho * Wo < (1 << 20);
    if (fits) {
        g.TH = TH;
        g.bands = (int)((H + TH - 1) / TH);
        const int64_t n_units = planes * g.bands;
        const int upb = 1;                               // bands per workgroup: 1, 2 and 4 measured alike on 112 x 112 planes, 8 slower
        const int64_t grid = (n_units + upb - 1) / upb;
        if (grid <= 2147483647LL) {
#define SWS_PG(KH, KW, SH, SW)                                                                                   \
    hipLaunchKernelGGL((maxpool2d_grad_kernel<KH, KW, SH, SW>), dim3((unsigned)grid), dim3(kThreads),                \
                       (size_t)g.slice * 4, s, x, gy, gx, g, n_units, upb)
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

hipError_t launch_avgpool2d_grad(const float *gy, float *gx, int64_t planes, int64_t H, int64_t W, int64_t Ho, int64_t Wo,
                                 int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, int div_real,
                                 float scale, hipStream_t s)
{
    if (!div_real && g_opt.pool2d_variant != 1 && !(g_opt.pool2d_variant & 128)) {
        // At stride 1 with one divisor the adjoint IS the forward sliding sum, over gy padded by k - 1 - p
        // (a cell's windows are the k x k block of gy around it): the forward kernels take it.
        if (sh == 1 && sw == 1)
            return launch_pool2d(SWS_OP_ADD, gy, gx, planes, Ho, Wo, H, W, kh, kw, 1, 1, kh - 1 - ph, kw - 1 - pw, scale, 0, s);
        bool taken = false;
        const hipError_t e = launch_avgpool2d_grad_rows(gy, gx, planes, (int)H, (int)W, (int)Ho, (int)Wo, kh, kw, sh, sw, ph,
                                                        pw, scale, s, &taken);
        if (taken) return e;
    }
    PgGeom g;
    g.H = (int)H; g.W = (int)W; g.Ho = (int)Ho; g.Wo = (int)Wo; g.kh = kh; g.kw = kw; g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.pwl = pw; g.PX = 0; g.x_rows = 0; g.cwx = g.kmx = g.cwg = g.kmg = 0;
    g.CA = (kh + sh - 1) / sh;
    g.CB = (kw + sw - 1) / sw;
    g.colpad = g.CB - 1;
    const int last_col = (int)((W - 1 + pw) / sw);   // the last window column a cell can ask for
    g.PO = g.colpad + (last_col + 1 > (int)Wo ? last_col + 1 : (int)Wo);
    // rows per band: a band of th rows asks for at most ceil((th - 1) / sh) + CA window rows; 16 KB
    // of LDS per workgroup keeps several workgroups on a compute unit
    constexpr int kLds = 16 * 1024;
    auto plan = [&](int th) {
        g.w_rows = (th - 1 + sh - 1) / sh + g.CA;
        g.slice = g.w_rows * g.PO;
        return (size_t)g.slice * 4 <= (size_t)kLds;
    };
    int TH = H < 64 ? (int)H : 64;
    while (TH >= 1 && !plan(TH)) --TH;
    if (TH >= 1) {                                   // bands of equal height
        const int nb = (int)((H + TH - 1) / TH);
        TH = (int)((H + nb - 1) / nb);
        plan(TH);
    }
    if (TH >= 1 && g_opt.pool2d_variant != 1 && H * W < (1 << 20) && Ho * Wo < (1 << 20)) {
        g.TH = TH;
        g.bands = (int)((H + TH - 1) / TH);
        const int64_t n_units = planes * g.bands;
        if (n_units <= 2147483647LL) {
#define SWS_AG(KH, KW, SH, SW)                                                                                   \
    hipLaunchKernelGGL((avgpool2d_grad_kernel<KH, KW, SH, SW>), dim3((unsigned)n_units), dim3(kThreads),             \
                       (size_t)g.slice * 4, s, gy, gx, g, n_units, scale, div_real)
            if (kh == 3 && kw == 3 && sh == 1 && sw == 1) SWS_AG(3, 3, 1, 1);
            else if (kh == 3 && kw == 3 && sh == 2 && sw == 2) SWS_AG(3, 3, 2, 2);
            else if (kh == 2 && kw == 2 && sh == 2 && sw == 2) SWS_AG(2, 2, 2, 2);
            else SWS_AG(0, 0, 1, 1);
#undef SWS_AG
            return hipGetLastError();
        }
    }
    int64_t grid = (planes * H * W + kThreads - 1) / kThreads;
    if (grid > 1048576) grid = 1048576;
    hipLaunchKernelGGL(avgpool2d_grad_naive_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, gy, gx, planes, (int)H, (int)W,
                       (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw, scale, div_real);
    return hipGetLastError();
}

}  // namespace sws
