// sws_slide1d on short rows — sliding window sums (Section 2.2, Eq. 3) for windows up to 33 when a
// row is much shorter than the 1024-element wave tile of the scan kernel.
//
// A lane owns four consecutive outputs and reads the w + 3 inputs under them as 128-bit loads; a
// wavefront takes several whole rows side by side (lane -> (row, strip) by a 16-bit reciprocal), or
// 256 outputs of one row, so that no lane idles on rows of a few dozen elements.  Up to w = 4 each
// output combines its inputs left to right (Eq. 3 as written); from w = 5 the four windows share
// the strip's inputs 3 .. w-1: that core is combined once, and output c adds the suffix c .. 2 in
// front of it and the prefix w .. w+c-1 behind it (running sums: the register-level form of Section
// 3's prefix / suffix split), about w + 6 operations for the four outputs instead of 4 (w - 1).
// A 128-bit load may run past the end of its row (those values reach no valid output) but not past
// the ends of x: there it is replaced by element loads.  Rows extended by a boundary rule
// (sws_slide1d_padded) take the same path with the border strips read through the rule.
#include "sws_internal.h"

namespace sws {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef v4f v4f_u __attribute__((aligned(4)));

constexpr int kRowsMaxW = 33;                        // nine 128-bit loads per strip of four outputs

// PAD: rows extended by a boundary rule (pad_left virtual elements in front; lo counts the outputs
// of the extended row).  Loads that lie inside the physical row stay 128-bit; the others go element
// by element through the rule.  (Two variants measured slower for w >= 16: one test per strip with
// all-vector loads for strips clear of the borders, and border strips gathered unconditionally.)
template <int OP, int W, bool PAD>
__global__ __launch_bounds__(kWave) void slide_rows_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                           int64_t rows, int len, int lo, float scale, int strips,
                                                           int wg_per_row, int rows_per_wg, int recip, int pad_left,
                                                           int pad_mode)
{
    using O = Op<OP>;
    constexpr int NL = (W + 3 + 3) / 4;              // 128-bit loads per strip
    const int lane = threadIdx.x;
    int64_t r;
    int sidx;
    if (rows_per_wg == 1) {
        const int br = blockIdx.x / (unsigned)wg_per_row;
        r = br;
        sidx = (blockIdx.x - br * wg_per_row) * kWave + lane;
    } else {
        const int lr = (lane * recip) >> 16;         // lane / strips, exact for lane < 64
        if (lr >= rows_per_wg) return;
        r = (int64_t)blockIdx.x * rows_per_wg + lr;
        sidx = lane - lr * strips;
    }
    if (r >= rows || sidx >= strips) return;
    const int q = 4 * sidx;                          // first of this lane's four outputs
    float v[4 * NL];
    if constexpr (PAD) {
        const float *xrow = x + r * (int64_t)len;
        const int lv = lo + W - 1;                   // length of the extended row
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            const int p0 = q + 4 * k - pad_left;     // physical position of the load's first element
            if (p0 >= 0 && p0 + 4 <= len) {
                const v4f a = *(const v4f_u *)(xrow + p0);
                v[4 * k] = a.x; v[4 * k + 1] = a.y; v[4 * k + 2] = a.z; v[4 * k + 3] = a.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int e = q + 4 * k + c;
                    const int p = e < lv ? pad_src(e, len, pad_left, pad_mode) : -1;
                    v[4 * k + c] = p >= 0 ? xrow[p] : O::id();
                }
            }
        }
    } else {
        const int64_t g = r * (int64_t)len + q;      // the strip's first input in x
        const int64_t total = rows * (int64_t)len;
        const float *xr = x + g;
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            if (g + 4 * k + 4 <= total) {
                const v4f a = *(const v4f_u *)(xr + 4 * k);
                v[4 * k] = a.x; v[4 * k + 1] = a.y; v[4 * k + 2] = a.z; v[4 * k + 3] = a.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) v[4 * k + c] = (g + 4 * k + c < total) ? xr[4 * k + c] : 0.0f;
            }
        }
    }
    float o[4];
    if constexpr (W <= 4) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float acc = v[c];
#pragma unroll
            for (int j = 1; j < W; ++j) acc = O::f(acc, v[c + j]);
            o[c] = acc;
        }
    } else {
        float core = v[3];
#pragma unroll
        for (int j = 4; j < W; ++j) core = O::f(core, v[j]);
        const float suf2 = v[2], suf1 = O::f(v[1], suf2), suf0 = O::f(v[0], suf1);
        const float pre1 = v[W], pre2 = O::f(pre1, v[W + 1]), pre3 = O::f(pre2, v[W + 2]);
        o[0] = O::f(suf0, core);
        o[1] = O::f(O::f(suf1, core), pre1);
        o[2] = O::f(O::f(suf2, core), pre2);
        o[3] = O::f(core, pre3);
    }
    if (OP == SWS_OP_ADD) {
        if (PAD && pad_mode == SWS_PAD_SHRINK) {
            // the window shrinks at the ends of the row: rescale by w / (real elements in it)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int e = q + c;                 // first element of the window, in the extended row
                const int hi = e + W < pad_left + len ? e + W : pad_left + len;
                const int n = hi - (e > pad_left ? e : pad_left);
                o[c] *= scale * (float)W / (float)(n > 0 ? n : 1);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] *= scale;
        }
    }
    float *yr = y + r * (int64_t)lo + q;
    if (q + 4 <= lo) {
        const v4f a = {o[0], o[1], o[2], o[3]};
        __builtin_nontemporal_store(a, (v4f_u *)yr);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (q + c < lo) yr[c] = o[c];
    }
}

template <int OP, int W>
hipError_t launch_rows_w(const float *x, float *y, int64_t rows, int len, int lo, float scale, bool padded,
                         int pad_left, int pad_mode, hipStream_t s)
{
    const int strips = (lo + 3) / 4;
    const int wg_per_row = (strips + kWave - 1) / kWave;
    const int rows_per_wg = strips < kWave ? kWave / strips : 1;
    const int recip = 65536 / strips + 1;
    const int64_t grid = rows_per_wg == 1 ? rows * wg_per_row : (rows + rows_per_wg - 1) / rows_per_wg;
    if (grid > 2147483647LL) return kNotTaken;
    if (padded)
        hipLaunchKernelGGL((slide_rows_kernel<OP, W, true>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, rows, len,
                           lo, scale, strips, wg_per_row, rows_per_wg, recip, pad_left, pad_mode);
    else
        hipLaunchKernelGGL((slide_rows_kernel<OP, W, false>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, rows, len,
                           lo, scale, strips, wg_per_row, rows_per_wg, recip, 0, 0);
    return hipGetLastError();
}

template <int OP, int W0>
hipError_t launch_rows(const float *x, float *y, int64_t rows, int len, int lo, int w, float scale, bool padded,
                       int pad_left, int pad_mode, hipStream_t s)
{
    if constexpr (W0 > kRowsMaxW) {
        return kNotTaken;
    } else {
        if (w == W0) return launch_rows_w<OP, W0>(x, y, rows, len, lo, scale, padded, pad_left, pad_mode, s);
        return launch_rows<OP, W0 + 1>(x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, s);
    }
}

}  // namespace

int slide1d_rows_max_w() { return kRowsMaxW; }

// len: the physical row; lo: outputs per row (of the extended row when padded).
// kNotTaken: w beyond the kernel's reach or a grid beyond the launch limit (the caller
// then takes another kernel).
hipError_t launch_slide1d_rows(int op, const float *x, float *y, int64_t rows, int len, int lo, int32_t w, float scale,
                               bool padded, int pad_left, int pad_mode, hipStream_t s)
{
    if (w < 1 || w > kRowsMaxW) return kNotTaken;
    switch (op) {
    case SWS_OP_ADD: return launch_rows<SWS_OP_ADD, 1>(x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, s);
    case SWS_OP_MAX: return launch_rows<SWS_OP_MAX, 1>(x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, s);
    default: return launch_rows<SWS_OP_MIN, 1>(x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, s);
    }
}

}  // namespace sws
