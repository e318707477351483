/*
 * sws_ref — CPU oracle for sliding window sums.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct definition that the GPU library is
 * checked against.  It is never part of the product path: only the tests, the
 * smoke check and the bench's cpu_baseline leg load it.  It shares no code,
 * header, table or helper with the HIP kernels.
 *
 * Everything is the plain definition written out as nested loops, accumulated
 * in fp64, on host pointers:
 *
 *   sws_ref_slide1d  Section 2.2, Eq. 3 (sliding window sum): every output is
 *                    the left-to-right combination of exactly w inputs, so a
 *                    row of length len has len-w+1 outputs ("valid").  Naive
 *                    O(w*N), the cost the paper quotes for the direct method.
 *   sws_ref_pool2d   Section 2.3 (pooling = sliding sum with + or max) taken to
 *                    two dimensions as a direct kh x kw window scan, NOT as two
 *                    separable passes, so that a separable GPU evaluation is
 *                    checked against an independent formulation.  Taps that
 *                    fall into the padding contribute the identity of the
 *                    operator (they are skipped).
 *   sws_ref_pool2d_ex  the same window scan with separate padding on the four sides and, for
 *                    ADD, the choice of dividing by the number of window cells that lie inside
 *                    the plane (average pooling that does not count the padding).
 *   sws_ref_maxpool2d_grad  the adjoint of max pooling at a point x (Section 2.3's max operator,
 *                    training side): every window sends its output gradient to the cell that
 *                    holds its maximum — the first such cell in row-major order when several tie.
 *   sws_ref_avgpool2d_grad  the adjoint of sws_ref_pool2d_ex for ADD with symmetric padding: every
 *                    window sends f * gy to each of its cells inside the plane, f = scale or
 *                    scale / (number of such cells) — the forward sum's terms, scattered.
 *   sws_ref_slide1d_padded  Eq. 3 on rows extended at both ends (the boundary conditions
 *                    named in Section 3: padding, mirroring, periodicity; plus edge
 *                    replication).  Every window element's index is mapped back into
 *                    the row by the rule of the mode, then combined as in Eq. 3.
 *   sws_ref_pool2d_padded  the same boundary conditions in two dimensions: Eq. 3 over kh x kw
 *                    windows of planes extended on their four sides, both indices of every
 *                    window cell mapped back into the plane by the rule of the mode.
 *   sws_ref_conv1d_padded  Eq. 4 per output over rows extended by the same boundary conditions:
 *                    every tap's input index mapped back into the row (or dropped: zero padding).
 *   sws_ref_conv2d_padded  the 2-D convolution over planes extended on four sides by those conditions,
 *                    the row and the column index of every tap's input cell mapped independently.
 *   sws_ref_slide1d_pair  Eq. 3 with the pair operator of Section 2.4, Eq. 8:
 *                    (u_i, v_i) (+) (u_j, v_j) = (u_i*u_j, u_j*v_i + v_j), i older.
 *                    Non-commutative; folded strictly left to right.
 *   sws_ref_conv1d_grad_input / _grad_weight  the two adjoints of sws_ref_conv1d (the training
 *                    side of Section 2.5's sliding dot product), written as SCATTER loops over
 *                    the forward sum's terms: every term wgt*x of output (b,co,i) sends
 *                    wgt*gy to gx at x's index and x*gy to gw at wgt's index.  The GPU
 *                    gathers instead (flipped taps, swapped channels; a reduction).
 *   sws_ref_conv2d_grad_input / _grad_weight  the same two adjoints for sws_ref_conv2d.
 *   sws_ref_round16  the value of the bf16 / fp16 number nearest to a double (ties to the even
 *                    significand, overflow to infinity): how a result computed on 16-bit
 *                    storage (the quantised inputs the paper's introduction mentions) is
 *                    written back.  The 16-bit sliding sum is round16(slide1d(widened x)).
 *   sws_ref_conv1d   Section 2.5 (convolution = sliding dot product, Eq. 4 per
 *   sws_ref_conv2d   output): cross-correlation (no tap flip), zero padding by
 *                    skipping out-of-range taps, accumulation order ci, kh, kw.
 *
 * The paper fixes no precision; fp64 accumulation of fp32 data leaves the
 * oracle's own rounding (~1e-16 * sum|terms|) far below the fp32 tolerance
 * the GPU results are held to.  max/min of fp32 values is exact in fp64.
 *
 * abs_sum (optional, may be NULL) receives sum|terms| per output, the scale
 * of the tolerance |err| <= 1e-5 * sum|terms|.
 *
 * Rows / planes / images are independent; the only parallelism is an OpenMP
 * "parallel for" over them.  Nothing here is tuned.
 *
 * Pins (tests/test_oracle_pins.py): hand-enumerated tiny cases, closed forms
 * for constant and ramp inputs, prefix-sum differences, window membership for
 * max, the paper's Vector Input algorithm emulated with a non-commutative
 * operator, the dot-product-as-prefix-sum construction of Eq. 7-9, and
 * cross-operator identities (all-ones taps, one-hot taps, rank-1 2-D taps,
 * separability of pooling, strided = subsampled); for the pair operator a
 * hand-folded case, u = 1 (sliding add of v), v = 0 (sliding product of u),
 * exact rational arithmetic on small integers, order sensitivity, and the
 * Eq. 7 sequence whose full-length window yields the dot product; for round16 the
 * library's own fp16 / bf16 casts, hand-written ties, subnormals and overflow; for the
 * adjoints the inner-product identities <conv(x;W), g> = <x, gx> = <W, gw> against the pinned
 * forward function, one-hot cases written out by hand, and central differences of the
 * (bilinear, hence exactly differentiated) loss <conv(x;W), g>.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_ADD = 0, REF_MAX = 1, REF_MIN = 2 };

int sws_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of OpenMP threads for the calls that follow (timing the oracle on one core); no-op
 * without OpenMP.  Has no effect on results. */
void sws_ref_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* a (+) b with a the older (left) operand. */
static double combine(int op, double a, double b)
{
    switch (op) {
    case REF_ADD: return a + b;
    case REF_MAX: return (a < b) ? b : a;
    default:      return (b < a) ? b : a;
    }
}

/* Eq. 3:  y[r,i] = scale * (x[r,i] (+) x[r,i+1] (+) ... (+) x[r,i+w-1]),  0 <= i <= len-w.
 * x: rows*len floats.  y, abs_sum: rows*(len-w+1) doubles.  scale applies to ADD only. */
int sws_ref_slide1d(int op, const float *x, double *y, double *abs_sum,
                    int64_t rows, int64_t len, int32_t w, double scale)
{
    if (op < 0 || op > 2 || rows < 0 || len < 0 || w < 1 || w > len) return 1;
    if (rows > 0 && (!x || !y)) return 1;
    const int64_t lo = len - w + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *xr = x + r * len;
        for (int64_t i = 0; i < lo; ++i) {
            double acc = (double)xr[i];
            double mag = fabs((double)xr[i]);
            for (int32_t j = 1; j < w; ++j) {
                acc = combine(op, acc, (double)xr[i + j]);
                mag += fabs((double)xr[i + j]);
            }
            if (op == REF_ADD) { acc *= scale; mag *= fabs(scale); }
            y[r * lo + i] = acc;
            if (abs_sum) abs_sum[r * lo + i] = mag;
        }
    }
    return 0;
}

/* NCHW pooling by direct window scan.  Ho = (H + 2*ph - kh)/sh + 1, Wo likewise.
 * Padding holds the identity of op, i.e. out-of-range taps are skipped.  ADD is
 * multiplied by scale (average pooling that counts the padding: scale = 1/(kh*kw)). */
int sws_ref_pool2d(int op, const float *x, double *y, double *abs_sum,
                   int64_t N, int64_t C, int64_t H, int64_t W,
                   int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                   int32_t ph, int32_t pw, double scale)
{
    if (op < 0 || op > 2 || N < 0 || C < 0 || H < 0 || W < 0) return 1;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return 1;
    if (ph >= kh || pw >= kw) return 1;            /* no window may lie wholly in padding */
    if (kh > H + 2 * (int64_t)ph || kw > W + 2 * (int64_t)pw) return 1;
    const int64_t Ho = (H + 2 * (int64_t)ph - kh) / sh + 1;
    const int64_t Wo = (W + 2 * (int64_t)pw - kw) / sw + 1;
    const int64_t planes = N * C;
    if (planes > 0 && (!x || !y)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        const float *xp = x + p * H * W;
        for (int64_t ho = 0; ho < Ho; ++ho) {
            for (int64_t wo = 0; wo < Wo; ++wo) {
                int first = 1;
                double acc = 0.0, mag = 0.0;
                for (int32_t a = 0; a < kh; ++a) {
                    const int64_t h = ho * sh - ph + a;
                    if (h < 0 || h >= H) continue;
                    for (int32_t b = 0; b < kw; ++b) {
                        const int64_t c = wo * sw - pw + b;
                        if (c < 0 || c >= W) continue;
                        const double v = (double)xp[h * W + c];
                        acc = first ? v : combine(op, acc, v);
                        mag += fabs(v);
                        first = 0;
                    }
                }
                if (op == REF_ADD) { acc *= scale; mag *= fabs(scale); }
                y[(p * Ho + ho) * Wo + wo] = acc;
                if (abs_sum) abs_sum[(p * Ho + ho) * Wo + wo] = mag;
            }
        }
    }
    return 0;
}

/* y[b,co,i] = sum_{ci in group(co)} sum_{t<k} wgt[co,ci,t] * x[b, g*Cin/groups + ci, i*stride + t*dilation - pad]
 * x [B,Cin,L], wgt [Cout,Cin/groups,k], y [B,Cout,Lo], Lo = (L + 2*pad - dilation*(k-1) - 1)/stride + 1. */
int sws_ref_conv1d(const float *x, const float *wgt, double *y, double *abs_sum,
                   int64_t B, int64_t Cin, int64_t L, int64_t Cout,
                   int32_t k, int32_t stride, int32_t pad, int32_t dilation, int32_t groups)
{
    if (B < 0 || Cin < 1 || L < 0 || Cout < 1 || k < 1 || stride < 1 || pad < 0 || dilation < 1 || groups < 1) return 1;
    if (Cin % groups || Cout % groups) return 1;
    const int64_t span = (int64_t)dilation * (k - 1) + 1;
    if (span > L + 2 * (int64_t)pad) return 1;
    const int64_t Lo = (L + 2 * (int64_t)pad - span) / stride + 1;
    const int64_t cig = Cin / groups, cog = Cout / groups;
    if (B > 0 && (!x || !wgt || !y)) return 1;
    const int64_t units = B * Cout;
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < units; ++u) {
        const int64_t b = u / Cout, co = u % Cout, g = co / cog;
        for (int64_t i = 0; i < Lo; ++i) {
            double acc = 0.0, mag = 0.0;
            for (int64_t ci = 0; ci < cig; ++ci) {
                const float *xr = x + (b * Cin + g * cig + ci) * L;
                const float *wr = wgt + (co * cig + ci) * k;
                for (int32_t t = 0; t < k; ++t) {
                    const int64_t j = i * stride + (int64_t)t * dilation - pad;
                    if (j < 0 || j >= L) continue;
                    const double term = (double)wr[t] * (double)xr[j];
                    acc += term;
                    mag += fabs(term);
                }
            }
            y[u * Lo + i] = acc;
            if (abs_sum) abs_sum[u * Lo + i] = mag;
        }
    }
    return 0;
}

/* NCHW x, OIHW wgt, zero padding, no bias, groups = 1:
 * y[n,co,ho,wo] = sum_ci sum_a sum_b wgt[co,ci,a,b] * x[n,ci,ho*sh - ph + a, wo*sw - pw + b]. */
int sws_ref_conv2d(const float *x, const float *wgt, double *y, double *abs_sum,
                   int64_t N, int64_t Cin, int64_t H, int64_t W, int64_t Cout,
                   int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw)
{
    if (N < 0 || Cin < 1 || H < 0 || W < 0 || Cout < 1) return 1;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return 1;
    if (kh > H + 2 * (int64_t)ph || kw > W + 2 * (int64_t)pw) return 1;
    const int64_t Ho = (H + 2 * (int64_t)ph - kh) / sh + 1;
    const int64_t Wo = (W + 2 * (int64_t)pw - kw) / sw + 1;
    if (N > 0 && (!x || !wgt || !y)) return 1;
    const int64_t units = N * Cout;
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < units; ++u) {
        const int64_t n = u / Cout, co = u % Cout;
        for (int64_t ho = 0; ho < Ho; ++ho) {
            for (int64_t wo = 0; wo < Wo; ++wo) {
                double acc = 0.0, mag = 0.0;
                for (int64_t ci = 0; ci < Cin; ++ci) {
                    const float *xp = x + (n * Cin + ci) * H * W;
                    const float *wp = wgt + (co * Cin + ci) * kh * kw;
                    for (int32_t a = 0; a < kh; ++a) {
                        const int64_t h = ho * sh - ph + a;
                        if (h < 0 || h >= H) continue;
                        for (int32_t b = 0; b < kw; ++b) {
                            const int64_t c = wo * sw - pw + b;
                            if (c < 0 || c >= W) continue;
                            const double term = (double)wp[a * kw + b] * (double)xp[h * W + c];
                            acc += term;
                            mag += fabs(term);
                        }
                    }
                }
                y[(u * Ho + ho) * Wo + wo] = acc;
                if (abs_sum) abs_sum[(u * Ho + ho) * Wo + wo] = mag;
            }
        }
    }
    return 0;
}

/* Sliding window sum (Eq. 3) of the pairs (u_i, v_i) under the operator of Eq. 8,
 *   (u_a, v_a) (+) (u_b, v_b) = (u_a*u_b, u_b*v_a + v_b),   a the older (left) operand,
 * i.e. the composition of the maps z -> u*z + v in index order.  u, v: rows*len floats;
 * yu, yv: rows*(len-w+1) doubles.  mag_u / mag_v (optional) receive the tolerance scales
 * |prod u| and sum_j |v_j| * prod_{m>j} |u_m| (the absolute values of the terms of yv). */
int sws_ref_slide1d_pair(const float *u, const float *v, double *yu, double *yv, double *mag_u, double *mag_v,
                         int64_t rows, int64_t len, int32_t w)
{
    if (rows < 0 || len < 0 || w < 1 || w > len) return 1;
    if (rows > 0 && (!u || !v || !yu || !yv)) return 1;
    const int64_t lo = len - w + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *ur = u + r * len, *vr = v + r * len;
        for (int64_t i = 0; i < lo; ++i) {
            double U = (double)ur[i], V = (double)vr[i], MV = fabs((double)vr[i]);
            for (int32_t t = 1; t < w; ++t) {
                const double uj = (double)ur[i + t], vj = (double)vr[i + t];
                V = uj * V + vj;                     /* uses the old U nowhere: order of the two lines is free */
                MV = fabs(uj) * MV + fabs(vj);
                U = U * uj;
            }
            yu[r * lo + i] = U;
            yv[r * lo + i] = V;
            if (mag_u) mag_u[r * lo + i] = fabs(U);
            if (mag_v) mag_v[r * lo + i] = MV;
        }
    }
    return 0;
}

/* Eq. 3 over rows extended by pad_left / pad_right virtual elements.  mode: 0 = the identity of
 * the operator (0 for ADD, -inf for MAX, +inf for MIN; such elements are skipped), 1 = mirror
 * about the end elements without repeating them (x[-i] = x[i]), 2 = periodic (x[-i] = x[len-i]),
 * 3 = the end element repeated, 4 = the window shrinks at the ends: the virtual elements are
 * skipped as in mode 0 and an ADD result is multiplied by w / n, n = the number of real elements
 * in the window (so that scale = 1/w gives the mean over real elements; pads must be < w).
 * y, abs_sum: rows*(len+pad_left+pad_right-w+1) doubles. */
int sws_ref_slide1d_padded(int op, const float *x, double *y, double *abs_sum, int64_t rows, int64_t len,
                           int32_t w, int32_t pad_left, int32_t pad_right, int mode, double scale)
{
    if (op < 0 || op > 2 || mode < 0 || mode > 4 || rows < 0 || len < 1 || w < 1 || pad_left < 0 || pad_right < 0)
        return 1;
    if (mode == 4 && (pad_left >= w || pad_right >= w)) return 1;     /* every window holds a real element */
    const int64_t lv = len + pad_left + pad_right, lo = lv - w + 1;
    if (lo < 1) return 1;
    if (mode == 1 && (pad_left > len - 1 || pad_right > len - 1)) return 1;
    if (mode == 2 && (pad_left > len || pad_right > len)) return 1;
    if (rows > 0 && (!x || !y)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *xr = x + r * len;
        for (int64_t i = 0; i < lo; ++i) {
            double acc = 0.0, mag = 0.0;
            int64_t have = 0;                            /* real or mapped elements combined so far */
            for (int32_t t = 0; t < w; ++t) {
                int64_t p = i + t - pad_left;            /* index into the physical row, may be outside */
                if (p < 0 || p >= len) {
                    if (mode == 0 || mode == 4) continue;   /* identity element: contributes nothing */
                    if (mode == 1) p = p < 0 ? -p : 2 * (len - 1) - p;
                    else if (mode == 2) p = p < 0 ? p + len : p - len;
                    else p = p < 0 ? 0 : len - 1;
                }
                const double v = (double)xr[p];
                acc = have ? combine(op, acc, v) : v;
                ++have;
                mag += fabs(v);
            }
            if (!have) acc = op == REF_ADD ? 0.0 : (op == REF_MAX ? -INFINITY : INFINITY);
            const double f = (mode == 4 && have) ? scale * (double)w / (double)have : scale;
            y[r * lo + i] = op == REF_ADD ? acc * f : acc;
            if (abs_sum) abs_sum[r * lo + i] = op == REF_ADD ? mag * fabs(f) : mag;
        }
    }
    return 0;
}

/* Index of the physical element that virtual index p (0 <= p < len is physical) of a line extended
 * by the rule `mode` stands for; -1: the operator's identity (mode 0). */
static int64_t map_index(int64_t p, int64_t len, int mode)
{
    if (p >= 0 && p < len) return p;
    if (mode == 1) return p < 0 ? -p : 2 * (len - 1) - p;            /* mirror, end elements not repeated */
    if (mode == 2) return p < 0 ? p + len : p - len;                 /* periodic */
    if (mode == 3) return p < 0 ? 0 : len - 1;                       /* edge */
    return -1;
}

/* 2-D pooling (Section 2.3) over planes extended on their four sides by a boundary condition of
 * Section 3 (mode 0 identity padding, 1 mirror, 2 periodic, 3 edge replication):
 *   y[p,ho,wo] = scale_if_add * (+)_{a<kh, b<kw} X[p, ho*sh - pad_top + a, wo*sw - pad_left + b],
 * X = x inside the plane, the mapped cell (or the identity) outside.  Row-major window order.
 * x: planes*H*W floats; y, abs_sum: planes*Ho*Wo doubles, Ho = (H+pad_top+pad_bottom-kh)/sh + 1. */
int sws_ref_pool2d_padded(int op, const float *x, double *y, double *abs_sum, int64_t planes, int64_t H, int64_t W,
                          int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t pad_top, int32_t pad_left,
                          int32_t pad_bottom, int32_t pad_right, int mode, double scale)
{
    if (op < 0 || op > 2 || mode < 0 || mode > 3 || planes < 0 || H < 1 || W < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1)
        return 1;
    if (pad_top < 0 || pad_left < 0 || pad_bottom < 0 || pad_right < 0) return 1;
    if (mode == 1 && (pad_top > H - 1 || pad_bottom > H - 1 || pad_left > W - 1 || pad_right > W - 1)) return 1;
    if (mode == 2 && (pad_top > H || pad_bottom > H || pad_left > W || pad_right > W)) return 1;
    const int64_t He = H + pad_top + pad_bottom, We = W + pad_left + pad_right;
    if (kh > He || kw > We) return 1;
    const int64_t Ho = (He - kh) / sh + 1, Wo = (We - kw) / sw + 1;
    if (planes > 0 && (!x || !y)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        const float *xp = x + p * H * W;
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo) {
                double acc = 0.0, mag = 0.0;
                int64_t have = 0;
                for (int32_t a = 0; a < kh; ++a)
                    for (int32_t b = 0; b < kw; ++b) {
                        const int64_t r = map_index(ho * sh - pad_top + a, H, mode);
                        const int64_t c = map_index(wo * sw - pad_left + b, W, mode);
                        if (r < 0 || c < 0) continue;                /* identity element */
                        const double v = (double)xp[r * W + c];
                        acc = have ? combine(op, acc, v) : v;
                        ++have;
                        mag += fabs(v);
                    }
                if (!have) acc = op == REF_ADD ? 0.0 : (op == REF_MAX ? -INFINITY : INFINITY);
                y[(p * Ho + ho) * Wo + wo] = op == REF_ADD ? acc * scale : acc;
                if (abs_sum) abs_sum[(p * Ho + ho) * Wo + wo] = op == REF_ADD ? mag * fabs(scale) : mag;
            }
    }
    return 0;
}

/* Nearest number with `frac_bits` fraction bits whose smallest normal exponent is min_exp:
 * spacing 2^(e - frac_bits) in the binade of v (the smallest normal's spacing below it),
 * rint() rounds ties to even in the default rounding mode, anything beyond the largest finite
 * value becomes infinity. */
static double round_to_format(double v, int frac_bits, int min_exp, double max_finite)
{
    if (v == 0.0 || !isfinite(v)) return v;
    int e;
    (void)frexp(fabs(v), &e);                 /* |v| = m * 2^e with m in [0.5, 1): leading bit 2^(e-1) */
    int lead = e - 1;
    if (lead < min_exp) lead = min_exp;
    const double ulp = ldexp(1.0, lead - frac_bits);
    const double r = rint(v / ulp) * ulp;     /* division and product by a power of two are exact */
    return fabs(r) > max_finite ? copysign(INFINITY, v) : r;
}

/* dtype 1 = bf16 (7 fraction bits, exponents of fp32), 2 = fp16 (10 fraction bits, smallest
 * normal 2^-14, largest finite 65504). */
int sws_ref_round16(const double *in, double *out, int64_t n, int dtype)
{
    if (n < 0 || (dtype != 1 && dtype != 2) || (n > 0 && (!in || !out))) return 1;
    for (int64_t i = 0; i < n; ++i)
        out[i] = dtype == 1 ? round_to_format(in[i], 7, -126, ldexp(2.0 - ldexp(1.0, -7), 127))
                            : round_to_format(in[i], 10, -14, 65504.0);
    return 0;
}

/* Adjoint of sws_ref_conv1d with respect to x: gx[b,ci,j] = sum of wgt[co,ci,t] * gy[b,co,i]
 * over every (co, i, t) whose forward term reads x[b,ci,j], i.e. j = i*stride + t*dilation - pad.
 * Scatter form; one image per thread so that no two threads write the same gx.
 * abs_sum (optional) receives sum|terms| per gx element. */
int sws_ref_conv1d_grad_input(const float *gy, const float *wgt, double *gx, double *abs_sum,
                              int64_t B, int64_t Cin, int64_t L, int64_t Cout,
                              int32_t k, int32_t stride, int32_t pad, int32_t dilation, int32_t groups)
{
    if (B < 0 || Cin < 1 || L < 0 || Cout < 1 || k < 1 || stride < 1 || pad < 0 || dilation < 1 || groups < 1) return 1;
    if (Cin % groups || Cout % groups) return 1;
    const int64_t span = (int64_t)dilation * (k - 1) + 1;
    if (span > L + 2 * (int64_t)pad) return 1;
    const int64_t Lo = (L + 2 * (int64_t)pad - span) / stride + 1;
    const int64_t cig = Cin / groups, cog = Cout / groups;
    if (B > 0 && (!gy || !wgt || !gx)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t e = 0; e < Cin * L; ++e) {
            gx[b * Cin * L + e] = 0.0;
            if (abs_sum) abs_sum[b * Cin * L + e] = 0.0;
        }
        for (int64_t co = 0; co < Cout; ++co) {
            const int64_t g = co / cog;
            for (int64_t i = 0; i < Lo; ++i) {
                const double gyv = (double)gy[(b * Cout + co) * Lo + i];
                for (int64_t ci = 0; ci < cig; ++ci)
                    for (int32_t t = 0; t < k; ++t) {
                        const int64_t j = i * stride + (int64_t)t * dilation - pad;
                        if (j < 0 || j >= L) continue;
                        const double term = (double)wgt[(co * cig + ci) * k + t] * gyv;
                        const int64_t at = (b * Cin + g * cig + ci) * L + j;
                        gx[at] += term;
                        if (abs_sum) abs_sum[at] += fabs(term);
                    }
            }
        }
    }
    return 0;
}

/* Adjoint with respect to wgt: gw[co,ci,t] = sum over (b, i) of x[b, g*cig+ci, i*stride + t*dilation - pad]
 * * gy[b,co,i] (terms in the padding are absent).  Scatter form; one output channel per thread. */
int sws_ref_conv1d_grad_weight(const float *x, const float *gy, double *gw, double *abs_sum,
                               int64_t B, int64_t Cin, int64_t L, int64_t Cout,
                               int32_t k, int32_t stride, int32_t pad, int32_t dilation, int32_t groups)
{
    if (B < 0 || Cin < 1 || L < 0 || Cout < 1 || k < 1 || stride < 1 || pad < 0 || dilation < 1 || groups < 1) return 1;
    if (Cin % groups || Cout % groups) return 1;
    const int64_t span = (int64_t)dilation * (k - 1) + 1;
    if (span > L + 2 * (int64_t)pad) return 1;
    const int64_t Lo = (L + 2 * (int64_t)pad - span) / stride + 1;
    const int64_t cig = Cin / groups, cog = Cout / groups;
    if (!gw || (B > 0 && (!x || !gy))) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t co = 0; co < Cout; ++co) {
        const int64_t g = co / cog;
        for (int64_t e = 0; e < cig * k; ++e) {
            gw[co * cig * k + e] = 0.0;
            if (abs_sum) abs_sum[co * cig * k + e] = 0.0;
        }
        for (int64_t b = 0; b < B; ++b)
            for (int64_t i = 0; i < Lo; ++i) {
                const double gyv = (double)gy[(b * Cout + co) * Lo + i];
                for (int64_t ci = 0; ci < cig; ++ci)
                    for (int32_t t = 0; t < k; ++t) {
                        const int64_t j = i * stride + (int64_t)t * dilation - pad;
                        if (j < 0 || j >= L) continue;
                        const double term = (double)x[(b * Cin + g * cig + ci) * L + j] * gyv;
                        gw[(co * cig + ci) * k + t] += term;
                        if (abs_sum) abs_sum[(co * cig + ci) * k + t] += fabs(term);
                    }
            }
    }
    return 0;
}

/* NCHW pooling with padding pt / pl / pb / pr on the top / left / bottom / right side:
 * Ho = (H + pt + pb - kh)/sh + 1, Wo = (W + pl + pr - kw)/sw + 1.  Padding holds the identity.
 * ADD: y = scale * sum when div_valid = 0; y = scale * sum / n when div_valid = 1, n = number of
 * cells of the window inside the plane (scale = 1: the mean over real cells). */
int sws_ref_pool2d_ex(int op, const float *x, double *y, double *abs_sum,
                      int64_t N, int64_t C, int64_t H, int64_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                      int32_t pt, int32_t pl, int32_t pb, int32_t pr, int div_valid, double scale)
{
    if (op < 0 || op > 2 || N < 0 || C < 0 || H < 1 || W < 1) return 1;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || pt < 0 || pl < 0 || pb < 0 || pr < 0) return 1;
    if (pt >= kh || pb >= kh || pl >= kw || pr >= kw) return 1;      /* every window holds a real cell */
    if (kh > H + pt + (int64_t)pb || kw > W + pl + (int64_t)pr) return 1;
    const int64_t Ho = (H + pt + (int64_t)pb - kh) / sh + 1;
    const int64_t Wo = (W + pl + (int64_t)pr - kw) / sw + 1;
    const int64_t planes = N * C;
    if (planes > 0 && (!x || !y)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        const float *xp = x + p * H * W;
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo) {
                int64_t n = 0;
                double acc = 0.0, mag = 0.0;
                for (int32_t a = 0; a < kh; ++a)
                    for (int32_t b = 0; b < kw; ++b) {
                        const int64_t h = ho * sh - pt + a, c = wo * sw - pl + b;
                        if (h < 0 || h >= H || c < 0 || c >= W) continue;
                        const double v = (double)xp[h * W + c];
                        acc = n ? combine(op, acc, v) : v;
                        mag += fabs(v);
                        ++n;
                    }
                if (op == REF_ADD) {
                    const double f = div_valid ? scale / (double)n : scale;
                    acc *= f;
                    mag *= fabs(f);
                }
                y[(p * Ho + ho) * Wo + wo] = acc;
                if (abs_sum) abs_sum[(p * Ho + ho) * Wo + wo] = mag;
            }
    }
    return 0;
}

/* Adjoints of sws_ref_conv2d in scatter form: every forward term wgt[co,ci,a,b] * x[n,ci,h,c] of
 * output (n,co,ho,wo), h = ho*sh - ph + a, c = wo*sw - pw + b, sends wgt * gy to gx[n,ci,h,c]
 * (which = 0) or x * gy to gw[co,ci,a,b] (which = 1).  `other` is wgt for which = 0 and x for
 * which = 1; out / abs_sum have the shape of x resp. wgt. */
static int conv2d_adjoint(int which, const float *other, const float *gy, double *out, double *abs_sum,
                          int64_t N, int64_t Cin, int64_t H, int64_t W, int64_t Cout,
                          int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw)
{
    if (N < 0 || Cin < 1 || H < 0 || W < 0 || Cout < 1) return 1;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return 1;
    if (kh > H + 2 * (int64_t)ph || kw > W + 2 * (int64_t)pw) return 1;
    const int64_t Ho = (H + 2 * (int64_t)ph - kh) / sh + 1;
    const int64_t Wo = (W + 2 * (int64_t)pw - kw) / sw + 1;
    if (!out || (N > 0 && (!other || !gy))) return 1;
    const int64_t n_out = which == 0 ? N * Cin * H * W : Cout * Cin * kh * kw;
    for (int64_t e = 0; e < n_out; ++e) {
        out[e] = 0.0;
        if (abs_sum) abs_sum[e] = 0.0;
    }
    for (int64_t n = 0; n < N; ++n)
        for (int64_t co = 0; co < Cout; ++co)
            for (int64_t ho = 0; ho < Ho; ++ho)
                for (int64_t wo = 0; wo < Wo; ++wo) {
                    const double g = (double)gy[((n * Cout + co) * Ho + ho) * Wo + wo];
                    for (int64_t ci = 0; ci < Cin; ++ci)
                        for (int32_t a = 0; a < kh; ++a)
                            for (int32_t b = 0; b < kw; ++b) {
                                const int64_t h = ho * sh - ph + a, c = wo * sw - pw + b;
                                if (h < 0 || h >= H || c < 0 || c >= W) continue;
                                const int64_t xi = ((n * Cin + ci) * H + h) * W + c;
                                const int64_t wi = ((co * Cin + ci) * kh + a) * kw + b;
                                const double term = (double)other[which == 0 ? wi : xi] * g;
                                const int64_t at = which == 0 ? xi : wi;
                                out[at] += term;
                                if (abs_sum) abs_sum[at] += fabs(term);
                            }
                }
    return 0;
}

int sws_ref_conv2d_grad_input(const float *gy, const float *wgt, double *gx, double *abs_sum,
                              int64_t N, int64_t Cin, int64_t H, int64_t W, int64_t Cout,
                              int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw)
{
    return conv2d_adjoint(0, wgt, gy, gx, abs_sum, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw);
}

int sws_ref_conv2d_grad_weight(const float *x, const float *gy, double *gw, double *abs_sum,
                               int64_t N, int64_t Cin, int64_t H, int64_t W, int64_t Cout,
                               int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw)
{
    return conv2d_adjoint(1, x, gy, gw, abs_sum, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw);
}

/* Gradient of loss = sum(gy * maxpool(x)) with respect to x (sws_ref_pool2d with op = max, same
 * geometry).  Scatter form: for every window, scan its cells inside the plane in row-major order,
 * keep the first cell whose value is strictly greater than all before it, add gy there.
 * gx: N*C*H*W doubles, overwritten. */
int sws_ref_maxpool2d_grad(const float *x, const float *gy, double *gx, int64_t N, int64_t C, int64_t H, int64_t W,
                           int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw)
{
    if (N < 0 || C < 0 || H < 0 || W < 0) return 1;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return 1;
    if (ph >= kh || pw >= kw) return 1;
    if (kh > H + 2 * (int64_t)ph || kw > W + 2 * (int64_t)pw) return 1;
    const int64_t Ho = (H + 2 * (int64_t)ph - kh) / sh + 1;
    const int64_t Wo = (W + 2 * (int64_t)pw - kw) / sw + 1;
    const int64_t planes = N * C;
    if (planes > 0 && (!x || !gy || !gx)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        const float *xp = x + p * H * W;
        double *gp = gx + p * H * W;
        for (int64_t e = 0; e < H * W; ++e) gp[e] = 0.0;
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo) {
                int64_t best = -1;
                for (int32_t a = 0; a < kh; ++a)
                    for (int32_t b = 0; b < kw; ++b) {
                        const int64_t h = ho * sh - ph + a, c = wo * sw - pw + b;
                        if (h < 0 || h >= H || c < 0 || c >= W) continue;
                        if (best < 0 || xp[h * W + c] > xp[best]) best = h * W + c;
                    }
                gp[best] += (double)gy[(p * Ho + ho) * Wo + wo];
            }
    }
    return 0;
}

/* The adjoint of average pooling (sws_ref_pool2d_ex, ADD, padding ph / pw on both sides): with
 * loss = sum(gy * y) and y = f * sum of the window's cells inside the plane, every such cell
 * receives f * gy of every window that holds it; f = scale (div_valid = 0) or scale / n with n
 * the number of cells of that window inside the plane.  Scatter form, windows in row-major order.
 * gx, abs_sum (optional): N*C*H*W doubles, overwritten. */
int sws_ref_avgpool2d_grad(const float *gy, double *gx, double *abs_sum, int64_t N, int64_t C, int64_t H, int64_t W,
                           int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, int div_valid,
                           double scale)
{
    if (N < 0 || C < 0 || H < 1 || W < 1) return 1;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return 1;
    if (ph >= kh || pw >= kw) return 1;
    if (kh > H + 2 * (int64_t)ph || kw > W + 2 * (int64_t)pw) return 1;
    const int64_t Ho = (H + 2 * (int64_t)ph - kh) / sh + 1;
    const int64_t Wo = (W + 2 * (int64_t)pw - kw) / sw + 1;
    const int64_t planes = N * C;
    if (planes > 0 && (!gy || !gx)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        double *gp = gx + p * H * W;
        double *mp = abs_sum ? abs_sum + p * H * W : 0;
        for (int64_t e = 0; e < H * W; ++e) {
            gp[e] = 0.0;
            if (mp) mp[e] = 0.0;
        }
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo) {
                int64_t n = 0;
                for (int32_t a = 0; a < kh; ++a)
                    for (int32_t b = 0; b < kw; ++b) {
                        const int64_t h = ho * sh - ph + a, c = wo * sw - pw + b;
                        if (h >= 0 && h < H && c >= 0 && c < W) ++n;
                    }
                const double term = (div_valid ? scale / (double)n : scale) * (double)gy[(p * Ho + ho) * Wo + wo];
                for (int32_t a = 0; a < kh; ++a)
                    for (int32_t b = 0; b < kw; ++b) {
                        const int64_t h = ho * sh - ph + a, c = wo * sw - pw + b;
                        if (h < 0 || h >= H || c < 0 || c >= W) continue;
                        gp[h * W + c] += term;
                        if (mp) mp[h * W + c] += fabs(term);
                    }
            }
    }
    return 0;
}

/* 1-D convolution (Section 2.5, Eq. 4 per output) over rows extended by pad_left elements in front and
 * pad_right behind under a boundary condition of Section 3 (mode 0 zero padding, 1 mirror, 2 periodic,
 * 3 edge replication):
 *   y[b,co,i] = sum_ci sum_t wgt[co,ci,t] * xe[b, g*cig+ci, i*stride + t*dilation],  xe[e] = x[map(e - pad_left)]
 * x: [B,Cin,L]; wgt: [Cout,Cin/groups,k]; y, abs_sum: [B,Cout,Lo], Lo = (L+pad_left+pad_right-span)/stride + 1. */
int sws_ref_conv1d_padded(const float *x, const float *wgt, double *y, double *abs_sum, int64_t B, int64_t Cin,
                          int64_t L, int64_t Cout, int32_t k, int32_t stride, int32_t pad_left, int32_t pad_right,
                          int32_t dilation, int32_t groups, int mode)
{
    if (B < 0 || Cin < 1 || L < 1 || Cout < 1 || k < 1 || stride < 1 || pad_left < 0 || pad_right < 0 || dilation < 1 ||
        groups < 1 || mode < 0 || mode > 3)
        return 1;
    if (Cin % groups || Cout % groups) return 1;
    if (mode == 1 && (pad_left > L - 1 || pad_right > L - 1)) return 1;
    if (mode == 2 && (pad_left > L || pad_right > L)) return 1;
    const int64_t span = (int64_t)dilation * (k - 1) + 1, Le = L + pad_left + pad_right;
    if (span > Le) return 1;
    const int64_t Lo = (Le - span) / stride + 1;
    const int64_t cig = Cin / groups, cog = Cout / groups;
    if (B > 0 && (!x || !wgt || !y)) return 1;
    const int64_t units = B * Cout;
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < units; ++u) {
        const int64_t b = u / Cout, co = u % Cout, g = co / cog;
        for (int64_t i = 0; i < Lo; ++i) {
            double acc = 0.0, mag = 0.0;
            for (int64_t ci = 0; ci < cig; ++ci) {
                const float *xr = x + (b * Cin + g * cig + ci) * L;
                const float *wr = wgt + (co * cig + ci) * k;
                for (int32_t t = 0; t < k; ++t) {
                    const int64_t j = map_index(i * stride + (int64_t)t * dilation - pad_left, L, mode);
                    if (j < 0) continue;                             /* zero padding */
                    const double term = (double)wr[t] * (double)xr[j];
                    acc += term;
                    mag += fabs(term);
                }
            }
            y[u * Lo + i] = acc;
            if (abs_sum) abs_sum[u * Lo + i] = mag;
        }
    }
    return 0;
}

/* 2-D convolution (Section 2.5's sliding dot product on NCHW planes, OIHW taps, groups = 1) over planes
 * extended on their four sides under a boundary condition of Section 3 (mode 0 zero padding, 1 mirror,
 * 2 periodic, 3 edge replication); the rule maps the row index and the column index independently:
 *   y[n,co,ho,wo] = sum_ci sum_a sum_b wgt[co,ci,a,b] * x[n,ci, map(ho*sh - pad_top + a), map(wo*sw - pad_left + b)]
 * y, abs_sum: [N,Cout,Ho,Wo], Ho = (H+pad_top+pad_bottom-kh)/sh + 1, Wo likewise. */
int sws_ref_conv2d_padded(const float *x, const float *wgt, double *y, double *abs_sum, int64_t N, int64_t Cin,
                          int64_t H, int64_t W, int64_t Cout, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                          int32_t pad_top, int32_t pad_left, int32_t pad_bottom, int32_t pad_right, int mode)
{
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || mode < 0 || mode > 3) return 1;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || pad_top < 0 || pad_left < 0 || pad_bottom < 0 || pad_right < 0) return 1;
    if (mode == 1 && (pad_top > H - 1 || pad_bottom > H - 1 || pad_left > W - 1 || pad_right > W - 1)) return 1;
    if (mode == 2 && (pad_top > H || pad_bottom > H || pad_left > W || pad_right > W)) return 1;
    const int64_t He = H + pad_top + pad_bottom, We = W + pad_left + pad_right;
    if (kh > He || kw > We) return 1;
    const int64_t Ho = (He - kh) / sh + 1, Wo = (We - kw) / sw + 1;
    if (N > 0 && (!x || !wgt || !y)) return 1;
    const int64_t units = N * Cout;
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < units; ++u) {
        const int64_t n = u / Cout, co = u % Cout;
        for (int64_t ho = 0; ho < Ho; ++ho) {
            for (int64_t wo = 0; wo < Wo; ++wo) {
                double acc = 0.0, mag = 0.0;
                for (int64_t ci = 0; ci < Cin; ++ci) {
                    const float *xp = x + (n * Cin + ci) * H * W;
                    const float *wp = wgt + (co * Cin + ci) * kh * kw;
                    for (int32_t a = 0; a < kh; ++a) {
                        const int64_t h = map_index(ho * sh - pad_top + a, H, mode);
                        if (h < 0) continue;
                        for (int32_t b = 0; b < kw; ++b) {
                            const int64_t c = map_index(wo * sw - pad_left + b, W, mode);
                            if (c < 0) continue;
                            const double term = (double)wp[a * kw + b] * (double)xp[h * W + c];
                            acc += term;
                            mag += fabs(term);
                        }
                    }
                }
                y[(u * Ho + ho) * Wo + wo] = acc;
                if (abs_sum) abs_sum[(u * Ho + ho) * Wo + wo] = mag;
            }
        }
    }
    return 0;
}
