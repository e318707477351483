/*
 * sws.h — C ABI of libsws: sliding window sums on one AMD MI355X (gfx950).
 *
 * Implements the hot path of "Sliding Window Sum Algorithms for Deep Neural
 * Networks" (arXiv 2305.16513): the sliding window sum of Section 2.2 (Eq. 3)
 * used as average / max pooling (Section 2.3) and as convolution that reads
 * the unmodified input and never builds an im2col column matrix (Section 2.5).
 *
 * Conventions common to every entry point
 *   - Every data pointer is DEVICE memory owned by the caller (fp32, densely
 *     packed, row-major in the stated index order, 4-byte aligned; 16-byte
 *     aligned bases are fastest).  Inputs are read-only and must not overlap
 *     the output.  The library allocates nothing, frees nothing and keeps no
 *     pointer after the call returns.
 *   - `stream` is a hipStream_t (sws_stream_t is the same pointer type, declared
 *     here so that the header needs no HIP include; NULL = the default stream).
 *     Work is enqueued on it; calls are asynchronous and never synchronise.
 *   - Errors are reported by return code only.  Arguments are checked before
 *     anything is launched; a problem with zero outputs returns SWS_OK without
 *     launching.  A failed launch returns SWS_ERR_HIP; the thread's HIP
 *     last-error state is cleared on entry, so that an error left by earlier
 *     calls of the caller is not reported as a failure of this one.
 *   - Inputs are assumed finite.  NaN propagation through MAX / MIN is
 *     unspecified, and so is the sign of a zero result when a MAX / MIN window
 *     holds both +0.0 and -0.0.  ADD and the convolutions accumulate in fp32:
 *     once a partial sum of a window (or of the up to 2w elements around it
 *     that a scan segment covers) overflows fp32, the outputs near it are
 *     unspecified (inf or NaN), even where the window's own sum is finite.
 *   - Row lengths and plane extents are indexed in int32: at most
 *     2^31 - 1 - 65536 = 2147418111 elements ("the int32 limit" below).
 *   - Reentrant: the entry points of this header keep no mutable global state.
 *     (The measurement knobs of sws_dev.h are process-wide and are not part of
 *     this contract.)
 */
#ifndef SWS_H
#define SWS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* hipStream_t is `struct ihipStream_t *` in <hip/hip_runtime_api.h>; a caller that includes the HIP
 * headers passes its hipStream_t unchanged. */
typedef struct ihipStream_t *sws_stream_t;

typedef enum {
    SWS_OK = 0,
    SWS_ERR_INVALID_ARG = 1,   /* null pointer, bad size, window larger than input, overflow */
    SWS_ERR_UNSUPPORTED = 2,   /* legal request that no kernel variant covers */
    SWS_ERR_HIP = 3            /* the HIP runtime refused the launch */
} sws_status;

/* The associative operator (+) of Eq. 3.  ADD and MAX are pooling (Section 2.3);
 * MIN is the paper's example of another associative operator (Section 3). */
typedef enum { SWS_OP_ADD = 0, SWS_OP_MAX = 1, SWS_OP_MIN = 2 } sws_op;

/* Boundary conditions of an extended row (Section 3 names padding, mirroring and periodicity):
 * what the virtual elements in front of x[0] and behind x[len-1] stand for. */
typedef enum {
    SWS_PAD_IDENTITY = 0,      /* the identity of the operator: 0 for ADD, -inf for MAX, +inf for MIN */
    SWS_PAD_MIRROR = 1,        /* x[-i] = x[i], x[len-1+i] = x[len-1-i] (end elements not repeated) */
    SWS_PAD_PERIODIC = 2,      /* x[-i] = x[len-i], x[len-1+i] = x[i-1] */
    SWS_PAD_EDGE = 3,          /* x[-i] = x[0], x[len-1+i] = x[len-1] */
    SWS_PAD_SHRINK = 4         /* the window shrinks at the ends: virtual elements are skipped and an ADD
                                  result is multiplied by w / n, n = real elements in the window, so that
                                  scale = 1/w gives the mean over real elements (pads must be < w) */
} sws_pad_mode;

/* Sliding window sum, Section 2.2 Eq. 3, applied to `rows` independent sequences:
 *
 *   y[r, i] = scale * ( x[r,i] (+) x[r,i+1] (+) ... (+) x[r,i+w-1] ),   0 <= i <= len - w
 *
 * Every output combines exactly w inputs ("valid"), operands in index order.
 *   x : device, rows*len floats          y : device, rows*(len-w+1) floats
 *   scale multiplies ADD results (1/w gives 1-D average pooling); ignored for MAX / MIN.
 * Errors: INVALID_ARG if op is unknown, rows < 0, len < 0, w < 1, w > len, a pointer is
 * NULL while there is output, or a size overflows int64 / len exceeds the int32 limit. */
sws_status sws_slide1d(sws_op op, const float *x, float *y, int64_t rows, int64_t len,
                       int32_t w, float scale, sws_stream_t stream);

/* The same sliding window sum over rows extended by pad_left virtual elements in front and
 * pad_right behind, filled by the boundary rule `mode`:
 *
 *   y[r, i] = scale * ( xe[r,i] (+) ... (+) xe[r,i+w-1] ),   0 <= i <= len + pad_left + pad_right - w
 *
 * with xe the extended row.  pad_left = pad_right = (w-1)/2 with odd w gives one output per
 * input ("same" pooling).  scale multiplies ADD results, padding included.
 *   x : device, rows*len floats     y : device, rows*(len+pad_left+pad_right-w+1) floats
 * Errors: as sws_slide1d, and INVALID_ARG if len < 1, a pad is negative, w exceeds the extended
 * row, the mode is unknown, a MIRROR pad exceeds len-1, a PERIODIC pad exceeds len or a SHRINK
 * pad is not smaller than w. */
sws_status sws_slide1d_padded(sws_op op, const float *x, float *y, int64_t rows, int64_t len,
                              int32_t w, int32_t pad_left, int32_t pad_right, sws_pad_mode mode,
                              float scale, sws_stream_t stream);

/* Storage types of sws_slide1d_16.  Arithmetic is fp32 for both. */
typedef enum {
    SWS_DTYPE_BF16 = 1,        /* 1 sign, 8 exponent, 7 fraction bits (the upper half of an fp32) */
    SWS_DTYPE_F16 = 2          /* IEEE 754 binary16 */
} sws_dtype;

/* sws_slide1d on 16-bit storage: the input quantised to fewer bits (the paper's introduction
 * names quantisation as the way to shrink what a layer moves; Eq. 3 itself is unchanged).
 * x and y hold bf16 or fp16 elements; each element is widened to fp32 exactly, the window is
 * combined in fp32 as in sws_slide1d, multiplied by scale (ADD), and rounded to the storage
 * type once, to nearest even.  MAX / MIN results are therefore exact.  Half the bytes of the
 * fp32 entry point cross HBM.
 *   x : device, rows*len 16-bit elements     y : device, rows*(len-w+1) 16-bit elements
 *   (2-byte aligned; densely packed)
 * Errors: as sws_slide1d, and INVALID_ARG for an unknown dtype. */
sws_status sws_slide1d_16(sws_op op, sws_dtype dtype, const void *x, void *y, int64_t rows,
                          int64_t len, int32_t w, float scale, sws_stream_t stream);

/* Sliding window sum (Eq. 3) under the pair operator of Section 2.4, Eq. 8 — the associative,
 * NON-commutative operator with which the paper writes a dot product as a prefix sum:
 *
 *   (u_i, v_i) (+) (u_j, v_j) = (u_i * u_j,  u_j * v_i + v_j),      i older than j
 *   (yu, yv)[r, i] = (u, v)[r, i] (+) (u, v)[r, i+1] (+) ... (+) (u, v)[r, i+w-1],   0 <= i <= len - w
 *
 * i.e. the composition, oldest first, of the w maps z -> u z + v.  Pairs are passed as two
 * planes.  u = 1 gives the sliding add of v; v = 0 gives the sliding product of u.
 *   u, v : device, rows*len floats each        yu, yv : device, rows*(len-w+1) floats each
 * Errors: INVALID_ARG if rows < 0, len < 0, w < 1, w > len, a pointer is NULL while there is
 * output, or a size overflows int64 / len exceeds the int32 limit. */
sws_status sws_slide1d_pair(const float *u, const float *v, float *yu, float *yv, int64_t rows,
                            int64_t len, int32_t w, sws_stream_t stream);

/* 2-D pooling (Section 2.3 extended to two dimensions) evaluated as separable sliding
 * sums, first along H then along W, on NCHW data:
 *
 *   y[n,c,ho,wo] = scale * (+)_{a<kh} (+)_{b<kw} x[n,c, ho*sh - ph + a, wo*sw - pw + b]
 *
 * Ho = (H + 2*ph - kh)/sh + 1, Wo = (W + 2*pw - kw)/sw + 1 (floor).  Padding cells hold
 * the identity of op (0 for ADD, -inf for MAX, +inf for MIN).  scale multiplies ADD
 * results (1/(kh*kw) = average pooling that counts the padding); ignored for MAX / MIN.
 *   x : device, N*C*H*W floats          y : device, N*C*Ho*Wo floats
 * Errors: INVALID_ARG for unknown op, negative sizes, kh/kw/sh/sw < 1, ph/pw < 0,
 * ph >= kh or pw >= kw (a window wholly inside padding), window larger than the padded
 * input, NULL pointer with output, H or W above the int32 limit. */
sws_status sws_pool2d(sws_op op, const float *x, float *y, int64_t N, int64_t C, int64_t H,
                      int64_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                      int32_t ph, int32_t pw, float scale, sws_stream_t stream);

/* The adjoint of max pooling (sws_pool2d with SWS_OP_MAX, same geometry) at the point x: with
 * loss = sum(gy * y), every window adds its gy to the gx of the cell that holds its maximum — the
 * first such cell in row-major order of the window when several tie (padding never wins).
 *   x, gx : device, N*C*H*W floats     gy : device, N*C*Ho*Wo floats
 * gx is overwritten (cells no window chose get 0).  Deterministic: a cell adds the gradients of
 * the windows that chose it in a fixed order, without atomic operations.
 * Errors: as sws_pool2d. */
sws_status sws_maxpool2d_grad(const float *x, const float *gy, float *gx, int64_t N, int64_t C,
                              int64_t H, int64_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                              int32_t ph, int32_t pw, sws_stream_t stream);

/* sws_pool2d on 16-bit storage, defined like sws_slide1d_16: x and y hold bf16 or fp16 elements,
 * each widened to fp32 exactly; the window is combined in fp32 as in sws_pool2d, multiplied by
 * scale (ADD) and rounded to the storage type once, to nearest even.  MAX / MIN are exact.
 *   x : device, N*C*H*W 16-bit elements     y : device, N*C*Ho*Wo 16-bit elements
 * Errors: as sws_pool2d, and INVALID_ARG for an unknown dtype. */
sws_status sws_pool2d_16(sws_op op, sws_dtype dtype, const void *x, void *y, int64_t N, int64_t C,
                         int64_t H, int64_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                         int32_t ph, int32_t pw, float scale, sws_stream_t stream);

/* What an ADD result of sws_pool2d_ex is divided by. */
typedef enum {
    SWS_DIV_SCALE = 0,         /* nothing: y = scale * sum (scale = 1/(kh*kw): the average that counts padding) */
    SWS_DIV_REAL_CELLS = 1     /* the number of window cells inside the plane: y = scale * sum / n
                                  (scale = 1: the average that does not count padding) */
} sws_divisor;

/* sws_pool2d with separate padding on the four sides and a choice of averaging rule (boundary
 * handling beyond the symmetric padding of sws_pool2d; Section 3 leaves boundary conditions to
 * the application):
 *
 *   y[n,c,ho,wo] = f * (+)_{a<kh} (+)_{b<kw} x[n,c, ho*sh - pad_top + a, wo*sw - pad_left + b]
 *   Ho = (H + pad_top + pad_bottom - kh)/sh + 1,  Wo = (W + pad_left + pad_right - kw)/sw + 1
 *
 * Cells outside the plane hold the identity of op.  f = scale, or scale / n with n the number of
 * window cells inside the plane (divisor; ADD only, MAX / MIN ignore both).
 *   x : device, N*C*H*W floats          y : device, N*C*Ho*Wo floats
 * Errors: as sws_pool2d; every pad must be smaller than the kernel extent on its axis (each
 * window then holds a real cell); H, W >= 1; unknown divisor. */
sws_status sws_pool2d_ex(sws_op op, const float *x, float *y, int64_t N, int64_t C, int64_t H,
                         int64_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                         int32_t pad_top, int32_t pad_left, int32_t pad_bottom, int32_t pad_right,
                         sws_divisor divisor, float scale, sws_stream_t stream);

/* 2-D pooling over planes extended by the boundary conditions of Section 3 (padding with the
 * identity, mirroring, periodicity; also the repeated edge and shrinking windows) on all four
 * sides — sws_slide1d_padded carried to two dimensions; the rule applies to rows and columns
 * independently (a corner cell mirrors / wraps on both axes):
 *
 *   y[n,c,ho,wo] = scale * (+)_{a<kh} (+)_{b<kw} xe[n,c, ho*sh + a, wo*sw + b]
 *   xe[n,c,i,j]  = x[n,c, src(i - pad_top, H), src(j - pad_left, W)],  0 <= i < H + pad_top + pad_bottom,
 *   Ho = (H + pad_top + pad_bottom - kh)/sh + 1,  Wo = (W + pad_left + pad_right - kw)/sw + 1
 *
 * with src the index rule of `mode` as in sws_pad_mode (IDENTITY: the cell holds the identity of
 * op; SHRINK: identity, and an ADD result is divided by the number of window cells inside the
 * plane, i.e. sws_pool2d_ex with SWS_DIV_REAL_CELLS).  scale multiplies ADD results only.
 *   x : device, N*C*H*W floats          y : device, N*C*Ho*Wo floats
 * Errors: as sws_pool2d; INVALID_ARG if H or W < 1, a pad is negative, the window exceeds the
 * extended plane, the mode is unknown, a MIRROR pad exceeds the extent of its axis minus 1, a
 * PERIODIC pad exceeds that extent, or a SHRINK pad is not smaller than the window on its axis;
 * UNSUPPORTED if the extended plane has more than 2^31 - 1 - 65536 cells. */
sws_status sws_pool2d_padded(sws_op op, const float *x, float *y, int64_t N, int64_t C, int64_t H,
                             int64_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                             int32_t pad_top, int32_t pad_left, int32_t pad_bottom, int32_t pad_right,
                             sws_pad_mode mode, float scale, sws_stream_t stream);

/* The adjoint of average pooling (Section 2.3's pooling with the + operator, training side): of
 * sws_pool2d_ex with SWS_OP_ADD, padding ph on top and bottom and pw left and right, and the same
 * divisor and scale.  With loss = sum(gy * y),
 *   gx[n,c,h,w] = sum over the windows (ho, wo) that hold (h, w) of f(ho, wo) * gy[n,c,ho,wo],
 * f = scale, or scale / n(ho, wo) with n the number of cells of that window inside the plane
 * (SWS_DIV_REAL_CELLS).  At stride 1 with SWS_DIV_SCALE this is itself a sliding add of gy over a
 * plane padded by k - 1 - pad; at larger strides cells between windows receive 0.
 *   gy : device, N*C*Ho*Wo floats     gx : device, N*C*H*W floats, overwritten
 * Deterministic: a cell adds its windows in a fixed order, without atomic operations.
 * Errors: as sws_pool2d; INVALID_ARG for an unknown divisor. */
sws_status sws_avgpool2d_grad(const float *gy, float *gx, int64_t N, int64_t C, int64_t H, int64_t W,
                              int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                              sws_divisor divisor, float scale, sws_stream_t stream);

/* 1-D convolution as a sliding dot product (Section 2.5; Eq. 4 per output), in the DNN
 * sense: cross-correlation, taps not flipped, zero padding, no bias.
 *
 *   y[b,co,i] = sum_{ci < Cin/groups} sum_{t < k}
 *                 wgt[co,ci,t] * x[b, g*Cin/groups + ci, i*stride + t*dilation - pad]
 *   g = co / (Cout/groups),  Lo = (L + 2*pad - dilation*(k-1) - 1)/stride + 1
 *
 *   x : device [B,Cin,L]    wgt : device [Cout,Cin/groups,k]    y : device [B,Cout,Lo]
 * groups = 1 is the dense-channel contraction; groups = Cin = Cout is depthwise.
 * Errors: INVALID_ARG for sizes < 0, Cin/Cout/k/stride/dilation/groups < 1, pad < 0,
 * Cin or Cout not divisible by groups, kernel span above the padded length, NULL pointer
 * with output, L above the int32 limit. */
sws_status sws_conv1d(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin,
                      int64_t L, int64_t Cout, int32_t k, int32_t stride, int32_t pad,
                      int32_t dilation, int32_t groups, sws_stream_t stream);

/* sws_conv1d over rows extended by pad_left elements in front and pad_right behind under a boundary
 * condition of Section 3 (the convolution of Section 2.5 with mirrored, periodic or edge-repeated
 * ends instead of zeros; periodic with pad_right = k - 1 is the circular correlation):
 *
 *   y[b,co,i] = sum_{ci < Cin/groups} sum_{t < k} wgt[co,ci,t] * xe[b, g*Cin/groups + ci, i*stride + t*dilation]
 *   xe[.., e] = x[.., src(e - pad_left)],  Lo = (L + pad_left + pad_right - dilation*(k-1) - 1)/stride + 1
 *
 * with src the index rule of `mode` as in sws_pad_mode (IDENTITY: the element is zero).
 *   x : device [B,Cin,L]    wgt : device [Cout,Cin/groups,k]    y : device [B,Cout,Lo]
 * Errors: as sws_conv1d; INVALID_ARG if L < 1, a pad is negative, the mode is unknown or
 * SWS_PAD_SHRINK (a dot product has no shrinking form), a MIRROR pad exceeds L-1 or a PERIODIC pad
 * exceeds L. */
sws_status sws_conv1d_padded(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L,
                             int64_t Cout, int32_t k, int32_t stride, int32_t pad_left, int32_t pad_right,
                             int32_t dilation, int32_t groups, sws_pad_mode mode, sws_stream_t stream);

/* sws_conv1d on 16-bit storage (the paper's introduction names quantisation as the way to shrink
 * what a layer moves; Section 2.5 itself is unchanged): x and y hold bf16 or fp16 elements, the taps
 * stay fp32.  Each element is widened to fp32 exactly, the sliding dot product is accumulated in
 * fp32 as in sws_conv1d, and each output is rounded to the storage type once, to nearest even.
 * The depthwise layer (groups = Cin = Cout, stride 1, dilation 1, k <= 64), which is bound by
 * memory traffic, moves half the bytes of the fp32 entry point; other geometries are evaluated
 * directly.
 *   x : device [B,Cin,L] 16-bit    wgt : device [Cout,Cin/groups,k] fp32    y : device [B,Cout,Lo] 16-bit
 *   (x, y 2-byte aligned, wgt 4-byte aligned; densely packed)
 * Errors: as sws_conv1d, and INVALID_ARG for an unknown dtype. */
sws_status sws_conv1d_16(sws_dtype dtype, const void *x, const float *wgt, void *y, int64_t B, int64_t Cin,
                         int64_t L, int64_t Cout, int32_t k, int32_t stride, int32_t pad, int32_t dilation,
                         int32_t groups, sws_stream_t stream);

/* The two adjoints of sws_conv1d (the training side of the sliding dot product of Section 2.5;
 * the abstract names training next to inference).  With loss = sum(gy * y):
 *
 *   gx[b,c,j]     = sum over (co, t) of the group of c with j + pad - t*dilation = i*stride,
 *                   0 <= i < Lo:   wgt[co, ci, t] * gy[b, co, i]                (d loss / d x)
 *   gw[co,ci,t]   = sum over (b, i) with 0 <= i*stride + t*dilation - pad < L:
 *                   gy[b, co, i] * x[b, g*Cin/groups + ci, i*stride + t*dilation - pad]
 *                                                                              (d loss / d wgt)
 *
 * All sizes are those of the forward call (L is the length of x, Lo = sws_out_len(...) that of
 * gy).  gx and gw are overwritten, not accumulated into.  gw is summed with atomic adds whose
 * order is not fixed: its last bits may differ between runs.  On dense layers (groups = 1, stride and
 * dilation 1, k = 1, 3 or 5, channel counts in multiples of 32) a product of gw is evaluated as six
 * exact products of bf16 pieces of its fp32 operands, which drops less than 2^-23 of it (inputs
 * must be finite there: an infinite operand splits into inf and NaN).
 *   gy : device [B,Cout,Lo]   wgt, gw : device [Cout,Cin/groups,k]   x, gx : device [B,Cin,L]
 * Errors: as sws_conv1d. */
sws_status sws_conv1d_grad_input(const float *gy, const float *wgt, float *gx, int64_t B,
                                 int64_t Cin, int64_t L, int64_t Cout, int32_t k, int32_t stride,
                                 int32_t pad, int32_t dilation, int32_t groups, sws_stream_t stream);
sws_status sws_conv1d_grad_weight(const float *x, const float *gy, float *gw, int64_t B,
                                  int64_t Cin, int64_t L, int64_t Cout, int32_t k, int32_t stride,
                                  int32_t pad, int32_t dilation, int32_t groups, sws_stream_t stream);

/* 2-D convolution (same reading of Section 2.5 on NCHW x and OIHW wgt, groups = 1):
 *
 *   y[n,co,ho,wo] = sum_ci sum_{a<kh} sum_{b<kw} wgt[co,ci,a,b] * x[n,ci, ho*sh-ph+a, wo*sw-pw+b]
 *
 * Zero padding, no bias, no dilation.  Ho, Wo as for sws_pool2d.
 *   x : device [N,Cin,H,W]   wgt : device [Cout,Cin,kh,kw]   y : device [N,Cout,Ho,Wo]
 * Accumulation is fp32 and the summation order is unspecified; every output is within
 * 1e-5 * sum|terms| of the exact sum.  On some layers (64 input channels, 3 x 3, stride 1) a product
 * x * w is evaluated as six exact products of bf16 pieces of the fp32 operands, which drops less than
 * 2^-23 of it; products of integers below 2^8 stay exact.  (The same holds for sws_conv1d on dense
 * layers of 32 / 64 input channels.)
 * Errors: as sws_conv1d. */
sws_status sws_conv2d(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin,
                      int64_t H, int64_t W, int64_t Cout, int32_t kh, int32_t kw,
                      int32_t sh, int32_t sw, int32_t ph, int32_t pw, sws_stream_t stream);

/* sws_conv2d over planes extended on their four sides under a boundary condition of Section 3 (mirrored,
 * periodic or edge-repeated borders instead of zeros; the rule maps the row index and the column index
 * independently, as in sws_pool2d_padded):
 *
 *   y[n,co,ho,wo] = sum_ci sum_{a<kh} sum_{b<kw} wgt[co,ci,a,b] * xe[n,ci, ho*sh + a, wo*sw + b]
 *   xe[n,ci,i,j]  = x[n,ci, src(i - pad_top, H), src(j - pad_left, W)]
 *   Ho = (H + pad_top + pad_bottom - kh)/sh + 1,  Wo = (W + pad_left + pad_right - kw)/sw + 1
 *
 *   x : device [N,Cin,H,W]    wgt : device [Cout,Cin,kh,kw]    y : device [N,Cout,Ho,Wo]
 * With equal pads on opposite sides the result is the zero-padding convolution (sws_conv2d's kernels
 * and accuracy) plus the virtual cells' terms added to the outputs at the border in a second launch on
 * the same stream; otherwise every output is evaluated directly.
 * Errors: as sws_conv2d; INVALID_ARG if H or W < 1, a pad is negative, the mode is unknown or
 * SWS_PAD_SHRINK, a MIRROR pad exceeds the extent of its axis minus 1 or a PERIODIC pad that extent. */
sws_status sws_conv2d_padded(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                             int64_t W, int64_t Cout, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                             int32_t pad_top, int32_t pad_left, int32_t pad_bottom, int32_t pad_right,
                             sws_pad_mode mode, sws_stream_t stream);

/* The two adjoints of sws_conv2d, defined like those of sws_conv1d (loss = sum(gy * y)):
 *   gx[n,ci,h,c]     = sum over (co, a, b) with h + ph - a = ho*sh, c + pw - b = wo*sw inside the
 *                      output:  wgt[co,ci,a,b] * gy[n,co,ho,wo]
 *   gw[co,ci,a,b]    = sum over (n, ho, wo) whose tap (a, b) lies inside the plane:
 *                      gy[n,co,ho,wo] * x[n,ci, ho*sh - ph + a, wo*sw - pw + b]
 * Sizes are those of the forward call.  gx and gw are overwritten; gw is summed with atomic adds
 * whose order is not fixed.  Accuracy as for sws_conv2d; on some layers (3 x 3 at stride 1 or 2, and
 * 1 x 1, 1 x 3, 1 x 5 at stride 1 without padding above and below, channel counts in multiples of 32)
 * a product of gw is evaluated as six exact products of bf16 pieces of its fp32
 * operands, which drops less than 2^-23 of it (inputs must be finite there: an infinite operand splits
 * into inf and NaN).
 *   gy : device [N,Cout,Ho,Wo]   wgt, gw : device [Cout,Cin,kh,kw]   x, gx : device [N,Cin,H,W]
 * Errors: as sws_conv2d. */
sws_status sws_conv2d_grad_input(const float *gy, const float *wgt, float *gx, int64_t N,
                                 int64_t Cin, int64_t H, int64_t W, int64_t Cout, int32_t kh,
                                 int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                                 sws_stream_t stream);
sws_status sws_conv2d_grad_weight(const float *x, const float *gy, float *gw, int64_t N,
                                  int64_t Cin, int64_t H, int64_t W, int64_t Cout, int32_t kh,
                                  int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                                  sws_stream_t stream);

/* Plain device-to-device copy of n floats with the same 128-bit access pattern the
 * sliding kernels use.  Not part of the method: it measures the HBM ceiling a
 * one-read-one-write kernel can reach on this device, and calibrates byte counters. */
sws_status sws_copy(const float *src, float *dst, int64_t n, sws_stream_t stream);

/* Host helper: number of outputs of a sliding window of `w` taps spaced `dilation`
 * apart over `len` inputs padded by `pad` on both sides, moved in steps of `stride`.
 * Returns -1 if the arguments are invalid or no window fits. */
int64_t sws_out_len(int64_t len, int32_t w, int32_t stride, int32_t pad, int32_t dilation);

/* Static, never-freed description of a status code. */
const char *sws_status_string(int status);

/* Library version, "major.minor". */
const char *sws_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SWS_H */
