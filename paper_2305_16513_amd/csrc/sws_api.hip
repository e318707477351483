// C ABI of libsws: argument checks and dispatch.  Nothing here touches device data.
#include <string.h>

#include "sws_internal.h"

namespace sws {
Options g_opt;

int device_cus()
{
    static std::atomic<int> cus{0};
    int v = cus.load(std::memory_order_relaxed);
    if (v == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            return 256;
        cus.store(v, std::memory_order_relaxed);
    }
    return v;
}
}

namespace {

constexpr int64_t kMaxDim = 2147483647LL - 65536;   // per-row / per-plane extents are indexed in int32
                                                    // with headroom for one tile of look-ahead

bool mul3(int64_t a, int64_t b, int64_t c, int64_t *out)
{
    int64_t t;
    if (__builtin_mul_overflow(a, b, &t)) return false;
    if (__builtin_mul_overflow(t, c, out)) return false;
    return *out <= (INT64_MAX / 4);        // byte offsets must fit as well
}

bool valid_op(int op) { return op == SWS_OP_ADD || op == SWS_OP_MAX || op == SWS_OP_MIN; }

// kNotTaken reaching the boundary: no kernel covers the request (a grid beyond the launch limit).
sws_status from_hip(hipError_t e)
{
    return e == hipSuccess ? SWS_OK : e == sws::kNotTaken ? SWS_ERR_UNSUPPORTED : SWS_ERR_HIP;
}
// Launchers report hipGetLastError() after their launch; an error left over from the caller's earlier
// HIP calls is cleared first so that it is not taken for a failure of this launch.
#define SWS_LAUNCH(call) ((void)hipGetLastError(), from_hip(call))

}  // namespace

extern "C" {

const char *sws_version(void) { return "0.1"; }

const char *sws_status_string(int status)
{
    switch (status) {
    case SWS_OK: return "ok";
    case SWS_ERR_INVALID_ARG: return "invalid argument";
    case SWS_ERR_UNSUPPORTED: return "unsupported configuration";
    case SWS_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int64_t sws_out_len(int64_t len, int32_t w, int32_t stride, int32_t pad, int32_t dilation)
{
    if (len < 0 || w < 1 || stride < 1 || pad < 0 || dilation < 1) return -1;
    const int64_t span = (int64_t)dilation * (w - 1) + 1;
    const int64_t padded = len + 2 * (int64_t)pad;
    if (span > padded) return -1;
    return (padded - span) / stride + 1;
}

sws_status sws_set_option(const char *key, int64_t value)
{
    if (!key) return SWS_ERR_INVALID_ARG;
    const int v = (int)value;
    if (!strcmp(key, "slide_variant")) sws::g_opt.slide_variant = v;
    else if (!strcmp(key, "slide_chunk")) sws::g_opt.slide_chunk = v;
    else if (!strcmp(key, "slide_group")) sws::g_opt.slide_group = v;
    else if (!strcmp(key, "pool2d_variant")) sws::g_opt.pool2d_variant = v;
    else if (!strcmp(key, "conv1d_variant")) sws::g_opt.conv1d_variant = v;
    else if (!strcmp(key, "conv2d_variant")) sws::g_opt.conv2d_variant = v;
    else if (!strcmp(key, "copy_variant")) sws::g_opt.copy_variant = v;
    else return SWS_ERR_INVALID_ARG;
    return SWS_OK;
}

sws_status sws_copy(const float *src, float *dst, int64_t n, sws_stream_t stream)
{
    if (n < 0 || n > INT64_MAX / 4) return SWS_ERR_INVALID_ARG;
    if (n == 0) return SWS_OK;
    if (!src || !dst) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_copy(src, dst, n, (hipStream_t)stream));
}

sws_status sws_slide1d(sws_op op, const float *x, float *y, int64_t rows, int64_t len, int32_t w,
                       float scale, sws_stream_t stream)
{
    if (!valid_op((int)op) || rows < 0 || len < 0 || w < 1) return SWS_ERR_INVALID_ARG;
    if (len > kMaxDim || (int64_t)w > len) return SWS_ERR_INVALID_ARG;
    int64_t n_in;
    if (!mul3(rows, len, 1, &n_in)) return SWS_ERR_INVALID_ARG;
    if (rows == 0) return SWS_OK;
    if (!x || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_slide1d((int)op, x, y, rows, len, w, 0, 0, SWS_PAD_IDENTITY, scale, (hipStream_t)stream));
}

sws_status sws_slide1d_16(sws_op op, sws_dtype dtype, const void *x, void *y, int64_t rows, int64_t len, int32_t w,
                          float scale, sws_stream_t stream)
{
    if (!valid_op((int)op) || rows < 0 || len < 0 || w < 1) return SWS_ERR_INVALID_ARG;
    if (dtype != SWS_DTYPE_BF16 && dtype != SWS_DTYPE_F16) return SWS_ERR_INVALID_ARG;
    if (len > kMaxDim || (int64_t)w > len) return SWS_ERR_INVALID_ARG;
    int64_t n_in;
    if (!mul3(rows, len, 1, &n_in)) return SWS_ERR_INVALID_ARG;
    if (rows == 0) return SWS_OK;
    if (!x || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_slide1d_16((int)op, (int)dtype, x, y, rows, len, w, scale, (hipStream_t)stream));
}

sws_status sws_slide1d_padded(sws_op op, const float *x, float *y, int64_t rows, int64_t len, int32_t w,
                              int32_t pad_left, int32_t pad_right, sws_pad_mode mode, float scale, sws_stream_t stream)
{
    if (!valid_op((int)op) || rows < 0 || len < 1 || w < 1 || pad_left < 0 || pad_right < 0) return SWS_ERR_INVALID_ARG;
    if ((int)mode < SWS_PAD_IDENTITY || (int)mode > SWS_PAD_SHRINK) return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_SHRINK && (pad_left >= w || pad_right >= w)) return SWS_ERR_INVALID_ARG;
    const int64_t lv = len + pad_left + pad_right;
    if (lv > kMaxDim || (int64_t)w > lv) return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_MIRROR && (pad_left > len - 1 || pad_right > len - 1)) return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_PERIODIC && (pad_left > len || pad_right > len)) return SWS_ERR_INVALID_ARG;
    int64_t n_out;
    if (!mul3(rows, lv, 1, &n_out)) return SWS_ERR_INVALID_ARG;
    if (rows == 0) return SWS_OK;
    if (!x || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_slide1d((int)op, x, y, rows, len, w, pad_left, pad_right, (int)mode, scale,
                                        (hipStream_t)stream));
}

sws_status sws_slide1d_pair(const float *u, const float *v, float *yu, float *yv, int64_t rows, int64_t len,
                            int32_t w, sws_stream_t stream)
{
    if (rows < 0 || len < 0 || w < 1) return SWS_ERR_INVALID_ARG;
    if (len > kMaxDim || (int64_t)w > len) return SWS_ERR_INVALID_ARG;
    int64_t n_in;
    if (!mul3(rows, len, 1, &n_in)) return SWS_ERR_INVALID_ARG;
    if (rows == 0) return SWS_OK;
    if (!u || !v || !yu || !yv) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_slide1d_pair(u, v, yu, yv, rows, len, w, (hipStream_t)stream));
}

sws_status sws_pool2d(sws_op op, const float *x, float *y, int64_t N, int64_t C, int64_t H, int64_t W,
                      int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                      float scale, sws_stream_t stream)
{
    if (!valid_op((int)op) || N < 0 || C < 0 || H < 0 || W < 0) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return SWS_ERR_INVALID_ARG;
    if (ph >= kh || pw >= kw) return SWS_ERR_INVALID_ARG;
    if (H > kMaxDim || W > kMaxDim) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = sws_out_len(H, kh, sh, ph, 1), Wo = sws_out_len(W, kw, sw, pw, 1);
    if (Ho < 1 || Wo < 1) return SWS_ERR_INVALID_ARG;
    int64_t planes, n_in, n_out;
    if (!mul3(N, C, 1, &planes) || !mul3(planes, H, W, &n_in) || !mul3(planes, Ho, Wo, &n_out))
        return SWS_ERR_INVALID_ARG;
    if (H * W > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (planes == 0) return SWS_OK;
    if (!x || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_pool2d((int)op, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale, 0,
                                       (hipStream_t)stream));
}

sws_status sws_avgpool2d_grad(const float *gy, float *gx, int64_t N, int64_t C, int64_t H, int64_t W, int32_t kh,
                              int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, sws_divisor divisor, float scale,
                              sws_stream_t stream)
{
    if (N < 0 || C < 0 || H < 0 || W < 0) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return SWS_ERR_INVALID_ARG;
    if (ph >= kh || pw >= kw) return SWS_ERR_INVALID_ARG;
    if (divisor != SWS_DIV_SCALE && divisor != SWS_DIV_REAL_CELLS) return SWS_ERR_INVALID_ARG;
    if (H > kMaxDim || W > kMaxDim) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = sws_out_len(H, kh, sh, ph, 1), Wo = sws_out_len(W, kw, sw, pw, 1);
    if (Ho < 1 || Wo < 1) return SWS_ERR_INVALID_ARG;
    int64_t planes, n_in, n_out;
    if (!mul3(N, C, 1, &planes) || !mul3(planes, H, W, &n_in) || !mul3(planes, Ho, Wo, &n_out))
        return SWS_ERR_INVALID_ARG;
    if (H * W > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (planes == 0) return SWS_OK;
    if (!gy || !gx) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_avgpool2d_grad(gy, gx, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw,
                                               divisor == SWS_DIV_REAL_CELLS ? 1 : 0, scale, (hipStream_t)stream));
}

sws_status sws_maxpool2d_grad(const float *x, const float *gy, float *gx, int64_t N, int64_t C, int64_t H, int64_t W,
                              int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, sws_stream_t stream)
{
    if (N < 0 || C < 0 || H < 0 || W < 0) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return SWS_ERR_INVALID_ARG;
    if (ph >= kh || pw >= kw) return SWS_ERR_INVALID_ARG;
    if (H > kMaxDim || W > kMaxDim) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = sws_out_len(H, kh, sh, ph, 1), Wo = sws_out_len(W, kw, sw, pw, 1);
    if (Ho < 1 || Wo < 1) return SWS_ERR_INVALID_ARG;
    int64_t planes, n_in, n_out;
    if (!mul3(N, C, 1, &planes) || !mul3(planes, H, W, &n_in) || !mul3(planes, Ho, Wo, &n_out))
        return SWS_ERR_INVALID_ARG;
    if (H * W > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (planes == 0) return SWS_OK;
    if (!x || !gy || !gx) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_maxpool2d_grad(x, gy, gx, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, (hipStream_t)stream));
}

sws_status sws_pool2d_16(sws_op op, sws_dtype dtype, const void *x, void *y, int64_t N, int64_t C, int64_t H, int64_t W,
                         int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, float scale, sws_stream_t stream)
{
    if (!valid_op((int)op) || N < 0 || C < 0 || H < 0 || W < 0) return SWS_ERR_INVALID_ARG;
    if (dtype != SWS_DTYPE_BF16 && dtype != SWS_DTYPE_F16) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return SWS_ERR_INVALID_ARG;
    if (ph >= kh || pw >= kw) return SWS_ERR_INVALID_ARG;
    if (H > kMaxDim || W > kMaxDim) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = sws_out_len(H, kh, sh, ph, 1), Wo = sws_out_len(W, kw, sw, pw, 1);
    if (Ho < 1 || Wo < 1) return SWS_ERR_INVALID_ARG;
    int64_t planes, n_in, n_out;
    if (!mul3(N, C, 1, &planes) || !mul3(planes, H, W, &n_in) || !mul3(planes, Ho, Wo, &n_out))
        return SWS_ERR_INVALID_ARG;
    if (H * W > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (planes == 0) return SWS_OK;
    if (!x || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_pool2d_16((int)op, (int)dtype, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, scale,
                                          (hipStream_t)stream));
}

sws_status sws_pool2d_ex(sws_op op, const float *x, float *y, int64_t N, int64_t C, int64_t H, int64_t W,
                         int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t pad_top, int32_t pad_left,
                         int32_t pad_bottom, int32_t pad_right, sws_divisor divisor, float scale, sws_stream_t stream)
{
    if (!valid_op((int)op) || N < 0 || C < 0 || H < 1 || W < 1) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1) return SWS_ERR_INVALID_ARG;
    if (pad_top < 0 || pad_left < 0 || pad_bottom < 0 || pad_right < 0) return SWS_ERR_INVALID_ARG;
    if (pad_top >= kh || pad_bottom >= kh || pad_left >= kw || pad_right >= kw) return SWS_ERR_INVALID_ARG;
    if (divisor != SWS_DIV_SCALE && divisor != SWS_DIV_REAL_CELLS) return SWS_ERR_INVALID_ARG;
    if (H > kMaxDim || W > kMaxDim) return SWS_ERR_INVALID_ARG;
    const int64_t He = H + pad_top + pad_bottom, We = W + pad_left + pad_right;
    if (kh > He || kw > We) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = (He - kh) / sh + 1, Wo = (We - kw) / sw + 1;
    int64_t planes, n_in, n_out;
    if (!mul3(N, C, 1, &planes) || !mul3(planes, H, W, &n_in) || !mul3(planes, Ho, Wo, &n_out))
        return SWS_ERR_INVALID_ARG;
    if (H * W > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (planes == 0) return SWS_OK;
    if (!x || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_pool2d((int)op, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, pad_top, pad_left, scale,
                                       divisor == SWS_DIV_REAL_CELLS ? 1 : 0, (hipStream_t)stream));
}

sws_status sws_pool2d_padded(sws_op op, const float *x, float *y, int64_t N, int64_t C, int64_t H, int64_t W,
                             int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t pad_top, int32_t pad_left,
                             int32_t pad_bottom, int32_t pad_right, sws_pad_mode mode, float scale, sws_stream_t stream)
{
    if (!valid_op((int)op) || N < 0 || C < 0 || H < 1 || W < 1) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1) return SWS_ERR_INVALID_ARG;
    if (pad_top < 0 || pad_left < 0 || pad_bottom < 0 || pad_right < 0) return SWS_ERR_INVALID_ARG;
    if ((int)mode < SWS_PAD_IDENTITY || (int)mode > SWS_PAD_SHRINK) return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_SHRINK && (pad_top >= kh || pad_bottom >= kh || pad_left >= kw || pad_right >= kw))
        return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_MIRROR && (pad_top > H - 1 || pad_bottom > H - 1 || pad_left > W - 1 || pad_right > W - 1))
        return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_PERIODIC && (pad_top > H || pad_bottom > H || pad_left > W || pad_right > W))
        return SWS_ERR_INVALID_ARG;
    const int64_t He = H + pad_top + pad_bottom, We = W + pad_left + pad_right;
    if (He > kMaxDim || We > kMaxDim) return SWS_ERR_INVALID_ARG;
    if (kh > He || kw > We) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = (He - kh) / sh + 1, Wo = (We - kw) / sw + 1;
    int64_t planes, n_in, n_out;
    if (!mul3(N, C, 1, &planes) || !mul3(planes, H, W, &n_in) || !mul3(planes, Ho, Wo, &n_out))
        return SWS_ERR_INVALID_ARG;
    if (He * We > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (planes == 0) return SWS_OK;
    if (!x || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_pool2d_padded((int)op, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, pad_top, pad_left,
                                               pad_bottom, pad_right, (int)mode, scale, (hipStream_t)stream));
}

sws_status sws_conv1d(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L,
                      int64_t Cout, int32_t k, int32_t stride, int32_t pad, int32_t dilation,
                      int32_t groups, sws_stream_t stream)
{
    if (B < 0 || Cin < 1 || L < 0 || Cout < 1 || k < 1 || stride < 1 || pad < 0 || dilation < 1 || groups < 1)
        return SWS_ERR_INVALID_ARG;
    if (Cin % groups || Cout % groups || L > kMaxDim || Cin > kMaxDim || Cout > kMaxDim)
        return SWS_ERR_INVALID_ARG;
    const int64_t Lo = sws_out_len(L, k, stride, pad, dilation);
    if (Lo < 1) return SWS_ERR_INVALID_ARG;
    int64_t n_in, n_out, n_w;
    if (!mul3(B, Cin, L, &n_in) || !mul3(B, Cout, Lo, &n_out) || !mul3(Cout, Cin / groups, k, &n_w))
        return SWS_ERR_INVALID_ARG;
    if (B == 0) return SWS_OK;
    if (!x || !wgt || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_conv1d(x, wgt, y, B, Cin, L, Cout, Lo, k, stride, pad, dilation, groups,
                                       (hipStream_t)stream));
}

sws_status sws_conv1d_padded(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L,
                             int64_t Cout, int32_t k, int32_t stride, int32_t pad_left, int32_t pad_right,
                             int32_t dilation, int32_t groups, sws_pad_mode mode, sws_stream_t stream)
{
    if (B < 0 || Cin < 1 || L < 1 || Cout < 1 || k < 1 || stride < 1 || pad_left < 0 || pad_right < 0 || dilation < 1 ||
        groups < 1)
        return SWS_ERR_INVALID_ARG;
    if ((int)mode < SWS_PAD_IDENTITY || (int)mode > SWS_PAD_EDGE) return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_MIRROR && (pad_left > L - 1 || pad_right > L - 1)) return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_PERIODIC && (pad_left > L || pad_right > L)) return SWS_ERR_INVALID_ARG;
    const int64_t Le = L + pad_left + pad_right;
    if (Cin % groups || Cout % groups || Le > kMaxDim || Cin > kMaxDim || Cout > kMaxDim) return SWS_ERR_INVALID_ARG;
    const int64_t span = (int64_t)dilation * (k - 1) + 1;
    if (span > Le) return SWS_ERR_INVALID_ARG;
    const int64_t Lo = (Le - span) / stride + 1;
    int64_t n_in, n_out, n_w;
    if (!mul3(B, Cin, L, &n_in) || !mul3(B, Cout, Lo, &n_out) || !mul3(Cout, Cin / groups, k, &n_w))
        return SWS_ERR_INVALID_ARG;
    if (B == 0) return SWS_OK;
    if (!x || !wgt || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_conv1d_padded(x, wgt, y, B, Cin, L, Cout, Lo, k, stride, pad_left, pad_right, dilation,
                                               groups, (int)mode, (hipStream_t)stream));
}

sws_status sws_conv1d_16(sws_dtype dtype, const void *x, const float *wgt, void *y, int64_t B, int64_t Cin, int64_t L,
                         int64_t Cout, int32_t k, int32_t stride, int32_t pad, int32_t dilation, int32_t groups,
                         sws_stream_t stream)
{
    if (dtype != SWS_DTYPE_BF16 && dtype != SWS_DTYPE_F16) return SWS_ERR_INVALID_ARG;
    if (B < 0 || Cin < 1 || L < 0 || Cout < 1 || k < 1 || stride < 1 || pad < 0 || dilation < 1 || groups < 1)
        return SWS_ERR_INVALID_ARG;
    if (Cin % groups || Cout % groups || L > kMaxDim || Cin > kMaxDim || Cout > kMaxDim)
        return SWS_ERR_INVALID_ARG;
    const int64_t Lo = sws_out_len(L, k, stride, pad, dilation);
    if (Lo < 1) return SWS_ERR_INVALID_ARG;
    int64_t n_in, n_out, n_w;
    if (!mul3(B, Cin, L, &n_in) || !mul3(B, Cout, Lo, &n_out) || !mul3(Cout, Cin / groups, k, &n_w))
        return SWS_ERR_INVALID_ARG;
    if (B == 0) return SWS_OK;
    if (!x || !wgt || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_conv1d_16((int)dtype, x, wgt, y, B, Cin, L, Cout, Lo, k, stride, pad, dilation, groups,
                                          (hipStream_t)stream));
}

namespace {

// Shared argument checks of the convolution and its adjoints; *Lo receives the output length.
sws_status check_conv1d(int64_t B, int64_t Cin, int64_t L, int64_t Cout, int32_t k, int32_t stride, int32_t pad,
                        int32_t dilation, int32_t groups, int64_t *Lo)
{
    if (B < 0 || Cin < 1 || L < 0 || Cout < 1 || k < 1 || stride < 1 || pad < 0 || dilation < 1 || groups < 1)
        return SWS_ERR_INVALID_ARG;
    if (Cin % groups || Cout % groups || L > kMaxDim || Cin > kMaxDim || Cout > kMaxDim)
        return SWS_ERR_INVALID_ARG;
    *Lo = sws_out_len(L, k, stride, pad, dilation);
    if (*Lo < 1) return SWS_ERR_INVALID_ARG;
    int64_t n_in, n_out, n_w;
    if (!mul3(B, Cin, L, &n_in) || !mul3(B, Cout, *Lo, &n_out) || !mul3(Cout, Cin / groups, k, &n_w))
        return SWS_ERR_INVALID_ARG;
    return SWS_OK;
}

}  // namespace

sws_status sws_conv1d_grad_input(const float *gy, const float *wgt, float *gx, int64_t B, int64_t Cin, int64_t L,
                                 int64_t Cout, int32_t k, int32_t stride, int32_t pad, int32_t dilation,
                                 int32_t groups, sws_stream_t stream)
{
    int64_t Lo;
    const sws_status st = check_conv1d(B, Cin, L, Cout, k, stride, pad, dilation, groups, &Lo);
    if (st != SWS_OK) return st;
    if (B == 0) return SWS_OK;
    if (!gy || !wgt || !gx) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_conv1d_grad_input(gy, wgt, gx, B, Cin, L, Cout, Lo, k, stride, pad, dilation, groups,
                                                  (hipStream_t)stream));
}

sws_status sws_conv1d_grad_weight(const float *x, const float *gy, float *gw, int64_t B, int64_t Cin, int64_t L,
                                  int64_t Cout, int32_t k, int32_t stride, int32_t pad, int32_t dilation,
                                  int32_t groups, sws_stream_t stream)
{
    int64_t Lo;
    const sws_status st = check_conv1d(B, Cin, L, Cout, k, stride, pad, dilation, groups, &Lo);
    if (st != SWS_OK) return st;
    if (!gw || (B > 0 && (!x || !gy))) return SWS_ERR_INVALID_ARG;      // with no images gw is all zeros
    return SWS_LAUNCH(sws::launch_conv1d_grad_weight(x, gy, gw, B, Cin, L, Cout, Lo, k, stride, pad, dilation, groups,
                                                   (hipStream_t)stream));
}

namespace {

sws_status check_conv2d(int64_t N, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int32_t kh, int32_t kw, int32_t sh,
                        int32_t sw, int32_t ph, int32_t pw, int64_t *Ho, int64_t *Wo)
{
    if (N < 0 || Cin < 1 || H < 0 || W < 0 || Cout < 1) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return SWS_ERR_INVALID_ARG;
    if (H > kMaxDim || W > kMaxDim || Cin > kMaxDim || Cout > kMaxDim) return SWS_ERR_INVALID_ARG;
    *Ho = sws_out_len(H, kh, sh, ph, 1);
    *Wo = sws_out_len(W, kw, sw, pw, 1);
    if (*Ho < 1 || *Wo < 1) return SWS_ERR_INVALID_ARG;
    int64_t t, n_in, n_out, n_w;
    if (!mul3(N, Cin, H, &t) || !mul3(t, W, 1, &n_in)) return SWS_ERR_INVALID_ARG;
    if (!mul3(N, Cout, *Ho, &t) || !mul3(t, *Wo, 1, &n_out)) return SWS_ERR_INVALID_ARG;
    if (!mul3(Cout, Cin, (int64_t)kh * kw, &n_w)) return SWS_ERR_INVALID_ARG;
    if (H * W > kMaxDim || *Ho * *Wo > kMaxDim || n_w > kMaxDim) return SWS_ERR_UNSUPPORTED;
    return SWS_OK;
}

}  // namespace

sws_status sws_conv2d_grad_input(const float *gy, const float *wgt, float *gx, int64_t N, int64_t Cin, int64_t H,
                                 int64_t W, int64_t Cout, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph,
                                 int32_t pw, sws_stream_t stream)
{
    int64_t Ho, Wo;
    const sws_status st = check_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, &Ho, &Wo);
    if (st != SWS_OK) return st;
    if (N == 0) return SWS_OK;
    if (!gy || !wgt || !gx) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_conv2d_grad_input(gy, wgt, gx, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, ph, pw,
                                                  (hipStream_t)stream));
}

sws_status sws_conv2d_grad_weight(const float *x, const float *gy, float *gw, int64_t N, int64_t Cin, int64_t H,
                                  int64_t W, int64_t Cout, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph,
                                  int32_t pw, sws_stream_t stream)
{
    int64_t Ho, Wo;
    const sws_status st = check_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, &Ho, &Wo);
    if (st != SWS_OK) return st;
    if (!gw || (N > 0 && (!x || !gy))) return SWS_ERR_INVALID_ARG;      // with no images gw is all zeros
    return SWS_LAUNCH(sws::launch_conv2d_grad_weight(x, gy, gw, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, ph, pw,
                                                   (hipStream_t)stream));
}

sws_status sws_conv2d(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                      int64_t W, int64_t Cout, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph,
                      int32_t pw, sws_stream_t stream)
{
    if (N < 0 || Cin < 1 || H < 0 || W < 0 || Cout < 1) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return SWS_ERR_INVALID_ARG;
    if (H > kMaxDim || W > kMaxDim || Cin > kMaxDim || Cout > kMaxDim) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = sws_out_len(H, kh, sh, ph, 1), Wo = sws_out_len(W, kw, sw, pw, 1);
    if (Ho < 1 || Wo < 1) return SWS_ERR_INVALID_ARG;
    int64_t t, n_in, n_out, n_w;
    if (!mul3(N, Cin, H, &t) || !mul3(t, W, 1, &n_in)) return SWS_ERR_INVALID_ARG;
    if (!mul3(N, Cout, Ho, &t) || !mul3(t, Wo, 1, &n_out)) return SWS_ERR_INVALID_ARG;
    if (!mul3(Cout, Cin, (int64_t)kh * kw, &n_w)) return SWS_ERR_INVALID_ARG;
    if (H * W > kMaxDim || Ho * Wo > kMaxDim || n_w > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (N == 0) return SWS_OK;
    if (!x || !wgt || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_conv2d(x, wgt, y, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, ph, pw,
                                       (hipStream_t)stream));
}

sws_status sws_conv2d_padded(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                             int64_t W, int64_t Cout, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t pad_top,
                             int32_t pad_left, int32_t pad_bottom, int32_t pad_right, sws_pad_mode mode,
                             sws_stream_t stream)
{
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1) return SWS_ERR_INVALID_ARG;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1) return SWS_ERR_INVALID_ARG;
    if (pad_top < 0 || pad_left < 0 || pad_bottom < 0 || pad_right < 0) return SWS_ERR_INVALID_ARG;
    if ((int)mode < SWS_PAD_IDENTITY || (int)mode > SWS_PAD_EDGE) return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_MIRROR && (pad_top > H - 1 || pad_bottom > H - 1 || pad_left > W - 1 || pad_right > W - 1))
        return SWS_ERR_INVALID_ARG;
    if (mode == SWS_PAD_PERIODIC && (pad_top > H || pad_bottom > H || pad_left > W || pad_right > W))
        return SWS_ERR_INVALID_ARG;
    const int64_t He = H + pad_top + pad_bottom, We = W + pad_left + pad_right;
    if (He > kMaxDim || We > kMaxDim || Cin > kMaxDim || Cout > kMaxDim) return SWS_ERR_INVALID_ARG;
    if (kh > He || kw > We) return SWS_ERR_INVALID_ARG;
    const int64_t Ho = (He - kh) / sh + 1, Wo = (We - kw) / sw + 1;
    int64_t t, n_in, n_out, n_w;
    if (!mul3(N, Cin, H, &t) || !mul3(t, W, 1, &n_in)) return SWS_ERR_INVALID_ARG;
    if (!mul3(N, Cout, Ho, &t) || !mul3(t, Wo, 1, &n_out)) return SWS_ERR_INVALID_ARG;
    if (!mul3(Cout, Cin, (int64_t)kh * kw, &n_w)) return SWS_ERR_INVALID_ARG;
    if (He * We > kMaxDim || n_w > kMaxDim) return SWS_ERR_UNSUPPORTED;
    if (N == 0) return SWS_OK;
    if (!x || !wgt || !y) return SWS_ERR_INVALID_ARG;
    return SWS_LAUNCH(sws::launch_conv2d_padded(x, wgt, y, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, pad_top, pad_left,
                                               pad_bottom, pad_right, (int)mode, (hipStream_t)stream));
}

}  // extern "C"
