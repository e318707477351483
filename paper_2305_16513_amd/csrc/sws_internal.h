// Internal declarations shared by the libsws translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "sws.h"
#include "sws_dev.h"

namespace sws {

// Measurement knobs set through sws_set_option(); 0 means "choose automatically".  Host-side only;
// every launcher reads a knob once (relaxed atomic load through Knob's conversion).
struct Knob {
    std::atomic<int> v{0};
    operator int() const { return v.load(std::memory_order_relaxed); }
    Knob &operator=(int x) { v.store(x, std::memory_order_relaxed); return *this; }
};
struct Options {
    Knob slide_variant;
    Knob slide_chunk;
    Knob slide_group;
    Knob pool2d_variant;
    Knob conv1d_variant;
    Knob conv2d_variant;
    Knob copy_variant;
};
extern Options g_opt;

// A launcher's answer when its kernel does not cover the request (the caller then tries the next
// kernel); never a code the HIP runtime returns.
constexpr hipError_t kNotTaken = (hipError_t)2047;

constexpr int kWave = 64;    // CDNA wavefront width
constexpr int kXcd = 8;      // XCDs (separate L2s) on MI355X

typedef float v4f __attribute__((ext_vector_type(4)));
typedef v4f v4f_u __attribute__((aligned(4)));     // 16-byte access at 4-byte alignment
typedef float v2f __attribute__((ext_vector_type(2)));

// The operator (+) of the sliding window sum, with its identity element.  `a` is always
// the older (left) operand so the kernels stay valid for non-commutative operators.
template <int OP> struct Op;
template <> struct Op<SWS_OP_ADD> {
    static __device__ __forceinline__ float id() { return 0.0f; }
    static __device__ __forceinline__ float f(float a, float b) { return a + b; }
};
template <> struct Op<SWS_OP_MAX> {
    static __device__ __forceinline__ float id() { return -__builtin_huge_valf(); }
    static __device__ __forceinline__ float f(float a, float b) { return __builtin_fmaxf(a, b); }
};
template <> struct Op<SWS_OP_MIN> {
    static __device__ __forceinline__ float id() { return __builtin_huge_valf(); }
    static __device__ __forceinline__ float f(float a, float b) { return __builtin_fminf(a, b); }
};

// N sliding windows of K consecutive elements at stride 1, out[j] = in[j] (+) ... (+) in[j + K - 1], from what they
// share: the elements N - 1 .. K - 1 lie in all of them and are combined once; window j puts the rest of the head
// in front (in[j] .. in[N - 2]) and the start of the tail behind (in[K] .. in[K + j - 1]) — Section 3's suffix /
// prefix split between registers.  K + 3N - 6 operations instead of N (K - 1); operand order is kept.
// F(a, b) combines two elements (floats, or vectors of columns).
template <int K, int N, typename E, typename F>
__device__ __forceinline__ void windows_shared(const E *in, E *out, F f)
{
    // (windows of fewer than five elements are combined left to right as Eq. 3 writes them: nothing to gain, and the
    // strided kernels, which share nothing, then give the same bits)
    if constexpr (N < 2 || K < N || K < 5 || K + 3 * N - 6 >= N * (K - 1)) {
#pragma unroll
        for (int j = 0; j < N; ++j) {
            E acc = in[j];
#pragma unroll
            for (int b = 1; b < K; ++b) acc = f(acc, in[j + b]);
            out[j] = acc;
        }
    } else {
        E core = in[N - 1];
#pragma unroll
        for (int b = N; b < K; ++b) core = f(core, in[b]);
        E head[N - 1], tail[N - 1];                  // head[j] = in[j] .. in[N-2];  tail[j] = in[K] .. in[K+j]
        head[N - 2] = in[N - 2];
#pragma unroll
        for (int j = N - 3; j >= 0; --j) head[j] = f(in[j], head[j + 1]);
        tail[0] = in[K];
#pragma unroll
        for (int j = 1; j < N - 1; ++j) tail[j] = f(tail[j - 1], in[K + j]);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            E acc = j < N - 1 ? f(head[j], core) : core;
            out[j] = j > 0 ? f(acc, tail[j - 1]) : acc;
        }
    }
}

// Boundary conditions of a row extended by pad_left virtual elements in front (and more behind):
// the physical index that virtual element e stands for, or -1 for the operator's identity.
// mode: SWS_PAD_IDENTITY, SWS_PAD_MIRROR (x[-i] = x[i]), SWS_PAD_PERIODIC (x[-i] = x[len-i]),
// SWS_PAD_EDGE (the end element repeated), SWS_PAD_SHRINK (identity; the caller rescales ADD results).
// The caller keeps e inside the extended row.
__device__ __forceinline__ int pad_src(int e, int len, int pad_left, int mode)
{
    const int p = e - pad_left;
    if (p >= 0 && p < len) return p;
    if (mode == SWS_PAD_IDENTITY || mode == SWS_PAD_SHRINK) return -1;
    if (mode == SWS_PAD_MIRROR) return p < 0 ? -p : 2 * (len - 1) - p;
    if (mode == SWS_PAD_PERIODIC) return p < 0 ? p + len : p - len;
    return p < 0 ? 0 : len - 1;
}

// Workgroups are dealt round-robin to the 8 XCDs.  This maps blockIdx so that each XCD
// (one L2) walks a contiguous range of work units, keeping a tile's halo re-read in the
// L2 that fetched it.  Returns an id in [0, n_units) or -1 for the padding blocks.
__device__ __forceinline__ int64_t xcd_unit(int64_t n_units)
{
    const int64_t b = blockIdx.x;
    const int64_t per = (n_units + kXcd - 1) / kXcd;
    const int64_t u = (b % kXcd) * per + b / kXcd;
    return (b / kXcd < per && u < n_units) ? u : -1;
}
// Kernels pull every row's tile origins back by (r * lo) mod line elements so that stores start on
// 64-byte lines.  The largest such shift over all rows r: line - gcd(lo mod line, line), i.e. 0 when
// lo is a multiple of the line (then no row needs an extra tile).
inline int max_origin_shift(int64_t lo, int line)
{
    int a = (int)(lo % line), b = line;
    while (a) { const int t = b % a; b = a; a = t; }
    return line - b;
}

// Compute units of the current device (256 on MI355X), asked once.
int device_cus();

inline int64_t xcd_grid(int64_t n_units) { return ((n_units + kXcd - 1) / kXcd) * kXcd; }

hipError_t launch_copy(const float *src, float *dst, int64_t n, hipStream_t s);
hipError_t launch_slide1d(int op, const float *x, float *y, int64_t rows, int64_t len, int32_t w,
                          int32_t pad_left, int32_t pad_right, int pad_mode, float scale, hipStream_t s);
hipError_t launch_slide1d_16(int op, int dtype, const void *x, void *y, int64_t rows, int64_t len, int32_t w,
                             float scale, hipStream_t s);
// Generic-operator kernels (slide_generic.hip): the pair operator, and +, max, min as a cross-check.
hipError_t launch_slide1d_pair(const float *u, const float *v, float *yu, float *yv, int64_t rows, int64_t len,
                               int32_t w, hipStream_t s);
// Medium windows (slide1d_reg_min_w() .. slide1d_reg_max_w()) on plain rows: one 256-element strip per
// single-wavefront workgroup, held in registers, whole lanes summed across the wavefront (slide_reg.hip).
// kNotTaken: not its case, nothing launched.
int slide1d_reg_min_w();
int slide1d_reg_max_w();
hipError_t launch_slide1d_reg(int op, const float *x, float *y, int64_t rows, int len, int lo, int w, float scale,
                              hipStream_t s);

// Short rows, windows up to slide1d_rows_max_w(): four outputs per lane from shifted 128-bit loads,
// several rows per wavefront.  hipErrorInvalidValue: not taken (w or grid beyond its reach).
// 2-D pooling on planes of a few hundred elements: several whole planes per workgroup through LDS.
// *taken = false: not its case (the caller goes on to the other kernels).
hipError_t launch_pool2d_small(int op, const float *x, float *y, int64_t planes, int H, int W, int Ho, int Wo, int kh,
                               int kw, int sh, int sw, int ph, int pw, float scale, int div_valid, hipStream_t s,
                               bool *taken);
int slide1d_rows_max_w();
hipError_t launch_slide1d_rows(int op, const float *x, float *y, int64_t rows, int len, int lo, int32_t w, float scale,
                               bool padded, int pad_left, int pad_mode, hipStream_t s);
// Windows longer than a wave tile in one pass (slide_long.hip): w > 256, plain rows or rows extended by a boundary
// rule other than the shrinking window; kNotTaken otherwise.
hipError_t launch_slide1d_long(int op, const float *x, float *y, int64_t rows, int len, int lo, int w, float scale,
                               bool padded, int pad_left, int pad_mode, int lv, hipStream_t s);
hipError_t launch_slide1d_long_16(int op, int dtype, const void *x, void *y, int64_t rows, int len, int lo, int w,
                                  float scale, hipStream_t s);
hipError_t launch_slide1d_generic(int op, const float *x, float *y, int64_t rows, int64_t len, int32_t w, float scale,
                                  hipStream_t s);
hipError_t launch_pool2d(int op, const float *x, float *y, int64_t planes, int64_t H, int64_t W,
                         int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                         int32_t ph, int32_t pw, float scale, int div_valid, hipStream_t s);
// Pooling over planes extended by a boundary rule on four sides (pool2d_padded.hip).
hipError_t launch_pool2d_padded(int op, const float *x, float *y, int64_t planes, int64_t H, int64_t W, int64_t Ho,
                                int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t pt, int32_t pl,
                                int32_t pb, int32_t pr, int mode, float scale, hipStream_t s);
hipError_t launch_maxpool2d_grad(const float *x, const float *gy, float *gx, int64_t planes, int64_t H, int64_t W,
                                 int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph,
                                 int32_t pw, hipStream_t s);
hipError_t launch_avgpool2d_grad(const float *gy, float *gx, int64_t planes, int64_t H, int64_t W, int64_t Ho, int64_t Wo,
                                 int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, int div_real,
                                 float scale, hipStream_t s);
// Row-streaming adjoints of 3 x 3 pooling (pool_grad_rows.hip); *taken = false: shape not covered, nothing launched.
hipError_t launch_maxpool2d_grad_rows(const float *x, const float *gy, float *gx, int64_t planes, int H, int W, int Ho,
                                      int Wo, int kh, int kw, int sh, int sw, int ph, int pw, hipStream_t s, bool *taken);
hipError_t launch_avgpool2d_grad_rows(const float *gy, float *gx, int64_t planes, int H, int W, int Ho, int Wo, int kh,
                                      int kw, int sh, int sw, int ph, int pw, float scale, hipStream_t s, bool *taken);
hipError_t launch_pool2d_16(int op, int dtype, const void *x, void *y, int64_t planes, int64_t H, int64_t W, int64_t Ho,
                            int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                            float scale, hipStream_t s);
hipError_t launch_conv1d(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L,
                         int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad,
                         int32_t dilation, int32_t groups, hipStream_t s, int wadj = 0, bool *taken = nullptr);
// Rows extended by pad_left / pad_right elements under a boundary rule (mirror, periodic, edge; conv1d.hip).
hipError_t launch_conv1d_padded(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L,
                                int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad_left, int32_t pad_right,
                                int32_t dilation, int32_t groups, int mode, hipStream_t s);
// Dense 1-D layers of 32 / 64 input channels on the bf16 matrix cores with split fp32 operands (conv1d_split.hip);
// *taken = false: not one of its shapes, nothing launched.
hipError_t launch_conv1d_split(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L, int64_t Cout,
                               int64_t Lo, int32_t k, int32_t pad, hipStream_t s, bool *taken);
// 16-bit storage (conv1d16.hip): x, y bf16 / fp16, taps fp32.
hipError_t launch_conv1d_16(int dtype, const void *x, const float *wgt, void *y, int64_t B, int64_t Cin, int64_t L,
                            int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad, int32_t dilation,
                            int32_t groups, hipStream_t s);
// Adjoints of the 1-D convolution (conv_grad.hip).
hipError_t launch_conv1d_grad_input(const float *gy, const float *wgt, float *gx, int64_t B, int64_t Cin, int64_t L,
                                    int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad,
                                    int32_t dilation, int32_t groups, hipStream_t s);
hipError_t launch_conv1d_grad_weight(const float *x, const float *gy, float *gw, int64_t B, int64_t Cin, int64_t L,
                                     int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad,
                                     int32_t dilation, int32_t groups, hipStream_t s);
hipError_t launch_conv2d_grad_input(const float *gy, const float *wgt, float *gx, int64_t N, int64_t Cin, int64_t H,
                                    int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh,
                                    int32_t sw, int32_t ph, int32_t pw, hipStream_t s);
hipError_t launch_conv2d_grad_weight(const float *x, const float *gy, float *gw, int64_t N, int64_t Cin, int64_t H,
                                     int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh,
                                     int32_t sw, int32_t ph, int32_t pw, hipStream_t s);
hipError_t launch_conv2d(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                         int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw,
                         int32_t sh, int32_t sw, int32_t ph, int32_t pw, hipStream_t s);

// Planes extended on four sides under a boundary rule (conv2d_padded.hip).
hipError_t launch_conv2d_padded(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H, int64_t W,
                                int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                                int32_t pt, int32_t pl, int32_t pb, int32_t pr, int mode, hipStream_t s);

// Dense grad-weight on the bf16 matrix cores with split fp32 operands (conv_gw_split.hip): 3 x 3, horizontal
// stride 1, channel counts in multiples of 32; gw must hold zeros; *taken = false: not its case, nothing launched.
hipError_t launch_conv2d_gw_split(const float *x, const float *gy, float *gw, int64_t N, int64_t Cin, int64_t H, int64_t W,
                                  int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                                  int32_t ph, int32_t pw, hipStream_t s, bool *taken);

// The same for kernels one row high (the 1-D convolution; 1 x k layers): rows = images * RH rows of L inputs / Lo outputs.
hipError_t launch_conv1d_gw_split(const float *x, const float *gy, float *gw, int64_t rows, int RH, int64_t Cin, int64_t L,
                                  int64_t Cout, int64_t Lo, int32_t k, int32_t pad, int64_t x_cs, int64_t gy_cs, hipStream_t s,
                                  bool *taken);

// Matrix-core convolution (conv_mfma.hip); *taken = false: shape not covered, nothing launched.
hipError_t launch_conv2d_mfma(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                              int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh,
                              int32_t sw, int32_t ph, int32_t pw, int32_t dh, int32_t dw, hipStream_t s,
                              bool *taken, int wadj = 0);
// Weight-stationary streaming kernel (conv_stream.hip): 64 input channels, 3 x 3 on narrow images and
// 1 x 3 on 1-D rows, stride 1; *taken = false: not its case, nothing launched.
hipError_t launch_conv2d_stream(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H, int64_t W,
                                int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t ph, int32_t pw,
                                hipStream_t s, bool *taken, int wadj);
// Strided adjoint with respect to the input, one stride-1 launch chain per output phase; phases no
// tap reaches are NOT written (the caller clears gx first when kh < sh or kw < sw).
hipError_t launch_conv2d_grad_input_phases(const float *gy, const float *wgt, float *gx, int64_t N, int64_t Cin,
                                           int64_t H, int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh,
                                           int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, hipStream_t s,
                                           bool *taken);

// Direct-evaluation fallbacks (naive_kernels.hip).
hipError_t launch_slide1d_naive(int op, const float *x, float *y, int64_t rows, int64_t len, int32_t w,
                                int32_t pad_left, int32_t pad_right, int pad_mode, float scale, hipStream_t s);
hipError_t launch_pool2d_naive(int op, const float *x, float *y, int64_t planes, int64_t H, int64_t W,
                               int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                               int32_t ph, int32_t pw, float scale, int div_valid, hipStream_t s);
hipError_t launch_conv1d_naive(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin,
                               int64_t L, int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad,
                               int32_t dilation, int32_t groups, hipStream_t s, int mode = SWS_PAD_IDENTITY);
hipError_t launch_conv2d_naive(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin,
                               int64_t H, int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh,
                               int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, hipStream_t s);

}  // namespace sws
