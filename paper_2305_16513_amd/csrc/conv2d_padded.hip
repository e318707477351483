// sws_conv2d_padded — the 2-D convolution over planes extended on four sides by a boundary condition of
// Section 3 (mirror, periodic, repeated edge) instead of zeros.
//
// A convolution is linear in its input, so the extended plane splits into the plane itself on a field
// of zeros plus the virtual cells alone:  y = conv(x, zero padding) + (the terms whose input cell is
// virtual).  The first part is the library's tuned zero-padding convolution, untouched.  The second
// part exists only for the outputs whose window leaves the plane — a frame of a few rows and columns
// round the output plane (7 % of a 56 x 56 plane for 3 x 3) — and only for the taps that land
// outside; the border kernel below adds it into y: a small matrix product per 64 border outputs over
// only the taps that are virtual for one of them, the input cell read from where the rule points.  Unequal pads on opposite sides, and any geometry with the knob conv2d_variant = 1, are
// evaluated directly through the same index rule.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kCoPer = 64;                           // output channels per workgroup of the border kernel

// The frame: output rows [0, r0) and [r1, Ho) whole, and of the rows between them the columns [0, c0)
// and [c1, Wo).  Outputs inside [r0, r1) x [c0, c1) see real cells only.  The four sides are numbered one
// after the other, each rounded up to whole groups of 64, so that the 64 outputs of a workgroup lie on
// one side and share the taps that fall outside the plane.
struct Frame {
    int r0, r1, c0, c1;
    int nT, nB, nL, nR;                              // outputs on the top, bottom, left, right
    int gT, gB, gL, gR;                              // ... in groups of 64
};

// Slot q of the numbering -> (ho, wo); false: a slot of the rounding.
__device__ __forceinline__ bool frame_cell(const Frame &f, int Wo, int q, int *ho, int *wo)
{
    int i = q;
    if (i < 64 * f.gT) {
        if (i >= f.nT) return false;
        *ho = i / Wo; *wo = i - *ho * Wo;
        return true;
    }
    i -= 64 * f.gT;
    if (i < 64 * f.gB) {
        if (i >= f.nB) return false;
        const int r = i / Wo;
        *ho = f.r1 + r; *wo = i - r * Wo;
        return true;
    }
    i -= 64 * f.gB;
    const int rows = f.r1 - f.r0;
    if (i < 64 * f.gL) {
        if (i >= f.nL) return false;
        const int c = i / rows;
        *ho = f.r0 + (i - c * rows); *wo = c;
        return true;
    }
    i -= 64 * f.gL;
    if (i >= f.nR) return false;
    const int c = i / rows;
    *ho = f.r0 + (i - c * rows); *wo = f.c1 + c;
    return true;
}

// A workgroup: 64 border outputs of one image x 64 output channels, a chunk of 16 input channels at a
// time — a small matrix product  D[output][co] += X[output][(tap, ci)] * W[(tap, ci)][co]  on
// v_mfma_f32_32x32x2_f32, one 32 x 32 block of D per wavefront.  The taps that are virtual for at least
// one of the 64 outputs are taken four at a time: the input cells they meet (zero where the tap is real
// for that output: the zero-padding pass has it) and the matching weights are gathered into LDS, every
// load of a thread independent of the others, then each wavefront runs its block over them.  No sums
// across wavefronts, a fixed order of additions.
constexpr int kSlots = 4;                            // taps gathered together
constexpr int kCc = 16;                              // input channels per chunk
constexpr int kWp = kCoPer + 1;                      // pitch of a weight row in LDS (bank spread for the transposing writes)
typedef float v16f __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(kThreads) void conv2d_border_kernel(const float *__restrict__ x, const float *__restrict__ wgt,
                                                                 float *__restrict__ y, int Cin, int H, int W, int Cout,
                                                                 int Ho, int Wo, int kh, int kw, int sh, int sw, int pt,
                                                                 int pl, int mode, Frame f, int cgroups)
{
    __shared__ float lw[kSlots][kCc][kWp];           // weights  [tap slot][ci][co]
    __shared__ float xt[kSlots][kCc][kWave];         // inputs   [tap slot][ci][output]
    __shared__ int cpos[kWave];                      // ho * Wo + wo of the 64 outputs (-1: none)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t n = blockIdx.y / cgroups;
    const int co0 = (int)(blockIdx.y - n * cgroups) * kCoPer;
    const int q = blockIdx.x * kWave + lane;
    int ho = 0, wo = 0;
    const bool live = frame_cell(f, Wo, q, &ho, &wo);
    if (wave == 0) cpos[lane] = live ? ho * Wo + wo : -1;
    __syncthreads();
    const int plane = H * W;
    const float *xn = x + n * Cin * (int64_t)plane;
    const int ktaps = kh * kw;
    // the taps that leave the plane for one of the 64 outputs (the same set in all four wavefronts)
    uint64_t mask = 0;
    for (int t = 0; t < ktaps; ++t) {
        const int a = t / kw, b = t - a * kw;
        const int hr = ho * sh + a - pt, cr = wo * sw + b - pl;
        const bool virt = live && !(hr >= 0 && hr < H && cr >= 0 && cr < W);
        if (__builtin_amdgcn_ballot_w64(virt) != 0) mask |= 1ull << t;
    }
    const int l32 = lane & 31, half = lane >> 5;
    const int row0 = (wave & 1) * 32, col0 = (wave >> 1) * 32;      // my block of D: outputs row0.., channels col0..
    // staging roles: inputs — lane = output, wavefront = ci mod 4; weights — 16 lanes along ci, 16 along co
    const int w_ci = threadIdx.x & 15, w_co = threadIdx.x >> 4;
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    uint64_t m = mask;
    while (m != 0) {
        // the next four taps of the set: where each of them lands for my output
        int tap[kSlots], off[kSlots], ns = 0;
        bool virt[kSlots];
#pragma unroll
        for (int s = 0; s < kSlots; ++s) {
            tap[s] = 0; off[s] = 0; virt[s] = false;
            if (m != 0) {
                const int t = __builtin_ctzll(m);
                m &= m - 1;
                ns = s + 1;
                const int a = t / kw, b = t - a * kw;
                const int hr = ho * sh + a - pt, cr = wo * sw + b - pl;
                tap[s] = t;
                virt[s] = live && !(hr >= 0 && hr < H && cr >= 0 && cr < W);
                off[s] = virt[s] ? pad_src(ho * sh + a, H, pt, mode) * W + pad_src(wo * sw + b, W, pl, mode) : 0;
            }
        }
        float gx[kCc / 4][kSlots], gw[kCoPer / 16][kSlots];
        // a chunk's loads: inputs (lane = output, wavefront = ci mod 4) and weights (16 lanes along ci, 16 along co)
        auto gather = [&](int c0) {
            const int cc = Cin - c0 < kCc ? Cin - c0 : kCc;
#pragma unroll
            for (int j = 0; j < kCc / 4; ++j) {
                const int ci = wave + 4 * j;
                const float *xc = xn + (int64_t)(c0 + (ci < cc ? ci : 0)) * plane;
#pragma unroll
                for (int s = 0; s < kSlots; ++s) gx[j][s] = xc[off[s]];
            }
#pragma unroll
            for (int j = 0; j < kCoPer / 16; ++j) {
                const int co = co0 + w_co + 16 * j;
                const float *wr = wgt + ((int64_t)(co < Cout ? co : co0) * Cin + c0 + (w_ci < cc ? w_ci : 0)) * ktaps;
#pragma unroll
                for (int s = 0; s < kSlots; ++s) gw[j][s] = wr[tap[s]];
            }
        };
        gather(0);
        for (int c0 = 0; c0 < Cin; c0 += kCc) {
            const int cc = Cin - c0 < kCc ? Cin - c0 : kCc;      // input channels of this chunk
            __syncthreads();                                     // the previous chunk has been consumed
#pragma unroll
            for (int j = 0; j < kCc / 4; ++j)
#pragma unroll
                for (int s = 0; s < kSlots; ++s) xt[s][wave + 4 * j][lane] = (virt[s] && wave + 4 * j < cc) ? gx[j][s] : 0.0f;
#pragma unroll
            for (int j = 0; j < kCoPer / 16; ++j)
#pragma unroll
                for (int s = 0; s < kSlots; ++s)
                    lw[s][w_ci][w_co + 16 * j] = (co0 + w_co + 16 * j < Cout && w_ci < cc && s < ns) ? gw[j][s] : 0.0f;
            __syncthreads();
            if (c0 + kCc < Cin) gather(c0 + kCc);                // the next chunk's loads fly during the matrix work
#pragma unroll
            for (int s = 0; s < kSlots; ++s) {
                if (s >= ns) break;
#pragma unroll
                for (int ci = 0; ci < kCc; ci += 2) {            // rows beyond cc hold zeros
                    const float av = xt[s][ci + half][row0 + l32];
                    const float bv = lw[s][ci + half][col0 + l32];
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
                }
            }
        }
    }
    // register v of lane (l32, half) is output row0 + 8*(v/4) + 4*half + v%4, channel col0 + l32
    const int co = co0 + col0 + l32;
    if (co < Cout) {
        float *yc = y + (n * Cout + co) * (int64_t)Ho * Wo;
        float old[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {                           // all reads of y before the first write
            const int p = cpos[row0 + 8 * (v / 4) + 4 * half + (v % 4)];
            old[v] = yc[p >= 0 ? p : 0];
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int p = cpos[row0 + 8 * (v / 4) + 4 * half + (v % 4)];
            if (p >= 0) yc[p] = old[v] + acc[v];
        }
    }
}

// Direct evaluation through the index rule: one thread per output.
__global__ __launch_bounds__(kThreads) void conv2d_padded_naive_kernel(const float *__restrict__ x,
                                                                       const float *__restrict__ wgt,
                                                                       float *__restrict__ y, int64_t N, int Cin, int H,
                                                                       int W, int Cout, int Ho, int Wo, int kh, int kw,
                                                                       int sh, int sw, int pt, int pl, int mode)
{
    const int64_t total = N * (int64_t)Cout * Ho * Wo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int wo = (int)(o % Wo);
        const int ho = (int)((o / Wo) % Ho);
        const int co = (int)((o / ((int64_t)Wo * Ho)) % Cout);
        const int64_t n = o / ((int64_t)Wo * Ho * Cout);
        float acc = 0.0f;
        for (int ci = 0; ci < Cin; ++ci) {
            const float *xp = x + (n * Cin + ci) * (int64_t)H * W;
            const float *wp = wgt + ((int64_t)co * Cin + ci) * kh * kw;
            for (int a = 0; a < kh; ++a) {
                const int sr = pad_src(ho * sh + a, H, pt, mode);
                if (sr < 0) continue;
                for (int b = 0; b < kw; ++b) {
                    const int sc = pad_src(wo * sw + b, W, pl, mode);
                    if (sc >= 0) acc = fmaf(wp[a * kw + b], xp[(int64_t)sr * W + sc], acc);
                }
            }
        }
        y[o] = acc;
    }
}

// First output index whose window starts inside the plane, and one past the last whose window ends inside it.
void interior(int len, int k, int s, int pad, int lo, int *i0, int *i1)
{
    int a = (pad + s - 1) / s;
    int b = len - k + pad >= 0 ? (len - k + pad) / s + 1 : 0;
    if (a > lo) a = lo;
    if (b > lo) b = lo;
    if (b < a) b = a;
    *i0 = a;
    *i1 = b;
}

}  // namespace

hipError_t launch_conv2d_padded(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H, int64_t W,
                                int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                                int32_t pt, int32_t pl, int32_t pb, int32_t pr, int mode, hipStream_t s)
{
    const bool even = pt == pb && pl == pr;
    if (mode == SWS_PAD_IDENTITY && even) return launch_conv2d(x, wgt, y, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, pt, pl, s);
    const int64_t cgroups = (Cout + kCoPer - 1) / kCoPer;
    // the tap set of a workgroup is a 64-bit mask
    if (mode != SWS_PAD_IDENTITY && even && g_opt.conv2d_variant != 1 && N * cgroups <= 65535 && kh * (int64_t)kw <= 64) {
        const hipError_t e = launch_conv2d(x, wgt, y, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, pt, pl, s);
        if (e != hipSuccess) return e;
        Frame f;
        interior((int)H, kh, sh, pt, (int)Ho, &f.r0, &f.r1);
        interior((int)W, kw, sw, pl, (int)Wo, &f.c0, &f.c1);
        if (f.r1 == f.r0 || f.c1 == f.c0) {          // no output sees real cells only: every output is frame
            f.r0 = f.r1 = (int)Ho;
            f.c0 = 0;
            f.c1 = (int)Wo;
        }
        f.nT = f.r0 * (int)Wo;
        f.nB = ((int)Ho - f.r1) * (int)Wo;
        f.nL = (f.r1 - f.r0) * f.c0;
        f.nR = (f.r1 - f.r0) * ((int)Wo - f.c1);
        f.gT = (f.nT + 63) / 64; f.gB = (f.nB + 63) / 64; f.gL = (f.nL + 63) / 64; f.gR = (f.nR + 63) / 64;
        const int groups = f.gT + f.gB + f.gL + f.gR;
        if (groups == 0) return hipSuccess;
        hipLaunchKernelGGL(conv2d_border_kernel, dim3((unsigned)groups, (unsigned)(N * cgroups)),
                           dim3(kThreads), 0, s, x, wgt, y, (int)Cin, (int)H, (int)W, (int)Cout, (int)Ho, (int)Wo, kh, kw,
                           sh, sw, pt, pl, mode, f, (int)cgroups);
        return hipGetLastError();
    }
    const int64_t total = N * Cout * Ho * Wo;
    int64_t grid = (total + kThreads - 1) / kThreads;
    const int64_t cap = (int64_t)device_cus() * 32;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL(conv2d_padded_naive_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, x, wgt, y, N, (int)Cin,
                       (int)H, (int)W, (int)Cout, (int)Ho, (int)Wo, kh, kw, sh, sw, pt, pl, mode);
    return hipGetLastError();
}

}  // namespace sws
