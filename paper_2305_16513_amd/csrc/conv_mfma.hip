// Dense-channel convolution (Section 2.5) on the fp32 matrix cores, without im2col.
//
// The convolution is evaluated as a sliding sum over taps of shifted, weighted input
// rows:  Y[co, p] = sum_tap  W_tap[co, :] . X[:, p + shift(tap)].  For each tap the inner
// product over input channels is a small dense matrix product (C_out x C_in times
// C_in x positions) — the "small matrix multiplication" form the paper's conclusion asks
// for — and runs on v_mfma_f32_32x32x2_f32.  The input tile (with its kh-1 / kw-1 halo and
// zero padding) is staged ONCE in LDS per block of input channels and is read at kh*kw
// shifted offsets; the column matrix of im2col never exists.
//
// Tile geometry.  A workgroup (4 wavefronts) computes 64 output channels for NP = 128*NBW
// output positions of one image.  Positions are numbered p = r*Wt + c over a tile of TR
// rows with pitch Wt = TC + kw - 1 (the staged row length), so that the input of tap
// (a, b) for position p is simply LDS element p + a*Wt + b: a shifted read of the same
// buffer.  Columns c >= TC are computed and thrown away.
//
// MFMA operand layout (32x32x2, wave64): lane l supplies A[i = l%32][k = l/32] and
// B[k = l/32][j = l%32]; accumulator register v of lane l holds
// D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kCoTile = 64;                           // output channels per workgroup

typedef float v16f __attribute__((ext_vector_type(16)));

struct ConvGeom {
    int Cin, H, W, Cout, Ho, Wo, kh, kw, ph, pw;
    int TR, TC, Wt, NRows, CP;                        // tile rows / cols, staged pitch, staged rows, channel pitch
    int tiles_r, tiles_c, co_blocks;
};

template <int NBW, int CIB>
__global__ __launch_bounds__(kThreads) void conv2d_mfma_kernel(const float *__restrict__ x,
                                                               const float *__restrict__ wgt,
                                                               float *__restrict__ y, ConvGeom g,
                                                               int64_t n_units)
{
    constexpr int KP = CIB / 2;                       // k-pairs (MFMA steps) per tap and channel block
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *Xl = lds;                                  // [CIB][CP] staged inputs
    float *Wl = lds + CIB * g.CP;                     // [tap][KP][2][64] weights, co fastest

    const int64_t unit = xcd_unit(n_units);
    if (unit < 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;

    // unit -> (image, co block, tile row, tile col)
    int64_t u = unit;
    const int tc = (int)(u % g.tiles_c); u /= g.tiles_c;
    const int tr = (int)(u % g.tiles_r); u /= g.tiles_r;
    const int cb = (int)(u % g.co_blocks); u /= g.co_blocks;
    const int64_t n = u;
    const int oh0 = tr * g.TR, ow0 = tc * g.TC;
    const int co0 = cb * kCoTile;
    const int KT = g.kh * g.kw;
    const int64_t plane = (int64_t)g.H * g.W;
    const float *xn = x + n * g.Cin * plane;

    v16f acc[2][NBW];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;

    const int a_lane0 = half * 64 + ((l32 + 32 * half) & 63);          // + mb*32 stays inside 0..63
    const int a_lane1 = half * 64 + ((32 + l32 + 32 * half) & 63);
    const int b_lane = half * g.CP + (wave * NBW) * 32 + l32;

    for (int ci0 = 0; ci0 < g.Cin; ci0 += CIB) {
        __syncthreads();                              // previous block fully consumed
        // ---- stage inputs: rows of the tile, zero outside the image, zero tail up to CP
        for (int rowid = wave; rowid < CIB * g.NRows; rowid += 4) {
            const int ci = rowid / g.NRows, rr = rowid - ci * g.NRows;
            const int gh = oh0 + rr - g.ph;
            const bool row_ok = (ci0 + ci < g.Cin) && gh >= 0 && gh < g.H;
            const float *src = xn + (int64_t)(ci0 + ci) * plane + (int64_t)gh * g.W;
            for (int cc = lane; cc < g.Wt; cc += 64) {
                const int gw = ow0 + cc - g.pw;
                Xl[ci * g.CP + rr * g.Wt + cc] = (row_ok && gw >= 0 && gw < g.W) ? src[gw] : 0.0f;
            }
        }
        {
            const int used = g.NRows * g.Wt, tail = g.CP - used;
            for (int i = threadIdx.x; i < CIB * tail; i += kThreads) {
                const int ci = i / tail, o = i - ci * tail;
                Xl[ci * g.CP + used + o] = 0.0f;
            }
        }
        // ---- stage weights: lane = output channel, (ci, tap) walks the contiguous block
        {
            const int per_co = CIB * KT;
            const bool co_ok = co0 + lane < g.Cout;
            const float *wsrc = wgt + ((int64_t)(co0 + lane) * g.Cin + ci0) * KT;
            for (int j = wave; j < per_co; j += 4) {
                const int ci = j / KT, tap = j - ci * KT;
                const float v = (co_ok && ci0 + ci < g.Cin) ? wsrc[j] : 0.0f;
                Wl[((tap * KP + (ci >> 1)) * 2 + (ci & 1)) * 64 + ((lane + 32 * (ci & 1)) & 63)] = v;
            }
        }
        __syncthreads();
        // ---- taps x channel pairs on the matrix cores
        int ta = 0, tb = 0;
        for (int tap = 0; tap < KT; ++tap) {
            const int shift = ta * g.Wt + tb;
            const float *wt = Wl + tap * KP * 128;
            const float *xt = Xl + b_lane + shift;
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) {
                const float a0 = wt[kp * 128 + a_lane0];
                const float a1 = wt[kp * 128 + a_lane1];
                float b[NBW];
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) b[nb] = xt[2 * kp * g.CP + nb * 32];
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) {
                    acc[0][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b[nb], acc[0][nb], 0, 0, 0);
                    acc[1][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b[nb], acc[1][nb], 0, 0, 0);
                }
            }
            if (++tb == g.kw) { tb = 0; ++ta; }
        }
    }

    // ---- epilogue: registers -> y (32 consecutive positions per store instruction)
    float *yn = y + n * g.Cout * (int64_t)g.Ho * g.Wo;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int p = (wave * NBW + nb) * 32 + l32;
        const int r = p / g.Wt, c = p - r * g.Wt;
        const int oh = oh0 + r, ow = ow0 + c;
        if (r >= g.TR || c >= g.TC || oh >= g.Ho || ow >= g.Wo) continue;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int co = co0 + mb * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (co < g.Cout) yn[((int64_t)co * g.Ho + oh) * g.Wo + ow] = acc[mb][nb][v];
            }
    }
}

template <int NBW>
bool plan(ConvGeom &g, int64_t N, int64_t *n_units, size_t *lds_bytes, int CIB)
{
    const int NP = 128 * NBW;
    if (g.Wo + g.kw - 1 <= NP) {                      // full-width tiles, several rows
        g.TC = g.Wo;
        g.Wt = g.TC + g.kw - 1;
        g.TR = NP / g.Wt;
        if (g.TR > g.Ho) g.TR = g.Ho;
    } else {                                          // one row, column tiles
        g.TR = 1;
        g.Wt = NP;
        g.TC = NP - g.kw + 1;
        if (g.TC < 1) return false;
    }
    g.NRows = g.TR + g.kh - 1;
    int need = NP + (g.kh - 1) * g.Wt + g.kw;         // furthest shifted read, any lane
    if (need < g.NRows * g.Wt) need = g.NRows * g.Wt;
    g.CP = (need + 31) / 64 * 64 + 32;                // == 32 (mod 64): the two k-halves of a wave
    if (g.CP < need) g.CP += 64;                      //   hit disjoint LDS banks
    g.tiles_r = (g.Ho + g.TR - 1) / g.TR;
    g.tiles_c = (g.Wo + g.TC - 1) / g.TC;
    g.co_blocks = (g.Cout + kCoTile - 1) / kCoTile;
    *n_units = N * g.co_blocks * g.tiles_r * g.tiles_c;
    *lds_bytes = 4 * ((size_t)CIB * g.CP + (size_t)g.kh * g.kw * (CIB / 2) * 128);
    return *lds_bytes <= 64 * 1024;
}

template <int NBW, int CIB>
hipError_t launch(const float *x, const float *wgt, float *y, const ConvGeom &g, int64_t n_units, size_t lds_bytes,
                  hipStream_t s)
{
    const int64_t grid = xcd_grid(n_units);
    if (grid > 2147483647LL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv2d_mfma_kernel<NBW, CIB>), dim3((unsigned)grid), dim3(kThreads), lds_bytes, s, x, wgt, y,
                       g, n_units);
    return hipGetLastError();
}

}  // namespace

// Stride-1, undilated, groups = 1 convolution on the matrix cores.  *taken = false means the
// shape is outside what this kernel covers and nothing was launched.
hipError_t launch_conv2d_mfma(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                              int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t ph,
                              int32_t pw, hipStream_t s, bool *taken)
{
    *taken = false;
    const int KT = kh * kw;
    const int CIB = (KT <= 9) ? 16 : (KT <= 36 ? 4 : 0);
    if (CIB == 0 || Cin < 2) return hipSuccess;
    ConvGeom g;
    g.Cin = (int)Cin; g.H = (int)H; g.W = (int)W; g.Cout = (int)Cout; g.Ho = (int)Ho; g.Wo = (int)Wo;
    g.kh = kh; g.kw = kw; g.ph = ph; g.pw = pw;
    ConvGeom g2 = g, g1 = g;
    int64_t u2 = 0, u1 = 0;
    size_t l2 = 0, l1 = 0;
    const bool ok2 = plan<2>(g2, N, &u2, &l2, CIB);
    const bool ok1 = plan<1>(g1, N, &u1, &l1, CIB);
    const bool use2 = ok2 && (u2 >= 512 || !ok1);
    if (!use2 && !ok1) return hipSuccess;
    *taken = true;
    if (use2) {
        if (CIB == 16) return launch<2, 16>(x, wgt, y, g2, u2, l2, s);
        return launch<2, 4>(x, wgt, y, g2, u2, l2, s);
    }
    if (CIB == 16) return launch<1, 16>(x, wgt, y, g1, u1, l1, s);
    return launch<1, 4>(x, wgt, y, g1, u1, l1, s);
}

}  // namespace sws
