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
// Tile geometry.  A workgroup computes 64 output channels for NP output positions of one
// image; each wavefront owns MB 32-channel blocks x NBW 32-position blocks of accumulators.
// Two ways to cut an image into tiles:
//   mode A (narrow images): NP consecutive positions of the flattened Ho*Wo output, which
//          span a few whole rows; the staged rows are full width plus halo.
//   mode B (wide images, and 1-D convolution as height 1): NP consecutive positions of one
//          output row; the staged rows are that column range plus halo.
// Either way a lane knows the LDS offset of its position inside the staged tile (row pitch
// Wt), and the input of tap (a, b) is that offset + a*Wt + b: a shifted read.
//
// MFMA operand layout (32x32x2, wave64): lane l supplies A[i = l%32][k = l/32] and
// B[k = l/32][j = l%32]; accumulator register v of lane l holds
// D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].
//
// Pipeline per block of CIB input channels: the global loads of block i+1 are issued into
// registers before the MFMA loop of block i and written to LDS after it, so their latency
// hides behind the matrix work.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kCoTile = 64;                           // output channels per workgroup

typedef float v16f __attribute__((ext_vector_type(16)));

struct ConvGeom {
    int Cin, H, W, Cout, Ho, Wo, kh, kw, ph, pw;
    int sh, sw;                                       // strides (the channel-fastest kernel only)
    int dh, dw;                                       // tap spacing (ditto)
    int wstride, wofs;                                // taps per (co, ci) pair in memory; first tap of this launch
    int wadj;                                         // weights read as the adjoint's: wgt[ci][co][last tap - t]
    int accum;                                        // add to what y already holds (a later chunk of taps)
    int mode_b;                                       // 0: flat tiles over rows, 1: column tiles of one row
    int NP;                                           // output positions per workgroup
    int Wt, NRows, CP;                                // staged row pitch, staged rows, channel pitch in LDS
    int CH;                                           // 64-column chunks per staged row
    int tiles_per_img, tiles_c, co_blocks;
    // (read by the general instance only; kept behind the fields every instance reads)
    int wlast, wrs, wcs;                              // adjoint view: index of the tap read first, and the steps (in taps of the
                                                      //   stored kernel) from one row / one tap of this launch's kernel to the next
    int yH, yW, ysh, ysw, yh0, yw0;                   // general instance: output (oh, ow) is stored at row yh0 + oh*ysh, column
                                                      //   yw0 + ow*ysw of planes of yH x yW (a phase of a strided adjoint)
    int vw, xsh, xsw, xH, xW;                         // general instance, 1 x 1 kernels: the launch's plane is a row of cells
                                                      //   numbered row-major over rows of vw cells; cell (r, c) of those rows is
                                                      //   input element (r*xsh, c*xsw) of the stored xH x xW plane, and output
                                                      //   row / column (r, c) before ysh / ysw apply.  vw = 2^30: no renumbering
};

// x / d for 0 <= x < 2^20 and 1 <= d < 2^12, exact, a handful of VALU ops instead of the
// long integer-division sequence (the margin 0.5/d dwarfs the fp32 rounding of the product).
__device__ __forceinline__ int fast_div(int x, float inv_d) { return (int)(((float)x + 0.5f) * inv_d); }

template <int WAVES, int MB, int NBW, int CIB>
__global__ __launch_bounds__(WAVES * 64, 2) void conv2d_mfma_kernel(const float *__restrict__ x,
                                                                 const float *__restrict__ wgt,
                                                                 float *__restrict__ y, ConvGeom g,
                                                                 int64_t n_units)
{
    constexpr int THREADS = WAVES * 64;
    constexpr int MG = 2 / MB;                        // wave groups along the 64 output channels
    constexpr int KP = CIB / 2;                       // k-pairs (MFMA steps) per tap and channel block
    constexpr int XS = (CIB == 16 ? 128 : 64) / WAVES;    // staged-input registers per lane
    constexpr int WS = (2304 + THREADS - 1) / THREADS;    // staged-weight 128-bit registers per lane
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *Xl = lds;                                  // [CIB][CP] staged inputs
    float *Wl = lds + CIB * g.CP;                     // [64 co][WP] weights of the block, as in memory

    const int64_t unit = xcd_unit(n_units);
    if (unit < 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wave % MG, wn = wave / MG;         // my channel group, my position group

    // unit -> (image, co block, tile)
    int64_t u = unit;
    const int tile = (int)(u % g.tiles_per_img); u /= g.tiles_per_img;
    const int cb = (int)(u % g.co_blocks); u /= g.co_blocks;
    const int64_t n = u;
    const int co0 = cb * kCoTile;
    const int KT = g.kh * g.kw;
    const int plane = g.H * g.W;
    const float *xn = x + n * g.Cin * (int64_t)plane;

    // tile origin: first output row / column, and the input coordinates of staged (0, 0)
    int oh_first, ow_first, p_base = 0;
    if (g.mode_b) {
        oh_first = tile / g.tiles_c;
        ow_first = (tile - oh_first * g.tiles_c) * g.NP;
    } else {
        p_base = tile * g.NP;
        oh_first = p_base / g.Wo;
        ow_first = 0;
    }
    const int row0 = oh_first - g.ph, col0 = ow_first - g.pw;

    // my positions: validity, output coordinates, offset inside the staged tile
    int oh[NBW], ow[NBW], boff[NBW];
    bool pok[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int idx = (wn * NBW + nb) * 32 + l32;
        if (g.mode_b) {
            oh[nb] = oh_first;
            ow[nb] = ow_first + idx;
            pok[nb] = ow[nb] < g.Wo;
        } else {
            const int p = p_base + idx;
            oh[nb] = p / g.Wo;
            ow[nb] = p - oh[nb] * g.Wo;
            pok[nb] = p < g.Ho * g.Wo;
        }
        boff[nb] = half * g.CP + (pok[nb] ? (oh[nb] - oh_first) * g.Wt + (ow[nb] - ow_first) : 0);
    }

    v16f acc[MB][NBW];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.0f;

    // Weights sit in LDS as 64 rows (output channels) of per_co = CIB*KT floats in memory order
    // (channel-major, tap fastest) with pitch WP = per_co + 2.  WP == 2 (mod 4) spreads 32
    // consecutive channels over 32 distinct even banks, and the k = 1 half of the wave reads KT
    // floats further on: the odd banks when KT is odd.
    const int per_co = CIB * KT;
    const int WP = per_co + 2;
    const int a_lane = (wm * MB * 32 + l32) * WP + half * KT;

    // Staging plan, fixed for the whole kernel.  Input segments (channel, staged row, 64-column
    // chunk) are dealt to the wavefronts round-robin; slot s of this lane moves one float of
    // segment wave + WAVES*s.  xg = offset of that float inside the channel block (-1: always
    // zero), xl = its LDS offset (-1: nothing to write).  Everything is straight-line code so
    // that all loads of a block are in flight together.
    const int nseg = CIB * g.NRows * g.CH;
    const float inv_rc = 1.0f / (float)(g.NRows * g.CH), inv_c = 1.0f / (float)g.CH;
    int xg[XS], xl[XS];
#pragma unroll
    for (int s = 0; s < XS; ++s) {
        const int seg = wave + WAVES * s;
        const int ci = fast_div(seg, inv_rc);
        const int r2 = seg - ci * g.NRows * g.CH;
        const int rr = fast_div(r2, inv_c), ch = r2 - rr * g.CH;
        const int gh = row0 + rr, cc = ch * 64 + lane, gw = col0 + cc;
        const bool act = seg < nseg && cc < g.Wt;
        xl[s] = act ? ci * g.CP + rr * g.Wt + cc : -1;
        xg[s] = (act && gh >= 0 && gh < g.H && gw >= 0 && gw < g.W) ? ci * plane + gh * g.W + gw : -1;
    }
    // Weight block: 64 runs (one per output channel) of per_co contiguous floats, moved as
    // 128-bit pieces; piece f = tid + THREADS*s belongs to channel f / (per_co/4).
    const int pf4 = per_co / 4, nf4 = kCoTile * pf4;
    const float inv_pf4 = 1.0f / (float)pf4;
    int wg[WS], wl[WS];
#pragma unroll
    for (int s = 0; s < WS; ++s) {
        const int f = threadIdx.x + THREADS * s;
        const int co = fast_div(f, inv_pf4), j4 = f - co * pf4;
        const bool ok = f < nf4 && co0 + co < g.Cout;
        wg[s] = ok ? (co0 + co) * g.Cin * KT + 4 * j4 : -1;
        wl[s] = f < nf4 ? co * WP + 4 * j4 : -1;
    }

    float xreg[XS];
    v4f wreg[WS];

    // Loads are unconditional (out-of-range slots read element 0 of the image / of the weights,
    // which is valid memory) and the validity test is applied when the registers are written to
    // LDS, on the far side of the matrix loop: nothing forces a wait on a single load.
    auto prefetch = [&](int ci0) {
        const int xb = ci0 * plane;
#pragma unroll
        for (int s = 0; s < XS; ++s) xreg[s] = xn[xg[s] >= 0 ? xb + xg[s] : 0];
        const int wb = ci0 * KT;
#pragma unroll
        for (int s = 0; s < WS; ++s) wreg[s] = *(const v4f_u *)(wgt + (wg[s] >= 0 ? wb + wg[s] : 0));
    };

    auto commit = [&]() {
#pragma unroll
        for (int s = 0; s < XS; ++s)
            if (xl[s] >= 0) Xl[xl[s]] = xg[s] >= 0 ? xreg[s] : 0.0f;
#pragma unroll
        for (int s = 0; s < WS; ++s) {
            if (wl[s] >= 0) {
                const v4f v = wg[s] >= 0 ? wreg[s] : (v4f){0.0f, 0.0f, 0.0f, 0.0f};
                *(v2f *)(Wl + wl[s]) = (v2f){v.x, v.y};          // rows are 8-byte aligned (WP is even)
                *(v2f *)(Wl + wl[s] + 2) = (v2f){v.z, v.w};
            }
        }
    };

    // zero the part of every channel slab that staging never writes (read by discarded lanes only)
    {
        const int used = g.NRows * g.Wt, tail = g.CP - used;
        for (int i = threadIdx.x; i < CIB * tail; i += THREADS) {
            const int ci = i / tail, o = i - ci * tail;
            Xl[ci * g.CP + used + o] = 0.0f;
        }
    }

    prefetch(0);
    for (int ci0 = 0; ci0 < g.Cin; ci0 += CIB) {
        __syncthreads();                              // the previous block has been consumed
        commit();
        __syncthreads();
        if (ci0 + CIB < g.Cin) prefetch(ci0 + CIB);   // in flight during the matrix work below
        int ta = 0, tb = 0;
        for (int tap = 0; tap < KT; ++tap) {
            const int shift = ta * g.Wt + tb;
            const float *wt = Wl + tap + a_lane;
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) {
                float a[MB], b[NBW];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) a[mb] = wt[2 * kp * KT + mb * 32 * WP];
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) b[nb] = Xl[2 * kp * g.CP + boff[nb] + shift];
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mb], b[nb], acc[mb][nb], 0, 0, 0);
            }
            if (++tb == g.kw) { tb = 0; ++ta; }
        }
    }

    // ---- epilogue: registers -> y (32 consecutive positions per store instruction)
    float *yn = y + n * g.Cout * (int64_t)g.Ho * g.Wo;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        if (!pok[nb]) continue;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int co = co0 + (wm * MB + mb) * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (co < g.Cout) yn[((int64_t)co * g.Ho + oh[nb]) * g.Wo + ow[nb]] = acc[mb][nb][v];
            }
    }
}

// ------------------------------------------------------------------------------------------
// Channel-fastest variant for kh*kw <= 9: 128-bit operand reads.
// ------------------------------------------------------------------------------------------
// Same tiling (64 output channels x 128 positions, 8 wavefronts, one 32x32 accumulator block
// each) but the LDS tiles keep the 8 input channels of a block next to each other:
//   Xl[position][12]      (8 channels + 4 floats of padding: pitch 48 bytes)
//   Wl[tap][channel out][12]
// The k index of the four MFMA steps of a tap is mapped as step j <-> channels (j, 4+j), so
// the half-wave h needs channels 4h .. 4h+3 of its position / output channel: ONE 128-bit
// LDS read per operand feeds four MFMAs (the scalar-read kernel above needs eight reads).
// With the 12-float pitch sixteen consecutive lanes of a 128-bit read hit sixteen distinct
// bank quads.
// Staging plan of the input tile, computed on the host and passed by value: segment i (one
// staged row of one channel, 64 columns wide) packs its channel, row and chunk into e[i].  Wavefront w moves segments w, w+8, ...; the lookups are scalar loads.
struct SegPlan {
    unsigned int e[128];                              // channel | row << 8 | chunk << 16
};

// (the second launch bound is wavefronts per SIMD: two workgroups per compute unit)
// GEN: the general instance — the input-channel count need not be a multiple of 8 (channels beyond
// it are staged as zeros) and the weights may be read through the adjoint view.  The plain
// instance keeps constant tap offsets and unguarded channel blocks.
template <int KTT, int WAVES, int NB, int SEG, bool GEN = false>
__global__ __launch_bounds__(WAVES * 64, (2 * WAVES + 3) / 4) void conv2d_mfma_c8_kernel(const float *__restrict__ x,
                                                                       const float *__restrict__ wgt,
                                                                       float *__restrict__ y, ConvGeom g,
                                                                       SegPlan sp)
{
    // NB blocks of 8 input channels are staged per barrier pair (NB > 1 for few taps, where one
    // block is too little matrix work between two barriers).
    constexpr int CIB = 8, XP = 12;
    constexpr int MAXSEG = SEG;                       // segments of one channel block (checked by the host)
    constexpr int XS = (MAXSEG + WAVES - 1) / WAVES;  // staged-input registers per lane and channel block
    constexpr int KTMAX = KTT > 0 ? KTT : 9;          // staged-weight registers per lane and channel block
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *Xl = lds;                                  // NB input tiles of CP floats
    float *Wl = lds + NB * g.CP;                      // NB weight blocks of KT * 64 * 12 floats

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;          // my channel block, my position block

    // grid: x = tile of the image, y = output-channel block, z = image
    const int tile = blockIdx.x;
    const int co0 = blockIdx.y * kCoTile;
    const int64_t n = blockIdx.z;
    const int KT = KTT > 0 ? KTT : g.kh * g.kw;
    const int plane = GEN ? g.xH * g.xW : g.H * g.W;
    const float *xn = x + n * g.Cin * (int64_t)plane;

    int oh_first, ow_first, p_base = 0;
    if (g.mode_b) {
        oh_first = tile / g.tiles_c;
        ow_first = (tile - oh_first * g.tiles_c) * g.NP;
    } else {
        p_base = tile * g.NP;
        oh_first = p_base / g.Wo;
        ow_first = 0;
    }
    const int row0 = oh_first * g.sh - g.ph, col0 = ow_first * g.sw - g.pw;

    // my position
    int oh, ow;
    bool pok;
    {
        const int idx = wn * 32 + l32;
        if (g.mode_b) {
            oh = oh_first;
            ow = ow_first + idx;
            pok = ow < g.Wo;
        } else {
            const int p = p_base + idx;
            oh = fast_div(p, 1.0f / (float)g.Wo);
            ow = p - oh * g.Wo;
            pok = p < g.Ho * g.Wo;
        }
    }
    const int b_lane = (pok ? (oh - oh_first) * g.sh * g.Wt + (ow - ow_first) * g.sw : 0) * XP + 4 * half;
    const int a_lane = (wm * 32 + l32) * XP + 4 * half;
    const bool useful = co0 + wm * 32 < g.Cout;       // wave-uniform

    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    // ---- input staging plan: slot s of this wavefront moves segment wave + 8*s
    const int nseg = CIB * g.NRows * g.CH;
    int xg[XS], xl[XS], xc[XS];
#pragma unroll
    for (int s = 0; s < XS; ++s) {
        const int seg = wave + WAVES * s;
        const int sq = seg < MAXSEG ? seg : MAXSEG - 1;
        const unsigned int pe = sp.e[sq];             // uniform index: a scalar load
        const int ci = pe & 255, rr = (pe >> 8) & 255, ch = pe >> 16;
        xc[s] = ci;
        const int gh = row0 + rr, cc = ch * 64 + lane, gw = col0 + cc;
        const bool act = seg < nseg && cc < g.Wt;
        xl[s] = act ? (rr * g.Wt + cc) * XP + ci : -1;
        if constexpr (GEN) {
            const int vr = gw >= 0 ? gw / g.vw : 0, vc = gw - vr * g.vw;     // (0, gw) unless the plane is renumbered
            xg[s] = (act && gh >= 0 && gh < g.H && gw >= 0 && gw < g.W) ? ci * plane + (gh + vr) * g.xsh * g.xW + vc * g.xsw : -1;
        } else {
            xg[s] = (act && gh >= 0 && gh < g.H && gw >= 0 && gw < g.W) ? ci * plane + gh * g.W + gw : -1;
        }
    }
    // ---- weight staging plan: thread (co = tid / 8, ci = tid % 8) moves the KT taps of one
    // (output channel, input channel) pair: KT contiguous floats in memory, and in LDS the
    // same word of KT consecutive tap planes (a constant stride).
    const int w_co = (threadIdx.x >> 3) & (kCoTile - 1), w_ci = threadIdx.x & 7;
    const bool w_mine = threadIdx.x < kCoTile * 8;    // the first 512 threads move the weights
    const bool w_ok = w_mine && co0 + w_co < g.Cout;
    // Plain view: wgt[co][ci][wofs + t].  Adjoint view (the convolution that maps output gradients
    // back to the input): this launch's output channel co is the stored array's input channel, so
    // the element is wgt[ci][co][wstride - 1 - wofs - t] with rows of g.Cout pairs.
    constexpr bool TAIL = GEN;
    const bool adj = GEN && g.wadj;
    const int64_t w_sci = adj ? (int64_t)g.Cout * g.wstride : g.wstride;
    const float *wsrc = wgt + (w_ok ? (adj ? (int64_t)w_ci * w_sci + (int64_t)(co0 + w_co) * g.wstride + g.wlast
                                           : ((int64_t)(co0 + w_co) * g.Cin + w_ci) * g.wstride + g.wofs)
                                    : 0);
    // general instance: tap t of this launch's kernel sits toff[t] elements from wsrc (plain view:
    // t; adjoint view: towards the front, by wrs per kernel row and wcs per tap)
    int toff[KTMAX];
    if constexpr (GEN) {
        int ta = 0, tb = 0;
#pragma unroll
        for (int t = 0; t < KTMAX; ++t) {
            toff[t] = t < KT ? (adj ? -(ta * g.wrs + tb * g.wcs) : t) : 0;
            if (++tb == g.kw) { tb = 0; ++ta; }
        }
    }
    float *wdst = Wl + w_co * XP + w_ci;

    float xreg[NB][XS], wreg[NB][KTMAX];
    const int wblock = KT * kCoTile * XP;             // floats of one weight block in LDS
    // Loads are unconditional (out-of-range slots read valid memory and are dropped when the
    // registers are written to LDS, on the far side of the matrix loop), so nothing forces a
    // wait on a single load.
    auto prefetch = [&](int ci0) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int cb = ci0 + nb * CIB;            // first channel of this block
            const int xb = cb * plane;
#pragma unroll
            for (int s = 0; s < XS; ++s)
                xreg[nb][s] = xn[(xg[s] >= 0 && (!TAIL || cb + xc[s] < g.Cin)) ? xb + xg[s] : 0];
            if constexpr (GEN) {
                const bool wk = w_ok && cb + w_ci < g.Cin;
                const float *w = wk ? wsrc + cb * w_sci : wgt;
#pragma unroll
                for (int t = 0; t < KTMAX; ++t) wreg[nb][t] = w[wk ? toff[t] : 0];
            } else {
                const float *w = wsrc + (w_ok ? cb * g.wstride : 0);
#pragma unroll
                for (int t = 0; t < KTMAX; ++t) wreg[nb][t] = w[t < KT ? t : 0];
            }
        }
    };
    auto commit = [&](int ci0) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int cb = ci0 + nb * CIB;
#pragma unroll
            for (int s = 0; s < XS; ++s)
                if (xl[s] >= 0)
                    Xl[nb * g.CP + xl[s]] = (xg[s] >= 0 && (!TAIL || cb + xc[s] < g.Cin)) ? xreg[nb][s] : 0.0f;
            const bool wk = w_ok && (!TAIL || cb + w_ci < g.Cin);
#pragma unroll
            for (int t = 0; t < KTMAX; ++t)
                if (t < KT && w_mine) wdst[nb * wblock + t * kCoTile * XP] = wk ? wreg[nb][t] : 0.0f;
        }
    };

    prefetch(0);
    for (int ci0 = 0; ci0 < g.Cin; ci0 += CIB * NB) {
        __syncthreads();                              // the previous blocks have been consumed
        commit(ci0);
        __syncthreads();
        if (ci0 + CIB * NB < g.Cin) prefetch(ci0 + CIB * NB);   // in flight during the matrix work below
        if (!useful) continue;                        // a block of 32 output channels beyond Cout: staging only
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const float *Xb = Xl + nb * g.CP, *Wb = Wl + nb * wblock;
            if (KTT > 0) {
#pragma unroll
                for (int tap = 0; tap < (KTT > 0 ? KTT : 1); ++tap) {
                    const int shift = (tap / 3) * g.dh * g.Wt + (tap % 3) * g.dw;    // KTT > 0 is only used with kw == 3
                    const v4f a4 = *(const v4f *)(Wb + tap * kCoTile * XP + a_lane);
                    const v4f b4 = *(const v4f *)(Xb + shift * XP + b_lane);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4.x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4.y, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4.z, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4.w, acc, 0, 0, 0);
                }
            } else {
                int ta = 0, tb = 0;
                for (int tap = 0; tap < KT; ++tap) {
                    const int shift = ta * g.dh * g.Wt + tb * g.dw;
                    const v4f a4 = *(const v4f *)(Wb + tap * kCoTile * XP + a_lane);
                    const v4f b4 = *(const v4f *)(Xb + shift * XP + b_lane);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4.x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4.y, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4.z, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4.w, acc, 0, 0, 0);
                    if (++tb == g.kw) { tb = 0; ++ta; }
                }
            }
        }
    }

    if (!pok) return;
    if constexpr (GEN) {
        float *yn = y + n * g.Cout * (int64_t)g.yH * g.yW;
        const int vr = ow / g.vw, vc = ow - vr * g.vw;
        const int64_t at = (int64_t)(g.yh0 + (oh + vr) * g.ysh) * g.yW + g.yw0 + vc * g.ysw;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int co = co0 + wm * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (co < g.Cout) {
                float *dst = yn + (int64_t)co * g.yH * g.yW + at;
                *dst = g.accum ? *dst + acc[v] : acc[v];
            }
        }
        return;
    }
    float *yn = y + n * g.Cout * (int64_t)g.Ho * g.Wo;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int co = co0 + wm * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        if (co < g.Cout) {
            float *dst = yn + ((int64_t)co * g.Ho + oh) * g.Wo + ow;
            *dst = g.accum ? *dst + acc[v] : acc[v];
        }
    }
}

bool plan(ConvGeom &g, int NP, int CIB, int xslots_total, int64_t N, int64_t *n_units, size_t *lds_bytes)
{
    g.NP = NP;
    const int span_h = (g.kh - 1) * g.dh + 1, span_w = (g.kw - 1) * g.dw + 1;     // reach of the taps
    if ((g.Wo - 1) * g.sw + span_w <= 192) {          // mode A: flat tiles, full-width rows
        g.mode_b = 0;
        g.Wt = (g.Wo - 1) * g.sw + span_w;
        // output rows a tile can touch (tiles of whole rows always start on a row)
        const int rows = (g.NP % g.Wo == 0) ? g.NP / g.Wo : (g.NP + g.Wo - 2) / g.Wo + 1;
        g.NRows = ((rows < g.Ho ? rows : g.Ho) - 1) * g.sh + span_h;
        g.tiles_c = 1;
        g.tiles_per_img = (g.Ho * g.Wo + g.NP - 1) / g.NP;
    } else {                                          // mode B: column tiles of single rows
        g.mode_b = 1;
        g.Wt = (g.NP - 1) * g.sw + span_w;
        g.NRows = span_h;
        g.tiles_c = (g.Wo + g.NP - 1) / g.NP;
        g.tiles_per_img = g.Ho * g.tiles_c;
    }
    g.CH = (g.Wt + 63) / 64;
    const int need = g.NRows * g.Wt;
    g.CP = (need + 31) / 64 * 64 + 32;                // == 32 (mod 64): the two k-halves of a wave
                                                      //   read disjoint LDS banks
    g.co_blocks = (g.Cout + kCoTile - 1) / kCoTile;
    *n_units = N * g.co_blocks * g.tiles_per_img;
    *lds_bytes = 4 * ((size_t)CIB * g.CP + (size_t)kCoTile * (CIB * g.kh * g.kw + 2));
    const int nseg = CIB * g.NRows * g.CH;
    // (the channel-fastest kernel passes xslots_total = 1 << 30 and checks its own LDS layout)
    const bool fits = xslots_total == (1 << 30) || (*lds_bytes <= 64 * 1024 && nseg <= xslots_total);
    return fits && kCoTile * (CIB * g.kh * g.kw / 4) <= 2304 && (int64_t)g.Cin * g.H * g.W < 2147483647LL;
}

template <int WAVES, int MB, int NBW, int CIB>
hipError_t launch(const float *x, const float *wgt, float *y, const ConvGeom &g, int64_t n_units, size_t lds_bytes,
                  hipStream_t s)
{
    const int64_t grid = xcd_grid(n_units);
    if (grid > 2147483647LL) return kNotTaken;
    hipLaunchKernelGGL((conv2d_mfma_kernel<WAVES, MB, NBW, CIB>), dim3((unsigned)grid), dim3(WAVES * 64), lds_bytes,
                       s, x, wgt, y, g, n_units);
    return hipGetLastError();
}

}  // namespace

namespace {

// One launch of the channel-fastest kernel, fully decided on the host before anything runs.
struct C8Launch {
    ConvGeom g;
    SegPlan sp;
    dim3 grid;
    size_t lds;
    int waves, ktt, nb, seg, tail;
};

// Decides tile width and template instance for the geometry in L->g (kh * kw <= 9).
bool c8_prepare(C8Launch *L, int64_t N)
{
    ConvGeom &g = L->g;
    const int KT = g.kh * g.kw;
    int64_t units = 0;
    size_t lds = 0;
    // Tile width: 8 to 14 wavefronts (128 to 224 positions).  Two workgroups share a compute unit,
    // so the launch takes ceil(workgroups / 512) rounds of `waves` accumulator blocks each.
    int best_w = 0;
    int64_t best_cost = 0;
    for (int wv = 8; wv <= 14; wv += 2) {
        if (g_opt.conv2d_variant >= 8 && g_opt.conv2d_variant != wv) continue;     // A/B: force a width
        ConvGeom t = g;
        if (!plan(t, 16 * wv, 16, 1 << 30, N, &units, &lds)) continue;
        const int xfl = (t.NRows * t.Wt * 12 + 3) / 4 * 4;
        // staging plan: up to 64 row segments per channel block, 128 with 8 wavefronts
        if (8 * t.NRows * t.CH > (wv == 8 ? 128 : 64) || t.NRows >= 256 ||
            4 * ((size_t)xfl + (size_t)KT * kCoTile * 12) > 64 * 1024)
            continue;
        const int64_t cost = ((units + 511) / 512) * wv;
        if (best_w == 0 || cost < best_cost) { best_w = wv; best_cost = cost; }
    }
    if (best_w == 0 || N > 65535 || (g.Cout + kCoTile - 1) / kCoTile > 65535) return false;
    plan(g, 16 * best_w, 16, 1 << 30, N, &units, &lds);
    const int xfloats = (g.NRows * g.Wt * 12 + 3) / 4 * 4;
    const size_t lds1 = 4 * ((size_t)xfloats + (size_t)KT * kCoTile * 12);
    // few taps: four channel blocks per barrier pair, if they fit
    const bool general = g.Cin % 8 != 0 || g.wadj || g.vw != (1 << 30);    // the general instance stages one channel block per barrier pair
    // (the general instance has it for 1 x 1 kernels only: the adjoint of a 1 x 1 convolution)
    const bool nb4 = ((!general && KT == 3 && g.kw == 3) || KT == 1) && g.Cin % 32 == 0 && 8 * g.NRows * g.CH <= 32 &&
                     4 * lds1 <= 64 * 1024 && g_opt.conv2d_variant != 5;
    const bool seg128 = 8 * g.NRows * g.CH > 64;          // only reached with 8 wavefronts (strided: tall tiles)
    g.CP = xfloats;
    for (int i = 0; i < 128; ++i) {
        const int ci = i / (g.NRows * g.CH), r2 = i % (g.NRows * g.CH);
        L->sp.e[i] = (unsigned)(ci < 8 ? ci : 0) | (unsigned)(r2 / g.CH) << 8 | (unsigned)(r2 % g.CH) << 16;
    }
    L->grid = dim3((unsigned)g.tiles_per_img, (unsigned)g.co_blocks, (unsigned)N);
    L->lds = (nb4 ? 4 : 1) * lds1;
    L->waves = seg128 ? 8 : best_w;
    L->tail = general;
    L->ktt = (KT == 9 && g.kw == 3) ? 9 : ((KT == 3 && g.kw == 3) ? 3 : ((KT == 1 && nb4 && !seg128) ? 1 : 0));
    L->nb = (nb4 && !seg128) ? 4 : 1;
    L->seg = seg128 ? 128 : (L->nb == 4 ? 32 : 64);
    return true;
}

hipError_t c8_launch(const C8Launch &L, const float *x, const float *wgt, float *y, hipStream_t s)
{
#define SWS_C8(KTT, WV, NB, SEG)                                                                                \
    hipLaunchKernelGGL((conv2d_mfma_c8_kernel<KTT, WV, NB, SEG>), L.grid, dim3(WV * 64), L.lds, s, x, wgt, y, L.g, L.sp)
#define SWS_C8_W(KTT, NB, SEG)                                                                                  \
    switch (L.waves) {                                                                                          \
    case 8: SWS_C8(KTT, 8, NB, SEG); break;                                                                     \
    case 10: SWS_C8(KTT, 10, NB, SEG); break;                                                                   \
    case 12: SWS_C8(KTT, 12, NB, SEG); break;                                                                   \
    default: SWS_C8(KTT, 14, NB, SEG); break;                                                                   \
    }
    if (L.tail) {                                     // the general instance: one channel block per barrier pair
#define SWS_C8T(KTT, WV, SEG)                                                                                   \
    hipLaunchKernelGGL((conv2d_mfma_c8_kernel<KTT, WV, 1, SEG, true>), L.grid, dim3(WV * 64), L.lds, s, x, wgt, y, L.g, L.sp)
#define SWS_C8T_W(KTT)                                                                                          \
    if (L.seg == 128) SWS_C8T(KTT, 8, 128);                                                                     \
    else switch (L.waves) {                                                                                     \
        case 8: SWS_C8T(KTT, 8, 64); break;                                                                     \
        case 10: SWS_C8T(KTT, 10, 64); break;                                                                   \
        case 12: SWS_C8T(KTT, 12, 64); break;                                                                   \
        default: SWS_C8T(KTT, 14, 64); break;                                                                   \
    }
        if (L.nb == 4) {                              // 1 x 1 through the adjoint view, four channel blocks per barrier pair
            switch (L.waves) {
            case 8: hipLaunchKernelGGL((conv2d_mfma_c8_kernel<1, 8, 4, 32, true>), L.grid, dim3(8 * 64), L.lds, s, x, wgt, y, L.g, L.sp); break;
            case 10: hipLaunchKernelGGL((conv2d_mfma_c8_kernel<1, 10, 4, 32, true>), L.grid, dim3(10 * 64), L.lds, s, x, wgt, y, L.g, L.sp); break;
            case 12: hipLaunchKernelGGL((conv2d_mfma_c8_kernel<1, 12, 4, 32, true>), L.grid, dim3(12 * 64), L.lds, s, x, wgt, y, L.g, L.sp); break;
            default: hipLaunchKernelGGL((conv2d_mfma_c8_kernel<1, 14, 4, 32, true>), L.grid, dim3(14 * 64), L.lds, s, x, wgt, y, L.g, L.sp); break;
            }
        }
        else if (L.ktt == 9) { SWS_C8T_W(9) }
        else if (L.ktt == 3) { SWS_C8T_W(3) }
        else { SWS_C8T_W(0) }
#undef SWS_C8T_W
#undef SWS_C8T
    } else if (L.seg == 128) {
        if (L.ktt == 9) SWS_C8(9, 8, 1, 128);
        else if (L.ktt == 3) SWS_C8(3, 8, 1, 128);
        else SWS_C8(0, 8, 1, 128);
    } else if (L.ktt == 9) {
        SWS_C8_W(9, 1, 64)
    } else if (L.nb == 4 && L.ktt == 1) {             // 1 x 1: four channel blocks per barrier pair
        SWS_C8_W(1, 4, 32)
    } else if (L.nb == 4) {
        SWS_C8_W(3, 4, 32)
    } else if (L.ktt == 3) {
        SWS_C8_W(3, 1, 64)
    } else {
        SWS_C8_W(0, 1, 64)
    }
#undef SWS_C8_W
#undef SWS_C8
    return hipGetLastError();
}

}  // namespace

// groups = 1 convolution on the matrix cores.  The channel-fastest kernel takes strides and tap
// spacing, and kernels of more than 9 taps run as a chain of launches over chunks of taps (whole
// kernel rows, or runs of taps of a one-row kernel), each adding to what the earlier ones left in
// y: the sliding sum over taps, cut into pieces.  *taken = false means the shape is outside what
// these kernels cover and nothing was launched.
hipError_t launch_conv2d_mfma(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H,
                              int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh,
                              int32_t sw, int32_t ph, int32_t pw, int32_t dh, int32_t dw, hipStream_t s, bool *taken,
                              int wadj)
{
    *taken = false;
    const bool plain = sh == 1 && sw == 1 && dh == 1 && dw == 1;
    const int KT = kh * kw;
    if (Ho * Wo > 2147483647LL / 2 || Cout * Cin * KT > 2147483647LL / 2) return hipSuccess;
    // A 1 x 1 kernel without stride or padding does not see the rows: the plane is one long row, cut
    // into column tiles (narrow planes would otherwise stage half-empty 64-column segments).
    if (KT == 1 && plain && ph == 0 && pw == 0 && H > 1) {
        W *= H; H = 1;
        Wo *= Ho; Ho = 1;
    }
    // the weight-stationary streaming kernel where it applies (option conv2d_variant 16 switches it off,
    // 17 takes it for small problems too)
    if (plain && (g_opt.conv2d_variant == 0 || g_opt.conv2d_variant == 17 || g_opt.conv2d_variant == 18)) {
        const hipError_t e = launch_conv2d_stream(x, wgt, y, N, Cin, H, W, Cout, Ho, Wo, kh, kw, ph, pw, s, taken, wadj);
        if (*taken || e != hipSuccess) return e;
    }
    ConvGeom g;
    g.Cin = (int)Cin; g.H = (int)H; g.W = (int)W; g.Cout = (int)Cout; g.Ho = (int)Ho; g.Wo = (int)Wo;
    g.kh = kh; g.kw = kw; g.ph = ph; g.pw = pw; g.sh = sh; g.sw = sw; g.dh = dh; g.dw = dw;
    g.wstride = KT; g.wofs = 0; g.accum = 0; g.wadj = wadj;
    g.wlast = KT - 1; g.wrs = kw; g.wcs = 1;
    g.yH = (int)Ho; g.yW = (int)Wo; g.ysh = 1; g.ysw = 1; g.yh0 = 0; g.yw0 = 0;
    g.vw = 1 << 30; g.xsh = 1; g.xsw = 1; g.xH = (int)H; g.xW = (int)W;
    // A strided 1 x 1 kernel without padding reads every sh-th row and sw-th column and nothing else:
    // the cells it reads, numbered row-major, are one long row for a stride-1 launch of the general
    // instance (which would otherwise stage the skipped cells too).
    if (KT == 1 && (sh > 1 || sw > 1) && ph == 0 && pw == 0 && !wadj && Cin * H * W < 2147483647LL) {
        g.vw = (int)Wo; g.xsh = sh; g.xsw = sw;
        g.H = 1; g.W = (int)(Ho * Wo); g.Ho = 1; g.Wo = (int)(Ho * Wo);
        g.sh = 1; g.sw = 1;
    }
    // Up to 36 adjacent taps at stride 1 the scalar-read kernel does the whole kernel in one pass,
    // which beats a chain of five or more launches (5 x 5 on [32,64,56,56]: 0.27 ms against 0.41 ms).
    const bool one_pass = !wadj && plain && KT > 9 && KT <= 36 && Cin % 4 == 0 && g_opt.conv2d_variant != 6;
    // preferred: channel-fastest tiles with 128-bit operand reads (8 input channels per block; a last
    // partial block is padded with zeros)
    // Cin = 4, 12, 20, ... at stride 1: the scalar-read kernel with blocks of 4 channels wastes none
    const bool quad_blocks = Cin % 8 != 0 && Cin % 4 == 0 && plain && !wadj && KT <= 36;
    if (!one_pass && !quad_blocks && g_opt.conv2d_variant != 3 && g_opt.conv2d_variant != 4) {
        // chunks of at most 9 taps: the whole kernel, whole rows of it (rows of up to 9 taps), or
        // runs of up to 9 taps of one row (wider rows)
        const int rows_per = KT <= 9 ? kh : (kw <= 9 ? 9 / kw : 1);
        const int taps_per = kw <= 9 ? kw : 9;
        const int row_chunks = (kh + rows_per - 1) / rows_per, run_chunks = (kw + taps_per - 1) / taps_per;
        const int n_chunks = row_chunks * run_chunks;
        if (n_chunks <= 64) {
            C8Launch L[64];
            bool ok = true;
            for (int c = 0; c < n_chunks && ok; ++c) {
                const int a0 = (c / run_chunks) * rows_per, b0 = (c % run_chunks) * taps_per;
                const int na = kh - a0 < rows_per ? kh - a0 : rows_per, nb = kw - b0 < taps_per ? kw - b0 : taps_per;
                L[c].g = g;
                L[c].g.kh = na; L[c].g.ph = ph - a0 * dh;
                L[c].g.kw = nb; L[c].g.pw = pw - b0 * dw;
                L[c].g.wofs = a0 * kw + b0;           // a chunk of several rows takes whole rows: its taps stay contiguous
                L[c].g.wlast = KT - 1 - (a0 * kw + b0);
                L[c].g.accum = c > 0;
                ok = c8_prepare(&L[c], N);
            }
            if (ok) {
                *taken = true;
                for (int c = 0; c < n_chunks; ++c) {
                    const hipError_t e = c8_launch(L[c], x, wgt, y, s);
                    if (e != hipSuccess) return e;
                }
                return hipSuccess;
            }
        }
    }
    if (!plain || wadj) return hipSuccess;            // the scalar-read kernels below: stride 1, taps adjacent, plain weights
    // channel blocks of 16 (or 4 for big kernels / odd channel counts) must divide Cin
    const int CIB = (KT <= 9 && Cin % 16 == 0) ? 16 : ((KT <= 36 && Cin % 4 == 0) ? 4 : 0);
    if (CIB == 0) return hipSuccess;
    int64_t units = 0;
    size_t lds = 0;
    if (!plan(g, 128, CIB, CIB == 16 ? 128 : 64, N, &units, &lds)) return hipSuccess;
    *taken = true;
    if (g_opt.conv2d_variant == 3) {                  // 4 wavefronts, two channel blocks each (A/B)
        if (CIB == 16) return launch<4, 2, 1, 16>(x, wgt, y, g, units, lds, s);
        return launch<4, 2, 1, 4>(x, wgt, y, g, units, lds, s);
    }
    // 8 wavefronts, one 32x32 accumulator block each: short workgroups, four waves per SIMD
    if (CIB == 16) return launch<8, 1, 1, 16>(x, wgt, y, g, units, lds, s);
    return launch<8, 1, 1, 4>(x, wgt, y, g, units, lds, s);
}

// The adjoint of a strided convolution with respect to its input, one output phase at a time.
// Cells (h, c) of gx with (h + ph) mod sh = rh and (c + pw) mod sw = rc are reached only by the
// taps a = rh, rh + sh, ..., b = rc, rc + sw, ...; over such a phase the adjoint is a stride-1
// convolution of gy with that sub-kernel (flipped, channels swapped: the adjoint weight view with a
// step of sh*kw / sw stored taps per row / tap), written to every sh-th row and sw-th column of gx.
// Sub-kernels of more than 9 taps run as chains of launches like any other kernel.  A phase no tap
// reaches (kernel smaller than the stride) is cleared by the caller.  *taken = false: nothing was
// launched.
hipError_t launch_conv2d_grad_input_phases(const float *gy, const float *wgt, float *gx, int64_t N, int64_t Cin,
                                           int64_t H, int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh,
                                           int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, hipStream_t s,
                                           bool *taken)
{
    *taken = false;
    const int KTF = kh * kw;
    if (H * W > 2147483647LL / 2 || Cout * Cin * KTF > 2147483647LL / 2 || sh * sw > 16) return hipSuccess;
    constexpr int kMaxLaunch = 64;
    C8Launch L[kMaxLaunch];
    int n_launch = 0;
    for (int rh = 0; rh < sh; ++rh)
        for (int rc = 0; rc < sw; ++rc) {
            const int KA = rh < kh ? (kh - rh + sh - 1) / sh : 0, KB = rc < kw ? (kw - rc + sw - 1) / sw : 0;
            if (KA == 0 || KB == 0) continue;         // no tap reaches this phase
            // first cell of the phase and the index i0 of its row among "h = sh*i + rh - ph"
            const int i0 = ph > rh ? (ph - rh + sh - 1) / sh : 0, j0 = pw > rc ? (pw - rc + sw - 1) / sw : 0;
            const int h0 = sh * i0 + rh - ph, c0 = sw * j0 + rc - pw;
            if (h0 >= H || c0 >= W) continue;         // no cell of the plane is in this phase
            const int nH = (int)((H - h0 + sh - 1) / sh), nW = (int)((W - c0 + sw - 1) / sw);
            ConvGeom g;
            g.Cin = (int)Cout; g.H = (int)Ho; g.W = (int)Wo; g.Cout = (int)Cin; g.Ho = nH; g.Wo = nW;
            g.sh = 1; g.sw = 1; g.dh = 1; g.dw = 1;
            g.wstride = KTF; g.wofs = 0; g.wadj = 1;
            g.wrs = sh * kw; g.wcs = sw;
            g.yH = (int)H; g.yW = (int)W; g.ysh = sh; g.ysw = sw; g.yh0 = h0; g.yw0 = c0;
            g.vw = 1 << 30; g.xsh = 1; g.xsw = 1; g.xH = (int)Ho; g.xW = (int)Wo;
            const int last = (rh + sh * (KA - 1)) * kw + rc + sw * (KB - 1);     // the sub-kernel's last tap, read first
            // out[i][j] = sum_{u,v} K[u][v] * gy[i + i0 - (KA-1) + u][j + j0 - (KB-1) + v]: padding KA-1-i0, KB-1-j0
            const int PA = KA - 1 - i0, PB = KB - 1 - j0;
            const int KT = KA * KB;
            if (KT == 1 && PA == 0 && PB == 0 && nH == Ho && nW == Wo && Ho > 1) {
                // a one-tap phase maps gy cell for cell onto its cells of gx: one long row (full tiles on narrow planes)
                g.vw = (int)Wo;
                g.H = 1; g.W = (int)(Ho * Wo); g.Ho = 1; g.Wo = (int)(Ho * Wo);
            }
            const int rows_per = KT <= 9 ? KA : (KB <= 9 ? 9 / KB : 1);
            const int taps_per = KB <= 9 ? KB : 9;
            const int row_chunks = (KA + rows_per - 1) / rows_per, run_chunks = (KB + taps_per - 1) / taps_per;
            for (int c = 0; c < row_chunks * run_chunks; ++c) {
                if (n_launch == kMaxLaunch) return hipSuccess;
                const int a0 = (c / run_chunks) * rows_per, b0 = (c % run_chunks) * taps_per;
                const int na = KA - a0 < rows_per ? KA - a0 : rows_per, nb = KB - b0 < taps_per ? KB - b0 : taps_per;
                C8Launch &Lc = L[n_launch];
                Lc.g = g;
                Lc.g.kh = na; Lc.g.ph = PA - a0;
                Lc.g.kw = nb; Lc.g.pw = PB - b0;
                Lc.g.wlast = last - (a0 * g.wrs + b0 * g.wcs);
                Lc.g.accum = c > 0;
                if (!c8_prepare(&Lc, N)) return hipSuccess;
                ++n_launch;
            }
        }
    *taken = true;
    for (int c = 0; c < n_launch; ++c) {
        const hipError_t e = c8_launch(L[c], gy, wgt, gx, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sws
