// sws_conv1d — 1-D convolution as a sliding sum of shifted, weighted rows (Section 2.5;
// the Vector Slide loop of Section 3, Algorithm 4, with X <- X + f_t * Slide(...)).
// The unmodified input row is staged once per tile; no column matrix is ever built.
//
//  * dense channels (groups = 1): handed to the matrix-core kernel of conv_mfma.hip.
//
//  * conv1d_thin_kernel: one input channel per output channel (depthwise, or a single
//    sequence).  There is no channel contraction, so this is plain VALU work bounded by
//    HBM: a lane keeps a window of 16 + k - 1 consecutive inputs in registers and slides
//    the k taps (held in scalar registers) over it, producing 16 consecutive outputs.
//    Global traffic is coalesced 128-bit strips; LDS turns strips into per-lane windows
//    and the per-lane outputs back into strips.
//
//  * conv1d_thin_dilated_kernel: the same with taps spaced d > 1 apart.  A dilated
//    correlation is d independent undilated ones on the phase subsequences x[p + d*m], so the
//    tile is staged phase-major in LDS and a lane slides the taps over a register window of
//    one phase, exactly as above; outputs return through LDS to coalesced strips.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerWg = kThreads / kWave;
constexpr int kTileOut = 1024;                       // outputs per wave tile (16 per lane)

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// LDS layout of a wave tile: element q lives at q + 4*(q >> 4) — 4 floats of padding after every
// 16.  A lane's window (16 + k - 1 consecutive elements from 16*lane) then starts 20 floats after
// its neighbour's, so the 128-bit reads of eight consecutive lanes fall on eight different bank
// quads, and every access of a lane is one base address plus a compile-time offset.  Strips
// (lane l at 4*l) see one two-way conflict per eight lanes.
__host__ __device__ constexpr int lds_pos(int q) { return q + 4 * (q >> 4); }

// RULE: the row is extended by `pad` elements in front and p_hi - L behind under the boundary rule
// `pmode` (mirror, periodic, edge) instead of zeros; only the tiles at the ends of a row differ.
// STREAM: the tiles' strips are loaded streamed (non-temporal) — inputs far beyond the caches.
template <int KB4, bool RULE, bool STREAM = false>
__global__ __launch_bounds__(kThreads, (KB4 <= 8 ? 5 : 4)) void conv1d_thin_kernel(
    const float *__restrict__ x, const float *__restrict__ wgt, float *__restrict__ y, int L, int Lo, int k,
    int pad, int Cin, int Cout, int cog, int tiles_per_row, int group, int chunks_per_row, int64_t n_units,
    int wflip, int p_hi, int pmode)
{
    constexpr int K4 = 4 * KB4;                      // taps, zero-padded to a multiple of 4
    constexpr int NI = kTileOut + K4;                // staged inputs per tile
    constexpr int NG = KB4 + 4;                      // 4-float groups in a lane's window
    constexpr int REGION = (lds_pos(NI) + 63) / 64 * 64;
    __shared__ __attribute__((aligned(16))) float lds[kWavesPerWg * REGION];

    const int64_t unit = xcd_unit(n_units);
    if (unit < 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float *A = lds + wave * REGION;
    const int64_t ro = unit / chunks_per_row;        // output row = b*Cout + co
    const int chunk = (int)(unit - ro * chunks_per_row);
    const int64_t b = ro / Cout;
    const int co = (int)(ro - b * Cout);
    const float *xr = x + (b * Cin + co / cog) * (int64_t)L;
    const float *wr = wgt + (int64_t)co * k;
    float *yr = y + ro * (int64_t)Lo;
    // Tile origins are pulled back by c so that (ro*Lo + t0) is a multiple of 16 floats: every
    // 1 KB strip store starts on a 64-byte line of y.  Outputs before the row start are dropped.
    const int c = (int)((ro * Lo) & 15);

    // Taps: one coalesced load (lane t holds tap t, zero beyond k), then broadcast into scalar registers.
    float f[K4];
    {
        float tv = wr[lane < k ? (wflip ? k - 1 - lane : lane) : 0];   // wflip: the adjoint's taps, last first
        tv = lane < k ? tv : 0.0f;
#pragma unroll
        for (int t = 0; t < K4; ++t) f[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(tv), t));
    }

    const int wbase = 20 * lane;                     // my window: lds_pos(16*lane + 4u) = wbase + 4u + 4*(u >> 2)
    const int sbase = 4 * lane + 4 * (lane >> 2);    // my strip element: lds_pos(256j + 4*lane) = sbase + 320j

    // Strips of one tile (inputs [p0, p0 + NI)): 4 full strips plus the k-1 halo, zero outside the row.
    auto load_tile = [&](int t, v4f (&g)[5]) {
        const int p0 = t * kTileOut - c - pad;
        if (p0 >= 0 && p0 <= L - NI) {
            // (streamed loads on inputs far beyond the caches, as in the sliding-sum scan kernel; the halo strip, which
            // the next tile reads again, stays a plain load)
            // (A template parameter: two run-time branches that differ in nothing but the hint are merged by the
            // compiler into plain loads.)
            if constexpr (STREAM) {
#pragma unroll
                for (int j = 0; j < 4; ++j) g[j] = __builtin_nontemporal_load((const v4f_u *)(xr + p0 + j * 256 + 4 * lane));
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) g[j] = *(const v4f_u *)(xr + p0 + j * 256 + 4 * lane);
            }
            g[4] = (4 * lane < K4) ? *(const v4f_u *)(xr + p0 + kTileOut + 4 * lane) : (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        } else {
            // a tile at an end of its row: strip by strip (wave-uniform tests) — whole strips inside
            // the row are still 128-bit loads, strips wholly outside are zero
#pragma unroll
            for (int j = 0; j < 5; ++j) {
                const int s0 = p0 + j * 256;
                const int p = s0 + 4 * lane;
                if (s0 >= 0 && s0 + 256 <= L) {
                    g[j] = *(const v4f_u *)(xr + p);
                } else if (RULE) {
                    // virtual elements stand for the row element the rule names; beyond the extended row: zero
                    float e4[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int q = p + u;
                        const int src = (q >= -pad && q < p_hi) ? pad_src(q + pad, L, pad, pmode) : -1;
                        e4[u] = src >= 0 ? xr[src] : 0.0f;
                    }
                    g[j] = (v4f){e4[0], e4[1], e4[2], e4[3]};
                } else if (s0 >= L || s0 + 256 <= 0) {
                    g[j] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
                } else {
                    g[j].x = (p + 0 >= 0 && p + 0 < L) ? xr[p + 0] : 0.0f;
                    g[j].y = (p + 1 >= 0 && p + 1 < L) ? xr[p + 1] : 0.0f;
                    g[j].z = (p + 2 >= 0 && p + 2 < L) ? xr[p + 2] : 0.0f;
                    g[j].w = (p + 3 >= 0 && p + 3 < L) ? xr[p + 3] : 0.0f;
                }
            }
        }
    };

    int t_end = (chunk + 1) * group;
    if (t_end > tiles_per_row) t_end = tiles_per_row;
    int t = chunk * group + wave;
    v4f cur[5];
    if (t < t_end) load_tile(t, cur);
    for (; t < t_end; t += kWavesPerWg) {
        const int t0 = t * kTileOut - c;             // first output of the tile (may be < 0 for t = 0)
        // ---- the next tile's loads go out before this tile's arithmetic
        v4f nxt[5];
        if (t + kWavesPerWg < t_end) load_tile(t + kWavesPerWg, nxt);
        // ---- stage: strips -> LDS
#pragma unroll
        for (int j = 0; j < 4; ++j) *(v4f *)(A + sbase + 320 * j) = cur[j];
        if (4 * lane < K4) *(v4f *)(A + sbase + 1280) = cur[4];
        wave_lds_sync();
        // ---- my window: inputs 16*lane .. 16*lane + K4 + 15
        float xw[K4 + 16];
#pragma unroll
        for (int u = 0; u < NG; ++u) {
            const v4f g = *(const v4f *)(A + wbase + 4 * u + 4 * (u >> 2));
            xw[4 * u] = g.x; xw[4 * u + 1] = g.y; xw[4 * u + 2] = g.z; xw[4 * u + 3] = g.w;
        }
        // ---- slide the taps: acc[e] = sum_t f[t] * x[e + t]
        float acc[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
#pragma unroll
        for (int tt = 0; tt < K4; ++tt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = fmaf(f[tt], xw[e + tt], acc[e]);
        wave_lds_sync();                             // every lane has its window: A may be reused
        // ---- per-lane outputs -> strips
#pragma unroll
        for (int u = 0; u < 4; ++u)
            *(v4f *)(A + wbase + 4 * u) = (v4f){acc[4 * u], acc[4 * u + 1], acc[4 * u + 2], acc[4 * u + 3]};
        wave_lds_sync();
        const int lim = Lo - t0;
        const int qlo = t0 < 0 ? -t0 : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = j * 256 + 4 * lane;
            if (q >= lim) continue;
            const v4f o = *(const v4f *)(A + sbase + 320 * j);
            if (q >= qlo && q + 4 <= lim) {
                __builtin_nontemporal_store(o, (v4f_u *)(yr + t0 + q));
            } else {
                if (q + 0 >= qlo && q + 0 < lim) yr[t0 + q + 0] = o.x;
                if (q + 1 >= qlo && q + 1 < lim) yr[t0 + q + 1] = o.y;
                if (q + 2 >= qlo && q + 2 < lim) yr[t0 + q + 2] = o.z;
                if (q + 3 >= qlo && q + 3 < lim) yr[t0 + q + 3] = o.w;
            }
        }
        wave_lds_sync();
#pragma unroll
        for (int j = 0; j < 5; ++j) cur[j] = nxt[j];
    }
}

template <int KB4, bool RULE = false>
hipError_t launch_thin(const float *x, const float *wgt, float *y, int64_t rows_out, int L, int Lo, int k, int pad,
                       int Cin, int Cout, int cog, hipStream_t s, int wflip, int p_hi = 0, int pmode = 0)
{
    const int tiles_per_row = (Lo + max_origin_shift(Lo, 16) + kTileOut - 1) / kTileOut;     // origins move back
    // Tiles per workgroup (measured): two per wavefront while HBM is the bound (the tiles in flight
    // stay a compact window of memory), many once the FMAs dominate (k > 32: fewer prologues).
    // (With streamed loads four per wavefront measured 2.5 % faster when the layer's launches follow each other, 0.833
    // against 0.855 ms on cfg 5's k = 31 layer, but 1 % slower between other kernels, 0.779 against 0.771: not taken.)
    const bool stream = !RULE && rows_out * (int64_t)L >= ((int64_t)1 << 27) && !(g_opt.slide_chunk & 256);
    int64_t g = (KB4 <= 8 ? 2 : 16) * kWavesPerWg;
    if (g_opt.slide_group > 0) g = g_opt.slide_group;
    if (g > tiles_per_row) g = tiles_per_row;
    const int chunks_per_row = (int)((tiles_per_row + g - 1) / g);
    const int group = (tiles_per_row + chunks_per_row - 1) / chunks_per_row;     // even chunks
    const int64_t n_units = rows_out * chunks_per_row;
    const int64_t grid = xcd_grid(n_units);
    if (grid > 2147483647LL) return kNotTaken;
    // inputs far beyond the caches are loaded streamed (slide_chunk bit 256: plain loads, as for the sliding sums)
    if constexpr (!RULE) {
        if (stream) {
            hipLaunchKernelGGL((conv1d_thin_kernel<KB4, false, true>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, wgt, y, L,
                               Lo, k, pad, Cin, Cout, cog, tiles_per_row, group, chunks_per_row, n_units, wflip, p_hi, pmode);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((conv1d_thin_kernel<KB4, RULE>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, wgt, y, L, Lo, k,
                       pad, Cin, Cout, cog, tiles_per_row, group, chunks_per_row, n_units, wflip, p_hi, pmode);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------
// Dilated thin convolution.  A wave tile is TO = 16*d*G consecutive outputs (G = 64 / d lanes per
// phase); lane (p, g) produces the 16 outputs p + d*(16g + e), e < 16, which need phase p of the
// input at indices 16g .. 16g + 15 + k - 1.  LDS holds the tile phase-major: input q of the tile
// (phase q % d, index m = q / d) lives at  (q % d) * MP + m + 4*(m >> 4)  — 4 floats of padding
// per 16 keep the 128-bit window reads of neighbouring lanes on different banks.  Where each
// element of each staged strip goes does not depend on the tile, so the workgroup computes that
// table once (in LDS) and every tile's scatter is a table read plus four 32-bit writes.
// Outputs travel back at q + 4*(q / (16 d)): a lane's 16 outputs are base + d*e, and the lanes of
// one phase start 16d + 4 floats apart (different banks).
constexpr int kDilSliceMax = 3072;                   // floats of LDS per wavefront
constexpr int kDilMaxD = 64;

struct DilPlan {
    int d, G, MP, slice, TO, NI, tab_strips;
    float inv_d, inv_16d;
    int wadj;                                        // weights read as the adjoint's (see the kernel)
    int wstride, wofs, accum;                        // a chunk of a longer kernel: taps per channel pair in memory,
                                                     // first tap of this launch, add to what y already holds
};

// MULTI: every output channel sums over the `cig` input channels of its group (few dense channels,
// grouped convolution): the tile of each input channel is staged in turn and the taps of the
// (output channel, input channel) pair are broadcast anew, all accumulating into the same
// registers.  With MULTI the spacing d may be 1 (one phase).
//
// STRIDED (taps adjacent, outputs `d` inputs apart — here d is the stride): the staged tile is
// phase-major in the same way, but now a lane's 16 consecutive outputs draw on every phase: output
// i, tap r + j*d reads phase r at index i + j.  So the lane walks the phases, each with its own
// window and its own taps (every d-th tap from r on); KB4 then counts the taps of ONE phase.
template <int KB4, bool MULTI, bool STRIDED>
__global__ __launch_bounds__(kThreads) void conv1d_thin_dilated_kernel(
    const float *__restrict__ x, const float *__restrict__ wgt, float *__restrict__ y, int L, int Lo, int k,
    int pad, DilPlan pl, int Cin, int Cout, int cog, int cig, int tiles_per_row, int group, int chunks_per_row,
    int64_t n_units)
{
    constexpr int K4 = 4 * KB4;
    constexpr int NG = KB4 + 4;
    extern __shared__ __attribute__((aligned(16))) float lds_dyn[];

    const int64_t unit = xcd_unit(n_units);
    if (unit < 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int4 *tab = (int4 *)lds_dyn;                     // [tab_strips][64]: LDS offsets of a strip's 4 elements
    float *A = lds_dyn + pl.tab_strips * 256 + wave * pl.slice;
    const int64_t ro = unit / chunks_per_row;
    const int chunk = (int)(unit - ro * chunks_per_row);
    const int64_t b = ro / Cout;
    const int co = (int)(ro - b * Cout);
    const float *xg = x + (b * Cin + (int64_t)(co / cog) * cig) * (int64_t)L;     // first input channel of my group
    // Plain view: wgt[co][ci][wofs + t].  Adjoint view (pl.wadj; this launch maps output gradients
    // back to the input): my output channel is the stored array's input channel a = co % cog of
    // group co / cog, my input channel ci its output channel, the taps run backwards:
    // wgt[(group*cig + ci)][a][wstride - 1 - wofs - t].
    const int64_t w_sci = pl.wadj ? (int64_t)cog * pl.wstride : pl.wstride;
    const float *wr = wgt + (pl.wadj ? ((int64_t)(co / cog) * cig * cog + co % cog) * pl.wstride + pl.wstride - 1 - pl.wofs
                                     : (int64_t)co * cig * pl.wstride + pl.wofs);
    const int w_st = pl.wadj ? -1 : 1;
    float *yr = y + ro * (int64_t)Lo;
    const int c = (int)((ro * Lo) & 15);             // 64-byte-aligned strip stores, as in the undilated kernel
    const int d = pl.d, MP = pl.MP, TO = pl.TO, NI = pl.NI;

    // ---- scatter table: element q of the tile -> its phase-major LDS offset; elements the tile does
    //      not need go to a per-lane dummy slot at the end of the slice
    {
        const int dummy = pl.slice - 64 + lane;
        for (int idx = threadIdx.x; idx < pl.tab_strips * 64; idx += kThreads) {
            const int q = (idx >> 6) * 256 + 4 * (idx & 63);
            int m = (int)(((float)q + 0.5f) * pl.inv_d);      // q / d, exact for q < 2^20
            int p = q - m * d;
            int a[4];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                a[cc] = (q + cc < NI) ? p * MP + m + 4 * (m >> 4) : dummy;
                if (++p == d) { p = 0; ++m; }
            }
            tab[idx] = make_int4(a[0], a[1], a[2], a[3]);
        }
    }

    // Taps: one coalesced load (lane t holds tap t, zero beyond k), then broadcast into scalar registers.
    float f[K4];
    auto load_taps = [&](int ci) {
        const float tv = wr[ci * w_sci + (lane < k ? lane : 0) * w_st];
        return lane < k ? tv : 0.0f;
    };
    auto spread_taps = [&](float tv) {
#pragma unroll
        for (int t = 0; t < K4; ++t) f[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(tv), t));
    };
    // every d-th tap from r on (strided mode): phase r's taps
    auto spread_phase_taps = [&](float tv, int r) {
#pragma unroll
        for (int j = 0; j < K4; ++j) {
            const int idx = r + j * d;               // wave-uniform
            const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(tv), idx < 64 ? idx : 63));
            f[j] = idx < k ? v : 0.0f;
        }
    };
    float tv_one = 0.0f;                             // the tap vector when there is one input channel
    if (!MULTI) {
        tv_one = load_taps(0);
        if (!STRIDED) spread_taps(tv_one);
    }

    const int ph = STRIDED ? 0 : lane / pl.G, gl = STRIDED ? lane : lane - ph * pl.G;
    const bool active = STRIDED ? lane < pl.G : lane < d * pl.G;
    const int wbase = active ? ph * MP + 20 * gl : 0;
    const int obase = STRIDED ? 20 * lane : ph + (16 * d + 4) * gl;   // my outputs on their way back
    const int n_strips = (NI + 255) >> 8;
    int rpos[4];                                     // my strip groups on their way out
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int q = j * 256 + 4 * lane;
        if (STRIDED) rpos[j] = q < TO ? q + 4 * (q >> 4) : 0;
        else rpos[j] = q < TO ? q + 4 * (int)(((float)q + 0.5f) * pl.inv_16d) : 0;
    }
    __syncthreads();                                 // table complete

    int t_end = (chunk + 1) * group;
    if (t_end > tiles_per_row) t_end = tiles_per_row;
    for (int t = chunk * group + wave; t < t_end; t += kWavesPerWg) {
        const int t0 = t * TO - c;
        const int p0 = (STRIDED ? t0 * d : t0) - pad;    // global index of tile input 0
        float acc[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
        float tv_next = MULTI ? load_taps(0) : 0.0f;
        for (int ci = 0; ci < (MULTI ? cig : 1); ++ci) {
        const float *xr = xg + (int64_t)ci * L;
        float tv_cur = tv_one;
        if (MULTI) {
            tv_cur = tv_next;
            if (!STRIDED) spread_taps(tv_cur);
            tv_next = load_taps(ci + 1 < cig ? ci + 1 : ci);       // in flight during this channel's work
        }
        // ---- stage: coalesced strips -> phase-major LDS, four strips in flight at a time
        for (int j0 = 0; j0 < n_strips; j0 += 4) {
            v4f g4[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                if (j0 + jj >= n_strips) break;      // wave-uniform
                const int pg = p0 + (j0 + jj) * 256 + 4 * lane;
                int pc = pg < 0 ? 0 : pg;
                pc = pc > L - 4 ? L - 4 : pc;        // always a legal address (L >= 4)
                g4[jj] = *(const v4f_u *)(xr + pc);
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                if (j0 + jj >= n_strips) break;
                const int pg = p0 + (j0 + jj) * 256 + 4 * lane;
                const int4 ad = tab[(j0 + jj) * 64 + lane];
                float e[4] = {g4[jj].x, g4[jj].y, g4[jj].z, g4[jj].w};
                if (pg < 0 || pg > L - 4) {          // row border: pick the wanted elements, zero outside
                    int pc = pg < 0 ? 0 : pg;
                    pc = pc > L - 4 ? L - 4 : pc;
                    const int sft = pg - pc;
                    float r[4];
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) {
                        const int want = cc + sft;   // index into the loaded group
                        float v = 0.0f;
                        v = want == 0 ? e[0] : v;
                        v = want == 1 ? e[1] : v;
                        v = want == 2 ? e[2] : v;
                        v = want == 3 ? e[3] : v;
                        r[cc] = (pg + cc >= 0 && pg + cc < L) ? v : 0.0f;
                    }
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) e[cc] = r[cc];
                }
                A[ad.x] = e[0];
                A[ad.y] = e[1];
                A[ad.z] = e[2];
                A[ad.w] = e[3];
            }
        }
        wave_lds_sync();
        // ---- my window: phase ph, indices 16*gl .. 16*gl + K4 + 15 (strided: every phase in turn)
        for (int r = 0; r < (STRIDED ? d : 1); ++r) {
            if (STRIDED) spread_phase_taps(tv_cur, r);
            float xw[K4 + 16];
#pragma unroll
            for (int u = 0; u < NG; ++u) {
                const v4f g = *(const v4f *)(A + wbase + r * MP + 4 * u + 4 * (u >> 2));
                xw[4 * u] = g.x; xw[4 * u + 1] = g.y; xw[4 * u + 2] = g.z; xw[4 * u + 3] = g.w;
            }
#pragma unroll
            for (int tt = 0; tt < K4; ++tt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[e] = fmaf(f[tt], xw[e + tt], acc[e]);
        }
        wave_lds_sync();                             // every lane has its window: the slice may be reused
        }
        // ---- outputs p + d*(16 gl + e) -> LDS -> strips
        if (STRIDED) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                *(v4f *)(A + obase + 4 * u) = (v4f){acc[4 * u], acc[4 * u + 1], acc[4 * u + 2], acc[4 * u + 3]};
        } else if (active) {
            int o = obase;
#pragma unroll
            for (int e = 0; e < 16; ++e) { A[o] = acc[e]; o += d; }
        }
        wave_lds_sync();
        int lim = Lo - t0;
        if (lim > TO) lim = TO;
        const int qlo = t0 < 0 ? -t0 : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = j * 256 + 4 * lane;
            if (q >= lim) continue;
            v4f o = *(const v4f *)(A + rpos[j]);
            if (q >= qlo && q + 4 <= lim) {
                if (pl.accum) o += *(const v4f_u *)(yr + t0 + q);
                __builtin_nontemporal_store(o, (v4f_u *)(yr + t0 + q));
            } else {
                if (q + 0 >= qlo && q + 0 < lim) yr[t0 + q + 0] = pl.accum ? yr[t0 + q + 0] + o.x : o.x;
                if (q + 1 >= qlo && q + 1 < lim) yr[t0 + q + 1] = pl.accum ? yr[t0 + q + 1] + o.y : o.y;
                if (q + 2 >= qlo && q + 2 < lim) yr[t0 + q + 2] = pl.accum ? yr[t0 + q + 2] + o.z : o.z;
                if (q + 3 >= qlo && q + 3 < lim) yr[t0 + q + 3] = pl.accum ? yr[t0 + q + 3] + o.w : o.w;
            }
        }
        wave_lds_sync();
    }
}

// Tile geometry of the dilated kernel; false if the tile does not fit a wavefront's LDS slice.
bool plan_dilated(int d, int K4, DilPlan *pl)
{
    if (d < 1 || d > kDilMaxD) return false;
    pl->d = d;
    pl->G = 64 / d;
    const int M = 16 * pl->G + K4;                   // staged indices per phase
    int MP = M + 4 * ((M + 15) / 16);
    if (((MP / 4) & 1) == 0) MP += 4;                // odd number of bank quads between phases
    pl->MP = MP;
    pl->TO = 16 * d * pl->G;
    pl->NI = d * M;
    const int out_floats = pl->TO + 4 * pl->G;       // the output exchange reuses the slice
    pl->slice = (d * MP > out_floats ? d * MP : out_floats) + 64;   // + one dummy slot per lane
    pl->tab_strips = ((pl->NI + 255) / 256 + 3) & ~3;
    pl->inv_d = 1.0f / (float)d;
    pl->inv_16d = 1.0f / (float)(16 * d);
    pl->wstride = 0;
    pl->wofs = 0;
    pl->wadj = 0;
    pl->accum = 0;
    return pl->slice <= kDilSliceMax;
}

// Tile geometry of the strided mode: `s` phases of the staged input, as many lanes (16 outputs each)
// as fit the slice; K4 = taps of one phase, padded to a multiple of 4.
bool plan_strided(int s, int K4, DilPlan *pl)
{
    if (s < 2 || s > kDilMaxD) return false;
    int nl = 64;
    int MP = 0;
    for (; nl >= 4; --nl) {
        const int M = 16 * nl + K4;
        MP = M + 4 * ((M + 15) / 16);
        if (((MP / 4) & 1) == 0) MP += 4;
        if (s * MP + 64 <= kDilSliceMax) break;
    }
    if (nl < 4) return false;
    pl->d = s;
    pl->G = nl;                                      // active lanes
    pl->MP = MP;
    pl->TO = 16 * nl;
    pl->NI = s * (16 * nl + K4);
    const int out_floats = 1344;                     // 64 lanes x 20 floats + a strip's reach
    pl->slice = (s * MP > out_floats ? s * MP : out_floats) + 64;
    pl->tab_strips = ((pl->NI + 255) / 256 + 3) & ~3;
    pl->inv_d = 1.0f / (float)s;
    pl->inv_16d = 0.0f;
    pl->wstride = 0;
    pl->wofs = 0;
    pl->wadj = 0;
    pl->accum = 0;
    return pl->slice <= kDilSliceMax + 64;
}

template <int KB4>
hipError_t launch_thin_dilated(const float *x, const float *wgt, float *y, int64_t rows_out, int L, int Lo, int k,
                               int pad, const DilPlan &pl, int Cin, int Cout, int cog, int cig, hipStream_t s,
                               bool strided = false)
{
    const int tiles_per_row = (Lo + max_origin_shift(Lo, 16) + pl.TO - 1) / pl.TO;
    int64_t g = (KB4 <= 8 ? 4 : 8) * kWavesPerWg;    // the scatter table is built once per workgroup
    while (g > kWavesPerWg && rows_out * ((tiles_per_row + g - 1) / g) < 2048) g /= 2;   // small problems: more workgroups
    if (g_opt.slide_group > 0) g = g_opt.slide_group;
    if (g > tiles_per_row) g = tiles_per_row;
    const int chunks_per_row = (int)((tiles_per_row + g - 1) / g);
    const int group = (tiles_per_row + chunks_per_row - 1) / chunks_per_row;     // even chunks
    const int64_t n_units = rows_out * chunks_per_row;
    const int64_t grid = xcd_grid(n_units);
    if (grid > 2147483647LL) return kNotTaken;
    const size_t lds_bytes = ((size_t)pl.tab_strips * 256 + (size_t)kWavesPerWg * pl.slice) * sizeof(float);
#define SWS_DIL_LAUNCH(MULTI, STRIDED)                                                                          \
    hipLaunchKernelGGL((conv1d_thin_dilated_kernel<KB4, MULTI, STRIDED>), dim3((unsigned)grid), dim3(kThreads),  \
                       lds_bytes, s, x, wgt, y, L, Lo, k, pad, pl, Cin, Cout, cog, cig, tiles_per_row, group,    \
                       chunks_per_row, n_units)
    if (strided) {
        if (cig > 1) SWS_DIL_LAUNCH(true, true);
        else SWS_DIL_LAUNCH(false, true);
    } else {
        if (cig > 1) SWS_DIL_LAUNCH(true, false);
        else SWS_DIL_LAUNCH(false, false);
    }
#undef SWS_DIL_LAUNCH
    return hipGetLastError();
}

constexpr int kThinMaxK = 64;

// Dense channels: the vector-ALU kernel against the matrix-core kernel.  Measured on
// x[64, C, 16384], C -> C channels (TFLOP/s, vector ALU / matrix cores): k = 51: 52 / 11 (C = 8),
// 58 / 27 (16), 61 / 56 (32), 63 / 87 (64); k = 9: 16 / 11, 23 / 27, 27 / 62, 29 / 101; k = 3:
// 7 / 6, 11 / 19, 13 / 43, 14 / 89.  The vector-ALU rate depends on the taps per staged tile,
// the matrix rate on how much of its 64-channel tile the output channels fill.
// With stride 2 the vector-ALU kernel has half the taps per staged phase: k = 51: 36-44, k = 31:
// 29-38, k = 9: 6-8, k = 3: 2-3, against 10 / 24 / 52 / 80 on the matrix cores for C = 8 / 16 / 32 / 64.
bool prefer_few(int64_t Cin, int64_t Cout, int k, bool strided)
{
    if (Cin % 8 != 0) return true;                   // the matrix kernel stages 8 input channels at a time
    const double cm = (double)(Cout < 64 ? Cout : 64);
    if (strided) {
        const double valu_est = k >= 40 ? 38.0 : (k >= 24 ? 31.0 : (k >= 12 ? 14.0 : (k >= 6 ? 7.0 : 2.5)));
        return valu_est > 1.05 * 1.5 * cm;
    }
    const double valu_est = k >= 24 ? 55.0 : (k >= 12 ? 35.0 : (k >= 6 ? 22.0 : 11.0));
    return valu_est > 1.05 * 1.6 * cm;
}

}  // namespace

hipError_t launch_conv1d(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L,
                         int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad, int32_t dilation,
                         int32_t groups, hipStream_t s, int wadj, bool *taken)
{
    // wadj: wgt is the [Cin, Cout/groups, k] array of the convolution whose adjoint this call
    // evaluates (x holds output gradients); the kernels read it transposed inside each group, taps
    // last first.  The direct-evaluation fallback does not know that view: *taken = false then.
    if (taken) *taken = true;
    int variant = g_opt.conv1d_variant;
    const int cig = (int)(Cin / groups);
    const bool thin_ok = cig == 1 && stride == 1 && dilation == 1 && k <= kThinMaxK;
    const bool dense_ok = groups == 1 && Cin >= 2;
    // The phase-major kernel: taps spaced apart, several input channels per output channel, and — as
    // a chain of launches over chunks of at most 64 taps, each adding to y — kernels of any length.
    const int k_chunk = k <= kThinMaxK ? k : kThinMaxK;
    DilPlan dpl;
    const bool plan_ok = stride == 1 && L >= 4 && (cig > 1 || dilation > 1 || k > kThinMaxK) &&
                         plan_dilated(dilation, 4 * ((k_chunk + 3) / 4), &dpl);
    const bool thin_dil_ok = cig == 1 && plan_ok;
    const bool few_ok = cig > 1 && plan_ok;          // a few input channels per output channel, on the vector ALU
    // strides (taps adjacent): the same kernel walking the phases of the input
    DilPlan spl;
    const int k_phase = (k + stride - 1) / stride;                 // taps of one phase
    const bool strided_ok = !wadj && stride > 1 && dilation == 1 && k <= kThinMaxK && L >= 4 &&
                            plan_strided(stride, 4 * ((k_phase + 3) / 4), &spl);
    if (variant == 2 && !thin_ok) variant = 0;
    if (variant == 4 && !thin_dil_ok) variant = 0;
    if (variant == 3 && !dense_ok) variant = 0;
    if (variant == 6 && !few_ok) variant = 0;
    if (variant == 7 && !strided_ok) variant = 0;
    const bool valu_ok = few_ok || (strided_ok && cig > 1);
    if (variant == 0) {
        if (thin_ok) variant = 2;
        else if (thin_dil_ok) variant = 4;
        else if (dense_ok && !(valu_ok && prefer_few(Cin, Cout, k, stride > 1))) variant = 3;
        else variant = few_ok ? 6 : (strided_ok ? 7 : 1);
    }
    if (variant == 3 && g_opt.conv1d_variant == 0 && !wadj && stride == 1 && dilation == 1) {
        // a few dozen channels: the split-operand kernel that streams the input straight from memory
        bool taken_s = false;
        const hipError_t e = launch_conv1d_split(x, wgt, y, B, Cin, L, Cout, Lo, k, pad, s, &taken_s);
        if (taken_s || e != hipSuccess) return e;
    }
    if (variant == 3) {
        // the dense contraction is the 2-D kernel on images of height 1
        bool taken_m = false;
        const hipError_t e = launch_conv2d_mfma(x, wgt, y, B, Cin, 1, L, Cout, 1, Lo, 1, k, 1, stride, 0, pad, 1, dilation, s, &taken_m, wadj);
        if (taken_m) return e;
        variant = few_ok ? 6 : (strided_ok ? 7 : 1);
    }
    if (variant == 7) {
        const int cog = (int)(Cout / groups);
        spl.wstride = k;
#define SWS_THIN_STR(KB)                                                                                        \
    case KB:                                                                                                    \
        return launch_thin_dilated<KB>(x, wgt, y, B * Cout, (int)L, (int)Lo, k, pad, spl, (int)Cin, (int)Cout, cog, \
                                       cig, s, true)
        switch ((k_phase + 3) / 4) {
            SWS_THIN_STR(1); SWS_THIN_STR(2); SWS_THIN_STR(3); SWS_THIN_STR(4); SWS_THIN_STR(5); SWS_THIN_STR(6);
            SWS_THIN_STR(7); SWS_THIN_STR(8);
        default: break;
        }
#undef SWS_THIN_STR
        variant = 1;
    }
    if (variant == 2) {
        const int cog = (int)(Cout / groups);
#define SWS_THIN(KB)                                                                                            \
    case KB:                                                                                                    \
        return launch_thin<KB>(x, wgt, y, B * Cout, (int)L, (int)Lo, k, pad, (int)Cin, (int)Cout, cog, s, wadj)
        switch ((k + 3) / 4) {
            SWS_THIN(1); SWS_THIN(2); SWS_THIN(3); SWS_THIN(4); SWS_THIN(5); SWS_THIN(6); SWS_THIN(7); SWS_THIN(8);
            SWS_THIN(9); SWS_THIN(10); SWS_THIN(11); SWS_THIN(12); SWS_THIN(13); SWS_THIN(14); SWS_THIN(15);
            SWS_THIN(16);
        default: break;
        }
#undef SWS_THIN
    }
    if (variant == 4 || variant == 6) {
        const int cog = (int)(Cout / groups);
        const int n_chunks = (k + kThinMaxK - 1) / kThinMaxK;
        for (int c = 0; c < n_chunks; ++c) {
            const int first = c * kThinMaxK, kc = (k - first < kThinMaxK) ? k - first : kThinMaxK;
            DilPlan pc = dpl;
            pc.wstride = k;
            pc.wofs = first;
            pc.wadj = wadj;
            pc.accum = c > 0;
            const int pad_c = pad - first * dilation;           // the chunk's first tap sits first * dilation further on
            hipError_t e = kNotTaken;
#define SWS_THIN_DIL(KB)                                                                                        \
    case KB:                                                                                                    \
        e = launch_thin_dilated<KB>(x, wgt, y, B * Cout, (int)L, (int)Lo, kc, pad_c, pc, (int)Cin, (int)Cout, cog,  \
                                    cig, s);                                                                    \
        break
            switch ((kc + 3) / 4) {
                SWS_THIN_DIL(1); SWS_THIN_DIL(2); SWS_THIN_DIL(3); SWS_THIN_DIL(4); SWS_THIN_DIL(5); SWS_THIN_DIL(6);
                SWS_THIN_DIL(7); SWS_THIN_DIL(8); SWS_THIN_DIL(9); SWS_THIN_DIL(10); SWS_THIN_DIL(11);
                SWS_THIN_DIL(12); SWS_THIN_DIL(13); SWS_THIN_DIL(14); SWS_THIN_DIL(15); SWS_THIN_DIL(16);
            default: break;
            }
#undef SWS_THIN_DIL
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    if (wadj) {
        *taken = false;
        return hipSuccess;
    }
    return launch_conv1d_naive(x, wgt, y, B, Cin, L, Cout, Lo, k, stride, pad, dilation, groups, s);
}

// Boundary rules other than zeros.  One input channel per output channel with adjacent taps at stride 1
// (the paper's own 1-D case and the depthwise layers) runs on the sliding kernel, whose end tiles read
// their virtual elements through the rule; zero padding, the same on both sides, is the plain entry
// point's case; every other geometry is evaluated directly.
hipError_t launch_conv1d_padded(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L,
                                int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad_left, int32_t pad_right,
                                int32_t dilation, int32_t groups, int mode, hipStream_t s)
{
    if (mode == SWS_PAD_IDENTITY && pad_left == pad_right)
        return launch_conv1d(x, wgt, y, B, Cin, L, Cout, Lo, k, stride, pad_left, dilation, groups, s);
    const int cig = (int)(Cin / groups), cog = (int)(Cout / groups);
    if (cig == 1 && stride == 1 && dilation == 1 && k <= kThinMaxK && g_opt.conv1d_variant != 1) {
        hipError_t e = kNotTaken;
#define SWS_THIN_RULE(KB)                                                                                       \
    case KB:                                                                                                    \
        e = launch_thin<KB, true>(x, wgt, y, B * Cout, (int)L, (int)Lo, k, pad_left, (int)Cin, (int)Cout, cog, s, 0, \
                                  (int)L + pad_right, mode);                                                    \
        break
        switch ((k + 3) / 4) {
            SWS_THIN_RULE(1); SWS_THIN_RULE(2); SWS_THIN_RULE(3); SWS_THIN_RULE(4); SWS_THIN_RULE(5); SWS_THIN_RULE(6);
            SWS_THIN_RULE(7); SWS_THIN_RULE(8); SWS_THIN_RULE(9); SWS_THIN_RULE(10); SWS_THIN_RULE(11); SWS_THIN_RULE(12);
            SWS_THIN_RULE(13); SWS_THIN_RULE(14); SWS_THIN_RULE(15); SWS_THIN_RULE(16);
        default: break;
        }
#undef SWS_THIN_RULE
        if (e != kNotTaken) return e;
    }
    return launch_conv1d_naive(x, wgt, y, B, Cin, L, Cout, Lo, k, stride, pad_left, dilation, groups, s, mode);
}

}  // namespace sws
