// sws_pool2d_padded — 2-D pooling over planes extended on all four sides by the boundary
// conditions Section 3 names (identity padding, mirroring, periodicity; also the repeated edge):
// the sliding window sum of Eq. 3 down H and along W of the extended plane, which is never
// written to memory.
//
// Work is laid out in the coordinates of the extended plane.  A wavefront takes a band of TH output
// rows of one plane and a tile of TWO output columns, and stages the (TH-1)*sh + kh extended rows by
// (TWO-1)*sw + kw extended columns its windows see in its own LDS slice: every staged cell is read
// from the plane cell that the boundary rule makes it stand for (or holds the operator's identity), so
// the rule costs index arithmetic at staging time only and the two reductions that follow — down H
// into a second LDS array, then along W from there, kh + kw combines per output — need no bounds.
// Interior tiles read each plane cell once (plus the tile halo); a boundary tile re-reads the few rows
// and columns its virtual cells mirror, which the L2 holds.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int OP>
__global__ __launch_bounds__(kThreads) void pool2d_padded_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                 int H, int W, int We, int Ho, int Wo, int kh, int kw,
                                                                 int sh, int sw, int pt, int pl, int mode, int P, int TH,
                                                                 int TWO, int bands, int ctiles, float scale,
                                                                 int64_t n_units, int lds_floats)
{
    using O = Op<OP>;
    extern __shared__ __attribute__((aligned(16))) float lds_all[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t unit = (int64_t)blockIdx.x * kWaves + wave;
    if (unit >= n_units) return;
    // in:  [rows_need][P]  the extended rows er0 .. of the band; position q of a row holds extended column
    //                      ec0 - lead + q, with lead in 0..3 chosen so that plane columns 4g .. 4g+3 sit on
    //                      16-byte aligned positions
    // col: [nr][P]         those rows reduced down H
    const int ct = (int)(unit % ctiles);
    const int64_t pb = unit / ctiles;
    const int64_t plane = pb / bands;
    const int band = (int)(pb - plane * bands);
    const float *xp = x + plane * (int64_t)H * W;
    float *yp = y + plane * (int64_t)Ho * Wo;
    const int ho0 = band * TH;
    const int nr = (ho0 + TH < Ho ? ho0 + TH : Ho) - ho0;
    const int wo0 = ct * TWO;
    const int nwo = (wo0 + TWO < Wo ? wo0 + TWO : Wo) - wo0;
    const int er0 = ho0 * sh, ec0 = wo0 * sw;        // first extended row and column the windows see
    const int rows_need = (nr - 1) * sh + kh;
    const int lead = (((ec0 - pl) % 4) + 4) % 4;
    const int shift = ec0 - pl - lead;               // plane column of position 0 (a multiple of 4)
    const int used = lead + (nwo - 1) * sw + kw;     // positions the windows read
    float *in = lds_all + wave * lds_floats;
    float *col = in + ((TH - 1) * sh + kh) * P;
    const v4f id4 = {O::id(), O::id(), O::id(), O::id()};
    // ---- stage, part 1: the plane columns of the tile in whole groups of four — one 128-bit load and one
    //      128-bit LDS write per group, the boundary rule applied to the row only
    const int c_lo = ec0 - pl > 0 ? ec0 - pl : 0, c_hi = shift + used < W ? shift + used : W;
    const int g_lo = (c_lo + 3) >> 2;
    int g_hi = c_hi >> 2;
    if (g_hi < g_lo) g_hi = g_lo;
    const int ng = g_hi - g_lo;
    if (ng > 0) {
        const int n = rows_need * ng;
        const float inv_ng = 1.0f / (float)ng;
        constexpr int U = 4;
        for (int i0 = 0; i0 < n; i0 += kWave * U) {
            v4f v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                const int r = (int)(((float)i + 0.5f) * inv_ng), g = g_lo + i - r * ng;
                const int sr = pad_src(er0 + r, H, pt, mode);
                const bool ok = i < n && sr >= 0;
                v[u] = *(const v4f_u *)(xp + (ok ? (int64_t)sr * W + 4 * g : 0));
                v[u] = ok ? v[u] : id4;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                const int r = (int)(((float)i + 0.5f) * inv_ng), g = g_lo + i - r * ng;
                if (i < n) *(v4f *)(in + r * P + 4 * g - shift) = v[u];
            }
        }
    }
    // ---- stage, part 2: the positions in front of and behind those groups (virtual columns, ragged ends),
    //      one by one through the boundary rule of both axes
    {
        const int q_front = ng > 0 ? 4 * g_lo - shift : P;   // positions 0 .. q_front - 1
        const int q_back = ng > 0 ? 4 * g_hi - shift : P;    // positions q_back .. P - 1
        const int nrem = q_front + P - q_back;
        const int n = rows_need * nrem;
        const float inv_n = 1.0f / (float)nrem;
        constexpr int U = 4;
        for (int i0 = 0; i0 < n; i0 += kWave * U) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                const int r = (int)(((float)i + 0.5f) * inv_n), e = i - r * nrem;
                const int q = e < q_front ? e : e - q_front + q_back;
                const int ec = ec0 - lead + q;
                const int sr = pad_src(er0 + r, H, pt, mode);
                const int sc = (q >= lead && ec < We) ? pad_src(ec, W, pl, mode) : -1;
                const bool ok = i < n && sr >= 0 && sc >= 0;
                v[u] = xp[ok ? (int64_t)sr * W + sc : 0];
                v[u] = ok ? v[u] : O::id();
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + kWave * u + lane;
                const int r = (int)(((float)i + 0.5f) * inv_n), e = i - r * nrem;
                const int q = e < q_front ? e : e - q_front + q_back;
                if (i < n) in[r * P + q] = v[u];
            }
        }
    }
    wave_lds_sync();
    // ---- down H: col[r][c] = (+)_{a < kh} in[r*sh + a][c], four columns per item
    const int P4 = P >> 2;
    const float inv_p4 = 1.0f / (float)P4;
    for (int item = lane; item < nr * P4; item += kWave) {
        const int r = (int)(((float)item + 0.5f) * inv_p4), g = item - r * P4;
        const float *p = in + r * sh * P + 4 * g;
        v4f acc = *(const v4f *)p;
        int a = 1;
#define SWS_ACC4(v) acc.x = O::f(acc.x, v.x); acc.y = O::f(acc.y, v.y); acc.z = O::f(acc.z, v.z); acc.w = O::f(acc.w, v.w)
        for (; a + 4 <= kh; a += 4) {                // four reads in flight per wait
            const v4f v0 = *(const v4f *)(p + a * P), v1 = *(const v4f *)(p + (a + 1) * P);
            const v4f v2 = *(const v4f *)(p + (a + 2) * P), v3 = *(const v4f *)(p + (a + 3) * P);
            SWS_ACC4(v0); SWS_ACC4(v1); SWS_ACC4(v2); SWS_ACC4(v3);
        }
        for (; a < kh; ++a) {
            const v4f v = *(const v4f *)(p + a * P);
            SWS_ACC4(v);
        }
#undef SWS_ACC4
        *(v4f *)(col + r * P + 4 * g) = acc;
    }
    wave_lds_sync();
    // ---- along W: one output per lane, consecutive lanes on consecutive outputs
    const float inv_wo = 1.0f / (float)nwo;
    for (int item = lane; item < nr * nwo; item += kWave) {
        const int r = (int)(((float)item + 0.5f) * inv_wo), wq = item - r * nwo;
        const float *cr = col + r * P + lead + wq * sw;
        float acc = cr[0];
        int b = 1;
        for (; b + 4 <= kw; b += 4) {
            const float v0 = cr[b], v1 = cr[b + 1], v2 = cr[b + 2], v3 = cr[b + 3];
            acc = O::f(O::f(O::f(O::f(acc, v0), v1), v2), v3);
        }
        for (; b < kw; ++b) acc = O::f(acc, cr[b]);
        if (OP == SWS_OP_ADD) acc *= scale;
        __builtin_nontemporal_store(acc, yp + (int64_t)(ho0 + r) * Wo + wo0 + wq);
    }
}

// ------------------------------------------------------------------------------------------------
// The pooling layers' own shapes — 3 x 3 with one virtual column on the left (stride 1: and one on the
// right), 5 x 5 and 7 x 7 at stride 1 with two / three a side, 2 x 2 stride 2 without virtual columns, rows of
// 4 .. 256 elements in multiples of 4 — without
// LDS: a lane owns four adjacent columns, the W/4 lanes of a group hold one input row, the 64 / (W/4)
// groups of a wavefront take consecutive bands of TH output rows.  A lane keeps the (TH-1)*S + K rows
// of its band in registers (each read from the plane row the boundary rule names), forms the sum down
// H on them, and takes the column beside its four from the neighbouring lane (DPP).  The rule acts on
// rows and columns independently, so a virtual column of the row-reduced values is the reduced value
// of the column it stands for: elements of the same lane (mirror: columns 1 .. 3 for the left edge;
// repeated edge: column 0), or elements of the group's last lane (periodic; one ds_bpermute each) — and
// likewise on the right.  A workgroup is one short-lived wavefront; XCD x takes planes 8q + x.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float lane_before(float v)       // the value held by lane - 1
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_after(float v)        // the value held by lane + 1
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130, 0xf, 0xf, false));
}
__device__ __forceinline__ float from_lane(float v, int src)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(4 * src, __builtin_bit_cast(int, v)));
}

template <int OP, int K, int S, int PW, int TH>
__global__ __launch_bounds__(kWave) void pool2d_padded_rows_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                   int H, int W, int He, int Ho, int Wo, int pt, int mode,
                                                                   int LPR, int G, int lpr_rcp, int64_t planes,
                                                                   float scale)
{
    using O = Op<OP>;
    constexpr int NL = PW;                                           // columns wanted from the lane before
    constexpr int NRT = (S == 1) ? K - 1 - PW : (K - 2 - PW > 0 ? K - 2 - PW : 0);   // ... from the lane after
    constexpr int NOUT = (S == 1) ? 4 : 2;                           // outputs per lane and row
    constexpr int NR = (TH - 1) * S + K;                             // rows of a band
    static_assert(NL <= 3 && NRT <= 3, "the virtual columns of an edge lane are cells of that lane or of the group's other edge lane");
    const int lane = threadIdx.x;
    const int grp = (lane * lpr_rcp) >> 16, l = lane - grp * LPR;    // lane / LPR (exact for lane < 64)
    if (grp >= G) return;
    const int sl = (int)(blockIdx.x >> 3);
    const int64_t plane = (int64_t)blockIdx.y * kXcd + (blockIdx.x & 7);
    if (plane >= planes) return;
    const int ho0 = (sl * G + grp) * TH;                             // first output row of my band
    if (ho0 >= Ho) return;
    const float *xp = x + plane * (int64_t)H * W + 4 * l;
    float *yp = y + plane * (int64_t)Ho * Wo + NOUT * l;
    v4f r[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) {                                   // all loads in flight together
        const int er = ho0 * S + j;                                  // rows past the extended plane feed no stored output
        const int row = er < He ? pad_src(er, H, pt, mode) : 0;
        r[j] = *(const v4f_u *)(xp + (int64_t)row * W);
    }
    const bool first = l == 0, last = l == LPR - 1;
    // the sums down the columns of all TH output rows at once where they share rows (stride 1)
    v4f vs[TH];
    if constexpr (S == 1) {
        windows_shared<K, TH>(r, vs, [](v4f a, v4f b) {
            return (v4f){O::f(a.x, b.x), O::f(a.y, b.y), O::f(a.z, b.z), O::f(a.w, b.w)};
        });
    }
#pragma unroll
    for (int i = 0; i < TH; ++i) {
        float e[NL + 4 + NRT];
        v4f v = r[i * S];
        if constexpr (S == 1) {
            v = vs[i];
        } else {
#pragma unroll
            for (int a = 1; a < K; ++a) {
                v.x = O::f(v.x, r[i * S + a].x); v.y = O::f(v.y, r[i * S + a].y);
                v.z = O::f(v.z, r[i * S + a].z); v.w = O::f(v.w, r[i * S + a].w);
            }
        }
        e[NL] = v.x; e[NL + 1] = v.y; e[NL + 2] = v.z; e[NL + 3] = v.w;
        const float own[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int t = 0; t < NL; ++t) {                                   // column -(t + 1) of my four
            const float nb = lane_before(own[3 - t]);
            float edge = mode == SWS_PAD_MIRROR ? own[t + 1] : own[0];   // mirror: column t + 1; repeated edge: column 0
            if (mode == SWS_PAD_PERIODIC) edge = from_lane(own[3 - t], lane + LPR - 1);   // uniform branch: every lane takes part
            e[NL - 1 - t] = first ? edge : nb;
        }
#pragma unroll
        for (int t = 0; t < NRT; ++t) {                                  // column 4 + t of my four
            const float nb = lane_after(own[t]);
            float edge = mode == SWS_PAD_MIRROR ? own[2 - t] : own[3];   // mirror: column W - 2 - t; repeated edge: W - 1
            if (mode == SWS_PAD_PERIODIC) edge = from_lane(own[t], lane - LPR + 1);
            e[NL + 4 + t] = last ? edge : nb;
        }
        float o[NOUT];
        if constexpr (S == 1) {
            windows_shared<K, NOUT>(e, o, [](float a, float b) { return O::f(a, b); });
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) o[cc] = (OP == SWS_OP_ADD) ? o[cc] * scale : o[cc];
        } else {
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) {
                float acc = e[cc * S];
#pragma unroll
                for (int b = 1; b < K; ++b) acc = O::f(acc, e[cc * S + b]);
                o[cc] = (OP == SWS_OP_ADD) ? acc * scale : acc;
            }
        }
        const int ho = ho0 + i;
        if (ho < Ho) {
            if constexpr (NOUT == 4) __builtin_nontemporal_store((v4f){o[0], o[1], o[2], o[3]}, (v4f_u *)(yp + (int64_t)ho * Wo));
            else {
                __builtin_nontemporal_store(o[0], yp + (int64_t)ho * Wo);
                __builtin_nontemporal_store(o[1], yp + (int64_t)ho * Wo + 1);
            }
        }
    }
}

template <int OP, int K, int S, int PW, int TH>
hipError_t launch_padded_rows(const float *x, float *y, int64_t planes, int H, int W, int He, int Ho, int Wo, int pt,
                              int mode, float scale, hipStream_t s, bool *taken)
{
    const int LPR = W / 4, G = kWave / LPR;
    const int bands = (Ho + TH - 1) / TH;
    const int spp = (bands + G - 1) / G;                             // wavefronts per plane
    const int64_t rounds = (planes + kXcd - 1) / kXcd;
    *taken = rounds <= 65535;
    if (!*taken) return hipSuccess;
    hipLaunchKernelGGL((pool2d_padded_rows_kernel<OP, K, S, PW, TH>), dim3((unsigned)(spp * kXcd), (unsigned)rounds),
                       dim3(kWave), 0, s, x, y, H, W, He, Ho, Wo, pt, mode, LPR, G, (65536 + LPR - 1) / LPR, planes, scale);
    return hipGetLastError();
}

// The same kernel for planes wider than a wavefront's 256 columns.  A wavefront takes a strip of 256 columns of the
// extended plane, of which the two lanes at either end only serve their neighbours (strips overlap by 16 columns and
// yield 240 columns of outputs each).  A lane whose four columns lie outside the plane holds what the rule puts
// there — periodic: the group W columns away; mirror: the four columns the rule points to, loaded as one group and
// reversed; repeated edge: the edge column four times — so every lane finds its neighbours' columns by the same two
// lane shifts, at the plane's edges too.  (Only the lanes next to the plane feed a stored output.)
constexpr int kStripCols = 240, kStripHalo = 8;

template <int OP, int K, int S, int PW, int TH>
__global__ __launch_bounds__(kWave) void pool2d_padded_rows_wide_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                        int H, int W, int He, int Ho, int Wo, int pt,
                                                                        int mode, int nstrips, int64_t planes, float scale)
{
    using O = Op<OP>;
    constexpr int NL = PW;
    constexpr int NRT = (S == 1) ? K - 1 - PW : (K - 2 - PW > 0 ? K - 2 - PW : 0);
    constexpr int NOUT = (S == 1) ? 4 : 2;
    constexpr int NR = (TH - 1) * S + K;
    static_assert(NL <= kStripHalo && NRT <= kStripHalo, "windows reach no further than the lanes a strip gives away");
    const int lane = threadIdx.x;
    const int sl = (int)(blockIdx.x >> 3);                          // (band, strip) of the plane
    const int64_t plane = (int64_t)blockIdx.y * kXcd + (blockIdx.x & 7);
    if (plane >= planes) return;
    const int band = sl / nstrips, strip = sl - band * nstrips;
    const int ho0 = band * TH;
    if (ho0 >= Ho) return;
    const int c = strip * kStripCols - kStripHalo + 4 * lane;       // my four columns (a multiple of 4: wholly in or out)
    const bool inside = c >= 0 && c < W;
    // where an outside lane's columns come from, and how the loaded group is rearranged
    int src = c;
    bool reversed = false, all_first = false, all_last = false;
    if (!inside) {
        if (mode == SWS_PAD_PERIODIC) src = c < 0 ? c + W : c - W;
        else if (mode == SWS_PAD_MIRROR) { src = c < 0 ? -c - 3 : 2 * W - 5 - c; reversed = true; }
        else { src = c < 0 ? 0 : W - 4; all_first = c < 0; all_last = c >= W; }
        src = src < 0 ? 0 : (src > W - 4 ? W - 4 : src);             // (lanes far outside: any valid group)
    }
    const float *xp = x + plane * (int64_t)H * W + src;
    v4f r[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) {                                   // all loads in flight together
        const int er = ho0 * S + j;                                  // rows past the extended plane feed no stored output
        const int row = er < He ? pad_src(er, H, pt, mode) : 0;
        r[j] = *(const v4f_u *)(xp + (int64_t)row * W);
    }
    const bool mine = lane >= kStripHalo / 4 && lane < kWave - kStripHalo / 4 && inside;
    float *yp = y + plane * (int64_t)Ho * Wo + (S == 1 ? c : c / 2);
    // the sums down the columns of all TH output rows at once where they share rows (stride 1)
    v4f vs[TH];
    if constexpr (S == 1) {
        windows_shared<K, TH>(r, vs, [](v4f a, v4f b) {
            return (v4f){O::f(a.x, b.x), O::f(a.y, b.y), O::f(a.z, b.z), O::f(a.w, b.w)};
        });
    }
#pragma unroll
    for (int i = 0; i < TH; ++i) {
        float e[NL + 4 + NRT];
        v4f v = r[i * S];
        if constexpr (S == 1) {
            v = vs[i];
        } else {
#pragma unroll
            for (int a = 1; a < K; ++a) {
                v.x = O::f(v.x, r[i * S + a].x); v.y = O::f(v.y, r[i * S + a].y);
                v.z = O::f(v.z, r[i * S + a].z); v.w = O::f(v.w, r[i * S + a].w);
            }
        }
        // the rearrangement commutes with the sums down the columns: once per output row
        const v4f u = reversed ? (v4f){v.w, v.z, v.y, v.x}
                               : (all_first ? (v4f){v.x, v.x, v.x, v.x} : (all_last ? (v4f){v.w, v.w, v.w, v.w} : v));
        e[NL] = u.x; e[NL + 1] = u.y; e[NL + 2] = u.z; e[NL + 3] = u.w;
        // column -(t + 1) of my four is element 3 - t % 4 of the lane t / 4 + 1 before me: one or two lane shifts
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            const float one = lane_before(e[NL + 3 - (t & 3)]);
            e[NL - 1 - t] = t < 4 ? one : lane_before(one);
        }
#pragma unroll
        for (int t = 0; t < NRT; ++t) {
            const float one = lane_after(e[NL + (t & 3)]);
            e[NL + 4 + t] = t < 4 ? one : lane_after(one);
        }
        float o[NOUT];
        if constexpr (S == 1) {
            windows_shared<K, NOUT>(e, o, [](float a, float b) { return O::f(a, b); });
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) o[cc] = (OP == SWS_OP_ADD) ? o[cc] * scale : o[cc];
        } else {
#pragma unroll
            for (int cc = 0; cc < NOUT; ++cc) {
                float acc = e[cc * S];
#pragma unroll
                for (int b = 1; b < K; ++b) acc = O::f(acc, e[cc * S + b]);
                o[cc] = (OP == SWS_OP_ADD) ? acc * scale : acc;
            }
        }
        const int ho = ho0 + i;
        if (mine && ho < Ho) {
            if constexpr (NOUT == 4) __builtin_nontemporal_store((v4f){o[0], o[1], o[2], o[3]}, (v4f_u *)(yp + (int64_t)ho * Wo));
            else {
                __builtin_nontemporal_store(o[0], yp + (int64_t)ho * Wo);
                __builtin_nontemporal_store(o[1], yp + (int64_t)ho * Wo + 1);
            }
        }
    }
}

template <int OP, int K, int S, int PW, int TH>
hipError_t launch_padded_rows_wide(const float *x, float *y, int64_t planes, int H, int W, int He, int Ho, int Wo, int pt,
                                   int mode, float scale, hipStream_t s, bool *taken)
{
    const int nstrips = (W + kStripCols - 1) / kStripCols;
    const int bands = (Ho + TH - 1) / TH;
    const int64_t spp = (int64_t)bands * nstrips;                    // wavefronts per plane
    const int64_t rounds = (planes + kXcd - 1) / kXcd;
    *taken = rounds <= 65535 && spp * kXcd <= 2147483647LL;
    if (!*taken) return hipSuccess;
    hipLaunchKernelGGL((pool2d_padded_rows_wide_kernel<OP, K, S, PW, TH>), dim3((unsigned)(spp * kXcd), (unsigned)rounds),
                       dim3(kWave), 0, s, x, y, H, W, He, Ho, Wo, pt, mode, nstrips, planes, scale);
    return hipGetLastError();
}

// Band heights as for the kernel without boundary rules: two output rows per lane at stride 1, one at stride 2.
template <int OP>
hipError_t dispatch_padded_rows(const float *x, float *y, int64_t planes, int H, int W, int He, int Ho, int Wo, int kh,
                                int kw, int sh, int sw, int pt, int pl, int pr, int mode, float scale, hipStream_t s,
                                bool *taken)
{
    *taken = false;
    if (kh != kw || sh != sw || (W & 3) || W < 4 || g_opt.pool2d_variant != 0) return hipSuccess;
    if (mode != SWS_PAD_MIRROR && mode != SWS_PAD_PERIODIC && mode != SWS_PAD_EDGE) return hipSuccess;
    if (W > 256) {                                   // strips of 256 columns
        if (kh == 3 && sh == 1 && pl == 1 && pr == 1)
            return launch_padded_rows_wide<OP, 3, 1, 1, 2>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        if (kh == 5 && sh == 1 && pl == 2 && pr == 2)
            return launch_padded_rows_wide<OP, 5, 1, 2, 2>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        if (kh == 7 && sh == 1 && pl == 3 && pr == 3)
            return launch_padded_rows_wide<OP, 7, 1, 3, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        if (kh == 9 && sh == 1 && pl == 4 && pr == 4)
            return launch_padded_rows_wide<OP, 9, 1, 4, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        if (kh == 11 && sh == 1 && pl == 5 && pr == 5)
            return launch_padded_rows_wide<OP, 11, 1, 5, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        if (kh == 13 && sh == 1 && pl == 6 && pr == 6)
            return launch_padded_rows_wide<OP, 13, 1, 6, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        if (kh == 3 && sh == 2 && pl == 1 && Wo == W / 2)
            return launch_padded_rows_wide<OP, 3, 2, 1, 1>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        if (kh == 2 && sh == 2 && pl == 0 && Wo == W / 2)
            return launch_padded_rows_wide<OP, 2, 2, 0, 1>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
        return hipSuccess;
    }
    if (kh == 9 && sh == 1 && pl == 4 && pr == 4 && W >= 64)   // (four and more virtual columns a side: the strip kernel, one strip)
        return launch_padded_rows_wide<OP, 9, 1, 4, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    if (kh == 11 && sh == 1 && pl == 5 && pr == 5 && W >= 64)
        return launch_padded_rows_wide<OP, 11, 1, 5, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    if (kh == 13 && sh == 1 && pl == 6 && pr == 6 && W >= 64)
        return launch_padded_rows_wide<OP, 13, 1, 6, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    if (kh == 3 && sh == 1 && pl == 1 && pr == 1)
        return launch_padded_rows<OP, 3, 1, 1, 2>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    if (kh == 5 && sh == 1 && pl == 2 && pr == 2)
        return launch_padded_rows<OP, 5, 1, 2, 2>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    if (kh == 7 && sh == 1 && pl == 3 && pr == 3)
        return launch_padded_rows<OP, 7, 1, 3, 4>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    if (kh == 3 && sh == 2 && pl == 1 && Wo == W / 2)
        return launch_padded_rows<OP, 3, 2, 1, 1>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    if (kh == 2 && sh == 2 && pl == 0 && Wo == W / 2)
        return launch_padded_rows<OP, 2, 2, 0, 1>(x, y, planes, H, W, He, Ho, Wo, pt, mode, scale, s, taken);
    return hipSuccess;
}

// Direct evaluation for windows whose tile does not fit an LDS slice: one thread per output.
template <int OP>
__global__ __launch_bounds__(kThreads) void pool2d_padded_naive_kernel(const float *__restrict__ x,
                                                                       float *__restrict__ y, int H, int W, int Ho,
                                                                       int Wo, int kh, int kw, int sh, int sw, int pt,
                                                                       int pl, int mode, float scale, int64_t n_out)
{
    using O = Op<OP>;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < n_out; o += stride) {
        const int wo = (int)(o % Wo);
        const int64_t t = o / Wo;
        const int ho = (int)(t % Ho);
        const float *xp = x + (t / Ho) * (int64_t)H * W;
        float acc = O::id();
        for (int a = 0; a < kh; ++a) {
            const int sr = pad_src(ho * sh + a, H, pt, mode);
            if (sr < 0) continue;
            for (int b = 0; b < kw; ++b) {
                const int sc = pad_src(wo * sw + b, W, pl, mode);
                if (sc >= 0) acc = O::f(acc, xp[(int64_t)sr * W + sc]);
            }
        }
        if (OP == SWS_OP_ADD) acc *= scale;
        y[o] = acc;
    }
}

template <int OP>
hipError_t launch_padded(const float *x, float *y, int64_t planes, int H, int W, int He, int We, int Ho, int Wo, int kh,
                         int kw, int sh, int sw, int pt, int pl, int mode, float scale, hipStream_t s)
{
    // Tile sizing.  A slice holds (TH-1)*sh + kh staged rows and TH reduced rows of P floats.  Whole
    // rows of outputs where they fit; otherwise a few output rows per band, the widest pitch the slice
    // then allows (at least 16 outputs per tile) and as many outputs per tile as that pitch covers.
    bool taken = false;
    const hipError_t e = dispatch_padded_rows<OP>(x, y, planes, H, W, He, Ho, Wo, kh, kw, sh, sw, pt, pl, We - W - pl, mode,
                                                  scale, s, &taken);
    if (taken) return e;
    int P = 0, TH = 0, TWO = Wo, ctiles = 1, budget = 0;
    if (g_opt.pool2d_variant != 1) {
        for (const int bytes : {12 * 1024, 16 * 1024}) {
            budget = bytes / 4;
            P = ((Wo - 1) * sw + kw + 3 + 3) / 4 * 4;   // up to three positions in front for alignment
            TWO = Wo;
            ctiles = 1;
            TH = (int)(((int64_t)budget / P - (kh - sh)) / (sh + 1));
            if (TH > Ho) TH = Ho;
            if (TH < 1 || (g_opt.pool2d_variant == 2 && Wo > 16)) {
                for (TH = Ho < 4 ? Ho : 4; TH >= 1; --TH) {
                    P = budget / ((TH - 1) * sh + kh + TH) / 4 * 4;
                    if (P >= kw + 15 * sw + 3) break;
                }
                if (TH >= 1) {
                    if (g_opt.pool2d_variant == 2) P = (kw + 15 * sw + 3 + 3) / 4 * 4;   // test knob: the narrowest tiles
                    TWO = (P - 3 - kw) / sw + 1;
                    if (TWO > Wo) TWO = Wo;
                    ctiles = (Wo + TWO - 1) / TWO;
                }
            }
            if (TH >= 1) break;
        }
    }
    const int64_t n_out = planes * Ho * Wo;
    if (TH >= 1) {
        const int bands0 = (Ho + TH - 1) / TH;
        TH = (Ho + bands0 - 1) / bands0;             // even bands
        const int bands = (Ho + TH - 1) / TH;
        const int lds_floats = ((TH - 1) * sh + kh + TH) * P;
        const int64_t n_units = planes * bands * ctiles;
        const int64_t grid = (n_units + kWaves - 1) / kWaves;
        if (lds_floats <= budget && grid <= 2147483647LL && (int64_t)((TH - 1) * sh + kh) * P < (1 << 20)) {
            hipLaunchKernelGGL((pool2d_padded_kernel<OP>), dim3((unsigned)grid), dim3(kThreads),
                               (size_t)lds_floats * 4 * kWaves, s, x, y, H, W, We, Ho, Wo, kh, kw, sh, sw, pt, pl, mode,
                               P, TH, TWO, bands, ctiles, scale, n_units, lds_floats);
            return hipGetLastError();
        }
    }
    int64_t grid = (n_out + kThreads - 1) / kThreads;
    const int64_t cap = (int64_t)device_cus() * 32;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL((pool2d_padded_naive_kernel<OP>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, H, W, Ho, Wo,
                       kh, kw, sh, sw, pt, pl, mode, scale, n_out);
    return hipGetLastError();
}

}  // namespace

// pool2d_variant: 1 = direct evaluation, 2 = column tiles of the narrowest width (both for tests).
hipError_t launch_pool2d_padded(int op, const float *x, float *y, int64_t planes, int64_t H, int64_t W, int64_t Ho,
                                int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t pt, int32_t pl,
                                int32_t pb, int32_t pr, int mode, float scale, hipStream_t s)
{
    const int He = (int)(H + pt + pb), We = (int)(W + pl + pr);
    // identity padding narrower than the window is the case the tuned pooling kernels cover;
    // shrinking windows are their real-cell divisor
    const bool narrow = pt < kh && pb < kh && pl < kw && pr < kw;
    if (mode == SWS_PAD_SHRINK || (mode == SWS_PAD_IDENTITY && narrow && g_opt.pool2d_variant == 0))
        return launch_pool2d(op, x, y, planes, H, W, Ho, Wo, kh, kw, sh, sw, pt, pl, scale, mode == SWS_PAD_SHRINK, s);
    switch (op) {
    case SWS_OP_ADD:
        return launch_padded<SWS_OP_ADD>(x, y, planes, (int)H, (int)W, He, We, (int)Ho, (int)Wo, kh, kw, sh, sw, pt, pl,
                                         mode, scale, s);
    case SWS_OP_MAX:
        return launch_padded<SWS_OP_MAX>(x, y, planes, (int)H, (int)W, He, We, (int)Ho, (int)Wo, kh, kw, sh, sw, pt, pl,
                                         mode, scale, s);
    default:
        return launch_padded<SWS_OP_MIN>(x, y, planes, (int)H, (int)W, He, We, (int)Ho, (int)Wo, kh, kw, sh, sw, pt, pl,
                                         mode, scale, s);
    }
}

}  // namespace sws
