// Adjoints of 3 x 3 pooling (stride 1 with one column of padding, stride 2 with one or none) and of 2 x 2
// pooling at stride 2 — the backward passes of the row-streaming pooling kernel (Section 2.3 used for
// training), without LDS.  Rows of up to 256 columns fit a wavefront, wider ones go in strips (see locate());
// rows that are not a multiple of 4 long end in a lane that holds fewer than four columns (see Cols).
//
// As in the forward kernel a lane owns four adjacent columns, the W/4 lanes of a group move a row as
// one contiguous run of 128-bit accesses, the G = 64 / (W/4) groups of a wavefront take G consecutive
// bands of TH rows of gx, a wavefront is a workgroup of its own, and XCD b mod 8 takes the planes
// 8q + (b mod 8) band by band.  What a lane needs from beside its columns comes from the neighbouring
// lanes by DPP shifts.
//
// Max pooling: every window's gradient goes to the first cell (row-major) that holds its maximum.
// A band's lane keeps the x rows its windows see; per row it forms, for each of its window columns,
// the maximum of the three cells and WHICH cell it was, as the number 8 * (row of the band) + (column
// among the lane's six, its neighbours' included) — strict comparisons, so the first of equal cells
// wins; three rows combine the same way down H.  A window thus ends up with the number of the one
// cell that receives its gradient, and a cell adds the gradients of the windows whose number is its
// own — no window-relative arithmetic, no range tests: a window that does not contain a cell cannot
// carry its number.  Windows outside the plane are given gradient 0; cells outside the plane hold -inf.
//
// Average pooling at stride 2: the same bands with sums instead of numbers (at stride 1 the adjoint is
// the forward sliding sum over gy and runs on the forward kernels).
#include "sws_internal.h"

namespace sws {

namespace {

typedef v2f v2f_u __attribute__((aligned(4)));

__device__ __forceinline__ float lane_before(float v)       // the value held by lane - 1
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_after(float v)        // the value held by lane + 1
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130, 0xf, 0xf, false));
}
__device__ __forceinline__ int lane_before(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x138, 0xf, 0xf, false); }
__device__ __forceinline__ int lane_after(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x130, 0xf, 0xf, false); }

// Where a wavefront's lane works: group (band) and lane within the row; false = nothing to do.
// Planes wider than 256 columns (nstrips > 0): the wavefront takes one band and a strip of 256 columns of it, of
// which the two lanes at either end only serve their neighbours — strips overlap by 16 columns and write 240.  A
// lane whose columns lie outside the plane holds -inf cells and zero gradients, so there are no edge lanes.
constexpr int kStripCols = 240, kStripHalo = 8;
struct Where {
    int c;                  // my columns: c .. c + 3 (a multiple of 4)
    int r0;                 // first gx row of the band
    int64_t plane;
    bool first, last;       // the row's edge lanes (narrow planes)
    bool inside;            // my columns lie in the plane
    bool store;             // ... and are mine to write
};
__device__ __forceinline__ bool locate(Where &w, int LPR, int G, int lpr_rcp, int TH, int H, int W, int nstrips,
                                       int64_t planes)
{
    const int lane = threadIdx.x;
    w.plane = (int64_t)blockIdx.y * kXcd + (blockIdx.x & 7);        // gridDim.x is a multiple of 8: XCD = x & 7
    if (w.plane >= planes) return false;
    if (nstrips > 0) {
        const int sl = (int)(blockIdx.x >> 3), band = sl / nstrips, strip = sl - band * nstrips;
        w.r0 = band * TH;
        if (w.r0 >= H) return false;
        w.c = strip * kStripCols - kStripHalo + 4 * lane;
        w.inside = w.c >= 0 && w.c < W;
        w.store = w.inside && lane >= kStripHalo / 4 && lane < kWave - kStripHalo / 4;
        w.first = w.last = false;
        return true;
    }
    const int grp = (lane * lpr_rcp) >> 16;                          // lane / LPR (exact for lane < 64)
    const int l = lane - grp * LPR;
    if (grp >= G) return false;
    w.r0 = ((int)(blockIdx.x >> 3) * G + grp) * TH;
    if (w.r0 >= H) return false;
    w.c = 4 * l;
    w.inside = w.store = true;
    w.first = l == 0;
    w.last = l == LPR - 1;
    return true;
}

// A lane's columns in memory.  Rows whose length is not a multiple of 4 (RAG) end inside a lane: that lane
// (part) reads the row's last four elements instead of its own four and shifts them down, so that every lane
// still issues one 128-bit load per row, and writes its nv < 4 columns one by one.
struct Cols {
    int cx;                 // column at which the lane's load starts
    int nv;                 // columns of mine that exist (meaningful where part)
    bool part;
};
template <bool RAG>
__device__ __forceinline__ Cols columns(const Where &w, int W)
{
    Cols k;
    k.part = RAG && w.inside && w.c + 4 > W;
    k.nv = W - w.c;
    k.cx = !w.inside ? 0 : k.part ? W - 4 : w.c;     // (lanes outside the plane read column 0 and drop it)
    return k;
}
template <bool RAG>
__device__ __forceinline__ v4f load4(const float *row, const Cols &k, float fill)
{
    v4f v = *(const v4f_u *)(row + k.cx);
    if constexpr (RAG) {
        const float a = k.nv == 1 ? v.w : k.nv == 2 ? v.z : v.y;
        const float b = k.nv == 1 ? fill : k.nv == 2 ? v.w : v.z;
        const float c = k.nv == 3 ? v.w : fill;
        if (k.part) v = (v4f){a, b, c, fill};
    }
    return v;
}
template <bool RAG>
__device__ __forceinline__ void store4(float *p, const float (&o)[4], const Cols &k)
{
    if (!RAG || !k.part) {
        __builtin_nontemporal_store((v4f){o[0], o[1], o[2], o[3]}, (v4f_u *)p);
    } else {
#pragma unroll
        for (int e = 0; e < 3; ++e)
            if (e < k.nv) p[e] = o[e];
    }
}
// Window columns wo0, wo0 + 1 of a gy row at stride 2; those beyond the row's end read as 0.
__device__ __forceinline__ void load_windows2(const float *row, int wo0, int Wo, bool ok, float &g0, float &g1)
{
    const float a = row[wo0 < Wo ? wo0 : Wo - 1], b = row[wo0 + 1 < Wo ? wo0 + 1 : Wo - 1];
    g0 = (ok && wo0 < Wo) ? a : 0.0f;
    g1 = (ok && wo0 + 1 < Wo) ? b : 0.0f;
}

// One x row -> for each of the lane's NW window columns the maximum of its three cells (hm) and the
// number of the first cell holding it (hc), numbers being base + (column among e[0..5]).
// STEP = 1: windows u = 0..3 see e[u .. u+2]; STEP = 2: windows u = 0, 1 see e[OFF + 2u .. OFF + 2u+2].
template <int STEP, int NW, int OFF>
__device__ __forceinline__ void row_maxima(const float (&e)[6], int base, float (&hm)[NW], int (&hc)[NW])
{
#pragma unroll
    for (int u = 0; u < NW; ++u) {
        const int c = STEP * u + OFF;
        float m = e[c];
        int k = base + c;
        if (e[c + 1] > m) { m = e[c + 1]; k = base + c + 1; }
        if (e[c + 2] > m) { m = e[c + 2]; k = base + c + 2; }
        hm[u] = m;
        hc[u] = k;
    }
}

// ------------------------------------------------------------------------------------------------
// Max pooling, stride S.  gx rows r0 .. r0 + TH - 1 of a plane; TH even for S = 2.
//   S = 1: window row ho covers x rows ho - ph .. + 2; the band's windows are ho = r0 + ph - 2 + i,
//          i < TH + 2, over x rows r0 - 2 + j, j < TH + 4: window i = rows j = i, i+1, i+2; cell row t
//          is j = t + 2 and lies in windows t, t+1, t+2.
//   S = 2: window row ho covers x rows 2 ho - ph .. + 2; windows ho = hf + i, hf = ceil((r0 + ph - 2) / 2),
//          i < TH/2 + 1, over x rows 2 hf - ph + j, j < TH + 3: window i = rows 2i, 2i+1, 2i+2; cell row t
//          is j = d0 + t with d0 = r0 + ph - 2 hf (1 or 2).
// Columns.  S = 1: window wo covers columns wo - 1 .. wo + 1; the lane's windows are wo = 4l + u, u < 4,
//          over e[0..5] = columns 4l - 1 .. 4l + 4; cell v (column 4l + v, e[v + 1]) lies in windows
//          v - 1, v, v + 1, of which u = -1 is the previous lane's u = 3 (where the cell is e[5]) and
//          u = 4 the next lane's u = 0 (where it is e[0]).
//          S = 2, PW = 1: window wo covers columns 2 wo - 1 .. 2 wo + 1; the lane's windows are wo = 2l + u, u < 2,
//          over e[0..4]; cell 0 lies in window 0, cell 1 in 0 and 1, cell 2 in 1, cell 3 in 1 and in the
//          next lane's window 0 (where it is e[0]).
//          S = 2, PW = 0: window wo covers columns 2 wo .. 2 wo + 2, the lane's two windows lie over e[1..5]; cell 0
//          lies in window 0 and in the previous lane's window 1 (where it is e[5]), cell 1 in 0, cell 2 in 0 and 1,
//          cell 3 in 1.  Windows beyond the row's last (wo >= Wo) are given gradient 0.
// ------------------------------------------------------------------------------------------------
template <int S, int TH, int PW, bool RAG>
__global__ __launch_bounds__(kWave) void maxpool_grad_rows_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                  float *__restrict__ gx, int H, int W, int Ho, int Wo,
                                                                  int ph, int LPR, int G, int lpr_rcp, int nstrips,
                                                                  int64_t planes)
{
    static_assert(S == 1 || (S == 2 && TH % 2 == 0), "bands of an even number of rows at stride 2");
    static_assert(PW == 1 || (S == 2 && PW == 0), "stride 1: one column of padding");
    constexpr int NW = S == 1 ? 4 : 2;                               // window columns of a lane
    constexpr int NWR = S == 1 ? TH + 2 : TH / 2 + 1;                // window rows of a band
    constexpr int NXR = S == 1 ? TH + 4 : TH + 3;                    // x rows of a band
    constexpr int OFF = 1 - PW;                                      // e[] index at which the lane's first window starts
    constexpr bool kBefore = S == 1 || PW == 1, kAfter = S == 1 || PW == 0;    // the neighbours' columns a lane sees
    const float ninf = -__builtin_huge_valf();
    Where w;
    if (!locate(w, LPR, G, lpr_rcp, TH, H, W, nstrips, planes)) return;
    const Cols k = columns<RAG>(w, W);
    const int hf = S == 1 ? w.r0 + ph - 2 : (w.r0 + ph - 1) >> 1;    // first window row (may be < 0)
    const int xr0 = S == 1 ? w.r0 - 2 : 2 * hf - ph;                 // first x row (may be < 0)
    const int d0 = S == 1 ? 2 : w.r0 - xr0;                          // cell row t is x row j = d0 + t
    const int cc = w.inside ? w.c : 0;
    const float *xp = x + w.plane * (int64_t)H * W;
    const float *gp = gy + w.plane * (int64_t)Ho * Wo;
    float *op = gx + w.plane * (int64_t)H * W + cc;

    // ---- all loads in flight together; rows and columns outside the plane: -inf cells, zero gradients
    v4f xr[NXR];
#pragma unroll
    for (int j = 0; j < NXR; ++j) {
        const int row = xr0 + j;
        const bool in_rows = row >= 0 && row < H, ok = in_rows && w.inside;
        const v4f v = load4<RAG>(xp + (int64_t)(in_rows ? row : 0) * W, k, ninf);
        xr[j] = ok ? v : (v4f){ninf, ninf, ninf, ninf};
    }
    float g[NWR][NW];
#pragma unroll
    for (int i = 0; i < NWR; ++i) {
        const int ho = hf + i;
        const bool in_rows = ho >= 0 && ho < Ho, ok = in_rows && w.inside;
        const float *src = gp + (int64_t)(in_rows ? ho : 0) * Wo;
        if constexpr (NW == 4) {                                     // (Wo = W: the same columns as x)
            const v4f v = load4<RAG>(src, k, 0.0f);
            g[i][0] = ok ? v.x : 0.0f; g[i][1] = ok ? v.y : 0.0f; g[i][2] = ok ? v.z : 0.0f; g[i][3] = ok ? v.w : 0.0f;
        } else if constexpr (!RAG && PW == 1) {                      // (Wo = W / 2: both windows exist)
            const v2f v = *(const v2f_u *)(src + cc / 2);
            g[i][0] = ok ? v.x : 0.0f; g[i][1] = ok ? v.y : 0.0f;
        } else {
            load_windows2(src, cc / 2, Wo, ok, g[i][0], g[i][1]);
        }
    }

    // ---- per x row: maxima along W with the number of the cell that holds them, folded at once into the
    //      (up to three) windows the row belongs to: down H the first row wins ties.  wn = number of the
    //      cell that receives the window's gradient.
    float wm[NWR][NW];
    int wn[NWR][NW];
#pragma unroll
    for (int j = 0; j < NXR; ++j) {
        float e[6];
        e[0] = ninf; e[1] = xr[j].x; e[2] = xr[j].y; e[3] = xr[j].z; e[4] = xr[j].w; e[5] = ninf;
        if constexpr (kBefore) {
            const float b = lane_before(xr[j].w);
            e[0] = w.first ? ninf : b;
        }
        if constexpr (kAfter) {
            const float a = lane_after(xr[j].x);
            e[5] = w.last ? ninf : a;
        }
        float hm[NW];
        int hc[NW];
        row_maxima<S, NW, OFF>(e, 8 * j, hm, hc);
#pragma unroll
        for (int i = 0; i < NWR; ++i) {
            const int a = j - S * i;                                 // the row's place in window i
            if (a < 0 || a > 2) continue;
#pragma unroll
            for (int u = 0; u < NW; ++u) {
                if (a == 0) {
                    wm[i][u] = hm[u];
                    wn[i][u] = hc[u];
                } else {
                    const bool better = hm[u] > wm[i][u];
                    wm[i][u] = better ? hm[u] : wm[i][u];
                    wn[i][u] = better ? hc[u] : wn[i][u];
                }
            }
        }
    }
    // ---- the windows beside the lane's: the previous lane's last and the next lane's first, where they reach
    //      into the lane's columns
    int wn_b[NWR], wn_a[NWR];
    float g_b[NWR], g_a[NWR];
#pragma unroll
    for (int i = 0; i < NWR; ++i) {
        wn_b[i] = wn_a[i] = 0;
        g_b[i] = g_a[i] = 0.0f;
        if constexpr (S == 1 || PW == 0) {
            wn_b[i] = lane_before(wn[i][NW - 1]);
            const float t = lane_before(g[i][NW - 1]);
            g_b[i] = w.first ? 0.0f : t;
        }
        if constexpr (S == 1 || PW == 1) {
            wn_a[i] = lane_after(wn[i][0]);
            const float t = lane_after(g[i][0]);
            g_a[i] = w.last ? 0.0f : t;
        }
    }
    // ---- every cell adds the gradients of the windows that carry its number
#pragma unroll
    for (int t = 0; t < TH; ++t) {
        const int row = w.r0 + t;
        float o[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int me = 8 * (d0 + t) + v + 1;                     // my number in this lane's numbering
            float acc = 0.0f;
            if constexpr (S == 1) {
#pragma unroll
                for (int di = 0; di < 3; ++di) {
                    const int i = t + di;
#pragma unroll
                    for (int du = 0; du < 3; ++du) {
                        const int u = v - 1 + du;
                        if (u < 0) acc += (wn_b[i] == 8 * (d0 + t) + 5) ? g_b[i] : 0.0f;
                        else if (u > 3) acc += (wn_a[i] == 8 * (d0 + t) + 0) ? g_a[i] : 0.0f;
                        else acc += (wn[i][u] == me) ? g[i][u] : 0.0f;
                    }
                }
            } else if constexpr (PW == 1) {
#pragma unroll
                for (int i = 0; i < NWR; ++i) {
                    if (v <= 1) acc += (wn[i][0] == me) ? g[i][0] : 0.0f;
                    if (v >= 1) acc += (wn[i][1] == me) ? g[i][1] : 0.0f;
                    if (v == 3) acc += (wn_a[i] == 8 * (d0 + t) + 0) ? g_a[i] : 0.0f;
                }
            } else {
#pragma unroll
                for (int i = 0; i < NWR; ++i) {
                    if (v == 0) acc += (wn_b[i] == 8 * (d0 + t) + 5) ? g_b[i] : 0.0f;
                    if (v <= 2) acc += (wn[i][0] == me) ? g[i][0] : 0.0f;
                    if (v >= 2) acc += (wn[i][1] == me) ? g[i][1] : 0.0f;
                }
            }
            o[v] = acc;
        }
        if (row < H && w.store) store4<RAG>(op + (int64_t)row * W, o, k);
    }
}

// ------------------------------------------------------------------------------------------------
// Max pooling, 2 x 2 windows at stride 2 without padding: windows do not overlap, a lane's four columns of two
// rows are two whole windows and nothing comes from a neighbour.  The gradient goes to the first cell
// (row-major) that holds the window's maximum; rows and windows past the last whole window get 0.
// ------------------------------------------------------------------------------------------------
template <int TH, bool RAG>
__global__ __launch_bounds__(kWave) void maxpool_grad_rows_k2s2_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                       float *__restrict__ gx, int H, int W, int Ho, int Wo,
                                                                       int LPR, int G, int lpr_rcp, int nstrips, int64_t planes)
{
    static_assert(TH % 2 == 0, "bands of whole windows");
    Where w;
    if (!locate(w, LPR, G, lpr_rcp, TH, H, W, nstrips, planes)) return;
    const Cols k = columns<RAG>(w, W);
    const int cc = w.inside ? w.c : 0;
    const float *xp = x + w.plane * (int64_t)H * W;
    const float *gp = gy + w.plane * (int64_t)Ho * Wo;
    float *op = gx + w.plane * (int64_t)H * W + cc;
    v4f xr[TH];
    v2f g[TH / 2];
#pragma unroll
    for (int j = 0; j < TH; ++j) {                                   // all loads in flight together
        const int row = w.r0 + j;
        xr[j] = load4<RAG>(xp + (int64_t)(row < H ? row : 0) * W, k, 0.0f);
    }
#pragma unroll
    for (int i = 0; i < TH / 2; ++i) {
        const int ho = (w.r0 >> 1) + i;
        const bool ok = ho < Ho;                                     // (a last odd row belongs to no window)
        const float *src = gp + (int64_t)(ok ? ho : 0) * Wo;
        if constexpr (!RAG) {
            const v2f v = *(const v2f_u *)(src + cc / 2);
            g[i] = ok ? v : (v2f){0.0f, 0.0f};
        } else {                                                     // (a last odd column belongs to no window)
            float g0, g1;
            load_windows2(src, cc / 2, Wo, ok, g0, g1);
            g[i] = (v2f){g0, g1};
        }
    }
#pragma unroll
    for (int i = 0; i < TH / 2; ++i) {
        const float a[4] = {xr[2 * i].x, xr[2 * i].y, xr[2 * i].z, xr[2 * i].w};
        const float b[4] = {xr[2 * i + 1].x, xr[2 * i + 1].y, xr[2 * i + 1].z, xr[2 * i + 1].w};
        const float gg[2] = {g[i].x, g[i].y};
        float oa[4], ob[4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            float m = a[2 * u];
            int k4 = 0;
            if (a[2 * u + 1] > m) { m = a[2 * u + 1]; k4 = 1; }
            if (b[2 * u] > m) { m = b[2 * u]; k4 = 2; }
            if (b[2 * u + 1] > m) { k4 = 3; }
            oa[2 * u] = k4 == 0 ? gg[u] : 0.0f;
            oa[2 * u + 1] = k4 == 1 ? gg[u] : 0.0f;
            ob[2 * u] = k4 == 2 ? gg[u] : 0.0f;
            ob[2 * u + 1] = k4 == 3 ? gg[u] : 0.0f;
        }
        const int row = w.r0 + 2 * i;
        if (w.store && row < H) store4<RAG>(op + (int64_t)row * W, oa, k);
        if (w.store && row + 1 < H) store4<RAG>(op + (int64_t)(row + 1) * W, ob, k);
    }
}

// ------------------------------------------------------------------------------------------------
// Average pooling, stride 2 (same bands): a cell adds f * gy over the windows that contain it.
// ------------------------------------------------------------------------------------------------
template <int TH, int PW, bool RAG>
__global__ __launch_bounds__(kWave) void avgpool_grad_rows_s2_kernel(const float *__restrict__ gy, float *__restrict__ gx,
                                                                     int H, int W, int Ho, int Wo, int ph, int LPR, int G,
                                                                     int lpr_rcp, int nstrips, int64_t planes, float scale)
{
    static_assert(TH % 2 == 0, "bands of an even number of rows");
    constexpr int NWR = TH / 2 + 1;
    Where w;
    if (!locate(w, LPR, G, lpr_rcp, TH, H, W, nstrips, planes)) return;
    const Cols k = columns<RAG>(w, W);
    const int hf = (w.r0 + ph - 1) >> 1;
    const int d0 = w.r0 - (2 * hf - ph);                             // 1 or 2
    const int cc = w.inside ? w.c : 0;
    const float *gp = gy + w.plane * (int64_t)Ho * Wo;
    float *op = gx + w.plane * (int64_t)H * W + cc;
    // per window row: the sums along W that the lane's four cells receive
    float c[NWR][4];
#pragma unroll
    for (int i = 0; i < NWR; ++i) {
        const int ho = hf + i;
        const bool in_rows = ho >= 0 && ho < Ho, ok = in_rows && w.inside;
        const float *src = gp + (int64_t)(in_rows ? ho : 0) * Wo;
        float g0, g1;
        if constexpr (!RAG && PW == 1) {
            const v2f v = *(const v2f_u *)(src + cc / 2);
            g0 = ok ? v.x : 0.0f; g1 = ok ? v.y : 0.0f;
        } else {
            load_windows2(src, cc / 2, Wo, ok, g0, g1);
        }
        g0 *= scale; g1 *= scale;
        if constexpr (PW == 1) {                                     // windows over columns 2 wo - 1 .. 2 wo + 1
            const float t = lane_after(g0);
            const float ga = w.last ? 0.0f : t;
            c[i][0] = g0; c[i][1] = g0 + g1; c[i][2] = g1; c[i][3] = g1 + ga;
        } else {                                                     // windows over columns 2 wo .. 2 wo + 2
            const float t = lane_before(g1);
            const float gb = w.first ? 0.0f : t;
            c[i][0] = gb + g0; c[i][1] = g0; c[i][2] = g0 + g1; c[i][3] = g1;
        }
    }
#pragma unroll
    for (int t = 0; t < TH; ++t) {
        const int row = w.r0 + t;
        const int j = d0 + t;                                        // x row among the band's: windows i with 2i <= j <= 2i + 2
        float o[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float acc = 0.0f;
#pragma unroll
            for (int i = 0; i < NWR; ++i) acc += (2 * i <= j && j <= 2 * i + 2) ? c[i][v] : 0.0f;
            o[v] = acc;
        }
        if (row < H && w.store) store4<RAG>(op + (int64_t)row * W, o, k);
    }
}

// Average pooling, 2 x 2 windows at stride 2 without padding: every cell of a window gets scale * gy of that window;
// a last odd row or column gets 0.
template <int TH, bool RAG>
__global__ __launch_bounds__(kWave) void avgpool_grad_rows_k2s2_kernel(const float *__restrict__ gy, float *__restrict__ gx,
                                                                       int H, int W, int Ho, int Wo, int LPR, int G,
                                                                       int lpr_rcp, int nstrips, int64_t planes, float scale)
{
    static_assert(TH % 2 == 0, "bands of whole windows");
    Where w;
    if (!locate(w, LPR, G, lpr_rcp, TH, H, W, nstrips, planes)) return;
    const Cols k = columns<RAG>(w, W);
    const int cc = w.inside ? w.c : 0;
    const float *gp = gy + w.plane * (int64_t)Ho * Wo;
    float *op = gx + w.plane * (int64_t)H * W + cc;
    v2f g[TH / 2];
#pragma unroll
    for (int i = 0; i < TH / 2; ++i) {
        const int ho = (w.r0 >> 1) + i;
        const bool ok = ho < Ho;
        const float *src = gp + (int64_t)(ok ? ho : 0) * Wo;
        if constexpr (!RAG) {
            const v2f v = *(const v2f_u *)(src + cc / 2);
            g[i] = ok ? (v2f){v.x * scale, v.y * scale} : (v2f){0.0f, 0.0f};
        } else {
            float g0, g1;
            load_windows2(src, cc / 2, Wo, ok, g0, g1);
            g[i] = (v2f){g0 * scale, g1 * scale};
        }
    }
#pragma unroll
    for (int i = 0; i < TH / 2; ++i) {
        const float o[4] = {g[i].x, g[i].x, g[i].y, g[i].y};
        const int row = w.r0 + 2 * i;
        if (w.store && row < H) store4<RAG>(op + (int64_t)row * W, o, k);
        if (w.store && row + 1 < H) store4<RAG>(op + (int64_t)(row + 1) * W, o, k);
    }
}

struct RowsGrid {
    int LPR, G, rcp, nstrips;
    dim3 grid;
    bool ok;
};
RowsGrid rows_grid(int64_t planes, int H, int W, int TH)
{
    RowsGrid r;
    const int bands = (H + TH - 1) / TH;
    const int64_t rounds = (planes + kXcd - 1) / kXcd;
    int64_t spp;                                                     // wavefronts per plane
    if (W > 256) {                                                   // strips of 256 columns
        r.LPR = kWave; r.G = 1; r.rcp = 0;
        r.nstrips = (W + kStripCols - 1) / kStripCols;
        spp = (int64_t)bands * r.nstrips;
    } else {
        r.LPR = (W + 3) / 4;                                         // (a last lane may hold fewer than 4 columns)
        r.G = kWave / r.LPR;
        r.rcp = (65536 + r.LPR - 1) / r.LPR;
        r.nstrips = 0;
        spp = (bands + r.G - 1) / r.G;
    }
    r.ok = rounds <= 65535 && spp * kXcd <= 2147483647LL;
    r.grid = dim3((unsigned)(spp * kXcd), (unsigned)rounds);
    return r;
}

// 3 x 3 windows: stride 1 with one column of padding, stride 2 with one or none; up to two rows of padding.
bool rows_shape(int H, int W, int Ho, int Wo, int kh, int kw, int sh, int sw, int ph, int pw)
{
    if (kh != 3 || kw != 3 || sh != sw || (sh != 1 && sh != 2) || ph < 0 || ph > 2) return false;
    if (pw != 1 && !(sh == 2 && pw == 0)) return false;
    if (W < 4 || H < 1 || Wo < 1) return false;
    return Wo == (W + 2 * pw - 3) / sh + 1;
}
bool k2s2_shape(int H, int W, int Ho, int Wo, int kh, int kw, int sh, int sw, int ph, int pw)
{
    return kh == 2 && kw == 2 && sh == 2 && sw == 2 && ph == 0 && pw == 0 && W >= 4 && H >= 2 && Wo == W / 2 && Ho == H / 2;
}

}  // namespace

hipError_t launch_maxpool2d_grad_rows(const float *x, const float *gy, float *gx, int64_t planes, int H, int W, int Ho,
                                      int Wo, int kh, int kw, int sh, int sw, int ph, int pw, hipStream_t s, bool *taken)
{
    *taken = false;
    constexpr int TH = 4;
    const bool rag = (W & 3) != 0;
    const bool k2 = k2s2_shape(H, W, Ho, Wo, kh, kw, sh, sw, ph, pw);
    if (!k2 && !rows_shape(H, W, Ho, Wo, kh, kw, sh, sw, ph, pw)) return hipSuccess;
    const RowsGrid r = rows_grid(planes, H, W, TH);
    if (!r.ok) return hipSuccess;
    *taken = true;
#define SWS_MPG(S_, PW_, RAG_)                                                                                          \
    hipLaunchKernelGGL((maxpool_grad_rows_kernel<S_, TH, PW_, RAG_>), r.grid, dim3(kWave), 0, s, x, gy, gx, H, W, Ho, Wo, ph, \
                       r.LPR, r.G, r.rcp, r.nstrips, planes)
    if (k2) {
        if (rag)
            hipLaunchKernelGGL((maxpool_grad_rows_k2s2_kernel<TH, true>), r.grid, dim3(kWave), 0, s, x, gy, gx, H, W, Ho, Wo,
                               r.LPR, r.G, r.rcp, r.nstrips, planes);
        else
            hipLaunchKernelGGL((maxpool_grad_rows_k2s2_kernel<TH, false>), r.grid, dim3(kWave), 0, s, x, gy, gx, H, W, Ho, Wo,
                               r.LPR, r.G, r.rcp, r.nstrips, planes);
    } else if (sh == 1) {
        if (rag) SWS_MPG(1, 1, true); else SWS_MPG(1, 1, false);
    } else if (pw == 1) {
        if (rag) SWS_MPG(2, 1, true); else SWS_MPG(2, 1, false);
    } else {
        if (rag) SWS_MPG(2, 0, true); else SWS_MPG(2, 0, false);
    }
#undef SWS_MPG
    return hipGetLastError();
}

hipError_t launch_avgpool2d_grad_rows(const float *gy, float *gx, int64_t planes, int H, int W, int Ho, int Wo, int kh,
                                      int kw, int sh, int sw, int ph, int pw, float scale, hipStream_t s, bool *taken)
{
    *taken = false;
    constexpr int TH = 4;
    const bool rag = (W & 3) != 0;
    const bool k2 = k2s2_shape(H, W, Ho, Wo, kh, kw, sh, sw, ph, pw);
    if (!k2 && (sh != 2 || !rows_shape(H, W, Ho, Wo, kh, kw, sh, sw, ph, pw))) return hipSuccess;
    const RowsGrid r = rows_grid(planes, H, W, TH);
    if (!r.ok) return hipSuccess;
    *taken = true;
#define SWS_APG(PW_, RAG_)                                                                                              \
    hipLaunchKernelGGL((avgpool_grad_rows_s2_kernel<TH, PW_, RAG_>), r.grid, dim3(kWave), 0, s, gy, gx, H, W, Ho, Wo, ph, r.LPR, \
                       r.G, r.rcp, r.nstrips, planes, scale)
    if (k2) {
        if (rag)
            hipLaunchKernelGGL((avgpool_grad_rows_k2s2_kernel<TH, true>), r.grid, dim3(kWave), 0, s, gy, gx, H, W, Ho, Wo, r.LPR,
                               r.G, r.rcp, r.nstrips, planes, scale);
        else
            hipLaunchKernelGGL((avgpool_grad_rows_k2s2_kernel<TH, false>), r.grid, dim3(kWave), 0, s, gy, gx, H, W, Ho, Wo, r.LPR,
                               r.G, r.rcp, r.nstrips, planes, scale);
    } else if (pw == 1) {
        if (rag) SWS_APG(1, true); else SWS_APG(1, false);
    } else {
        if (rag) SWS_APG(0, true); else SWS_APG(0, false);
    }
#undef SWS_APG
    return hipGetLastError();
}

}  // namespace sws
