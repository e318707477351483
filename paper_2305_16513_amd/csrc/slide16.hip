// sws_slide1d_16 — sliding window sums (Section 2.2, Eq. 3) on bf16 / fp16 storage.
//
// The segment prefix / suffix scheme of the fp32 kernel (the block form of Section 3's
// Algorithm 2): a wavefront owns a tile of 1024 consecutive inputs cut into segments of
// S = w - 1 elements, builds the in-segment prefix sums Pre and suffix sums Suf, and every output
// costs one more (+): y[q] = Suf[q] (+) Pre[q+S].  Elements are 16 bits wide in memory only: a
// lane's strip element is EIGHT of them (one 128-bit load), widened exactly to fp32 on the way
// into LDS; the scans and the combine are fp32; the eight results of a strip element are rounded
// to nearest even once and leave as one 128-bit non-temporal store.  With half the bytes per
// element the kernel is bound by instruction issue and latency rather than by HBM, hence the wide
// strips (half as many staging and combine steps per element as the fp32 kernel's four-element
// strips) and the software prefetch of the next tile.
// Windows up to 33 also have a kernel on shifted loads (eight outputs per lane straight from
// 128-bit loads, no LDS); it serves the windows up to 9 everywhere, and the others on short rows
// and small tensors, where 1024-element wave tiles fit badly.
// Plain rows only (no boundary rules, no chains of windows).
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerWg = kThreads / kWave;
constexpr int kC = 16;                               // consecutive elements a lane scans
constexpr int kN = kWave * kC;                       // inputs per wave tile
constexpr int kLine = 32;                            // 16-bit elements per 64-byte line

__device__ __forceinline__ float lane_read(float v, int src_lane)
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute((src_lane & 63) << 2, __float_as_int(v)));
}

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// LDS layout of a wave tile: 256 groups of 4 floats, group g stored at
//     g ^ ((g >> 3) & 3) ^ (((g >> 5) & 1) << 3).
// Conflict-free for the three 128-bit access shapes used here: chunks (lane l reads groups
// 4l .. 4l+3), strip halves on the way in and out (lane l touches group 2l, then 2l+1: eight
// consecutive lanes cover the groups {0,2,4,6,9,11,13,15} mod 16 — eight different bank quads) and
// the shifted Pre groups.  Only bits 0-3 of g change, so adding 128 groups (a strip) commutes.
__device__ __forceinline__ int lds_group(int g) { return g ^ ((g >> 3) & 3) ^ (((g >> 5) & 1) << 3); }

// In-segment scan step, the reset folded into arithmetic (one VALU op for ADD, two for MAX / MIN).
template <int OP> struct SegStep;
template <> struct SegStep<SWS_OP_ADD> {
    static __device__ __forceinline__ float mask(bool start) { return start ? 0.0f : 1.0f; }
    static __device__ __forceinline__ float f(float acc, float m, float x) { return __builtin_fmaf(acc, m, x); }
};
template <> struct SegStep<SWS_OP_MAX> {
    static __device__ __forceinline__ float mask(bool start) { return start ? -__builtin_huge_valf() : __builtin_huge_valf(); }
    static __device__ __forceinline__ float f(float acc, float m, float x) { return __builtin_fmaxf(__builtin_fminf(acc, m), x); }
};
template <> struct SegStep<SWS_OP_MIN> {
    static __device__ __forceinline__ float mask(bool start) { return start ? __builtin_huge_valf() : -__builtin_huge_valf(); }
    static __device__ __forceinline__ float f(float acc, float m, float x) { return __builtin_fminf(__builtin_fmaxf(acc, m), x); }
};

typedef float v8f __attribute__((ext_vector_type(8)));

// Eight 16-bit elements <-> eight floats.  Widening is exact; narrowing rounds to nearest even.
template <typename T> struct Io {
    typedef T v8 __attribute__((ext_vector_type(8)));
    typedef v8 v8_u __attribute__((aligned(2)));
    static __device__ __forceinline__ v8 load_raw(const T *p) { return *(const v8_u *)p; }
    static __device__ __forceinline__ v8f widen(v8 r) { return __builtin_convertvector(r, v8f); }
    static __device__ __forceinline__ v8f load8(const T *p) { return widen(load_raw(p)); }
    static __device__ __forceinline__ float load1(const T *p) { return (float)*p; }
    static __device__ __forceinline__ void store1(T *p, float v) { *p = (T)v; }
    static __device__ __forceinline__ void store8(T *p, v8f o)
    {
        __builtin_nontemporal_store(__builtin_convertvector(o, v8), (v8_u *)p);
    }
};

template <int OP, typename T>
__global__ __launch_bounds__(kThreads) void slide16_scan_kernel(const T *__restrict__ x, T *__restrict__ y, int len,
                                                                int lo, int S, float scale, int tiles_per_row,
                                                                int tout, int group, int64_t n_tiles,
                                                                int64_t n_units, int remap)
{
    using O = Op<OP>;
    using G = SegStep<OP>;
    using IO = Io<T>;
    constexpr int C = kC, N = kN;
    __shared__ __attribute__((aligned(16))) float lds[kWavesPerWg * 2 * N];

    const int64_t unit = remap ? xcd_unit(n_units) : (int64_t)blockIdx.x;
    if (unit < 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *Bf = lds + wave * 2 * N;                  // Suf
    float *A = Bf + N;                               // staged inputs, later Pre
    int64_t gt = unit * group + wave;
    int64_t gt_end = (unit + 1) * group;
    if (gt_end > n_tiles) gt_end = n_tiles;
    int64_t r = gt / tiles_per_row;
    int t = (int)(gt - r * tiles_per_row);

    // Lane constants (as in the fp32 kernel): this lane scans local positions C*lane .. C*lane+C-1;
    // m[k] is the reset mask of element k (a segment of S elements, counted from the tile origin,
    // starts there); m[C] belongs to the first element of the next lane.
    const float inv_s = 1.0f / (float)S;
    const int q0 = (C * lane) - S * (int)(((float)(C * lane) + 0.5f) * inv_s);                // (C*lane) % S
    float m[C + 1];
    if (S > C) {
        const int kb = q0 == 0 ? 0 : S - q0;
#pragma unroll
        for (int k = 0; k <= C; ++k) m[k] = G::mask(k == kb);
    } else {
        int q = q0;
#pragma unroll
        for (int k = 0; k <= C; ++k) {
            m[k] = G::mask(q == 0);
            q = (q + 1 == S) ? 0 : q + 1;
        }
    }
    const int n_pre = (q0 + C - 1) / C;             // earlier lanes holding part of my first segment
    int qe = q0 + C;
    if (S > C) qe = qe >= S ? qe - S : qe;
    else qe -= S * (int)(((float)qe + 0.5f) * inv_s);
    const int rem = qe == 0 ? 0 : S - qe;           // elements of my last segment beyond my chunk
    const int n_suf = (rem + C - 1) / C;
    const int max_reach = (S - 1 + C - 1) / C;
    const int sh = S & 3;                           // misalignment of Pre[q+S] against groups
    const int s4 = (S - sh) >> 2;
    const int chunk_pos = 4 * lds_group(4 * lane);  // my chunk: group u of it sits at chunk_pos ^ (4*u)
    // strip element of lane l: local positions 512*j + 8*l .. +7, i.e. groups 128*j + 2l, 2l+1
    const int sp0 = 4 * lds_group(2 * lane), sp1 = 4 * lds_group(2 * lane + 1);
    // the three aligned groups that hold Pre[q+S .. q+S+7+sh] (past the tile: wrapped, discarded lanes only)
    const int pp0 = 4 * lds_group((2 * lane + s4) & 255), pp1 = 4 * lds_group((2 * lane + s4 + 1) & 255),
              pp2 = 4 * lds_group((2 * lane + s4 + 2) & 255);

    // The strips of my next tile are requested before the current tile is worked on (raw 16-bit
    // registers, widened when their turn comes): with 2 KB per tile a wavefront would otherwise
    // have too few bytes in flight to cover the memory latency (measured on 2^29 elements, w = 16:
    // 0.59 ms without, 0.43 ms with; requesting two tiles ahead gains nothing more).  Tiles at an
    // end of their row are not requested ahead; they are staged strip by strip at their turn.
    typename IO::v8 raw0[2];                         // my current tile, later my next tile
    auto request = [&](int64_t rr, int tt, int64_t g_idx, typename IO::v8 (&dst)[2]) -> bool {
        if (g_idx >= gt_end) return false;
        const int t0n = tt * tout - (int)((rr * lo) & (kLine - 1));
        if (t0n < 0 || t0n > len - N) return false;
        const T *xn = x + rr * (int64_t)len + t0n;
#pragma unroll
        for (int j = 0; j < 2; ++j) dst[j] = IO::load_raw(xn + 512 * j + 8 * lane);
        return true;
    };
    int t1 = t + kWavesPerWg;
    int64_t r1 = r;
    while (t1 >= tiles_per_row) { t1 -= tiles_per_row; ++r1; }
    bool have0 = request(r, t, gt, raw0);
    for (; gt < gt_end; gt += kWavesPerWg) {
        const T *xr = x + r * (int64_t)len;
        // tile origins pulled back so that (r*lo + t0) is a multiple of 32 elements: every strip
        // store starts on a 64-byte line of y; outputs before the row start are not stored
        const int t0 = t * tout - (int)((r * lo) & (kLine - 1));
        const int qlo = t0 < 0 ? -t0 : 0;
        const T *xt = xr + t0;
        T *yt = y + r * (int64_t)lo + t0;
        // ---- stage: two strips of 512 elements -> LDS as fp32
        v8f g8[2];
        if (have0) {
#pragma unroll
            for (int j = 0; j < 2; ++j) g8[j] = IO::widen(raw0[j]);
        } else {
            // a tile at an end of its row: whole strips inside the row are still 128-bit loads,
            // strips wholly outside hold the identity (wave-uniform tests)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int s0 = t0 + 512 * j;
                if (s0 >= 0 && s0 + 512 <= len) {
                    g8[j] = IO::load8(xt + 512 * j + 8 * lane);
                } else if (s0 >= len || s0 + 512 <= 0) {
#pragma unroll
                    for (int c = 0; c < 8; ++c) g8[j][c] = O::id();
                } else {
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        const int e = s0 + 8 * lane + c;
                        g8[j][c] = (e >= 0 && e < len) ? IO::load1(xr + e) : O::id();
                    }
                }
            }
        }
        // ---- my next tile: request it now
        have0 = request(r1, t1, gt + kWavesPerWg, raw0);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            *(v4f *)(A + sp0 + 512 * j) = (v4f){g8[j][0], g8[j][1], g8[j][2], g8[j][3]};
            *(v4f *)(A + sp1 + 512 * j) = (v4f){g8[j][4], g8[j][5], g8[j][6], g8[j][7]};
        }
        wave_lds_sync();
        // ---- my chunk of C consecutive elements
        float v[C];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const v4f g = *(const v4f *)(A + (chunk_pos ^ (4 * u)));
            v[4 * u] = g.x; v[4 * u + 1] = g.y; v[4 * u + 2] = g.z; v[4 * u + 3] = g.w;
        }
        // ---- pass 1: lane totals (tail: my last segment's part, head: my first segment's part)
        float tail = v[0], head = v[C - 1];
#pragma unroll
        for (int k = 1; k < C; ++k) tail = G::f(tail, m[k], v[k]);
#pragma unroll
        for (int k = C - 2; k >= 0; --k) head = G::f(head, m[k + 1], v[k]);
        // ---- cross-lane carries: e from the n_pre lanes before me, g from the n_suf lanes after me
        float e = lane_read(tail, lane - 1);
        float g = lane_read(head, lane + 1);
        for (int d = 1; d < max_reach; d <<= 1) {
            const float te = lane_read(e, lane - d);
            const float tg = lane_read(g, lane + d);
            if (n_pre > d) e = O::f(te, e);
            if (n_suf > d) g = O::f(g, tg);
        }
        // ---- pass 2: the scans seeded with the carries: in-segment prefix sums (over v) and suffix sums
        float suf[C];
        suf[C - 1] = G::f(g, m[C], v[C - 1]);
#pragma unroll
        for (int k = C - 2; k >= 0; --k) suf[k] = G::f(suf[k + 1], m[k + 1], v[k]);
        v[0] = G::f(e, m[0], v[0]);
#pragma unroll
        for (int k = 1; k < C; ++k) v[k] = G::f(v[k - 1], m[k], v[k]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *(v4f *)(A + (chunk_pos ^ (4 * u))) = (v4f){v[4 * u], v[4 * u + 1], v[4 * u + 2], v[4 * u + 3]};
            *(v4f *)(Bf + (chunk_pos ^ (4 * u))) = (v4f){suf[4 * u], suf[4 * u + 1], suf[4 * u + 2], suf[4 * u + 3]};
        }
        wave_lds_sync();
        // ---- combine on strips of eight: y[q] = Suf[q] (+) Pre[q+S], one rounding, 128-bit stores
        int lim = lo - t0;
        if (lim > tout) lim = tout;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int q = 512 * j + 8 * lane;
            if (q >= lim) continue;
            const v4f sa = *(const v4f *)(Bf + sp0 + 512 * j), sb = *(const v4f *)(Bf + sp1 + 512 * j);
            const v4f p0 = *(const v4f *)(A + ((pp0 + 512 * j) & (N - 1)));
            const v4f p1 = *(const v4f *)(A + ((pp1 + 512 * j) & (N - 1)));
            const v4f p2 = *(const v4f *)(A + ((pp2 + 512 * j) & (N - 1)));
            v8f pn;
            switch (sh) {                            // wave-uniform
            case 0: pn = (v8f){p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w}; break;
            case 1: pn = (v8f){p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w, p2.x}; break;
            case 2: pn = (v8f){p0.z, p0.w, p1.x, p1.y, p1.z, p1.w, p2.x, p2.y}; break;
            default: pn = (v8f){p0.w, p1.x, p1.y, p1.z, p1.w, p2.x, p2.y, p2.z}; break;
            }
            const v8f sv = {sa.x, sa.y, sa.z, sa.w, sb.x, sb.y, sb.z, sb.w};
            v8f o;
#pragma unroll
            for (int c = 0; c < 8; ++c) o[c] = O::f(sv[c], pn[c]);
            if (OP == SWS_OP_ADD) o *= scale;
            if (q >= qlo && q + 8 <= lim) {
                IO::store8(yt + q, o);
            } else {
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    if (q + c >= qlo && q + c < lim) IO::store1(yt + q + c, o[c]);
            }
        }
        wave_lds_sync();                             // the next tile overwrites A
        t = t1;
        r = r1;
        t1 += kWavesPerWg;
        while (t1 >= tiles_per_row) { t1 -= tiles_per_row; ++r1; }
    }
}

// Direct evaluation (windows beyond the scan kernel's reach): one thread per output,
// fp32 accumulation left to right, one rounding at the end.
template <int OP, typename T>
__global__ __launch_bounds__(kThreads) void slide16_naive_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                                 int64_t rows, int len, int lo, int w, float scale)
{
    using O = Op<OP>;
    const int64_t total = rows * (int64_t)lo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int64_t r = o / lo;
        const T *xr = x + r * (int64_t)len + (o - r * lo);
        float acc = (float)xr[0];
        for (int j = 1; j < w; ++j) acc = O::f(acc, (float)xr[j]);
        if (OP == SWS_OP_ADD) acc *= scale;
        y[o] = (T)acc;
    }
}

// Small windows on shifted loads: a lane owns eight consecutive outputs and reads the w + 7 inputs
// under them as 128-bit loads.  Up to w = 8 each output combines its inputs left to right (Eq. 3 as
// written).  From w = 9 the eight windows share the inputs 7 .. w-1 of the strip: that core is
// combined once, and output c adds the suffix c .. 6 in front of it and the prefix w .. w+c-1
// behind it (running sums, the register-level form of Section 3's prefix / suffix split), about
// w + 20 operations for the eight outputs instead of 8 (w - 1).  All of it in fp32, one rounding.
// Workgroups are one wavefront and short-lived (512 outputs of a row, or several short rows side
// by side), which streams better than long-lived tiles.
// A 128-bit load may run past the end of its row (those values reach no valid output) but not
// past the ends of x: there it is replaced by element loads.
template <int OP, typename T, int W>
__global__ __launch_bounds__(kWave) void slide16_direct_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                               int64_t rows, int len, int lo, float scale,
                                                               int strips, int wg_per_row, int rows_per_wg, int recip,
                                                               int align)
{
    using O = Op<OP>;
    using IO = Io<T>;
    constexpr int NL = (W + 7 + 7) / 8;              // 128-bit loads per strip
    const int lane = threadIdx.x;
    int64_t r;
    int sidx;
    if (rows_per_wg == 1) {
        const int br = blockIdx.x / (unsigned)wg_per_row;
        r = br;
        sidx = (blockIdx.x - br * wg_per_row) * kWave + lane;
    } else {
        const int lr = (lane * recip) >> 16;         // lane / strips, exact for lane < 64
        if (lr >= rows_per_wg) return;
        r = (int64_t)blockIdx.x * rows_per_wg + lr;
        sidx = lane - lr * strips;
    }
    if (r >= rows || sidx >= strips) return;
    // long rows: strips sit on the 16-byte boundaries of y, so a row that starts between two
    // boundaries has a partial first strip (short rows would spend too many lanes on those)
    T *yrow = y + r * (int64_t)lo;
    const int q = 8 * sidx - (align ? (int)(((uintptr_t)yrow >> 1) & 7) : 0);
    if (q >= lo) return;
    const int64_t g = r * (int64_t)len + q;          // the strip's first input in x
    const int64_t total = rows * (int64_t)len;
    const T *xr = x + g;
    float v[8 * NL];
#pragma unroll
    for (int k = 0; k < NL; ++k) {
        if (g + 8 * k >= 0 && g + 8 * k + 8 <= total) {
            const v8f a = IO::load8(xr + 8 * k);
#pragma unroll
            for (int c = 0; c < 8; ++c) v[8 * k + c] = a[c];
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int64_t e = g + 8 * k + c;
                v[8 * k + c] = (e >= 0 && e < total) ? IO::load1(xr + 8 * k + c) : 0.0f;
            }
        }
    }
    v8f o;
    if constexpr (W <= 8) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float acc = v[c];
#pragma unroll
            for (int j = 1; j < W; ++j) acc = O::f(acc, v[c + j]);
            o[c] = acc;
        }
    } else {
        float core = v[7];
#pragma unroll
        for (int j = 8; j < W; ++j) core = O::f(core, v[j]);
        float suf[7], pre[8];
        suf[6] = v[6];
#pragma unroll
        for (int c = 5; c >= 0; --c) suf[c] = O::f(v[c], suf[c + 1]);
        pre[1] = v[W];
#pragma unroll
        for (int c = 2; c < 8; ++c) pre[c] = O::f(pre[c - 1], v[W + c - 1]);
        o[0] = O::f(suf[0], core);
        o[7] = O::f(core, pre[7]);
#pragma unroll
        for (int c = 1; c < 7; ++c) o[c] = O::f(O::f(suf[c], core), pre[c]);
    }
    if (OP == SWS_OP_ADD) o *= scale;
    T *yr = yrow + q;
    if (q >= 0 && q + 8 <= lo) {
        IO::store8(yr, o);
    } else {
#pragma unroll
        for (int c = 0; c < 8; ++c)
            if (q + c >= 0 && q + c < lo) IO::store1(yr + c, o[c]);
    }
}

constexpr int kDirectMaxW = 33;                      // five 128-bit loads per strip of eight outputs

template <int OP, typename T, int W>
hipError_t launch_16_direct_w(const T *x, T *y, int64_t rows, int len, int lo, float scale, hipStream_t s)
{
    // aligned strips pay from about a thousand outputs per row (measured: 4.5 against 4.3 TB/s at
    // 4096, 2.7 against 3.7 at 224); rows of y that all start on a boundary need no shift
    const int align = lo >= 1024 && !(lo % 8 == 0 && (uintptr_t)y % 16 == 0);
    const int strips = (lo + (align ? 14 : 7)) / 8;
    const int wg_per_row = (strips + kWave - 1) / kWave;
    const int rows_per_wg = strips < kWave ? kWave / strips : 1;
    const int recip = 65536 / strips + 1;
    const int64_t grid = rows_per_wg == 1 ? rows * wg_per_row : (rows + rows_per_wg - 1) / rows_per_wg;
    if (grid > 2147483647LL) return kNotTaken;
    hipLaunchKernelGGL((slide16_direct_kernel<OP, T, W>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, rows, len, lo,
                       scale, strips, wg_per_row, rows_per_wg, recip, align);
    return hipGetLastError();
}

template <int OP, typename T, int W0>
hipError_t launch_16_direct(const T *x, T *y, int64_t rows, int len, int lo, int w, float scale, hipStream_t s)
{
    if constexpr (W0 > kDirectMaxW) {
        return kNotTaken;
    } else {
        if (w == W0) return launch_16_direct_w<OP, T, W0>(x, y, rows, len, lo, scale, s);
        return launch_16_direct<OP, T, W0 + 1>(x, y, rows, len, lo, w, scale, s);
    }
}

constexpr int kScanMaxW = kN - 64 + 1;               // leaves at least 64 outputs per wave tile
constexpr int kLong16MinW = 600;                     // from here the long-window kernel (bf16, 16384-long rows: w = 513 level, 700 1.3 x, 961 5 x the scan)

template <int OP, typename T>
hipError_t launch_16(const T *x, T *y, int64_t rows, int len, int lo, int w, float scale, hipStream_t s)
{
    const int variant = g_opt.slide_variant;
    // Measured on bf16: up to w = 9 (two loads per strip) the shifted loads win at every size (5.2 to
    // 5.8 TB/s against the scan's 4.9 to 5.1 on a 1 GB tensor); beyond that they win where the scan
    // kernel's 1024-element wave tiles fit badly: rows under 2048 outputs (3 to 25 times faster at
    // 56 to 224 elements per row) and tensors under 2^25 elements (2 to 5 times).
    const bool direct_auto = w <= 9 || lo < 2048 || rows * (int64_t)len <= (1LL << 25);
    if (w <= kDirectMaxW && variant != 1 && (variant == 3 || w == 1 || (variant != 2 && direct_auto))) {
        const hipError_t e = launch_16_direct<OP, T, 1>(x, y, rows, len, lo, w, scale, s);
        if (e != kNotTaken) return e;     // a grid beyond the launch limit: the kernels below
    }
    if (w >= 2 && w <= kScanMaxW && variant != 1) {
        const int S = w - 1;
        const int tout = (kN - S) & ~(kLine - 1);    // a multiple of 64 bytes of y (at least 64 outputs)
        const int tiles = (lo + max_origin_shift(lo, kLine) + tout - 1) / tout;
        const int64_t n_tiles = rows * tiles;
        // sixteen tiles per wavefront (measured best: 8 to 32), the next one in flight while one is
        // worked on; workgroups in launch order
        int64_t g = 16 * kWavesPerWg;
        int remap = 0;
        // ... halved while that leaves fewer than 2048 workgroups (measured on 64 rows of 2^20:
        // 5.8 against 4.9 TB/s; a limit of 4096 loses again on 4096 x 4096)
        while (g > kWavesPerWg && n_tiles / g < 2048) g /= 2;
        if (g_opt.slide_group > 0) g = (g_opt.slide_group + kWavesPerWg - 1) / kWavesPerWg * kWavesPerWg;
        if (g_opt.slide_chunk & 4) remap = 1;
        if (g_opt.slide_chunk & 8) remap = 0;
        const int64_t n_units = (n_tiles + g - 1) / g;
        const int64_t grid = remap ? xcd_grid(n_units) : n_units;
        if (grid > 2147483647LL) return kNotTaken;
        hipLaunchKernelGGL((slide16_scan_kernel<OP, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, len, lo, S,
                           scale, tiles, tout, (int)g, n_tiles, n_units, remap);
        return hipGetLastError();
    }
    int64_t grid = (rows * (int64_t)lo + kThreads - 1) / kThreads;
    if (grid > 1048576) grid = 1048576;
    hipLaunchKernelGGL((slide16_naive_kernel<OP, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, rows, len, lo,
                       w, scale);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_16_op(int op, const void *x, void *y, int64_t rows, int len, int lo, int w, float scale,
                        hipStream_t s)
{
    switch (op) {
    case SWS_OP_ADD: return launch_16<SWS_OP_ADD, T>((const T *)x, (T *)y, rows, len, lo, w, scale, s);
    case SWS_OP_MAX: return launch_16<SWS_OP_MAX, T>((const T *)x, (T *)y, rows, len, lo, w, scale, s);
    default: return launch_16<SWS_OP_MIN, T>((const T *)x, (T *)y, rows, len, lo, w, scale, s);
    }
}

}  // namespace

// 16-bit storage (dtype SWS_DTYPE_BF16 / SWS_DTYPE_F16), fp32 arithmetic, one rounding per output.
hipError_t launch_slide1d_16(int op, int dtype, const void *x, void *y, int64_t rows, int64_t len64, int32_t w,
                             float scale, hipStream_t s)
{
    const int len = (int)len64, lo = len - w + 1;
    // windows longer than a wave tile: the one-pass long-window kernel (slide_long.hip); slide_variant 8 takes it
    // from w = 257, 1 and 5 keep it out
    const int variant = g_opt.slide_variant;
    if ((w >= kLong16MinW || (variant == 8 && w > 256)) && variant != 1 && variant != 5) {
        const hipError_t e = launch_slide1d_long_16(op, dtype, x, y, rows, len, lo, w, scale, s);
        if (e != kNotTaken) return e;
    }
    if (dtype == SWS_DTYPE_BF16) return launch_16_op<__bf16>(op, x, y, rows, len, lo, w, scale, s);
    return launch_16_op<_Float16>(op, x, y, rows, len, lo, w, scale, s);
}

}  // namespace sws
