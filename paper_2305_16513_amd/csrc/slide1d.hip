// sws_slide1d — sliding window sums over rows (Section 2.2, Eq. 3) for gfx950.
//
// Two tuned kernels plus the direct-evaluation fallback (rows of a few hundred elements with
// windows up to 33 go to a third, slide_rows.hip, which packs several rows into a wavefront):
//
//  * slide_direct_kernel: the Vector Slide idea of Section 3 (Algorithm 4) — the output
//    vector is the (+) of w shifted copies of the input vector.  A lane owns four consecutive
//    outputs and reads its shifted operands as 128-bit loads at +4, +8, +12 elements.  Two launch
//    shapes: 1024-output tiles, four wavefronts per workgroup (w <= 9 on short rows or small
//    problems), and 256-output strips, one wavefront per workgroup (large inputs: w <= 4 and w = 9
//    where the scan below does not load streamed, max / min at w = 9 where it does).
//    Also w = 1 (a scaled copy).
//
//  * slide_scan_kernel (every w >= 2): the block form of the Vector Input algorithm
//    (Section 3, Algorithm 2).  A wavefront owns a tile of 64*C consecutive inputs cut
//    into segments of length S = w-1 (counted from the tile origin).  It builds
//       Pre[q] = x[seg_start(q)] (+) ... (+) x[q]      (in-segment prefix sums, "X1")
//       Suf[q] = x[q] (+) ... (+) x[seg_end(q)]        (in-segment suffix sums, "Y1")
//    and every output costs ONE more (+):  y[q] = Suf[q] (+) Pre[q+S]  (older operand on
//    the left), which holds exactly w terms because q and q+S sit at the same offset of
//    adjacent segments.  Each lane scans C consecutive elements sequentially; the lane
//    totals are combined by O(log(S/C)) cross-lane steps, so the work per output does not
//    grow with w.  Global memory is touched only with fully coalesced 128-bit accesses
//    (lane l <-> bytes 16*l of each 1 KB strip); LDS does the strip <-> chunk transposes.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerWg = kThreads / kWave;

__device__ __forceinline__ float lane_read(float v, int src_lane)
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute((src_lane & 63) << 2, __float_as_int(v)));
}

// Orders the LDS traffic of one wavefront: everything written before is visible to the
// lanes reading after.  No workgroup barrier — each wavefront owns its LDS slice.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ------------------------------------------------------------------------------------------
// Small windows: y[i] = x[i] (+) x[i+1] (+) ... (+) x[i+W-1] from shifted 128-bit loads.
// ------------------------------------------------------------------------------------------
// STRIPS = 4: one 1024-output tile per wavefront, four wavefronts per workgroup.  STRIPS = 1: one
// 256-output strip per wavefront and one wavefront per workgroup — the shape in which a plain copy
// measures fastest on this GPU (6.7 against 6.1 TB/s), used for large inputs.
template <int OP, int W, int STRIPS>
__global__ __launch_bounds__(STRIPS == 1 ? kWave : kThreads) void slide_direct_kernel(const float *__restrict__ x,
                                                                float *__restrict__ y, int len, int lo,
                                                                float scale, int tiles_per_row, int64_t n_tiles,
                                                                int remap)
{
    using O = Op<OP>;
    constexpr int NV = (W + 2) / 4 + 1;            // float4 groups covering x[q .. q+W+2]
    constexpr int WPW = STRIPS == 1 ? 1 : kWavesPerWg;     // wavefronts per workgroup
    // Tiles numbered over all rows; consecutive tiles per workgroup (the tiles in flight then stay
    // a compact window of memory).
    const int64_t n_units = (n_tiles + WPW - 1) / WPW;
    const int64_t unit = remap ? xcd_unit(n_units) : (int64_t)blockIdx.x;
    if (unit < 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t gt = unit * WPW + wave;
    if (gt >= n_tiles) return;
    const int64_t r = gt / tiles_per_row;
    const int t = (int)(gt - r * tiles_per_row);
    const float *xr = x + r * (int64_t)len;
    float *yr = y + r * (int64_t)lo;
    // tile origins pulled back so that every 1 KB strip store starts on a 64-byte line of y
    const int t0 = t * (256 * STRIPS) - (int)((r * lo) & 15);
#pragma unroll
    for (int j = 0; j < STRIPS; ++j) {
        const int q = t0 + j * 256 + 4 * lane;       // first of this lane's four outputs
        if (q >= lo || q + 4 <= 0) continue;
        float a[4 * NV];
        if (q >= 0 && q <= len - 4 * NV) {
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                const v4f g = *(const v4f_u *)(xr + q + 4 * u);
                a[4 * u] = g.x; a[4 * u + 1] = g.y; a[4 * u + 2] = g.z; a[4 * u + 3] = g.w;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4 * NV; ++u) a[u] = (q + u >= 0 && q + u < len) ? xr[q + u] : O::id();
        }
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float acc = a[e];
#pragma unroll
            for (int s = 1; s < W; ++s) acc = O::f(acc, a[e + s]);
            o[e] = (OP == SWS_OP_ADD) ? acc * scale : acc;
        }
        if (q >= 0 && q + 4 <= lo) {
            const v4f g = {o[0], o[1], o[2], o[3]};
            __builtin_nontemporal_store(g, (v4f_u *)(yr + q));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (q + e >= 0 && q + e < lo) yr[q + e] = o[e];
        }
    }
}

// ------------------------------------------------------------------------------------------
// Large windows: in-segment prefix + suffix sums, one (+) per output.
// ------------------------------------------------------------------------------------------
// LDS layout of one wave tile: the tile is 256 groups of 4 floats, and group g is stored at
//     g ^ ((g >> 3) & 3) ^ (((g >> 5) & 1) << 3).
// Folding bits 3-4 into bits 0-1 and bit 5 into bit 3 makes both access shapes of a 128-bit
// LDS instruction conflict-free, whether the hardware serves 8 lanes (32 banks) or 16 lanes
// (64 banks) per cycle: strips (consecutive lanes read consecutive groups) and chunks (lane l
// reads groups 4*l .. 4*l+3, i.e. consecutive lanes are 4 groups apart).  The permutation
// only touches bits 0-3 of g, so it commutes with adding multiples of 64 groups (a strip).
__device__ __forceinline__ int lds_pos(int q)
{
    const int g = q >> 2;                            // group of 4 floats
    return ((g ^ ((g >> 3) & 3) ^ (((g >> 5) & 1) << 3)) << 2) | (q & 3);
}

// In-segment scan step with the reset folded into arithmetic: acc is forgotten where a new
// segment starts.  The per-element mask is a lane constant (see seg_mask) — one VALU op for
// ADD (fma with 0/1), two for MAX / MIN (clamp against -/+inf, then combine).
template <int OP> struct SegStep;
template <> struct SegStep<SWS_OP_ADD> {
    static __device__ __forceinline__ float mask(bool start) { return start ? 0.0f : 1.0f; }
    static __device__ __forceinline__ float f(float acc, float m, float x) { return __builtin_fmaf(acc, m, x); }
};
template <> struct SegStep<SWS_OP_MAX> {
    static __device__ __forceinline__ float mask(bool start)
    {
        return start ? -__builtin_huge_valf() : __builtin_huge_valf();
    }
    static __device__ __forceinline__ float f(float acc, float m, float x)
    {
        return __builtin_fmaxf(__builtin_fminf(acc, m), x);
    }
};
template <> struct SegStep<SWS_OP_MIN> {
    static __device__ __forceinline__ float mask(bool start)
    {
        return start ? __builtin_huge_valf() : -__builtin_huge_valf();
    }
    static __device__ __forceinline__ float f(float acc, float m, float x)
    {
        return __builtin_fminf(__builtin_fmaxf(acc, m), x);
    }
};

// MODE 0: plain rows.  MODE 1: rows extended by a boundary rule.  MODE 2: one link of a chain of
// windows (see launch_chain): rows `pitch` apart of which `len` elements are used, results
// combined with what an earlier link left in y.
template <int OP, int C, int MODE, int WPW = kWavesPerWg, bool STREAM = false>
__global__ __launch_bounds__(WPW * kWave) void slide_scan_kernel(const float *__restrict__ x,
                                                              float *__restrict__ y, int len, int lo, int S,
                                                              float scale, int tiles_per_row, int tout,
                                                              int group, int64_t n_tiles, int64_t n_units,
                                                              int flags, int pad_left_arg, int pad_mode_arg,
                                                              int lv_arg)
{
    // The row the windows slide over is the physical row of `len` elements extended to `lv`
    // (pad_left in front, the rest behind) by the boundary rule pad_mode; lo = lv - S outputs.
    // The plain instantiation sees constants, so the common path carries none of this.
    // MODE 3: a chain link over extended rows — pad_left may then be negative (the link's windows
    // start inside the row), pad_mode_arg carries the boundary rule in its low byte and the
    // "combine with y" flag in bit 8.
    constexpr bool PADDED = MODE == 1 || MODE == 3;
    constexpr bool CHAIN = MODE == 2 || MODE == 3;
    const int pad_left = PADDED ? pad_left_arg : 0, pad_mode = PADDED ? (pad_mode_arg & 255) : SWS_PAD_IDENTITY;
    const int lv = PADDED ? lv_arg : len;
    const int pitch = MODE == 2 ? lv_arg : len;     // distance between rows of x
    const bool chain_acc = (MODE == 2 && (pad_mode_arg & 1)) || (MODE == 3 && (pad_mode_arg & 256));   // combine with the earlier links' result in y
    using O = Op<OP>;
    using G = SegStep<OP>;
    static_assert(C == 16, "the LDS layout assumes 16-element chunks");
    constexpr int N = kWave * C;                    // inputs per wave tile
    constexpr int NS = C / 4;                       // 256-element strips per tile
    constexpr int REGION = N;
    __shared__ __attribute__((aligned(16))) float lds[WPW * 2 * REGION];

    // kernel flag bits: 2 = non-temporal stores, 4 = aligned tile origins, 32 = workgroups keep
    // their launch order instead of the XCD-contiguous mapping
    const int64_t unit = (flags & 32) ? (int64_t)blockIdx.x : xcd_unit(n_units);
    if (unit < 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *Bf = lds + wave * 2 * REGION;            // Suf
    float *A = Bf + REGION;                         // staged inputs, later Pre
    // Tiles are numbered over all rows (row-major) and dealt out in groups of `group`
    // consecutive tiles per workgroup, wavefront w taking every fourth: equal work per
    // wavefront whatever the row length.
    int64_t gt = unit * group + wave;
    int64_t gt_end = (unit + 1) * group;
    if (gt_end > n_tiles) gt_end = n_tiles;
    // row and tile-in-row of my first tile; the float reciprocal is exact below 2^22 tiles
    int64_t r;
    if (n_tiles < (1LL << 22)) r = (int)(((float)(int)gt + 0.5f) * (1.0f / (float)tiles_per_row));
    else if (n_tiles < 4294967296LL) r = (uint32_t)gt / (uint32_t)tiles_per_row;
    else r = gt / tiles_per_row;
    int t = (int)(gt - r * tiles_per_row);
    const bool aligned = (flags & 4) != 0;          // tile origins on 64-byte boundaries of y

    // Lane constants.  This lane scans local positions C*lane .. C*lane+C-1; m[k] is the reset
    // mask of element k: a segment (S elements, counted from the tile origin) starts there.
    // m[C] belongs to the first element of the next lane.
    const float inv_s = 1.0f / (float)S;
    const int q0 = (C * lane) - S * (int)(((float)(C * lane) + 0.5f) * inv_s);                // (C*lane) % S
    float m[C + 1];
    if (S > C) {
        // at most one segment start inside k = 0 .. C: at kb = distance to the next multiple of S
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
    int qe = q0 + C;                                // (q0 + C) % S: offset of the next lane's first element
    if (S > C) qe = qe >= S ? qe - S : qe;
    else qe -= S * (int)(((float)qe + 0.5f) * inv_s);
    const int rem = qe == 0 ? 0 : S - qe;           // elements of my last segment beyond my chunk
    const int n_suf = (rem + C - 1) / C;            // later lanes holding them
    const int max_reach = (S - 1 + C - 1) / C;
    const int sh = S & 3;                           // misalignment of Pre[q+S] against strips
    const int chunk_pos = lds_pos(C * lane);        // my chunk: group u of it sits at chunk_pos ^ (4*u)
    // Strip j of lane l is local position 256*j + 4*l, i.e. group 64*j + l: the swizzle depends
    // on (group mod 64) only, so one address per lane serves all strips (+256 floats per strip).
    // The same holds for the two aligned groups that hold Pre[q+S .. q+S+3].
    const int s4 = (S - sh) >> 2;
    const int strip_pos = lds_pos(4 * lane);
    const int pre_pos0 = lds_pos(4 * (lane + s4)), pre_pos1 = lds_pos(4 * (lane + s4 + 1));

    for (; gt < gt_end; gt += WPW) {
        const float *xr = x + r * (int64_t)pitch;
        // With aligned tiles the origin is pulled back so that (r*lo + t0) is a multiple of 16
        // floats: every 1 KB strip store then starts on a 64-byte line.  The first tile of a row
        // may start before the row (t0 < 0); those outputs are not stored.
        const int t0 = t * tout - (aligned ? (int)((r * lo) & 15) : 0);
        const int qlo = t0 < 0 ? -t0 : 0;
        // tile-relative bases: uniform 64-bit arithmetic once, 32-bit lane offsets afterwards
        const float *xt = xr + (t0 - pad_left);
        float *yt = y + r * (int64_t)lo + t0;
        // ---- stage the tile: coalesced strips -> LDS; boundary rule in the padding, identity
        //      outside the extended row
        if (t0 - pad_left >= 0 && t0 - pad_left <= len - N) {
            // STREAM: streamed (non-temporal) loads, the launcher's choice for large inputs and windows up to 129 /
            // 173.  (Streaming all strips but those that reach into a neighbouring tile's inputs gains half as much
            // where streaming gains and loses half as much where it loses.  A template parameter: run-time branches
            // that differ in nothing but the hint are merged by the compiler into plain loads.)
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const int q = j * 256 + 4 * lane;
                if constexpr (STREAM) *(v4f *)(A + strip_pos + 256 * j) = __builtin_nontemporal_load((const v4f_u *)(xt + q));
                else *(v4f *)(A + strip_pos + 256 * j) = *(const v4f_u *)(xt + q);
            }
        } else {
            // a tile at an end of its row: strip by strip (wave-uniform tests) — whole strips inside
            // the row are still 128-bit loads, strips wholly outside hold the identity
            v4f g4[NS];
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const int q = j * 256 + 4 * lane;
                const int s0 = t0 - pad_left + j * 256;          // physical index of the strip's first element
                if (s0 >= 0 && s0 + 256 <= len) {
                    g4[j] = *(const v4f_u *)(xt + q);
                } else if (!PADDED && (s0 >= len || s0 + 256 <= 0)) {
                    g4[j] = (v4f){O::id(), O::id(), O::id(), O::id()};
                } else {
                    float e4[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int e = t0 + q + c;    // element of the extended row
                        const int src = (e >= 0 && e < lv) ? pad_src(e, len, pad_left, pad_mode) : -1;
                        e4[c] = src >= 0 ? xr[src] : O::id();
                    }
                    g4[j] = (v4f){e4[0], e4[1], e4[2], e4[3]};
                }
            }
#pragma unroll
            for (int j = 0; j < NS; ++j) *(v4f *)(A + strip_pos + 256 * j) = g4[j];
        }
        wave_lds_sync();
        // ---- my chunk of C consecutive elements
        float v[C];
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            const v4f g = *(const v4f *)(A + (chunk_pos ^ (4 * u)));
            v[4 * u] = g.x; v[4 * u + 1] = g.y; v[4 * u + 2] = g.z; v[4 * u + 3] = g.w;
        }
        // ---- pass 1: lane totals.  tail = my last segment's part inside the chunk (end of a
        //      forward scan), head = my first segment's part (end of a backward scan).
        float tail = v[0], head = v[C - 1];
#pragma unroll
        for (int k = 1; k < C; ++k) tail = G::f(tail, m[k], v[k]);
#pragma unroll
        for (int k = C - 2; k >= 0; --k) head = G::f(head, m[k + 1], v[k]);
        // ---- cross-lane: e = (+) of the tails of the n_pre lanes before me,
        //                  g = (+) of the heads of the n_suf lanes after me.
        float e = lane_read(tail, lane - 1);
        float g = lane_read(head, lane + 1);
        for (int d = 1; d < max_reach; d <<= 1) {
            const float te = lane_read(e, lane - d);
            const float tg = lane_read(g, lane + d);
            if (n_pre > d) e = O::f(te, e);
            if (n_suf > d) g = O::f(g, tg);
        }
        // ---- pass 2: the same scans seeded with the carries give the final in-segment
        //      prefix sums (in place over v) and suffix sums
        float suf[C];
        suf[C - 1] = G::f(g, m[C], v[C - 1]);
#pragma unroll
        for (int k = C - 2; k >= 0; --k) suf[k] = G::f(suf[k + 1], m[k + 1], v[k]);
        v[0] = G::f(e, m[0], v[0]);
#pragma unroll
        for (int k = 1; k < C; ++k) v[k] = G::f(v[k - 1], m[k], v[k]);
        // ---- chunks -> LDS (Pre over the staged inputs, Suf beside it)
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            *(v4f *)(A + (chunk_pos ^ (4 * u))) = (v4f){v[4 * u], v[4 * u + 1], v[4 * u + 2], v[4 * u + 3]};
            *(v4f *)(Bf + (chunk_pos ^ (4 * u))) = (v4f){suf[4 * u], suf[4 * u + 1], suf[4 * u + 2], suf[4 * u + 3]};
        }
        wave_lds_sync();
        // ---- combine on strips: y[q] = Suf[q] (+) Pre[q+S], then coalesced stores
        int lim = lo - t0;
        if (lim > tout) lim = tout;                              // (a tile past the row end has lim <= 0)
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const int q = j * 256 + 4 * lane;
            if (q >= lim) continue;
            const v4f s4v = *(const v4f *)(Bf + strip_pos + 256 * j);
            // the aligned groups holding Pre[q+S ..]; past the tile (discarded lanes only) wrap around
            const v4f p0 = *(const v4f *)(A + ((pre_pos0 + 256 * j) & (N - 1)));
            const v4f p1 = *(const v4f *)(A + ((pre_pos1 + 256 * j) & (N - 1)));
            v4f pn;
            switch (sh) {
            case 0: pn = p0; break;
            case 1: pn = (v4f){p0.y, p0.z, p0.w, p1.x}; break;
            case 2: pn = (v4f){p0.z, p0.w, p1.x, p1.y}; break;
            default: pn = (v4f){p0.w, p1.x, p1.y, p1.z}; break;
            }
            v4f o;
            o.x = O::f(s4v.x, pn.x); o.y = O::f(s4v.y, pn.y); o.z = O::f(s4v.z, pn.z); o.w = O::f(s4v.w, pn.w);
            if (!CHAIN) {
                if (PADDED && OP == SWS_OP_ADD && pad_mode == SWS_PAD_SHRINK) {
                    // the window shrinks at the ends of the row: rescale by w / (real elements in it)
                    float ov[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int e = t0 + q + c;    // first element of the window, in the extended row
                        const int hi = e + S + 1 < pad_left + len ? e + S + 1 : pad_left + len;
                        const int n = hi - (e > pad_left ? e : pad_left);
                        ov[c] *= scale * (float)(S + 1) / (float)(n > 0 ? n : 1);
                    }
                    o = (v4f){ov[0], ov[1], ov[2], ov[3]};
                } else if (OP == SWS_OP_ADD) o *= scale;
            } else {
                if (chain_acc) {                     // earlier links cover older elements: they go on the left
                    if (q >= qlo && q + 4 <= lim) {
                        const v4f old = *(const v4f_u *)(yt + q);
                        o.x = O::f(old.x, o.x); o.y = O::f(old.y, o.y); o.z = O::f(old.z, o.z); o.w = O::f(old.w, o.w);
                    } else {
                        if (q + 0 >= qlo && q + 0 < lim) o.x = O::f(yt[q + 0], o.x);
                        if (q + 1 >= qlo && q + 1 < lim) o.y = O::f(yt[q + 1], o.y);
                        if (q + 2 >= qlo && q + 2 < lim) o.z = O::f(yt[q + 2], o.z);
                        if (q + 3 >= qlo && q + 3 < lim) o.w = O::f(yt[q + 3], o.w);
                    }
                }
                if (OP == SWS_OP_ADD) o *= scale;    // 1 in every link but the last
            }
            if (q >= qlo && q + 4 <= lim) {
                if (flags & 2) __builtin_nontemporal_store(o, (v4f_u *)(yt + q));
                else *(v4f_u *)(yt + q) = o;
            } else {
                if (q + 0 >= qlo && q + 0 < lim) yt[q + 0] = o.x;
                if (q + 1 >= qlo && q + 1 < lim) yt[q + 1] = o.y;
                if (q + 2 >= qlo && q + 2 < lim) yt[q + 2] = o.z;
                if (q + 3 >= qlo && q + 3 < lim) yt[q + 3] = o.w;
            }
        }
        wave_lds_sync();                                         // the next tile overwrites A
        t += WPW;
        while (t >= tiles_per_row) { t -= tiles_per_row; ++r; }
    }
}

template <int OP>
hipError_t launch_direct(const float *x, float *y, int64_t rows, int len, int lo, int w, float scale,
                         hipStream_t s)
{
    // One strip per single-wavefront workgroup for large inputs (6.1-6.4 TB/s against 5.6 on x[32768,16384],
    // w = 2 .. 9) and for small ones (1 M elements: 3.4 us against 4.3 us cold, 3.1 against 3.2 warm, in a
    // graph); in between (4 M elements: 7.8 us against 8.9 us cold, but 6.3 against 4.7 us warm from the
    // last-level cache, where the launch rate of 16 K tiny workgroups is the limit) the tiles stay.
    // slide_chunk bit 16 forces tiles, bit 32 strips.
    const int64_t n_out = rows * (int64_t)lo;
    const bool fine = (n_out >= ((int64_t)1 << 24) || n_out <= ((int64_t)1 << 21) || (g_opt.slide_chunk & 32)) &&
                      !(g_opt.slide_chunk & 16);
    const int tile_out = fine ? 256 : 1024;
    const int tiles_per_row = (lo + max_origin_shift(lo, 16) + tile_out - 1) / tile_out;          // origins move back
    const int64_t n_tiles = rows * tiles_per_row;
    const int64_t n_units = fine ? n_tiles : (n_tiles + kWavesPerWg - 1) / kWavesPerWg;
    // strips go out in launch order (measured equal or better than the XCD-contiguous mapping: w = 9 6.38
    // against 6.18 TB/s); slide_chunk bit 4 forces the mapping on, bit 8 off
    const int remap = (g_opt.slide_chunk & 8) ? 0 : ((g_opt.slide_chunk & 4) || !fine ? 1 : 0);
    const int64_t grid = remap ? xcd_grid(n_units) : n_units;
    if (grid > 2147483647LL) return kNotTaken;
#define SWS_DIRECT(WV)                                                                                     \
    case WV:                                                                                               \
        if (fine)                                                                                          \
            hipLaunchKernelGGL((slide_direct_kernel<OP, WV, 1>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, \
                               len, lo, scale, tiles_per_row, n_tiles, remap);                             \
        else                                                                                               \
            hipLaunchKernelGGL((slide_direct_kernel<OP, WV, 4>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, \
                               len, lo, scale, tiles_per_row, n_tiles, remap);                             \
        break
    switch (w) {
        SWS_DIRECT(1); SWS_DIRECT(2); SWS_DIRECT(3); SWS_DIRECT(4); SWS_DIRECT(5);
        SWS_DIRECT(6); SWS_DIRECT(7); SWS_DIRECT(8); SWS_DIRECT(9);
        SWS_DIRECT(10); SWS_DIRECT(11);
    default: return kNotTaken;
    }
#undef SWS_DIRECT
    return hipGetLastError();
}

// slide_chunk option bits (A/B measurements): 1 = never align tiles, 2 = plain instead of
// non-temporal stores on aligned tiles, 4 = force the XCD-contiguous unit mapping on,
// 8 = force it off.
template <int OP>
hipError_t launch_scan(const float *x, float *y, int64_t rows, int len, int lo, int w, float scale,
                       int pad_left, int pad_mode, int lv, hipStream_t s, int chain = 0, int pitch = 0)
{
    constexpr int C = 16, N = kWave * C;
    const int S = w - 1;
    const int max_tout = N - S;
    const int opt = g_opt.slide_chunk;
    int flags = 0;
    // Unaligned plan: as few tiles per row as possible.  Aligned plan (preferred; measured
    // faster even when it costs one more tile per row): tile length a multiple of 16 floats and
    // origins pulled back per row so that every strip store starts on a 64-byte line of y,
    // which also makes non-temporal stores pay off.
    int tiles = (lo + max_tout - 1) / max_tout;
    int tout = (lo + tiles - 1) / tiles;
    if (!(opt & 1) && max_tout >= 16) {
        tout = max_tout & ~15;
        tiles = (lo + max_origin_shift(lo, 16) + tout - 1) / tout;
        flags |= 4;
        if (!(opt & 2)) flags |= 2;
    }
    // Few tiles per workgroup and many workgroups: the set of tiles in flight then stays a
    // compact window sweeping through memory.  Measured on 2 GiB inputs: one tile per wavefront
    // is best while the halo is small; with a large halo two tiles per wavefront and plain
    // round-robin placement of workgroups over the XCDs win.
    const int64_t n_tiles = rows * tiles;
    // (For + the first form stays ahead up to w = 170 — x[32768,16384], w = 80 .. 160: 5.98-6.08 TB/s
    // against 5.5-5.7 — while max / min already prefer the second from w = 80 on: 5.7-5.94 against 5.6-5.85.)
    const bool one_tile = S <= 64 || (OP == SWS_OP_ADD && S <= 172);
    // Nothing ties the four wavefronts of a workgroup together (no barrier, private LDS slices), and
    // single-wavefront workgroups measure a little faster on large plain inputs where the halo is
    // small or the scan is the slower one (x[32768,16384], TB/s, one / four wavefronts: w = 16 + 6.05 /
    // 5.94, max 5.98 / 5.92; w = 64 equal; w = 255 max 5.87 / 5.77, + with one tile per workgroup in
    // launch order 6.10 / 5.90; beyond w = 320 + is faster in the four-wavefront shape again: w = 400 0.79 against
    // 0.84 ms, w = 700 1.21 against 1.38).  Option slide_chunk bit 64 forces them, bit 128 the four-wavefront shape.
    const bool plain = !chain && lv == len;
    const bool big = rows * (int64_t)tiles >= 16384;
    const bool single = plain && !(opt & 128) && ((opt & 64) || (big && (S <= 32 || (S > 172 && (OP != SWS_OP_ADD || S <= 320)))));
    const int wpw = single ? 1 : kWavesPerWg;
    int64_t g = one_tile ? wpw : 2 * wpw;
    bool remap = one_tile;
    // one tile per workgroup for 172 < S <= 320, max / min too: with two, 1.17 x the input came from HBM (counters,
    // max w = 255) against 1.04 x with one, and the bench step's max w = 255 launch went from 0.725 to 0.705 ms
    if (single && S > 172 && S <= 320) g = 1;
    if (g_opt.slide_group > 0) g = (g_opt.slide_group + wpw - 1) / wpw * wpw;
    if (opt & 4) remap = true;
    if (opt & 8) remap = false;
    if (!remap) flags |= 32;
    // Inputs far beyond the caches are streamed while the halo is small (x[32768,16384], ms per launch, plain /
    // streamed loads: w = 16 0.725 / 0.661, 32 0.708 / 0.658, 64 0.709 / 0.677, 128 + 0.702 / 0.679, max 0.745 /
    // 0.714, 173 + 0.712 / 0.693, max level; beyond that streaming loses: w = 200 0.73 / 0.76-0.79, 255 0.71 / 0.80).
    // slide_chunk bit 256: plain loads.
    bool stream = false;
    if (!chain && rows * (int64_t)len >= ((int64_t)1 << 27) && !(opt & 256) && (S <= 128 || (OP == SWS_OP_ADD && S <= 172)))
        stream = true;
    const int64_t n_units = (n_tiles + g - 1) / g;
    const int64_t grid = remap ? xcd_grid(n_units) : n_units;
    if (grid > 2147483647LL) return kNotTaken;
    if (chain & 8) {                                  // a link over extended rows (chain bits: 1 = combine with y, 2 = last)
        if (!(chain & 2)) flags &= ~2;
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 3>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, len, lo,
                           S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, pad_left, pad_mode | ((chain & 1) << 8), lv);
    } else if (chain) {                               // chain bits: 1 = combine with y, 2 = last link
        if (!(chain & 2)) flags &= ~2;                // y is read again by the next link: plain stores
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 2>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, len, lo,
                           S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, 0, chain & 1, pitch);
    } else if (lv != len && stream) {                 // (the tiles at the ends of a row stage strip by strip, plainly)
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 1, kWavesPerWg, true>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y,
                           len, lo, S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, pad_left, pad_mode, lv);
    } else if (lv != len) {
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 1>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, len, lo,
                           S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, pad_left, pad_mode, lv);
    } else if (single && stream) {
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 0, 1, true>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, len, lo,
                           S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, 0, 0, len);
    } else if (stream) {
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 0, kWavesPerWg, true>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y,
                           len, lo, S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, 0, 0, len);
    } else if (single) {
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 0, 1>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, len, lo,
                           S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, 0, 0, len);
    } else {
        hipLaunchKernelGGL((slide_scan_kernel<OP, C, 0>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, len, lo,
                           S, scale, tiles, tout, (int)g, n_tiles, n_units, flags, 0, 0, len);
    }
    return hipGetLastError();
}

// Windows longer than one tile can hold: w = w_0 + w_1 + ... with every w_j within the scan
// kernel's reach, and  y[i] = Y_0[i] (+) Y_1[i + w_0] (+) Y_2[i + w_0 + w_1] ...  where Y_j is the
// sliding sum of window w_j (associativity; the links go oldest first, so operand order holds).
// Link j runs the scan kernel on the rows shifted by the earlier links' widths and combines its
// result with what is already in y.  Each link after the first re-reads y, so a window of P links
// moves 3P - 1 arrays instead of 2 — the work stays independent of w, where direct evaluation
// does w operations per output.
template <int OP>
hipError_t launch_chain(const float *x, float *y, int64_t rows, int len, int lo, int w, float scale, hipStream_t s)
{
    int reach = 768;                                 // longest link (a tile keeps >= 25 % of its elements as outputs)
    if ((g_opt.slide_chunk >> 8) > 1) reach = g_opt.slide_chunk >> 8;      // A/B: link length
    int links = (w + reach - 1) / reach;
    if (links < 2) links = 2;
    int done = 0;
    for (int j = 0; j < links; ++j) {
        const int wj = (w - done) / (links - j);    // near-equal widths, each >= 2
        const bool last = j == links - 1;
        const hipError_t e = launch_scan<OP>(x + done, y, rows, lo + wj - 1, lo, wj, last ? scale : 1.0f, 0, 0,
                                             lo + wj - 1, s, 4 | (j > 0 ? 1 : 0) | (last ? 2 : 0), len);
        if (e != hipSuccess) return e;
        done += wj;
    }
    return hipSuccess;
}

// The same over rows extended by a boundary rule: link j slides its window over the extended row
// from element off_j = w_0 + ... + w_{j-1} on, i.e. with pad_left - off_j elements in front (negative
// once the link starts inside the row) and an extended length of lo + w_j - 1.
template <int OP>
hipError_t launch_chain_padded(const float *x, float *y, int64_t rows, int len, int lo, int w, int pad_left, int pad_mode,
                               float scale, hipStream_t s)
{
    const int reach = 768;
    int links = (w + reach - 1) / reach;
    if (links < 2) links = 2;
    int done = 0;
    for (int j = 0; j < links; ++j) {
        const int wj = (w - done) / (links - j);
        const bool last = j == links - 1;
        const hipError_t e = launch_scan<OP>(x, y, rows, len, lo, wj, last ? scale : 1.0f, pad_left - done, pad_mode,
                                             lo + wj - 1, s, 8 | 4 | (j > 0 ? 1 : 0) | (last ? 2 : 0), 0);
        if (e != hipSuccess) return e;
        done += wj;
    }
    return hipSuccess;
}

constexpr int kStreamMinLen = 4096;                 // rows from this length on: large inputs go to the scan kernel's streamed loads
constexpr int kDirectMaxW = 11;                      // widest window of the shifted-load kernel (four 128-bit loads per lane)
constexpr int kScanMaxW = kWave * 16 - 64 + 1;      // leaves at least 64 outputs per wave tile
constexpr int kLongMinW = 449;                      // from here the long-window kernel beats the scan kernel (16384-long rows: w = 400 level, 512 1.1-1.4 x, 850 3 x)
constexpr int kLongMaxW = 8192;                     // the long-window kernel reads w - 1 extra inputs per tile: beyond this the chain moves less

}  // namespace

hipError_t launch_slide1d(int op, const float *x, float *y, int64_t rows, int64_t len64, int32_t w,
                          int32_t pad_left, int32_t pad_right, int pad_mode, float scale, hipStream_t s)
{
    const int len = (int)len64, lv = (int)(len64 + pad_left + pad_right), lo = lv - w + 1;
    const bool padded = pad_left != 0 || pad_right != 0;
    int variant = g_opt.slide_variant;
    if ((variant == 2 || variant == 4) && padded) variant = 0;      // those kernels know no boundary rule
    if (variant == 2 && w > kDirectMaxW) variant = 0;
    if (variant == 3 && (w < 2 || w > kScanMaxW)) variant = 0;
    if (variant == 4) return launch_slide1d_generic(op, x, y, rows, len64, w, scale, s);   // generic-operator kernel (A/B)
    if (variant == 7 && w > slide1d_rows_max_w()) variant = 0;
    if (variant == 8 && (w <= 256 || (padded && pad_mode == SWS_PAD_SHRINK))) variant = 0;   // the long-window kernel: w > 256
    if (variant == 9 && (padded || w < slide1d_reg_min_w() || w > slide1d_reg_max_w())) variant = 0;   // strips in registers: plain rows
    // Measured on 16384-long rows: the scan kernel's tiles are more and more halo as w grows; from w = 449 the
    // long-window kernel takes over, beyond its reach a chain of shorter windows.
    if (variant == 0) {
        // Windows up to 9 on short rows (every fifth tile of a 4096-long row is a border tile of
        // the scan kernel) or on small problems (latency-bound: fewer phases per tile): the
        // shifted-load kernel.  Measured, max, 2 GiB: 4096-long rows 0.76 ms against 0.79-0.82;
        // 16384-long rows 0.76-0.77 against 0.73-0.76; cfg 1 in a HIP graph 3.0-3.4 us against 4.3.
        // On large inputs its one-strip-per-wavefront form beats the scan kernel at any row length
        // (x[32768,16384], w = 2 .. 9: 6.1-6.4 TB/s against 5.9-6.0).
        // (Strips against the scan kernel there, TB/s: w = 10 6.07 / 5.85, w = 12 6.01 / 5.96, w = 16 4.7 / 5.96 —
        // beyond four 128-bit loads per lane the re-reads through L1 cost more than the scan's LDS passes.)
        // (Of the large inputs only w <= 4 and w = 9 stay here: the strips-in-registers kernel below measured level
        // or ahead for the other windows at every row length — x of 2^29 elements, ms, shifted loads / registers:
        // w = 5 rows of 1024 0.767 / 0.709, 2048 0.731 / 0.675, 8192 0.728 / 0.680, 65536 0.702 / 0.698; w = 11 rows of
        // 2048 1.04 / 0.70, 8192 0.83 / 0.675, 65536 level; w = 9 level everywhere.)
        const bool big_out = rows * (int64_t)lo >= (1LL << 24);
        const bool small_w = (w <= 9 && (lo <= 8192 || rows * len64 <= (8LL << 20))) || ((w <= 4 || w == 9) && big_out);
        // Rows too short for either: up to 256 outputs (one strip of the shifted-load kernel, a
        // quarter of the scan's wave tile) the short-row kernel for every window it has, several
        // rows per wavefront; up to 1024 outputs for the windows the shifted loads do not take.
        // Measured, max, TB/s, short-row kernel against the above: 262144 rows of 56 5.4-6.7 / 0.4-2.8;
        // 65536 x 224 5.4-6.7 / 5.2-6.0 (w <= 9), 1.9 (w >= 12); 32768 x 512 5.3-6.2 / 6.3-6.6 (w <= 9),
        // 5.8-6.5 / 3.5-4.3 (w >= 12); 16384 x 1024 5.9-6.3 / 3.7-6.2 (w >= 12); from 2048 no gain.
        // With a boundary rule the alternative is the scan kernel alone and the border strips cost
        // more as w grows (mirror, max, TB/s, short-row kernel / scan): rows of 56 5.5-1.4 / 0.4 for
        // w = 3 .. 33; 224 5.6-2.4 / 1.6 up to w = 16, 1.4 / 1.6 at 33; 1024 5.8-3.9 / 3.5 up to 16;
        // 2048 5.7-5.4 / 4.8-4.6 up to 9, 3.8 / 4.6 at 16.
        const bool streamed = !padded && w >= 2 && rows * len64 >= (1LL << 27) && len64 >= kStreamMinLen;
        const bool short_rows = w <= slide1d_rows_max_w() &&
                                (padded ? (lo <= 128 || (w <= 16 && lo <= 1024) || (w <= 9 && lo <= 2048))
                                        : (lo <= 256 || (w > 9 && lo <= 1024)));
        // A row that is exactly one tile of the scan kernel (1024-long rows with w - 1 a multiple of 16: all its
        // outputs in one aligned tile): x[524288,1024], w = 17 0.66 ms against 0.70 on the short-row kernel, w = 33
        // 0.65 against 0.98.
        const int tout1 = (kWave * 16 - (w - 1)) & ~15;
        const bool one_tile_rows = !padded && w > 16 && w < kLongMinW && lo > 768 && lo + max_origin_shift(lo, 16) <= tout1;
        if (one_tile_rows) variant = 3;
        else if (short_rows) variant = 7;
        else if (w == 1) variant = padded ? 1 : 2;
        else if (padded && pad_mode == SWS_PAD_SHRINK) variant = w <= kScanMaxW ? 3 : 1;   // one pass rescales by the real elements
        else if (padded) variant = w < kLongMinW ? 3 : (w <= kLongMaxW ? 8 : 6);   // 6: a chain over extended rows
        // Inputs far beyond the caches on long rows: the scan kernel loads streamed there (launch_scan) and is then
        // the fastest for nearly every small window too.  x[32768,16384], ms per launch, scan / the kernels below:
        // + w = 2 .. 8 0.656-0.660 / 0.688-0.706, 9 0.667 / 0.673, 10 0.661 / 0.702, 11 0.661 / 0.745, 12 .. 16
        // 0.662 / 0.681, 17 level; max w = 2 .. 8 0.673-0.678 / 0.694-0.708, 9 0.687 / 0.673, 10 0.681 / 0.703,
        // 11 0.683 / 0.741, 12 .. 16 level, 17 0.701 / 0.675.
        else if (streamed && w <= kDirectMaxW && !(w == 9 && op != SWS_OP_ADD)) variant = 3;
        else if (streamed && w >= 12 && w <= 16) variant = 3;
        // Large inputs, w = 5 .. 17 except 9: one strip per wavefront held in registers (strips overlap by 16 elements).
        // Measured on x[32768,16384], ms per 2 GiB, that kernel / the scan with plain loads: max 0.700-0.711 / 0.738,
        // + 0.699-0.703 / 0.710-0.715; from w = 18 the overlap is 32 elements and + loses (0.73 / 0.714), max gains
        // under 1.5 %.
        else if (w >= slide1d_reg_min_w() && w <= 17 && w != 9 && big_out) variant = 9;
        else if (small_w) variant = 2;
        else variant = w < kLongMinW ? 3 : (w <= kLongMaxW ? 8 : 5);
    }
    if (variant == 8) {
        const hipError_t e = launch_slide1d_long(op, x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, lv, s);
        if (e != kNotTaken) return e;
        variant = padded ? 6 : 5;
    }
    if (variant == 5) {                              // longer than a tile: a chain of windows
        if (padded || w < 4) variant = 1;
        else switch (op) {
            case SWS_OP_ADD: return launch_chain<SWS_OP_ADD>(x, y, rows, len, lo, w, scale, s);
            case SWS_OP_MAX: return launch_chain<SWS_OP_MAX>(x, y, rows, len, lo, w, scale, s);
            default: return launch_chain<SWS_OP_MIN>(x, y, rows, len, lo, w, scale, s);
        }
    }
    if (variant == 6) {
        switch (op) {
        case SWS_OP_ADD: return launch_chain_padded<SWS_OP_ADD>(x, y, rows, len, lo, w, pad_left, pad_mode, scale, s);
        case SWS_OP_MAX: return launch_chain_padded<SWS_OP_MAX>(x, y, rows, len, lo, w, pad_left, pad_mode, scale, s);
        default: return launch_chain_padded<SWS_OP_MIN>(x, y, rows, len, lo, w, pad_left, pad_mode, scale, s);
        }
    }
    if (variant == 9) {
        const hipError_t e = launch_slide1d_reg(op, x, y, rows, len, lo, w, scale, s);
        if (e != kNotTaken) return e;
        variant = 3;
    }
    if (variant == 7) {
        const hipError_t e = launch_slide1d_rows(op, x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, s);
        if (e != kNotTaken) return e;
        variant = w == 1 ? (padded ? 1 : 2) : 3;     // a grid beyond the launch limit
    }
    if (variant == 1) return launch_slide1d_naive(op, x, y, rows, len64, w, pad_left, pad_right, pad_mode, scale, s);
    if (variant == 2) {
        switch (op) {
        case SWS_OP_ADD: return launch_direct<SWS_OP_ADD>(x, y, rows, len, lo, w, scale, s);
        case SWS_OP_MAX: return launch_direct<SWS_OP_MAX>(x, y, rows, len, lo, w, scale, s);
        default: return launch_direct<SWS_OP_MIN>(x, y, rows, len, lo, w, scale, s);
        }
    }
    switch (op) {
    case SWS_OP_ADD: return launch_scan<SWS_OP_ADD>(x, y, rows, len, lo, w, scale, pad_left, pad_mode, lv, s);
    case SWS_OP_MAX: return launch_scan<SWS_OP_MAX>(x, y, rows, len, lo, w, scale, pad_left, pad_mode, lv, s);
    default: return launch_scan<SWS_OP_MIN>(x, y, rows, len, lo, w, scale, pad_left, pad_mode, lv, s);
    }
}

}  // namespace sws
