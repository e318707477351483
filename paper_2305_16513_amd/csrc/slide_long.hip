// Sliding window sums whose window is longer than a wave tile, in one pass (Section 3: the prefix and
// suffix sums of Algorithm 2, with the carry between vectors that a window spanning several of them
// needs).  For a tile of B outputs starting at i0 and a window w > B every window of the tile contains
// the same middle stretch, so
//
//   y[i0 + q] = Suf[q] (+) M (+) Pre[q]
//   Suf[q] = x[i0+q] (+) ... (+) x[i0+B-1]             suffix sums of the tile's own inputs
//   M      = x[i0+B] (+) ... (+) x[i0+w-2]             one reduction, shared by the B windows
//   Pre[q] = x[i0+w-1] (+) ... (+) x[i0+w-1+q]         prefix sums of the B inputs where the windows end
//
// — two scans of B elements and a reduction of w - 1 - B per tile, operands in window order.  A
// wavefront owns a tile; every element is read as part of a coalesced 128-bit strip (lane l holds
// elements 256 j + 4 l .. + 3 of strip j) and the scans run in that layout: inside a lane's four
// elements, across the 64 lanes of a strip (six ds_bpermute steps, the strips independent of each other),
// across the strips.  No LDS.  HBM sees x once and y once; the w - 1 inputs a tile shares with the tiles
// after it come from the L2 that neighbouring tiles (same XCD) have just filled.  The reduction uses that
// (+) is commutative for the three operators this kernel is instantiated for.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerWg = kThreads / kWave;

// Four consecutive elements of a row in memory: fp32, or bf16 / fp16 widened exactly on the way in and rounded
// to nearest even once on the way out.
template <typename T> struct Quad;
template <> struct Quad<float> {
    static __device__ __forceinline__ v4f load(const float *p) { return *(const v4f_u *)p; }
    static __device__ __forceinline__ float load1(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, v4f o) { __builtin_nontemporal_store(o, (v4f_u *)p); }
    static __device__ __forceinline__ void store1(float *p, float o) { *p = o; }
};
template <typename T> struct Quad {
    typedef T v4 __attribute__((ext_vector_type(4)));
    typedef v4 v4_u __attribute__((aligned(2)));
    static __device__ __forceinline__ v4f load(const T *p) { return __builtin_convertvector(*(const v4_u *)p, v4f); }
    static __device__ __forceinline__ float load1(const T *p) { return (float)*p; }
    static __device__ __forceinline__ void store(T *p, v4f o) { *(v4_u *)p = __builtin_convertvector(o, v4); }
    static __device__ __forceinline__ void store1(T *p, float o) { *p = (T)o; }
};

__device__ __forceinline__ float lane_read(float v, int src)        // v of lane src (any lane if src is out of range)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(4 * src, __builtin_bit_cast(int, v)));
}

// PADDED: the windows slide over the row extended by pad_left elements in front (and more behind, lv in all)
// under the boundary rule pad_mode; an element of the extended row is read from the row element the rule names.
template <int OP, int NS, bool PADDED, typename T>
__global__ __launch_bounds__(kThreads) void slide_long_kernel(const T *__restrict__ x, T *__restrict__ y, int len,
                                                              int lo, int w, float scale, int tiles_per_row,
                                                              int64_t n_tiles, int64_t n_units, int pad_left, int pad_mode,
                                                              int lv)
{
    using O = Op<OP>;
    constexpr int B = 256 * NS;                      // outputs per tile
    const int64_t unit = xcd_unit(n_units);
    if (unit < 0) return;
    const int lane = threadIdx.x & 63;
    const int64_t tile = unit * kWavesPerWg + (threadIdx.x >> 6);
    if (tile >= n_tiles) return;
    const int64_t r = tile / tiles_per_row;
    const int i0 = (int)(tile - r * tiles_per_row) * B;
    using Q = Quad<T>;
    const T *xr = x + r * (int64_t)len;
    T *yr = y + r * (int64_t)lo;
    const v4f id4 = {O::id(), O::id(), O::id(), O::id()};
    // four elements at index p .. p + 3 of the (extended) row, the identity beyond it
    auto load4 = [&](int p) -> v4f {
        if (PADDED) {
            const int q = p - pad_left;              // index in the physical row
            if (q >= 0 && q + 4 <= len) return Q::load(xr + q);
            float e[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int src = p + u < lv ? pad_src(p + u, len, pad_left, pad_mode) : -1;
                e[u] = src >= 0 ? Q::load1(xr + src) : O::id();
            }
            return (v4f){e[0], e[1], e[2], e[3]};
        }
        if (p + 4 <= len) return Q::load(xr + p);
        v4f v = id4;
        if (p < len) v.x = Q::load1(xr + p);
        if (p + 1 < len) v.y = Q::load1(xr + p + 1);
        if (p + 2 < len) v.z = Q::load1(xr + p + 2);
        return v;
    };
    v4f own[NS], end[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) own[j] = load4(i0 + 256 * j + 4 * lane);
#pragma unroll
    for (int j = 0; j < NS; ++j) end[j] = load4(i0 + w - 1 + 256 * j + 4 * lane);
    // ---- M: the middle stretch, w - 1 - B elements from i0 + B
    float mid = O::id();
    {
        const int cnt = w - 1 - B, m0 = i0 + B;
        v4f acc = id4;
        for (int k = 4 * lane; k < cnt; k += 256) {
            v4f v = load4(m0 + k);
            if (k + 4 > cnt) {                       // the stretch ends inside this group
                if (k + 1 >= cnt) v.y = O::id();
                if (k + 2 >= cnt) v.z = O::id();
                if (k + 3 >= cnt) v.w = O::id();
            }
            acc.x = O::f(acc.x, v.x); acc.y = O::f(acc.y, v.y); acc.z = O::f(acc.z, v.z); acc.w = O::f(acc.w, v.w);
        }
        mid = O::f(O::f(acc.x, acc.y), O::f(acc.z, acc.w));
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) mid = O::f(mid, lane_read(mid, lane ^ d));      // every lane ends with the total
    }
    // ---- Suf: suffix sums of the tile's own elements, in place
    {
        float tot[NS];
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            own[j].z = O::f(own[j].z, own[j].w);
            own[j].y = O::f(own[j].y, own[j].z);
            own[j].x = O::f(own[j].x, own[j].y);
            tot[j] = own[j].x;                       // my four elements of strip j
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1)             // inclusive suffix over the lanes of a strip
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const float u = lane_read(tot[j], lane + d);
                tot[j] = lane + d < 64 ? O::f(tot[j], u) : tot[j];
            }
        float carry = O::id();                       // the strips after strip j
#pragma unroll
        for (int j = NS - 1; j >= 0; --j) {
            const float after = lane_read(tot[j], lane + 1);             // the lanes after me in strip j
            const float rest = lane < 63 ? O::f(after, carry) : carry;
            own[j].x = O::f(own[j].x, rest); own[j].y = O::f(own[j].y, rest);
            own[j].z = O::f(own[j].z, rest); own[j].w = O::f(own[j].w, rest);
            carry = O::f(lane_read(tot[j], 0), carry);                   // strip j whole, then what followed it
        }
    }
    // ---- Pre: prefix sums of the elements where the windows end, in place
    {
        float tot[NS];
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            end[j].y = O::f(end[j].x, end[j].y);
            end[j].z = O::f(end[j].y, end[j].z);
            end[j].w = O::f(end[j].z, end[j].w);
            tot[j] = end[j].w;
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1)             // inclusive prefix over the lanes of a strip
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const float u = lane_read(tot[j], lane - d);
                tot[j] = lane >= d ? O::f(u, tot[j]) : tot[j];
            }
        float carry = O::id();                       // the strips before strip j
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const float before = lane_read(tot[j], lane - 1);
            const float rest = lane > 0 ? O::f(carry, before) : carry;
            end[j].x = O::f(rest, end[j].x); end[j].y = O::f(rest, end[j].y);
            end[j].z = O::f(rest, end[j].z); end[j].w = O::f(rest, end[j].w);
            carry = O::f(carry, lane_read(tot[j], 63));
        }
    }
    // ---- combine and store
#pragma unroll
    for (int j = 0; j < NS; ++j) {
        const int q = i0 + 256 * j + 4 * lane;
        v4f o;
        o.x = O::f(O::f(own[j].x, mid), end[j].x); o.y = O::f(O::f(own[j].y, mid), end[j].y);
        o.z = O::f(O::f(own[j].z, mid), end[j].z); o.w = O::f(O::f(own[j].w, mid), end[j].w);
        if (OP == SWS_OP_ADD) { o.x *= scale; o.y *= scale; o.z *= scale; o.w *= scale; }
        if (q + 4 <= lo) {
            Q::store(yr + q, o);
        } else {
            if (q < lo) Q::store1(yr + q, o.x);
            if (q + 1 < lo) Q::store1(yr + q + 1, o.y);
            if (q + 2 < lo) Q::store1(yr + q + 2, o.z);
        }
    }
}

template <int OP, int NS, typename T>
hipError_t launch_long(const T *x, T *y, int64_t rows, int len, int lo, int w, float scale, bool padded,
                       int pad_left, int pad_mode, int lv, hipStream_t s)
{
    constexpr int B = 256 * NS;
    const int tiles_per_row = (lo + B - 1) / B;
    const int64_t n_tiles = rows * tiles_per_row;
    const int64_t n_units = (n_tiles + kWavesPerWg - 1) / kWavesPerWg;
    const int64_t grid = xcd_grid(n_units);
    if (grid > 2147483647LL) return kNotTaken;
    if (padded)
        hipLaunchKernelGGL((slide_long_kernel<OP, NS, true, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, len, lo, w,
                           scale, tiles_per_row, n_tiles, n_units, pad_left, pad_mode, lv);
    else
        hipLaunchKernelGGL((slide_long_kernel<OP, NS, false, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, y, len, lo, w,
                           scale, tiles_per_row, n_tiles, n_units, 0, 0, len);
    return hipGetLastError();
}

}  // namespace

// Windows of more than 256 elements (tiles of 256, 512 or 1024 outputs: the largest the window exceeds), on plain
// rows or on rows extended by the identity / mirror / periodic / edge rule (lv = len + pads, lo = lv - w + 1
// outputs); kNotTaken: a shorter window, the shrinking-window mode, or a grid beyond the launch limit.
hipError_t launch_slide1d_long(int op, const float *x, float *y, int64_t rows, int len, int lo, int w, float scale,
                               bool padded, int pad_left, int pad_mode, int lv, hipStream_t s)
{
    if (w <= 256 || (padded && pad_mode == SWS_PAD_SHRINK)) return kNotTaken;
#define SWS_LONG(NS_)                                                                                              \
    switch (op) {                                                                                                  \
    case SWS_OP_ADD: return launch_long<SWS_OP_ADD, NS_>(x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, lv, s); \
    case SWS_OP_MAX: return launch_long<SWS_OP_MAX, NS_>(x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, lv, s); \
    default: return launch_long<SWS_OP_MIN, NS_>(x, y, rows, len, lo, w, scale, padded, pad_left, pad_mode, lv, s);         \
    }
    if (w <= 512) { SWS_LONG(1) }
    if (w <= 1024) { SWS_LONG(2) }
    SWS_LONG(4)
#undef SWS_LONG
}

// The same on 16-bit storage (dtype SWS_DTYPE_BF16 / SWS_DTYPE_F16; fp32 arithmetic, one rounding per output).
hipError_t launch_slide1d_long_16(int op, int dtype, const void *x, void *y, int64_t rows, int len, int lo, int w,
                                  float scale, hipStream_t s)
{
    if (w <= 256) return kNotTaken;
#define SWS_LONG16(T_, NS_)                                                                                        \
    switch (op) {                                                                                                  \
    case SWS_OP_ADD: return launch_long<SWS_OP_ADD, NS_, T_>((const T_ *)x, (T_ *)y, rows, len, lo, w, scale, false, 0, 0, len, s); \
    case SWS_OP_MAX: return launch_long<SWS_OP_MAX, NS_, T_>((const T_ *)x, (T_ *)y, rows, len, lo, w, scale, false, 0, 0, len, s); \
    default: return launch_long<SWS_OP_MIN, NS_, T_>((const T_ *)x, (T_ *)y, rows, len, lo, w, scale, false, 0, 0, len, s);         \
    }
    if (dtype == SWS_DTYPE_BF16) {
        if (w <= 512) { SWS_LONG16(__bf16, 1) }
        if (w <= 1024) { SWS_LONG16(__bf16, 2) }
        SWS_LONG16(__bf16, 4)
    }
    if (w <= 512) { SWS_LONG16(_Float16, 1) }
    if (w <= 1024) { SWS_LONG16(_Float16, 2) }
    SWS_LONG16(_Float16, 4)
#undef SWS_LONG16
}

}  // namespace sws
