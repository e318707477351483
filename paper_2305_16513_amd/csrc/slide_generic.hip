// Sliding window sum (Section 2.2, Eq. 3) for ANY associative operator on small tuples of
// floats, operand order preserved (older (+) newer), so it holds for non-commutative operators.
// Instantiated for the pair operator of Section 2.4 (Eq. 8),
//     (u_i, v_i) (+) (u_j, v_j) = (u_i * u_j, u_j * v_i + v_j),
// the composition of the maps z -> u z + v that turns a dot product into a prefix sum, and —
// as a cross-check of the tuned kernel — for plain +, max and min.
//
// Same scheme as the tuned scan kernel (the block form of Section 3, Algorithm 2): a wavefront
// owns a tile of 512 (1024 for w > 208) consecutive elements of a row, cut into segments of S = w - 1 elements
// counted from the tile origin.  For every element it forms
//     Pre[q] = x[segment start] (+) ... (+) x[q]      Suf[q] = x[q] (+) ... (+) x[segment end]
// and every output is one more operation:  y[q] = Suf[q] (+) Pre[q + S] — done in the lane's own chunk
// (Suf stays in registers, Pre[q + S ..] is read back from LDS at the window's offset), so that a tile
// needs one set of LDS planes, not two.
// A lane scans 8 (16) consecutive elements; lane totals are joined by segmented log-step scans across
// the wavefront (flag = "my elements contain a segment boundary"), then the in-lane scans run
// again seeded with the carries.  Segment resets are selects, so nothing is assumed about the
// operator beyond associativity.  Tuples are stored as separate planes (one array per component),
// which keeps every global access a coalesced 128-bit strip.
#include "sws_internal.h"

namespace sws {

namespace {

// Two tile shapes: 8 elements per lane (tile 512, 4 wavefronts per workgroup) for short windows,
// 16 per lane (tile 1024, 2 wavefronts per workgroup: the same LDS per workgroup) for long ones.
// Pairs on [16384,16384], % of HBM peak, tile 512 / 1024: w = 16 67 / 63, 128 67 / 61, 200 60 / 59,
// 255 52 / 58, 400 28 / 49.
constexpr int kSmallMaxW = 208;                      // measured break-even of the two shapes (pairs, 16384-long rows)
constexpr int kGenericMaxW = 961;                    // tile 1024: at least 64 outputs per tile

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// LDS position of element q of a plane: group g (4 floats) is moved within its block of 8 (16)
// groups so that 128-bit accesses are conflict-free both for strips (lane l at group l) and for
// per-lane chunks (lane l at groups 2l, 2l+1, or 4l .. 4l+3).
template <int PER> __device__ __forceinline__ int gpos(int q)
{
    const int g = q >> 2;
    const int gs = PER == 8 ? (g ^ ((g >> 3) & 1)) : (g ^ ((g >> 3) & 3) ^ (((g >> 5) & 1) << 3));
    return (gs << 2) | (q & 3);
}

// ---- operators: NP components, identity, r = a (+) b with a the older operand
struct PairOp {                                      // Section 2.4, Eq. 8
    static constexpr int NP = 2;
    static constexpr bool kScaled = false;
    static __device__ __forceinline__ void id(float (&a)[2]) { a[0] = 1.0f; a[1] = 0.0f; }
    static __device__ __forceinline__ void f(const float (&a)[2], const float (&b)[2], float (&r)[2])
    {
        r[0] = a[0] * b[0];
        r[1] = fmaf(b[0], a[1], b[1]);
    }
};
template <int OP> struct ScalarOp {                  // +, max, min of Eq. 3 / Section 2.3
    static constexpr int NP = 1;
    static constexpr bool kScaled = OP == SWS_OP_ADD;
    static __device__ __forceinline__ void id(float (&a)[1]) { a[0] = Op<OP>::id(); }
    static __device__ __forceinline__ void f(const float (&a)[1], const float (&b)[1], float (&r)[1])
    {
        r[0] = Op<OP>::f(a[0], b[0]);
    }
};

template <class O, int kPer>
__global__ __launch_bounds__(kPer == 8 ? 256 : 128) void slide_generic_kernel(const float *__restrict__ x0,
                                                                 const float *__restrict__ x1,
                                                                 float *__restrict__ y0, float *__restrict__ y1,
                                                                 int len, int lo, int S, int tout, int tiles_per_row,
                                                                 int64_t n_tiles, float scale, float inv_S, int pitch,
                                                                 int accum)
{
    // Rows are `pitch` apart and `len` of their elements are used; with `accum` the result is combined
    // with what y already holds (an earlier link of a chain of windows, which covers older elements).
    constexpr int NP = O::NP;
    constexpr int kTile = 64 * kPer, kWavesPerWg = kPer == 8 ? 4 : 2;
    // planes [0, NP): the inputs, then Pre, then the results (Suf never leaves the registers).  One
    // private slice per wavefront.
    __shared__ __attribute__((aligned(16))) float lds[kWavesPerWg][NP][kTile];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gt = (int64_t)blockIdx.x * kWavesPerWg + wave;
    if (gt >= n_tiles) return;                       // whole wavefronts leave; no workgroup barrier below
    const int64_t r = gt / tiles_per_row;
    const int t0 = (int)(gt - r * tiles_per_row) * tout;
    const float *xr[2] = {x0 + r * (int64_t)pitch, NP > 1 ? x1 + r * (int64_t)pitch : nullptr};
    float *yr[2] = {y0 + r * (int64_t)lo, NP > 1 ? y1 + r * (int64_t)lo : nullptr};
    float(*L)[kTile] = lds[wave];

    float ident[NP];
    O::id(ident);

    // ---- stage: two coalesced strips per plane, identity past the end of the row
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int j = 0; j < kTile / 256; ++j) {
            const int q = 256 * j + 4 * lane, gi = t0 + q;
            v4f v;
            if (gi + 4 <= len) {
                v = *(const v4f_u *)(xr[p] + gi);
            } else {
                v.x = gi + 0 < len ? xr[p][gi + 0] : ident[p];
                v.y = gi + 1 < len ? xr[p][gi + 1] : ident[p];
                v.z = gi + 2 < len ? xr[p][gi + 2] : ident[p];
                v.w = gi + 3 < len ? xr[p][gi + 3] : ident[p];
            }
            *(v4f *)(&L[p][gpos<kPer>(q)]) = v;
        }
    wave_lds_sync();

    // ---- my 8 consecutive elements
    float xe[kPer][NP];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int h = 0; h < kPer / 4; ++h) {
            const v4f v = *(const v4f *)(&L[p][gpos<kPer>(kPer * lane + 4 * h)]);
            xe[4 * h + 0][p] = v.x; xe[4 * h + 1][p] = v.y; xe[4 * h + 2][p] = v.z; xe[4 * h + 3][p] = v.w;
        }
    wave_lds_sync();                                 // every lane holds its inputs: the planes may be overwritten

    // ---- where the segments (S elements, counted from the tile origin) begin and end in my chunk
    bool st[kPer], en[kPer];
    {
        const int q0 = kPer * lane;
        int rr = q0 - (int)(((float)q0 + 0.5f) * inv_S) * S;      // q0 mod S (q0 < 1024: exact)
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            st[e] = rr == 0;
            en[e] = rr == S - 1;
            rr = rr + 1 == S ? 0 : rr + 1;
        }
    }
    auto sel = [](bool c, const float (&a)[NP], const float (&b)[NP], float (&r)[NP]) {
#pragma unroll
        for (int p = 0; p < NP; ++p) r[p] = c ? a[p] : b[p];
    };

    // ---- pass 1: what my chunk adds to a segment entering from the left (tail) / from the right (head)
    float tail[NP], head[NP], t[NP];
    bool has_start = false, has_end = false;
    O::id(tail);
    O::id(head);
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        O::f(tail, xe[e], t);
        sel(st[e], xe[e], t, tail);
        has_start |= st[e];
    }
#pragma unroll
    for (int e = kPer - 1; e >= 0; --e) {
        O::f(xe[e], head, t);
        sel(en[e], xe[e], t, head);
        has_end |= en[e];
    }

    // ---- segmented inclusive scans over the lanes, older operand always on the left
    {
        int fu = has_start, fd = has_end;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            float o[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p) o[p] = __shfl_up(tail[p], d, 64);
            const int fo = __shfl_up(fu, d, 64);
            O::f(o, tail, t);
            const bool take = lane >= d && !fu;
            sel(take, t, tail, tail);
            fu = take ? fo : fu;
#pragma unroll
            for (int p = 0; p < NP; ++p) o[p] = __shfl_down(head[p], d, 64);
            const int go = __shfl_down(fd, d, 64);
            O::f(head, o, t);
            const bool take_d = lane + d < 64 && !fd;
            sel(take_d, t, head, head);
            fd = take_d ? go : fd;
        }
    }
    // exclusive: what arrives from the lanes below / above me
    float carry_p[NP], carry_s[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const float a = __shfl_up(tail[p], 1, 64), b = __shfl_down(head[p], 1, 64);
        carry_p[p] = lane > 0 ? a : ident[p];
        carry_s[p] = lane < 63 ? b : ident[p];
    }

    // ---- pass 2: the in-lane scans again, seeded with the carries
    float pre[kPer][NP], suf[kPer][NP];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        O::f(carry_p, xe[e], t);
        sel(st[e], xe[e], t, carry_p);
#pragma unroll
        for (int p = 0; p < NP; ++p) pre[e][p] = carry_p[p];
    }
#pragma unroll
    for (int e = kPer - 1; e >= 0; --e) {
        O::f(xe[e], carry_s, t);
        sel(en[e], xe[e], t, carry_s);
#pragma unroll
        for (int p = 0; p < NP; ++p) suf[e][p] = carry_s[p];
    }

    // ---- exchange: Pre goes to LDS over the input planes; Suf stays in registers
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int h = 0; h < kPer / 4; ++h) {
            const int pos = gpos<kPer>(kPer * lane + 4 * h);
            *(v4f *)(&L[p][pos]) = (v4f){pre[4 * h][p], pre[4 * h + 1][p], pre[4 * h + 2][p], pre[4 * h + 3][p]};
        }
    wave_lds_sync();

    // ---- combine in the lane's own chunk: y[q + e] = Suf[q + e] (+) Pre[q + e + S], q = kPer * lane.  The
    //      kPer elements from q + S on lie in kPer/4 + 1 aligned groups (S mod 4 is the same for every
    //      lane); groups past the tile belong to outputs that are not stored and are read clamped.
    const int sh = S & 3;
    float o[kPer][NP];
    {
        const int g0 = (kPer * lane + S) >> 2;
        float wv[kPer + 4][NP];
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int h = 0; h <= kPer / 4; ++h) {
                const int gq = g0 + h < kTile / 4 ? g0 + h : kTile / 4 - 1;
                const v4f v = *(const v4f *)(&L[p][gpos<kPer>(4 * gq)]);
                wv[4 * h][p] = v.x; wv[4 * h + 1][p] = v.y; wv[4 * h + 2][p] = v.z; wv[4 * h + 3][p] = v.w;
            }
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            float b[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p)
                b[p] = sh == 0 ? wv[e][p] : (sh == 1 ? wv[e + 1][p] : (sh == 2 ? wv[e + 2][p] : wv[e + 3][p]));
            O::f(suf[e], b, o[e]);
        }
    }
    wave_lds_sync();                                 // every lane has read its Pre values: the planes are free again
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int h = 0; h < kPer / 4; ++h) {
            const int pos = gpos<kPer>(kPer * lane + 4 * h);
            *(v4f *)(&L[p][pos]) = (v4f){o[4 * h][p], o[4 * h + 1][p], o[4 * h + 2][p], o[4 * h + 3][p]};
        }
    wave_lds_sync();

    // ---- results back as strips, coalesced stores
    int lim = lo - t0;
    if (lim > tout) lim = tout;
#pragma unroll
    for (int j = 0; j < kTile / 256; ++j) {
        const int q = 256 * j + 4 * lane;
        if (q >= lim) continue;
        float o4[4][NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const v4f v = *(const v4f *)(&L[p][gpos<kPer>(q)]);
            o4[0][p] = v.x; o4[1][p] = v.y; o4[2][p] = v.z; o4[3][p] = v.w;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (accum && q + c < lim) {
                float old[NP], t2[NP];
#pragma unroll
                for (int p = 0; p < NP; ++p) old[p] = yr[p][t0 + q + c];
                O::f(old, o4[c], t2);
#pragma unroll
                for (int p = 0; p < NP; ++p) o4[c][p] = t2[p];
            }
            if (O::kScaled) o4[c][0] *= scale;
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (q + 4 <= lim) {
                *(v4f_u *)(yr[p] + t0 + q) = (v4f){o4[0][p], o4[1][p], o4[2][p], o4[3][p]};
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (q + c < lim) yr[p][t0 + q + c] = o4[c][p];
            }
        }
    }
}

// One thread per output, the window folded left to right: w = 1.
template <class O>
__global__ __launch_bounds__(256) void slide_generic_direct_kernel(const float *__restrict__ x0,
                                                                    const float *__restrict__ x1,
                                                                    float *__restrict__ y0, float *__restrict__ y1,
                                                                    int64_t rows, int len, int lo, int w, float scale)
{
    constexpr int NP = O::NP;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * lo) return;
    const int64_t r = idx / lo;
    const int i = (int)(idx - r * lo);
    const float *xr[2] = {x0 + r * (int64_t)len + i, NP > 1 ? x1 + r * (int64_t)len + i : nullptr};
    float acc[NP], b[NP], t[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = xr[p][0];
    for (int k = 1; k < w; ++k) {
#pragma unroll
        for (int p = 0; p < NP; ++p) b[p] = xr[p][k];
        O::f(acc, b, t);
#pragma unroll
        for (int p = 0; p < NP; ++p) acc[p] = t[p];
    }
    if (O::kScaled) acc[0] *= scale;
    y0[idx] = acc[0];
    if (NP > 1) y1[idx] = acc[NP - 1];
}

template <class O>
hipError_t launch_generic_tiles(const float *x0, const float *x1, float *y0, float *y1, int64_t rows, int len, int lo,
                                int w, float scale, int pitch, int accum, hipStream_t s)
{
    // (slide_group: A/B of the break-even; the 512-tile is never taken above w = 448, where it has 64 outputs left)
    const int small_max = g_opt.slide_group > 0 ? (g_opt.slide_group < 448 ? (int)g_opt.slide_group : 448) : kSmallMaxW;
    const bool small = w <= small_max;
    const int S = w - 1, tout = (small ? 512 : 1024) - S, waves = small ? 4 : 2;
    const int64_t tiles_per_row = (lo + tout - 1) / tout;
    const int64_t n_tiles = rows * tiles_per_row;
    const int64_t grid = (n_tiles + waves - 1) / waves;
    if (grid > 2147483647LL) return kNotTaken;
    if (small)
        hipLaunchKernelGGL((slide_generic_kernel<O, 8>), dim3((unsigned)grid), dim3(256), 0, s, x0, x1, y0, y1, len, lo, S,
                           tout, (int)tiles_per_row, n_tiles, scale, 1.0f / (float)S, pitch, accum);
    else
        hipLaunchKernelGGL((slide_generic_kernel<O, 16>), dim3((unsigned)grid), dim3(128), 0, s, x0, x1, y0, y1, len, lo, S,
                           tout, (int)tiles_per_row, n_tiles, scale, 1.0f / (float)S, pitch, accum);
    return hipGetLastError();
}

template <class O>
hipError_t launch_generic(const float *x0, const float *x1, float *y0, float *y1, int64_t rows, int64_t len, int32_t w,
                          float scale, hipStream_t s)
{
    const int64_t lo = len - w + 1;
    if (w >= 2 && w <= kGenericMaxW)
        return launch_generic_tiles<O>(x0, x1, y0, y1, rows, (int)len, (int)lo, w, scale, (int)len, 0, s);
    if (w > kGenericMaxW) {
        // A chain of shorter windows, w = w_0 + w_1 + ...:  y[i] = Y_0[i] (+) Y_1[i + w_0] (+) ...
        // (associativity; links oldest first, so the operand order holds).
        const int links = (w + 767) / 768;
        int done = 0;
        for (int j = 0; j < links; ++j) {
            const int wj = (w - done) / (links - j);
            const bool last = j == links - 1;
            const hipError_t e = launch_generic_tiles<O>(x0 + done, O::NP > 1 ? x1 + done : nullptr, y0, y1, rows,
                                                         (int)lo + wj - 1, (int)lo, wj, last ? scale : 1.0f, (int)len,
                                                         j > 0, s);
            if (e != hipSuccess) return e;
            done += wj;
        }
        return hipSuccess;
    }
    const int64_t grid = (rows * lo + 255) / 256;
    if (grid > 2147483647LL) return kNotTaken;
    hipLaunchKernelGGL((slide_generic_direct_kernel<O>), dim3((unsigned)grid), dim3(256), 0, s, x0, x1, y0, y1, rows,
                       (int)len, (int)lo, w, scale);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_slide1d_pair(const float *u, const float *v, float *yu, float *yv, int64_t rows, int64_t len,
                               int32_t w, hipStream_t s)
{
    return launch_generic<PairOp>(u, v, yu, yv, rows, len, w, 1.0f, s);
}

hipError_t launch_slide1d_generic(int op, const float *x, float *y, int64_t rows, int64_t len, int32_t w, float scale,
                                  hipStream_t s)
{
    switch (op) {
    case SWS_OP_ADD: return launch_generic<ScalarOp<SWS_OP_ADD>>(x, nullptr, y, nullptr, rows, len, w, scale, s);
    case SWS_OP_MAX: return launch_generic<ScalarOp<SWS_OP_MAX>>(x, nullptr, y, nullptr, rows, len, w, scale, s);
    default: return launch_generic<ScalarOp<SWS_OP_MIN>>(x, nullptr, y, nullptr, rows, len, w, scale, s);
    }
}

}  // namespace sws
