// sws_conv1d_16 — the 1-D convolution of conv1d.hip on 16-bit storage: x and y hold bf16 or fp16
// elements, the taps stay fp32.  Every element is widened to fp32 exactly, the sliding dot product
// (Section 2.5; Algorithm 4 with X <- X + f_t * Slide(...)) is accumulated in fp32 as in the fp32
// kernel, and each output is rounded to the storage type once, to nearest even.  The layer that is
// bound by HBM — one input channel per output channel (depthwise), stride 1, taps adjacent — moves
// half the bytes of the fp32 kernel; it is the tuned path.  Every other legal geometry runs on a
// direct-evaluation kernel (one thread per output).
//
// conv1d16_thin_kernel: a wavefront owns 1024 consecutive outputs of a row.  A lane's strip element
// is EIGHT 16-bit values (one 128-bit load, two strips of 512 per tile plus the k-1 halo), widened on
// the way into LDS, which turns strips into per-lane windows (16 + k - 1 consecutive inputs) and the
// per-lane outputs back into strips; eight results leave as one 128-bit non-temporal store.  Tile
// origins are pulled back so that every strip store starts on a 64-byte line of y.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerWg = kThreads / kWave;
constexpr int kTileOut = 1024;                       // outputs per wave tile (16 per lane)
constexpr int kThinMaxK16 = 64;

typedef float v8f __attribute__((ext_vector_type(8)));

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Eight 16-bit elements <-> eight floats.  Widening is exact; narrowing rounds to nearest even.
template <typename T> struct Io {
    typedef T v8 __attribute__((ext_vector_type(8)));
    typedef v8 v8_u __attribute__((aligned(2)));
    static __device__ __forceinline__ v8f load8(const T *p) { return __builtin_convertvector(*(const v8_u *)p, v8f); }
    static __device__ __forceinline__ float load1(const T *p) { return (float)*p; }
    static __device__ __forceinline__ void store1(T *p, float v) { *p = (T)v; }
    static __device__ __forceinline__ void store8(T *p, v8f o)
    {
        __builtin_nontemporal_store(__builtin_convertvector(o, v8), (v8_u *)p);
    }
};

// LDS layout of a wave tile (fp32): element q lives at q + 4*(q >> 4) — 4 floats of padding after every
// 16, so that a lane's window (from 16*lane on) starts 20 floats after its neighbour's and the 128-bit
// reads of eight consecutive lanes fall on eight different bank quads.
__host__ __device__ constexpr int lds_pos(int q) { return q + 4 * (q >> 4); }

template <int KB4, typename T>
__global__ __launch_bounds__(kThreads, (KB4 <= 8 ? 5 : 4)) void conv1d16_thin_kernel(
    const T *__restrict__ x, const float *__restrict__ wgt, T *__restrict__ y, int L, int Lo, int k, int pad,
    int Cin, int Cout, int cog, int tiles_per_row, int group, int chunks_per_row, int64_t n_units)
{
    using IO = Io<T>;
    constexpr int K4 = 4 * KB4;                      // taps, zero-padded to a multiple of 4
    constexpr int NI = kTileOut + K4;                // staged inputs per tile
    constexpr int NG = KB4 + 4;                      // 4-float groups in a lane's window
    constexpr int REGION = (lds_pos(NI + 8) + 63) / 64 * 64;
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
    const T *xr = x + (b * Cin + co / cog) * (int64_t)L;
    const float *wr = wgt + (int64_t)co * k;
    T *yr = y + ro * (int64_t)Lo;
    // Tile origins are pulled back by c so that (ro*Lo + t0) is a multiple of 32 elements: every
    // 1 KB strip store starts on a 64-byte line of y.  Outputs before the row start are dropped.
    const int c = (int)((ro * Lo) & 31);

    // Taps: one coalesced load (lane t holds tap t, zero beyond k), then broadcast into scalar registers.
    float f[K4];
    {
        float tv = wr[lane < k ? lane : 0];
        tv = lane < k ? tv : 0.0f;
#pragma unroll
        for (int t = 0; t < K4; ++t) f[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(tv), t));
    }

    const int wbase = 20 * lane;                     // my window: lds_pos(16*lane + 4u) = wbase + 4u + 4*(u >> 2)
    const int sbase = 8 * lane + 4 * (lane >> 1);    // my strip element: lds_pos(512j + 8*lane) = sbase + 640j

    // Strips of one tile (inputs [p0, p0 + NI)): 2 full strips plus the k-1 halo, zero outside the row.
    auto load_tile = [&](int t, v8f (&g)[3]) {
        const int p0 = t * kTileOut - c - pad;
        if (p0 >= 0 && p0 <= L - NI - 4) {           // (the halo strip reads whole groups of eight)
#pragma unroll
            for (int j = 0; j < 2; ++j) g[j] = IO::load8(xr + p0 + j * 512 + 8 * lane);
            g[2] = (8 * lane < K4) ? IO::load8(xr + p0 + kTileOut + 8 * lane) : (v8f){0, 0, 0, 0, 0, 0, 0, 0};
        } else {
            // a tile at an end of its row: strip by strip (wave-uniform tests) — whole strips inside
            // the row are still 128-bit loads, strips wholly outside are zero
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int s0 = p0 + j * 512;
                const int p = s0 + 8 * lane;
                if (s0 >= 0 && s0 + 512 <= L) {
                    g[j] = IO::load8(xr + p);
                } else if (s0 >= L || s0 + 512 <= 0) {
                    g[j] = (v8f){0, 0, 0, 0, 0, 0, 0, 0};
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) g[j][e] = (p + e >= 0 && p + e < L) ? IO::load1(xr + p + e) : 0.0f;
                }
            }
        }
    };

    int t_end = (chunk + 1) * group;
    if (t_end > tiles_per_row) t_end = tiles_per_row;
    int t = chunk * group + wave;
    v8f cur[3];
    if (t < t_end) load_tile(t, cur);
    for (; t < t_end; t += kWavesPerWg) {
        const int t0 = t * kTileOut - c;             // first output of the tile (may be < 0 for t = 0)
        // ---- the next tile's loads go out before this tile's arithmetic
        v8f nxt[3];
        if (t + kWavesPerWg < t_end) load_tile(t + kWavesPerWg, nxt);
        // ---- stage: strips -> LDS
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            *(v4f *)(A + sbase + 640 * j) = (v4f){cur[j][0], cur[j][1], cur[j][2], cur[j][3]};
            *(v4f *)(A + sbase + 640 * j + 4) = (v4f){cur[j][4], cur[j][5], cur[j][6], cur[j][7]};
        }
        if (8 * lane < K4) {                         // the halo: K4 elements, in groups of eight
            *(v4f *)(A + sbase + 1280) = (v4f){cur[2][0], cur[2][1], cur[2][2], cur[2][3]};
            *(v4f *)(A + sbase + 1284) = (v4f){cur[2][4], cur[2][5], cur[2][6], cur[2][7]};
        }
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
        for (int j = 0; j < 2; ++j) {
            const int q = j * 512 + 8 * lane;
            if (q >= lim) continue;
            const v4f o0 = *(const v4f *)(A + sbase + 640 * j), o1 = *(const v4f *)(A + sbase + 640 * j + 4);
            const v8f o = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w};
            if (q >= qlo && q + 8 <= lim) {
                IO::store8(yr + t0 + q, o);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (q + e >= qlo && q + e < lim) IO::store1(yr + t0 + q + e, o[e]);
            }
        }
        wave_lds_sync();
#pragma unroll
        for (int j = 0; j < 3; ++j) cur[j] = nxt[j];
    }
}

template <int KB4, typename T>
hipError_t launch_thin16(const T *x, const float *wgt, T *y, int64_t rows_out, int L, int Lo, int k, int pad, int Cin,
                         int Cout, int cog, hipStream_t s)
{
    const int tiles_per_row = (Lo + max_origin_shift(Lo, 32) + kTileOut - 1) / kTileOut;     // origins move back
    int64_t g = (KB4 <= 8 ? 2 : 16) * kWavesPerWg;
    if (g_opt.slide_group > 0) g = g_opt.slide_group;
    if (g > tiles_per_row) g = tiles_per_row;
    const int chunks_per_row = (int)((tiles_per_row + g - 1) / g);
    const int group = (tiles_per_row + chunks_per_row - 1) / chunks_per_row;     // even chunks
    const int64_t n_units = rows_out * chunks_per_row;
    const int64_t grid = xcd_grid(n_units);
    if (grid > 2147483647LL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv1d16_thin_kernel<KB4, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, wgt, y, L, Lo, k,
                       pad, Cin, Cout, cog, tiles_per_row, group, chunks_per_row, n_units);
    return hipGetLastError();
}

// Direct evaluation: one thread per output, taps in the oracle's order (input channel, then tap).
template <typename T>
__global__ __launch_bounds__(kThreads) void conv1d16_naive_kernel(const T *__restrict__ x, const float *__restrict__ wgt,
                                                                  T *__restrict__ y, int64_t B, int Cin, int L, int Cout,
                                                                  int Lo, int k, int stride, int pad, int dilation,
                                                                  int groups)
{
    const int cig = Cin / groups, cog = Cout / groups;
    const int64_t total = B * Cout * (int64_t)Lo;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int i = (int)(o % Lo);
        const int co = (int)((o / Lo) % Cout);
        const int64_t b = o / ((int64_t)Lo * Cout);
        const int g0 = (co / cog) * cig;
        float acc = 0.0f;
        for (int ci = 0; ci < cig; ++ci) {
            const T *xr = x + (b * Cin + g0 + ci) * (int64_t)L;
            const float *wr = wgt + ((int64_t)co * cig + ci) * k;
            for (int t = 0; t < k; ++t) {
                const int64_t p = (int64_t)i * stride - pad + (int64_t)t * dilation;
                if (p >= 0 && p < L) acc = fmaf(wr[t], (float)xr[p], acc);
            }
        }
        y[o] = (T)acc;
    }
}

template <typename T>
hipError_t conv1d_16(const T *x, const float *wgt, T *y, int64_t B, int64_t Cin, int64_t L, int64_t Cout, int64_t Lo,
                     int32_t k, int32_t stride, int32_t pad, int32_t dilation, int32_t groups, hipStream_t s)
{
    const int cig = (int)(Cin / groups);
    const bool thin_ok = cig == 1 && stride == 1 && dilation == 1 && k <= kThinMaxK16 && g_opt.conv1d_variant != 1;
    if (thin_ok) {
        const int cog = (int)(Cout / groups);
        hipError_t e = hipErrorInvalidValue;
#define SWS_THIN16(KB)                                                                                          \
    case KB:                                                                                                    \
        e = launch_thin16<KB, T>(x, wgt, y, B * Cout, (int)L, (int)Lo, k, pad, (int)Cin, (int)Cout, cog, s);    \
        break
        switch ((k + 3) / 4) {
            SWS_THIN16(1); SWS_THIN16(2); SWS_THIN16(3); SWS_THIN16(4); SWS_THIN16(5); SWS_THIN16(6); SWS_THIN16(7);
            SWS_THIN16(8); SWS_THIN16(9); SWS_THIN16(10); SWS_THIN16(11); SWS_THIN16(12); SWS_THIN16(13);
            SWS_THIN16(14); SWS_THIN16(15); SWS_THIN16(16);
        default: break;
        }
#undef SWS_THIN16
        if (e != hipErrorInvalidValue) return e;     // (a grid beyond the launch limit falls through)
    }
    int64_t grid = (B * Cout * Lo + kThreads - 1) / kThreads;
    if (grid > 1048576) grid = 1048576;
    hipLaunchKernelGGL((conv1d16_naive_kernel<T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, wgt, y, B, (int)Cin, (int)L,
                       (int)Cout, (int)Lo, k, stride, pad, dilation, groups);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv1d_16(int dtype, const void *x, const float *wgt, void *y, int64_t B, int64_t Cin, int64_t L,
                            int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad, int32_t dilation,
                            int32_t groups, hipStream_t s)
{
    if (dtype == SWS_DTYPE_BF16)
        return conv1d_16<__bf16>((const __bf16 *)x, wgt, (__bf16 *)y, B, Cin, L, Cout, Lo, k, stride, pad, dilation, groups, s);
    return conv1d_16<_Float16>((const _Float16 *)x, wgt, (_Float16 *)y, B, Cin, L, Cout, Lo, k, stride, pad, dilation,
                               groups, s);
}

}  // namespace sws
