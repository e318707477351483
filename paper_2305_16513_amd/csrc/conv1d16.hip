// sws_conv1d_16 — the 1-D convolution of conv1d.hip on 16-bit storage: x and y hold bf16 or fp16
// elements, the taps stay fp32.  Every element is widened to fp32 exactly, the sliding dot product
// (Section 2.5; Algorithm 4 with X <- X + f_t * Slide(...)) is accumulated in fp32 as in the fp32
// kernel, and each output is rounded to the storage type once, to nearest even.  The layer that is
// bound by HBM — one input channel per output channel (depthwise), stride 1, taps adjacent — moves
// half the bytes of the fp32 kernel; it is the tuned path.  Every other legal geometry runs on a
// direct-evaluation kernel (one thread per output).
//
// At half the bytes the vector ALU, not HBM, bounds a kernel that spends one FMA per tap and output
// (31 taps: 0.43 ms of FMA issue for the 256 x 128 x 16384 layer against 0.27 ms of HBM time), so the
// tuned kernel does the arithmetic on the matrix cores, exactly:
//
// conv1d16_mfma_kernel: a wavefront owns 1024 consecutive outputs of a row, seen as 32 blocks of 32:
//     out[32m + j] = sum_s T[j][s] * x[32m + s],   T[j][s] = f[s - j] (0 <= s - j < k, else 0),
// a (32 x S) by (S x 32) product with S = 31 + k rounded up to 16.  The B operand of
// v_mfma_f32_32x32x16_bf16 wants, per lane, eight consecutive k-indices of one column: eight
// consecutive elements of x, i.e. one 128-bit global load per 16 values of s with no LDS and no
// widening.  bf16 inputs are used as they are; an fp16 input is the exact sum of two bf16 numbers
// (8 + 3 significant bits).  An fp32 tap is the exact sum of three bf16 numbers (8 + 8 + 8 bits),
// so T is three bf16 matrices built once per wavefront and kept in registers.  Every product of two
// bf16 numbers is exact in fp32 and the matrix core accumulates in fp32: the result differs from the
// fp32 kernel's only in summation order.  The D layout leaves a lane with groups of four consecutive
// outputs; v_permlane32_swap pairs them into 128-bit non-temporal stores.  Tile origins are pulled
// back so that every store starts on a 64-byte line of y.  (Structural zeros of T multiply inputs up
// to 63 elements away from an output: the inputs must be finite.)
//
// conv1d16_thin_kernel (the vector-ALU kernel, kept for comparison): a wavefront owns 1024
// consecutive outputs of a row.  A lane's strip element is EIGHT 16-bit values (one 128-bit load, two
// strips of 512 per tile plus the k-1 halo), widened on the way into LDS, which turns strips into
// per-lane windows (16 + k - 1 consecutive inputs) and the per-lane outputs back into strips.
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
    if (grid > 2147483647LL) return kNotTaken;
    hipLaunchKernelGGL((conv1d16_thin_kernel<KB4, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, wgt, y, L, Lo, k,
                       pad, Cin, Cout, cog, tiles_per_row, group, chunks_per_row, n_units);
    return hipGetLastError();
}

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef v4u v4u_u __attribute__((aligned(2)));

template <typename T> struct Bits;
template <> struct Bits<__bf16> {
    static constexpr bool kSplit = false;            // the input is a bf16 number already
    static __device__ __forceinline__ unsigned pack2(float a, float b)
    {
        typedef __bf16 v2 __attribute__((ext_vector_type(2)));
        const v2 r = {(__bf16)a, (__bf16)b};
        return __builtin_bit_cast(unsigned, r);
    }
};
template <> struct Bits<_Float16> {
    static constexpr bool kSplit = true;             // fp16 = bf16 (top 8 bits) + bf16 (the other 3), exactly
    static __device__ __forceinline__ unsigned pack2(float a, float b)
    {
        typedef _Float16 v2 __attribute__((ext_vector_type(2)));
        const v2 r = {(_Float16)a, (_Float16)b};
        return __builtin_bit_cast(unsigned, r);
    }
};

__device__ __forceinline__ unsigned short bf16_bits(float f) { return __builtin_bit_cast(unsigned short, (__bf16)f); }

// Two fp16 values in a dword -> their leading bf16 parts and the exact remainders, each as a dword.
__device__ __forceinline__ void split_half2(unsigned w, unsigned &hi, unsigned &lo)
{
    typedef _Float16 v2h __attribute__((ext_vector_type(2)));
    const v2h p = __builtin_bit_cast(v2h, w);
    const float a = (float)p[0], b = (float)p[1];
    const unsigned ab = __float_as_uint(a), bb = __float_as_uint(b);
    const unsigned ah = ab & 0xffff0000u, bh = bb & 0xffff0000u;
    hi = (ab >> 16) | bh;
    const float al = a - __uint_as_float(ah), bl = b - __uint_as_float(bh);          // 3 significant bits
    lo = (__float_as_uint(al) >> 16) | (__float_as_uint(bl) & 0xffff0000u);
}

// NCH: 16-wide slices of s that a block of 32 outputs reads: 31 + k <= 16 * NCH.
template <int NCH, int PF, typename T>
__global__ __launch_bounds__(kThreads, (NCH <= 4 ? 4 : 3)) void conv1d16_mfma_kernel(
    const T *__restrict__ x, const float *__restrict__ wgt, T *__restrict__ y, int L, int Lo, int k, int pad, int Cin,
    int Cout, int cog, int tiles_per_row, int group, int chunks_per_row, int64_t n_wave_units)
{
    using BT = Bits<T>;
    constexpr int TLEN = 16 * NCH + 48;              // tap indices -32 .. 16*NCH + 15, one slot each
    constexpr int HALO = 16 * NCH - 32;              // inputs of a tile beyond its 1024: 0 .. 64
    constexpr int kInLen = 1152, kOutLen = 1088;     // padded lengths of 1024 + 64 inputs and of 1024 results
    __shared__ __attribute__((aligned(16))) unsigned short taps[kWavesPerWg][3][2][TLEN];
    __shared__ __attribute__((aligned(16))) unsigned short stage[kWavesPerWg][kInLen + kOutLen];

    // A work unit (a run of `group` tiles of one row) belongs to a wavefront, not to the workgroup.
    const int64_t ug = xcd_unit((n_wave_units + kWavesPerWg - 1) / kWavesPerWg);
    if (ug < 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t unit = ug * kWavesPerWg + wave;
    if (unit >= n_wave_units) return;                // (no workgroup barrier below)
    const int64_t ro = unit / chunks_per_row;        // output row = b*Cout + co
    const int chunk = (int)(unit - ro * chunks_per_row);
    const int64_t b = ro / Cout;
    const int co = (int)(ro - b * Cout);
    const unsigned short *xs = (const unsigned short *)(x + (b * Cin + co / cog) * (int64_t)L);
    const float *wr = wgt + (int64_t)co * k;
    unsigned short *ys = (unsigned short *)(y + ro * (int64_t)Lo);
    const int cshift = (int)((ro * Lo) & 31);        // (ro*Lo + tile origin) is a multiple of 32 elements
    const int m = lane & 31, h = lane >> 5;

    // ---- T as three bf16 matrices.  Slot p of copy X holds tap p - 32 - X (zero outside [0, k)), so
    // that the eight taps a lane needs, from tap 16c + 8h - j on, start on a dword in copy j & 1.
#pragma unroll
    for (int X = 0; X < 2; ++X)
        for (int p = lane; p < TLEN; p += kWave) {
            const int i = p - 32 - X;
            const float f = (i >= 0 && i < k) ? wr[i] : 0.0f;
            const __bf16 f1 = (__bf16)f;
            const float r1 = f - (float)f1;
            const __bf16 f2 = (__bf16)r1;
            const float r2 = r1 - (float)f2;
            taps[wave][0][X][p] = __builtin_bit_cast(unsigned short, f1);
            taps[wave][1][X][p] = __builtin_bit_cast(unsigned short, f2);
            taps[wave][2][X][p] = bf16_bits(r2);
        }
    wave_lds_sync();
    v8bf A[3][NCH];
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int pos = 16 * c + 8 * h - m + 32 + (m & 1);       // even, >= 2, pos + 7 < TLEN
            const unsigned *src = (const unsigned *)&taps[wave][p][m & 1][pos];
            const v4u q = {src[0], src[1], src[2], src[3]};
            A[p][c] = __builtin_bit_cast(v8bf, q);
        }

    // ---- LDS staging areas of this wavefront (16-bit elements).  Element q of a tile lives at
    // q + 8 * (q >> 7): 16 bytes of padding after every 256, which spreads the 64-byte stride of the
    // operand reads (and of the result writes) over all banks.  LDS operations of one wavefront execute
    // in order, so the areas need no double buffering.
    unsigned short *in = stage[wave];
    unsigned short *out = stage[wave] + kInLen;
    const int strip_pos = 8 * lane + 8 * (lane >> 4);                // element 512j + 8*lane sits at strip_pos + 544j
    int bpos[NCH];                                                   // operand slice c: elements 32m + 16c + 8h .. + 8
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int q = 32 * m + 16 * c + 8 * h;
        bpos[c] = q + 8 * (q >> 7);
    }
    const int dpos = 32 * m + 8 * (m >> 2) + 4 * h;                  // results 32m + 4h + 8g .. + 4 sit at dpos + 8g

    // ---- a tile's strips: lane l, strip j holds x[p0 + 512j + 8l .. + 8), zero outside the row
    auto load8 = [&](int q) -> v4u {
        if (q >= 0 && q + 8 <= L) return *(const v4u_u *)(xs + q);
        v4u z = {0u, 0u, 0u, 0u};
        if (q + 8 > 0 && q < L) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned v = (q + e >= 0 && q + e < L) ? (unsigned)xs[q + e] : 0u;
                z[e >> 1] |= v << (16 * (e & 1));
            }
        }
        return z;
    };
    auto load_tile = [&](int t, v4u (&g)[2], bool both) {            // `both` is false for the tile that only lends its head
        const int p0 = t * kTileOut - cshift - pad;
        if (p0 >= 0 && p0 + kTileOut <= L) {
            g[0] = *(const v4u_u *)(xs + p0 + 8 * lane);
            if (both) g[1] = *(const v4u_u *)(xs + p0 + 512 + 8 * lane);
        } else {
            g[0] = load8(p0 + 8 * lane);
            if (both) g[1] = load8(p0 + 512 + 8 * lane);
        }
    };

    // ---- one tile: strips (and the head of the next tile: the last HALO inputs) -> LDS -> operand
    // slices, 3 * NCH (bf16) or 6 * NCH (fp16) matrix instructions, results -> LDS -> strips -> y
    auto compute_tile = [&](int t, const v4u (&cur)[2], const v4u (&nxt)[2]) {
        const int t0 = t * kTileOut - cshift;        // first output of the tile (may be < 0 for t = 0)
        *(v4u *)(in + strip_pos) = cur[0];
        *(v4u *)(in + strip_pos + 544) = cur[1];
        if (8 * lane < HALO) *(v4u *)(in + 1088 + 8 * lane) = nxt[0];
        wave_lds_sync();
        v16f acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const v4u raw = *(const v4u *)(in + bpos[c]);
            if constexpr (BT::kSplit) {
                v4u hi, lo;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    unsigned hd, ld;
                    split_half2(raw[d], hd, ld);
                    hi[d] = hd;
                    lo[d] = ld;
                }
                const v8bf bh = __builtin_bit_cast(v8bf, hi), bl = __builtin_bit_cast(v8bf, lo);
#pragma unroll
                for (int p = 2; p >= 0; --p) {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[p][c], bl, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[p][c], bh, acc, 0, 0, 0);
                }
            } else {
                const v8bf bx = __builtin_bit_cast(v8bf, raw);
#pragma unroll
                for (int p = 2; p >= 0; --p) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[p][c], bx, acc, 0, 0, 0);
            }
        }
        // acc[v] is output 32m + 8*(v/4) + 4h + v%4: round, groups of four -> LDS, strips of eight back
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const v2u pr = {BT::pack2(acc[4 * g], acc[4 * g + 1]), BT::pack2(acc[4 * g + 2], acc[4 * g + 3])};
            *(v2u *)(out + dpos + 8 * g) = pr;
        }
        wave_lds_sync();
        const int lim = Lo - t0;
        const int qlo = t0 < 0 ? -t0 : 0;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int q = 512 * j + 8 * lane;
            if (q >= lim) continue;
            const v4u o = *(const v4u *)(out + strip_pos + 544 * j);
            if (q >= qlo && q + 8 <= lim) {
                __builtin_nontemporal_store(o, (v4u_u *)(ys + t0 + q));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (q + e >= qlo && q + e < lim) ys[t0 + q + e] = (unsigned short)(o[e >> 1] >> (16 * (e & 1)));
            }
        }
        wave_lds_sync();
    };

    // ---- the run of tiles t .. t_end - 1, with the loads of the next PF tiles in flight (PF + 1 register
    // slots in rotation).  Tile t_end is loaded too, first strip only: its head is the last tile's tail.
    int t_end = (chunk + 1) * group;
    if (t_end > tiles_per_row) t_end = tiles_per_row;
    int t = chunk * group;
    constexpr int D = PF + 1;
    v4u buf[D][2];
#pragma unroll
    for (int u = 0; u < D; ++u) buf[u][0] = buf[u][1] = (v4u){0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (t + u <= t_end) load_tile(t + u, buf[u], t + u < t_end);
    for (; t < t_end; t += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            if (t + u < t_end) {
                if (t + u + PF <= t_end) load_tile(t + u + PF, buf[(u + PF) % D], t + u + PF < t_end);
                compute_tile(t + u, buf[u], buf[(u + 1) % D]);
            }
        }
    }
}

template <int NCH, int PF, typename T>
hipError_t launch_mfma16(const T *x, const float *wgt, T *y, int64_t rows_out, int L, int Lo, int k, int pad, int Cin,
                         int Cout, int cog, hipStream_t s)
{
    const int tiles_per_row = (Lo + max_origin_shift(Lo, 32) + kTileOut - 1) / kTileOut;     // origins move back
    int64_t g = 16;
    if (g_opt.slide_group > 0) g = g_opt.slide_group;
    if (g > tiles_per_row) g = tiles_per_row;
    const int chunks_per_row = (int)((tiles_per_row + g - 1) / g);
    const int group = (tiles_per_row + chunks_per_row - 1) / chunks_per_row;     // even chunks
    const int64_t n_wave_units = rows_out * chunks_per_row;
    const int64_t grid = xcd_grid((n_wave_units + kWavesPerWg - 1) / kWavesPerWg);
    if (grid > 2147483647LL) return kNotTaken;
    hipLaunchKernelGGL((conv1d16_mfma_kernel<NCH, PF, T>), dim3((unsigned)grid), dim3(kThreads), 0, s, x, wgt, y, L, Lo, k,
                       pad, Cin, Cout, cog, tiles_per_row, group, chunks_per_row, n_wave_units);
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
    // conv1d_variant (A/B and tests): 1 forces direct evaluation, 2 the vector-ALU kernel
    const bool thin_ok = cig == 1 && stride == 1 && dilation == 1 && k <= kThinMaxK16 && g_opt.conv1d_variant != 1;
    if (thin_ok && g_opt.conv1d_variant != 2) {
        const int cog = (int)(Cout / groups);
        hipError_t e = kNotTaken;
        const int pf = g_opt.slide_chunk;            // tiles in flight ahead of the arithmetic: 2 (A/B: 1)
#define SWS_MFMA16(N)                                                                                           \
    case N:                                                                                                     \
        e = pf == 1 ? launch_mfma16<N, 1, T>(x, wgt, y, B * Cout, (int)L, (int)Lo, k, pad, (int)Cin, (int)Cout, cog, s) \
                    : launch_mfma16<N, 2, T>(x, wgt, y, B * Cout, (int)L, (int)Lo, k, pad, (int)Cin, (int)Cout, cog, s); \
        break
        switch ((31 + k + 15) / 16) {
            SWS_MFMA16(2); SWS_MFMA16(3); SWS_MFMA16(4); SWS_MFMA16(5); SWS_MFMA16(6);
        default: break;
        }
#undef SWS_MFMA16
        if (e != kNotTaken) return e;     // (a grid beyond the launch limit falls through)
    } else if (thin_ok) {
        const int cog = (int)(Cout / groups);
        hipError_t e = kNotTaken;
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
        if (e != kNotTaken) return e;     // (a grid beyond the launch limit falls through)
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
