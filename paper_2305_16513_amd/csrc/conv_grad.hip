// Adjoints of sws_conv1d (the training side of Section 2.5's sliding dot product).
//
//  * with respect to the input: at stride 1 the adjoint is itself a sliding dot product — over
//    the output gradients, taps last first, channels swapped inside each group, padding
//    span - 1 - pad — so it runs on the forward kernels, which read the weight array through
//    that view (no transformed copy is made).  At larger strides (dense channels) the cells of gx
//    fall into stride-many phases, each reached by every stride-th tap only: one stride-1 launch
//    of the matrix-core kernel per phase, stored with the stride.  Other cases: one thread per
//    input element.
//
//  * with respect to the weights: gw[co,ci,t] = sum over images and positions of
//    gy[b,co,i] * x[b,ci,i*stride + t*dilation - pad], a reduction over everything the forward
//    pass slides over.  Two tuned kernels (thin: stride 1; dense: stride 1 or 2 along the row,
//    any stride between rows, short rows packed several to a slab):
//      - thin (one input channel per output channel): a wavefront stages a tile of x and of gy
//        in LDS, a lane keeps 16 gradients and its window of x in registers and adds
//        gy[e] * x[e+t] into one accumulator per tap; tiles of the same channel follow each other,
//        so the cross-lane reduction happens once per workgroup, then one atomic add per tap.
//      - dense channels: per tap the product GY[co, positions] * X[ci, positions + t*d]^T on the
//        fp32 matrix cores (positions are the contraction index, split over workgroups and over
//        the wavefronts of a workgroup), partial blocks added through LDS, then atomic adds.
//    gw is cleared by a fill kernel first.  The order of the atomic adds is not fixed, so the
//    last bits of gw can differ from run to run; every other case: one workgroup per element.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerWg = kThreads / kWave;
constexpr int kTileOut = 1024;

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(float *__restrict__ p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) p[i] = 0.0f;
}

// ---------------------------------------------------------------------------------------------
// Direct evaluation.
// ---------------------------------------------------------------------------------------------
// gx[b, cin, j] = sum over co in the group and taps t with (j + pad - t*dilation) = i*stride,
// 0 <= i < Lo, of wgt[co, ci, t] * gy[b, co, i].
__global__ __launch_bounds__(kThreads) void conv1d_grad_input_naive_kernel(
    const float *__restrict__ gy, const float *__restrict__ wgt, float *__restrict__ gx, int64_t B, int Cin, int L,
    int Cout, int Lo, int k, int stride, int pad, int dilation, int groups)
{
    const int cig = Cin / groups, cog = Cout / groups;
    const int64_t total = B * (int64_t)Cin * L;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int j = (int)(o % L);
        const int c = (int)((o / L) % Cin);
        const int64_t b = o / ((int64_t)L * Cin);
        const int g = c / cig, ci = c - g * cig;
        float acc = 0.0f;
        for (int a = 0; a < cog; ++a) {
            const int co = g * cog + a;
            const float *gr = gy + (b * Cout + co) * (int64_t)Lo;
            const float *wr = wgt + ((int64_t)co * cig + ci) * k;
            for (int t = 0; t < k; ++t) {
                const int num = j + pad - t * dilation;
                if (num < 0 || num % stride) continue;
                const int i = num / stride;
                if (i < Lo) acc += wr[t] * gr[i];
            }
        }
        gx[o] = acc;
    }
}

// One workgroup per gw element: threads stride over (image, position), then a tree in LDS.
__global__ __launch_bounds__(kThreads) void conv1d_grad_weight_naive_kernel(
    const float *__restrict__ x, const float *__restrict__ gy, float *__restrict__ gw, int64_t B, int Cin, int L,
    int Cout, int Lo, int k, int stride, int pad, int dilation, int groups)
{
    __shared__ float part[kThreads];
    const int cig = Cin / groups, cog = Cout / groups;
    const int64_t e = blockIdx.x;                    // (co * cig + ci) * k + t
    const int t = (int)(e % k);
    const int ci = (int)((e / k) % cig);
    const int co = (int)(e / ((int64_t)k * cig));
    const int c = (co / cog) * cig + ci;
    float acc = 0.0f;
    const int64_t n = B * (int64_t)Lo;
    for (int64_t o = threadIdx.x; o < n; o += kThreads) {
        const int64_t b = o / Lo;
        const int i = (int)(o - b * Lo);
        const int j = i * stride + t * dilation - pad;
        if (j >= 0 && j < L) acc += gy[(b * Cout + co) * (int64_t)Lo + i] * x[(b * Cin + c) * (int64_t)L + j];
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int h = kThreads / 2; h > 0; h >>= 1) {
        if ((int)threadIdx.x < h) part[threadIdx.x] += part[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) gw[e] = part[0];
}

// ---------------------------------------------------------------------------------------------
// Thin channels (one input channel per output channel), stride 1, taps adjacent, k <= 64.
// ---------------------------------------------------------------------------------------------
// LDS layout of a staged tile: element q at q + 4*(q >> 4), so that a lane's window (from 16*lane)
// starts 20 floats after its neighbour's and the 128-bit reads of eight lanes hit eight bank quads.
__host__ __device__ constexpr int gpos(int q) { return q + 4 * (q >> 4); }

// Strips of 256 elements of row `src` (valid indices [0, n)) from index p0 on -> LDS, zero outside.
template <int STRIPS>
__device__ __forceinline__ void stage_row(float *dst, const float *__restrict__ src, int p0, int n, int lane)
{
    v4f g4[STRIPS];
#pragma unroll
    for (int j = 0; j < STRIPS; ++j) {
        const int s0 = p0 + 256 * j;                 // wave-uniform
        const int q = s0 + 4 * lane;
        if (s0 >= 0 && s0 + 256 <= n) {
            g4[j] = *(const v4f_u *)(src + q);
        } else if (s0 >= n || s0 + 256 <= 0) {
            g4[j] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        } else {
            float e4[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) e4[c] = (q + c >= 0 && q + c < n) ? src[q + c] : 0.0f;
            g4[j] = (v4f){e4[0], e4[1], e4[2], e4[3]};
        }
    }
#pragma unroll
    for (int j = 0; j < STRIPS; ++j) *(v4f *)(dst + gpos(256 * j + 4 * lane)) = g4[j];
}

template <int KB4>
__global__ __launch_bounds__(kThreads) void conv1d_thin_grad_weight_kernel(
    const float *__restrict__ x, const float *__restrict__ gy, float *__restrict__ gw, int B, int Cin, int L,
    int Cout, int Lo, int k, int pad, int cog, int tiles_per_row, int bgroup, int64_t n_units)
{
    constexpr int K4 = 4 * KB4;
    constexpr int XS = (kTileOut + K4 + 255) / 256;  // strips of x per tile
    constexpr int XREG = (gpos(256 * XS) + 63) / 64 * 64;
    constexpr int GREG = (gpos(kTileOut) + 63) / 64 * 64;
    constexpr int NG = KB4 + 4;                      // 4-float groups in a lane's window of x
    __shared__ __attribute__((aligned(16))) float lds[kWavesPerWg * (XREG + GREG)];
    __shared__ float red[kWavesPerWg][K4];

    const int64_t unit = blockIdx.x;
    if (unit >= n_units) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float *X = lds + wave * (XREG + GREG), *G = X + XREG;
    // consecutive workgroups take consecutive channels of the same images: adjacent rows of memory
    const int co = (int)(unit % Cout);
    const int b0 = (int)(unit / Cout) * bgroup;
    int b1 = b0 + bgroup;
    if (b1 > B) b1 = B;
    const int ci = co / cog;

    float acc[K4];
#pragma unroll
    for (int t = 0; t < K4; ++t) acc[t] = 0.0f;

    const int n_tiles = (b1 - b0) * tiles_per_row;
    for (int j = wave; j < n_tiles; j += kWavesPerWg) {
        const int b = b0 + j / tiles_per_row;
        const int t0 = (j % tiles_per_row) * kTileOut;
        const float *xr = x + ((int64_t)b * Cin + ci) * L;
        const float *gr = gy + ((int64_t)b * Cout + co) * Lo;
        stage_row<XS>(X, xr, t0 - pad, L, lane);
        stage_row<kTileOut / 256>(G, gr, t0, Lo, lane);
        wave_lds_sync();
        float gv[16], xw[4 * NG];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const v4f g = *(const v4f *)(G + 20 * lane + 4 * u);
            gv[4 * u] = g.x; gv[4 * u + 1] = g.y; gv[4 * u + 2] = g.z; gv[4 * u + 3] = g.w;
        }
#pragma unroll
        for (int u = 0; u < NG; ++u) {
            const v4f g = *(const v4f *)(X + 20 * lane + 20 * (u >> 2) + 4 * (u & 3));
            xw[4 * u] = g.x; xw[4 * u + 1] = g.y; xw[4 * u + 2] = g.z; xw[4 * u + 3] = g.w;
        }
#pragma unroll
        for (int t = 0; t < K4; ++t) {
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t] = __builtin_fmaf(gv[e], xw[e + t], acc[t]);
        }
        wave_lds_sync();                             // the next tile overwrites X and G
    }
    // ---- one total per tap: across lanes, then across the workgroup's wavefronts, then to memory
#pragma unroll
    for (int t = 0; t < K4; ++t) {
        float v = acc[t];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
        if (lane == 0) red[wave][t] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < k) {
        float v = 0.0f;
#pragma unroll
        for (int wv = 0; wv < kWavesPerWg; ++wv) v += red[wv][threadIdx.x];
        atomicAdd(gw + (int64_t)co * k + threadIdx.x, v);
    }
}

// ---------------------------------------------------------------------------------------------
// Dense channels (groups = 1), stride 1: per tap a 32 x 32 block of gw on the matrix cores.
// ---------------------------------------------------------------------------------------------
// A workgroup owns output channels [co0, co0+32), input channels [ci0, ci0+32) and KT taps from
// t0 on.  The contraction index is (image, position); it is split first over workgroups and then
// over the four wavefronts of a workgroup: wavefront w takes every fourth slab of 64 positions of
// the workgroup's range, stages GY[32][64] and X[32][64 + (KT-1)*d] (zero outside the rows) in its
// own LDS slice (row pitch = 2 mod 64: the 64 lanes of an operand read, 32 rows x 2 adjacent
// positions, hit 64 banks), the next slab's global loads in flight during the matrix work.  At
// the end the four accumulator sets are added through LDS and leave as atomic adds whose lanes run
// over (ci, tap), i.e. over contiguous memory.  Adds to one cache line serialise (measured
// roughly 0.1 us each), so the number of workgroups per block is kept near what fills the device.
constexpr int kPw = 64;                              // positions per wavefront slab
constexpr int kGPitch = kPw + 2;

// The same kernel serves the 2-D convolution: its contraction runs over (image, output row,
// position in the row), and a tap group is one kernel row a (or a part of it): the x row that
// output row ho meets is ho*sh - ph + a, or none (zeros) outside the plane.  1-D: H = Ho = kh = 1.
struct GwGeom {
    int Cin, Cout, L, Lo, k, pad, dilation;          // row lengths of x and gy, taps per kernel row, left padding
    int H, Ho, kh, sh, ph;                           // rows of x and gy per image, kernel rows, row stride, top padding
    int sw;                                          // stride along the row (1 or 2)
    int64_t x_cs, gy_cs;                             // channel strides (H*L, Ho*Lo)
    int segp, nseg;                                  // packed mode: positions per row segment, row segments per slab
    int64_t rows_total;                              // packed mode: images * Ho
};

// PACK: rows shorter than half a slab.  A slab then holds nseg row segments of segp = Lo + (KT-1)*d
// positions each: segment s is (image, output row) number slab*nseg + s, its gy values followed by
// (KT-1)*d zeros, and beside it the x positions those outputs meet, so that position p + t*d of the x
// slice is still the tap-t partner of position p of the gy slice.  What the zeros of gy multiply is
// real x data or zero, never stale LDS.  (Without it a 14-wide row would fill 14 of a slab's 64
// positions.)
// SW: stride along the row.  gy position p meets x position p*SW + t*d, so the x slice is
// (64 - 1)*SW + 1 + (KT-1)*d positions wide and, in packed mode, an x segment is segp*SW positions.
template <int KT, int XC, bool PACK = false, int SW = 1>
__global__ __launch_bounds__(kThreads) void conv1d_dense_grad_weight_kernel(
    const float *__restrict__ x, const float *__restrict__ gy, float *__restrict__ gw, GwGeom gm, int XPITCH,
    int slabs_per_row, int64_t total_slabs, int slabs, int co_blocks, int ci_blocks, int tap_groups)
{
    const int Cin = gm.Cin, Cout = gm.Cout, L = gm.L, Lo = gm.Lo, k = gm.k, pad = gm.pad, dilation = gm.dilation;
    extern __shared__ __attribute__((aligned(16))) float lds_dyn[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int slice = 32 * kGPitch + 32 * XPITCH;
    float *Gl = lds_dyn + wave * slice;              // [32][kGPitch]
    float *Xl = Gl + 32 * kGPitch;                   // [32][XPITCH]

    int64_t u = blockIdx.x;
    const int tg_all = (int)(u % tap_groups); u /= tap_groups;
    const int cib = (int)(u % ci_blocks); u /= ci_blocks;
    const int cob = (int)(u % co_blocks); u /= co_blocks;
    const int64_t slab0 = u * slabs;
    int64_t slab1 = slab0 + slabs;
    if (slab1 > total_slabs) slab1 = total_slabs;
    const int groups_per_krow = tap_groups / gm.kh;  // tap groups of one kernel row
    const int ka = tg_all / groups_per_krow, tg = tg_all - ka * groups_per_krow;     // my kernel row, my group in it
    const int co0 = cob * 32, ci0 = cib * 32, t0 = tg * KT;
    const int nt = (k - t0 < KT) ? k - t0 : KT;      // live taps of this group
    const int xw = (kPw - 1) * SW + 1 + (KT - 1) * dilation;     // staged x positions per slab
    // staging plan: 16 lanes per row of 64 positions (one float4 each), 4 rows per pass;
    // x rows are xw long: XV passes of 16 float4 columns
    const int srow = lane >> 4, scol = 4 * (lane & 15);
    constexpr int GV = 8;                            // 32 rows / 4
    constexpr int XCMAX = XC;                        // 64-position column blocks of an x row: ceil(xw / 64)

    v16f acc[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    v4f greg[GV], xreg[XCMAX][GV];
    auto load4 = [&](const float *row, int j, int n, bool row_ok) -> v4f {
        // elements j .. j+3 of a row of n elements, zero outside
        if (row_ok && j >= 0 && j + 4 <= n) return *(const v4f_u *)(row + j);
        v4f r;
        r.x = (row_ok && j >= 0 && j < n) ? row[j] : 0.0f;
        r.y = (row_ok && j + 1 >= 0 && j + 1 < n) ? row[j + 1] : 0.0f;
        r.z = (row_ok && j + 2 >= 0 && j + 2 < n) ? row[j + 2] : 0.0f;
        r.w = (row_ok && j + 3 >= 0 && j + 3 < n) ? row[j + 3] : 0.0f;
        return r;
    };
    auto prefetch_rows = [&](int64_t slab) {
        const int64_t rho = slab / slabs_per_row;    // (image, output row)
        const int i0 = (int)(slab - rho * slabs_per_row) * kPw;
        const int j0 = i0 * SW + t0 * dilation - pad;
        const int64_t b = rho / gm.Ho;
        const int ho = (int)(rho - b * gm.Ho);
        const int h = ho * gm.sh - gm.ph + ka;       // the x row this output row meets under kernel row ka
        const bool h_ok = h >= 0 && h < gm.H;
        const float *gyb = gy + b * Cout * gm.gy_cs + (int64_t)ho * Lo;
        const float *xb_ = x + b * Cin * gm.x_cs + (int64_t)(h_ok ? h : 0) * L;
#pragma unroll
        for (int p = 0; p < GV; ++p) {
            const int row = 4 * p + srow;
            const int co = co0 + row, ci = ci0 + row;
            greg[p] = load4(gyb + (co < Cout ? co : 0) * gm.gy_cs, i0 + scol, Lo, co < Cout);
#pragma unroll
            for (int c = 0; c < XCMAX; ++c) {
                // lanes whose four columns lie beyond the staged width load nothing
                xreg[c][p] = load4(xb_ + (ci < Cin ? ci : 0) * gm.x_cs, j0 + 64 * c + scol, L,
                                   h_ok && ci < Cin && 64 * c + scol < xw);
            }
        }
    };
    // packed mode: which (segment, offset) each of my columns is does not change from slab to slab
    auto prefetch_packed = [&](int64_t slab) {
        const int64_t rho0 = slab * gm.nseg;
        const int64_t b0 = rho0 / gm.Ho;
        const int ho0 = (int)(rho0 - b0 * gm.Ho);
        int64_t goff[4], xoff[XCMAX][4];
        bool gok[4], xok[XCMAX][4];
#pragma unroll
        for (int c = 0; c <= XCMAX; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int q = (c == 0 ? 0 : 64 * (c - 1)) + scol + e;     // c = 0: gy columns; c >= 1: x column block c - 1
                const int sp = c == 0 ? gm.segp : gm.segp * SW;           // positions per segment in this slice
                const int sg = q / sp, o = q - sg * sp;
                const int tr = ho0 + sg;
                const int64_t b = b0 + tr / gm.Ho;
                const int ho = tr % gm.Ho;
                const bool seg_ok = sg < gm.nseg && rho0 + sg < gm.rows_total;
                if (c == 0) {
                    gok[e] = seg_ok && o < Lo;
                    goff[e] = b * Cout * gm.gy_cs + (int64_t)ho * Lo + o;
                } else {
                    const int col = t0 * dilation - pad + o;
                    const int h = ho * gm.sh - gm.ph + ka;
                    xok[c > 0 ? c - 1 : 0][e] = seg_ok && q < xw && col >= 0 && col < L && h >= 0 && h < gm.H;
                    xoff[c > 0 ? c - 1 : 0][e] = b * Cin * gm.x_cs + (int64_t)h * L + col;
                }
            }
#pragma unroll
        for (int p = 0; p < GV; ++p) {
            const int row = 4 * p + srow;
            const int co = co0 + row, ci = ci0 + row;
            const float *gr = gy + (co < Cout ? co : 0) * gm.gy_cs;
            const float *xr = x + (ci < Cin ? ci : 0) * gm.x_cs;
            greg[p].x = (gok[0] && co < Cout) ? gr[goff[0]] : 0.0f;
            greg[p].y = (gok[1] && co < Cout) ? gr[goff[1]] : 0.0f;
            greg[p].z = (gok[2] && co < Cout) ? gr[goff[2]] : 0.0f;
            greg[p].w = (gok[3] && co < Cout) ? gr[goff[3]] : 0.0f;
#pragma unroll
            for (int c = 0; c < XCMAX; ++c) {
                xreg[c][p].x = (xok[c][0] && ci < Cin) ? xr[xoff[c][0]] : 0.0f;
                xreg[c][p].y = (xok[c][1] && ci < Cin) ? xr[xoff[c][1]] : 0.0f;
                xreg[c][p].z = (xok[c][2] && ci < Cin) ? xr[xoff[c][2]] : 0.0f;
                xreg[c][p].w = (xok[c][3] && ci < Cin) ? xr[xoff[c][3]] : 0.0f;
            }
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int p = 0; p < GV; ++p) {
            const int row = 4 * p + srow;
            float *gd = Gl + row * kGPitch + scol;
            gd[0] = greg[p].x; gd[1] = greg[p].y; gd[2] = greg[p].z; gd[3] = greg[p].w;
#pragma unroll
            for (int c = 0; c < XCMAX; ++c) {
                const int col = 64 * c + scol;
                float *xd = Xl + row * XPITCH + col;
                if (col + 0 < xw) xd[0] = xreg[c][p].x;
                if (col + 1 < xw) xd[1] = xreg[c][p].y;
                if (col + 2 < xw) xd[2] = xreg[c][p].z;
                if (col + 3 < xw) xd[3] = xreg[c][p].w;
            }
        }
    };

    int64_t slab = slab0 + wave;
    if (slab < slab1) {
        if constexpr (PACK) prefetch_packed(slab);
        else prefetch_rows(slab);
    }
    for (; slab < slab1; slab += kWavesPerWg) {
        commit();
        wave_lds_sync();
        if (slab + kWavesPerWg < slab1) {            // in flight during the matrix work
            if constexpr (PACK) prefetch_packed(slab + kWavesPerWg);
            else prefetch_rows(slab + kWavesPerWg);
        }
        const float *ga = Gl + l32 * kGPitch + half;
        const float *xb = Xl + l32 * XPITCH + half * SW;   // my gy position is ip + half
#pragma unroll 4
        for (int ip = 0; ip < kPw; ip += 2) {
            const float a = ga[ip];
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const float bv = xb[ip * SW + t * dilation];
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc[t], 0, 0, 0);
            }
        }
        wave_lds_sync();                             // the next slab overwrites the slice
    }
    // ---- add the four wavefronts' accumulators through LDS.  Register v of lane (l32, half) is
    //      row 8*(v/4) + 4*half + v%4 (co), column l32 (ci); it goes to red[wave][row][ci*KT + t].
    constexpr int RP = 32 * KT + 1;                  // row pitch of a reduction plane
    __syncthreads();                                 // every slice is free
    float *red = lds_dyn + wave * (32 * RP);
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[(8 * (v >> 2) + 4 * half + (v & 3)) * RP + l32 * KT + t] = acc[t][v];
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * 32 * KT; idx += kThreads) {
        const int row = idx / (32 * KT), rest = idx - row * (32 * KT);      // rest = ci*KT + t
        const int ci = rest / KT, t = rest - ci * KT;
        float v = 0.0f;
#pragma unroll
        for (int wv = 0; wv < kWavesPerWg; ++wv) v += lds_dyn[wv * (32 * RP) + row * RP + rest];
        if (co0 + row < Cout && ci0 + ci < Cin && t < nt)
            atomicAdd(gw + (((int64_t)(co0 + row) * Cin + ci0 + ci) * gm.kh + ka) * k + t0 + t, v);
    }
}

template <int KB4>
hipError_t launch_thin_gw(const float *x, const float *gy, float *gw, int B, int Cin, int L, int Cout, int Lo, int k,
                          int pad, int cog, hipStream_t s)
{
    const int tiles_per_row = (Lo + kTileOut - 1) / kTileOut;
    // images per workgroup: at least 16 tiles per wavefront (the reduction at the end costs about
    // one tile's worth of work), but keep a few thousand workgroups when the problem allows
    int bgroup = (64 + tiles_per_row - 1) / tiles_per_row;
    while (bgroup > 1 && (int64_t)Cout * ((B + bgroup - 1) / bgroup) < 2048) bgroup = (bgroup + 1) / 2;
    const int64_t n_units = (int64_t)Cout * ((B + bgroup - 1) / bgroup);
    if (n_units > 2147483647LL) return kNotTaken;
    hipLaunchKernelGGL((conv1d_thin_grad_weight_kernel<KB4>), dim3((unsigned)n_units), dim3(kThreads), 0, s, x, gy, gw,
                       B, Cin, L, Cout, Lo, k, pad, cog, tiles_per_row, bgroup, n_units);
    return hipGetLastError();
}

template <int KT, int SW>
hipError_t launch_dense_gw(const float *x, const float *gy, float *gw, int64_t B, const GwGeom &gm_in, hipStream_t s,
                           bool *taken)
{
    GwGeom gm = gm_in;
    const int xw = (kPw - 1) * SW + 1 + (KT - 1) * gm.dilation;
    const int XPITCH = (xw + 61) / 64 * 64 + 2;      // >= xw, = 2 mod 64
    const size_t stage = (size_t)kWavesPerWg * (32 * kGPitch + 32 * XPITCH) * sizeof(float);
    const size_t red = (size_t)kWavesPerWg * 32 * (32 * KT + 1) * sizeof(float);
    const size_t lds = stage > red ? stage : red;
    *taken = lds <= 156 * 1024 && xw <= 256;        // above 64 KB the kernel's LDS limit is raised below
    if (!*taken) return hipSuccess;
    const int slabs_per_row = (gm.Lo + kPw - 1) / kPw;
    // rows of at most half a slab (with their tap margin) are packed several to a slab
    gm.segp = gm.Lo + ((KT - 1) * gm.dilation + SW - 1) / SW;
    gm.nseg = kPw / gm.segp;
    gm.rows_total = B * gm.Ho;
    const bool pack = gm.nseg >= 2 && xw <= 64 * (SW + 1) && g_opt.conv2d_variant != 3;
    const int64_t total_slabs = pack ? (gm.rows_total + gm.nseg - 1) / gm.nseg : B * gm.Ho * slabs_per_row;
    const int co_blocks = (gm.Cout + 31) / 32, ci_blocks = (gm.Cin + 31) / 32;
    const int tap_groups = gm.kh * ((gm.k + KT - 1) / KT);
    const int64_t blocks = (int64_t)co_blocks * ci_blocks * tap_groups;
    // Split of the contraction over workgroups: about 128 per block of gw (each ends with atomic
    // adds to the same cache lines, which serialise), more when there are so few blocks that 128
    // would leave the device idle; at least one slab per wavefront.  Measured, slabs per workgroup
    // 8 / 12 / 16 / 32 / 64: x[16,64,4096], 64 -> 64, k = 3 (4 blocks, 1024 slabs): 39 / 44 / 44 / 70 /
    // 124 us; [32,64,56,56], 3 x 3 (12 blocks, 1792 slabs): 199 / 176 / 180 / 190 / 204 us.
    int64_t nsplit = 512 / blocks > 128 ? 512 / blocks : 128;
    int64_t slabs = (total_slabs + nsplit - 1) / nsplit;
    if (slabs < kWavesPerWg) slabs = kWavesPerWg;
    if (g_opt.slide_group > 0) slabs = g_opt.slide_group;           // A/B: slabs per workgroup
    const int64_t grid = blocks * ((total_slabs + slabs - 1) / slabs);
    if (grid > 2147483647LL || slabs > 2147483647LL) { *taken = false; return hipSuccess; }
#define SWS_DGW(XC, PACK)                                                                                         \
    case XC:                                                                                                      \
        if (lds > 64 * 1024) {                                                                                    \
            const hipError_t ea = hipFuncSetAttribute((const void *)conv1d_dense_grad_weight_kernel<KT, XC, PACK, SW>, \
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);      \
            if (ea != hipSuccess) return ea;                                                                      \
        }                                                                                                         \
        hipLaunchKernelGGL((conv1d_dense_grad_weight_kernel<KT, XC, PACK, SW>), dim3((unsigned)grid), dim3(kThreads), \
                           lds, s, x, gy, gw, gm, XPITCH, slabs_per_row, total_slabs, (int)slabs, co_blocks,      \
                           ci_blocks, tap_groups);                                                                \
        break
    if constexpr (SW == 2) {                         // slices of 127 + (KT-1)*d positions: two or three column blocks
        if (pack) {
            switch ((xw + 63) / 64) {
                SWS_DGW(2, true); SWS_DGW(3, true);
            default: *taken = false; return hipSuccess;
            }
        } else {
            switch ((xw + 63) / 64) {
                SWS_DGW(2, false); SWS_DGW(3, false);
            default: *taken = false; return hipSuccess;
            }
        }
    } else {
        if (pack) {
            switch ((xw + 63) / 64) {
                SWS_DGW(1, true); SWS_DGW(2, true);
            default: *taken = false; return hipSuccess;
            }
        } else {
            switch ((xw + 63) / 64) {
                SWS_DGW(1, false); SWS_DGW(2, false); SWS_DGW(3, false); SWS_DGW(4, false);
            default: *taken = false; return hipSuccess;
            }
        }
    }
#undef SWS_DGW
    return hipGetLastError();
}

// taps per workgroup: all of a kernel row up to 4, else groups of 4 (16 accumulator registers per tap)
hipError_t launch_dense_gw_taps(const float *x, const float *gy, float *gw, int64_t B, const GwGeom &gm, hipStream_t s,
                                bool *taken)
{
    if (gm.sw == 2) {
        if (gm.k == 1) return launch_dense_gw<1, 2>(x, gy, gw, B, gm, s, taken);
        if (gm.k == 2) return launch_dense_gw<2, 2>(x, gy, gw, B, gm, s, taken);
        if (gm.k == 3) return launch_dense_gw<3, 2>(x, gy, gw, B, gm, s, taken);
        return launch_dense_gw<4, 2>(x, gy, gw, B, gm, s, taken);
    }
    if (gm.sw != 1) { *taken = false; return hipSuccess; }
    if (gm.k == 1) return launch_dense_gw<1, 1>(x, gy, gw, B, gm, s, taken);
    if (gm.k == 2) return launch_dense_gw<2, 1>(x, gy, gw, B, gm, s, taken);
    if (gm.k == 3) return launch_dense_gw<3, 1>(x, gy, gw, B, gm, s, taken);
    return launch_dense_gw<4, 1>(x, gy, gw, B, gm, s, taken);
}

// ---------------------------------------------------------------------------------------------
// Direct evaluation of the 2-D adjoints.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void conv2d_grad_input_naive_kernel(
    const float *__restrict__ gy, const float *__restrict__ wgt, float *__restrict__ gx, int64_t N, int Cin, int H,
    int W, int Cout, int Ho, int Wo, int kh, int kw, int sh, int sw, int ph, int pw)
{
    const int64_t total = N * (int64_t)Cin * H * W;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int c = (int)(o % W);
        const int h = (int)((o / W) % H);
        const int ci = (int)((o / ((int64_t)W * H)) % Cin);
        const int64_t n = o / ((int64_t)W * H * Cin);
        // the taps that reach this cell: a = (h + ph) mod sh, + sh, ... while the output row
        // (h + ph - a) / sh exists; the same along the row
        const int a_lo_raw = h + ph - (Ho - 1) * sh, b_lo_raw = c + pw - (Wo - 1) * sw;
        int a0 = (h + ph) % sh, b0 = (c + pw) % sw;
        if (a0 < a_lo_raw) a0 += (a_lo_raw - a0 + sh - 1) / sh * sh;
        if (b0 < b_lo_raw) b0 += (b_lo_raw - b0 + sw - 1) / sw * sw;
        const int a1 = h + ph < kh - 1 ? h + ph : kh - 1, b1 = c + pw < kw - 1 ? c + pw : kw - 1;
        float acc = 0.0f;
        for (int a = a0; a <= a1; a += sh) {
            const int nh = (h + ph - a) / sh;
            for (int b = b0; b <= b1; b += sw) {
                const float *wr = wgt + ((int64_t)ci * kh + a) * kw + b;
                const float *gr = gy + (n * Cout * (int64_t)Ho + nh) * Wo + (c + pw - b) / sw;
                for (int co = 0; co < Cout; ++co) acc += wr[(int64_t)co * Cin * kh * kw] * gr[(int64_t)co * Ho * Wo];
            }
        }
        gx[o] = acc;
    }
}

__global__ __launch_bounds__(kThreads) void conv2d_grad_weight_naive_kernel(
    const float *__restrict__ x, const float *__restrict__ gy, float *__restrict__ gw, int64_t N, int Cin, int H, int W,
    int Cout, int Ho, int Wo, int kh, int kw, int sh, int sw, int ph, int pw)
{
    __shared__ float part[kThreads];
    const int64_t e = blockIdx.x;                    // ((co * Cin + ci) * kh + a) * kw + b
    const int b = (int)(e % kw);
    const int a = (int)((e / kw) % kh);
    const int ci = (int)((e / ((int64_t)kw * kh)) % Cin);
    const int co = (int)(e / ((int64_t)kw * kh * Cin));
    float acc = 0.0f;
    const int64_t cnt = N * (int64_t)Ho * Wo;
    for (int64_t o = threadIdx.x; o < cnt; o += kThreads) {
        const int wo = (int)(o % Wo);
        const int ho = (int)((o / Wo) % Ho);
        const int64_t n = o / ((int64_t)Wo * Ho);
        const int h = ho * sh - ph + a, c = wo * sw - pw + b;
        if (h >= 0 && h < H && c >= 0 && c < W)
            acc += gy[((n * Cout + co) * (int64_t)Ho + ho) * Wo + wo] * x[((n * Cin + ci) * (int64_t)H + h) * W + c];
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int hh = kThreads / 2; hh > 0; hh >>= 1) {
        if ((int)threadIdx.x < hh) part[threadIdx.x] += part[threadIdx.x + hh];
        __syncthreads();
    }
    if (threadIdx.x == 0) gw[e] = part[0];
}

}  // namespace

// Adjoints of sws_conv2d.  With respect to the input at stride 1: the matrix-core kernel on the
// output gradients, weights read through the adjoint view (both tap axes reversed = the flattened
// tap index reversed), padding (kh-1-ph, kw-1-pw).  With respect to the weights at horizontal
// stride 1: the dense kernel above, one kernel row per tap group.
hipError_t launch_conv2d_grad_input(const float *gy, const float *wgt, float *gx, int64_t N, int64_t Cin, int64_t H,
                                    int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh,
                                    int32_t sw, int32_t ph, int32_t pw, hipStream_t s)
{
    if (sh == 1 && sw == 1 && ph <= kh - 1 && pw <= kw - 1 && g_opt.conv2d_variant != 1) {
        bool taken = false;
        const hipError_t e = launch_conv2d_mfma(gy, wgt, gx, N, Cout, Ho, Wo, Cin, H, W, kh, kw, 1, 1, kh - 1 - ph,
                                                kw - 1 - pw, 1, 1, s, &taken, 1);
        if (taken || e != hipSuccess) return e;
    }
    if ((sh > 1 || sw > 1) && N > 0 && g_opt.conv2d_variant != 1) {
        if (kh < sh || kw < sw) {                     // some phases of gx are reached by no tap
            const int64_t n_gx = N * Cin * H * W;
            int64_t fg = (n_gx + kThreads - 1) / kThreads;
            if (fg > 65536) fg = 65536;
            hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)fg), dim3(kThreads), 0, s, gx, n_gx);
        }
        bool taken = false;
        const hipError_t e = launch_conv2d_grad_input_phases(gy, wgt, gx, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, ph,
                                                             pw, s, &taken);
        if (taken || e != hipSuccess) return e;
    }
    int64_t grid = (N * Cin * H * W + kThreads - 1) / kThreads;
    if (grid > 1048576) grid = 1048576;
    hipLaunchKernelGGL(conv2d_grad_input_naive_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, gy, wgt, gx, N,
                       (int)Cin, (int)H, (int)W, (int)Cout, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw);
    return hipGetLastError();
}

hipError_t launch_conv2d_grad_weight(const float *x, const float *gy, float *gw, int64_t N, int64_t Cin, int64_t H,
                                     int64_t W, int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh,
                                     int32_t sw, int32_t ph, int32_t pw, hipStream_t s)
{
    const int64_t n_gw = Cout * Cin * kh * kw;
    if (n_gw > 2147483647LL) return kNotTaken;
    if (N > 0 && sw <= 2 && Cin >= 2 && g_opt.conv2d_variant != 1 && H * W <= 2147483647LL && Ho * Wo <= 2147483647LL) {
        int64_t fg = (n_gw + kThreads - 1) / kThreads;
        if (fg > 4096) fg = 4096;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)fg), dim3(kThreads), 0, s, gw, n_gw);
        {
            bool taken_s = false;
            const hipError_t es = launch_conv2d_gw_split(x, gy, gw, N, Cin, H, W, Cout, Ho, Wo, kh, kw, sh, sw, ph, pw, s, &taken_s);
            if (taken_s || es != hipSuccess) return es;
        }
        if (kh == 1 && sh == 1 && sw == 1 && ph == 0) {
            // kernels one row high: the rows of all images as rows of a 1-D problem; a 1 x 1 kernel does not see the rows
            // either, and the plane is then one long row
            bool taken_s = false;
            const bool flat = kw == 1 && pw == 0;
            const hipError_t es = flat ? launch_conv1d_gw_split(x, gy, gw, N, 1, Cin, H * W, Cout, Ho * Wo, 1, 0, H * W, Ho * Wo, s, &taken_s)
                                       : launch_conv1d_gw_split(x, gy, gw, N * H, (int)H, Cin, W, Cout, Wo, kw, pw, H * W, Ho * Wo, s, &taken_s);
            if (taken_s || es != hipSuccess) return es;
        }
        GwGeom gm;
        gm.Cin = (int)Cin; gm.Cout = (int)Cout; gm.L = (int)W; gm.Lo = (int)Wo; gm.k = kw; gm.pad = pw; gm.dilation = 1;
        gm.H = (int)H; gm.Ho = (int)Ho; gm.kh = kh; gm.sh = sh; gm.ph = ph; gm.sw = sw; gm.x_cs = H * W; gm.gy_cs = Ho * Wo;
        if (kh == 1 && kw == 1 && sh == 1 && sw == 1 && ph == 0 && pw == 0 && H > 1) {
            // a 1 x 1 kernel does not see the rows: the plane may be taken as one long row, if that fills the
            // 64-position slabs better than whole rows (or several short rows packed into one) do
            const int64_t hw = H * W;
            const double flat = (double)hw / (double)((hw + 63) / 64 * 64);
            const double rows = W >= 64 ? (double)W / (double)((W + 63) / 64 * 64) : (double)((64 / W) * W) / 64.0;
            if (flat > rows) { gm.L = gm.Lo = (int)hw; gm.H = gm.Ho = 1; }
        }
        bool taken = false;
        const hipError_t e = launch_dense_gw_taps(x, gy, gw, N, gm, s, &taken);
        if (taken || e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(conv2d_grad_weight_naive_kernel, dim3((unsigned)n_gw), dim3(kThreads), 0, s, x, gy, gw, N,
                       (int)Cin, (int)H, (int)W, (int)Cout, (int)Ho, (int)Wo, kh, kw, sh, sw, ph, pw);
    return hipGetLastError();
}

hipError_t launch_conv1d_grad_input(const float *gy, const float *wgt, float *gx, int64_t B, int64_t Cin, int64_t L,
                                    int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad,
                                    int32_t dilation, int32_t groups, hipStream_t s)
{
    const int64_t back_pad = (int64_t)dilation * (k - 1) - pad;
    if (stride == 1 && back_pad >= 0 && g_opt.conv1d_variant != 1) {
        // the adjoint as a forward call: Cout channels of length Lo in, Cin channels of length L out
        bool taken = false;
        const hipError_t e = launch_conv1d(gy, wgt, gx, B, Cout, Lo, Cin, L, k, 1, (int32_t)back_pad, dilation, groups, s,
                                           1, &taken);
        if (taken || e != hipSuccess) return e;
    }
    if (stride > 1 && dilation == 1 && groups == 1 && Cin >= 2 && B > 0 && g_opt.conv1d_variant != 1) {
        // dense channels: the phases of the strided adjoint on the matrix-core kernel (rows of height 1)
        if (k < stride) {
            const int64_t n_gx = B * Cin * L;
            int64_t fg = (n_gx + kThreads - 1) / kThreads;
            if (fg > 65536) fg = 65536;
            hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)fg), dim3(kThreads), 0, s, gx, n_gx);
        }
        bool taken = false;
        const hipError_t e = launch_conv2d_grad_input_phases(gy, wgt, gx, B, Cin, 1, L, Cout, 1, Lo, 1, k, 1, stride, 0, pad,
                                                             s, &taken);
        if (taken || e != hipSuccess) return e;
    }
    int64_t grid = (B * Cin * L + kThreads - 1) / kThreads;
    if (grid > 1048576) grid = 1048576;
    hipLaunchKernelGGL(conv1d_grad_input_naive_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, gy, wgt, gx, B,
                       (int)Cin, (int)L, (int)Cout, (int)Lo, k, stride, pad, dilation, groups);
    return hipGetLastError();
}

hipError_t launch_conv1d_grad_weight(const float *x, const float *gy, float *gw, int64_t B, int64_t Cin, int64_t L,
                                     int64_t Cout, int64_t Lo, int32_t k, int32_t stride, int32_t pad,
                                     int32_t dilation, int32_t groups, hipStream_t s)
{
    const int cig = (int)(Cin / groups), cog = (int)(Cout / groups);
    const int64_t n_gw = Cout * cig * k;
    const int variant = g_opt.conv1d_variant;        // 1 forces direct evaluation (A/B and tests)
    if (n_gw > 2147483647LL) return kNotTaken;
    const bool thin_ok = B > 0 && cig == 1 && stride == 1 && dilation == 1 && k <= 64 && B <= 2147483647LL && variant != 1;
    const bool dense_ok = B > 0 && groups == 1 && stride <= 2 && Cin >= 2 && variant != 1;
    if (thin_ok || dense_ok) {
        int64_t fg = (n_gw + kThreads - 1) / kThreads;
        if (fg > 4096) fg = 4096;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)fg), dim3(kThreads), 0, s, gw, n_gw);
    }
    if (thin_ok) {
#define SWS_TGW(KB)                                                                                              \
    case KB:                                                                                                     \
        return launch_thin_gw<KB>(x, gy, gw, (int)B, (int)Cin, (int)L, (int)Cout, (int)Lo, k, pad, cog, s)
        switch ((k + 3) / 4) {
            SWS_TGW(1); SWS_TGW(2); SWS_TGW(3); SWS_TGW(4); SWS_TGW(5); SWS_TGW(6); SWS_TGW(7); SWS_TGW(8);
            SWS_TGW(9); SWS_TGW(10); SWS_TGW(11); SWS_TGW(12); SWS_TGW(13); SWS_TGW(14); SWS_TGW(15); SWS_TGW(16);
        default: break;
        }
#undef SWS_TGW
    }
    if (dense_ok && stride == 1 && dilation == 1) {
        bool taken_s = false;
        const hipError_t es = launch_conv1d_gw_split(x, gy, gw, B, 1, Cin, L, Cout, Lo, k, pad, L, Lo, s, &taken_s);
        if (taken_s || es != hipSuccess) return es;
    }
    if (dense_ok) {
        GwGeom gm;
        gm.Cin = (int)Cin; gm.Cout = (int)Cout; gm.L = (int)L; gm.Lo = (int)Lo; gm.k = k; gm.pad = pad; gm.dilation = dilation;
        gm.H = 1; gm.Ho = 1; gm.kh = 1; gm.sh = 1; gm.ph = 0; gm.sw = stride; gm.x_cs = L; gm.gy_cs = Lo;
        bool taken = false;
        const hipError_t e = launch_dense_gw_taps(x, gy, gw, B, gm, s, &taken);
        if (taken || e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(conv1d_grad_weight_naive_kernel, dim3((unsigned)n_gw), dim3(kThreads), 0, s, x, gy, gw, B,
                       (int)Cin, (int)L, (int)Cout, (int)Lo, k, stride, pad, dilation, groups);
    return hipGetLastError();
}

}  // namespace sws
