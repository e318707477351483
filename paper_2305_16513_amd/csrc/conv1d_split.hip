// Dense 1-D convolution (Section 2.5: y[co][i] = sum over ci and taps of w[co][ci][t] * x[ci][i + t - pad]) for
// layers of a few dozen channels, on the bf16 matrix cores with exactly split fp32 operands.
//
// Per tap the layer is a matrix product W_t[co][ci] * X[ci][i + t]; v_mfma_f32_32x32x16_bf16 contracts 16 input
// channels at a time.  The weights are the stationary operand: a workgroup splits the W_t of its 64 output
// channels once into three bf16 pieces each (truncation: 8 + 8 + 8 bits of mantissa, the pieces sum to the value)
// and lays them out in LDS exactly as the matrix instruction reads them, 16 bytes per lane and piece.  The input is
// the streaming operand and is never staged: a lane owns one output position and eight input channels, so its
// operand is eight loads of one element each, coalesced across the 32 lanes of a half-wavefront; all loads of a
// tile of 32 positions are issued up front and converted (split, packed with v_perm) as they arrive.  Six of the
// nine piece products are kept — what is dropped is below 2^-23 of a term — so the result has fp32 accuracy at
// 6/16 of the fp32 matrix instruction's time.  Output registers hold one output channel and 32 consecutive
// positions: stores are 128-byte runs.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 512;                        // eight wavefronts share one set of split weights
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned pack_hi(float lo, float hi)     // the upper halves of two floats: two bf16
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
__device__ __forceinline__ void split3(float v, float &p2, float &p3)   // v = upper(v) + upper(p2) + upper(p3) ...
{
    p2 = v - __uint_as_float(__float_as_uint(v) & 0xffff0000u);
    p3 = p2 - __uint_as_float(__float_as_uint(p2) & 0xffff0000u);
}
// eight values -> three operands of eight bf16
__device__ __forceinline__ void pieces(const float (&v)[8], v4u (&out)[3])
{
    float p2[8], p3[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) split3(v[e], p2[e], p3[e]);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[0][i] = pack_hi(v[2 * i], v[2 * i + 1]);
        out[1][i] = pack_hi(p2[2 * i], p2[2 * i + 1]);
        out[2][i] = pack_hi(p3[2 * i], p3[2 * i + 1]);
    }
}

// NC chunks of 16 input channels, K taps; a workgroup: 64 output channels (two blocks of 32), its wavefronts
// on tiles of 32 positions.
template <int NC, int K>
__global__ __launch_bounds__(kThreads) void conv1d_split_kernel(const float *__restrict__ x, const float *__restrict__ wgt,
                                                                float *__restrict__ y, int L, int Cout, int Lo, int pad,
                                                                int tiles_per_row, int64_t n_tiles)
{
    constexpr int Cin = 16 * NC;
    extern __shared__ __attribute__((aligned(16))) v4u wl[];    // [operand][piece][lane]
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int co0 = blockIdx.y * 64;
    // ---- the weights of my 64 output channels (one contiguous range of the weight array), split and laid out as
    //      operands (A[i = co][k = ci]: lane i + 32 (k / 8), element k % 8): a thread takes two neighbouring input
    //      channels of one tap at a time, so that every LDS store is a whole register of two bf16
    {
        unsigned *w32 = (unsigned *)wl;
        const float *wb = wgt + (int64_t)co0 * Cin * K;
        const int n_mine = (Cout - co0 < 64 ? Cout - co0 : 64) * Cin * K;
        constexpr int PK = (Cin / 2) * K;            // pairs per output channel
        for (int pidx = threadIdx.x; pidx < 64 * PK; pidx += kThreads) {
            const int col = pidx / PK, rem = pidx - col * PK, cp = rem / K, t = rem - cp * K;
            const int idx = (col * Cin + 2 * cp) * K + t;
            const float v0 = idx < n_mine ? wb[idx] : 0.0f, v1 = idx < n_mine ? wb[idx + K] : 0.0f;
            float a2, a3, b2, b3;
            split3(v0, a2, a3);
            split3(v1, b2, b3);
            const int ci = 2 * cp;
            const int o = ((col >> 5) * NC + (ci >> 4)) * K + t, ln = (col & 31) + 32 * ((ci & 15) >> 3);
            unsigned *dst = w32 + ((o * 3) * 64 + ln) * 4 + ((ci & 7) >> 1);
            dst[0] = pack_hi(v0, v1);
            dst[64 * 4] = pack_hi(a2, b2);
            dst[2 * 64 * 4] = pack_hi(a3, b3);
        }
    }
    __syncthreads();
    // ---- tiles of 32 positions of one row (image), all Cin input channels
    const int64_t stride = (int64_t)gridDim.x * (kThreads / kWave);
    for (int64_t tile = (int64_t)blockIdx.x * (kThreads / kWave) + wave; tile < n_tiles; tile += stride) {
        const int64_t b = tile / tiles_per_row;
        const int pos0 = (int)(tile - b * tiles_per_row) * 32;
        const float *xb = x + b * Cin * (int64_t)L;
        // all loads of the tile: xr[c][t][e] = x[16c + 8 half + e][pos0 + l32 + t - pad]; out-of-row positions are
        // read from a clamped address and zeroed at conversion time (nothing waits here)
        float xr[NC][K][8];
        bool ok[K];
#pragma unroll
        for (int t = 0; t < K; ++t) {
            const int p = pos0 + l32 + t - pad;
            ok[t] = p >= 0 && p < L;
            const float *xp = xb + (int64_t)(8 * half) * L + (ok[t] ? p : 0);
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int e = 0; e < 8; ++e) xr[c][t][e] = xp[(int64_t)(16 * c + e) * L];
        }
        v16f acc[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[cb][v] = 0.0f;
        // the weight operands are read from LDS where they are used; an index the compiler cannot see through keeps it
        // from hoisting all of them (288 registers) out of the loop over tiles
        int wlane = lane;
        asm volatile("" : "+v"(wlane));
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int t = 0; t < K; ++t) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = ok[t] ? xr[c][t][e] : 0.0f;
                v4u pc[3];
                pieces(v, pc);
                const v8bf b1 = __builtin_bit_cast(v8bf, pc[0]), b2 = __builtin_bit_cast(v8bf, pc[1]),
                           b3 = __builtin_bit_cast(v8bf, pc[2]);
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    const int o = (cb * NC + c) * K + t;
                    const v8bf a1 = __builtin_bit_cast(v8bf, wl[(o * 3 + 0) * 64 + wlane]);
                    const v8bf a2 = __builtin_bit_cast(v8bf, wl[(o * 3 + 1) * 64 + wlane]);
                    const v8bf a3 = __builtin_bit_cast(v8bf, wl[(o * 3 + 2) * 64 + wlane]);
                    v16f d = acc[cb];                            // smallest products first
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a3, b1, d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b2, d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b3, d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b1, d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b2, d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, d, 0, 0, 0);
                    acc[cb] = d;
                }
            }
        // ---- register v of lane (l32, half) of block cb: output channel co0 + 32 cb + 8 (v / 4) + 4 half + v % 4, position pos0 + l32
        const int pos = pos0 + l32;
        if (pos < Lo) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int co = co0 + 32 * cb + 8 * (v / 4) + 4 * half + (v % 4);
                    if (co < Cout) __builtin_nontemporal_store(acc[cb][v], y + (b * Cout + co) * (int64_t)Lo + pos);
                }
        }
    }
}

template <int NC, int K>
hipError_t launch_split(const float *x, const float *wgt, float *y, int64_t B, int L, int Cout, int Lo, int pad,
                        hipStream_t s)
{
    const int tiles_per_row = (Lo + 31) / 32;
    const int64_t n_tiles = B * tiles_per_row;
    const int co_blocks = (Cout + 63) / 64;
    const size_t lds = (size_t)2 * NC * K * 3 * 64 * 16;
    // one tile per wavefront while one workgroup per CU (eight wavefronts, two per SIMD) holds them all: the chain of
    // a wavefront — split the weights, load a tile, convert and multiply — is what the kernel's time is made of
    int64_t wgs = (n_tiles + 7) / 8;
    if (g_opt.slide_group > 0) wgs = (n_tiles + g_opt.slide_group - 1) / g_opt.slide_group;   // A/B: tiles per workgroup
    const int64_t cap = (int64_t)device_cus() / co_blocks > 0 ? (int64_t)device_cus() / co_blocks : 1;
    if (wgs > cap) wgs = cap;
    if (wgs < 1) wgs = 1;
    static std::atomic<int> raised{0};
    if (lds > 64 * 1024 && !raised.load(std::memory_order_relaxed)) {
        const hipError_t e = hipFuncSetAttribute((const void *)conv1d_split_kernel<NC, K>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        raised.store(1, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL((conv1d_split_kernel<NC, K>), dim3((unsigned)wgs, (unsigned)co_blocks), dim3(kThreads), lds, s, x, wgt, y,
                       L, Cout, Lo, pad, tiles_per_row, n_tiles);
    return hipGetLastError();
}

}  // namespace

// Dense channels, stride 1, adjacent taps; *taken = false: not one of the shapes this kernel is built for.
hipError_t launch_conv1d_split(const float *x, const float *wgt, float *y, int64_t B, int64_t Cin, int64_t L, int64_t Cout,
                               int64_t Lo, int32_t k, int32_t pad, hipStream_t s, bool *taken)
{
    *taken = false;
    if ((Cout & 31) || Cout > 32768 || B < 1 || L < 1) return hipSuccess;
    *taken = true;
    if (Cin == 64 && k == 3) return launch_split<4, 3>(x, wgt, y, B, (int)L, (int)Cout, (int)Lo, pad, s);
    if (Cin == 32 && k == 3) return launch_split<2, 3>(x, wgt, y, B, (int)L, (int)Cout, (int)Lo, pad, s);
    if (Cin == 64 && k == 1) return launch_split<4, 1>(x, wgt, y, B, (int)L, (int)Cout, (int)Lo, pad, s);
    if (Cin == 32 && k == 5) return launch_split<2, 5>(x, wgt, y, B, (int)L, (int)Cout, (int)Lo, pad, s);
    *taken = false;
    return hipSuccess;
}

}  // namespace sws
