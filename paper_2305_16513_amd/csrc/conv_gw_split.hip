// The adjoint of the dense 2-D convolution with respect to its weights (the training side of
// Section 2.5's sliding dot product), horizontal stride 1, on the bf16 matrix cores with exactly split
// fp32 operands:
//
//   gw[co][ci][a][b] = sum over (n, ho, wo) of  gy[n][co][ho][wo] * x[n][ci][ho*sh - ph + a][wo - pw + b]
//
// is, for each tap (a, b), a matrix product GY[co][positions] * X_ab[positions][ci] whose contraction
// index — the position — is also the index that is contiguous in memory for both operands.  The
// operand layout of v_mfma_f32_32x32x16_bf16 (a lane holds 8 consecutive contraction indices of one row /
// column) therefore reads straight from memory: a lane loads 8 consecutive gradients of its output
// channel, and the 8 + KW - 1 consecutive inputs of its input channel that those positions meet under
// the KW taps of one kernel row; nothing is staged in LDS and no column matrix is built.  Every fp32
// value is split into three bf16 pieces by truncation (8 + 8 + 8 bits of mantissa; the pieces sum to
// the value exactly) and six of the nine piece products are kept — what is dropped is below 2^-23 of
// the term — so the result has fp32 accuracy at 6/16 of the fp32 matrix instruction's time.
//
// A workgroup owns a 64 x 64 block of (co, ci) — one 32 x 32 block and all KH*KW taps per wavefront,
// 16 accumulator registers per tap — and a contiguous share of the positions, walked in groups of 8 along
// the output rows (the two halves of a wavefront take consecutive groups, which need not lie in the
// same row).  At the end the blocks go through LDS, 16 output channels at a time, and leave as atomic
// adds whose lanes run over contiguous (ci, tap) — adds to one cache line serialise, so as few
// instructions as possible touch each line.  gw is cleared by the caller first; the order of the adds
// is not fixed.
#include "sws_internal.h"

namespace sws {

namespace {

constexpr int kThreads = 256;
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// the upper halves of two floats as one register of two bf16 (lo in the low half)
__device__ __forceinline__ unsigned pack_hi(float lo, float hi)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
// v = p1 + p2 + p3 with every piece's significant bits in the upper half of a float
__device__ __forceinline__ void split3(float v, float &p2, float &p3)
{
    p2 = v - __uint_as_float(__float_as_uint(v) & 0xffff0000u);
    p3 = p2 - __uint_as_float(__float_as_uint(p2) & 0xffff0000u);
}

template <int KH, int KW>
__global__ __launch_bounds__(kThreads) void conv2d_gw_split_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                   float *__restrict__ gw, int Cin, int H, int W, int Cout,
                                                                   int Ho, int Wo, int sh, int ph, int pw, int g8,
                                                                   int64_t n_groups, int64_t groups_per_wg, int ci_blocks,
                                                                   int64_t x_total)
{
    constexpr int T = KH * KW;
    constexpr int NV = 8 + KW - 1;                   // inputs a lane needs per kernel row
    constexpr int NCH = (NV + 3) / 4;                // ... in 128-bit loads
    __shared__ float red[16][64 * T + 1];
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int co_blk = (int)(blockIdx.y / ci_blocks), ci_blk = (int)(blockIdx.y - co_blk * ci_blocks);
    const int co_base = co_blk * 64 + (wave & 1) * 32, ci_base = ci_blk * 64 + (wave >> 1) * 32;
    const bool active = co_base < Cout && ci_base < Cin;         // channel counts are multiples of 32
    const int co = co_base + l32, ci = ci_base + l32;
    v16f acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    const int64_t G0 = blockIdx.x * groups_per_wg;
    const int64_t G1 = G0 + groups_per_wg < n_groups ? G0 + groups_per_wg : n_groups;
    if (active) {
        // my first group of 8 positions: output row (n, ho), group gi of the row; then two groups further per step
        int64_t n;
        int ho, gi;
        {
            const int64_t mg0 = G0 + half, row0 = mg0 / g8;
            gi = (int)(mg0 - row0 * g8);
            n = row0 / Ho;
            ho = (int)(row0 - n * Ho);
        }
        for (int64_t G = G0; G < G1; G += 2) {
            const bool valid = G + half < G1;
            const int64_t nn = valid ? n : 0;                    // a lane without a group points at the first row
            const int hh = valid ? ho : 0;
            const int wo0 = valid ? gi * 8 : 0;
            // ---- gradients: 8 consecutive positions of my output channel
            float ga[8];
            {
                const float *gp = gy + ((nn * Cout + co) * Ho + hh) * (int64_t)Wo + wo0;
                const bool fast = valid && wo0 + 8 <= Wo;
                if (__builtin_amdgcn_ballot_w64(valid && !fast) == 0) {
                    const v4f a0 = *(const v4f_u *)(fast ? gp : gy), a1 = *(const v4f_u *)(fast ? gp + 4 : gy);
                    ga[0] = a0.x; ga[1] = a0.y; ga[2] = a0.z; ga[3] = a0.w; ga[4] = a1.x; ga[5] = a1.y; ga[6] = a1.z; ga[7] = a1.w;
#pragma unroll
                    for (int e = 0; e < 8; ++e) ga[e] = fast ? ga[e] : 0.0f;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const bool ok = valid && wo0 + e < Wo;
                        const float t = gp[ok ? e : 0];
                        ga[e] = ok ? t : 0.0f;
                    }
                }
            }
            unsigned A[3][4];
            {
                float p2[8], p3[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) split3(ga[e], p2[e], p3[e]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    A[0][i] = pack_hi(ga[2 * i], ga[2 * i + 1]);
                    A[1][i] = pack_hi(p2[2 * i], p2[2 * i + 1]);
                    A[2][i] = pack_hi(p3[2 * i], p3[2 * i + 1]);
                }
            }
            const v8bf a1 = __builtin_bit_cast(v8bf, (v4u){A[0][0], A[0][1], A[0][2], A[0][3]});
            const v8bf a2 = __builtin_bit_cast(v8bf, (v4u){A[1][0], A[1][1], A[1][2], A[1][3]});
            const v8bf a3 = __builtin_bit_cast(v8bf, (v4u){A[2][0], A[2][1], A[2][2], A[2][3]});
#pragma unroll
            for (int a = 0; a < KH; ++a) {
                // ---- inputs: positions wo0 - pw .. wo0 - pw + NV - 1 of row ho*sh - ph + a of my input channel
                const int r = hh * sh - ph + a;
                const bool rowok = valid && r >= 0 && r < H;
                const int p0 = wo0 - pw;
                const float *xr = x + ((nn * Cin + ci) * H + (rowok ? r : 0)) * (int64_t)W;
                float xv[4 * NCH];
                // the 128-bit loads may run over the ends of the row (into the neighbouring rows: masked below);
                // only at the two ends of the whole tensor must they not
                const int64_t at = (xr - x) + p0;
                const bool fast = rowok && at >= 0 && at + 4 * NCH <= x_total;
                if (__builtin_amdgcn_ballot_w64(rowok && !fast) == 0) {
#pragma unroll
                    for (int j = 0; j < NCH; ++j) {
                        const v4f q = *(const v4f_u *)(fast ? xr + p0 + 4 * j : x);
                        const float qe[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            xv[4 * j + e] = (fast && p0 + 4 * j + e >= 0 && p0 + 4 * j + e < W) ? qe[e] : 0.0f;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < NV; ++e) {
                        const bool ok = rowok && p0 + e >= 0 && p0 + e < W;
                        const float t = xr[ok ? p0 + e : 0];
                        xv[e] = ok ? t : 0.0f;
                    }
                }
                float q2[NV], q3[NV];
#pragma unroll
                for (int e = 0; e < NV; ++e) split3(xv[e], q2[e], q3[e]);
#pragma unroll
                for (int b = 0; b < KW; ++b) {
                    unsigned Bp[3][4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        Bp[0][i] = pack_hi(xv[b + 2 * i], xv[b + 2 * i + 1]);
                        Bp[1][i] = pack_hi(q2[b + 2 * i], q2[b + 2 * i + 1]);
                        Bp[2][i] = pack_hi(q3[b + 2 * i], q3[b + 2 * i + 1]);
                    }
                    const v8bf b1 = __builtin_bit_cast(v8bf, (v4u){Bp[0][0], Bp[0][1], Bp[0][2], Bp[0][3]});
                    const v8bf b2 = __builtin_bit_cast(v8bf, (v4u){Bp[1][0], Bp[1][1], Bp[1][2], Bp[1][3]});
                    const v8bf b3 = __builtin_bit_cast(v8bf, (v4u){Bp[2][0], Bp[2][1], Bp[2][2], Bp[2][3]});
                    v16f c = acc[a * KW + b];                    // smallest products first
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a3, b1, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b2, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b3, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b1, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b2, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, c, 0, 0, 0);
                    acc[a * KW + b] = c;
                }
            }
            gi += 2;
            while (gi >= g8) {
                gi -= g8;
                if (++ho == Ho) { ho = 0; ++n; }
            }
        }
    }
    // ---- out: register v of lane (l32, half) of tap t is gw[co_base + 8*(v/4) + 4*half + v%4][ci_base + l32][t];
    //      16 output channels at a time through LDS, then atomic adds over contiguous (ci, tap)
    const int co0 = co_blk * 64, ci0 = ci_blk * 64;
    const int ci_n = Cin - ci0 < 64 ? Cin - ci0 : 64;            // input channels of this block (32 or 64)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        __syncthreads();
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if ((wave & 1) * 2 + g / 2 != q) continue;           // rows 8g .. 8g+7 of my block lie in quarter (wave&1)*2 + g/2
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int rl = 8 * (g & 1) + 4 * half + u;       // row inside the quarter
#pragma unroll
                for (int t = 0; t < T; ++t) red[rl][((wave >> 1) * 32 + l32) * T + t] = acc[t][4 * g + u];
            }
        }
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * ci_n * T; e += kThreads) {
            const int rl = e / (ci_n * T), in = e - rl * (ci_n * T);
            const int c = co0 + 16 * q + rl;
            if (c < Cout) atomicAdd(gw + ((int64_t)c * Cin + ci0) * T + in, red[rl][in]);
        }
    }
}

}  // namespace

// *taken = false: not this kernel's case (nothing launched).  gw must hold zeros.
hipError_t launch_conv2d_gw_split(const float *x, const float *gy, float *gw, int64_t N, int64_t Cin, int64_t H, int64_t W,
                                  int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                                  int32_t ph, int32_t pw, hipStream_t s, bool *taken)
{
    *taken = false;
    if (sw != 1 || kh != 3 || kw != 3 || (Cin & 31) || (Cout & 31) || N < 1) return hipSuccess;
    if (g_opt.conv2d_variant != 0 || Cin > 32768 || Cout > 32768) return hipSuccess;
    if (N * Cout * Ho * Wo < 8 || N * Cin * H * W < 12) return hipSuccess;      // the masked lanes' dummy loads
    const int g8 = (int)((Wo + 7) / 8);
    const int64_t n_groups = N * Ho * g8;
    const int co_blocks = (int)((Cout + 63) / 64), ci_blocks = (int)((Cin + 63) / 64);
    // Split of the positions over workgroups: enough to fill the GPU once, no more — every workgroup ends
    // with atomic adds of its whole block.
    int64_t split = (int64_t)device_cus() / ((int64_t)co_blocks * ci_blocks);
    if (split < 1) split = 1;
    int64_t per = (n_groups + split - 1) / split;
    per = (per + 1) / 2 * 2;                             // whole pairs of groups
    split = (n_groups + per - 1) / per;
    if (split > 2147483647LL || (int64_t)co_blocks * ci_blocks > 65535) return hipSuccess;
    *taken = true;
    hipLaunchKernelGGL((conv2d_gw_split_kernel<3, 3>), dim3((unsigned)split, (unsigned)(co_blocks * ci_blocks)), dim3(kThreads),
                       0, s, x, gy, gw, (int)Cin, (int)H, (int)W, (int)Cout, (int)Ho, (int)Wo, sh, ph, pw, g8, n_groups, per,
                       ci_blocks, N * Cin * H * W);
    return hipGetLastError();
}

}  // namespace sws
