// The adjoint of the dense 2-D convolution with respect to its weights (the training side of
// Section 2.5's sliding dot product), horizontal stride 1, on the bf16 matrix cores with exactly split
// fp32 operands (3 x 3, stride s = 1 or 2 on both axes):
//
//   gw[co][ci][a][b] = sum over (n, ho, wo) of  gy[n][co][ho][wo] * x[n][ci][s*ho - ph + a][s*wo - pw + b]
//
// is, for each tap (a, b), a matrix product GY[co][positions] * X_ab[positions][ci] whose contraction
// index — the position — is also the index that is contiguous in memory for both operands.  The
// operand layout of v_mfma_f32_32x32x16_bf16 (a lane holds 8 consecutive contraction indices of one row /
// column) therefore reads straight from memory: a lane loads 8 consecutive gradients of its output
// channel, and the 7s + KW consecutive inputs of its input channel that those positions meet under
// the KW taps of one kernel row (every s-th of them per tap); nothing is staged in LDS and no column matrix is built.  Every fp32
// value is split into three bf16 pieces by truncation (8 + 8 + 8 bits of mantissa; the pieces sum to
// the value exactly) and six of the nine piece products are kept — what is dropped is below 2^-23 of
// the term — so the result has fp32 accuracy at 6/16 of the fp32 matrix instruction's time.
//
// A workgroup owns a 64 x 64 block of (co, ci) — one 32 x 32 block and all KH*KW taps per wavefront,
// 16 accumulator registers per tap — and a share of the positions, cut into tasks of a column of 8
// positions by S output rows (the two halves of a wavefront take two tasks).  Walking down a column, a step
// converts (splits, packs) the s new input rows and keeps what it shares with the step before; that
// conversion runs in the shadow of the matrix instructions, and loads run two steps ahead of it.  At the end the blocks go through LDS, 16 output channels at a time, and leave as atomic
// adds whose lanes run over contiguous (ci, tap) — adds to one cache line serialise, so as few
// instructions as possible touch each line.  gw is cleared by the caller first; the order of the adds
// is not fixed.
#include "sws_internal.h"

#include <atomic>

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

// One kernel row's inputs of a lane as matrix operands: for each of the KW taps the 8 positions it meets,
// in three bf16 pieces.
template <int KW> struct RowOperand {
    v8bf b[KW][3];
};

template <int KH, int KW, int PW, int ST, bool DYN>
__global__ __launch_bounds__(kThreads) void conv2d_gw_split_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                   float *__restrict__ gw, int Cin, int H, int W, int Cout,
                                                                   int Ho, int Wo, int ph, int g8, int S, int nseg,
                                                                   int64_t n_tasks, int64_t pairs_per_wg, int ci_blocks,
                                                                   int64_t x_total, int64_t gy_total)
{
    static_assert(KH == 3 && (ST == 1 || ST == 2), "the ring of kernel rows below is written for three rows, strides 1 and 2");
    constexpr int T = KH * KW;
    constexpr int NV = 7 * ST + KW;                  // inputs a lane needs per kernel row: 8 windows ST apart
    // W and Wo are multiples of 4 and a column starts at a multiple of 8, so the first input a lane needs sits
    // D elements into a 16-byte group of the tensor: loads of whole groups never straddle an end of the tensor
    // (DYN: rows of any length — every element is then loaded on its own, from an offset clamped into the lane's
    // plane)
    constexpr int D = DYN ? 0 : (4 - PW % 4) % 4;
    constexpr int NCH = (D + NV + 3) / 4;            // groups per kernel row
    constexpr int NGG = 2;                           // groups per 8 gradients
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

    // A task: S consecutive output rows of one column of 8 positions of one image.  Walking down the column,
    // the input rows of consecutive steps overlap: a step converts one new input row and keeps two.
    const int64_t P0 = blockIdx.x * pairs_per_wg;
    const int64_t P1 = P0 + pairs_per_wg < (n_tasks + 1) / 2 ? P0 + pairs_per_wg : (n_tasks + 1) / 2;
    if (active) {
        for (int64_t P = P0; P < P1; ++P) {
            const int64_t task = 2 * P + half;
            const bool tv = task < n_tasks;
            const int64_t col = tv ? task / nseg : 0;
            const int seg = tv ? (int)(task - col * nseg) : 0;
            const int64_t n = col / g8;
            const int wo0 = (int)(col - n * g8) * 8, h0 = seg * S;
            const float *xp = x + (n * Cin + ci) * (int64_t)H * W;       // my input plane
            const float *gp = gy + (n * Cout + co) * (int64_t)Ho * Wo;   // my gradient plane
            const int p0 = ST * wo0 - PW;
            const int64_t x_groups = x_total >> 2, gy_groups = gy_total >> 2;
            // the groups that hold positions p0 .. p0 + NV - 1 of input row r, as loaded (no branches, nothing
            // waits here): groups beyond an end of the tensor are taken from its first / last group, and every
            // cell outside the plane is zeroed at conversion time (position < wlim)
            auto load_row = [&](int r, float (&xv)[4 * NCH], unsigned &wlim, unsigned &dsel) {
                const bool rowok = tv && r >= 0 && r < H;
                wlim = rowok ? (unsigned)W : 0u;
                dsel = 0;
                if constexpr (DYN) {
                    const int o0 = (rowok ? r : 0) * W + p0, last = H * W - 1;
#pragma unroll
                    for (int e = 0; e < NV; ++e) {
                        const int o = o0 + e;
                        xv[e] = xp[o < 0 ? 0 : (o > last ? last : o)];
                    }
                } else {
                    const int64_t g0 = ((xp - x) + (int64_t)(rowok ? r : 0) * W + (p0 - D)) >> 2;    // may be -1
#pragma unroll
                    for (int j = 0; j < NCH; ++j) {
                        int64_t g = g0 + j;
                        g = g < 0 ? 0 : (g >= x_groups ? x_groups - 1 : g);
                        // only what is used is loaded: a register of a load still in flight that nothing reads would
                        // be handed out again, and writing it waits for the load
                        if (4 * j >= D && 4 * j + 4 <= D + NV) {
                            const v4f q = *(const v4f_u *)(x + 4 * g);
                            xv[4 * j] = q.x; xv[4 * j + 1] = q.y; xv[4 * j + 2] = q.z; xv[4 * j + 3] = q.w;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (4 * j + e >= D && 4 * j + e < D + NV) xv[4 * j + e] = x[4 * g + e];
                        }
                    }
                }
            };
            auto convert_row = [&](const float (&raw)[4 * NCH], unsigned wlim, unsigned dsel, RowOperand<KW> &R) {
                float xv[NV], q2[NV], q3[NV];
                (void)dsel;
#pragma unroll
                for (int e = 0; e < NV; ++e) xv[e] = raw[D + e];
#pragma unroll
                for (int e = 0; e < NV; ++e) {
                    xv[e] = (unsigned)(p0 + e) < wlim ? xv[e] : 0.0f;
                    split3(xv[e], q2[e], q3[e]);
                }
#pragma unroll
                for (int b = 0; b < KW; ++b) {
                    unsigned Bp[3][4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        Bp[0][i] = pack_hi(xv[b + ST * 2 * i], xv[b + ST * (2 * i + 1)]);
                        Bp[1][i] = pack_hi(q2[b + ST * 2 * i], q2[b + ST * (2 * i + 1)]);
                        Bp[2][i] = pack_hi(q3[b + ST * 2 * i], q3[b + ST * (2 * i + 1)]);
                    }
#pragma unroll
                    for (int pc = 0; pc < 3; ++pc)
                        R.b[b][pc] = __builtin_bit_cast(v8bf, (v4u){Bp[pc][0], Bp[pc][1], Bp[pc][2], Bp[pc][3]});
                }
            };
            // 8 consecutive gradients of output row ho, as loaded; glim = how many of them count (none beyond the
            // segment or the plane)
            auto load_grad = [&](int ho, int i, float (&ga)[4 * NGG], unsigned &glim) {
                const bool ok_row = tv && i < S && ho < Ho;
                glim = ok_row ? (unsigned)(Wo - wo0) : 0u;
                if constexpr (DYN) {
                    const int o0 = (ok_row ? ho : 0) * Wo + wo0, last = Ho * Wo - 1;
#pragma unroll
                    for (int e = 0; e < 8; ++e) ga[e] = gp[o0 + e > last ? last : o0 + e];
                } else {
                    const int64_t g0 = ((gp - gy) + (int64_t)(ok_row ? ho : 0) * Wo + wo0) >> 2;
#pragma unroll
                    for (int j = 0; j < NGG; ++j) {
                        const int64_t g = g0 + j < gy_groups ? g0 + j : gy_groups - 1;
                        const v4f q = *(const v4f_u *)(gy + 4 * g);
                        ga[4 * j] = q.x; ga[4 * j + 1] = q.y; ga[4 * j + 2] = q.z; ga[4 * j + 3] = q.w;
                    }
                }
            };
            struct GradOperand { v8bf a[3]; };
            auto convert_grad = [&](const float (&raw)[4 * NGG], unsigned gl_, GradOperand &A) {
                float ga[8], p2[8], p3[8];
                const unsigned glim = gl_;
#pragma unroll
                for (int e = 0; e < 8; ++e) ga[e] = raw[e];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    ga[e] = (unsigned)e < glim ? ga[e] : 0.0f;
                    split3(ga[e], p2[e], p3[e]);
                }
                unsigned w[3][4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    w[0][k] = pack_hi(ga[2 * k], ga[2 * k + 1]);
                    w[1][k] = pack_hi(p2[2 * k], p2[2 * k + 1]);
                    w[2][k] = pack_hi(p3[2 * k], p3[2 * k + 1]);
                }
#pragma unroll
                for (int pc = 0; pc < 3; ++pc) A.a[pc] = __builtin_bit_cast(v8bf, (v4u){w[pc][0], w[pc][1], w[pc][2], w[pc][3]});
            };
            // Step i (output row h0 + i) meets input rows r0 + ST*i + a, r0 = ST*h0 - ph, kept in ring[(ST*i + a) % 3].
            // Its matrix instructions for the kernel rows whose ring slots the next step does not need (the first ST
            // of them) go first; those slots then take the next step's new rows, which are converted — with the
            // next step's gradients — in the shadow of the remaining matrix instructions.  Loads run two steps
            // ahead of their conversion.
            const int r0 = ST * h0 - ph;
            RowOperand<KW> ring[KH];
            GradOperand A;
            constexpr int NB = 2;                                // steps the loads run ahead
            float nx[NB][ST][4 * NCH], ng[NB][4 * NGG];
            unsigned wl[NB][ST], dl[NB][ST], gl[NB];
            // rows r0 + 0, 1, 2 (step 0), then the new rows of steps 1 and 2 into the two buffers
#pragma unroll
            for (int a = 0; a < KH; ++a) {
                load_row(r0 + a, nx[0][0], wl[0][0], dl[0][0]);
                convert_row(nx[0][0], wl[0][0], dl[0][0], ring[a]);
            }
            load_grad(h0, 0, ng[0], gl[0]);
            convert_grad(ng[0], gl[0], A);
#pragma unroll
            for (int k = 1; k <= NB; ++k) {                      // the new rows and gradients of steps 1 .. NB
#pragma unroll
                for (int u = 0; u < ST; ++u) load_row(r0 + k * ST + KH - ST + u, nx[k % NB][u], wl[k % NB][u], dl[k % NB][u]);
                load_grad(h0 + k, k, ng[k % NB], gl[k % NB]);
            }
            auto taps_of_row = [&](int a, const RowOperand<KW> &R) {
#pragma unroll
                for (int b = 0; b < KW; ++b) {
                    v16f c = acc[a * KW + b];                    // smallest products first
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.a[2], R.b[b][0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.a[1], R.b[b][1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.a[0], R.b[b][2], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.a[1], R.b[b][0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.a[0], R.b[b][1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.a[0], R.b[b][0], c, 0, 0, 0);
                    acc[a * KW + b] = c;
                }
            };
            for (int i6 = 0; i6 < S; i6 += 6) {
#pragma unroll
                for (int j6 = 0; j6 < 6; ++j6) {
                    const int i = i6 + j6;
                    if (i >= S) break;                           // S need not be a whole number of rounds
                    const int bsel = (j6 + 1) % NB;              // what step i + 1 needs, loaded NB steps ago
#pragma unroll
                    for (int a = 0; a < ST; ++a) taps_of_row(a, ring[(ST * j6 + a) % 3]);
                    GradOperand An;
#pragma unroll
                    for (int u = 0; u < ST; ++u)                 // step i + 1's kernel row KH - ST + u: the slot of my row u
                        convert_row(nx[bsel][u], wl[bsel][u], dl[bsel][u], ring[(ST * j6 + u) % 3]);
                    convert_grad(ng[bsel], gl[bsel], An);
#pragma unroll
                    for (int u = 0; u < ST; ++u) load_row(r0 + ST * (i + 1 + NB) + KH - ST + u, nx[bsel][u], wl[bsel][u], dl[bsel][u]);   // step i + 1 + NB's
                    load_grad(h0 + i + 1 + NB, i + 1 + NB, ng[bsel], gl[bsel]);
#pragma unroll
                    for (int a = ST; a < KH; ++a) taps_of_row(a, ring[(ST * j6 + a) % 3]);
                    A = An;
                    // the order asked of the scheduler: a few vector instructions after every matrix instruction,
                    // so that the conversions hide behind the matrix pipe instead of running in a block of their own
#pragma unroll
                    for (int k = 0; k < 6 * T; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, ST == 1 ? 6 : 8, 0);
                    }
                }
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
        // all reads of a thread first, then its adds back to back: one read, one add at a time would pay the
        // LDS latency 36 times over
        constexpr int NE = 16 * 64 * T / kThreads;
        static_assert(16 * 64 * T % kThreads == 0, "whole rounds of the workgroup");
        float val[NE];
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int e = k * kThreads + threadIdx.x, rl = e / (64 * T);
            val[k] = red[rl][e - rl * (64 * T)];
        }
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int e = k * kThreads + threadIdx.x, rl = e / (64 * T), in = e - rl * (64 * T);
            const int c = co0 + 16 * q + rl;
            if (c < Cout && in < ci_n * T) atomicAdd(gw + ((int64_t)c * Cin + ci0) * T + in, val[k]);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Kernels one row high (1 x KW: the 1-D convolution, and 1 x 1 layers with a plane taken as one long row).
// The products run over positions, so a matrix operand is 8 consecutive positions of one channel — across a
// wavefront that is 32 different rows of memory.  The workgroup therefore stages a chunk of 64 output positions
// through LDS: every thread loads pairs of neighbouring positions along the rows (coalesced), splits them once
// into three bf16 pieces and stores each pair as one register into a [piece][channel][pair] array whose rows are
// 36 registers long (144 bytes: 128-bit reads of 16 consecutive channels fall into different banks).  The eight
// wavefronts (32 output x 32 input channels x one half of the chunk's positions each; two per SIMD, so that one's
// waits pass behind the other's work) then read their operands from there: 8 positions are four registers, and
// a tap at an odd offset takes the halves of neighbouring registers (one byte permute each).  Two staging buffers
// and two sets of load registers: while the matrix instructions of chunk c run, chunk c + 1 is split into the
// other buffer and the loads of chunk c + 3 go out.
//   rows: row r of x starts at x + (r / RH * Cin + ci) * x_cs + (r % RH) * L, of gy likewise with Cout, gy_cs,
//   Lo (RH = rows per image: 1 for the 1-D convolution, H for 1 x KW kernels on planes).
// ------------------------------------------------------------------------------------------------
constexpr int kRowThreads = 512;                                 // eight wavefronts: (output half, input half, half of a chunk's positions)
constexpr int kRowPairs = 36;                                    // registers per staged row: 72 positions >= 64 + KW - 1
constexpr int kXRows = 72;                                       // staged rows of x: 64 channels, and 8 that only round the
                                                                 // workgroup's share of pairs up to five per thread
constexpr int kXPiece = kXRows * kRowPairs, kGPiece = 64 * kRowPairs;    // registers per bf16 piece
constexpr int kStage = 3 * (kXPiece + kGPiece);                  // registers per staging buffer (x, then gy)
constexpr int kRowLds = 2 * kStage * 4;                          // bytes: two buffers

// One phase of the row kernel's loop: the matrix products of the chunk staged in (xc, gc), and the splitting of the
// loaded chunk (vx, vg; first output position p0) into the other buffer (xn, gn).  The splitting is written out in
// slices between the groups of six matrix instructions (one group per tap and 16 positions), so that the vector
// unit works on the next chunk while the matrix unit works on this one; issue_loads() refills (vx, vg) and is called
// once they are split, a few groups before the end.  SH: the staged row starts one position early (an even
// position: pairs loaded as one 64-bit access, PAIR); NA sets of accumulators take turns, so that a matrix
// instruction seldom waits for the one before it.
template <int KW, int SH, bool PAIR, int NA, int NX, int NG, class Loads>
__device__ __forceinline__ void row_phase(const unsigned *__restrict__ xc, const unsigned *__restrict__ gc,
                                          unsigned *__restrict__ xn, unsigned *__restrict__ gn, v16f (&acc)[NA][KW],
                                          const float (&vx)[NX][2], const float (&vg)[NG][2], int p0, int pad, int L, int Lo,
                                          const int (&xpr)[NX], int gpr, int tid, int wave, int l32, int half, Loads &&issue_loads)
{
    constexpr int ND = (KW + SH + 6) / 2 + 1;                    // registers that hold positions 0 .. KW + SH + 6 of a run
    constexpr int G = 2 * KW;                                    // groups of matrix instructions (my half of the chunk)
    constexpr int GS = G - (KW == 1 ? 1 : 2);                    // the splitting is spread over the first GS of them
    const int kh = wave >> 2;                                    // my half of the chunk's positions
    const unsigned *ga = gc + ((wave & 1) * 32 + l32) * kRowPairs + 4 * half + 16 * kh;
    const unsigned *xa = xc + (((wave >> 1) & 1) * 32 + l32) * kRowPairs + 4 * half + 16 * kh;
    // positions outside the row count as zero
    auto stage_pair = [&](int q) {
        if (q < NX) {
            const int j = q;
            const int o = p0 - pad - SH + 2 * xpr[j];
            const bool in0 = (unsigned)o < (unsigned)L, in1 = PAIR ? in0 : (unsigned)(o + 1) < (unsigned)L;
            const float v0 = in0 ? vx[j][0] : 0.0f, v1 = in1 ? vx[j][1] : 0.0f;
            float a2, a3, b2, b3;
            split3(v0, a2, a3);
            split3(v1, b2, b3);
            const int at = j * kRowThreads + tid;                 // = row * kRowPairs + pair
            xn[at] = pack_hi(v0, v1);
            xn[kXPiece + at] = pack_hi(a2, b2);
            xn[2 * kXPiece + at] = pack_hi(a3, b3);
        } else {
            const int j = q - NX;
            const int o = p0 + 2 * gpr;
            const bool in0 = o < Lo, in1 = PAIR ? in0 : o + 1 < Lo;
            const float v0 = in0 ? vg[j][0] : 0.0f, v1 = in1 ? vg[j][1] : 0.0f;
            float a2, a3, b2, b3;
            split3(v0, a2, a3);
            split3(v1, b2, b3);
            const int at = (j * (kRowThreads / 32) + (tid >> 5)) * kRowPairs + gpr;
            gn[at] = pack_hi(v0, v1);
            gn[kGPiece + at] = pack_hi(a2, b2);
            gn[2 * kGPiece + at] = pack_hi(a3, b3);
        }
    };
    // operands of 16 positions (8 per half-wavefront): read one step ahead of the matrix instructions that use them,
    // so that the LDS latency passes behind the step before
    v4u A[2][3];
    unsigned d[2][3][ND];
    auto read_operands = [&](int ks, v4u (&Ao)[3], unsigned (&dd)[3][ND]) {
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            Ao[p] = *reinterpret_cast<const v4u *>(ga + p * kGPiece + 8 * ks);
            const unsigned *src = xa + p * kXPiece + 8 * ks;
            const v4u q = *reinterpret_cast<const v4u *>(src);
            dd[p][0] = q[0]; dd[p][1] = q[1]; dd[p][2] = q[2]; dd[p][3] = q[3];
#pragma unroll
            for (int e = 4; e < ND; ++e) dd[p][e] = src[e];
        }
    };
    read_operands(0, A[0], d[0]);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        if (ks < 1) read_operands(ks + 1, A[(ks + 1) & 1], d[(ks + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);                       // the reads above stay above
        const int cur = ks & 1;
        // registers, from here on: keeps the compiler from fetching a shifted run from LDS a second time
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int e = 0; e < ND; ++e) asm volatile("" : "+v"(d[cur][p][e]));
        const v8bf a1 = __builtin_bit_cast(v8bf, A[cur][0]), a2 = __builtin_bit_cast(v8bf, A[cur][1]), a3 = __builtin_bit_cast(v8bf, A[cur][2]);
#pragma unroll
        for (int b = 0; b < KW; ++b) {
            v4u Bp[3];
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    Bp[p][i] = ((b + SH) & 1) ? __builtin_amdgcn_perm(d[cur][p][(b + SH) / 2 + i + 1], d[cur][p][(b + SH) / 2 + i], 0x05040302u)
                                              : d[cur][p][(b + SH) / 2 + i];
            const v8bf b1 = __builtin_bit_cast(v8bf, Bp[0]), b2 = __builtin_bit_cast(v8bf, Bp[1]), b3 = __builtin_bit_cast(v8bf, Bp[2]);
            v16f cc = acc[ks % NA][b];                           // smallest products first
            cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a3, b1, cc, 0, 0, 0);
            cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b2, cc, 0, 0, 0);
            cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b3, cc, 0, 0, 0);
            cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b1, cc, 0, 0, 0);
            cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b2, cc, 0, 0, 0);
            cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, cc, 0, 0, 0);
            acc[ks % NA][b] = cc;
            // this group's slice of the splitting, issued behind its matrix instructions
            const int g = ks * KW + b;
#pragma unroll
            for (int q = 0; q < NX + NG; ++q)
                if (q * GS / (NX + NG) == g) stage_pair(q);
            // the registers are free again: the next loads go out behind the last groups
            if (g == GS - 1) issue_loads();
        }
    }
}

template <int KW, int SH, bool PAIR>
__global__ __launch_bounds__(kRowThreads) void conv1d_gw_split_kernel(const float *__restrict__ x, const float *__restrict__ gy,
                                                                   float *__restrict__ gw, int Cin, int L, int Cout, int Lo,
                                                                   int pad, int RH, int64_t x_cs, int64_t gy_cs, int cpr,
                                                                   int64_t n_chunks, int64_t chunks_per_wg, int ci_blocks)
{
    constexpr int T = KW;
    constexpr int NX = kXPiece / kRowThreads, NG = 64 * 32 / kRowThreads;       // pairs per thread: 5 of x, 4 of gy
    static_assert(kXPiece >= NX * kRowThreads, "every thread's pairs lie inside the staged array");
    constexpr int NA = KW == 5 ? 1 : 2;                          // sets of accumulators
    static_assert(KW + SH + 63 <= 2 * kRowPairs && (KW & 1) && (PAIR || !SH), "a chunk's inputs fit the staged row");
    static_assert(16 * (64 * T + 1) <= 2 * kStage, "the transposition of the results fits the staging buffers");
    extern __shared__ __align__(16) unsigned lds[];              // [buffer][x, gy][piece][channel][pair]
    float (*red)[64 * T + 1] = reinterpret_cast<float (*)[64 * T + 1]>(lds);
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int co_blk = (int)(blockIdx.y / ci_blocks), ci_blk = (int)(blockIdx.y - co_blk * ci_blocks);
    const int co0 = co_blk * 64, ci0 = ci_blk * 64;
    v16f acc[NA][T];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][t][v] = 0.0f;
    // my pairs of the staging: fixed rows and columns for the whole kernel (rows past the last channel are read
    // from the last one: what is computed from them is not written)
    unsigned xrow[NX], grow[NG];                                 // byte offsets of my rows from the block's first channel
    int xpr[NX], gpr;
#pragma unroll
    for (int j = 0; j < NX; ++j) {
        const int idx = j * kRowThreads + tid, r = idx / kRowPairs;
        xpr[j] = idx - r * kRowPairs;
        const int rr = r < 64 ? r : 63;                          // the rounding rows: loaded from a real one, never read
        xrow[j] = (unsigned)(ci0 + rr < Cin ? rr : Cin - 1 - ci0) * (unsigned)x_cs * 4u;
    }
    gpr = tid & 31;
#pragma unroll
    for (int j = 0; j < NG; ++j) {
        const int r = j * (kRowThreads / 32) + (tid >> 5);
        grow[j] = (unsigned)(co0 + r < Cout ? r : Cout - 1 - co0) * (unsigned)gy_cs * 4u;
    }
    const int64_t C0 = blockIdx.x * chunks_per_wg;
    const int64_t C1 = C0 + chunks_per_wg < n_chunks ? C0 + chunks_per_wg : n_chunks;
    // the next chunk to load: (image, row inside the image, chunk inside the row), stepped without divisions
    int64_t img;
    int hr, cr;
    {
        const int64_t r = C0 / cpr;
        cr = (int)(C0 - r * cpr);
        img = r / RH;
        hr = (int)(r - img * RH);
    }
    int64_t c_load = C0;
    int cr_over = 0;
    // two sets of load registers: a chunk is loaded during one phase of the loop and split during the next
    float rx[2][NX][2], rg[2][NG][2];
    int p0r[2] = {0, 0};                                         // first output position of the chunk in a set
    auto load_chunk = [&](float (&vx)[NX][2], float (&vg)[NG][2], int &p0s) {   // every offset clamped into its row: no branch
        const int p0 = cr * 64;
        p0s = (cr + cr_over) * 64;
        const char *xb = reinterpret_cast<const char *>(x + (img * Cin + ci0) * x_cs + (int64_t)hr * L);
        const char *gb = reinterpret_cast<const char *>(gy + (img * Cout + co0) * gy_cs + (int64_t)hr * Lo);
        auto at = [](const char *base, unsigned byte_off) { return *reinterpret_cast<const float *>(base + byte_off); };
        auto at2 = [](const char *base, unsigned byte_off) { return *reinterpret_cast<const float2 *>(base + byte_off); };
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int o = p0 - pad - SH + 2 * xpr[j];
            if constexpr (PAIR) {                                // even position, even row length: both inside or both outside
                const float2 v = at2(xb, xrow[j] + 4u * (unsigned)(o < 0 ? 0 : (o >= L ? L - 2 : o)));
                vx[j][0] = v.x;
                vx[j][1] = v.y;
            } else {
                vx[j][0] = at(xb, xrow[j] + 4u * (unsigned)(o < 0 ? 0 : (o >= L ? L - 1 : o)));
                vx[j][1] = at(xb, xrow[j] + 4u * (unsigned)(o + 1 < 0 ? 0 : (o + 1 >= L ? L - 1 : o + 1)));
            }
        }
#pragma unroll
        for (int j = 0; j < NG; ++j) {
            const int o = p0 + 2 * gpr;
            if constexpr (PAIR) {
                const float2 v = at2(gb, grow[j] + 4u * (unsigned)(o >= Lo ? Lo - 2 : o));
                vg[j][0] = v.x;
                vg[j][1] = v.y;
            } else {
                vg[j][0] = at(gb, grow[j] + 4u * (unsigned)(o >= Lo ? Lo - 1 : o));
                vg[j][1] = at(gb, grow[j] + 4u * (unsigned)(o + 1 >= Lo ? Lo - 1 : o + 1));
            }
        }
        // past the last chunk the last one is loaded again and taken as zeros: every phase issues the same number
        // of loads, so the waits on them can be counted exactly
        if (++c_load < C1) {
            if (++cr == cpr) {
                cr = 0;
                if (++hr == RH) { hr = 0; ++img; }
            }
        } else {
            cr_over = 1 << 23;                                    // splits into zeros: the positions lie outside every row
        }
    };
    // split a loaded chunk (positions outside the row count as zero) into a staging buffer
    auto stage = [&](const float (&vx)[NX][2], const float (&vg)[NG][2], int p0, unsigned *xl, unsigned *gl) {
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int o = p0 - pad - SH + 2 * xpr[j];
            const float v0 = (unsigned)o < (unsigned)L ? vx[j][0] : 0.0f, v1 = (unsigned)(o + 1) < (unsigned)L ? vx[j][1] : 0.0f;
            float a2, a3, b2, b3;
            split3(v0, a2, a3);
            split3(v1, b2, b3);
            const int at = j * kRowThreads + tid;                 // = row * kRowPairs + pair
            xl[at] = pack_hi(v0, v1);
            xl[kXPiece + at] = pack_hi(a2, b2);
            xl[2 * kXPiece + at] = pack_hi(a3, b3);
        }
#pragma unroll
        for (int j = 0; j < NG; ++j) {
            const int o = p0 + 2 * gpr;
            const float v0 = o < Lo ? vg[j][0] : 0.0f, v1 = o + 1 < Lo ? vg[j][1] : 0.0f;
            float a2, a3, b2, b3;
            split3(v0, a2, a3);
            split3(v1, b2, b3);
            const int at = (j * (kRowThreads / 32) + (tid >> 5)) * kRowPairs + gpr;
            gl[at] = pack_hi(v0, v1);
            gl[kGPiece + at] = pack_hi(a2, b2);
            gl[2 * kGPiece + at] = pack_hi(a3, b3);
        }
    };
    unsigned *const xl0 = lds, *const gl0 = lds + 3 * kXPiece, *const xl1 = lds + kStage, *const gl1 = lds + kStage + 3 * kXPiece;
    // A phase of the loop: the products of one chunk out of its buffer with the splitting of the next chunk into the
    // other buffer in between, then the loads of the chunk after that into the registers just emptied.
#define SWS_ROW_PHASE(XC_, GC_, XN_, GN_, SET_)                                                                  \
    {                                                                                                             \
        const int p0_ = p0r[SET_];                                                                                \
        row_phase<KW, SH, PAIR, NA, NX, NG>(XC_, GC_, XN_, GN_, acc, rx[SET_], rg[SET_], p0_, pad, L, Lo, xpr, gpr, tid, wave, l32, half, \
                              [&]() { load_chunk(rx[SET_], rg[SET_], p0r[SET_]); });                              \
    }                                                                                                             \
    __syncthreads()
    load_chunk(rx[0], rg[0], p0r[0]);
    load_chunk(rx[1], rg[1], p0r[1]);
    stage(rx[0], rg[0], p0r[0], xl0, gl0);
    load_chunk(rx[0], rg[0], p0r[0]);
    __syncthreads();
    // phases in pairs (one straight loop body, so that the compiler can count the loads in flight): a workgroup with
    // an odd number of chunks runs its last phase on a buffer of zeros
    for (int64_t c = C0; c < C1; c += 2) {
        SWS_ROW_PHASE(xl0, gl0, xl1, gl1, 1);                    // chunk c; stages c + 1 (set 1), then loads c + 3 into it
        SWS_ROW_PHASE(xl1, gl1, xl0, gl0, 0);                    // chunk c + 1; stages c + 2 (set 0), then loads c + 4
    }
#undef SWS_ROW_PHASE
    // ---- out: a quarter of the block's rows at a time through LDS, so that consecutive lanes add to consecutive
    // (input channel, tap) of gw
#pragma unroll
    for (int a = 1; a < NA; ++a)
#pragma unroll
        for (int t = 0; t < T; ++t) acc[0][t] += acc[a][t];
    const int ci_n = Cin - ci0 < 64 ? Cin - ci0 : 64;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // the wavefronts of the chunks' first halves write their quarter, those of the second halves add theirs
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            if (q || kh) __syncthreads();
            if ((wave >> 2) != kh) continue;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if ((wave & 1) * 2 + g / 2 != q) continue;       // rows 8g .. 8g+7 of my block lie in quarter (wave&1)*2 + g/2
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int rl = 8 * (g & 1) + 4 * half + u;   // row inside the quarter
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        float &cell = red[rl][(((wave >> 1) & 1) * 32 + l32) * T + t];
                        cell = kh ? cell + acc[0][t][4 * g + u] : acc[0][t][4 * g + u];
                    }
                }
            }
        }
        __syncthreads();
        constexpr int NE = (16 * 64 * T + kRowThreads - 1) / kRowThreads;
        float val[NE];
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int e = k * kRowThreads + tid, rl = e / (64 * T);
            val[k] = e < 16 * 64 * T ? red[rl][e - rl * (64 * T)] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int e = k * kRowThreads + tid, rl = e / (64 * T), in = e - rl * (64 * T);
            const int cc = co0 + 16 * q + rl;
            if (e < 16 * 64 * T && cc < Cout && in < ci_n * T) atomicAdd(gw + ((int64_t)cc * Cin + ci0) * T + in, val[k]);
        }
    }
}

}  // namespace

// Kernels one row high on dense channels (stride 1, channel counts in multiples of 32, k = 1, 3 or 5); rows: see the
// kernel.  gw must hold zeros; *taken = false: not its case, nothing launched.
hipError_t launch_conv1d_gw_split(const float *x, const float *gy, float *gw, int64_t rows, int RH, int64_t Cin, int64_t L,
                                  int64_t Cout, int64_t Lo, int32_t k, int32_t pad, int64_t x_cs, int64_t gy_cs, hipStream_t s,
                                  bool *taken)
{
    *taken = false;
    if ((Cin & 31) || (Cout & 31) || rows < 1 || Lo < 1 || L < 1 || Cin > 32768 || Cout > 32768) return hipSuccess;
    if (pad < 0 || pad > (1 << 20) || RH < 1) return hipSuccess;
    if (64 * x_cs + L >= (1 << 30) || 64 * gy_cs + Lo >= (1 << 30)) return hipSuccess;       // 32-bit byte offsets inside a block
    if (g_opt.conv2d_variant != 0 || g_opt.conv1d_variant != 0 || (k != 1 && k != 3 && k != 5)) return hipSuccess;
    const int cpr = (int)((Lo + 63) / 64);                         // chunks of 64 output positions per row
    const int64_t n_chunks = rows * cpr;
    const int co_blocks = (int)((Cout + 63) / 64), ci_blocks = (int)((Cin + 63) / 64);
    const int64_t blocks = (int64_t)co_blocks * ci_blocks;
    if (blocks > 65535) return hipSuccess;
    // Workgroups per block of gw: more of them shorten the walk over the chunks, and every one of them ends with
    // 4096 k adds to memory, which the chip takes at about a third of a million per microsecond.  One workgroup
    // fills a CU (LDS); a chunk takes it two microseconds or so (1.6 with the operands in the last-level cache, 3 from
    // memory).
    const int cus = device_cus();
    int64_t best = 1;
    double best_t = 1e30;
    for (int64_t sgroups = 1; sgroups * blocks <= (int64_t)cus && sgroups <= n_chunks; ++sgroups) {
        const double t = (double)((n_chunks + sgroups - 1) / sgroups) * 2.0 + (double)(sgroups * blocks) * 4096.0 * k / 350000.0;
        if (t < best_t) { best_t = t; best = sgroups; }
    }
    int64_t wgs = best;
    if (g_opt.slide_group > 0) wgs = g_opt.slide_group;
    if (wgs > n_chunks) wgs = n_chunks;
    const int64_t per = (n_chunks + wgs - 1) / wgs;
    const int64_t grid = (n_chunks + per - 1) / per;
    if (grid > 2147483647LL) return hipSuccess;
    *taken = true;
    // pairs of positions as one 64-bit access where every pair is aligned and lies wholly inside or outside its row
    const bool pair = !((uintptr_t)x & 7) && !((uintptr_t)gy & 7) && !(x_cs & 1) && !(gy_cs & 1) && !(L & 1) && !(Lo & 1);
    const int shift = pair ? (pad & 1) : 0;
#define SWS_GW1(KW_, SH_, PAIR_)                                                                                   \
    do {                                                                                                           \
        static std::atomic<int> raised{0};                                                                         \
        if (!raised.load(std::memory_order_relaxed)) {                                                             \
            const hipError_t e = hipFuncSetAttribute((const void *)conv1d_gw_split_kernel<KW_, SH_, PAIR_>,        \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, kRowLds);         \
            if (e != hipSuccess) return e;                                                                         \
            raised.store(1, std::memory_order_relaxed);                                                            \
        }                                                                                                          \
        hipLaunchKernelGGL((conv1d_gw_split_kernel<KW_, SH_, PAIR_>), dim3((unsigned)grid, (unsigned)blocks), dim3(kRowThreads), \
                           kRowLds, s, x, gy, gw, (int)Cin, (int)L, (int)Cout, (int)Lo, pad, RH, x_cs, gy_cs, cpr, n_chunks, per, \
                           ci_blocks);                                                                             \
    } while (0)
#define SWS_GW1_K(KW_)                                                                                             \
    do {                                                                                                           \
        if (!pair) SWS_GW1(KW_, 0, false);                                                                         \
        else if (shift) SWS_GW1(KW_, 1, true);                                                                     \
        else SWS_GW1(KW_, 0, true);                                                                                \
    } while (0)
    if (k == 1) SWS_GW1_K(1);
    else if (k == 3) SWS_GW1_K(3);
    else SWS_GW1_K(5);
#undef SWS_GW1_K
#undef SWS_GW1
    return hipGetLastError();
}

// *taken = false: not this kernel's case (nothing launched).  gw must hold zeros.
hipError_t launch_conv2d_gw_split(const float *x, const float *gy, float *gw, int64_t N, int64_t Cin, int64_t H, int64_t W,
                                  int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                                  int32_t ph, int32_t pw, hipStream_t s, bool *taken)
{
    *taken = false;
    if (sw != sh || (sw != 1 && sw != 2) || kh != 3 || kw != 3 || (Cin & 31) || (Cout & 31) || N < 1) return hipSuccess;
    if ((pw != 0 && pw != 1) || (sw == 2 && pw != 1) || W >= (1 << 28)) return hipSuccess;
    const bool dyn = (W & 3) || (Wo & 3);
    if (g_opt.conv2d_variant != 0 || Cin > 32768 || Cout > 32768) return hipSuccess;
    const int g8 = (int)((Wo + 7) / 8);
    const int co_blocks = (int)((Cout + 63) / 64), ci_blocks = (int)((Cin + 63) / 64);
    if ((int64_t)co_blocks * ci_blocks > 65535) return hipSuccess;
    // Workgroups per block of gw: enough to fill the GPU once, no more — every workgroup ends with atomic adds
    // of its whole block.  Rows per task S: the one whose rounds of whole tasks cost least, counting a step and a
    // half for a task's start (three rows loaded and converted with nothing to hide behind).
    int64_t wgs = (int64_t)device_cus() / ((int64_t)co_blocks * ci_blocks);
    if (wgs < 1) wgs = 1;
    if (g_opt.slide_group > 0) wgs = g_opt.slide_group;      // A/B: workgroups per block of gw
    int S = 1, nseg = (int)Ho;
    int64_t pairs = 1, per = 1;
    double best = 1e300;
    for (int s1 = 1; s1 <= 32 && s1 <= Ho; ++s1) {
        const int ns = (int)((Ho + s1 - 1) / s1);
        const int64_t pr = (N * g8 * ns + 1) / 2;
        const int64_t pw_ = (pr + wgs - 1) / wgs;
        const double cost = (double)pw_ * (s1 + 1.5);
        if (cost < best) { best = cost; S = s1; nseg = ns; pairs = pr; per = pw_; }
    }
    const int64_t n_tasks = N * g8 * nseg;
    const int64_t grid = (pairs + per - 1) / per;
    if (grid > 2147483647LL) return hipSuccess;
    *taken = true;
#define SWS_GW_SPLIT(PW_, ST_, DYN_)                                                                                  \
    hipLaunchKernelGGL((conv2d_gw_split_kernel<3, 3, PW_, ST_, DYN_>), dim3((unsigned)grid, (unsigned)(co_blocks * ci_blocks)), \
                       dim3(kThreads), 0, s, x, gy, gw, (int)Cin, (int)H, (int)W, (int)Cout, (int)Ho, (int)Wo, ph, g8, S,   \
                       nseg, n_tasks, per, ci_blocks, N * Cin * H * W, N * Cout * Ho * Wo)
    if (dyn) {
        if (sw == 2) SWS_GW_SPLIT(1, 2, true);
        else if (pw == 1) SWS_GW_SPLIT(1, 1, true);
        else SWS_GW_SPLIT(0, 1, true);
    } else {
        if (sw == 2) SWS_GW_SPLIT(1, 2, false);
        else if (pw == 1) SWS_GW_SPLIT(1, 1, false);
        else SWS_GW_SPLIT(0, 1, false);
    }
#undef SWS_GW_SPLIT
    return hipGetLastError();
}

}  // namespace sws
