// Dense-channel convolution (Section 2.5) as a sliding window sum that streams: weights stay in
// registers, the input rows a window needs are carried from one step to the next in an LDS ring
// (the carry of Algorithm 2 between vectors, here between blocks of 32 output positions), and the
// contraction over input channels runs on v_mfma_f32_32x32x2_f32 — no im2col, no column matrix.
//
// One persistent workgroup of 8 wavefronts per compute unit walks a contiguous run of position
// blocks (32 consecutive outputs of one image, flattened Ho*Wo; or 32 outputs of a 1-D row).  For a
// block the 64 x 32 outputs (64 output channels) are 2 accumulator blocks of 32 x 32; each is
// computed by FOUR wavefronts, one per quarter of the input channels, whose partial sums are
// combined through LDS (each of the four keeps a quarter of the 32 x 32 block and stores it).
// Splitting the contraction instead of the outputs makes a step cost 1/8 of a position block per
// wavefront, so that a layer with few position blocks per compute unit (configuration 4:
// 12.25) still divides evenly.
//
// Wavefront (wm, wq): output channels 32 wm .. 32 wm + 31, input channels wq*CIN/4 .. (wq+1)*CIN/4 - 1.
// Its A operands — W[co][ci][tap] for its channels and all taps, CIN*KT/8 floats per lane — are loaded
// once and live in registers.  Its B operands are 128-bit LDS reads of the staged input, layout
// [line][column][CIN + 4] (channel fastest, 4 floats of padding so that consecutive positions fall on
// consecutive bank quads): four consecutive channels of one position feed four MFMAs.
//
// MFMA operand layout (32x32x2, wave64): lane l supplies A[i = l%32][k = l/32] and B[k = l/32][j = l%32];
// accumulator register v of lane l holds D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].
//
// Lines.  Images (MODE_B = false): a line is one zero-padded input row of one image, all channels;
// block k of an image needs the lines oh_first .. oh_last + KH - 1.  1-D rows (MODE_B = true, H = 1): a
// line is 32 consecutive columns of the zero-padded row; block k needs lines k and k + 1.  Lines are
// numbered through the whole run (image after image), needed in increasing order, and line i sits in
// ring slot i mod R.  A line is requested two steps before its block and written to the ring one step
// before it; one workgroup barrier per block.
//
// What shapes the inner loop (measured on this GPU): a vector-ALU instruction between two MFMAs of a
// SIMD delays the matrix pipe by about 3 cycles (a pure MFMA stream runs at 98 % of the matrix peak
// with one wavefront and one dependent accumulator chain per SIMD), scalar and memory instructions do
// not.  So the per-step vector work is kept small — tap offsets are instruction immediates, the zero
// padding columns of the ring are written once, the staging of a line uses one lane offset for all its
// loads — and what remains is spread between the groups of four MFMAs.
//
// Split operands (template flag X3, images only).  An fp32 number is the exact sum of three bf16
// numbers (the leading, middle and last 8 bits of its mantissa, each the upper half of an fp32 word),
// and a product of two bf16 numbers is exact in fp32.  Of the nine piece products of x * w the three
// smallest are below 2^-23 of the product; the other six, accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16, give the fp32 result to within less than one fp32 rounding per term — in
// 6 instructions of 32 cycles per 16 channels and tap instead of 8 of 64 cycles.  The input is split when
// a line is written to the ring (three bf16 planes per position, 384 bytes for 64 channels, 16-byte
// channel groups permuted by the column so that the operand reads need no padding); the weights are
// split once per run (108 registers).  The larger ring leaves room for one hand-over buffer only, so
// this form has two workgroup barriers per block.
#include "sws_internal.h"

namespace sws {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int kPad = 4;                               // floats of padding per staged position
constexpr int kScratchFloats = 2 * 2 * 4 * 3 * 64 * 4;  // [buffer][wm][owner quarter][source][lane][4]
constexpr int kSpareFloats = 128;                     // where lanes without a column of their own write
constexpr int kPitch3 = 384;                          // bytes per staged position, three bf16 planes of 64 channels

struct StreamGeom {
    int N, H, W, Ho, Wo, ph, pw, Cout;
    int LW;                                           // positions per line
    int LPI, BPI;                                     // lines / position blocks per image
    int R;                                            // ring slots
    float inv_R, inv_Wo;
    int q31, r31;                                     // 31 / Wo and 31 % Wo
    int co_tiles;
    int wadj;                                         // weights read as the adjoint's: wgt[ci][co][last tap - t]
    long long T;                                      // position blocks in all: co_tiles * N * BPI
};

// x / d for 0 <= x < 2^20 and 1 <= d < 2^12, exact (the margin 0.5/d dwarfs the rounding of the product)
__device__ __forceinline__ int fdiv(int x, float inv_d) { return (int)(((float)x + 0.5f) * inv_d); }

// CGS = log2 of the 16-column groups per line, rounded up to a power of two (0 .. 2)
// X3: the arithmetic runs on the bf16 matrix cores with operands split exactly (see the file header).
template <int CIN, int KH, int KW, bool MODE_B, int CGS, bool WADJ, bool X3 = false>
__global__ __launch_bounds__(kThreads) void conv_stream_kernel(const float *__restrict__ x,
                                                               const float *__restrict__ wgt,
                                                               float *__restrict__ y, StreamGeom g)
{
    constexpr int KT = KH * KW;
    constexpr int PITCH = CIN + kPad;
    constexpr int PB = X3 ? kPitch3 : PITCH * 4;      // bytes per staged position
    static_assert(!X3 || (CIN == 64 && !MODE_B), "the split-operand path is built for 64-channel images");
    constexpr int CQ = CIN / 4;                       // input channels per wavefront
    constexpr int NCB = CQ / 8;                       // blocks of 8 channels among them
    // staging: a group is 16 columns x 4 channels (lane = column + 16 * channel); slot s of this wavefront
    // moves group wave + 8 s.  With 2^CGS column groups all my slots have the same column group and
    // channels CH_STEP groups apart.
    constexpr int CH_STEP = 8 >> CGS;
    constexpr int XS = (CIN / 4 + CH_STEP - 1) / CH_STEP;     // slots per line and wavefront
    constexpr int H2 = XS / 2;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *ring = lds;
    float *scratch = lds + g.R * g.LW * (PB / 4);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wave & 1, wq = wave >> 1;
    const int HW = g.H * g.W, HoWo = g.Ho * g.Wo;

    // my run of position blocks.  Workgroup b runs on XCD b mod 8: each XCD takes one contiguous
    // eighth of the runs, so neighbouring runs (which share input rows) meet in one L2.
    const int G = gridDim.x;
    const int gi = (G & 7) ? (int)blockIdx.x : (int)(blockIdx.x & 7) * (G >> 3) + (int)(blockIdx.x >> 3);
    const long long b0 = (long long)gi * g.T / G, b1 = (long long)(gi + 1) * g.T / G;
    if (b0 >= b1) return;
    const long long img0 = b0 / g.BPI;                // combined index: co tile * N + image
    int k = (int)(b0 - img0 * g.BPI);
    int ct = (int)(img0 / g.N), n = (int)(img0 - (long long)ct * g.N);

    // last input line (exclusive) that block kk of an image needs, given the row (q) of its last position
    auto hi_of = [&](int kk, int q) { return MODE_B ? kk + 2 : (kk == g.BPI - 1 ? g.LPI : q + KH); };
    const int lo0 = MODE_B ? k : __builtin_amdgcn_readfirstlane(fdiv(32 * k, g.inv_Wo));
    // line numbers relative to the first line of the run: image i, line r  ->  (i - img0) * LPI + r - lo0
    int img_base = -lo0;                              // relative number of line 0 of the current block's image
    int next_line = 0;                                // first line not yet requested
    int st_n = n, st_pr = lo0;                        // image and line-in-image of next_line

    // ---- staging of a line: one lane offset serves all my slots
    const int cg0 = wave & ((1 << CGS) - 1), chg0 = wave >> CGS;
    const int st_pc = 16 * cg0 + (lane & 15), st_ci = 4 * chg0 + (lane >> 4);
    const int st_c = st_pc - g.pw;                    // images: the column inside the image; rows: plus 32 * line
    const bool st_in = st_pc < g.LW;
    const bool st_colok = st_in && st_c >= 0 && st_c < g.W;
    const int st_src = st_ci * HW + ((MODE_B || st_colok) ? st_c : 0);     // element offset inside an image at line 0
    // Byte offset inside a ring slot.  Images: lanes whose column is padding or beyond the line write to a
    // spare area behind the scratch buffers instead — the ring is cleared once, so the zero padding
    // columns of every slot stay zero.  Rows: every lane inside the line writes (zero where the row ends).
    const bool st_wr = MODE_B ? st_in : st_colok;
    // (X3: position st_pc, plane p, channel ci at p * 128 + 16 * ((ci >> 3) ^ ((st_pc >> 1) & 7)) + 2 * (ci & 7):
    // the 16-byte groups of eight channels are permuted by the column.  With the 384-byte position pitch,
    // sixteen consecutive positions reading the same group then fall on sixteen different 16-byte bank
    // groups: even and odd columns differ in bank bit 7, and eight columns of one parity in the permutation)
    const int st_dst = X3 ? st_pc * PB + 2 * (st_ci & 7) : (st_pc * PITCH + st_ci) * 4;
    const int st_key = (st_pc >> 1) & 7, st_c8 = st_ci >> 3;
    char *const spare = (char *)(scratch + (X3 ? kScratchFloats / 2 : kScratchFloats));
    constexpr int SRC_STEP = 4 * CH_STEP, DST_STEP = 16 * CH_STEP;          // channels / bytes from one slot to the next
    auto line_begin = [&](int &l_n, int &l_pr, int &l_rel) {
        l_n = st_n; l_pr = st_pr; l_rel = next_line;
        ++next_line;
        if (++st_pr == g.LPI) { st_pr = 0; if (++st_n == g.N) st_n = 0; }
    };
    // a line's loads (issue) and, later, its LDS writes (commit), each in two halves of the slots so that
    // they can be spread between the matrix instructions
    auto issue = [&](float (&xr)[XS], int l_n, int l_pr, int s0, int s1) {
        const float *xi = x + (long long)l_n * CIN * HW;
        const int r = MODE_B ? 0 : l_pr - g.ph;
        if (r >= 0 && r < g.H) {
            const int line_off = MODE_B ? 32 * l_pr : r * g.W;
            const bool ok = !MODE_B || (unsigned)(st_c + line_off) < (unsigned)g.W;
            const unsigned at = ok ? (unsigned)(st_src + line_off) : 0u;
#pragma unroll
            for (int s = 0; s < XS; ++s) {
                if (s < s0 || s >= s1) continue;
                if (chg0 + s * CH_STEP < CIN / 4) xr[s] = (xi + (long long)s * SRC_STEP * HW)[at];
            }
        }
    };
    auto commit = [&](const float (&xr)[XS], int l_pr, int l_rel, int s0, int s1) {
        const int slot = l_rel - g.R * __builtin_amdgcn_readfirstlane(fdiv(l_rel, g.inv_R));
        char *dst = st_wr ? (char *)ring + slot * (g.LW * PB) + st_dst : spare;
        const int r = MODE_B ? 0 : l_pr - g.ph;
        if constexpr (X3) {
            const bool real = r >= 0 && r < g.H;
#pragma unroll
            for (int s = 0; s < XS; ++s) {
                if (s < s0 || s >= s1) continue;
                if (chg0 + s * CH_STEP < CIN / 4) {
                    // x = x1 + x2 + x3 exactly: the leading 8, the next 8 and the last 8 bits of the mantissa,
                    // each the upper half of an fp32 word (a bf16 number), both differences exact
                    const float v = real ? xr[s] : 0.0f;
                    const unsigned u1 = __float_as_uint(v) & 0xffff0000u;
                    const float r1 = v - __uint_as_float(u1);
                    const unsigned u2 = __float_as_uint(r1) & 0xffff0000u;
                    const unsigned u3 = __float_as_uint(r1 - __uint_as_float(u2));
                    char *d = dst + 16 * ((st_c8 + s * (SRC_STEP / 8)) ^ st_key);
                    *(unsigned short *)d = (unsigned short)(u1 >> 16);
                    *(unsigned short *)(d + 128) = (unsigned short)(u2 >> 16);
                    *(unsigned short *)(d + 256) = (unsigned short)(u3 >> 16);
                }
            }
            return;
        }
        if (MODE_B) {
            const bool ok = (unsigned)(st_c + 32 * l_pr) < (unsigned)g.W;
#pragma unroll
            for (int s = 0; s < XS; ++s) {
                if (s < s0 || s >= s1) continue;
                if (chg0 + s * CH_STEP < CIN / 4) *(float *)(dst + s * DST_STEP) = ok ? xr[s] : 0.0f;
            }
        } else if (r >= 0 && r < g.H) {
#pragma unroll
            for (int s = 0; s < XS; ++s) {
                if (s < s0 || s >= s1) continue;
                if (chg0 + s * CH_STEP < CIN / 4) *(float *)(dst + s * DST_STEP) = xr[s];
            }
        } else {                                      // a line above or below the image
#pragma unroll
            for (int s = 0; s < XS; ++s) {
                if (s < s0 || s >= s1) continue;
                if (chg0 + s * CH_STEP < CIN / 4) *(float *)(dst + s * DST_STEP) = 0.0f;
            }
        }
    };
    // stages the lines [next_line, need), one after the other (the start of a run, a step into the next image)
    float xr0[XS];
    int n0r = 0, p0r = 0, r0r = 0;
    auto stage_sync = [&](int need) {
        while (next_line < need) {
            line_begin(n0r, p0r, r0r);
            issue(xr0, n0r, p0r, 0, XS);
            commit(xr0, p0r, r0r, 0, XS);
        }
    };
    // the same at the start of a run, two lines' loads in flight at a time (X3)
    auto stage_first = [&](int need) {
        float xr1[XS];
        int n1r = 0, p1r = 0, r1r = 0;
        while (next_line + 1 < need) {
            line_begin(n0r, p0r, r0r);
            issue(xr0, n0r, p0r, 0, XS);
            line_begin(n1r, p1r, r1r);
            issue(xr1, n1r, p1r, 0, XS);
            commit(xr0, p0r, r0r, 0, XS);
            commit(xr1, p1r, r1r, 0, XS);
        }
        stage_sync(need);
    };

    // ---- weights: A operands of all my MFMAs, loaded once per output-channel tile.  A lane's weights
    // lie 2304 bytes from its neighbour's, so the tile is first copied to LDS with coalesced loads (in
    // two halves of 32 output channels, rows padded by one float: lane = output channel then reads
    // conflict-free) and the registers are filled from there.  Uses the ring's memory: called before
    // the first line is staged, or (a later tile of output channels) re-stages the ring afterwards.
    float w[X3 ? 1 : KT][NCB][4];
    // X3: W[co][ci = 16 wq + 8 half + e][t] as three bf16 pieces, eight channels per register quad — the A
    // operand of v_mfma_f32_32x32x16_bf16 (lane = output channel + 32 * (k / 8), element = k % 8)
    v8bf w3[X3 ? KT : 1][3];
    auto load_weights = [&](int tile) {
        constexpr int ROW = CIN * KT, WP = ROW + 1;
        constexpr int PER = 32 * ROW / 4 / kThreads;  // 128-bit loads per thread and half tile
        static_assert(32 * ROW % (4 * kThreads) == 0 && ROW % 4 == 0, "half a tile divides over the threads");
        float *wl = lds;
        constexpr int HALF = WADJ ? 32 * ROW : 32 * WP;        // floats of a staged half tile
        if constexpr (X3) {
            // the larger LDS of this form holds both halves side by side: one round of loads, every
            // wavefront fills its registers at the same time
            __syncthreads();                          // (the memory is the ring's: its last readers are done)
#pragma unroll 1
            for (int h = 0; h < 2; ++h) {
                v4f v[PER];
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int e = 4 * (threadIdx.x + u * kThreads);
                    if (WADJ) {
                        const int ci = e / (32 * KT), q = e - ci * (32 * KT);
                        v[u] = *(const v4f_u *)(wgt + (unsigned)((ci * g.Cout + tile * 64 + 32 * h) * KT + q));
                    } else {
                        v[u] = *(const v4f_u *)(wgt + (unsigned)((tile * 64 + 32 * h) * ROW) + e);
                    }
                }
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int e = 4 * (threadIdx.x + u * kThreads);
                    if (WADJ) {
                        ((v4f *)(wl + h * HALF))[threadIdx.x + u * kThreads] = v[u];
                    } else {
                        float *d = wl + h * HALF + e + e / ROW;
                        d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
                    }
                }
            }
            __syncthreads();
            const float *wh = wl + wm * HALF;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int ci = wq * CQ + 8 * half + e;
                const float *rd = WADJ ? wh + ci * (32 * KT) + l32 * KT : wh + l32 * WP + ci * KT;
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    const float f = rd[WADJ ? KT - 1 - t : t];
                    const __bf16 f1 = (__bf16)f;
                    const float r1 = f - (float)f1;
                    const __bf16 f2 = (__bf16)r1;
                    w3[t][0][e] = f1;
                    w3[t][1][e] = f2;
                    w3[t][2][e] = (__bf16)(r1 - (float)f2);
                }
                __builtin_amdgcn_sched_barrier(0);            // (one channel's reads in flight at a time: registers)
            }
        } else
#pragma unroll 1
        for (int h = 0; h < 2; ++h) {
            v4f v[PER];
            if (WADJ) {
                // stored as wgt[ci][co][KT - 1 - t] with rows of Cout pairs: for every ci the half tile is one
                // contiguous range of 32 * KT floats; it is copied as it is (lane = output channel then
                // reads addresses 9 floats apart: conflict-free)
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int e = 4 * (threadIdx.x + u * kThreads);
                    const int ci = e / (32 * KT), q = e - ci * (32 * KT);
                    v[u] = *(const v4f_u *)(wgt + (unsigned)((ci * g.Cout + tile * 64 + 32 * h) * KT + q));
                }
                __syncthreads();
#pragma unroll
                for (int u = 0; u < PER; ++u) ((v4f *)wl)[threadIdx.x + u * kThreads] = v[u];
            } else {
                // stored as wgt[co][ci][t]: the half tile is one contiguous range; rows padded by one float in LDS
                const float *src = wgt + (unsigned)((tile * 64 + 32 * h) * ROW);
#pragma unroll
                for (int u = 0; u < PER; ++u) v[u] = *(const v4f_u *)(src + 4 * (threadIdx.x + u * kThreads));
                __syncthreads();
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int e = 4 * (threadIdx.x + u * kThreads);
                    float *d = wl + e + e / ROW;      // row e / ROW starts (e / ROW) floats later
                    d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
                }
            }
            __syncthreads();
            if (wm == h) {
                if constexpr (X3) {
                } else {
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int ci = wq * CQ + cb * 8 + 4 * half + j;
                            const float *rd = WADJ ? wl + ci * (32 * KT) + l32 * KT : wl + l32 * WP + ci * KT;
#pragma unroll
                            for (int t = 0; t < KT; ++t) w[t][cb][j] = rd[WADJ ? KT - 1 - t : t];
                        }
                }
            }
        }
        __syncthreads();
        // the registers are settled here, so that no matrix instruction of the loop below waits on a counter
        if constexpr (X3) {
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    v4u q = __builtin_bit_cast(v4u, w3[t][p]);
                    asm volatile("" : "+v"(q));
                    w3[t][p] = __builtin_bit_cast(v8bf, q);
                }
        } else {
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(w[t][cb][j]));
        }
    };

    // ---- where my position's taps are in the ring, for block kk of the image whose line 0 has number `base`:
    // images: one byte offset per kernel row (the taps of a row are immediates); rows: one per tap
    constexpr int NB = X3 ? KT : (MODE_B ? KW : KH);
    const int lane_const = (wq * CQ + 4 * half) * 4;
    const int oct = 2 * wq + half;                    // X3: my eight channels are group `oct` of a plane
    auto bases = [&](int kk, int base, int (&rb)[NB], bool &pok, int &pp) {
        const int p = 32 * kk + l32;
        pok = p < HoWo;
        pp = pok ? p : 32 * kk;
        if (MODE_B) {
#pragma unroll
            for (int b = 0; b < KW; ++b) {
                const int pc = pp + b;
                const int line = base + (pc >> 5);
                const int slot = line - g.R * fdiv(line, g.inv_R);
                rb[b] = ((slot * 32 + (pc & 31)) * PITCH) * 4 + lane_const;
            }
        } else {
            const int oh = fdiv(pp, g.inv_Wo), ow = pp - oh * g.Wo;
            const int line = base + oh;
            int slot = line - g.R * fdiv(line, g.inv_R);
#pragma unroll
            for (int a = 0; a < KH; ++a) {
                if constexpr (X3) {
#pragma unroll
                    for (int b = 0; b < KW; ++b)
                        rb[a * KW + b] = (slot * g.LW + ow + b) * PB + 16 * (oct ^ (((ow + b) >> 1) & 7));
                } else {
                    rb[a] = ((slot * g.LW + ow) * PITCH) * 4 + lane_const;
                }
                slot = slot + 1 == g.R ? 0 : slot + 1;
            }
        }
    };

    // the block finished in the previous step: my quarter of its sums, where it goes
    float mine[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float *y_prev = y;
    bool pok_prev = false, have_prev = false;
    int buf = 0;
    const v4f *sc_rd = (const v4f *)scratch + ((wm * 4 + wq) * 3) * 64 + lane;      // + buffer * 1536
    v4f *sc_wr = (v4f *)scratch + (wm * 4) * 3 * 64 + lane;
    const long long co_off = (long long)(32 * wm + 8 * wq + 4 * half) * HoWo;
    constexpr int SCB = X3 ? 0 : 2 * 4 * 3 * 64;      // v4f per hand-over buffer (X3: one buffer, two barriers per block)
    auto finish = [&](int b) {
        const v4f *sp = sc_rd + b * SCB;
        const v4f f = sp[0] + sp[64] + sp[128];
        if (pok_prev) {
#pragma unroll
            for (int q = 0; q < 4; ++q) y_prev[(long long)q * HoWo] = mine[q] + f[q];
        }
    };

    int rb[NB];
    bool pok = false;
    int pp = 0;
    long long gb = b0;
    while (gb < b1) {
    // a stretch of the run with one tile of output channels: its weights are loaded here, outside the
    // loop over blocks, through the ring's memory — so the previous block is finished first and the
    // lines the current block needs are staged (again) afterwards
    if (have_prev) { finish(buf ^ 1); have_prev = false; }
    load_weights(ct);
    if (!MODE_B) {                                    // clear the ring: its zero padding columns are never written again
        const int n4 = g.R * g.LW * (PB / 16);
        for (int i = threadIdx.x; i < n4; i += kThreads) ((v4f *)ring)[i] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        __syncthreads();
    }
    // (q, r) = (row, column) of the last position of a block, carried from block to block
    int q1 = 0, r1 = 0;
    if (!MODE_B) {
        q1 = __builtin_amdgcn_readfirstlane(fdiv(32 * k + 31, g.inv_Wo));
        r1 = 32 * k + 31 - q1 * g.Wo;
    }
    {
        // rewind the staging state to the current block's first line
        const int lo_c = MODE_B ? k : __builtin_amdgcn_readfirstlane(fdiv(32 * k, g.inv_Wo));
        next_line = img_base + lo_c; st_n = n; st_pr = lo_c;
        if constexpr (X3) stage_first(img_base + hi_of(k, q1));
        else stage_sync(img_base + hi_of(k, q1));
    }
    bases(k, img_base, rb, pok, pp);
    long long seg_end = (long long)(ct + 1) * g.N * g.BPI;
    if (seg_end > b1) seg_end = b1;
    // the blocks after the current one: (k2 ..) the next, (k3 ..) the one after it
    auto advance = [&](int &kk, int &nn, int &cc, int &bb, int &q, int &r) {
        if (++kk == g.BPI) {
            kk = 0; bb += g.LPI; q = g.q31; r = g.r31;
            if (++nn == g.N) { nn = 0; ++cc; }
        } else {
            r += 32;
            while (r >= g.Wo) { r -= g.Wo; ++q; }
        }
    };
    int k2 = k, n2 = n, ct2 = ct, base2 = img_base, q2 = q1, r2 = r1;
    advance(k2, n2, ct2, base2, q2, r2);
    int k3 = k2, n3 = n2, ct3 = ct2, base3 = base2, q3 = q2, r3 = r2;
    advance(k3, n3, ct3, base3, q3, r3);
    int need2 = gb + 1 < b1 ? base2 + hi_of(k2, q2) : 0;      // lines (numbers below) the next block needs
    int need3 = gb + 2 < b1 ? base3 + hi_of(k3, q3) : need2;  // ... and the one after it
    bool pending = false;                             // a line requested in the previous step, not yet in the ring
    __syncthreads();
    for (; gb < seg_end; ++gb) {
        // ---- lines: the one requested in the previous step goes into the ring early in this step's matrix
        // work, and the next line that the block after the next one needs is requested — two steps ahead
        // of its use, so that its loads have a whole step to come back.  Whatever the next block still
        // lacks after the matrix work (the first step of a run, a step into the next image) is staged then.
        const bool more = gb + 1 < b1;
        const bool commit_now = pending;
        const int cp = p0r, cr = r0r;                 // the pending line's place
        const bool issue_now = next_line < need3;

        // ---- matrix work: the B operands are read DEPTH groups ahead; the rest of the step's work sits
        // between the groups of four MFMAs
        v16f acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
        // (X3: a group is one operand read — piece p of the input under tap t — and the matrix instructions
        // it feeds: the products of input piece p with weight pieces 1 .. 3 - p, i.e. every pair whose
        // product is not below 2^-24 of the full product)
        constexpr int STEPS = X3 ? KT * 3 : KT * NCB, DEPTH = 2;
        constexpr int I_COM = 0, I_ISS = 2, I_FIN = STEPS >= 7 ? 4 : 0, I_ADR = STEPS >= 7 ? 6 : 1, I_BAS = STEPS - 1 - DEPTH;
        static_assert(STEPS >= 4 && STEPS > DEPTH, "room for the pieces between the groups");
        v4f bq[DEPTH + 1];
        float *y_cur = y;
        int t_k3 = k3, t_n3 = n3, t_ct3 = ct3, t_base3 = base3, t_q3 = q3, t_r3 = r3, t_need3 = need3;
        auto bread = [&](int i) {
            if constexpr (X3) {
                return *(const v4f *)((const char *)ring + rb[i / 3] + (i % 3) * 128);
            } else {
                const int t = i / NCB, cb = i % NCB;
                const int ofs = MODE_B ? cb * 32 : (t % KW) * PITCH * 4 + cb * 32;      // an instruction immediate
                return *(const v4f *)((const char *)ring + rb[MODE_B ? t : t / KW] + ofs);
            }
        };
#pragma unroll
        for (int i = 0; i < DEPTH; ++i) bq[i] = bread(i);
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            if (i + DEPTH < STEPS) bq[(i + DEPTH) % (DEPTH + 1)] = bread(i + DEPTH);
            __builtin_amdgcn_sched_barrier(0);        // keep the read ahead of the MFMAs below
            const v4f b4 = bq[i % (DEPTH + 1)];
            if constexpr (X3) {
                const v8bf b8 = __builtin_bit_cast(v8bf, b4);
                const int t = i / 3, p = i % 3;
                if (p == 0) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w3[t][2], b8, acc, 0, 0, 0);
                if (p <= 1) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w3[t][1], b8, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w3[t][0], b8, acc, 0, 0, 0);
            } else {
                const int t = i / NCB, cb = i % NCB;
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w[t][cb][0], b4.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w[t][cb][1], b4.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w[t][cb][2], b4.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w[t][cb][3], b4.w, acc, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (i == I_COM && commit_now) commit(xr0, cp, cr, 0, H2);
            if (i == I_COM + 1 && commit_now) commit(xr0, cp, cr, H2, XS);
            if (i == I_ISS && issue_now) { line_begin(n0r, p0r, r0r); issue(xr0, n0r, p0r, 0, H2); }
            if (i == I_ISS + 1 && issue_now) issue(xr0, n0r, p0r, H2, XS);
            if (i == I_FIN && have_prev) {            // the previous block: the other quarters' partial sums
                const v4f *sp = sc_rd + (buf ^ 1) * SCB;
                const v4f f = sp[0] + sp[64] + sp[128];
                mine[0] += f.x; mine[1] += f.y; mine[2] += f.z; mine[3] += f.w;
            }
            if (i == I_FIN + 1 && have_prev && pok_prev) {
#pragma unroll
                for (int q = 0; q < 4; ++q) y_prev[(long long)q * HoWo] = mine[q];
            }
            // accumulator register 4 wq + i is output channel 8 wq + 4 half + i of my block of 32
            if (i == I_ADR) {
                y_cur = y + ((long long)n * g.Cout + ct * 64) * HoWo + co_off + pp;
                // scalar bookkeeping for the step after the next, here where it costs no matrix time
                advance(t_k3, t_n3, t_ct3, t_base3, t_q3, t_r3);
                t_need3 = gb + 3 < b1 ? t_base3 + hi_of(t_k3, t_q3) : need3;
            }
            // after the last read of this block has been issued: the next block's tap addresses
            if (i == I_BAS) {
                pok_prev = pok;
                if (more) bases(k2, base2, rb, pok, pp);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- hand the three quarters I do not own to their owners; keep mine.  Quarter (wq + 1 + j) & 3 lists
        // me as its source 2 - j, so the three addresses are wave constants; which accumulator registers go
        // where depends on wq: one branch over four short copies of the code.
        {
            if constexpr (X3) __syncthreads();        // one hand-over buffer: every wavefront has read the previous block's sums
            v4f *wr = sc_wr + buf * SCB;
#define SWS_HAND(Q0, Q1, Q2, Q3)                                                                    \
    mine[0] = acc[4 * Q0]; mine[1] = acc[4 * Q0 + 1]; mine[2] = acc[4 * Q0 + 2]; mine[3] = acc[4 * Q0 + 3];       \
    wr[(Q1 * 3 + 2) * 64] = (v4f){acc[4 * Q1], acc[4 * Q1 + 1], acc[4 * Q1 + 2], acc[4 * Q1 + 3]};                \
    wr[(Q2 * 3 + 1) * 64] = (v4f){acc[4 * Q2], acc[4 * Q2 + 1], acc[4 * Q2 + 2], acc[4 * Q2 + 3]};                \
    wr[(Q3 * 3 + 0) * 64] = (v4f){acc[4 * Q3], acc[4 * Q3 + 1], acc[4 * Q3 + 2], acc[4 * Q3 + 3]}
            if (wq == 0) { SWS_HAND(0, 1, 2, 3); }
            else if (wq == 1) { SWS_HAND(1, 2, 3, 0); }
            else if (wq == 2) { SWS_HAND(2, 3, 0, 1); }
            else { SWS_HAND(3, 0, 1, 2); }
#undef SWS_HAND
        }
        y_prev = y_cur;
        have_prev = true;

        // ---- lines the next block still lacks
        pending = issue_now;
        if (more) {
            if (pending && r0r < need2) { commit(xr0, p0r, r0r, 0, XS); pending = false; }
            stage_sync(need2);
        }
        __syncthreads();
        buf ^= 1;
        k = k2; n = n2; ct = ct2; img_base = base2;
        k2 = k3; n2 = n3; ct2 = ct3; base2 = base3; q2 = q3; r2 = r3;
        need2 = need3;
        k3 = t_k3; n3 = t_n3; ct3 = t_ct3; base3 = t_base3; q3 = t_q3; r3 = t_r3;
        need3 = t_need3;
    }
    }
    finish(buf ^ 1);
}

template <int CIN, int KH, int KW, bool MODE_B, int CGS, bool WADJ, bool X3 = false>
hipError_t launch_stream1(const float *x, const float *wgt, float *y, const StreamGeom &g, size_t lds, int grid,
                         hipStream_t s)
{
    static bool raised = false;                       // (set once per process; the attribute is per function)
    if (!raised && lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute((const void *)conv_stream_kernel<CIN, KH, KW, MODE_B, CGS, WADJ, X3>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((conv_stream_kernel<CIN, KH, KW, MODE_B, CGS, WADJ, X3>), dim3((unsigned)grid), dim3(kThreads), lds, s, x,
                       wgt, y, g);
    return hipGetLastError();
}

template <int CIN, int KH, int KW, bool MODE_B, int CGS>
hipError_t launch_stream(const float *x, const float *wgt, float *y, const StreamGeom &g, size_t lds, int grid,
                         hipStream_t s)
{
    if (g.wadj) return launch_stream1<CIN, KH, KW, MODE_B, CGS, true>(x, wgt, y, g, lds, grid, s);
    return launch_stream1<CIN, KH, KW, MODE_B, CGS, false>(x, wgt, y, g, lds, grid, s);
}

}  // namespace

// Stride 1, taps adjacent, groups = 1, 64 input channels, output channels in multiples of 64, kernels of
// 3 x 3 (images whose padded rows have at most 64 columns) and 1 x 3 (1-D rows).  *taken = false:
// not one of these, or too little work to fill the device — nothing was launched.
hipError_t launch_conv2d_stream(const float *x, const float *wgt, float *y, int64_t N, int64_t Cin, int64_t H, int64_t W,
                                int64_t Cout, int64_t Ho, int64_t Wo, int32_t kh, int32_t kw, int32_t ph, int32_t pw,
                                hipStream_t s, bool *taken, int wadj)
{
    *taken = false;
    if (Cin != 64 || Cout % 64 != 0 || Cout < 64 || kw != 3 || (kh != 3 && kh != 1) || ph < 0 || pw < 0 ||
        ph >= kh || pw >= kw)
        return hipSuccess;
    const bool mode_b = H == 1 && kh == 1;
    if (!mode_b && kh != 3) return hipSuccess;
    if (N > (1 << 20) || Ho * Wo >= (1 << 20) || H >= (1 << 16) || W >= (1LL << 30) || Cin * H * W >= 2147483647LL ||
        Cout * Cin * kh * kw >= 2147483647LL)
        return hipSuccess;
    StreamGeom g;
    g.N = (int)N; g.H = (int)H; g.W = (int)W; g.Ho = (int)Ho; g.Wo = (int)Wo; g.ph = ph; g.pw = pw; g.Cout = (int)Cout;
    g.wadj = wadj;
    g.co_tiles = (int)(Cout / 64);
    g.q31 = (int)(31 / Wo); g.r31 = (int)(31 % Wo);
    const int64_t HoWo = Ho * Wo;
    g.BPI = (int)((HoWo + 31) / 32);
    int need = 0;                                     // most lines alive at once: this block's and the next one's
    int cgs = 1;
    if (mode_b) {
        g.LW = 32;
        g.LPI = g.BPI + 1;
        need = 4;                                     // lines k, k+1 and, stepping into the next row, its lines 0, 1
    } else {
        const int64_t Wt = Wo + kw - 1;               // columns of a padded row that the windows reach
        if (Wt > 64) return hipSuccess;
        g.LW = (int)Wt;
        cgs = Wt <= 16 ? 0 : (Wt <= 32 ? 1 : 2);
        g.LPI = (int)(Ho + kh - 1);
        // lines [lo(k), hi(k+1)) must fit the ring: walk the blocks of one image and the step into the next image
        for (int k = 0; k < g.BPI; ++k) {
            const int64_t p0 = 32LL * k, pl = p0 + 31 < HoWo ? p0 + 31 : HoWo - 1;
            const int lo = (int)(p0 / Wo);
            int hi2;
            if (k + 1 < g.BPI) {
                const int64_t q0 = 32LL * (k + 1), ql = q0 + 31 < HoWo ? q0 + 31 : HoWo - 1;
                hi2 = (int)(ql / Wo) + kh;
            } else {
                const int64_t ql = 31 < HoWo ? 31 : HoWo - 1;
                hi2 = g.LPI + (int)(ql / Wo) + kh;
            }
            const int hi = (int)(pl / Wo) + kh;
            const int alive = (hi2 > hi ? hi2 : hi) - lo;
            if (alive > need) need = alive;
        }
    }
    g.R = need;
    size_t lds = 4 * ((size_t)g.R * g.LW * (64 + kPad) + kScratchFloats + kSpareFloats);
    const size_t wtmp = 4 * (size_t)32 * (64 * kh * kw + 1);      // half a tile of weights passes through LDS
    if (lds < wtmp) lds = wtmp;
    if (lds > 160 * 1024) return hipSuccess;
    g.inv_R = 1.0f / (float)g.R;
    g.inv_Wo = 1.0f / (float)g.Wo;
    g.T = (long long)g.co_tiles * N * g.BPI;
    const int cus = device_cus();
    // line numbers inside a run stay below 2^20 (the reciprocal division), and a run must be long enough
    // for the weights and the first lines to pay off: about 13000 cycles of set-up against 1024 cycles of
    // matrix work per block and tap.  Measured: [16,64,4096] x [64,64,3] (24 block-taps per CU) 25.2 us here
    // against 21.6 us on the tile kernel; [32,64,56,56] x [64,64,3,3] (110 per CU) 75 - 83 us against 83 - 85 us.
    const int64_t lines_per_run = (g.T / cus + 2) / g.BPI * g.LPI + 2LL * g.LPI;
    if ((g.T * kh * kw < 60LL * cus && g_opt.conv2d_variant != 17 && g_opt.conv2d_variant != 18) || lines_per_run >= (1 << 20))
        return hipSuccess;
    *taken = true;
    // the split-operand instance: images, forward weights, and its larger ring must fit
    size_t lds3 = (size_t)g.R * g.LW * kPitch3 + 4 * (kScratchFloats / 2 + kSpareFloats);
    if (lds3 < 2 * wtmp) lds3 = 2 * wtmp;             // the whole weight tile passes through LDS at once
    if (!mode_b && g_opt.conv2d_variant != 17 && lds3 <= 160 * 1024) {
        if (wadj) {
            if (cgs == 0) return launch_stream1<64, 3, 3, false, 0, true, true>(x, wgt, y, g, lds3, cus, s);
            if (cgs == 1) return launch_stream1<64, 3, 3, false, 1, true, true>(x, wgt, y, g, lds3, cus, s);
            return launch_stream1<64, 3, 3, false, 2, true, true>(x, wgt, y, g, lds3, cus, s);
        }
        if (cgs == 0) return launch_stream1<64, 3, 3, false, 0, false, true>(x, wgt, y, g, lds3, cus, s);
        if (cgs == 1) return launch_stream1<64, 3, 3, false, 1, false, true>(x, wgt, y, g, lds3, cus, s);
        return launch_stream1<64, 3, 3, false, 2, false, true>(x, wgt, y, g, lds3, cus, s);
    }
    if (mode_b) return launch_stream<64, 1, 3, true, 1>(x, wgt, y, g, lds, cus, s);
    if (cgs == 0) return launch_stream<64, 3, 3, false, 0>(x, wgt, y, g, lds, cus, s);
    if (cgs == 1) return launch_stream<64, 3, 3, false, 1>(x, wgt, y, g, lds, cus, s);
    return launch_stream<64, 3, 3, false, 2>(x, wgt, y, g, lds, cus, s);
}

}  // namespace sws
