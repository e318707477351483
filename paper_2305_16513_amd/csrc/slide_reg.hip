// Sliding window sums of medium windows (Section 2.2, Eq. 3), 5 <= w <= 65, on strips held in registers.
//
// A wavefront loads 256 consecutive inputs of a row as one 128-bit load per lane (a 1 KB strip: the
// launch shape in which this GPU moves memory fastest) and keeps them there: no LDS, no second load.
// Lane L owns outputs 4L .. 4L+3 of the strip.  With P_L[t] the sum of the lane's first t+1 elements,
// T_L = P_L[3] and F_L[j] the sum of its elements j .. 3, the window of output 4L + j ends in lane
// L + q at element t, where 4q + t = j + w - 1, and
//
//     y[4L + j] = F_L[j] (+) T_{L+1} (+) ... (+) T_{L+q-1} (+) P_{L+q}[t]
//
// — Section 3's split of a window into the tail of one vector, whole vectors and the head of another
// (Algorithm 2's suffix and prefix sums), with lanes as the vectors.  The run of whole lanes is summed
// from power-of-two runs (1, 2, 4, 8 lanes, built by doubling with ds_bpermute) chosen by the bits of its
// length, oldest first, so operand order is kept.  Lanes whose windows would leave the strip produce
// nothing: strips overlap by the window's reach rounded up to 16 elements, so a strip yields 256 - that
// many outputs and its store still starts on a 64-byte line of y (row origins pulled back as in the
// other kernels).  The overlap is read again by the neighbouring strip's workgroup, which is what keeps the kernel
// from a plain copy's rate in this launch shape (0.70 ms against 0.635 per 2 GiB at 16 elements of overlap, 0.73
// at 32, 0.84-0.89 at 64): it is used where that still beats the scan kernel's LDS passes.

#include "sws_internal.h"

namespace sws {

namespace {

__device__ __forceinline__ float from_lane(float v, int byte_addr)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(byte_addr, __builtin_bit_cast(int, v)));
}

// R = (w - 1) mod 4: the element of lane L + q0 at which output 4L's window ends (q0 = (w - 1) / 4).
template <int OP, int R>
__global__ __launch_bounds__(kWave) void slide_reg_kernel(const float *__restrict__ x, float *__restrict__ y, int len,
                                                          int lo, int w, float scale, int n_out, int tiles_per_row,
                                                          int64_t n_tiles, int remap)
{
    using O = Op<OP>;
    const int64_t gt = remap ? xcd_unit(n_tiles) : (int64_t)blockIdx.x;
    if (gt < 0 || gt >= n_tiles) return;
    const int lane = threadIdx.x;
    const int64_t r = gt / tiles_per_row;
    const int t = (int)(gt - r * tiles_per_row);
    const float *xr = x + r * (int64_t)len;
    float *yr = y + r * (int64_t)lo;
    // strip origins pulled back so that every store starts on a 64-byte line of y
    const int q = t * n_out - (int)((r * lo) & 15) + 4 * lane;     // first of this lane's four elements / outputs
    float v[4];
    if (q >= 0 && q + 4 <= len) {
        // streamed (measured on 2 GiB, w = 16: 0.700-0.706 ms against 0.72 with plain loads; keeping only the
        // lines that the next strip reads again in the cache costs a second load instruction: 0.71-0.72)
        const v4f g = __builtin_nontemporal_load((const v4f_u *)(xr + q));
        v[0] = g.x; v[1] = g.y; v[2] = g.z; v[3] = g.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (q + e >= 0 && q + e < len) ? xr[q + e] : O::id();
    }
    // ---- inside the lane
    float P[4], F[4];
    P[0] = v[0];
#pragma unroll
    for (int e = 1; e < 4; ++e) P[e] = O::f(P[e - 1], v[e]);
    F[3] = v[3];
#pragma unroll
    for (int e = 2; e >= 0; --e) F[e] = O::f(v[e], F[e + 1]);
    // ---- whole lanes L + 1 .. L + n (n = q0 - 1 for the outputs that end in lane L + q0)
    const int q0 = (w - 1) >> 2, n = q0 - 1;         // w >= 5: q0 >= 1
    const int la = lane << 2;                        // ds_bpermute addresses are lane * 4; wrapped lanes feed no stored output
    float run[4];                                    // run[k]: T of lanes L .. L + 2^k - 1
    run[0] = P[3];
#pragma unroll
    for (int k = 1; k < 4; ++k)
        run[k] = (n >> k) ? O::f(run[k - 1], from_lane(run[k - 1], (la + (4 << (k - 1))) & 255)) : run[k - 1];
    float M = O::id();
    bool have = false;
    int off = 1;                                     // next lane of the run, relative to L
#pragma unroll
    for (int k = 3; k >= 0; --k) {
        if (n & (1 << k)) {                          // wave-uniform
            const float part = from_lane(run[k], (la + 4 * off) & 255);
            M = have ? O::f(M, part) : part;
            have = true;
            off += 1 << k;
        }
    }
    // ---- the heads: outputs j <= 3 - R end in lane L + q0 at element R + j, the others in lane L + q0 + 1
    // at element R + j - 4, after the whole of lane L + q0
    const int a0 = (la + 4 * q0) & 255, a1 = (la + 4 * q0 + 4) & 255;
    float o[4];
    float Tq = 0.0f;
    if (R > 0) Tq = from_lane(P[3], a0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float acc = F[j];
        if (have) acc = O::f(acc, M);
        if (R + j <= 3) {
            acc = O::f(acc, from_lane(P[R + j], a0));
        } else {
            acc = O::f(acc, Tq);
            acc = O::f(acc, from_lane(P[R + j - 4], a1));
        }
        o[j] = (OP == SWS_OP_ADD) ? acc * scale : acc;
    }
    // ---- out: the lanes whose windows stay inside the strip
    if (4 * lane >= n_out || q >= lo || q + 4 <= 0) return;
    if (q >= 0 && q + 4 <= lo) {
        const v4f g = {o[0], o[1], o[2], o[3]};
        __builtin_nontemporal_store(g, (v4f_u *)(yr + q));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (q + e >= 0 && q + e < lo) yr[q + e] = o[e];
    }
}

template <int OP>
hipError_t launch_reg(const float *x, float *y, int64_t rows, int len, int lo, int w, float scale, hipStream_t s)
{
    const int reach = (w - 1 + 15) & ~15;            // overlap of neighbouring strips: a multiple of 64 bytes
    const int n_out = 256 - reach;
    const int tiles_per_row = (lo + max_origin_shift(lo, 16) + n_out - 1) / n_out;
    const int64_t n_tiles = rows * tiles_per_row;
    // neighbouring strips share their overlap: each XCD (one L2) takes a contiguous range of them, unless
    // slide_chunk bit 8 asks for launch order
    const int remap = (g_opt.slide_chunk & 8) ? 0 : 1;
    const int64_t grid = remap ? xcd_grid(n_tiles) : n_tiles;
    if (grid > 2147483647LL) return kNotTaken;
#define SWS_REG(R_)                                                                                         \
    case R_:                                                                                                \
        hipLaunchKernelGGL((slide_reg_kernel<OP, R_>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, len, lo, w, scale, \
                           n_out, tiles_per_row, n_tiles, remap);                                          \
        break
    switch ((w - 1) & 3) {
        SWS_REG(0); SWS_REG(1); SWS_REG(2);
    default:
        hipLaunchKernelGGL((slide_reg_kernel<OP, 3>), dim3((unsigned)grid), dim3(kWave), 0, s, x, y, len, lo, w, scale,
                           n_out, tiles_per_row, n_tiles, remap);
        break;
    }
#undef SWS_REG
    return hipGetLastError();
}

}  // namespace

int slide1d_reg_min_w() { return 5; }
int slide1d_reg_max_w() { return 65; }

// Plain rows (no boundary rule), 5 <= w <= 65.  kNotTaken: a grid beyond the launch limit.
hipError_t launch_slide1d_reg(int op, const float *x, float *y, int64_t rows, int len, int lo, int w, float scale,
                              hipStream_t s)
{
    if (w < slide1d_reg_min_w() || w > slide1d_reg_max_w() || lo < 1) return kNotTaken;
    switch (op) {
    case SWS_OP_ADD: return launch_reg<SWS_OP_ADD>(x, y, rows, len, lo, w, scale, s);
    case SWS_OP_MAX: return launch_reg<SWS_OP_MAX>(x, y, rows, len, lo, w, scale, s);
    default: return launch_reg<SWS_OP_MIN>(x, y, rows, len, lo, w, scale, s);
    }
}

}  // namespace sws
