// Shared declarations of the libmrfmp kernels: grid / scanline geometry and wavefront
// helpers for gfx950 (64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#ifdef __HIPCC__
#include <utility>
#endif

#define MRF_WAVE 64
#define MRF_MAXR 16

// Grid, direction set and scanline bookkeeping, passed to kernels by value.
struct MrfGeom {
    int B, H, W, L, R;
    int dh[MRF_MAXR], dw[MRF_MAXR];
    int opp[MRF_MAXR];      // index of r^- in the direction set, or -1
    int nscan[MRF_MAXR];    // scanlines of direction r in one image
    long long N;            // B*H*W nodes
};

// Scanlines of direction (dh,dw) are the maximal in-grid chains i, i+r, i+2r, ...; each is one
// tree of the tree parallelisation and starts at its first node (Sec. 3.5, Appendix C).
// First nodes are the nodes whose
// predecessor is off the grid: the |dh| boundary rows on the side the sweep starts from,
// then |dw| boundary columns in every other row.  For |dh| = 1 the count is
// W + (H-1)|dw| (Eq. supp-wide).
__host__ __device__ inline int mrf_iabs(int v) { return v < 0 ? -v : v; }
__host__ __device__ inline int mrf_imin(int a, int b) { return a < b ? a : b; }

__host__ __device__ inline long long mrf_geom_scanlines(int H, int W, int dh, int dw)
{
    int adh = mrf_imin(mrf_iabs(dh), H), adw = mrf_imin(mrf_iabs(dw), W);
    return (long long)adh * W + (long long)(H - adh) * adw;
}

__host__ __device__ inline void mrf_geom_head(int H, int W, int dh, int dw, long long t,
                                              int &y0, int &x0, int &len)
{
    int adh = mrf_imin(mrf_iabs(dh), H), adw = mrf_imin(mrf_iabs(dw), W);
    long long band = (long long)adh * W;
    if (t < band) {
        int yy = (int)(t / W);
        x0 = (int)(t - (long long)yy * W);
        y0 = dh > 0 ? yy : H - adh + yy;
    } else {
        long long tt = t - band;
        int ry = (int)(tt / adw);
        int cx = (int)(tt - (long long)ry * adw);
        y0 = dh > 0 ? adh + ry : ry;
        x0 = dw > 0 ? cx : W - adw + cx;
    }
    int sy = dh > 0 ? (H - 1 - y0) / dh : (dh < 0 ? y0 / (-dh) : INT_MAX);
    int sx = dw > 0 ? (W - 1 - x0) / dw : (dw < 0 ? x0 / (-dw) : INT_MAX);
    len = 1 + mrf_imin(sy, sx);
}

#ifdef __HIPCC__
// ---- wavefront helpers (gfx950: 64 lanes, DPP row = 16 lanes) -------------------------
// DPP controls: quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_half_mirror = 0x141,
// row_mirror = 0x140.  After the four steps every lane holds the reduction of its row.
// (These four controls are permutations inside a row: every lane has a valid source, so no
// "old" value has to be prepared for the destination.)
template <int CTRL>
__device__ inline float mrf_dpp_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <int CTRL>
__device__ inline double mrf_dpp_f64(double v)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_mov_dpp((int)(b & 0xffffffffLL), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_mov_dpp((int)(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}

__device__ inline float mrf_readlane_f32(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

__device__ inline double mrf_readlane_f64(double v, int lane)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffLL), lane);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}

// Plain hardware minimum.  Inputs here are never NaN; fminf() would first canonicalise
// every operand that comes from memory (one extra instruction each).
__device__ inline float mrf_min(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

__device__ inline float mrf_min3(float a, float b, float c)
{
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// ---- running (minimum, lowest argmin) without wait states --------------------------------------
// On this chip a vector instruction that reads a lane mask (v_cndmask) must sit at least two vector
// instructions behind the compare that wrote the mask; left to itself the compiler routes every
// compare through VCC and pays an s_nop per candidate.  The blocks below keep G independent
// (best, index) chains in flight: all compares first, each into a scalar register pair of its own,
// then the minima, then the index selects, so that every select is 2 G - 1 >= 3 instructions behind
// its compare.  best' = min(best, d), index' = d < best ? K : index: strict '<' keeps the lowest
// index when candidates arrive in ascending order.  Inputs are never NaN.
template <int K>
__device__ inline void mrf_argmin_step(float (&b)[4], int (&i)[4], const float (&d)[4])
{
    unsigned long long m0, m1, m2, m3;
    asm("v_cmp_lt_f32_e64 %8, %12, %0\n\t"
        "v_cmp_lt_f32_e64 %9, %13, %1\n\t"
        "v_cmp_lt_f32_e64 %10, %14, %2\n\t"
        "v_cmp_lt_f32_e64 %11, %15, %3\n\t"
        "v_min_f32_e32 %0, %0, %12\n\t"
        "v_min_f32_e32 %1, %1, %13\n\t"
        "v_min_f32_e32 %2, %2, %14\n\t"
        "v_min_f32_e32 %3, %3, %15\n\t"
        "v_cndmask_b32_e64 %4, %4, %16, %8\n\t"
        "v_cndmask_b32_e64 %5, %5, %16, %9\n\t"
        "v_cndmask_b32_e64 %6, %6, %16, %10\n\t"
        "v_cndmask_b32_e64 %7, %7, %16, %11"
        : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(i[0]), "+v"(i[1]), "+v"(i[2]), "+v"(i[3]),
          "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3)
        : "v"(d[0]), "v"(d[1]), "v"(d[2]), "v"(d[3]), "n"(K));
}

template <int K>
__device__ inline void mrf_argmin_step(float (&b)[3], int (&i)[3], const float (&d)[3])
{
    unsigned long long m0, m1, m2;
    asm("v_cmp_lt_f32_e64 %6, %9, %0\n\t"
        "v_cmp_lt_f32_e64 %7, %10, %1\n\t"
        "v_cmp_lt_f32_e64 %8, %11, %2\n\t"
        "v_min_f32_e32 %0, %0, %9\n\t"
        "v_min_f32_e32 %1, %1, %10\n\t"
        "v_min_f32_e32 %2, %2, %11\n\t"
        "v_cndmask_b32_e64 %3, %3, %12, %6\n\t"
        "v_cndmask_b32_e64 %4, %4, %12, %7\n\t"
        "v_cndmask_b32_e64 %5, %5, %12, %8"
        : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(i[0]), "+v"(i[1]), "+v"(i[2]), "=&s"(m0), "=&s"(m1), "=&s"(m2)
        : "v"(d[0]), "v"(d[1]), "v"(d[2]), "n"(K));
}

template <int K>
__device__ inline void mrf_argmin_step(float (&b)[2], int (&i)[2], const float (&d)[2])
{
    unsigned long long m0, m1;
    asm("v_cmp_lt_f32_e64 %4, %6, %0\n\t"
        "v_cmp_lt_f32_e64 %5, %7, %1\n\t"
        "v_min_f32_e32 %0, %0, %6\n\t"
        "v_min_f32_e32 %1, %1, %7\n\t"
        "v_cndmask_b32_e64 %2, %2, %8, %4\n\t"
        "v_cndmask_b32_e64 %3, %3, %8, %5"
        : "+v"(b[0]), "+v"(b[1]), "+v"(i[0]), "+v"(i[1]), "=&s"(m0), "=&s"(m1)
        : "v"(d[0]), "v"(d[1]), "n"(K));
}

// one chain: two candidates in a row (indices K and K + 1), the second compared with the minimum
// that includes the first
template <int K>
__device__ inline void mrf_argmin_step2(float &b, int &i, float d0, float d1)
{
    unsigned long long m0, m1;
    asm("v_cmp_lt_f32_e64 %2, %4, %0\n\t"
        "v_min_f32_e32 %0, %0, %4\n\t"
        "v_cmp_lt_f32_e64 %3, %5, %0\n\t"
        "v_min_f32_e32 %0, %0, %5\n\t"
        "v_cndmask_b32_e64 %1, %1, %6, %2\n\t"
        "v_cndmask_b32_e64 %1, %1, %7, %3"
        : "+v"(b), "+v"(i), "=&s"(m0), "=&s"(m1)
        : "v"(d0), "v"(d1), "n"(K), "n"(K + 1));
}

// the same for candidates that bring their index in a register (merging partial results)
template <int G>
__device__ inline void mrf_argmin_merge(float (&b)[G], int (&i)[G], const float (&d)[G], const int (&k)[G])
{
    static_assert(G >= 1 && G <= 4, "chains per block");
    if constexpr (G == 4) {
        unsigned long long m0, m1, m2, m3;
        asm("v_cmp_lt_f32_e64 %8, %12, %0\n\t"
            "v_cmp_lt_f32_e64 %9, %13, %1\n\t"
            "v_cmp_lt_f32_e64 %10, %14, %2\n\t"
            "v_cmp_lt_f32_e64 %11, %15, %3\n\t"
            "v_min_f32_e32 %0, %0, %12\n\t"
            "v_min_f32_e32 %1, %1, %13\n\t"
            "v_min_f32_e32 %2, %2, %14\n\t"
            "v_min_f32_e32 %3, %3, %15\n\t"
            "v_cndmask_b32_e64 %4, %4, %16, %8\n\t"
            "v_cndmask_b32_e64 %5, %5, %17, %9\n\t"
            "v_cndmask_b32_e64 %6, %6, %18, %10\n\t"
            "v_cndmask_b32_e64 %7, %7, %19, %11"
            : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(i[0]), "+v"(i[1]), "+v"(i[2]), "+v"(i[3]),
              "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3)
            : "v"(d[0]), "v"(d[1]), "v"(d[2]), "v"(d[3]), "v"(k[0]), "v"(k[1]), "v"(k[2]), "v"(k[3]));
    } else if constexpr (G == 3) {
        unsigned long long m0, m1, m2;
        asm("v_cmp_lt_f32_e64 %6, %9, %0\n\t"
            "v_cmp_lt_f32_e64 %7, %10, %1\n\t"
            "v_cmp_lt_f32_e64 %8, %11, %2\n\t"
            "v_min_f32_e32 %0, %0, %9\n\t"
            "v_min_f32_e32 %1, %1, %10\n\t"
            "v_min_f32_e32 %2, %2, %11\n\t"
            "v_cndmask_b32_e64 %3, %3, %12, %6\n\t"
            "v_cndmask_b32_e64 %4, %4, %13, %7\n\t"
            "v_cndmask_b32_e64 %5, %5, %14, %8"
            : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(i[0]), "+v"(i[1]), "+v"(i[2]), "=&s"(m0), "=&s"(m1), "=&s"(m2)
            : "v"(d[0]), "v"(d[1]), "v"(d[2]), "v"(k[0]), "v"(k[1]), "v"(k[2]));
    } else if constexpr (G == 2) {
        unsigned long long m0, m1;
        asm("v_cmp_lt_f32_e64 %4, %6, %0\n\t"
            "v_cmp_lt_f32_e64 %5, %7, %1\n\t"
            "v_min_f32_e32 %0, %0, %6\n\t"
            "v_min_f32_e32 %1, %1, %7\n\t"
            "v_cndmask_b32_e64 %2, %2, %8, %4\n\t"
            "v_cndmask_b32_e64 %3, %3, %9, %5"
            : "+v"(b[0]), "+v"(b[1]), "+v"(i[0]), "+v"(i[1]), "=&s"(m0), "=&s"(m1)
            : "v"(d[0]), "v"(d[1]), "v"(k[0]), "v"(k[1]));
    } else {
        if (d[0] < b[0]) { b[0] = d[0]; i[0] = k[0]; }
    }
}

// lowest index among four candidates K .. K + 3 that equal `best`, else `i` unchanged: the four
// compares first, then the selects from the highest index down (the lowest one lands last)
template <int K>
__device__ inline void mrf_first_equal4(int &i, float best, float d0, float d1, float d2, float d3)
{
    unsigned long long m0, m1, m2, m3;
    asm("v_cmp_eq_f32_e64 %4, %6, %5\n\t"
        "v_cmp_eq_f32_e64 %3, %7, %5\n\t"
        "v_cmp_eq_f32_e64 %2, %8, %5\n\t"
        "v_cmp_eq_f32_e64 %1, %9, %5\n\t"
        "v_cndmask_b32_e64 %0, %0, %10, %4\n\t"
        "v_cndmask_b32_e64 %0, %0, %11, %3\n\t"
        "v_cndmask_b32_e64 %0, %0, %12, %2\n\t"
        "v_cndmask_b32_e64 %0, %0, %13, %1"
        : "+v"(i), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3)
        : "v"(best), "v"(d3), "v"(d2), "v"(d1), "v"(d0), "n"(K + 3), "n"(K + 2), "n"(K + 1), "n"(K));
}

// compile-time loop: f(std::integral_constant<int, 0>), ..., f(std::integral_constant<int, N - 1>)
template <class F, int... I>
__device__ inline void mrf_static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ inline void mrf_static_for(F &&f)
{
    mrf_static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// minimum over the 64 lanes, returned to every lane (wave-uniform).
// Six DPP minima in place: within quads, within half rows, within rows of 16, then the last
// lane of rows 0 and 2 into rows 1 and 3, then the last lane of row 1 into rows 2 and 3; lane 63
// ends up with the minimum of all.  Written out because the compiler's own sequence spends
// four instructions per stage (move, wait, DPP move, min).  Every DPP read of a register that
// a vector instruction has just written needs two wait states (the s_nop 1 before each).
// All 64 lanes must be active.
__device__ inline float mrf_wave_min(float v)
{
    float r;
    asm("s_nop 1\n\t"
        "v_min_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %1, %1, %1 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_readlane_b32 %0, %1, 63"
        : "=s"(r), "+v"(v));
    return r;
}

// sum over the 64 lanes in a fixed tree order, returned to every lane
__device__ inline double mrf_wave_sum_f64(double v)
{
    v += mrf_dpp_f64<0xB1>(v);
    v += mrf_dpp_f64<0x4E>(v);
    v += mrf_dpp_f64<0x141>(v);
    v += mrf_dpp_f64<0x140>(v);
    const double r0 = mrf_readlane_f64(v, 0), r1 = mrf_readlane_f64(v, 16);
    const double r2 = mrf_readlane_f64(v, 32), r3 = mrf_readlane_f64(v, 48);
    return (r0 + r1) + (r2 + r3);
}

// v[lane ^ 16] + v[lane] and v[lane ^ 32] + v[lane]: the swap instructions exchange the odd rows (upper half)
// of their first operand with the even rows (lower half) of their second, so two copies of v come back as the
// two terms
__device__ inline double mrf_add_xor16_f64(double v)
{
    const long long b = __builtin_bit_cast(long long, v);
    const unsigned lo = (unsigned)(b & 0xffffffffLL), hi = (unsigned)(b >> 32);
    const auto l = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto h = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __builtin_bit_cast(double, ((long long)h[0] << 32) | (long long)l[0]) +
           __builtin_bit_cast(double, ((long long)h[1] << 32) | (long long)l[1]);
}

__device__ inline double mrf_add_xor32_f64(double v)
{
    const long long b = __builtin_bit_cast(long long, v);
    const unsigned lo = (unsigned)(b & 0xffffffffLL), hi = (unsigned)(b >> 32);
    const auto l = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto h = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __builtin_bit_cast(double, ((long long)h[0] << 32) | (long long)l[0]) +
           __builtin_bit_cast(double, ((long long)h[1] << 32) | (long long)l[1]);
}

// Sums of three doubles over the 64 lanes in one tree (fixed order), returned to every lane.  The first
// two levels fold the three operands into one register: after them a lane holds the sum over its group of
// four lanes of a (lane & 3 == 0), of b (== 1) or of c (== 2, 3); the remaining four levels pair lanes of
// equal lane & 3.  About 40 vector instructions against 23 for each sum taken alone.
__device__ inline void mrf_wave_sum3_f64(double a, double b, double c, double &sa, double &sb, double &sc)
{
    const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const bool odd = lane & 1, high = lane & 2;
    double keep = odd ? b : a, give = odd ? a : b;
    double r = keep + mrf_dpp_f64<0xB1>(give);            // lane ^ 1
    const double c1 = c + mrf_dpp_f64<0xB1>(c);
    keep = high ? c1 : r;
    give = high ? r : c1;
    r = keep + mrf_dpp_f64<0x4E>(give);                   // lane ^ 2
    r += mrf_dpp_f64<0x124>(r);                           // row_ror:4
    r += mrf_dpp_f64<0x128>(r);                           // row_ror:8
    r = mrf_add_xor16_f64(r);
    r = mrf_add_xor32_f64(r);
    sa = mrf_readlane_f64(r, 0);
    sb = mrf_readlane_f64(r, 1);
    sc = mrf_readlane_f64(r, 2);
}

// Three segments of 21 lanes (lanes 0-20, 21-41, 42-62; lane 63 idle) do not line up with the DPP
// rows of 16.  Call the lanes of a row that belong to the segment that began in an earlier row its
// lower part, the others its upper part (row 0 is all upper): segment s is the upper part of row s
// plus the lower part of row s + 1.  Two row reductions (upper lanes only, lower lanes only), one
// row_bcast:15 that brings the previous row's upper minimum to the lower lanes and completes the
// segment minimum there, and one lane permutation that hands it back to the upper lanes of the
// row before.
__device__ inline bool mrf_seg21_upper(int lane)
{
    return lane < 16 || (lane >= 21 && lane < 32) || (lane >= 42 && lane < 48) || lane == 63;
}

// Orders this wavefront's LDS writes before its later LDS reads by other lanes (lanes of
// one wavefront run in lock step; only the compiler and the LDS queue need telling).
__device__ inline void mrf_wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- bounded waits --------------------------------------------------------------------------------
// Wavefronts of one workgroup that hand nodes to each other through LDS rings wait on counters
// that only grow.  The workgroup notes a deadline (constant-rate clock, 100 MHz) in LDS when it
// starts.  Only a wait that finds its condition unmet looks at the clock, so the wavefronts carry
// nothing for this in registers and the path of a wait that need not wait is untouched.  Past the
// deadline the waiting wavefront raises the launch's fault word in global memory (read by the host
// once the stream has drained) and ends on the spot; whoever waits for it follows.  A slip in the
// ring logic thus ends as an error code, not as a launch that never returns.
struct MrfWaitBlock {
    unsigned long long deadline;     // s_memrealtime ticks
    int *fault;
};

__device__ inline void mrf_wait_init(MrfWaitBlock *w, int *fault, int budget_us)   // one thread, before the first barrier
{
    w->deadline = __builtin_amdgcn_s_memrealtime() + (unsigned long long)budget_us * 100ull;
    w->fault = fault;
}

// Raises the fault word and ends the wavefront here.  Written as one opaque block of instructions,
// not as a store and the compiler's "end of program": the compiler then sees neither a second way
// out of the loops that wait nor anything that touches memory there, and the code it lays out for
// the case that nobody has to wait stays as it is without the deadline (with a visible exit the
// straight path of every wait picked up taken branches: 15 % on the launches that are bound by the
// latency of one wavefront).
__device__ inline void mrf_fault_and_end(int *fault)
{
    const int one = 1;
    asm volatile("global_store_dword %0, %1, off\n\ts_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_endpgm" : : "v"(fault), "v"(one));
}

// The condition of a wait was found unmet: end this wavefront if the deadline has passed.
__device__ inline void mrf_wait_check(const MrfWaitBlock *w)
{
    if (__builtin_expect(__builtin_amdgcn_s_memrealtime() > w->deadline, 0)) mrf_fault_and_end(w->fault);
}

// One turn of such a wait: sleep a little, the caller looks again.  The clock is looked at on the
// 8th turn of a wait and every 64 turns from there (`turn` is a counter local to the wait): the
// short waits of a pipeline that is running never touch it, and the time between two looks at the
// awaited counter stays what it is without the deadline.
__device__ inline void mrf_wait_turn(const MrfWaitBlock *w, int &turn)
{
    if ((++turn & 63) == 8) mrf_wait_check(w);
    __builtin_amdgcn_s_sleep(1);
}

// A zero the compiler cannot see through: keeps wave-uniform addresses in vector loads, so
// that they queue behind the other prefetches instead of going through the scalar cache.
__device__ inline int mrf_opaque_zero()
{
    int z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

// The same for floats: adding it to a wave-uniform value keeps that value in a vector
// register.  Kernels with many uniform constants (flags, small tables) otherwise run out of
// scalar registers and pay a v_readlane for every use of a spilled one.
__device__ inline float mrf_opaque_zero_f()
{
    float z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

// Workgroup barrier that orders LDS traffic only: global loads issued as prefetch stay in
// flight across it (a full __syncthreads would wait for them).
__device__ inline void mrf_block_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
#endif
