// Shared declarations of the libmrfmp kernels: grid / scanline geometry and wavefront
// helpers for gfx950 (64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>

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

// Scanlines of direction (dh,dw) are the maximal in-grid chains i, i+r, i+2r, ...
// ("each tree is headed by its first node", Sec. 3.5).  First nodes are the nodes whose
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
// ---- wavefront helpers ---------------------------------------------------------------
__device__ inline float mrf_wave_min(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, MRF_WAVE));
    return v;
}

__device__ inline float mrf_wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, MRF_WAVE);
    return v;
}

__device__ inline double mrf_wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, MRF_WAVE);
    return v;
}

// Orders this wavefront's LDS writes before its later LDS reads by other lanes (lanes of
// one wavefront run in lock step; only the compiler and the LDS queue need telling).
__device__ inline void mrf_wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
#endif
