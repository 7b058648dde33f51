// Backward passes of ISGMR (Alg. 3) and TRWP (Alg. 4): replay of the stored indices p, q
// in reverse scanline order.
//
// One wavefront walks one scanline from its last node back to the node after its first;
// lanes own labels (lambda = lane + 64*s).  Per node: reparametrisation backward through q
// (Eq. supp-isgmr-back-norm), edge-weight gradient (Eq. supp-gradient-edge), V gradient
// (Eq. supp-gradient-smoothness) into an accumulator private to the wavefront, and the
// index scatter s(mu) = sum_{lambda : p(lambda) = mu} g(lambda) through a wavefront-private
// LDS vector.  What the same direction passes on to node i-r stays in registers.
//
// Precision: tensors in memory are float; the chain a scanline carries from node to node
// (message gradient, its label sum, the scatter sums) and the V-gradient accumulators are
// kept in double, so that rounding does not build up along a scanline.  On this chip
// double adds issue at the same rate as unpacked float adds.
//
// ISGMR sweeps all directions in one launch, so cross-direction sums are not formed here:
// the sweep writes s per (direction, node) and mrf_isgmr_bwd_combine adds them up in a
// fixed order.  TRWP sweeps one direction per launch; every (node, label) is touched by
// exactly one wavefront of the launch, so its read-modify-writes need no atomics.
#pragma once

#include "mrfmp_device.h"

struct MrfBwdParams {
    MrfGeom g;
    int algo;                              // 0 = ISGMR, 1 = TRWP
    int r_first, r_count;
    long long blk_begin[MRF_MAXR + 1];     // prefix sums of B*nscan over the launch's directions
    long long total_scanlines;
    const float *V, *w;
    float w_scalar;
    const uint8_t *p, *q;                  // [R][N][L], [R][N] of this iteration
    const float *gin;                      // ISGMR: grad m-hat, direction r at gin + r*gin_stride
    long long gin_stride;                  //        (0 when every direction starts from grad c)
    float *S;                              // ISGMR: [R][N][L] per-direction scatter result
    float *G;                              // TRWP : [R][N][L] grad m, updated in place
    float *gunary;                         // TRWP : [N][L] grad theta_i, updated in place
    float *gw;                             // [R][N] or NULL, accumulated over iterations
    double *gV;                            // [slots][L][L] or NULL, one slot per wavefront
    float rho[MRF_MAXR];
};

#define MRF_BWD_WAVES 4   // wavefronts (= scanlines in flight) per workgroup

template <int LP>
__global__ void __launch_bounds__(64 * MRF_BWD_WAVES) mrf_bwd_sweep(const MrfBwdParams P)
{
    __shared__ double sbuf_all[MRF_BWD_WAVES][64 * LP];
    const int L = P.g.L, R = P.g.R;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    double *sbuf = sbuf_all[wv];
    const long long slot = (long long)blockIdx.x * MRF_BWD_WAVES + wv;
    const long long nslots = (long long)gridDim.x * MRF_BWD_WAVES;
    const long long N = P.g.N;
    const bool trwp = P.algo != 0;
    double *gVs = P.gV ? P.gV + (size_t)slot * L * L : nullptr;

    for (long long sl = slot; sl < P.total_scanlines; sl += nslots) {
        int ri = 0;
        while (ri + 1 < P.r_count && sl >= P.blk_begin[ri + 1]) ++ri;
        const int r = P.r_first + ri;
        const long long local = sl - P.blk_begin[ri];
        const int nsc = P.g.nscan[r];
        const int b = (int)(local / nsc);
        const long long t = local - (long long)b * nsc;
        const int dh = P.g.dh[r], dw = P.g.dw[r], rm = P.g.opp[r];
        int y0, x0, len;
        mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
        const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
        const long long nstep = (long long)dh * P.g.W + dw;
        const double rho = (double)P.rho[r];
        const float *gin = trwp ? P.G + (size_t)r * N * L : P.gin + (size_t)r * P.gin_stride;

        // the last node of the scanline has no successor in direction r
        if (!trwp) {
            const long long last = head + (long long)(len - 1) * nstep;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) P.S[((size_t)r * N + last) * L + lam] = 0.0f;
            }
        }

        double carry[LP];   // what node i+r of this direction passed back to node i
#pragma unroll
        for (int s = 0; s < LP; ++s) carry[s] = 0.0;

        for (int n = len - 1; n >= 1; --n) {
            const long long i = head + (long long)n * nstep;
            const long long j = i - nstep;
            double g[LP];
            int pv[LP];
            double part = 0.0;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                g[s] = 0.0;
                pv[s] = 0;
                if (lam < L) {
                    g[s] = (double)gin[(size_t)i * L + lam] + carry[s];
                    int pp = P.p[((size_t)r * N + i) * L + lam];
                    pv[s] = pp < L ? pp : L - 1;
                    if (trwp) P.G[((size_t)r * N + i) * L + lam] = 0.0f;   // zero-out (Alg. 4)
                }
                part += g[s];
            }
            // back Eq. isgmr-norm: g(q) -= sum_lambda g(lambda)
            const double tot = mrf_wave_sum_f64(part);
            int qv = P.q[(size_t)r * N + i];
            qv = qv < L ? qv : L - 1;
#pragma unroll
            for (int s = 0; s < LP; ++s)
                if (lane + 64 * s == qv) g[s] = g[s] - tot;

            const double wgt = (double)(P.w ? P.w[(size_t)r * N + i] : P.w_scalar);
            if (P.gw) {
                double acc = 0.0;
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    if (lam < L) acc += g[s] * (double)P.V[(size_t)pv[s] * L + lam];
                }
                acc = mrf_wave_sum_f64(acc);
                if (lane == 0) P.gw[(size_t)r * N + i] = (float)((double)P.gw[(size_t)r * N + i] + acc);
            }
            if (gVs) {
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    if (lam < L) gVs[(size_t)pv[s] * L + lam] += wgt * g[s];
                }
            }

            // index scatter through LDS: s(mu) = sum over lambda with p(lambda) = mu
#pragma unroll
            for (int s = 0; s < LP; ++s) sbuf[lane + 64 * s] = 0.0;
            mrf_wave_lds_fence();
#pragma unroll
            for (int s = 0; s < LP; ++s)
                if (lane + 64 * s < L)
                    __hip_atomic_fetch_add(&sbuf[pv[s]], g[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            mrf_wave_lds_fence();
            double sv[LP];
#pragma unroll
            for (int s = 0; s < LP; ++s) sv[s] = sbuf[lane + 64 * s];
            mrf_wave_lds_fence();

            if (!trwp) {
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    if (lam < L) P.S[((size_t)r * N + j) * L + lam] = (float)sv[s];
                    carry[s] = sv[s];
                }
            } else {
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    const double rs = rho * sv[s];
                    if (lam < L) {
                        const size_t e = (size_t)j * L + lam;
                        P.gunary[e] = (float)((double)P.gunary[e] + rs);
                        for (int d = 0; d < R; ++d) {
                            if (d == r) continue;
                            float *gd = P.G + (size_t)d * N * L;
                            double v = (double)gd[e] + rs;
                            if (d == rm) v = v - sv[s];
                            gd[e] = (float)v;
                        }
                    }
                    carry[s] = rs;
                }
            }
        }
        if (trwp) {
            // gradient that reached the first node belongs to a constant message: dropped
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) P.G[((size_t)r * N + head) * L + lam] = 0.0f;
            }
        }
    }
}

// ISGMR, after the sweeps of iteration k: grad theta_i += sum_r s^r_i, and the gradient of
// m^d (= m-hat^d of iteration k-1) is sum over r not in {d, d-} of s^r_i.
struct MrfCombineParams {
    long long NL;            // N*L
    int R;
    int opp[MRF_MAXR];
    const float *S;          // [R][N][L]
    const float *gc;         // grad c, read when first != 0
    float *gunary;           // [N][L]
    float *ghat;             // [R][N][L] out (next iteration's grad m-hat), NULL on the last
    int first;               // first processed iteration: grad theta starts from grad c
};

__global__ void __launch_bounds__(256) mrf_isgmr_bwd_combine(const MrfCombineParams P)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < P.NL; e += stride) {
        double tot = (double)(P.first ? P.gc[e] : P.gunary[e]);
        for (int r = 0; r < P.R; ++r) tot = tot + (double)P.S[(size_t)r * P.NL + e];
        P.gunary[e] = (float)tot;
        if (P.ghat) {
            for (int d = 0; d < P.R; ++d) {
                double v = 0.0;
                for (int r = 0; r < P.R; ++r)
                    if (r != d && r != P.opp[d]) v = v + (double)P.S[(size_t)r * P.NL + e];
                P.ghat[(size_t)d * P.NL + e] = (float)v;
            }
        }
    }
}

// dst[e] = sum over slots of src[slot][e], slots in ascending order
__global__ void __launch_bounds__(256) mrf_reduce_slots(const double *src, float *dst, long long n, long long slots)
{
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    double v = 0.0;
    for (long long s = 0; s < slots; ++s) v = v + src[(size_t)s * n + e];
    dst[e] = (float)v;
}

__global__ void __launch_bounds__(256) mrf_fill_f64(double *dst, long long n, double val)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) dst[e] = val;
}

__global__ void __launch_bounds__(256) mrf_fill_f32(float *dst, long long n, float val)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) dst[e] = val;
}

// dst[c][e] = src[e] for c < copies  (back Eq. isgmr-aggregation: every direction's message
// gradient and the unary gradient start from grad c)
__global__ void __launch_bounds__(256) mrf_broadcast_f32(const float *src, float *dst, long long n, int copies)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) {
        const float v = src[e];
        for (int c = 0; c < copies; ++c) dst[(size_t)c * n + e] = v;
    }
}
