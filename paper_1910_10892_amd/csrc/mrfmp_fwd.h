// Forward sweeps of ISGMR (Alg. 1) and TRWP (Alg. 2) and the final aggregation
// (Eq. isgmr-aggregation, Eq. disp), hand-written for gfx950.
//
// Dense sweep kernel: one workgroup walks one scanline, node after node.  The L x L
// min-plus of a node is split over the NW wavefronts of the workgroup by source label mu
// (wavefront w owns MCH consecutive mu); lanes own destination labels lambda
// (lambda = lane + 64*s, s < LP).  The wavefront's slice of V lives in registers for the
// whole sweep; h[mu] (the lambda-independent part of the update) is broadcast from LDS.
// Partial minima meet in LDS once per node (one workgroup barrier per node); every
// wavefront then finishes the node redundantly (merge in ascending mu, argmin over
// lambda, reparametrisation), so no second barrier is needed.
#pragma once

#include "mrfmp_device.h"

struct MrfFwdParams {
    MrfGeom g;
    int algo;                              // 0 = ISGMR, 1 = TRWP
    int r_first, r_count;                  // directions swept by this launch
    long long blk_begin[MRF_MAXR + 1];     // prefix sums of B*nscan over those directions
    unsigned live_mask;                    // bit d: message array d holds data (else reads as 0)
    const float *unary, *V, *w;
    float w_scalar;
    const float *m_in;                     // [R][N][L] messages read
    float *m_out;                          // [R][N][L] messages written (TRWP: same array)
    uint8_t *p, *q;                        // [R][N][L], [R][N] of this iteration
    float rho[MRF_MAXR];
    int NW;                                // wavefronts per workgroup = ceil(L / MCH)
};

template <int LP, int MCH>
__global__ void __launch_bounds__(64 * (64 * LP / MCH))
mrf_fwd_sweep(const MrfFwdParams P)
{
    extern __shared__ __align__(16) unsigned char mrf_smem[];
    const int L = P.g.L, NW = P.NW, R = P.g.R;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int LPAD = NW * MCH;
    constexpr int SLOTS = 64 * LP;
    float *hbuf = reinterpret_cast<float *>(mrf_smem) + wv * LPAD;      // private to this wavefront
    float *pval = reinterpret_cast<float *>(mrf_smem) + NW * LPAD;      // [2][NW][SLOTS]
    uint8_t *pidx = reinterpret_cast<uint8_t *>(pval + 2 * NW * SLOTS); // [2][NW][SLOTS]

    // workgroup -> (direction r, image b, scanline t)
    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r], rm = P.g.opp[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const bool trwp = P.algo != 0;
    const float rho = P.rho[r];

    // this wavefront's slice of V: rows mu0 .. mu0+MCH-1, columns = the lane's lambdas
    const int mu0 = wv * MCH;
    float Vr[MCH][LP];
#pragma unroll
    for (int i = 0; i < MCH; ++i)
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int mu = mu0 + i, lam = lane + 64 * s;
            Vr[i][s] = (mu < L && lam < L) ? P.V[(size_t)mu * L + lam] : 0.0f;
        }
    // padding of h beyond L can never win a strict '<'
    for (int i = L + lane; i < LPAD; i += 64) hbuf[i] = INFINITY;

    // first node of the scanline: message 0, p = q = 0
    if (wv == 0) {
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int lam = lane + 64 * s;
            if (lam < L) {
                P.m_out[((size_t)r * N + head) * L + lam] = 0.0f;
                P.p[((size_t)r * N + head) * L + lam] = 0;
            }
        }
        if (lane == 0) P.q[(size_t)r * N + head] = 0;
    }

    float carry[LP];   // normalised message of this direction at the previous node
#pragma unroll
    for (int s = 0; s < LP; ++s) carry[s] = 0.0f;
    int buf = 0;

    for (int n = 1; n < len; ++n) {
        const long long j = head + (long long)(n - 1) * nstep;   // i - r
        const long long i = j + nstep;

        // ---- lambda-independent part h[mu] at node i-r (lane's labels act as mu here) ----
        float a[LP];
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int lam = lane + 64 * s;
            float v = 0.0f;
            if (lam < L) {
                v = P.unary[(size_t)j * L + lam];
                if (!trwp) {
                    // Eq. isgmr: theta_{i-r} + m-hat^r_{i-r} + sum_{d not in {r, r-}} m^d_{i-r}
                    v = v + carry[s];
                    for (int d = 0; d < R; ++d)
                        if (d != r && d != rm && ((P.live_mask >> d) & 1u))
                            v = v + P.m_in[((size_t)d * N + j) * L + lam];
                } else {
                    // Eq. trwp: rho (theta_{i-r} + sum_d m^d_{i-r}) - m^{r-}_{i-r}
                    float mrm = 0.0f;
                    for (int d = 0; d < R; ++d) {
                        float md;
                        if (d == r) md = carry[s];
                        else if ((P.live_mask >> d) & 1u) md = P.m_in[((size_t)d * N + j) * L + lam];
                        else md = 0.0f;
                        v = v + md;
                        if (d == rm) mrm = md;
                    }
                    v = rho * v;
                    if (rm >= 0) v = v - mrm;
                }
            }
            a[s] = v;
        }
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int lam = lane + 64 * s;
            if (lam < L) hbuf[lam] = a[s];
        }
        mrf_wave_lds_fence();

        const float wgt = P.w ? P.w[(size_t)r * N + i] : P.w_scalar;

        // ---- min-plus over this wavefront's mu slice, lowest mu on ties ----
        float best[LP];
        int bidx[LP];
#pragma unroll
        for (int s = 0; s < LP; ++s) { best[s] = INFINITY; bidx[s] = 0; }
#pragma unroll
        for (int i4 = 0; i4 < MCH; i4 += 4) {
            const float4 hv = *reinterpret_cast<const float4 *>(&hbuf[mu0 + i4]);
            const float hq[4] = { hv.x, hv.y, hv.z, hv.w };
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const float dlt = __builtin_fmaf(wgt, Vr[i4 + c][s], hq[c]);
                    if (dlt < best[s]) { best[s] = dlt; bidx[s] = i4 + c; }
                }
        }

        float tv[LP];
        int tp[LP];
        if (NW > 1) {
            float *pv = pval + (size_t)buf * NW * SLOTS;
            uint8_t *pi = pidx + (size_t)buf * NW * SLOTS;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                pv[wv * SLOTS + lane + 64 * s] = best[s];
                pi[wv * SLOTS + lane + 64 * s] = (uint8_t)(mu0 + bidx[s]);
            }
            __syncthreads();
#pragma unroll
            for (int s = 0; s < LP; ++s) { tv[s] = INFINITY; tp[s] = 0; }
            for (int w2 = 0; w2 < NW; ++w2) {
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const float v = pv[w2 * SLOTS + lane + 64 * s];
                    const int ix = pi[w2 * SLOTS + lane + 64 * s];
                    if (v < tv[s]) { tv[s] = v; tp[s] = ix; }
                }
            }
            buf ^= 1;
        } else {
#pragma unroll
            for (int s = 0; s < LP; ++s) { tv[s] = best[s]; tp[s] = bidx[s]; }
        }

        // ---- q = lowest argmin over lambda, reparametrisation (Eq. isgmr-norm) ----
        float mn = INFINITY;
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            if (lane + 64 * s >= L) tv[s] = INFINITY;
            mn = fminf(mn, tv[s]);
        }
        mn = mrf_wave_min(mn);
        int qidx = -1;
        float tq = mn;
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const unsigned long long bal = __ballot(tv[s] == mn);
            if (qidx < 0 && bal != 0ull) {
                const int ql = __ffsll((long long)bal) - 1;
                qidx = 64 * s + ql;
                tq = __shfl(tv[s], ql, MRF_WAVE);
            }
        }
#pragma unroll
        for (int s = 0; s < LP; ++s) carry[s] = tv[s] - tq;

        // ---- outputs of node i (the wavefronts take turns) ----
        if (wv == n % NW) {
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) {
                    P.m_out[((size_t)r * N + i) * L + lam] = carry[s];
                    P.p[((size_t)r * N + i) * L + lam] = (uint8_t)tp[s];
                }
            }
            if (lane == 0) P.q[(size_t)r * N + i] = (uint8_t)qidx;
        }
    }
}

// ---- final costs and labels: c_i = theta_i + sum_r m^r_i (direction order), x_i = argmin ----
struct MrfAggParams {
    long long N;
    int L, R;
    const float *unary, *m;
    float *cost;
    uint8_t *labels;     // may be NULL
};

__global__ void __launch_bounds__(256) mrf_aggregate(const MrfAggParams P)
{
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * (blockDim.x >> 6);
    const int L = P.L;
    for (long long i = wave; i < P.N; i += nwaves) {
        float c[4];
        float mn = INFINITY;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int lam = lane + 64 * s;
            c[s] = INFINITY;
            if (lam < L) {
                float v = P.unary[(size_t)i * L + lam];
                for (int d = 0; d < P.R; ++d) v = v + P.m[((size_t)d * P.N + i) * L + lam];
                c[s] = v;
                P.cost[(size_t)i * L + lam] = v;
            }
            mn = fminf(mn, c[s]);
        }
        if (P.labels) {
            mn = mrf_wave_min(mn);
            int lab = -1;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const unsigned long long bal = __ballot(c[s] == mn);
                if (lab < 0 && bal != 0ull) lab = 64 * s + __ffsll((long long)bal) - 1;
            }
            if (lane == 0) P.labels[i] = (uint8_t)lab;
        }
    }
}
