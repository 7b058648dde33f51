// Backward passes of ISGMR (Alg. 3) and TRWP (Alg. 4): replay of the stored indices p, q
// in reverse scanline order.
//
// One wavefront walks one scanline from its last node back to its first; lanes own labels
// (lambda = lane + 64*s).  Per node: reparametrisation backward through q
// (Eq. supp-isgmr-back-norm), edge-weight gradient (Eq. supp-gradient-edge), V gradient
// (Eq. supp-gradient-smoothness) into an accumulator private to the wavefront, and the
// index scatter s(mu) = sum_{lambda : p(lambda) = mu} g(lambda) through a wavefront-private
// LDS vector.  What the same direction passes on to node i-r stays in registers; nothing
// the sweep reads from memory depends on the previous node, so all of it is prefetched a
// group of D nodes ahead.
//
// A sweep never read-modify-writes message gradients.  It stores s per (direction, node)
// and later sweeps rebuild the gradient of a message from those stores:
//   ISGMR  all directions of an iteration run in one launch; mrf_isgmr_bwd_combine then forms
//          grad theta_i += sum_r s^r_i and grad m^d_i = sum_{r not in {d,d-}} s^r_i.
//   TRWP   directions run one after the other (reverse forward order).  Between two sweeps
//          of direction d every other direction r sweeps exactly once and adds
//          rho_r s^r_i (minus s^r_i if r = d-) to grad m^d_i (Alg. 4 lines 10-11), after
//          which grad m^d is reset; so the sweep of d reads the latest s^r of the other
//          directions and sums them with those coefficients (plus grad c in the first
//          processed iteration).  The sweep of direction 0 also owns grad theta_i.
//
// Precision: tensors in memory are float; the chain a scanline carries from node to node
// (message gradient, its label sum, the scatter sums) and the V-gradient accumulators are
// kept in double, so that rounding does not build up along a scanline.  On this chip
// double adds issue at the same rate as unpacked float adds.
//
// Kernels in this file:
//   mrf_bwd_sweep          one wavefront per scanline (the description above)
//   mrf_bwd_sweep_chain    the node-to-node chain on a wavefront of its own, helper wavefronts
//                          for everything else (launches with few scanlines)
//   mrf_bwd_sweep_split    one wavefront per 64 labels in lock step
//   mrf_bwd_sweep_packed   L <= 32: several scanlines per wavefront
//   mrf_isgmr_bwd_combine  ISGMR's sums over directions between two iterations
//   mrf_reduce_slot_*      fixed-order reduction of the private V-gradient accumulators
// Which sweep a launch gets is host arithmetic on the launch shape (dispatch_bwd).
#pragma once

#include "mrfmp_device.h"

struct MrfBwdParams {
    MrfGeom g;
    int r_first, r_count;
    long long blk_begin[MRF_MAXR + 1];     // prefix sums of B*nscan over the launch's directions
    long long total_scanlines;
    const float *V;
    const float *w;                        // [R][N] edge weights, or one float when w_mul == 0
    int w_mul;
    const uint8_t *p, *q;                  // [R][N][L], [R][N] of this iteration
    // incoming message gradient of direction d at node i = sum_c coefG[d][c] * src_c[i], where
    // src_c = src_base + src_dir[d][c] * src_stride for c < n_src[d]; slot n_src[d] is grad c
    // when use_gc is set
    const float *src_base;
    long long src_stride;
    signed char src_dir[MRF_MAXR][MRF_MAXR];
    signed char n_src[MRF_MAXR];
    float coefG[MRF_MAXR][MRF_MAXR];
    float coefT[MRF_MAXR][MRF_MAXR];       // coefficients of the same sources in grad theta_i
    const float *gc;
    int use_gc;
    float *S;                              // [R][N][L] out: s of direction d at node i-d
    float *gunary;                         // [N][L]
    int unary_dir;                         // direction whose sweep forms grad theta_i, or -1
    int unary_init;                        // grad theta_i is assigned (first iteration) / accumulated
    float *gw;                             // [R][N] or NULL, accumulated over iterations
    double *gV;                            // [slots][L][L] or NULL, one slot per wavefront
    int gv_lds;                            // grad V accumulates in LDS: 1 = a table per wavefront, flushed once per wavefront;
                                           // 2 = one table per workgroup (LDS adds), flushed once into the workgroup's slot
    int v_mode;                            // V for grad w: 0 global, 1 copy in LDS, 2 first row in LDS
    int hot_label;                         // pre-reduce the most popular scatter target (truncated models)
    float carry_scale[MRF_MAXR];           // rho_d (TRWP) or 1 (ISGMR)
    const float *rho_e;                    // [R][N] rho of edge (i-r, i) at node i (TRWP), or NULL: then
                                           // coefG / coefT / carry_scale hold the per-direction values
    float *gE;                             // [R][N][L][L] gradient of per-edge pairwise tables (zeroed by the host,
                                           // accumulated over iterations), or NULL; mrf_bwd_sweep<..., RHOE> only
    int force_plain;                       // the problem has no V: only mrf_bwd_sweep may run
    double *gstore_buf;                    // [N][L] room for gstore (workspace), or NULL
    double *gstore;                        // mrf_bwd_sweep_chain: if not NULL, its helpers store the gradient vector g of
                                           // every node here (0 where no update is replayed) for mrf_bwd_gv_from_g
    int *fault;                            // launch-wide word raised when a wait between wavefronts is given up (mrf_wait_turn)
    int spin_limit;                        // microseconds after which a wait is given up
};

#define MRF_BWD_WAVES 4   // wavefronts (= scanlines in flight) per workgroup
#define MRF_CHAIN_MAX_HELPERS 12

// dynamic LDS of mrf_bwd_sweep_chain (host and device agree through this one expression)
__host__ __device__ inline size_t mrf_bwd_chain_lds_bytes(int LP, int NI, int L, bool with_theta, bool vg, bool gv)
{
    const size_t NR = 2 * (size_t)NI, LL = 64 * (size_t)LP;
    const size_t arrays = sizeof(double) * (3 * NR * LL + LL + ((gv && LP == 1) ? (size_t)NI * L * L : 0)) +
                          sizeof(float) * (with_theta ? NR * LL : 0) + sizeof(int) * (3 * MRF_CHAIN_MAX_HELPERS + 1) +
                          sizeof(float) * (gv ? (size_t)L * L : (vg ? 0 : (size_t)L)) + NR * LL;
    return (arrays + 7) / 8 * 8 + sizeof(MrfWaitBlock);      // the deadline of the waits sits behind the arrays
}

// LP labels per lane, NS source slots, D prefetch distance, VG: V for the edge-weight
// gradient is gathered from global memory (it fits neither LDS layout), HOT: pre-reduce the
// most popular scatter target, RHOE: the per-edge extras.  TRW coefficients per edge (P.rho_e)
// instead of per direction: what direction c scattered to node i came over the edge (i, i+c)
// and carries that edge's rho.  Gradient of per-edge pairwise tables (P.gE): entry
// (p(lambda), lambda) of the edge's table receives g(lambda) (Eq. supp-gradient-pairwise).
// UNARY = false: no direction of the launch forms grad theta_i (P.unary_dir < 0: ISGMR leaves it to
// mrf_isgmr_bwd_combine), so nothing of it is loaded or kept in registers.
// WAVES: wavefronts per workgroup (more of them share the one V-gradient table of P.gv_lds == 2).
// FULL: the launch has exactly 64 LP labels (the host checks it), so every label test folds away and the
// strides are constants.
template <int LP, int NS, int D, bool VG, bool HOT, bool RHOE = false, bool UNARY = true, int WAVES = MRF_BWD_WAVES, bool FULL = false>
__global__ void __launch_bounds__(64 * WAVES) mrf_bwd_sweep(const MrfBwdParams P)
{
    extern __shared__ __align__(16) unsigned char mrf_bsmem[];
    const int L = FULL ? 64 * LP : P.g.L;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform, and known to be
    double *sbuf = reinterpret_cast<double *>(mrf_bsmem) + wv * 64 * LP;
    double *gvl = reinterpret_cast<double *>(mrf_bsmem) + WAVES * 64 * LP + (P.gv_lds == 1 ? wv * L * L : 0);
    float *vl = reinterpret_cast<float *>(reinterpret_cast<double *>(mrf_bsmem) + WAVES * 64 * LP +
                                          (P.gv_lds == 1 ? WAVES * L * L : (P.gv_lds == 2 ? L * L : 0)));
    const long long slot = (long long)blockIdx.x * WAVES + wv;
    const long long nslots = (long long)gridDim.x * WAVES;
    const long long N = P.g.N;
    double *gVs = P.gV ? P.gV + (size_t)(P.gv_lds == 2 ? (long long)blockIdx.x : slot) * L * L : nullptr;
    const int vzero = mrf_opaque_zero();

    if (P.v_mode == 1)
        for (int e = threadIdx.x; e < L * L; e += blockDim.x) vl[e] = P.V[e];
    else if (P.v_mode == 2)
        for (int e = threadIdx.x; e < L; e += blockDim.x) vl[e] = P.V[e];
    if (gVs && P.gv_lds == 1)
        for (int e = lane; e < L * L; e += 64) gvl[e] = 0.0;
    if (gVs && P.gv_lds == 2)
        for (int e = threadIdx.x; e < L * L; e += blockDim.x) gvl[e] = 0.0;
    __syncthreads();

    for (long long sl = slot; sl < P.total_scanlines; sl += nslots) {
        int ri = 0;
        while (ri + 1 < P.r_count && sl >= P.blk_begin[ri + 1]) ++ri;
        const int r = P.r_first + ri;
        const long long local = sl - P.blk_begin[ri];
        const int nsc = P.g.nscan[r];
        const int b = (int)(local / nsc);
        const long long t = local - (long long)b * nsc;
        const int dh = P.g.dh[r], dw = P.g.dw[r];
        int y0, x0, len;
        mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
        const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
        const long long nstep = (long long)dh * P.g.W + dw;
        const double cscale = (double)P.carry_scale[r];
        const bool own_unary = UNARY && (r == P.unary_dir);
        const bool unary_old = own_unary && !P.unary_init;
        const size_t umul = unary_old ? 1 : 0;
        const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
        const uint8_t *pbase = P.p + (size_t)r * N * L;
        const uint8_t *qbase = P.q + (size_t)r * N;

        // source slots; unused ones re-read grad c / the first source with coefficient 0
        const float *src[NS];
        double cG[NS], cT[NS];
        const int nsrc = P.n_src[r];
#pragma unroll
        for (int c = 0; c < NS; ++c) {
            const bool live = c < nsrc;
            const bool isgc = (c == nsrc) && P.use_gc;
            src[c] = live ? P.src_base + (size_t)P.src_dir[r][c] * P.src_stride : P.gc;
            cG[c] = live ? (double)P.coefG[r][c] : (isgc ? 1.0 : 0.0);
            cT[c] = live ? (double)P.coefT[r][c] : (isgc ? 1.0 : 0.0);
        }
        // per-edge rho: where to find the rho of the edge that source slot c used at a node
        const float *rsrc[NS];
        long long rstep[NS];
        double ropp[NS];
        bool rlive[NS];
#pragma unroll
        for (int c = 0; c < NS; ++c) {
            const int sd = (RHOE && c < nsrc) ? P.src_dir[r][c] : r;
            rlive[c] = RHOE && P.rho_e && c < nsrc;
            rsrc[c] = (RHOE && P.rho_e) ? P.rho_e + (size_t)sd * N : nullptr;
            rstep[c] = (long long)P.g.dh[sd] * P.g.W + P.g.dw[sd];
            ropp[c] = (sd == P.g.opp[r]) ? 1.0 : 0.0;
        }

        // the last node of the scanline has no successor in direction r
        {
            const long long last = head + (long long)(len - 1) * nstep;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) P.S[((size_t)r * N + last) * L + lam] = 0.0f;
            }
        }

        // prefetch registers: step tt handles node len-1-tt (clamped at the first node)
        float cur[D][NS][LP], nxt[D][NS][LP];
        float ucur[D][UNARY ? LP : 1], unxt[D][UNARY ? LP : 1];       // old grad theta_i (only read when accumulating)
        int pcur[D][LP], pnxt[D][LP];
        int qcur[D], qnxt[D];
        float wcur[D], wnxt[D];
        float rcur[D][NS + 1], rnxt[D][NS + 1];   // RHOE: rho of each source slot's edge, then of this direction's own edge
        auto prefetch = [&](float (&dst)[NS][LP], float (&udst)[UNARY ? LP : 1], int (&pdst)[LP], int &qdst, float &wdst,
                            float (&rdst)[NS + 1], int tt) {
            int n = len - 1 - tt;
            n = n > 0 ? n : 0;
            const long long i = head + (long long)n * nstep;
            if (RHOE && P.rho_e) {
                // (a node without successor in direction c got zeros from that direction: any
                // finite coefficient will do, so the index is only kept inside the array)
#pragma unroll
                for (int c = 0; c < NS; ++c) {
                    long long e = i + rstep[c];
                    e = e < 0 ? 0 : (e > N - 1 ? N - 1 : e);
                    rdst[c] = rsrc[c][(size_t)e + vzero];
                }
                rdst[NS] = P.rho_e[(size_t)r * N + i + vzero];
            }
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                const int lc = lam < L ? lam : 0;
#pragma unroll
                for (int c = 0; c < NS; ++c) dst[c][s] = src[c][(size_t)i * L + lc];
                if constexpr (UNARY) udst[s] = P.gunary[((size_t)i * L + lc) * umul];   // one cached word unless it is needed
                pdst[s] = pbase[(size_t)i * L + lc];
            }
            qdst = qbase[(size_t)i + vzero];
            wdst = wbase[(size_t)(i * P.w_mul) + vzero];
        };
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], ucur[u], pcur[u], qcur[u], wcur[u], rcur[u], u);

        double carry[LP];   // what node i+r of this direction passed back to node i
#pragma unroll
        for (int s = 0; s < LP; ++s) { carry[s] = 0.0; sbuf[lane + 64 * s] = 0.0; }
        mrf_wave_lds_fence();

        for (int t0 = 0; t0 < len; t0 += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) prefetch(nxt[u], unxt[u], pnxt[u], qnxt[u], wnxt[u], rnxt[u], t0 + D + u);
#pragma unroll
            for (int u = 0; u < D; ++u) {
                // Steps past the first node (last group only) and the first node itself run the
                // same instructions with their stores switched off, so that the loop body has no
                // branches around the prefetched registers.
                const int tt = t0 + u;
                const bool past = tt >= len;
                const int n = past ? 0 : len - 1 - tt;
                const bool update = !past && n > 0;      // node i has a predecessor: replay its update
                const long long i = head + (long long)n * nstep;
                const long long j = i - nstep;
                double cGn[NS], cTn[NS];
#pragma unroll
                for (int c = 0; c < NS; ++c) {
                    // Alg. 4 lines 9-11 with the rho of the edge (i, i+c): rho s to every direction
                    // and to grad theta, minus s to the opposite direction
                    cGn[c] = rlive[c] ? (double)rcur[u][c] - ropp[c] : cG[c];
                    cTn[c] = rlive[c] ? (double)rcur[u][c] : cT[c];
                }
                const double cscale_n = (RHOE && P.rho_e) ? (double)rcur[u][NS] : cscale;
                double g[LP];
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    double acc = carry[s];
#pragma unroll
                    for (int c = 0; c < NS; ++c) acc = __builtin_fma(cGn[c], (double)cur[u][c][s], acc);
                    g[s] = (lane + 64 * s < L) ? acc : 0.0;
                }
                if constexpr (UNARY) if (own_unary) {
                    // grad theta_i: everything every direction passed back to node i
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        double accT = carry[s];
#pragma unroll
                        for (int c = 0; c < NS; ++c) accT = __builtin_fma(cTn[c], (double)cur[u][c][s], accT);
                        accT += unary_old ? (double)ucur[u][s] : 0.0;   // (the buffer may hold anything at first)
                        if (!past && lane + 64 * s < L) P.gunary[(size_t)i * L + lane + 64 * s] = (float)accT;
                    }
                }
                int pv[LP];
                double part = 0.0;
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    pv[s] = pcur[u][s] < L ? pcur[u][s] : L - 1;
                    part += g[s];
                }
                // Truncated models send most labels to one source label (the far-field minimiser),
                // which would serialise the LDS adds below.  Guess that label from p at the first
                // and at the last label (one of the two is far from it), take the commoner of the
                // two, and sum its lanes with a DPP tree instead.
                // (Only worth its instructions when the launch is not latency bound or L is large.)
                int hot = -1;
                double hpart = 0.0;
                if (HOT) {
                    const int c0 = __builtin_amdgcn_readlane(pv[0], 0);
                    int c1 = c0;
#pragma unroll
                    for (int s = 0; s < LP; ++s)
                        if (((L - 1) >> 6) == s) c1 = __builtin_amdgcn_readlane(pv[s], (L - 1) & 63);
                    int n0 = 0, n1 = 0;
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        const bool vld = lane + 64 * s < L;
                        n0 += __popcll(__ballot(vld && pv[s] == c0));
                        n1 += __popcll(__ballot(vld && pv[s] == c1));
                    }
                    hot = n1 > n0 ? c1 : c0;
#pragma unroll
                    for (int s = 0; s < LP; ++s)
                        if (lane + 64 * s < L && pv[s] == hot) hpart += g[s];
                }
                // back Eq. isgmr-norm: g(q) -= sum_lambda g(lambda)
                double tot, hsum = 0.0;
                int qv = __builtin_amdgcn_readfirstlane(qcur[u]);
                qv = qv < L ? qv : L - 1;
                // HOT: the edge-weight gradient sum_lambda g(lambda) V(p(lambda), lambda) is formed from g
                // before the correction at q, in the same reduction as the two other sums, and corrected
                // by tot V(p(q), q) afterwards
                double gw_sum = 0.0;
                if (HOT) {
                    double wpart = 0.0;
                    float vq = 0.0f;
                    if (P.gw) {
#pragma unroll
                        for (int s = 0; s < LP; ++s) {
                            const int lam = lane + 64 * s;
                            const int dist = pv[s] > lam ? pv[s] - lam : lam - pv[s];
                            const float vv = lam < L ? vl[P.v_mode == 1 ? __mul24(pv[s], L) + lam : dist] : 0.0f;
                            wpart = __builtin_fma(g[s], (double)vv, wpart);       // (g is 0 beyond L)
                            if ((qv >> 6) == s) vq = mrf_readlane_f32(vv, qv & 63);
                        }
                    }
                    mrf_wave_sum3_f64(part, hpart, wpart, tot, hsum, gw_sum);
                    int pq = 0;
#pragma unroll
                    for (int s = 0; s < LP; ++s)
                        if ((qv >> 6) == s) pq = __builtin_amdgcn_readlane(pv[s], qv & 63);
                    if (pq == hot) hsum -= tot;
                    gw_sum = __builtin_fma(-tot, (double)vq, gw_sum);
                } else {
                    tot = mrf_wave_sum_f64(part);
                }
#pragma unroll
                for (int s = 0; s < LP; ++s)
                    if (lane + 64 * s == qv) g[s] = g[s] - tot;

                // index scatter through LDS: s(mu) = sum over lambda with p(lambda) = mu
                // (sbuf was cleared right after the previous step read it)
#pragma unroll
                for (int s = 0; s < LP; ++s)
                    if (lane + 64 * s < L && pv[s] != hot)
                        __hip_atomic_fetch_add(&sbuf[pv[s]], g[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                mrf_wave_lds_fence();
                double sv[LP];
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    sv[s] = sbuf[lane + 64 * s];
                    if (lane + 64 * s == hot) sv[s] += hsum;
                }
                mrf_wave_lds_fence();
#pragma unroll
                for (int s = 0; s < LP; ++s) sbuf[lane + 64 * s] = 0.0;
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    if (update && lam < L) P.S[((size_t)r * N + j) * L + lam] = (float)sv[s];
                    carry[s] = cscale_n * sv[s];
                }

                // pairwise gradients (off the node-to-node chain)
                const double wgt = (double)wcur[u];
                if (HOT && P.gw) {
                    if (update && lane == 0)
                        __hip_atomic_fetch_add(&P.gw[(size_t)r * N + i], (float)gw_sum, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                } else if (P.gw) {
                    double acc = 0.0;
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        const int lam = lane + 64 * s;
                        if (lam < L) {
                            float vv;
                            if (VG) {
                                vv = P.V[(size_t)__mul24(pv[s], L) + lam];
                            } else {
                                const int dist = pv[s] > lam ? pv[s] - lam : lam - pv[s];
                                vv = vl[P.v_mode == 1 ? __mul24(pv[s], L) + lam : dist];
                            }
                            acc = __builtin_fma(g[s], (double)vv, acc);
                        }
                    }
                    acc = mrf_wave_sum_f64(acc);
                    // one writer per entry and launch: a no-return atomic is a plain accumulate
                    // that does not make the wavefront wait for the old value
                    if (update && lane == 0)
                        __hip_atomic_fetch_add(&P.gw[(size_t)r * N + i], (float)acc, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                }
                if (RHOE && P.gE) {
                    // one writer per table and launch: plain read-modify-write
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        const int lam = lane + 64 * s;
                        if (update && lam < L) {
                            float *e = P.gE + (((size_t)r * N + i) * L + pv[s]) * L + lam;
                            *e = *e + (float)g[s];
                        }
                    }
                }
                if (gVs) {
                    // lane lambda owns column lambda of the wavefront's private accumulator
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        const int lam = lane + 64 * s;
                        if (update && lam < L) {
                            if (P.gv_lds == 1) gvl[__mul24(pv[s], L) + lam] = __builtin_fma(wgt, g[s], gvl[__mul24(pv[s], L) + lam]);
                            else if (P.gv_lds == 2) __hip_atomic_fetch_add(&gvl[__mul24(pv[s], L) + lam], wgt * g[s], __ATOMIC_RELAXED,
                                                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                            else __hip_atomic_fetch_add(&gVs[(size_t)__mul24(pv[s], L) + lam], wgt * g[s],
                                                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < D; ++u) {
                qcur[u] = qnxt[u];
                wcur[u] = wnxt[u];
#pragma unroll
                for (int c = 0; c <= NS; ++c) rcur[u][c] = rnxt[u][c];
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    if constexpr (UNARY) ucur[u][s] = unxt[u][s];
                    pcur[u][s] = pnxt[u][s];
#pragma unroll
                    for (int c = 0; c < NS; ++c) cur[u][c][s] = nxt[u][c][s];
                }
            }
        }
    }
    if (gVs && P.gv_lds == 1) {
        mrf_wave_lds_fence();
        for (int e = lane; e < L * L; e += 64) gVs[e] += gvl[e];
    }
    if (P.gv_lds == 2) {
        // (every wavefront of the workgroup arrives here; the slot belongs to this workgroup alone)
        __syncthreads();
        if (gVs)
            for (int e = threadIdx.x; e < L * L; e += blockDim.x) gVs[e] += gvl[e];
    }
}

// ---- index replay with the node-to-node chain on a wavefront of its own ----------------------
//
// For launches with few scanlines, where the time of a sweep is the length of a scanline
// times the latency of one node step.  Of the work of a node only this depends on the
// previous node: add what it passed back (carry) to the gradient arriving from elsewhere
// (ext), subtract the label sum at q, scatter through p, scale.  The label sum itself does
// not: the scattered vector of a node sums to zero (the reparametrisation took exactly its
// sum off one entry, back Eq. isgmr-norm), hence so does the carry, and the label sum of
// carry + ext is the label sum of ext up to rounding in the last place of a double.  So the
// correction at q can be applied to ext before the carry is known.
//
// A scanline gets 1 + NI wavefronts.  The helpers take the nodes in turn: they load, form
// ext with the correction at q, and publish it with p through a ring in LDS (stage "pre");
// the chain wavefront touches only LDS: one add per label, the scatter, one read, one
// multiply; the same helpers later pick up what the chain left for a node (incoming carry
// and scattered vector) and do the rest: grad theta (Alg. 4 line 8), the stored s, the
// edge-weight gradient (Eq. supp-gradient-edge) (stage "post").  A helper runs pre(t) then
// post(t - NI), with a ring of 2 NI slots: every slot is free again exactly when its owner
// comes round to it, so only two kinds of wait exist (chain on pre, post on chain), each on
// a counter that only grows.  The chain reads one node ahead and frees a node for post one
// step late; with NI >= 2 no wait can depend on itself: post(t - 2 NI), which precedes
// pre(t) in its helper, needs the chain to have passed step t - 2 NI + 1 only.
//
// GV (L <= 64, as far as LDS has room): the launch also wants the V gradient; every helper keeps an accumulator of
// its own in LDS, lane lambda owning column lambda, and adds it to its own slot at the end.  With more than
// one label per lane the tables do not fit: GV then means that the helpers store the gradient vector g of every
// node in P.gstore (0 where no update is replayed), from which mrf_bwd_gv_from_g forms the table afterwards;
// V is still copied to LDS for the edge-weight gradient.
// HOT: truncated models send most labels to one source label, and the chain wavefront's LDS
// adds would queue at that one word; the helpers guess it (as in mrf_bwd_sweep) and the chain
// sums its lanes with a DPP tree while the LDS round trip is under way.  Costs the chain some
// twenty instructions per node: for launches that are bound by LDS throughput, not by the
// latency of the chain.
template <int LP, int NS, int D, int NI, bool VG, bool GV, bool HOT>
__global__ void __launch_bounds__(64 * (1 + NI)) mrf_bwd_sweep_chain(const MrfBwdParams P)
{
    constexpr int NR = 2 * NI;
    constexpr int LL = 64 * LP;
    static_assert(NI >= 2 && NI <= MRF_CHAIN_MAX_HELPERS, "helpers per scanline");
    extern __shared__ __align__(16) unsigned char mrf_bsmem[];
    // carved in the order of mrf_bwd_chain_lds_bytes
    double *a_ext = reinterpret_cast<double *>(mrf_bsmem);       // [NR][LL] pre -> chain, post
    double *b_cin = a_ext + NR * LL;                             // [NR][LL] chain -> post: carry that entered the node
    double *b_sv = b_cin + NR * LL;                              // [NR][LL]                scattered vector that left it
    double *sbuf = b_sv + NR * LL;                               // [LL] scatter target of the chain
    double *gvacc = sbuf + LL;                                   // [NI][L*L] V-gradient accumulators (GV)
    constexpr bool GVT = GV && LP == 1;      // V-gradient tables in LDS
    constexpr bool GS = GV && LP != 1;       // node gradients stored for mrf_bwd_gv_from_g
    float *a_extT = reinterpret_cast<float *>(gvacc + (GVT ? NI * P.g.L * P.g.L : 0));   // [NR][LL] pre -> post (launches that form grad theta)
    int *pre_done = reinterpret_cast<int *>(a_extT + (P.unary_dir >= 0 ? NR * LL : 0));   // [MRF_CHAIN_MAX_HELPERS] per helper: last step published
    int *chain_done = pre_done + MRF_CHAIN_MAX_HELPERS;          // last step the chain finished
    int *a_hot = chain_done + 1;                                 // [NR] pre -> chain: most popular scatter target, or -1
    float *vl = reinterpret_cast<float *>(a_hot + 2 * MRF_CHAIN_MAX_HELPERS);   // [L] first row of V (unless VG), all of V (GV)
    uint8_t *a_p = reinterpret_cast<uint8_t *>(vl + (GV ? P.g.L * P.g.L : (VG ? 0 : P.g.L)));   // [NR][LL]
    MrfWaitBlock &wait_lds = *reinterpret_cast<MrfWaitBlock *>(
        mrf_bsmem + ((a_p + NR * LL - mrf_bsmem) + 7) / 8 * 8);  // for the waits below (mrf_wait_turn)
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform, and known to be
    const long long N = P.g.N;

    if (GV) {
        for (int e = threadIdx.x; e < L * L; e += blockDim.x) vl[e] = P.V[e];
        if (GVT)
            for (int e = threadIdx.x; e < NI * L * L; e += blockDim.x) gvacc[e] = 0.0;
    } else if (!VG) {
        for (int e = threadIdx.x; e < L; e += blockDim.x) vl[e] = P.V[e];
    }
    if (threadIdx.x < MRF_CHAIN_MAX_HELPERS) pre_done[threadIdx.x] = (int)threadIdx.x - NI;
    if (threadIdx.x == 0) { *chain_done = -1; mrf_wait_init(&wait_lds, P.fault, P.spin_limit); }
    for (int e = threadIdx.x; e < LL; e += blockDim.x) sbuf[e] = 0.0;
    __syncthreads();

    const long long sl = blockIdx.x;       // one scanline per workgroup
    int ri = 0;
    while (ri + 1 < P.r_count && sl >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = sl - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;

    if (wv == 0) {
        // ---- the chain: step tt handles node len-1-tt ---------------------------------------
        // One wait per step: the read of the scattered vector.  What the step needs from the
        // ring is read one step ahead, and the counter that frees a step for the helpers is
        // written one step late, when the LDS queue is known to have drained past it.
        const double cscale = (double)P.carry_scale[r];
        double carry[LP], ext[LP];
        int pv[LP];
        auto await = [&](int u, int tt) {
            int sn;
            int wait_turns = 0;
            do {
                sn = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&pre_done[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                if (sn < tt) mrf_wait_turn(&wait_lds, wait_turns);
            } while (sn < tt);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        };
        await(0, 0);
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            carry[s] = 0.0;
            ext[s] = a_ext[lane + 64 * s];
            pv[s] = a_p[lane + 64 * s];
        }
        int hot = -1;
        if (HOT) hot = __builtin_amdgcn_readfirstlane(a_hot[0]);
        int sb = 0;                         // slot of step t0 (t0 is a multiple of NI)
        for (int t0 = 0; t0 < len; t0 += NI) {
#pragma unroll
            for (int u = 0; u < NI; ++u) {
                const int tt = t0 + u;
                if (tt < len) {
                    const int slot = sb + u;
                    const int un = (u + 1 == NI) ? 0 : u + 1;
                    const int slotn = (u + 1 == NI) ? (sb == 0 ? NI : 0) : slot + 1;
                    const bool more = tt + 1 < len;
                    // index scatter: s(mu) = sum over lambda with p(lambda) = mu (labels past L
                    // carry zeros to entries of their own)
                    double hpart = 0.0;
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        const int lam = lane + 64 * s;
                        const double g = carry[s] + ext[s];
                        b_cin[slot * LL + lam] = carry[s];
                        const bool ishot = HOT && pv[s] == hot;
                        if (!ishot)
                            __hip_atomic_fetch_add(&sbuf[pv[s]], g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        if (HOT) hpart += ishot ? g : 0.0;
                    }
                    mrf_wave_lds_fence();
                    // In one batch behind the scatter: the counter of the next node's helper, then
                    // (the LDS queue keeps this order) that node's ring entries, then the scattered
                    // vector.  If the counter turns out not to cover the node, its entries are read
                    // again after waiting.
                    const int flag = __hip_atomic_load(&pre_done[un], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    double sv[LP];
                    int hotn = -1;
                    if (HOT) hotn = a_hot[slotn];
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        ext[s] = a_ext[slotn * LL + lane + 64 * s];
                        pv[s] = a_p[slotn * LL + lane + 64 * s];
                        sv[s] = sbuf[lane + 64 * s];
                    }
                    double hsum = 0.0;
                    if (HOT) hsum = mrf_wave_sum_f64(hpart);
                    if (__builtin_expect(more && __builtin_amdgcn_readfirstlane(flag) < tt + 1, 0)) {
                        await(un, tt + 1);
                        if (HOT) hotn = a_hot[slotn];
#pragma unroll
                        for (int s = 0; s < LP; ++s) {
                            ext[s] = a_ext[slotn * LL + lane + 64 * s];
                            pv[s] = a_p[slotn * LL + lane + 64 * s];
                        }
                    }
                    // everything this wavefront sent to LDS before the reads above has landed
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
                    __builtin_amdgcn_wave_barrier();
                    // (written by every lane: the same word, and no exec-mask juggling in the step)
                    if (tt > 0)
                        __hip_atomic_store(chain_done, tt - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        if (HOT && lane + 64 * s == hot) sv[s] += hsum;
                        sbuf[lane + 64 * s] = 0.0;
                        b_sv[slot * LL + lane + 64 * s] = sv[s];
                        carry[s] = cscale * sv[s];
                    }
                    if (HOT) hot = __builtin_amdgcn_readfirstlane(hotn);
                }
            }
            sb = (sb == 0) ? NI : 0;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) __hip_atomic_store(chain_done, len - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return;
    }

    // ---- helpers ---------------------------------------------------------------------------
    const int jw = wv - 1;
    const bool own_unary = (r == P.unary_dir);
    const bool unary_old = own_unary && !P.unary_init;
    const size_t umul = unary_old ? 1 : 0;
    const uint8_t *pbase = P.p + (size_t)r * N * L;
    const uint8_t *qbase = P.q + (size_t)r * N;
    const int vzero = mrf_opaque_zero();

    // source slots; unused ones re-read grad c / the first source with coefficient 0
    const float *src[NS];
    double cG[NS], cT[NS];
    const int nsrc = P.n_src[r];
#pragma unroll
    for (int c = 0; c < NS; ++c) {
        const bool live = c < nsrc;
        const bool isgc = (c == nsrc) && P.use_gc;
        src[c] = live ? P.src_base + (size_t)P.src_dir[r][c] * P.src_stride : P.gc;
        cG[c] = live ? (double)P.coefG[r][c] : (isgc ? 1.0 : 0.0);
        cT[c] = live ? (double)P.coefT[r][c] : (isgc ? 1.0 : 0.0);
    }

    // the last node of the scanline has no successor in direction r
    if (jw == 0) {
        const long long last = head + (long long)(len - 1) * nstep;
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int lam = lane + 64 * s;
            if (lam < L) P.S[((size_t)r * N + last) * L + lam] = 0.0f;
        }
    }

    // own steps: tt = jw + it * NI, it = 0 .. T-1; one more turn for the last post
    const int T = len > jw ? (len - jw + NI - 1) / NI : 0;
    float cur[D][NS][LP], nxt[D][NS][LP];
    float ucur[D][LP], unxt[D][LP];
    int pcur[D][LP], pnxt[D][LP];
    int qcur[D], qnxt[D];
    float wcur[D], wnxt[D];                 // edge weight of the node's incoming edge (GV)
    // addresses relative to the head of the scanline: one 32 x 32 bit product per node (the
    // host has checked that a node step times L fits 32 bits)
    const int step_l = (int)nstep * L;
    const int step_n = (int)nstep;
    const float *srcb[NS];
#pragma unroll
    for (int c = 0; c < NS; ++c) srcb[c] = src[c] + (size_t)head * L;
    const float *gub = P.gunary + (size_t)head * L * umul;
    const int step_u = unary_old ? step_l : 0;
    const uint8_t *pb = pbase + (size_t)head * L;
    const uint8_t *qb = qbase + (size_t)head;
    const float *wb = P.w + (P.w_mul ? (size_t)r * N + head : 0);
    const int step_w = P.w_mul ? step_n : 0;
    auto prefetch = [&](float (&dst)[NS][LP], float (&udst)[LP], int (&pdst)[LP], int &qdst, float &wdst, int it) {
        int n = len - 1 - (jw + it * NI);
        n = n > 0 ? n : 0;
        const long long o = (long long)n * step_l;
        const long long ou = (long long)n * step_u;
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int lam = lane + 64 * s;
            const int lc = lam < L ? lam : 0;
#pragma unroll
            for (int c = 0; c < NS; ++c) dst[c][s] = srcb[c][o + lc];
            udst[s] = gub[ou + (unary_old ? lc : 0)];      // one cached word unless it is needed
            pdst[s] = pb[o + lc];
        }
        qdst = qb[(long long)n * step_n + vzero];
        wdst = GVT ? wb[(long long)n * step_w + vzero] : 0.0f;
    };
    if (T > 0) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], ucur[u], pcur[u], qcur[u], wcur[u], u);
    }
    double *gvl = gvacc + (GVT ? jw * L * L : 0);
    float wlast = 0.0f;                     // weight of the node whose post stage comes next
    float *guw = P.gunary + (size_t)head * L;                       // stores of stage "post"
    float *sw = P.S + ((size_t)r * N + head) * L;
    float *gww = P.gw ? P.gw + (size_t)r * N + head : nullptr;
    double *gsw = GS ? P.gstore + (size_t)head * L : nullptr;

    int chain_seen = -1;
    for (int it0 = 0; it0 < T + 1 && T > 0; it0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], unxt[u], pnxt[u], qnxt[u], wnxt[u], it0 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int tt = jw + (it0 + u) * NI;
            if (tt < len) {
                // ---- pre(tt): everything of node len-1-tt that does not need the carry -------
                const int slot = tt % NR;
                double part = 0.0;
                double ev[LP];
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    double e = 0.0, eT = 0.0;
#pragma unroll
                    for (int c = 0; c < NS; ++c) e = __builtin_fma(cG[c], (double)cur[u][c][s], e);
                    if (own_unary) {
#pragma unroll
                        for (int c = 0; c < NS; ++c) eT = __builtin_fma(cT[c], (double)cur[u][c][s], eT);
                        eT += unary_old ? (double)ucur[u][s] : 0.0;     // (the buffer may hold anything at first)
                    }
                    ev[s] = lam < L ? e : 0.0;
                    part += ev[s];
                    if (own_unary) a_extT[slot * LL + lam] = (float)eT;
                    // (labels past L scatter their zeros to entries of their own)
                    a_p[slot * LL + lam] = (uint8_t)(lam < L ? (pcur[u][s] < L ? pcur[u][s] : L - 1) : lam);
                }
                // the commoner of p at the first and at the last label: for a truncated model one
                // of the two is far from the far-field minimiser and points to it
                if (HOT) {
                    int hot = -1;
                    const int c0 = __builtin_amdgcn_readlane(pcur[u][0], 0);
                    int c1 = c0;
#pragma unroll
                    for (int s = 0; s < LP; ++s)
                        if (((L - 1) >> 6) == s) c1 = __builtin_amdgcn_readlane(pcur[u][s], (L - 1) & 63);
                    int n0 = 0, n1 = 0;
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        const bool vld = lane + 64 * s < L;
                        n0 += __popcll(__ballot(vld && pcur[u][s] == c0));
                        n1 += __popcll(__ballot(vld && pcur[u][s] == c1));
                    }
                    hot = n1 > n0 ? c1 : c0;
                    hot = hot < L ? hot : -1;
                    if (lane == 0) a_hot[slot] = hot;
                }
                // back Eq. isgmr-norm, on the part of g that is known here: the entry at q loses
                // the label sum
                const double tot = mrf_wave_sum_f64(part);
                int qv = __builtin_amdgcn_readfirstlane(qcur[u]);
                qv = qv < L ? qv : L - 1;
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    a_ext[slot * LL + lam] = (lam == qv) ? ev[s] - tot : ev[s];
                }
                // (LDS keeps a wavefront's operations in order: the counter lands behind the entries)
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                if (lane == 0) __hip_atomic_store(&pre_done[jw], tt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            const int tp = tt - NI;
            if (tp >= 0 && tp < len) {
                // ---- post(tp): what is left of node len-1-tp once the chain has passed --------
                int wait_turns = 0;
                while (chain_seen < tp) {
                    chain_seen = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(chain_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                    if (chain_seen < tp) mrf_wait_turn(&wait_lds, wait_turns);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                const int slot = tp % NR;
                const int n = len - 1 - tp;
                const bool update = n > 0;             // node i has a predecessor: its update is replayed
                const long long oi = (long long)n * step_l;              // node i, in label entries from the head
                const long long oj = oi - step_l;                        // node i - r
                double acc = 0.0;
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    const double cin = b_cin[slot * LL + lam];
                    if (own_unary && lam < L)
                        guw[oi + lam] = (float)(cin + (double)a_extT[slot * LL + lam]);
                    if (update && lam < L) sw[oj + lam] = (float)b_sv[slot * LL + lam];
                    if ((P.gw || GV) && lam < L) {
                        const double g = cin + a_ext[slot * LL + lam];    // as the chain formed it
                        const int pv = a_p[slot * LL + lam];
                        if constexpr (GS) gsw[oi + lam] = update ? g : 0.0;
                        if (P.gw) {
                            float vv;
                            if (GV) {
                                vv = vl[__mul24(pv, L) + lam];
                            } else if (VG) {
                                vv = P.V[(size_t)__mul24(pv, L) + lam];
                            } else {
                                const int dist = pv > lam ? pv - lam : lam - pv;
                                vv = vl[dist];
                            }
                            acc = __builtin_fma(g, (double)vv, acc);
                        }
                        if (GVT && update)
                            gvl[__mul24(pv, L) + lam] = __builtin_fma((double)wlast, g, gvl[__mul24(pv, L) + lam]);
                    }
                }
                if (P.gw) {
                    acc = mrf_wave_sum_f64(acc);
                    // one writer per entry and launch: a no-return atomic is a plain accumulate
                    if (update && lane == 0)
                        __hip_atomic_fetch_add(&gww[(long long)n * step_n], (float)acc, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            wlast = wcur[u];
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            qcur[u] = qnxt[u];
            wcur[u] = wnxt[u];
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                ucur[u][s] = unxt[u][s];
                pcur[u][s] = pnxt[u][s];
#pragma unroll
                for (int c = 0; c < NS; ++c) cur[u][c][s] = nxt[u][c][s];
            }
        }
    }
    if (GVT) {
        // one slot per helper of every workgroup
        mrf_wave_lds_fence();
        double *gVs = P.gV + ((size_t)blockIdx.x * NI + jw) * L * L;
        for (int e = lane; e < L * L; e += 64) gVs[e] += gvl[e];
    }
}

// ---- grad V apart from the sweep (65..128 labels beside mrf_bwd_sweep_chain) --------------------
// Eq. supp-gradient-smoothness: entry (p(lambda), lambda) of the table receives theta_{i-r,i} g(lambda) at
// every replayed update.  Nothing of it depends on the order of the nodes, so where the chain layout has no
// room for the table its helpers store g per node and this streaming pass does the additions: one wavefront
// per node, lanes over lambda, the L x L table of a workgroup in LDS (`ds_add_f64`), added to the workgroup's
// slot at the end.
struct MrfGvParams {
    long long N;
    int L;
    const double *g;         // [N][L]
    const uint8_t *p;        // [N][L] of this direction and iteration
    const float *w;          // [N] edge weights of this direction, or the scalar at w[0] when w_mul == 0
    int w_mul;
    double *gV;              // [gridDim.x][L][L] slots
};

__global__ void __launch_bounds__(512) mrf_bwd_gv_from_g(const MrfGvParams P)
{
    extern __shared__ __align__(16) unsigned char mrf_gvsmem[];
    double *tile = reinterpret_cast<double *>(mrf_gvsmem);
    const int L = P.L;
    for (int e = threadIdx.x; e < L * L; e += blockDim.x) tile[e] = 0.0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long nwaves = (long long)gridDim.x * (blockDim.x >> 6);
    for (long long i = wave; i < P.N; i += nwaves) {
        const double wgt = (double)P.w[(size_t)(i * P.w_mul)];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int lam = lane + 64 * s;
            if (lam < L) {
                const double g = P.g[(size_t)i * L + lam];
                if (g != 0.0) {
                    int pv = P.p[(size_t)i * L + lam];
                    pv = pv < L ? pv : L - 1;
                    __hip_atomic_fetch_add(&tile[__mul24(pv, L) + lam], wgt * g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
        }
    }
    __syncthreads();
    double *slot = P.gV + (size_t)blockIdx.x * L * L;
    for (int e = threadIdx.x; e < L * L; e += blockDim.x) slot[e] += tile[e];
}

// ---- index replay, one label per lane, ceil(L/64) wavefronts per scanline --------------------
//
// Same arithmetic as mrf_bwd_sweep for launches with few scanlines and many labels (a lone
// wavefront with 3-4 labels per lane is bound by instruction issue).  Every wavefront owns 64
// labels: it scatters their g into its own copy of the target vector and publishes their sum;
// after one LDS-only barrier each wavefront adds the copies for its own 64 targets in
// wavefront order (fixed order: reproducible), applies the reparametrisation correction
// (the target p(q) loses the label sum) and carries on.  Copies alternate between two sets so
// that one barrier per node is enough; the edge-weight gradient is assembled one node later.
template <int NS, int D, bool VG>
__global__ void __launch_bounds__(256) mrf_bwd_sweep_split(const MrfBwdParams P)
{
    extern __shared__ __align__(16) unsigned char mrf_bsmem[];
    __shared__ double cp[2][4][256];
    __shared__ double psum[2][4];
    __shared__ double gwp[2][4];
    __shared__ int pqs[2];
    float *vl = reinterpret_cast<float *>(mrf_bsmem);
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform, and known to be
    const int NWV = blockDim.x >> 6;
    const int lam = wv * 64 + lane;
    const bool valid = lam < L;
    const int lc = valid ? lam : 0;
    const long long N = P.g.N;
    double *gVs = P.gV ? P.gV + (size_t)blockIdx.x * L * L : nullptr;
    const int vzero = mrf_opaque_zero();

    if (P.v_mode == 1)
        for (int e = threadIdx.x; e < L * L; e += blockDim.x) vl[e] = P.V[e];
    else if (P.v_mode == 2)
        for (int e = threadIdx.x; e < L; e += blockDim.x) vl[e] = P.V[e];
    if (threadIdx.x < 8) { (&psum[0][0])[threadIdx.x] = 0.0; (&gwp[0][0])[threadIdx.x] = 0.0; }

    for (long long sl = blockIdx.x; sl < P.total_scanlines; sl += gridDim.x) {
        int ri = 0;
        while (ri + 1 < P.r_count && sl >= P.blk_begin[ri + 1]) ++ri;
        const int r = P.r_first + ri;
        const long long local = sl - P.blk_begin[ri];
        const int nsc = P.g.nscan[r];
        const int b = (int)(local / nsc);
        const long long t = local - (long long)b * nsc;
        const int dh = P.g.dh[r], dw = P.g.dw[r];
        int y0, x0, len;
        mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
        const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
        const long long nstep = (long long)dh * P.g.W + dw;
        const double cscale = (double)P.carry_scale[r];
        const bool own_unary = (r == P.unary_dir);
        const bool unary_old = own_unary && !P.unary_init;
        const size_t umul = unary_old ? 1 : 0;
        const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
        const uint8_t *pbase = P.p + (size_t)r * N * L;
        const uint8_t *qbase = P.q + (size_t)r * N;

        const float *src[NS];
        double cG[NS], cT[NS];
        const int nsrc = P.n_src[r];
#pragma unroll
        for (int c = 0; c < NS; ++c) {
            const bool live = c < nsrc;
            const bool isgc = (c == nsrc) && P.use_gc;
            src[c] = live ? P.src_base + (size_t)P.src_dir[r][c] * P.src_stride : P.gc;
            cG[c] = live ? (double)P.coefG[r][c] : (isgc ? 1.0 : 0.0);
            cT[c] = live ? (double)P.coefT[r][c] : (isgc ? 1.0 : 0.0);
        }

        __syncthreads();                       // previous scanline completely done with the copies
        for (int e = lane; e < 256; e += 64) { cp[0][wv][e] = 0.0; cp[1][wv][e] = 0.0; }
        int pv_prev = 0;                       // where this lane scattered in the previous step
        if (valid) P.S[((size_t)r * N + head + (long long)(len - 1) * nstep) * L + lam] = 0.0f;

        float cur[D][NS], nxt[D][NS];
        float ucur[D], unxt[D];
        int pcur[D], pnxt[D], qcur[D], qnxt[D];
        float wcur[D], wnxt[D];
        auto prefetch = [&](float (&dst)[NS], float &udst, int &pdst, int &qdst, float &wdst, int tt) {
            int n = len - 1 - tt;
            n = n > 0 ? n : 0;
            const long long i = head + (long long)n * nstep;
#pragma unroll
            for (int c = 0; c < NS; ++c) dst[c] = src[c][(size_t)i * L + lc];
            udst = P.gunary[((size_t)i * L + lc) * umul];
            pdst = pbase[(size_t)i * L + lc];
            qdst = qbase[(size_t)i + vzero];
            wdst = wbase[(size_t)(i * P.w_mul) + vzero];
        };
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], ucur[u], pcur[u], qcur[u], wcur[u], u);

        double carry = 0.0;
        int par = 0;
        long long gw_node = -1;     // node whose edge-weight gradient parts sit in gwp[par ^ 1]

        for (int t0 = 0; t0 < len; t0 += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) prefetch(nxt[u], unxt[u], pnxt[u], qnxt[u], wnxt[u], t0 + D + u);
#pragma unroll
            for (int u = 0; u < D; ++u) {
                const int tt = t0 + u;
                const bool past = tt >= len;
                const int n = past ? 0 : len - 1 - tt;
                const bool update = !past && n > 0;
                const long long i = head + (long long)n * nstep;
                const long long j = i - nstep;

                double g = carry;
#pragma unroll
                for (int c = 0; c < NS; ++c) g = __builtin_fma(cG[c], (double)cur[u][c], g);
                g = valid ? g : 0.0;
                if (own_unary) {
                    double accT = carry;
#pragma unroll
                    for (int c = 0; c < NS; ++c) accT = __builtin_fma(cT[c], (double)cur[u][c], accT);
                    accT += unary_old ? (double)ucur[u] : 0.0;
                    if (!past && valid) P.gunary[(size_t)i * L + lam] = (float)accT;
                }
                const int pv = pcur[u] < L ? pcur[u] : L - 1;
                int qv = __builtin_amdgcn_readfirstlane(qcur[u]);
                qv = qv < L ? qv : L - 1;

                if (valid) __hip_atomic_fetch_add(&cp[par][wv][pv], g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                const double part = mrf_wave_sum_f64(g);
                if (lane == 0) psum[par][wv] = part;
                if (lam == qv) pqs[par] = pv;
                mrf_block_sync_lds();

                // edge-weight gradient of the previous node: parts in wavefront order
                if (P.gw && wv == 0 && lane == 0 && gw_node >= 0) {
                    const double a = ((gwp[par ^ 1][0] + gwp[par ^ 1][1]) + gwp[par ^ 1][2]) + gwp[par ^ 1][3];
                    __hip_atomic_fetch_add(&P.gw[(size_t)r * N + gw_node], (float)a, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                }
                // back Eq. isgmr-norm: g(q) -= sum_lambda g(lambda); the target p(q) loses the sum
                const double tot = ((psum[par][0] + psum[par][1]) + psum[par][2]) + psum[par][3];
                const int pq = pqs[par];
                double sv = 0.0;
#pragma unroll
                for (int w2 = 0; w2 < 4; ++w2)
                    if (w2 < NWV) sv += cp[par][w2][lam];
                if (lam == pq) sv -= tot;
                const double gn = (lam == qv) ? g - tot : g;
                if (update && valid) P.S[((size_t)r * N + j) * L + lam] = (float)sv;
                carry = cscale * sv;
                // own copy of the other set: its readers are past the barrier, clear what was touched
                cp[par ^ 1][wv][pv_prev] = 0.0;
                pv_prev = pv;

                const double wgt = (double)wcur[u];
                if (P.gw) {
                    double acc = 0.0;
                    if (valid) {
                        float vv;
                        if (VG) {
                            vv = P.V[(size_t)__mul24(pv, L) + lam];
                        } else {
                            const int dist = pv > lam ? pv - lam : lam - pv;
                            vv = vl[P.v_mode == 1 ? __mul24(pv, L) + lam : dist];
                        }
                        acc = gn * (double)vv;
                    }
                    acc = mrf_wave_sum_f64(acc);
                    if (lane == 0) gwp[par][wv] = acc;
                    gw_node = update ? i : -1;
                }
                if (gVs && update && valid)
                    __hip_atomic_fetch_add(&gVs[(size_t)__mul24(pv, L) + lam], wgt * gn, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                par ^= 1;
            }
#pragma unroll
            for (int u = 0; u < D; ++u) {
                qcur[u] = qnxt[u];
                wcur[u] = wnxt[u];
                ucur[u] = unxt[u];
                pcur[u] = pnxt[u];
#pragma unroll
                for (int c = 0; c < NS; ++c) cur[u][c] = nxt[u][c];
            }
        }
        if (P.gw) {
            __syncthreads();
            if (wv == 0 && lane == 0 && gw_node >= 0) {
                const double a = ((gwp[par ^ 1][0] + gwp[par ^ 1][1]) + gwp[par ^ 1][2]) + gwp[par ^ 1][3];
                __hip_atomic_fetch_add(&P.gw[(size_t)r * N + gw_node], (float)a, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// ---- index replay for few labels: several scanlines per wavefront ---------------------------
//
// Counterpart of mrf_fwd_sweep_packed: the wavefront is cut into 64/SEG segments of SEG >= L
// lanes, each replaying its own scanline (any direction, any length).  Label sums are DPP
// row sums (plus one swizzle for 32-lane segments), the scatter vector and the V-gradient
// accumulator are per segment in LDS.
// sum over a segment of 21 lanes (three per wavefront, see mrf_seg21_upper): the upper and the lower
// lanes of every row are summed apart, the previous row's upper sum joins this row's lower sum,
// and the upper lanes fetch the result from the row after theirs; a fixed order
__device__ inline double mrf_segment_sum21_f64(double v, int lane)
{
    const bool up = mrf_seg21_upper(lane);
    double u = up ? v : 0.0, lo = up ? 0.0 : v;
    u += mrf_dpp_f64<0xB1>(u);
    lo += mrf_dpp_f64<0xB1>(lo);
    u += mrf_dpp_f64<0x4E>(u);
    lo += mrf_dpp_f64<0x4E>(lo);
    u += mrf_dpp_f64<0x141>(u);
    lo += mrf_dpp_f64<0x141>(lo);
    u += mrf_dpp_f64<0x140>(u);
    lo += mrf_dpp_f64<0x140>(lo);
    const long long ub = __builtin_bit_cast(long long, u);
    // row_bcast:15 into rows 1..3, zero for row 0
    const int plo = __builtin_amdgcn_update_dpp(0, (int)(ub & 0xffffffffLL), 0x142, 0xE, 0xF, false);
    const int phi = __builtin_amdgcn_update_dpp(0, (int)(ub >> 32), 0x142, 0xE, 0xF, false);
    const double full = lo + __builtin_bit_cast(double, ((long long)phi << 32) | (long long)(unsigned)plo);
    const int from = (up ? ((lane & 48) + 16) & 63 : lane) << 2;
    const long long fb = __builtin_bit_cast(long long, full);
    const int rlo = __builtin_amdgcn_ds_bpermute(from, (int)(fb & 0xffffffffLL));
    const int rhi = __builtin_amdgcn_ds_bpermute(from, (int)(fb >> 32));
    return __builtin_bit_cast(double, ((long long)rhi << 32) | (long long)(unsigned)rlo);
}

template <int SEG>
__device__ inline double mrf_segment_sum_f64(double v)
{
    if (SEG == 21) return mrf_segment_sum21_f64(v, (int)(threadIdx.x & 63));
    v += mrf_dpp_f64<0xB1>(v);
    v += mrf_dpp_f64<0x4E>(v);
    v += mrf_dpp_f64<0x141>(v);
    v += mrf_dpp_f64<0x140>(v);
    if (SEG == 32) {
        const long long b = __builtin_bit_cast(long long, v);
        const int lo = __builtin_amdgcn_ds_swizzle((int)(b & 0xffffffffLL), 0x401F);
        const int hi = __builtin_amdgcn_ds_swizzle((int)(b >> 32), 0x401F);
        v += __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
    }
    return v;
}

// UNARY = false: no direction of the launch forms grad theta_i (ISGMR with its combine passes)
template <int SEG, int NS, int D, bool UNARY = true>
__global__ void __launch_bounds__(64) mrf_bwd_sweep_packed(const MrfBwdParams P)
{
    constexpr int NSEG = 64 / SEG;
    extern __shared__ __align__(16) unsigned char mrf_bsmem[];
    const int L = P.g.L;
    const int lane = threadIdx.x;
    // (three segments of 21 lanes leave lane 63 over: it shadows the last segment and stores nothing)
    const bool lane_on = lane / SEG < NSEG;
    const int seg = lane_on ? lane / SEG : NSEG - 1, lam = lane % SEG;
    const bool valid = lane_on && lam < L;
    const int lc = valid ? lam : 0;
    const long long N = P.g.N;
    double *sbuf = reinterpret_cast<double *>(mrf_bsmem) + seg * SEG;                       // [NSEG][SEG]
    double *gvl = reinterpret_cast<double *>(mrf_bsmem) + NSEG * SEG + (P.gV ? seg * L * L : 0);  // [NSEG][L*L]
    float *vl = reinterpret_cast<float *>(reinterpret_cast<double *>(mrf_bsmem) + NSEG * SEG + (P.gV ? NSEG * L * L : 0));
    double *gVs = P.gV ? P.gV + ((size_t)blockIdx.x * NSEG + seg) * L * L : nullptr;

    for (int e = lane; e < L * L; e += 64) vl[e] = P.V[e];
    if (gVs && lane_on)
        for (int e = lam; e < L * L; e += SEG) gvl[e] = 0.0;
    sbuf[lam] = 0.0;
    __syncthreads();

    const bool any_unary = UNARY && P.unary_dir >= P.r_first && P.unary_dir < P.r_first + P.r_count;
    const long long npacks = (P.total_scanlines + NSEG - 1) / NSEG;
    for (long long pk = blockIdx.x; pk < npacks; pk += gridDim.x) {
        const long long sl = pk * NSEG + seg;
        const bool act_seg = lane_on && sl < P.total_scanlines;

        int r = P.r_first, nsc = 1, dh = 0, dw = 1, nsrc = 0;
        long long local = 0;
        float cscale_f = 1.0f;
        int sdir[NS];
        float cGf[NS], cTf[NS];
#pragma unroll
        for (int c = 0; c < NS; ++c) { sdir[c] = 0; cGf[c] = 0.0f; cTf[c] = 0.0f; }
        for (int ri = 0; ri < P.r_count; ++ri) {
            const int rr = P.r_first + ri;
            const bool mine = act_seg && sl >= P.blk_begin[ri] && sl < P.blk_begin[ri + 1];
            if (mine) {
                r = rr; local = sl - P.blk_begin[ri]; nsc = P.g.nscan[rr]; dh = P.g.dh[rr]; dw = P.g.dw[rr];
                cscale_f = P.carry_scale[rr]; nsrc = P.n_src[rr];
#pragma unroll
                for (int c = 0; c < NS; ++c) { sdir[c] = P.src_dir[rr][c]; cGf[c] = P.coefG[rr][c]; cTf[c] = P.coefT[rr][c]; }
            }
        }
        int y0 = 0, x0 = 0, len = 1;
        long long head = 0;
        if (act_seg) {
            const int b = (int)(local / nsc);
            const long long t = local - (long long)b * nsc;
            mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
            head = ((long long)b * P.g.H + y0) * P.g.W + x0;
        }
        const long long nstep = (long long)dh * P.g.W + dw;
        const double cscale = (double)cscale_f;
        const bool own_unary = UNARY && act_seg && (r == P.unary_dir);
        const bool unary_old = own_unary && !P.unary_init;
        const size_t umul = unary_old ? 1 : 0;
        const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
        const uint8_t *pbase = P.p + (size_t)r * N * L;
        const uint8_t *qbase = P.q + (size_t)r * N;

        const float *src[NS];
        double cG[NS], cT[NS];
#pragma unroll
        for (int c = 0; c < NS; ++c) {
            const bool live = c < nsrc;
            const bool isgc = (c == nsrc) && P.use_gc;
            src[c] = live ? P.src_base + (size_t)sdir[c] * P.src_stride : P.gc;
            cG[c] = live ? (double)cGf[c] : (isgc ? 1.0 : 0.0);
            cT[c] = live ? (double)cTf[c] : (isgc ? 1.0 : 0.0);
        }
        if (act_seg && valid) P.S[((size_t)r * N + head + (long long)(len - 1) * nstep) * L + lam] = 0.0f;

        int maxlen = 1;
#pragma unroll
        for (int sg = 0; sg < NSEG; ++sg) {
            const int l2 = __builtin_amdgcn_readlane(len, sg * SEG);
            maxlen = l2 > maxlen ? l2 : maxlen;
        }

        float cur[D][NS], nxt[D][NS];
        float ucur[D], unxt[D];
        int pcur[D], pnxt[D], qcur[D], qnxt[D];
        float wcur[D], wnxt[D];
        auto prefetch = [&](float (&dst)[NS], float &udst, int &pdst, int &qdst, float &wdst, int tt) {
            int n = len - 1 - tt;
            n = n > 0 ? n : 0;
            const long long i = head + (long long)n * nstep;
#pragma unroll
            for (int c = 0; c < NS; ++c) dst[c] = src[c][(size_t)i * L + lc];
            if constexpr (UNARY) udst = P.gunary[((size_t)i * L + lc) * umul]; else udst = 0.0f;
            pdst = pbase[(size_t)i * L + lc];
            qdst = qbase[(size_t)i];
            wdst = wbase[(size_t)(i * P.w_mul)];
        };
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], ucur[u], pcur[u], qcur[u], wcur[u], u);

        double carry = 0.0;
        for (int t0 = 0; t0 < maxlen; t0 += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) prefetch(nxt[u], unxt[u], pnxt[u], qnxt[u], wnxt[u], t0 + D + u);
            // What arrives from elsewhere, and its label sums, for the D nodes of the group at once
            // (independent reductions overlap).  The label sum of g = carry + ext is the label sum
            // of ext: the scattered vector of a node sums to zero, because the reparametrisation took
            // exactly its sum off one entry, hence so does the carry (up to double rounding).
            double ext[D], tot[D];
#pragma unroll
            for (int u = 0; u < D; ++u) {
                double e = 0.0;
#pragma unroll
                for (int c = 0; c < NS; ++c) e = __builtin_fma(cG[c], (double)cur[u][c], e);
                ext[u] = valid ? e : 0.0;
            }
#pragma unroll
            for (int u = 0; u < D; ++u) tot[u] = mrf_segment_sum_f64<SEG>(ext[u]);
#pragma unroll
            for (int u = 0; u < D; ++u) {
                const int tt = t0 + u;
                const bool past = !act_seg || tt >= len;
                const int n = past ? 0 : len - 1 - tt;
                const bool update = !past && n > 0;
                const long long i = head + (long long)n * nstep;
                const long long j = i - nstep;

                double g = valid ? carry + ext[u] : 0.0;
                if constexpr (UNARY) if (any_unary) {        // (uniform) some scanline of this launch forms grad theta
                    double accT = carry;
#pragma unroll
                    for (int c = 0; c < NS; ++c) accT = __builtin_fma(cT[c], (double)cur[u][c], accT);
                    accT += unary_old ? (double)ucur[u] : 0.0;
                    if (own_unary && !past && valid) P.gunary[(size_t)i * L + lam] = (float)accT;
                }
                const int pv = pcur[u] < L ? pcur[u] : L - 1;
                const int qv = qcur[u] < L ? qcur[u] : L - 1;
                // back Eq. isgmr-norm: g(q) -= sum_lambda g(lambda)
                if (lam == qv) g = g - tot[u];

                if (valid) __hip_atomic_fetch_add(&sbuf[pv], g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                mrf_wave_lds_fence();
                const double sv = sbuf[lam];
                mrf_wave_lds_fence();
                sbuf[lam] = 0.0;
                if (update && valid) P.S[((size_t)r * N + j) * L + lam] = (float)sv;
                carry = cscale * sv;

                const double wgt = (double)wcur[u];
                if (P.gw) {
                    double acc = valid ? g * (double)vl[__mul24(pv, L) + lc] : 0.0;
                    acc = mrf_segment_sum_f64<SEG>(acc);
                    if (update && lam == 0)
                        __hip_atomic_fetch_add(&P.gw[(size_t)r * N + i], (float)acc, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                }
                if (gVs && update && valid) gvl[__mul24(pv, L) + lam] = __builtin_fma(wgt, g, gvl[__mul24(pv, L) + lam]);
            }
#pragma unroll
            for (int u = 0; u < D; ++u) {
                qcur[u] = qnxt[u];
                wcur[u] = wnxt[u];
                ucur[u] = unxt[u];
                pcur[u] = pnxt[u];
#pragma unroll
                for (int c = 0; c < NS; ++c) cur[u][c] = nxt[u][c];
            }
        }
    }
    if (gVs) {
        mrf_wave_lds_fence();
        if (lane_on)
            for (int e = lam; e < L * L; e += SEG) gVs[e] += gvl[e];
    }
}

// ---- the chain layout for up to 32 labels: two scanlines per workgroup -------------------------
//
// mrf_bwd_sweep_chain with the lanes of every wavefront divided as in mrf_bwd_sweep_packed: lanes 0-31 hold
// the labels of one scanline, lanes 32-63 those of the next (one direction per launch, so everything but the
// head and the length of the scanline is shared).  Ring entries are indexed by lane; a scatter target is
// stored as 32 seg + p, so the chain wavefront's step is that of mrf_bwd_sweep_chain unchanged: it neither
// knows nor cares that its 64 entries are two vectors.  A scanline that is shorter than its neighbour gets
// zeros with targets of their own for the steps past its first node, and nothing of those steps is stored.
// For launches of more than 1,024 scanlines of up to 32 labels with one direction (TRWP), where
// mrf_bwd_sweep_packed leaves a lone wavefront per SIMD to do all of a node's work in sequence.
__host__ __device__ inline size_t mrf_bwd_chain_pk_lds_bytes(int NI, int L, bool gv)
{
    const size_t NR = 2 * (size_t)NI, LL = 64;
    const size_t arrays = sizeof(double) * (3 * NR * LL + LL + (gv ? (size_t)2 * L * L : 0)) +
                          sizeof(float) * (NR * LL + (size_t)L * L) + sizeof(int) * (MRF_CHAIN_MAX_HELPERS + 4) + NR * LL;
    return (arrays + 7) / 8 * 8 + sizeof(MrfWaitBlock);
}

template <int NS, int D, int NI, bool GV>
__global__ void __launch_bounds__(64 * (1 + NI)) mrf_bwd_sweep_chain_pk(const MrfBwdParams P)
{
    constexpr int NR = 2 * NI;
    constexpr int LL = 64;
    static_assert(NI >= 2 && NI <= MRF_CHAIN_MAX_HELPERS, "helpers per pair of scanlines");
    extern __shared__ __align__(16) unsigned char mrf_bsmem[];
    const int L = P.g.L;
    // carved in the order of mrf_bwd_chain_pk_lds_bytes
    double *a_ext = reinterpret_cast<double *>(mrf_bsmem);       // [NR][LL] pre -> chain, post
    double *b_cin = a_ext + NR * LL;                             // [NR][LL] chain -> post: carry that entered the node
    double *b_sv = b_cin + NR * LL;                              // [NR][LL]                scattered vector that left it
    double *sbuf = b_sv + NR * LL;                               // [LL] scatter target of the chain
    double *gvacc = sbuf + LL;                                   // [2][L*L] V-gradient tables of the two scanlines (GV): LDS adds by all helpers
    float *a_extT = reinterpret_cast<float *>(gvacc + (GV ? 2 * L * L : 0));   // [NR][LL] pre -> post (grad theta)
    float *vl = a_extT + NR * LL;                                // [L*L] V
    int *pre_done = reinterpret_cast<int *>(vl + L * L);         // [MRF_CHAIN_MAX_HELPERS] per helper: last step published
    int *chain_done = pre_done + MRF_CHAIN_MAX_HELPERS;          // last step the chain finished
    uint8_t *a_p = reinterpret_cast<uint8_t *>(chain_done + 4);  // [NR][LL]
    MrfWaitBlock &wait_lds = *reinterpret_cast<MrfWaitBlock *>(
        mrf_bsmem + ((a_p + NR * LL - mrf_bsmem) + 7) / 8 * 8);
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int seg = lane >> 5, lam = lane & 31;
    const bool valid = lam < L;
    const int lc = valid ? lam : 0;
    const long long N = P.g.N;

    for (int e = threadIdx.x; e < L * L; e += blockDim.x) vl[e] = P.V[e];
    if (GV)
        for (int e = threadIdx.x; e < 2 * L * L; e += blockDim.x) gvacc[e] = 0.0;
    if (threadIdx.x < MRF_CHAIN_MAX_HELPERS) pre_done[threadIdx.x] = (int)threadIdx.x - NI;
    if (threadIdx.x == 0) { *chain_done = -1; chain_done[1] = 0; mrf_wait_init(&wait_lds, P.fault, P.spin_limit); }
    for (int e = threadIdx.x; e < LL; e += blockDim.x) sbuf[e] = 0.0;
    __syncthreads();

    // one direction per launch; the two scanlines of the workgroup
    const int r = P.r_first;
    const long long sl = (long long)blockIdx.x * 2 + seg;
    const bool act_seg = sl < P.total_scanlines;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0 = 0, x0 = 0, len = 0;
    long long head = 0;
    if (act_seg) {
        const int nsc = P.g.nscan[r];
        const int b = (int)(sl / nsc);
        const long long t = sl - (long long)b * nsc;
        mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
        head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    }
    const long long nstep = (long long)dh * P.g.W + dw;
    const int len0 = __builtin_amdgcn_readlane(len, 0), len1 = __builtin_amdgcn_readlane(len, 32);
    const int maxlen = len0 > len1 ? len0 : len1;

    if (wv == 0) {
        // ---- the chain: step tt handles node len-1-tt of either scanline (mrf_bwd_sweep_chain's step) ----
        const double cscale = (double)P.carry_scale[r];
        double carry = 0.0, ext;
        int pv;
        auto await = [&](int u, int tt) {
            int sn;
            int wait_turns = 0;
            do {
                sn = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&pre_done[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                if (sn < tt) mrf_wait_turn(&wait_lds, wait_turns);
            } while (sn < tt);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        };
        if (maxlen > 0) {
            await(0, 0);
            ext = a_ext[lane];
            pv = a_p[lane];
        } else {
            ext = 0.0;
            pv = lane;
        }
        int sb = 0;
        for (int t0 = 0; t0 < maxlen; t0 += NI) {
#pragma unroll
            for (int u = 0; u < NI; ++u) {
                const int tt = t0 + u;
                if (tt < maxlen) {
                    const int slot = sb + u;
                    const int un = (u + 1 == NI) ? 0 : u + 1;
                    const int slotn = (u + 1 == NI) ? (sb == 0 ? NI : 0) : slot + 1;
                    const bool more = tt + 1 < maxlen;
                    const double g = carry + ext;
                    b_cin[slot * LL + lane] = carry;
                    __hip_atomic_fetch_add(&sbuf[pv], g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    mrf_wave_lds_fence();
                    const int flag = __hip_atomic_load(&pre_done[un], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    ext = a_ext[slotn * LL + lane];
                    pv = a_p[slotn * LL + lane];
                    const double sv = sbuf[lane];
                    if (__builtin_expect(more && __builtin_amdgcn_readfirstlane(flag) < tt + 1, 0)) {
                        await(un, tt + 1);
                        ext = a_ext[slotn * LL + lane];
                        pv = a_p[slotn * LL + lane];
                    }
                    // everything this wavefront sent to LDS before the reads above has landed
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
                    __builtin_amdgcn_wave_barrier();
                    if (tt > 0)
                        __hip_atomic_store(chain_done, tt - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    sbuf[lane] = 0.0;
                    b_sv[slot * LL + lane] = sv;
                    carry = cscale * sv;
                }
            }
            sb = (sb == 0) ? NI : 0;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) __hip_atomic_store(chain_done, maxlen - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return;
    }

    // ---- helpers ---------------------------------------------------------------------------
    const int jw = wv - 1;
    const bool own_unary = (r == P.unary_dir);
    const bool unary_old = own_unary && !P.unary_init;
    const uint8_t *pbase = P.p + (size_t)r * N * L;
    const uint8_t *qbase = P.q + (size_t)r * N;
    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);

    const float *src[NS];
    double cG[NS], cT[NS];
    const int nsrc = P.n_src[r];
#pragma unroll
    for (int c = 0; c < NS; ++c) {
        const bool live = c < nsrc;
        const bool isgc = (c == nsrc) && P.use_gc;
        src[c] = live ? P.src_base + (size_t)P.src_dir[r][c] * P.src_stride : P.gc;
        cG[c] = live ? (double)P.coefG[r][c] : (isgc ? 1.0 : 0.0);
        cT[c] = live ? (double)P.coefT[r][c] : (isgc ? 1.0 : 0.0);
    }

    // the last node of a scanline has no successor in direction r
    if (jw == 0 && act_seg && valid && len > 0)
        P.S[((size_t)r * N + head + (long long)(len - 1) * nstep) * L + lam] = 0.0f;

    // own steps: tt = jw + it * NI, it = 0 .. T-1; one more turn for the last post
    const int T = maxlen > jw ? (maxlen - jw + NI - 1) / NI : 0;
    float cur[D][NS], nxt[D][NS];
    float ucur[D], unxt[D];
    int pcur[D], pnxt[D], qcur[D], qnxt[D];
    float wcur[D], wnxt[D];                 // edge weight of the node's incoming edge (GV)
    auto prefetch = [&](float (&dst)[NS], float &udst, int &pdst, int &qdst, float &wdst, int it) {
        int n = len - 1 - (jw + it * NI);
        n = n > 0 ? n : 0;
        const long long i = head + (long long)n * nstep;
#pragma unroll
        for (int c = 0; c < NS; ++c) dst[c] = src[c][(size_t)i * L + lc];
        udst = P.gunary[unary_old ? (size_t)i * L + lc : 0];      // one cached word unless it is needed
        pdst = pbase[(size_t)i * L + lc];
        qdst = qbase[(size_t)i];
        wdst = GV ? wbase[(size_t)(i * P.w_mul)] : 0.0f;
    };
    if (T > 0) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], ucur[u], pcur[u], qcur[u], wcur[u], u);
    }
    double *gvl = gvacc + (GV ? seg * L * L : 0);
    float wlast = 0.0f;                     // weight of the node whose post stage comes next

    int chain_seen = -1;
    for (int it0 = 0; it0 < T + 1 && T > 0; it0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], unxt[u], pnxt[u], qnxt[u], wnxt[u], it0 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int tt = jw + (it0 + u) * NI;
            if (tt < maxlen) {
                // ---- pre(tt): everything of node len-1-tt that does not need the carry -------
                const int slot = tt % NR;
                const bool live = valid && tt < len;       // (false for the whole of a scanline that has ended)
                double e = 0.0, eT = 0.0;
#pragma unroll
                for (int c = 0; c < NS; ++c) e = __builtin_fma(cG[c], (double)cur[u][c], e);
                if (own_unary) {
#pragma unroll
                    for (int c = 0; c < NS; ++c) eT = __builtin_fma(cT[c], (double)cur[u][c], eT);
                    eT += unary_old ? (double)ucur[u] : 0.0;     // (the buffer may hold anything at first)
                    a_extT[slot * LL + lane] = (float)eT;
                }
                const double ev = live ? e : 0.0;
                // (labels past L and scanlines that have ended scatter their zeros to entries of their own)
                a_p[slot * LL + lane] = (uint8_t)(live ? 32 * seg + (pcur[u] < L ? pcur[u] : L - 1) : lane);
                // back Eq. isgmr-norm, on the part of g that is known here: the entry at q loses the label sum
                const double tot = mrf_segment_sum_f64<32>(ev);
                const int qv = qcur[u] < L ? qcur[u] : L - 1;
                a_ext[slot * LL + lane] = (live && lam == qv) ? ev - tot : ev;
                // (LDS keeps a wavefront's operations in order: the counter lands behind the entries)
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                if (lane == 0) __hip_atomic_store(&pre_done[jw], tt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            const int tp = tt - NI;
            if (tp >= 0 && tp < maxlen) {
                // ---- post(tp): what is left of node len-1-tp once the chain has passed --------
                int wait_turns = 0;
                while (chain_seen < tp) {
                    chain_seen = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(chain_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                    if (chain_seen < tp) mrf_wait_turn(&wait_lds, wait_turns);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                const int slot = tp % NR;
                const int n = len - 1 - tp;
                const bool act = valid && n >= 0;        // the node exists
                const bool update = valid && n > 0;      // and has a predecessor: its update is replayed
                const long long i = head + (long long)(n > 0 ? n : 0) * nstep;
                const double cin = b_cin[slot * LL + lane];
                if (own_unary && act) P.gunary[(size_t)i * L + lam] = (float)(cin + (double)a_extT[slot * LL + lane]);
                if (update) P.S[((size_t)r * N + i - nstep) * L + lam] = (float)b_sv[slot * LL + lane];
                if (P.gw || GV) {
                    const double g = cin + a_ext[slot * LL + lane];    // as the chain formed it
                    const int pv = update ? (int)a_p[slot * LL + lane] - 32 * seg : 0;
                    if (P.gw) {
                        double acc = update ? g * (double)vl[__mul24(pv, L) + lam] : 0.0;
                        acc = mrf_segment_sum_f64<32>(acc);
                        // one writer per entry and launch: a no-return atomic is a plain accumulate
                        if (n > 0 && lam == 0)
                            __hip_atomic_fetch_add(&P.gw[(size_t)r * N + i], (float)acc, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if (GV && update)
                        __hip_atomic_fetch_add(&gvl[__mul24(pv, L) + lam], (double)wlast * g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
            wlast = wcur[u];
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            qcur[u] = qnxt[u];
            wcur[u] = wnxt[u];
            ucur[u] = unxt[u];
            pcur[u] = pnxt[u];
#pragma unroll
            for (int c = 0; c < NS; ++c) cur[u][c] = nxt[u][c];
        }
    }
    if (GV) {
        // the helper that finishes last adds the two tables to the workgroup's two slots
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_wave_barrier();
        int before = 0;
        if (lane == 0) before = __hip_atomic_fetch_add(&chain_done[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        before = __builtin_amdgcn_readfirstlane(before);
        if (before == NI - 1) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            double *gVs = P.gV + ((size_t)blockIdx.x * 2 + seg) * L * L;
            if (valid)
                for (int e = lam; e < L * L; e += L) gVs[e] += gvl[e];
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
    float *ghat;             // [R][N][L] out (next iteration's grad m-hat), NULL on the last; only the slabs of
                             // directions d with canon[d] == d are written
    int canon[MRF_MAXR];     // a direction and its opposite exclude the same pair {d, d-}, so their grad m-hat
                             // is one and the same array: canon[d] = the lower index of the two
    int first;               // first processed iteration: grad theta starts from grad c
    int skip_dir;            // direction whose s does not enter the sums (already added elsewhere), or -1
};

// RT: number of directions rounded up to 4, 8 or 16 (the loops below are unrolled to it);
// VEC: consecutive entries per thread (4 needs N*L divisible by 4 and 16-byte aligned arrays)
template <int RT, int VEC>
__global__ void __launch_bounds__(256) mrf_isgmr_bwd_combine(const MrfCombineParams P)
{
    typedef float vecf __attribute__((ext_vector_type(VEC)));
    const long long stride = (long long)gridDim.x * blockDim.x * VEC;
    for (long long e = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * VEC; e < P.NL; e += stride) {
        // every s^r_i is read once; sums are formed in double, where removing the two excluded
        // directions from the total loses nothing that float storage would keep
        vecf sraw[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r)
            sraw[r] = (r < P.R) ? *reinterpret_cast<const vecf *>(P.S + (size_t)r * P.NL + e) : vecf(0.0f);
        const vecf braw = *reinterpret_cast<const vecf *>((P.first ? P.gc : P.gunary) + e);
        vecf uout;
        vecf gout[RT];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            double sv[RT];
            double tot = 0.0;
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                sv[r] = (r == P.skip_dir) ? 0.0 : (double)sraw[r][v];
                tot += sv[r];
            }
            uout[v] = (float)((double)braw[v] + tot);
#pragma unroll
            for (int d = 0; d < RT; ++d) {
                double g = tot - sv[d];
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    if (r == P.opp[d]) g -= sv[r];
                gout[d][v] = (float)g;
            }
        }
        *reinterpret_cast<vecf *>(P.gunary + e) = uout;
        if (P.ghat) {
#pragma unroll
            for (int d = 0; d < RT; ++d)
                if (d < P.R && P.canon[d] == d) *reinterpret_cast<vecf *>(P.ghat + (size_t)d * P.NL + e) = gout[d];
        }
    }
}

// Reduction of the wavefront-private V-gradient accumulators in a fixed order, two levels:
// first every chunk of `chunk` consecutive slots is summed into its first slot, then the
// chunk heads are summed into the output.
__global__ void __launch_bounds__(256) mrf_reduce_slot_chunks(double *buf, long long n, long long slots, long long chunk)
{
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    const long long first = (long long)blockIdx.y * chunk;
    const long long last = first + chunk < slots ? first + chunk : slots;
    double v = 0.0;
    for (long long s = first; s < last; ++s) v = v + buf[(size_t)s * n + e];
    buf[(size_t)first * n + e] = v;
}

__global__ void __launch_bounds__(256) mrf_reduce_slot_heads(const double *buf, float *dst, long long n, long long slots, long long chunk)
{
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    double v = 0.0;
    for (long long s = 0; s < slots; s += chunk) v = v + buf[(size_t)s * n + e];
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
