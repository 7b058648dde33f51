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
//
// The node-to-node dependence makes a sweep latency bound, so everything that does not
// depend on the previous node (unary, other directions' messages, edge weight) is loaded
// a group of D nodes ahead into a second register set, unconditionally (clamped
// addresses), so that a load is first waited for at least D node steps after its issue.
//
// Kernels in this file, all computing the same update in the same rounding order:
//   mrf_fwd_sweep               dense O(L^2), NW wavefronts per scanline split the source labels
//   mrf_fwd_sweep_sliced        dense, L > 64: the same with the O(L) work of a node divided among the wavefronts
//   mrf_fwd_sweep_packed        dense, L <= 32: several scanlines per wavefront
//   mrf_fwd_sweep_edge          pairwise potentials given per edge (L <= 64)
//   mrf_aggregate               final costs and labels
//   mrf_fwd_sweep_window        truncated models: window of 2 TW - 1 source labels per label
//   mrf_fwd_sweep_window_duo    the same with the dependency chain (values) on one wavefront and
//                               index / loader wavefronts beside it, connected by LDS rings
//   mrf_fwd_sweep_window_split  the same, one wavefront per 64 labels in lock step
//   mrf_fwd_sweep_window_squad  value wavefronts per 64 labels plus index wavefronts per node
// Which one a launch gets is host arithmetic on the launch shape (dispatch_fwd).
#pragma once

#include "mrfmp_device.h"

struct MrfFwdParams {
    MrfGeom g;
    int r_first, r_count;                  // directions swept by this launch
    long long blk_begin[MRF_MAXR + 1];     // prefix sums of B*nscan over those directions
    const float *unary, *V;
    const float *w;                        // [R][N] edge weights, or one float when w_mul == 0
    int w_mul;                             // 1: per-edge weights, 0: the scalar at w[0]
    const float *m_in;                     // [R][N][L] messages read
    float *m_out;                          // [R][N][L] messages written (TRWP: same array)
    uint8_t *p, *q;                        // [R][N][L], [R][N] of this iteration
    float rho[MRF_MAXR];
    const float *rho_e;                    // [R][N] rho of edge (i-r, i) at node i (TRWP), or NULL: then rho[] applies
                                           // (read by mrf_fwd_sweep, mrf_fwd_sweep_window and mrf_fwd_sweep_edge only)
    const float *Te;                       // [R][N][L][L] pairwise potentials per edge (mrf_fwd_sweep_edge), or NULL
    // per swept direction r: the message arrays that enter h, in summation order.  The first
    // n_pre[r] are added before this direction's own running message, the rest after it.
    signed char src_dir[MRF_MAXR][MRF_MAXR];
    signed char n_pre[MRF_MAXR], n_src[MRF_MAXR];
    signed char rm_slot[MRF_MAXR];         // position of r^- in src_dir[r], or -1 (term absent / still 0)
    int NW;                                // wavefronts per workgroup = ceil(L / MCH)
    int *fault;                            // launch-wide word raised when a wait between wavefronts is given up (mrf_wait_turn)
    int spin_limit;                        // microseconds after which a wait is given up
    signed char unary_slab[MRF_MAXR];      // direction r reads its lambda-independent start term at
                                           // unary + unary_slab[r] * N * L (0 unless mrf_isgmr_presum prepared them)
    int sgm_std;                           // standard single-pass SGM (Eq. sgm_old): the message carries the node's own
                                           // unary, m^r_i = theta_i + min_mu (m^r_{i-r} + theta_{i-r,i}); mrf_fwd_sweep only
};

// LP: labels per lane; MCH: source labels per wavefront; RMAX: bound on 1 + n_src;
// D: prefetch distance in nodes; TRWP: Eq. trwp (else Eq. isgmr)
template <int LP, int MCH, int RMAX, int D, bool TRWP>
__global__ void __launch_bounds__(64 * ((64 * LP + MCH - 1) / MCH))
mrf_fwd_sweep(const MrfFwdParams P)
{
    extern __shared__ __align__(16) unsigned char mrf_smem[];
    constexpr int NWMAX = (64 * LP + MCH - 1) / MCH;
    constexpr int LPAD = NWMAX * MCH;
    constexpr int SLOTS = 64 * LP;
    const int L = P.g.L, NW = P.NW;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform, and known to be
    float *hbuf = reinterpret_cast<float *>(mrf_smem) + wv * LPAD;          // private to this wavefront
    float2 *part = reinterpret_cast<float2 *>(reinterpret_cast<float *>(mrf_smem) + NWMAX * LPAD);  // [2][NWMAX][SLOTS]

    // workgroup -> (direction r, image b, scanline t)
    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const float rho = P.rho[r];
    const int n_pre = P.n_pre[r], n_src = P.n_src[r], rm_slot = P.rm_slot[r];

    // Sources of h: slot 0 = unary, slot c >= 1 = message array src_dir[r][c-1].  Unused
    // slots read the unary again and enter with factor 0: fma(0, x, v) = v exactly, and
    // fma(1, x, v) = v + x exactly, so the sum below is the plain left-to-right sum of the
    // live terms with this direction's running message inserted after the first n_pre.
    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    const float vz = mrf_opaque_zero_f();     // keeps the flags below in vector registers
    // standard SGM adds the unary of node i itself after the minimum (Eq. sgm_old): slot 0 then
    // holds theta_i, one node further along the scanline, instead of theta_{i-r}
    const bool sgm_std = !TRWP && P.sgm_std;
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L + (sgm_std ? nstep * L : 0);
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)P.src_dir[r][c - 1] * N * L : src[0];
        use[c] = ((c <= n_src) ? 1.0f : 0.0f) + vz;
        is_rm[c] = ((c - 1 == rm_slot) ? 1.0f : 0.0f) + vz;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = ((c == n_pre + 1) ? 1.0f : 0.0f) + vz;

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
    // padding of h beyond L, and partial minima of absent wavefronts, can never win a strict '<'
    for (int i = L + lane; i < LPAD; i += 64) hbuf[i] = INFINITY;
    if (NWMAX > 1) {
        for (int i = threadIdx.x; i < 2 * NWMAX * SLOTS; i += blockDim.x) part[i] = make_float2(INFINITY, 0.0f);
        __syncthreads();
    }

    // first node of the scanline: message 0, p = q = 0
    if (wv == 0) {
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int lam = lane + 64 * s;
            if (lam < L) {
                // (standard SGM: with nothing before it, the first node's message is its unary)
                P.m_out[((size_t)r * N + head) * L + lam] = sgm_std ? P.unary[(size_t)head * L + lam] : 0.0f;
                P.p[((size_t)r * N + head) * L + lam] = 0;
            }
        }
        if (lane == 0) P.q[(size_t)r * N + head] = 0;
    }

    // Prefetch in groups of D nodes: while the D nodes of one group are processed from the
    // registers `cur`, the inputs of the next group are in flight into `nxt`.
    const int vzero = mrf_opaque_zero();
    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
    const int lastsrc = len - 2;           // last node that is a predecessor
    float cur[D][RMAX][LP], nxt[D][RMAX][LP];
    float wcur[D], wnxt[D];
    float rcur[D], rnxt[D];                // rho of the edge (i-r, i): per edge if P.rho_e is given
    const float *rbase = P.rho_e ? P.rho_e + (size_t)r * N : nullptr;
    auto prefetch = [&](float (&dst)[RMAX][LP], float &wdst, float &rdst, int nj) {   // inputs of the update nj -> nj+1
        nj = nj < lastsrc ? nj : lastsrc;  // past the end: reload the last one, never used
        const long long j = head + (long long)nj * nstep;
#pragma unroll
        for (int c = 0; c < RMAX; ++c)
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                dst[c][s] = src[c][(size_t)j * L + (lam < L ? lam : 0)];
            }
        wdst = wbase[(size_t)((j + nstep) * P.w_mul) + vzero];
        rdst = rho;
        if (TRWP && rbase) rdst = rbase[(size_t)(j + nstep) + vzero];
    };
    if (len >= 2) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u], rcur[u], u);
    }

    float carry[LP];   // normalised message of this direction at the previous node
#pragma unroll
    for (int s = 0; s < LP; ++s)
        carry[s] = (sgm_std && lane + 64 * s < L) ? P.unary[(size_t)head * L + lane + 64 * s] : 0.0f;
    int buf = 0, turn = 0;

    for (int n0 = 1; n0 < len; n0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u], rnxt[u], n0 - 1 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            // node index of i on the scanline; i-r is node n-1.  The last group may run past
            // the end of the scanline: those steps recompute the last node and store nothing.
            const int nn = n0 + u;
            const bool past = nn >= len;
            const int n = past ? len - 1 : nn;
            const long long i = head + (long long)n * nstep;

            // ---- lambda-independent part h[mu] at node i-r (lane's labels act as mu here) ----
            float a[LP];
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                float v = cur[u][0][s];
                float mrm = 0.0f;
                if (TRWP) {
                    // Eq. trwp: rho (theta_{i-r} + sum_d m^d_{i-r}) - m^{r-}_{i-r}
#pragma unroll
                    for (int c = 1; c < RMAX; ++c) {
                        v = __builtin_fmaf(carry_at[c], carry[s], v);
                        v = __builtin_fmaf(use[c], cur[u][c][s], v);
                        mrm = __builtin_fmaf(is_rm[c], cur[u][c][s], mrm);
                    }
                    v = __builtin_fmaf(carry_at[RMAX], carry[s], v);
                    v = rcur[u] * v;
                    v = v - mrm;
                } else {
                    // Eq. isgmr: theta_{i-r} + sum_{d not in {r, r-}} m^d_{i-r} (what iteration k left), then m-hat^r_{i-r}
#pragma unroll
                    for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[u][c][s], v);
                    v = v + carry[s];
                    // Eq. sgm_old: the previous message alone (it holds theta_{i-r} already)
                    v = sgm_std ? carry[s] : v;
                }
                a[s] = v;
            }
            const float wgt = wcur[u];

#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) hbuf[lam] = a[s];
            }
            mrf_wave_lds_fence();

            // ---- min-plus over this wavefront's mu slice, lowest mu on ties ----
            float best[LP];
            int bidx[LP];
#pragma unroll
            for (int s = 0; s < LP; ++s) { best[s] = INFINITY; bidx[s] = 0; }
            // (compares, minima and index selects of the LP label slots go out in blocks that need
            // no wait states: mrf_argmin_step)
            mrf_static_for<MCH / 4>([&](auto q4) {
                constexpr int i4 = 4 * decltype(q4)::value;
                const float4 hv = *reinterpret_cast<const float4 *>(&hbuf[mu0 + i4]);
                const float hq[4] = { hv.x, hv.y, hv.z, hv.w };
                if constexpr (LP == 1) {
                    mrf_argmin_step2<i4>(best[0], bidx[0], __builtin_fmaf(wgt, Vr[i4][0], hq[0]),
                                         __builtin_fmaf(wgt, Vr[i4 + 1][0], hq[1]));
                    mrf_argmin_step2<i4 + 2>(best[0], bidx[0], __builtin_fmaf(wgt, Vr[i4 + 2][0], hq[2]),
                                             __builtin_fmaf(wgt, Vr[i4 + 3][0], hq[3]));
                } else {
                    mrf_static_for<4>([&](auto cc) {
                        constexpr int c = decltype(cc)::value;
                        float dlt[LP];
#pragma unroll
                        for (int s = 0; s < LP; ++s) dlt[s] = __builtin_fmaf(wgt, Vr[i4 + c][s], hq[c]);
                        mrf_argmin_step<i4 + c>(best, bidx, dlt);
                    });
                }
            });

            float tv[LP];
            int tp[LP];
            if (NWMAX > 1) {
                float2 *pb = part + (size_t)buf * NWMAX * SLOTS;
#pragma unroll
                for (int s = 0; s < LP; ++s)
                    pb[wv * SLOTS + lane + 64 * s] = make_float2(best[s], __int_as_float(mu0 + bidx[s]));
                mrf_block_sync_lds();
#pragma unroll
                for (int s = 0; s < LP; ++s) { tv[s] = INFINITY; tp[s] = 0; }
#pragma unroll
                for (int w2 = 0; w2 < NWMAX; ++w2) {
                    float ev[LP];
                    int ei[LP];
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        const float2 e = pb[w2 * SLOTS + lane + 64 * s];
                        ev[s] = e.x;
                        ei[s] = __float_as_int(e.y);
                    }
                    mrf_argmin_merge<LP>(tv, tp, ev, ei);
                }
                buf ^= 1;
            } else {
#pragma unroll
                for (int s = 0; s < LP; ++s) { tv[s] = best[s]; tp[s] = bidx[s]; }
            }

            if (sgm_std) {
#pragma unroll
                for (int s = 0; s < LP; ++s) tv[s] = cur[u][0][s] + tv[s];     // theta_i + min_mu (...)
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
                    tq = mrf_readlane_f32(tv[s], ql);
                }
            }
#pragma unroll
            for (int s = 0; s < LP; ++s) carry[s] = (lane + 64 * s < L) ? tv[s] - tq : 0.0f;

            // ---- outputs of node i (the wavefronts take turns) ----
            if (wv == turn && !past) {
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
            turn = (turn + 1 == NW) ? 0 : turn + 1;
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            wcur[u] = wnxt[u];
            rcur[u] = rnxt[u];
#pragma unroll
            for (int c = 0; c < RMAX; ++c)
#pragma unroll
                for (int s = 0; s < LP; ++s) cur[u][c][s] = nxt[u][c][s];
        }
    }
}

// ---- dense sweep, every wavefront owns a slice of the labels ------------------------------------
//
// The same O(L^2) update as mrf_fwd_sweep for more than 64 labels, with the O(L) work of a node
// divided instead of repeated.  Wavefront w holds rows [32 w, 32 w + 32) of V in registers as
// before and evaluates their candidates for all L destination labels; but only these 32 labels
// are also its "home": it alone loads the inputs of h for them, merges the partial results of all
// wavefronts for them, normalises, keeps the running message for them, and stores them.  (In
// mrf_fwd_sweep every wavefront does all of that for all L labels, so that one barrier per node
// suffices; at L = 256 that is a third of its instructions.)  The price is a second barrier per
// node: the minimum over all labels (Eq. isgmr-norm) is the minimum of the wavefronts' home minima,
// exchanged through LDS.  Home labels sit in 32 consecutive lanes of one label slot (lane + 64 s),
// so loads and stores of a wavefront are 128-byte runs.
//   per node:  h(home) -> private LDS copy -> candidates of the 32 source labels for all lambda
//              -> partial (min, argmin) per lambda to LDS -> barrier -> merge at home, home minimum
//              -> LDS -> barrier -> global minimum, q, running message, stores
// Same arithmetic in the same order as mrf_fwd_sweep: results are bit-identical.
template <int LP, int RMAX, int D, bool TRWP>
__global__ void __launch_bounds__(64 * 2 * LP)
mrf_fwd_sweep_sliced(const MrfFwdParams P)
{
    constexpr int MCH = 32;
    constexpr int NWMAX = 2 * LP;
    constexpr int SLOTS = 64 * LP;
    __shared__ __align__(16) float hbuf_all[NWMAX][MCH];         // h of every wavefront's slice (read by its owner only)
    __shared__ float2 part[NWMAX][SLOTS];                        // partial (min, argmin) of wavefront w for label lambda
    __shared__ float2 hmin[NWMAX];                               // home minimum and its label, per wavefront
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    float *hbuf = hbuf_all[wv];

    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const float rho = P.rho[r];
    const int n_pre = P.n_pre[r], n_src = P.n_src[r], rm_slot = P.rm_slot[r];

    // home label of this lane: lanes [32 (w & 1), +32) of the wavefront hold labels 32 w .. 32 w + 31
    const int mu0 = wv * MCH;
    const bool home_lane = (lane >> 5) == (wv & 1);
    const int hl = mu0 + (lane & 31);                 // home label (meaningful in home lanes)
    const bool home = home_lane && hl < L;
    const int hlc = home ? hl : 0;

    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    const float vz = mrf_opaque_zero_f();
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L;
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)P.src_dir[r][c - 1] * N * L : src[0];
        use[c] = ((c <= n_src) ? 1.0f : 0.0f) + vz;
        is_rm[c] = ((c - 1 == rm_slot) ? 1.0f : 0.0f) + vz;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = ((c == n_pre + 1) ? 1.0f : 0.0f) + vz;

    // rows mu0 .. mu0 + 31 of V, columns = the lane's destination labels
    float Vr[MCH][LP];
#pragma unroll
    for (int i = 0; i < MCH; ++i)
#pragma unroll
        for (int s = 0; s < LP; ++s) {
            const int mu = mu0 + i, lam = lane + 64 * s;
            Vr[i][s] = (mu < L && lam < L) ? P.V[(size_t)mu * L + lam] : 0.0f;
        }
    // entries of h past L never win a strict '<'; wavefronts that are absent (NW < NWMAX) neither
    if (lane < MCH) hbuf[lane] = INFINITY;
    for (int i = threadIdx.x; i < NWMAX * SLOTS; i += blockDim.x) (&part[0][0])[i] = make_float2(INFINITY, 0.0f);
    if (threadIdx.x < NWMAX) hmin[threadIdx.x] = make_float2(INFINITY, 0.0f);
    __syncthreads();

    // first node of the scanline: message 0, p = q = 0
    if (home) {
        P.m_out[((size_t)r * N + head) * L + hl] = 0.0f;
        P.p[((size_t)r * N + head) * L + hl] = 0;
    }
    if (threadIdx.x == 0) P.q[(size_t)r * N + head] = 0;

    const int vzero = mrf_opaque_zero();
    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
    const int lastsrc = len - 2;
    float cur[D][RMAX], nxt[D][RMAX];
    float wcur[D], wnxt[D];
    auto prefetch = [&](float (&dst)[RMAX], float &wdst, int nj) {      // inputs of the update nj -> nj + 1
        nj = nj < lastsrc ? nj : lastsrc;
        const long long j = head + (long long)nj * nstep;
#pragma unroll
        for (int c = 0; c < RMAX; ++c) dst[c] = src[c][(size_t)j * L + hlc];
        wdst = wbase[(size_t)((j + nstep) * P.w_mul) + vzero];
    };
    if (len >= 2) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u], u);
    }

    float carry = 0.0f;        // normalised message of this direction at the previous node, home label

    for (int n0 = 1; n0 < len; n0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u], n0 - 1 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int nn = n0 + u;
            const bool past = nn >= len;
            const int n = past ? len - 1 : nn;
            const long long i = head + (long long)n * nstep;

            // ---- h at node i-r for the home labels (same order of additions as mrf_fwd_sweep) ----
            float v = cur[u][0];
            if (TRWP) {
                float mrm = 0.0f;
#pragma unroll
                for (int c = 1; c < RMAX; ++c) {
                    v = __builtin_fmaf(carry_at[c], carry, v);
                    v = __builtin_fmaf(use[c], cur[u][c], v);
                    mrm = __builtin_fmaf(is_rm[c], cur[u][c], mrm);
                }
                v = __builtin_fmaf(carry_at[RMAX], carry, v);
                v = rho * v;
                v = v - mrm;
            } else {
#pragma unroll
                for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[u][c], v);
                v = v + carry;
            }
            const float wgt = wcur[u];
            if (home) hbuf[lane & 31] = v;
            mrf_wave_lds_fence();

            // ---- candidates of the 32 source labels of this wavefront, for every lambda ----
            float best[LP];
            int bidx[LP];
#pragma unroll
            for (int s = 0; s < LP; ++s) { best[s] = INFINITY; bidx[s] = 0; }
            // (all of the slice's h in one batch of LDS reads: the registers that the divided loads
            // freed pay for it, and the candidates then run without waiting for LDS)
            float hq[MCH];
#pragma unroll
            for (int i4 = 0; i4 < MCH; i4 += 4) {
                const float4 hv = *reinterpret_cast<const float4 *>(&hbuf[i4]);
                hq[i4] = hv.x; hq[i4 + 1] = hv.y; hq[i4 + 2] = hv.z; hq[i4 + 3] = hv.w;
            }
            mrf_static_for<MCH>([&](auto mm) {
                constexpr int m = decltype(mm)::value;
                float dlt[LP];
#pragma unroll
                for (int s = 0; s < LP; ++s) dlt[s] = __builtin_fmaf(wgt, Vr[m][s], hq[m]);
                mrf_argmin_step<m>(best, bidx, dlt);
            });
#pragma unroll
            for (int s = 0; s < LP; ++s)
                part[wv][lane + 64 * s] = make_float2(best[s], __int_as_float(mu0 + bidx[s]));
            mrf_block_sync_lds();

            // ---- merge at home, in ascending source label: the lowest index survives ----
            float tv = INFINITY;
            int tp = 0;
#pragma unroll
            for (int w2 = 0; w2 < NWMAX; ++w2) {
                const float2 e = part[w2][hlc];
                if (e.x < tv) { tv = e.x; tp = __float_as_int(e.y); }
            }
            if (!home) tv = INFINITY;
            // home minimum and the lowest home label that attains it
            const float lmin = mrf_wave_min(tv);
            const unsigned long long lbal = __ballot(tv == lmin);
            const int llab = mu0 + ((__ffsll((long long)lbal) - 1) & 31);
            if (lane == 0) hmin[wv] = make_float2(lmin, __int_as_float(llab));
            mrf_block_sync_lds();

            // ---- global minimum over the labels, q = lowest label attaining it (Eq. isgmr-norm) ----
            float tq = INFINITY;
            int qidx = 0;
#pragma unroll
            for (int w2 = 0; w2 < NWMAX; ++w2) {
                const float2 e = hmin[w2];
                if (e.x < tq) { tq = e.x; qidx = __float_as_int(e.y); }     // ascending wavefront = ascending label
            }
            carry = home ? tv - tq : 0.0f;

            if (!past) {
                if (home) {
                    P.m_out[((size_t)r * N + i) * L + hl] = carry;
                    P.p[((size_t)r * N + i) * L + hl] = (uint8_t)tp;
                }
                if (threadIdx.x == 0) P.q[(size_t)r * N + i] = (uint8_t)qidx;
            }
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            wcur[u] = wnxt[u];
#pragma unroll
            for (int c = 0; c < RMAX; ++c) cur[u][c] = nxt[u][c];
        }
    }
}

// ---- sweep for pairwise potentials given per edge ---------------------------------------------
//
// theta_{i-r,i}(mu,lambda) read from a table of its own per edge, [R][N][L][L] with entry
// (r, i) the edge that arrives at node i (Eq. isgmr / Eq. trwp as written, before the
// decomposition into edge weight times V); for L <= 64.  One wavefront per scanline, lanes
// over lambda.  Row mu of a node's table is one coalesced load of L floats; the table is
// fetched in two halves of HALF = 4, 8, ..., 32 rows into two register sets, each reloaded
// for the next node as soon as the current node is done with it, so that one half is always
// in flight behind the evaluation of the other.  h(mu) comes from the lane that owns mu
// (v_readlane with a constant lane).  The candidate is the plain sum h(mu) + theta(mu,lambda).
template <int HALF, int RMAX, bool TRWP>
__global__ void __launch_bounds__(64)
mrf_fwd_sweep_edge(const MrfFwdParams P)
{
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const bool valid = lane < L;
    const int lamc = valid ? lane : 0;

    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const float rho = P.rho[r];
    const int n_pre = P.n_pre[r], n_src = P.n_src[r], rm_slot = P.rm_slot[r];

    // sources of h as in mrf_fwd_sweep: unused slots read the unary with factor 0
    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L;
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)P.src_dir[r][c - 1] * N * L : src[0];
        use[c] = (c <= n_src) ? 1.0f : 0.0f;
        is_rm[c] = (c - 1 == rm_slot) ? 1.0f : 0.0f;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = (c == n_pre + 1) ? 1.0f : 0.0f;

    if (valid) {
        P.m_out[((size_t)r * N + head) * L + lane] = 0.0f;
        P.p[((size_t)r * N + head) * L + lane] = 0;
    }
    if (lane == 0) P.q[(size_t)r * N + head] = 0;
    if (len < 2) return;

    const int vzero = mrf_opaque_zero();
    const float *rbase = P.rho_e ? P.rho_e + (size_t)r * N : nullptr;
    const float *tbase = P.Te + (size_t)r * N * L * L;
    // rows mu0 .. mu0 + HALF - 1 of the table of the edge that arrives at node n of the scanline
    // (rows past L - 1 repeat the last row and are masked at use; a node past the end repeats the last)
    auto load_half = [&](float (&dst)[HALF], int n, int mu0) {
        n = n < len ? n : len - 1;
        const float *tb = tbase + (size_t)(head + (long long)n * nstep) * L * L + lamc;
#pragma unroll
        for (int m = 0; m < HALF; ++m) {
            const int mu = mu0 + m < L ? mu0 + m : L - 1;
            dst[m] = tb[(size_t)mu * L];
        }
    };
    float ta[HALF], tb2[HALF];
    float cur[RMAX], nxt[RMAX];
    float rcur = rho, rnxt = rho;
    auto prefetch = [&](float (&dst)[RMAX], float &rdst, int nj) {      // inputs of the update nj -> nj+1
        nj = nj < len - 2 ? nj : len - 2;
        const long long j = head + (long long)nj * nstep;
#pragma unroll
        for (int c = 0; c < RMAX; ++c) dst[c] = src[c][(size_t)j * L + lamc];
        rdst = rho;
        if (TRWP && rbase) rdst = rbase[(size_t)(j + nstep) + vzero];
    };
    prefetch(cur, rcur, 0);
    load_half(ta, 1, 0);
    load_half(tb2, 1, HALF);

    float carry = 0.0f;
    for (int n = 1; n < len; ++n) {
        prefetch(nxt, rnxt, n);
        const long long i = head + (long long)n * nstep;

        float v = cur[0];
        if (TRWP) {
            float mrm = 0.0f;
#pragma unroll
            for (int c = 1; c < RMAX; ++c) {
                v = __builtin_fmaf(carry_at[c], carry, v);
                v = __builtin_fmaf(use[c], cur[c], v);
                mrm = __builtin_fmaf(is_rm[c], cur[c], mrm);
            }
            v = __builtin_fmaf(carry_at[RMAX], carry, v);
            v = rcur * v;
            v = v - mrm;
        } else {
#pragma unroll
            for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[c], v);
            v = v + carry;
        }

        // ascending mu with a strict '<': the lowest minimiser survives
        float best = INFINITY;
        int arg = 0;
#pragma unroll
        for (int m = 0; m < HALF; ++m) {
            const float hm = mrf_readlane_f32(v, m);
            const float dl = (m < L) ? hm + ta[m] : INFINITY;
            if (dl < best) { best = dl; arg = m; }
        }
        load_half(ta, n + 1, 0);
#pragma unroll
        for (int m = 0; m < HALF; ++m) {
            const float hm = mrf_readlane_f32(v, (HALF + m) & 63);
            const float dl = (HALF + m < L) ? hm + tb2[m] : INFINITY;
            if (dl < best) { best = dl; arg = HALF + m; }
        }
        load_half(tb2, n + 1, HALF);

        const float tv = valid ? best : INFINITY;
        const float tq = mrf_wave_min(tv);
        const unsigned long long bal = __ballot(tv == tq);
        const int qidx = __ffsll((long long)bal) - 1;
        carry = valid ? tv - tq : 0.0f;
        if (valid) {
            P.m_out[((size_t)r * N + i) * L + lane] = carry;
            P.p[((size_t)r * N + i) * L + lane] = (uint8_t)arg;
        }
        if (lane == 0) P.q[(size_t)r * N + i] = (uint8_t)qidx;

        rcur = rnxt;
#pragma unroll
        for (int c = 0; c < RMAX; ++c) cur[c] = nxt[c];
    }
}

// ---- final costs and labels: c_i = theta_i + sum_r m^r_i (direction order), x_i = argmin ----
struct MrfAggParams {
    long long N;
    int L, R;
    int no_unary;        // Eq. isgmr-aggregation-old (standard SGM): c_i = sum_r m^r_i
    const float *unary, *m;
    float *cost;
    uint8_t *labels;     // may be NULL
};

// RT: bound on R (all loads of a node are issued before the first addition)
template <int RT>
__global__ void __launch_bounds__(256) mrf_aggregate(const MrfAggParams P)
{
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
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
                float v = P.no_unary ? 0.0f : P.unary[(size_t)i * L + lam];
                float mv[RT];
#pragma unroll
                for (int d = 0; d < RT; ++d)
                    if (d < P.R) mv[d] = P.m[((size_t)d * P.N + i) * L + lam];
#pragma unroll
                for (int d = 0; d < RT; ++d)
                    if (d < P.R) v = v + mv[d];
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

// ---- ISGMR with many directions: what iteration k left at a node, summed once per pair of directions ----
// Eq. isgmr's bracket holds, besides the running message, theta_i + sum over d not in {r, r-} of m^{d,k}_i:
// the same sum for r and for r-, and the same terms in the same order for every node that reads node i.
// One streaming pass per iteration forms it for every pair (2 R + 2 + R vectors moved per node instead of
// R (R - 1) read by the sweeps); the sweeps then read that one vector where they read the unary in the
// first iteration.  The additions are those of the sweeps, left to right in direction order.
struct MrfPresumParams {
    long long NL;            // entries per array
    int R;
    int opp[MRF_MAXR];       // opposite direction, or -1
    const float *unary;      // [N][L]
    const float *m;          // [R][N][L] messages of iteration k
    float *out;              // [R][N][L]: slab d is written for every d with no lower-indexed opposite
};

template <int RT, int VEC>
__global__ void __launch_bounds__(256) mrf_isgmr_presum(const MrfPresumParams P)
{
    typedef float vecf __attribute__((ext_vector_type(VEC)));
    const long long n = P.NL / VEC;
    for (long long e4 = (long long)blockIdx.x * blockDim.x + threadIdx.x; e4 < n; e4 += (long long)gridDim.x * blockDim.x) {
        const long long e = e4 * VEC;
        const vecf th = *reinterpret_cast<const vecf *>(P.unary + e);
        vecf mv[RT];
#pragma unroll
        for (int d = 0; d < RT; ++d)
            if (d < P.R) mv[d] = *reinterpret_cast<const vecf *>(P.m + (size_t)d * P.NL + e);
#pragma unroll
        for (int d = 0; d < RT; ++d) {
            if (d >= P.R) continue;
            const int od = P.opp[d];
            if (od >= 0 && od < d) continue;          // the pair was done at its lower index
            vecf a = th;
#pragma unroll
            for (int c = 0; c < RT; ++c)
                if (c < P.R && c != d && c != od) a = a + mv[c];
            *reinterpret_cast<vecf *>(P.out + (size_t)d * P.NL + e) = a;
        }
    }
}

// ---- fast path: V(mu, lambda) = f(|mu - lambda|) with f non-decreasing and constant (= fT)
// from distance TW on (truncated linear / quadratic models, Sec. 5.1) ------------------------
//
// With a non-negative edge weight every candidate inside the window |mu - lambda| < TW is
// <= g(mu) := fma(w, fT, h(mu)), and every candidate outside it equals g(mu).  Hence
//     min_mu Delta(lambda, mu) = min(W(lambda), gmin),   W = min over the window, gmin = min_mu g,
// and the lowest minimiser is  pW            if W <  gmin
//                              mu_g          if W >  gmin   (mu_g = lowest argmin of g; it is
//                                                            then provably outside the window)
//                              min(pW, mu_g) if W == gmin.
// Values and indices are bit-identical to the dense evaluation; the work per label drops
// from L to 2 TW - 1 candidates.  One wavefront walks one scanline: no workgroup barrier.
// A node with a negative weight falls back to the full loop over mu.
template <int LP, int RMAX, int D, bool TRWP, int TW>
__global__ void __launch_bounds__(64)
mrf_fwd_sweep_window(const MrfFwdParams P)
{
    constexpr int HB = 64 * LP + 2 * TW;          // h with TW entries of padding on both sides
    __shared__ float hpad[HB];
    __shared__ float ftab[TW + 1];
    const int L = P.g.L;
    const int lane = threadIdx.x;

    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const float rho = P.rho[r];
    const int n_pre = P.n_pre[r], n_src = P.n_src[r], rm_slot = P.rm_slot[r];

    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    const float vz = mrf_opaque_zero_f();     // keeps the flags below in vector registers
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L;
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)P.src_dir[r][c - 1] * N * L : src[0];
        use[c] = ((c <= n_src) ? 1.0f : 0.0f) + vz;
        is_rm[c] = ((c - 1 == rm_slot) ? 1.0f : 0.0f) + vz;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = ((c == n_pre + 1) ? 1.0f : 0.0f) + vz;

    // f(d) = V(0, d) for d < TW, fT = V(0, L-1) (the promise makes every farther entry equal it)
    float f[TW];
#pragma unroll
    for (int d = 0; d < TW; ++d) f[d] = P.V[d < L ? d : L - 1] + vz;
    const float fT = P.V[L - 1] + vz;
    const bool f0zero = (P.V[0] == 0.0f);
    if (lane <= TW) ftab[lane] = lane < TW ? P.V[lane < L ? lane : L - 1] : fT;
    for (int i = lane; i < HB; i += 64) hpad[i] = INFINITY;     // padding never wins a strict '<'
    __syncthreads();
    float *hbuf = hpad + TW;

#pragma unroll
    for (int s = 0; s < LP; ++s) {
        const int lam = lane + 64 * s;
        if (lam < L) {
            P.m_out[((size_t)r * N + head) * L + lam] = 0.0f;
            P.p[((size_t)r * N + head) * L + lam] = 0;
        }
    }
    if (lane == 0) P.q[(size_t)r * N + head] = 0;

    const int vzero = mrf_opaque_zero();
    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
    const int lastsrc = len - 2;
    float cur[D][RMAX][LP], nxt[D][RMAX][LP];
    float wcur[D], wnxt[D];
    float rcur[D], rnxt[D];                // rho of the edge (i-r, i): per edge if P.rho_e is given
    const float *rbase = P.rho_e ? P.rho_e + (size_t)r * N : nullptr;
    auto prefetch = [&](float (&dst)[RMAX][LP], float &wdst, float &rdst, int nj) {
        nj = nj < lastsrc ? nj : lastsrc;
        const long long j = head + (long long)nj * nstep;
#pragma unroll
        for (int c = 0; c < RMAX; ++c)
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                dst[c][s] = src[c][(size_t)j * L + (lam < L ? lam : 0)];
            }
        wdst = wbase[(size_t)((j + nstep) * P.w_mul) + vzero];
        rdst = rho;
        if (TRWP && rbase) rdst = rbase[(size_t)(j + nstep) + vzero];
    };
    if (len >= 2) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u], rcur[u], u);
    }

    float carry[LP];
#pragma unroll
    for (int s = 0; s < LP; ++s) carry[s] = 0.0f;

    for (int n0 = 1; n0 < len; n0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u], rnxt[u], n0 - 1 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int nn = n0 + u;
            const bool past = nn >= len;
            const int n = past ? len - 1 : nn;
            const long long i = head + (long long)n * nstep;
            const float wgt = wcur[u];

            float a[LP], gfar[LP];
            float hm = INFINITY;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                float v = cur[u][0][s];
                float mrm = 0.0f;
                if (TRWP) {
#pragma unroll
                    for (int c = 1; c < RMAX; ++c) {
                        v = __builtin_fmaf(carry_at[c], carry[s], v);
                        v = __builtin_fmaf(use[c], cur[u][c][s], v);
                        mrm = __builtin_fmaf(is_rm[c], cur[u][c][s], mrm);
                    }
                    v = __builtin_fmaf(carry_at[RMAX], carry[s], v);
                    v = rcur[u] * v;
                    v = v - mrm;
                } else {
#pragma unroll
                    for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[u][c][s], v);
                    v = v + carry[s];
                }
                const int lam = lane + 64 * s;
                if (lam < L) hbuf[lam] = v;
                a[s] = lam < L ? v : INFINITY;
                gfar[s] = lam < L ? __builtin_fmaf(wgt, fT, v) : INFINITY;
                hm = mrf_min(hm, a[s]);
            }
            mrf_wave_lds_fence();

            float tv[LP];
            int tp[LP];
            int qidx = -1;
            float tq;
            // (the weight is wave-uniform: take the branch on a scalar copy of its sign)
            if (__builtin_expect(__builtin_amdgcn_readfirstlane(__float_as_int(wgt)) >= 0, 1)) {
                // One reduction serves the whole node.  g is a non-decreasing function of h, so
                // gmin = fma(w, fT, hmin).  If moreover f(0) = 0, every candidate is >= its h(mu)
                // >= hmin and the candidate (lambda = mu = argmin h) equals hmin, so the minimum
                // over lambda of the new message is hmin itself: q is the lowest label that
                // attains it and no second reduction is needed.
                const float hmin = mrf_wave_min(hm);
                const float gmin = __builtin_fmaf(wgt, fT, hmin);
                int mug = 0;
                bool found = false;
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const unsigned long long bal = __ballot(gfar[s] == gmin);
                    if (!found && bal != 0ull) { found = true; mug = 64 * s + __ffsll((long long)bal) - 1; }
                }
                // window |mu - lambda| < TW, ascending mu
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    float dl[2 * TW - 1];
#pragma unroll
                    for (int o = 0; o < 2 * TW - 1; ++o) {
                        const int dist = o < TW - 1 ? TW - 1 - o : o - (TW - 1);
                        dl[o] = __builtin_fmaf(wgt, f[dist], hbuf[lam + o - (TW - 1)]);
                    }
                    float W = dl[0];
#pragma unroll
                    for (int o = 1; o + 1 < 2 * TW - 1; o += 2) W = mrf_min3(W, dl[o], dl[o + 1]);
                    int po = 2 * TW - 2;
#pragma unroll
                    for (int o = 2 * TW - 3; o >= 0; --o) po = (dl[o] == W) ? o : po;
                    const int pW = lam + po - (TW - 1);
                    const bool wlt = W < gmin, wgt_ = W > gmin;
                    tv[s] = (lam < L) ? (wlt ? W : gmin) : INFINITY;
                    const int tie = pW < mug ? pW : mug;
                    tp[s] = wlt ? pW : (wgt_ ? mug : tie);
                }
                if (__builtin_expect(f0zero, 1)) {
                    tq = hmin;
                } else {
                    float mn = INFINITY;
#pragma unroll
                    for (int s = 0; s < LP; ++s) mn = fminf(mn, tv[s]);
                    tq = mrf_wave_min(mn);
                }
            } else {
                // negative weight: the ordering argument does not hold, evaluate every mu
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    float best = INFINITY;
                    int bi = 0;
                    for (int mu = 0; mu < L; ++mu) {
                        int dist = mu > lam ? mu - lam : lam - mu;
                        dist = dist < TW ? dist : TW;
                        const float dlt = __builtin_fmaf(wgt, ftab[dist], hbuf[mu]);
                        if (dlt < best) { best = dlt; bi = mu; }
                    }
                    tv[s] = (lam < L) ? best : INFINITY;
                    tp[s] = bi;
                }
                float mn = INFINITY;
#pragma unroll
                for (int s = 0; s < LP; ++s) mn = fminf(mn, tv[s]);
                tq = mrf_wave_min(mn);
            }
            mrf_wave_lds_fence();

            // q = lowest label attaining the minimum; reparametrisation (Eq. isgmr-norm)
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const unsigned long long bal = __ballot(tv[s] == tq);
                if (qidx < 0 && bal != 0ull) qidx = 64 * s + __ffsll((long long)bal) - 1;
            }
#pragma unroll
            for (int s = 0; s < LP; ++s) carry[s] = (lane + 64 * s < L) ? tv[s] - tq : 0.0f;

            if (!past) {
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
#pragma unroll
        for (int u = 0; u < D; ++u) {
            wcur[u] = wnxt[u];
            rcur[u] = rnxt[u];
#pragma unroll
            for (int c = 0; c < RMAX; ++c)
#pragma unroll
                for (int s = 0; s < LP; ++s) cur[u][c][s] = nxt[u][c][s];
        }
    }
}

// ---- window sweep with an index wavefront ----------------------------------------------------
//
// Same arithmetic as mrf_fwd_sweep_window, for launches with few scanlines.  Only the VALUES
// of the new message are on the node-to-node dependency chain; the argmin tables p and q and
// every store are not.  Two wavefronts share a scanline: the value wavefront forms h, its
// minimum and the new message and passes h, hmin and the weight through a ring in LDS; the
// index wavefronts follow a little behind, repeat the window evaluation with the index
// bookkeeping (Alg. 1/2: p, q) and store m, p and q.  Both sides evaluate the same
// expressions on the same h, so what is stored equals what the value wavefront carries.
// The index work of a node does not depend on other nodes, so NI index wavefronts take the
// nodes of a scanline in turn (it is somewhat more work per node than the value chain).
// Nobody meets at a barrier: the producer only waits when the ring is full, a consumer when
// its next node is not there yet, and every counter only grows, so all waits end.
//
// LOADER (TRWP with at most three other directions) adds a fourth kind of wavefront in front
// of the value wavefront.  It does the global loads and whatever of h does not need the
// running message: the partial sum theta + (messages of the directions before r), in the
// order Eq. trwp is summed, and the vector of r-.  It hands these, the later directions'
// messages and the weight over through a second ring; the value wavefront then touches LDS
// only, adds the running message and the later directions to the partial sum (same order,
// same roundings), and reads the next node's entries while it reduces the current one.
template <int LP, int RMAX, int D, bool TRWP, int TW, int NI, bool LOADER>
__global__ void __launch_bounds__(64 * ((LOADER ? 2 : 1) + NI))
mrf_fwd_sweep_window_duo(const MrfFwdParams P)
{
    static_assert(!LOADER || (TRWP && RMAX == 4), "loader wavefront: TRWP with up to three other directions");
    constexpr int NW0 = LOADER ? 2 : 1;           // wavefronts in front of the index wavefronts
    constexpr int NRL = 8;                        // slots of the loader's ring (a power of two, >= D)
    constexpr int LL = 64 * LP;
    constexpr int HB = 64 * LP + 2 * TW;          // h with TW entries of padding on both sides
    constexpr int NR = 8;                         // ring slots (a power of two, >= D)
    static_assert(NR >= D && (NR & (NR - 1)) == 0 && NI <= 4, "ring depth");
    constexpr int NT = 64 * (NW0 + NI);
    // One block with the h ring at LDS address 0: the value wavefront's fifteen neighbour reads per
    // label slot then fit the 8-bit offsets of ds_read2_b32 and need no address arithmetic.
    struct Shared {
        float ring[NR][HB];
        float ringw[NR], ringhm[NR];
        float ftab[TW + 1];
        int produced;                             // last step published
        int loaded;                               // last step the loader has published
        MrfWaitBlock wait;                        // for the waits below (mrf_wait_turn)
        alignas(16) int consumed[4];              // per index wavefront: last step finished
        float lw[NRL];
        alignas(16) float lring[LOADER ? NRL : 1][5][LOADER ? LL : 1];   // partial sum, 3 messages, r- vector
    };
    __shared__ Shared sm;
    auto &ring = sm.ring;
    auto &ringw = sm.ringw;
    auto &ringhm = sm.ringhm;
    auto &ftab = sm.ftab;
    int &produced = sm.produced;
    int &loaded = sm.loaded;
    auto &consumed = sm.consumed;
    auto &lw = sm.lw;
    auto &lring = sm.lring;
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool index_wave = wave >= NW0;
    // the wavefronts on the node-to-node chain go first wherever they share a SIMD with the others
    if (!index_wave) __builtin_amdgcn_s_setprio(3);

    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const float vz = mrf_opaque_zero_f();     // keeps uniform constants in vector registers

    // f(d) = V(0, d) for d < TW, fT = V(0, L-1) (the promise makes every farther entry equal it)
    float f[TW];
#pragma unroll
    for (int d = 0; d < TW; ++d) f[d] = P.V[d < L ? d : L - 1] + vz;
    const float fT = P.V[L - 1] + vz;
    const bool f0zero = (P.V[0] == 0.0f);
    if ((int)threadIdx.x <= TW) ftab[threadIdx.x] = (int)threadIdx.x < TW ? P.V[(int)threadIdx.x < L ? threadIdx.x : L - 1] : fT;
    // padding and the entries of labels >= L are never written again: they never win a strict '<'
    for (int i = threadIdx.x; i < NR * HB; i += NT) (&ring[0][0])[i] = INFINITY;
    if (threadIdx.x == 0) { produced = 0; loaded = 0; mrf_wait_init(&sm.wait, P.fault, P.spin_limit); }
    const MrfWaitBlock *const wait_block = &sm.wait;
    // index wavefront j takes steps 1 + j, 1 + j + NI, ...; "finished" starts one turn before
    if (threadIdx.x < 4) consumed[threadIdx.x] = (int)threadIdx.x + 1 - NI;
    __syncthreads();

    if (index_wave) {
        // ---- p, q and all stores -----------------------------------------------------------
        const int jw = wave - NW0;
        if (jw == 0) {
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

        // stores relative to the head of the scanline (the host has checked that a node step
        // times L fits 32 bits)
        float *const mrow = P.m_out + ((size_t)r * N + head) * L;
        uint8_t *const prow = P.p + ((size_t)r * N + head) * L;
        uint8_t *const qrow = P.q + (size_t)r * N + head;
        const int istep_l = (int)nstep * L;
        int seen = 0;
        for (int n = 1 + jw; n < len; n += NI) {
            int wait_turns = 0;
            while (seen < n) {
                seen = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&produced, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                if (seen < n) mrf_wait_turn(wait_block, wait_turns);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            const int slot = n & (NR - 1);
            const float *hbuf = &ring[slot][TW];
            const float wgt = ringw[slot];
            const float hmin = ringhm[slot];
            const long long ol = (long long)n * istep_l;
            // the window's h in one batch of LDS reads behind the two words above (entries of labels
            // >= L and the padding hold +inf, so no lane needs a condition)
            float hv[LP][2 * TW - 1];
#pragma unroll
            for (int s = 0; s < LP; ++s)
#pragma unroll
                for (int o = 0; o < 2 * TW - 1; ++o) hv[s][o] = hbuf[lane + 64 * s + o - (TW - 1)];

            float tv[LP];
            int tp[LP];
            float tq;
            // The window evaluation runs for every node, so that the usual case is straight-line
            // code; for a negative weight its results are replaced below.
            {
                const float gmin = __builtin_fmaf(wgt, fT, hmin);
                int mug = 0;
                bool found = false;
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    const float gfar = lam < L ? __builtin_fmaf(wgt, fT, hv[s][TW - 1]) : INFINITY;
                    const unsigned long long bal = __ballot(gfar == gmin);
                    if (!found && bal != 0ull) { found = true; mug = 64 * s + __ffsll((long long)bal) - 1; }
                }
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    float dl[2 * TW - 1];
#pragma unroll
                    for (int o = 0; o < 2 * TW - 1; ++o) {
                        const int dist = o < TW - 1 ? TW - 1 - o : o - (TW - 1);
                        dl[o] = __builtin_fmaf(wgt, f[dist], hv[s][o]);
                    }
                    float W = dl[0];
#pragma unroll
                    for (int o = 1; o + 1 < 2 * TW - 1; o += 2) W = mrf_min3(W, dl[o], dl[o + 1]);
                    int po = 2 * TW - 2;
#pragma unroll
                    for (int o = 2 * TW - 3; o >= 0; --o) po = (dl[o] == W) ? o : po;
                    const int pW = lam + po - (TW - 1);
                    const bool wlt = W < gmin, wgt_ = W > gmin;
                    tv[s] = (lam < L) ? (wlt ? W : gmin) : INFINITY;
                    const int tie = pW < mug ? pW : mug;
                    tp[s] = wlt ? pW : (wgt_ ? mug : tie);
                }
                if (__builtin_expect(f0zero, 1)) {
                    tq = hmin;
                } else {
                    float mn = INFINITY;
#pragma unroll
                    for (int s = 0; s < LP; ++s) mn = fminf(mn, tv[s]);
                    tq = mrf_wave_min(mn);
                }
            }
            if (__builtin_expect(__builtin_amdgcn_readfirstlane(__float_as_int(wgt)) < 0, 0)) {
                // negative weight: the ordering argument does not hold, evaluate every mu
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    float best = INFINITY;
                    int bi = 0;
                    for (int mu = 0; mu < L; ++mu) {
                        int dist = mu > lam ? mu - lam : lam - mu;
                        dist = dist < TW ? dist : TW;
                        const float dlt = __builtin_fmaf(wgt, ftab[dist], hbuf[mu]);
                        if (dlt < best) { best = dlt; bi = mu; }
                    }
                    tv[s] = (lam < L) ? best : INFINITY;
                    tp[s] = bi;
                }
                float mn = INFINITY;
#pragma unroll
                for (int s = 0; s < LP; ++s) mn = fminf(mn, tv[s]);
                tq = mrf_wave_min(mn);
            }
            // this slot has been read: hand it back
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            if (lane == 0) __hip_atomic_store(&consumed[jw], n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);

            int qidx = -1;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const unsigned long long bal = __ballot(tv[s] == tq);
                if (qidx < 0 && bal != 0ull) qidx = 64 * s + __ffsll((long long)bal) - 1;
            }
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                if (__builtin_expect(lam < L, 1)) {
                    mrow[ol + lam] = tv[s] - tq;
                    prow[ol + lam] = (uint8_t)tp[s];
                }
            }
            if (lane == 0) qrow[(long long)n * nstep] = (uint8_t)qidx;
        }
        return;
    }

    // ---- values: the dependency chain ------------------------------------------------------
    const float rho = P.rho[r];
    const int n_pre = P.n_pre[r], n_src = P.n_src[r], rm_slot = P.rm_slot[r];
    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L;
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)P.src_dir[r][c - 1] * N * L : src[0];
        use[c] = ((c <= n_src) ? 1.0f : 0.0f) + vz;
        is_rm[c] = ((c - 1 == rm_slot) ? 1.0f : 0.0f) + vz;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = ((c == n_pre + 1) ? 1.0f : 0.0f) + vz;

    const int vzero = mrf_opaque_zero();
    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
    const int lastsrc = len - 2;
    // addresses relative to the head of the scanline: one 32 x 32 bit product per node (the
    // host has checked that a node step times L fits 32 bits)
    const int step_l = (int)nstep * L;
    const int step_w = (int)nstep * P.w_mul;
    const float *srcb[RMAX];
#pragma unroll
    for (int c = 0; c < RMAX; ++c) srcb[c] = src[c] + (size_t)head * L;
    const float *wb = wbase + (size_t)((head + nstep) * P.w_mul);
    float cur[D][RMAX][LP], nxt[D][RMAX][LP];
    float wcur[D], wnxt[D];
    auto prefetch = [&](float (&dst)[RMAX][LP], float &wdst, int nj) {
        nj = nj < lastsrc ? nj : lastsrc;
        const long long o = (long long)nj * step_l;
#pragma unroll
        for (int c = 0; c < RMAX; ++c)
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                const int lam = lane + 64 * s;
                dst[c][s] = srcb[c][o + (lam < L ? lam : 0)];
            }
        wdst = wb[(long long)nj * step_w + vzero];
    };
    if (LOADER && wave == 1) {
        // ---- loads and the part of h that does not wait for the running message -----------
        float before[RMAX];                   // sources summed before the running message
#pragma unroll
        for (int c = 1; c < RMAX; ++c) before[c] = ((c <= n_pre && c <= n_src) ? 1.0f : 0.0f) + vz;
        if (len >= 2) {
#pragma unroll
            for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u], u);
        }
        int pseen = 0;
        for (int n0 = 1; n0 < len; n0 += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u], n0 - 1 + D + u);
#pragma unroll
            for (int u = 0; u < D; ++u) {
                const int nn = n0 + u;
                if (nn < len) {
                    // the slot was last read for step nn - NRL, before that step was published
                    int wait_turns = 0;
                    while (pseen < nn - NRL) {
                        pseen = __builtin_amdgcn_readfirstlane(
                            __hip_atomic_load(&produced, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                        if (pseen < nn - NRL) mrf_wait_turn(wait_block, wait_turns);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                    const int ls = nn & (NRL - 1);
#pragma unroll
                    for (int s = 0; s < LP; ++s) {
                        float v = cur[u][0][s];
                        float mrm = 0.0f;
#pragma unroll
                        for (int c = 1; c < RMAX; ++c) {
                            v = __builtin_fmaf(before[c], cur[u][c][s], v);
                            mrm = __builtin_fmaf(is_rm[c], cur[u][c][s], mrm);
                            lring[ls][c][lane + 64 * s] = cur[u][c][s];
                        }
                        lring[ls][0][lane + 64 * s] = v;
                        lring[ls][4][lane + 64 * s] = mrm;
                    }
                    if (lane == 0) lw[ls] = wcur[u];
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
                    __builtin_amdgcn_wave_barrier();
                    if (lane == 0) __hip_atomic_store(&loaded, nn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
#pragma unroll
            for (int u = 0; u < D; ++u) {
                wcur[u] = wnxt[u];
#pragma unroll
                for (int c = 0; c < RMAX; ++c)
#pragma unroll
                    for (int s = 0; s < LP; ++s) cur[u][c][s] = nxt[u][c][s];
            }
        }
        return;
    }

    float carry[LP];
#pragma unroll
    for (int s = 0; s < LP; ++s) carry[s] = 0.0f;
    int freed = 0;          // every step <= freed is finished (a possibly stale, hence conservative, view)

    if (LOADER) {
        // ---- values, fed by the loader -------------------------------------------------------
        // With two labels per lane a lane holds two ADJACENT labels: its h pair is one 8-byte LDS
        // write, the windows of both labels come out of the same 2 TW + 2 neighbours (TW 8-byte
        // reads instead of 4 TW - 2 single ones), and a ring entry of the loader is one 8-byte read
        // per vector.  The rings are indexed by label, so the other wavefronts keep their own mapping.
        constexpr bool PAIR = LP == 2 && (TW % 2) == 0;
        auto lab = [&](int s) { return PAIR ? 2 * lane + s : lane + 64 * s; };
        auto read_entry = [&](float (&dst)[5][LP], int ls) {
            if constexpr (PAIR) {
#pragma unroll
                for (int c = 0; c < 5; ++c) {
                    const float2 t = *reinterpret_cast<const float2 *>(&lring[ls][c][2 * lane]);
                    dst[c][0] = t.x;
                    dst[c][LP - 1] = t.y;
                }
            } else {
#pragma unroll
                for (int c = 0; c < 5; ++c)
#pragma unroll
                    for (int s = 0; s < LP; ++s) dst[c][s] = lring[ls][c][lane + 64 * s];
            }
        };
        float after[RMAX];                    // sources summed after the running message
#pragma unroll
        for (int c = 1; c < RMAX; ++c) after[c] = ((c > n_pre && c <= n_src) ? 1.0f : 0.0f) + vz;
        auto await_loader = [&](int nn) {
            int sn;
            int wait_turns = 0;
            do {
                sn = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&loaded, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                if (sn < nn) mrf_wait_turn(wait_block, wait_turns);
            } while (sn < nn);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            return sn;
        };
        float in[5][LP], wgt = 0.0f;
        int lseen = 0;
        if (len >= 2) {
            lseen = await_loader(1);
            read_entry(in, 1);
            wgt = lw[1];
        }
        for (int nn = 1; nn < len; ++nn) {
            const int slot = nn & (NR - 1);
            float *hbuf = &ring[slot][TW];
            int wait_turns = 0;
            while (__builtin_expect(freed < nn - NR, 0)) {
                int lo = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&consumed[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
#pragma unroll
                for (int j = 1; j < NI; ++j) {
                    const int cj = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(&consumed[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                    lo = cj < lo ? cj : lo;
                }
                freed = lo + NI - 1;
                if (freed < nn - NR) mrf_wait_turn(wait_block, wait_turns);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");

            float a[LP];
            float hm = 0.0f;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                float v = in[0][s] + carry[s];
#pragma unroll
                for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(after[c], in[c][s], v);
                v = rho * v;
                v = v - in[4][s];
                const int lam = lab(s);
                // (lanes past L rewrite the +inf their ring entries hold anyway: no divergence; what
                // they carry from node to node is never looked at)
                a[s] = lam < L ? v : INFINITY;
                if (!PAIR) hbuf[lam] = a[s];
                hm = s == 0 ? a[s] : mrf_min(hm, a[s]);
            }
            if constexpr (PAIR) *reinterpret_cast<float2 *>(&hbuf[2 * lane]) = make_float2(a[0], a[LP - 1]);
            mrf_wave_lds_fence();
            float nb[LP][2 * TW - 1];
            if constexpr (PAIR) {
                // hn[k] = h(2 lane - TW + k), k = 0 .. 2 TW + 1; label 2 lane + s looks at hn[s + 1 ..]
                float hn[2 * TW + 2];
#pragma unroll
                for (int j = 0; j <= TW; ++j) {
                    if (j == TW / 2) {
                        hn[2 * j] = a[0];
                        hn[2 * j + 1] = a[LP - 1];
                    } else {
                        const float2 t = *reinterpret_cast<const float2 *>(&ring[slot][2 * lane + 2 * j]);
                        hn[2 * j] = t.x;
                        hn[2 * j + 1] = t.y;
                    }
                }
#pragma unroll
                for (int s = 0; s < LP; ++s)
#pragma unroll
                    for (int o = 0; o < 2 * TW - 1; ++o) nb[s][o] = hn[o + 1 + s];
            } else {
#pragma unroll
                for (int s = 0; s < LP; ++s)
#pragma unroll
                    for (int o = 0; o < 2 * TW - 1; ++o)
                        nb[s][o] = (o == TW - 1) ? a[s] : hbuf[lane + 64 * s + o - (TW - 1)];
            }
            // the next node's entries, in the same batch of LDS reads; if the loader's counter
            // (read first: the LDS queue keeps the order) does not cover them yet, they are read
            // again after waiting
            const bool more = nn + 1 < len;
            const int lsn = (nn + 1) & (NRL - 1);
            const int flag = __hip_atomic_load(&loaded, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            float nin[5][LP];
            read_entry(nin, lsn);
            float nwgt = lw[lsn];

            const float hmin = mrf_wave_min(hm);
            // LDS executes a wavefront's operations in order: whoever sees the counter also sees the
            // node's ring entries written before it, so no wait is needed in between
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            // (every lane writes the same three words: no divergent branch in the node step)
            ringw[slot] = wgt;
            ringhm[slot] = hmin;
            __hip_atomic_store(&produced, nn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

            float tv[LP];
            float tq;
            // (evaluated for every node, so that the usual case is straight-line code; replaced
            // below for a negative weight)
            {
                const float gmin = __builtin_fmaf(wgt, fT, hmin);
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    // The two candidates at distance d share f(d), and a correctly rounded fma is
                    // non-decreasing in its addend: the smaller of the two comes from the smaller h.
                    float dl[TW];
                    dl[0] = __builtin_fmaf(wgt, f[0], nb[s][TW - 1]);
#pragma unroll
                    for (int d = 1; d < TW; ++d)
                        dl[d] = __builtin_fmaf(wgt, f[d], mrf_min(nb[s][TW - 1 - d], nb[s][TW - 1 + d]));
                    float W = mrf_min(dl[0], gmin);
#pragma unroll
                    for (int d = 1; d + 1 < TW; d += 2) W = mrf_min3(W, dl[d], dl[d + 1]);
                    if ((TW & 1) == 0) W = mrf_min(W, dl[TW - 1]);
                    tv[s] = W;
                }
                if (__builtin_expect(f0zero, 1)) {
                    tq = hmin;
                } else {
                    float mn = INFINITY;
#pragma unroll
                    for (int s = 0; s < LP; ++s) mn = fminf(mn, (lab(s) < L) ? tv[s] : INFINITY);
                    tq = mrf_wave_min(mn);
                }
            }
            if (__builtin_expect(__builtin_amdgcn_readfirstlane(__float_as_int(wgt)) < 0, 0)) {
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lab(s);
                    float best = INFINITY;
                    for (int mu = 0; mu < L; ++mu) {
                        int dist = mu > lam ? mu - lam : lam - mu;
                        dist = dist < TW ? dist : TW;
                        const float dlt = __builtin_fmaf(wgt, ftab[dist], hbuf[mu]);
                        if (dlt < best) best = dlt;
                    }
                    tv[s] = (lam < L) ? best : INFINITY;
                }
                float mn = INFINITY;
#pragma unroll
                for (int s = 0; s < LP; ++s) mn = fminf(mn, tv[s]);
                tq = mrf_wave_min(mn);
            }
            // the next node's entries were read above with the loader's counter in front of them;
            // looked at only now, so that everything before is one straight block
            if (more) {
                lseen = __builtin_amdgcn_readfirstlane(flag);
                if (__builtin_expect(lseen < nn + 1, 0)) {
                    lseen = await_loader(nn + 1);
                    read_entry(nin, lsn);
                    nwgt = lw[lsn];
                }
            }
#pragma unroll
            for (int s = 0; s < LP; ++s) carry[s] = tv[s] - tq;
            wgt = nwgt;
#pragma unroll
            for (int c = 0; c < 5; ++c)
#pragma unroll
                for (int s = 0; s < LP; ++s) in[c][s] = nin[c][s];
        }
        return;
    }

    if (len >= 2) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u], u);
    }

    for (int n0 = 1; n0 < len; n0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u], n0 - 1 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int nn = n0 + u;
            const bool past = nn >= len;
            const float wgt = wcur[u];
            const int slot = nn & (NR - 1);
            float *hbuf = &ring[slot][TW];

            // the slot was last used by step nn - NR (steps past the end publish nothing
            // and write nothing)
            int wait_turns = 0;
            while (__builtin_expect(!past && freed < nn - NR, 0)) {
                int lo = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&consumed[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
#pragma unroll
                for (int j = 1; j < NI; ++j) {
                    const int cj = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(&consumed[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                    lo = cj < lo ? cj : lo;
                }
                freed = lo + NI - 1;
                if (freed < nn - NR) mrf_wait_turn(wait_block, wait_turns);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");

            float a[LP];
            float hm = 0.0f;
#pragma unroll
            for (int s = 0; s < LP; ++s) {
                float v = cur[u][0][s];
                float mrm = 0.0f;
                if (TRWP) {
#pragma unroll
                    for (int c = 1; c < RMAX; ++c) {
                        v = __builtin_fmaf(carry_at[c], carry[s], v);
                        v = __builtin_fmaf(use[c], cur[u][c][s], v);
                        mrm = __builtin_fmaf(is_rm[c], cur[u][c][s], mrm);
                    }
                    v = __builtin_fmaf(carry_at[RMAX], carry[s], v);
                    v = rho * v;
                    v = v - mrm;
                } else {
#pragma unroll
                    for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[u][c][s], v);
                    v = v + carry[s];
                }
                const int lam = lane + 64 * s;
                // (lanes past L rewrite the +inf their ring entries hold anyway: no divergence; what
                // they carry from node to node is never looked at)
                a[s] = lam < L ? v : INFINITY;
                if (!past) hbuf[lam] = a[s];
                hm = s == 0 ? a[s] : mrf_min(hm, a[s]);
            }
            // the neighbours' h for the window, requested before the reduction so that the LDS
            // latency passes behind it (the LDS queue keeps the order: writes above, then reads)
            mrf_wave_lds_fence();
            float nb[LP][2 * TW - 1];
#pragma unroll
            for (int s = 0; s < LP; ++s)
#pragma unroll
                for (int o = 0; o < 2 * TW - 1; ++o)
                    nb[s][o] = (o == TW - 1) ? a[s] : hbuf[lane + 64 * s + o - (TW - 1)];
            const float hmin = mrf_wave_min(hm);
            // LDS executes a wavefront's operations in order: whoever sees the counter also sees the
            // node's ring entries written before it, so no wait is needed in between
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            // (every lane writes the same three words: no divergent branch in the node step)
            if (!past) {
                ringw[slot] = wgt;
                ringhm[slot] = hmin;
                __hip_atomic_store(&produced, nn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

            // a past step re-reads the slot of an earlier step: its result is never used
            float tv[LP];
            float tq;
            // (evaluated for every node, so that the usual case is straight-line code; replaced
            // below for a negative weight)
            {
                const float gmin = __builtin_fmaf(wgt, fT, hmin);
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    // The two candidates at distance d share f(d), and a correctly rounded fma is
                    // non-decreasing in its addend: the smaller of the two comes from the smaller h.
                    float dl[TW];
                    dl[0] = __builtin_fmaf(wgt, f[0], nb[s][TW - 1]);
#pragma unroll
                    for (int d = 1; d < TW; ++d)
                        dl[d] = __builtin_fmaf(wgt, f[d], mrf_min(nb[s][TW - 1 - d], nb[s][TW - 1 + d]));
                    float W = mrf_min(dl[0], gmin);
#pragma unroll
                    for (int d = 1; d + 1 < TW; d += 2) W = mrf_min3(W, dl[d], dl[d + 1]);
                    if ((TW & 1) == 0) W = mrf_min(W, dl[TW - 1]);
                    tv[s] = W;
                }
                if (__builtin_expect(f0zero, 1)) {
                    tq = hmin;
                } else {
                    float mn = INFINITY;
#pragma unroll
                    for (int s = 0; s < LP; ++s) mn = fminf(mn, (lane + 64 * s < L) ? tv[s] : INFINITY);
                    tq = mrf_wave_min(mn);
                }
            }
            if (__builtin_expect(__builtin_amdgcn_readfirstlane(__float_as_int(wgt)) < 0, 0)) {
#pragma unroll
                for (int s = 0; s < LP; ++s) {
                    const int lam = lane + 64 * s;
                    float best = INFINITY;
                    for (int mu = 0; mu < L; ++mu) {
                        int dist = mu > lam ? mu - lam : lam - mu;
                        dist = dist < TW ? dist : TW;
                        const float dlt = __builtin_fmaf(wgt, ftab[dist], hbuf[mu]);
                        if (dlt < best) best = dlt;
                    }
                    tv[s] = (lam < L) ? best : INFINITY;
                }
                float mn = INFINITY;
#pragma unroll
                for (int s = 0; s < LP; ++s) mn = fminf(mn, tv[s]);
                tq = mrf_wave_min(mn);
            }
#pragma unroll
            for (int s = 0; s < LP; ++s) carry[s] = tv[s] - tq;
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            wcur[u] = wnxt[u];
#pragma unroll
            for (int c = 0; c < RMAX; ++c)
#pragma unroll
                for (int s = 0; s < LP; ++s) cur[u][c][s] = nxt[u][c][s];
        }
    }
}

// ---- window sweep, one label per lane, ceil(L/64) wavefronts per scanline ------------------
//
// Same arithmetic as mrf_fwd_sweep_window, laid out for launches with few scanlines (TRWP
// sweeps one direction at a time): a lone wavefront issues one instruction every four
// cycles, so the node step is spread over NWV wavefronts that each own 64 labels.  They
// meet once per node: every wavefront publishes its slice of h and its local minimum of h,
// then (after one LDS-only barrier) knows hmin, finds the lowest argmin of g by looking at
// all slices, evaluates its own windows and normalises by hmin without further exchange.
// q is assembled from per-wavefront candidates one node later, after the next barrier.
// Nodes where the single-reduction argument does not apply (negative weight, f(0) != 0)
// take a second barrier.
template <int RMAX, int D, bool TRWP, int TW>
__global__ void __launch_bounds__(256)
mrf_fwd_sweep_window_split(const MrfFwdParams P)
{
    constexpr int HB = 256 + 2 * TW;
    __shared__ float hpad[2][HB];
    __shared__ float ftab[TW + 1];
    __shared__ __align__(16) float hmslot[2][4];     // local minima of h
    __shared__ __align__(16) float tmslot[2][4];     // local minima of the new message (general path)
    __shared__ __align__(16) int qslot[2][4];        // local candidates for q
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform, and known to be
    const int NWV = blockDim.x >> 6;
    const int lam = wv * 64 + lane;
    const bool valid = lam < L;
    const int lamc = valid ? lam : 0;

    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const float rho = P.rho[r];
    const int n_pre = P.n_pre[r], n_src = P.n_src[r], rm_slot = P.rm_slot[r];

    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    const float vz = mrf_opaque_zero_f();     // keeps the flags below in vector registers
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L;
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)P.src_dir[r][c - 1] * N * L : src[0];
        use[c] = ((c <= n_src) ? 1.0f : 0.0f) + vz;
        is_rm[c] = ((c - 1 == rm_slot) ? 1.0f : 0.0f) + vz;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = ((c == n_pre + 1) ? 1.0f : 0.0f) + vz;

    float f[TW];
#pragma unroll
    for (int d = 0; d < TW; ++d) f[d] = P.V[d < L ? d : L - 1] + vz;
    const float fT = P.V[L - 1] + vz;
    const bool f0zero = (P.V[0] == 0.0f);
    if (threadIdx.x <= TW) ftab[threadIdx.x] = (int)threadIdx.x < TW ? P.V[(int)threadIdx.x < L ? threadIdx.x : L - 1] : fT;
    for (int i = threadIdx.x; i < 2 * HB; i += blockDim.x) (&hpad[0][0])[i] = INFINITY;
    if (threadIdx.x < 8) {
        (&hmslot[0][0])[threadIdx.x] = INFINITY;
        (&tmslot[0][0])[threadIdx.x] = INFINITY;
        (&qslot[0][0])[threadIdx.x] = -1;
    }
    __syncthreads();

    if (valid) {
        P.m_out[((size_t)r * N + head) * L + lam] = 0.0f;
        P.p[((size_t)r * N + head) * L + lam] = 0;
    }
    if (threadIdx.x == 0) P.q[(size_t)r * N + head] = 0;

    const int vzero = mrf_opaque_zero();
    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
    const int lastsrc = len - 2;
    float cur[D][RMAX], nxt[D][RMAX];
    float wcur[D], wnxt[D];
    auto prefetch = [&](float (&dst)[RMAX], float &wdst, int nj) {
        nj = nj < lastsrc ? nj : lastsrc;
        const long long j = head + (long long)nj * nstep;
#pragma unroll
        for (int c = 0; c < RMAX; ++c) dst[c] = src[c][(size_t)j * L + lamc];
        wdst = wbase[(size_t)((j + nstep) * P.w_mul) + vzero];
    };
    if (len >= 2) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u], u);
    }

    float carry = 0.0f;
    int par = 0, qpar = 0;
    long long qnode = -1;      // node whose q is still to be stored (wavefront 0), candidates in qslot[qpar]

    for (int n0 = 1; n0 < len; n0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u], n0 - 1 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int nn = n0 + u;
            const bool past = nn >= len;
            const int n = past ? len - 1 : nn;
            const long long i = head + (long long)n * nstep;
            const float wgt = wcur[u];
            float *hb = &hpad[par][TW];

            float v = cur[u][0];
            if (TRWP) {
                float mrm = 0.0f;
#pragma unroll
                for (int c = 1; c < RMAX; ++c) {
                    v = __builtin_fmaf(carry_at[c], carry, v);
                    v = __builtin_fmaf(use[c], cur[u][c], v);
                    mrm = __builtin_fmaf(is_rm[c], cur[u][c], mrm);
                }
                v = __builtin_fmaf(carry_at[RMAX], carry, v);
                v = rho * v;
                v = v - mrm;
            } else {
#pragma unroll
                for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[u][c], v);
                v = v + carry;
            }
            if (valid) hb[lam] = v;
            const float hloc = mrf_wave_min(valid ? v : INFINITY);
            if (lane == 0) hmslot[par][wv] = hloc;
            mrf_block_sync_lds();

            // q of the previous node: first wavefront that had a candidate
            if (wv == 0 && qnode >= 0) {
                const int4 qc = *reinterpret_cast<const int4 *>(&qslot[qpar][0]);
                const int qv = qc.x >= 0 ? qc.x : (qc.y >= 0 ? qc.y : (qc.z >= 0 ? qc.z : qc.w));
                if (lane == 0) P.q[(size_t)r * N + qnode] = (uint8_t)qv;
            }

            const float4 hm4 = *reinterpret_cast<const float4 *>(&hmslot[par][0]);
            const float hmin = fminf(fminf(hm4.x, hm4.y), fminf(hm4.z, hm4.w));
            const bool wpos = __builtin_amdgcn_readfirstlane(__float_as_int(wgt)) >= 0;
            float tv;
            int tp;
            if (wpos) {
                const float gmin = __builtin_fmaf(wgt, fT, hmin);
                // lowest argmin of g over all labels: look at every wavefront's slice of h
                int mug = 0;
                bool found = false;
#pragma unroll
                for (int w2 = 0; w2 < 4; ++w2) {
                    if (w2 < NWV) {
                        const float g2 = __builtin_fmaf(wgt, fT, hb[w2 * 64 + lane]);   // padding is +inf
                        const unsigned long long bal = __ballot(g2 == gmin);
                        if (!found && bal != 0ull) { found = true; mug = 64 * w2 + __ffsll((long long)bal) - 1; }
                    }
                }
                float dl[2 * TW - 1];
#pragma unroll
                for (int o = 0; o < 2 * TW - 1; ++o) {
                    const int dist = o < TW - 1 ? TW - 1 - o : o - (TW - 1);
                    dl[o] = __builtin_fmaf(wgt, f[dist], hb[lam + o - (TW - 1)]);
                }
                float W = dl[0];
#pragma unroll
                for (int o = 1; o + 1 < 2 * TW - 1; o += 2) W = mrf_min3(W, dl[o], dl[o + 1]);
                int po = 2 * TW - 2;
#pragma unroll
                for (int o = 2 * TW - 3; o >= 0; --o) po = (dl[o] == W) ? o : po;
                const int pW = lam + po - (TW - 1);
                const bool wlt = W < gmin, wgt_ = W > gmin;
                tv = valid ? (wlt ? W : gmin) : INFINITY;
                const int tie = pW < mug ? pW : mug;
                tp = wlt ? pW : (wgt_ ? mug : tie);
            } else {
                float best = INFINITY;
                int bi = 0;
                for (int mu = 0; mu < L; ++mu) {
                    int dist = mu > lam ? mu - lam : lam - mu;
                    dist = dist < TW ? dist : TW;
                    const float dlt = __builtin_fmaf(wgt, ftab[dist], hb[mu]);
                    if (dlt < best) { best = dlt; bi = mu; }
                }
                tv = valid ? best : INFINITY;
                tp = bi;
            }
            float tq = hmin;
            if (!(wpos && f0zero)) {
                // general case: the minimum of the new message needs its own exchange
                const float tloc = mrf_wave_min(tv);
                if (lane == 0) tmslot[par][wv] = tloc;
                mrf_block_sync_lds();
                const float4 t4 = *reinterpret_cast<const float4 *>(&tmslot[par][0]);
                tq = fminf(fminf(t4.x, t4.y), fminf(t4.z, t4.w));
            }
            const unsigned long long qb = __ballot(tv == tq);
            carry = valid ? tv - tq : 0.0f;

            // steps past the end of the scanline (last group only) leave no trace
            if (!past) {
                if (lane == 0) qslot[par][wv] = qb != 0ull ? wv * 64 + __ffsll((long long)qb) - 1 : -1;
                if (valid) {
                    P.m_out[((size_t)r * N + i) * L + lam] = carry;
                    P.p[((size_t)r * N + i) * L + lam] = (uint8_t)tp;
                }
                qnode = i;
                qpar = par;
            }
            par ^= 1;
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            wcur[u] = wnxt[u];
#pragma unroll
            for (int c = 0; c < RMAX; ++c) cur[u][c] = nxt[u][c];
        }
    }
    // q of the last node
    __syncthreads();
    if (wv == 0 && qnode >= 0) {
        const int4 qc = *reinterpret_cast<const int4 *>(&qslot[qpar][0]);
        const int qv = qc.x >= 0 ? qc.x : (qc.y >= 0 ? qc.y : (qc.z >= 0 ? qc.z : qc.w));
        if (lane == 0) P.q[(size_t)r * N + qnode] = (uint8_t)qv;
    }
}

// ---- window sweep: value wavefronts per 64 labels, index wavefronts per node -----------------
//
// Both ideas above together, for wide windows over many labels in small launches.  NWV =
// ceil(L/64) value wavefronts walk the scanline in lock step as in mrf_fwd_sweep_window_split
// but compute the values of the new message only; NI index wavefronts take the nodes in
// turn as in mrf_fwd_sweep_window_duo, each doing the argmin bookkeeping of a whole node (all
// labels) and the stores.  The value wavefronts publish h through a ring; all of a node's
// entries are written before the node's barrier, so the wavefront that raises the counter
// after the barrier needs no further wait.
template <int RMAX, int D, bool TRWP, int TW, int NI>
__global__ void __launch_bounds__(64 * (4 + NI))
mrf_fwd_sweep_window_squad(const MrfFwdParams P)
{
    constexpr int HB = 256 + 2 * TW;
    constexpr int NR = 8;                          // ring slots
    constexpr int LPI = 4;                         // label slots of an index wavefront
    static_assert(NR >= D && (NR & (NR - 1)) == 0 && NI >= 1 && NI <= 8, "ring depth");
    __shared__ float ring[NR][HB];
    __shared__ float ringw[NR];
    __shared__ float ftab[TW + 1];
    // exchanges among the value wavefronts: {step, float} per wavefront, two sets by step parity
    __shared__ __align__(16) unsigned long long hmx[2][4];     // local minima of h
    __shared__ __align__(16) unsigned long long tmx[2][4];     // local minima of the new message (general path)
    __shared__ int produced;
    __shared__ MrfWaitBlock wait_lds;             // for the waits below (mrf_wait_turn)
    __shared__ __align__(16) int consumed[8];
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int NWV = (int)(blockDim.x >> 6) - NI;   // value wavefronts come first

    const long long blk = blockIdx.x;
    int ri = 0;
    while (ri + 1 < P.r_count && blk >= P.blk_begin[ri + 1]) ++ri;
    const int r = P.r_first + ri;
    const long long local = blk - P.blk_begin[ri];
    const int nsc = P.g.nscan[r];
    const int b = (int)(local / nsc);
    const long long t = local - (long long)b * nsc;
    const int dh = P.g.dh[r], dw = P.g.dw[r];
    int y0, x0, len;
    mrf_geom_head(P.g.H, P.g.W, dh, dw, t, y0, x0, len);
    const long long N = P.g.N;
    const long long head = ((long long)b * P.g.H + y0) * P.g.W + x0;
    const long long nstep = (long long)dh * P.g.W + dw;
    const float vz = mrf_opaque_zero_f();     // keeps uniform constants in vector registers

    float f[TW];
#pragma unroll
    for (int d = 0; d < TW; ++d) f[d] = P.V[d < L ? d : L - 1] + vz;
    const float fT = P.V[L - 1] + vz;
    const bool f0zero = (P.V[0] == 0.0f);
    if ((int)threadIdx.x <= TW) ftab[threadIdx.x] = (int)threadIdx.x < TW ? P.V[(int)threadIdx.x < L ? threadIdx.x : L - 1] : fT;
    // padding and the entries of labels >= L are never written again: they never win a strict '<'
    for (int i = threadIdx.x; i < NR * HB; i += blockDim.x) (&ring[0][0])[i] = INFINITY;
    if (threadIdx.x < 8) {
        (&hmx[0][0])[threadIdx.x] = 0ull;                      // step 0: no step waits for it
        (&tmx[0][0])[threadIdx.x] = 0ull;
        consumed[threadIdx.x] = (int)threadIdx.x + 1 - NI;     // "finished" starts one turn before
    }
    if (threadIdx.x == 0) { produced = 0; mrf_wait_init(&wait_lds, P.fault, P.spin_limit); }
    const MrfWaitBlock *const wait_block = &wait_lds;
    __syncthreads();

    // the value wavefronts go first wherever they share a SIMD with index wavefronts
    if (wv < NWV) __builtin_amdgcn_s_setprio(3);
    if (wv >= NWV) {
        // ---- p, q and all stores: index wavefront jw takes steps 1 + jw, 1 + jw + NI, ... ------
        const int jw = wv - NWV;
        if (jw == 0) {
#pragma unroll
            for (int s = 0; s < LPI; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) {
                    P.m_out[((size_t)r * N + head) * L + lam] = 0.0f;
                    P.p[((size_t)r * N + head) * L + lam] = 0;
                }
            }
            if (lane == 0) P.q[(size_t)r * N + head] = 0;
        }
        int seen = 0;
        for (int n = 1 + jw; n < len; n += NI) {
            int wait_turns = 0;
            while (seen < n) {
                seen = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&produced, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                if (seen < n) mrf_wait_turn(wait_block, wait_turns);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            const int slot = n & (NR - 1);
            const float *hbuf = &ring[slot][TW];
            const float wgt = ringw[slot];
            const long long i = head + (long long)n * nstep;

            float hv[LPI];
            float hm = INFINITY;
#pragma unroll
            for (int s = 0; s < LPI; ++s) {
                hv[s] = hbuf[lane + 64 * s];           // +inf for labels >= L
                hm = mrf_min(hm, hv[s]);
            }
            const float hmin = mrf_wave_min(hm);

            float tv[LPI];
            int tp[LPI];
            float tq;
            if (__builtin_expect(__builtin_amdgcn_readfirstlane(__float_as_int(wgt)) >= 0, 1)) {
                const float gmin = __builtin_fmaf(wgt, fT, hmin);
                int mug = 0;
                bool found = false;
#pragma unroll
                for (int s = 0; s < LPI; ++s) {
                    const int lam = lane + 64 * s;
                    const float gfar = lam < L ? __builtin_fmaf(wgt, fT, hv[s]) : INFINITY;
                    const unsigned long long bal = __ballot(gfar == gmin);
                    if (!found && bal != 0ull) { found = true; mug = 64 * s + __ffsll((long long)bal) - 1; }
                }
#pragma unroll
                for (int s = 0; s < LPI; ++s) {
                    const int lam = lane + 64 * s;
                    float dl[2 * TW - 1];
#pragma unroll
                    for (int o = 0; o < 2 * TW - 1; ++o) {
                        const int dist = o < TW - 1 ? TW - 1 - o : o - (TW - 1);
                        dl[o] = __builtin_fmaf(wgt, f[dist], hbuf[lam + o - (TW - 1)]);
                    }
                    float W = dl[0];
#pragma unroll
                    for (int o = 1; o + 1 < 2 * TW - 1; o += 2) W = mrf_min3(W, dl[o], dl[o + 1]);
                    int po = 2 * TW - 2;
#pragma unroll
                    for (int o = 2 * TW - 3; o >= 0; --o) po = (dl[o] == W) ? o : po;
                    const int pW = lam + po - (TW - 1);
                    const bool wlt = W < gmin, wgt_ = W > gmin;
                    tv[s] = (lam < L) ? (wlt ? W : gmin) : INFINITY;
                    const int tie = pW < mug ? pW : mug;
                    tp[s] = wlt ? pW : (wgt_ ? mug : tie);
                }
                if (__builtin_expect(f0zero, 1)) {
                    tq = hmin;
                } else {
                    float mn = INFINITY;
#pragma unroll
                    for (int s = 0; s < LPI; ++s) mn = fminf(mn, tv[s]);
                    tq = mrf_wave_min(mn);
                }
            } else {
                // negative weight: the ordering argument does not hold, evaluate every mu
#pragma unroll
                for (int s = 0; s < LPI; ++s) {
                    const int lam = lane + 64 * s;
                    float best = INFINITY;
                    int bi = 0;
                    for (int mu = 0; mu < L; ++mu) {
                        int dist = mu > lam ? mu - lam : lam - mu;
                        dist = dist < TW ? dist : TW;
                        const float dlt = __builtin_fmaf(wgt, ftab[dist], hbuf[mu]);
                        if (dlt < best) { best = dlt; bi = mu; }
                    }
                    tv[s] = (lam < L) ? best : INFINITY;
                    tp[s] = bi;
                }
                float mn = INFINITY;
#pragma unroll
                for (int s = 0; s < LPI; ++s) mn = fminf(mn, tv[s]);
                tq = mrf_wave_min(mn);
            }
            // this slot has been read: hand it back
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            if (lane == 0) __hip_atomic_store(&consumed[jw], n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);

            int qidx = -1;
#pragma unroll
            for (int s = 0; s < LPI; ++s) {
                const unsigned long long bal = __ballot(tv[s] == tq);
                if (qidx < 0 && bal != 0ull) qidx = 64 * s + __ffsll((long long)bal) - 1;
            }
#pragma unroll
            for (int s = 0; s < LPI; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) {
                    P.m_out[((size_t)r * N + i) * L + lam] = tv[s] - tq;
                    P.p[((size_t)r * N + i) * L + lam] = (uint8_t)tp[s];
                }
            }
            if (lane == 0) P.q[(size_t)r * N + i] = (uint8_t)qidx;
        }
        return;
    }

    // ---- values: wavefront wv owns labels 64 wv .. 64 wv + 63 ---------------------------------
    const int lam = wv * 64 + lane;
    const bool valid = lam < L;
    const int lamc = valid ? lam : 0;
    const float rho = P.rho[r];
    const int n_pre = P.n_pre[r], n_src = P.n_src[r], rm_slot = P.rm_slot[r];
    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L;
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)P.src_dir[r][c - 1] * N * L : src[0];
        use[c] = ((c <= n_src) ? 1.0f : 0.0f) + vz;
        is_rm[c] = ((c - 1 == rm_slot) ? 1.0f : 0.0f) + vz;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = ((c == n_pre + 1) ? 1.0f : 0.0f) + vz;

    const int vzero = mrf_opaque_zero();
    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
    const int lastsrc = len - 2;
    float cur[D][RMAX], nxt[D][RMAX];
    float wcur[D], wnxt[D];
    auto prefetch = [&](float (&dst)[RMAX], float &wdst, int nj) {
        nj = nj < lastsrc ? nj : lastsrc;
        const long long j = head + (long long)nj * nstep;
#pragma unroll
        for (int c = 0; c < RMAX; ++c) dst[c] = src[c][(size_t)j * L + lamc];
        wdst = wbase[(size_t)((j + nstep) * P.w_mul) + vzero];
    };
    if (len >= 2) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u], u);
    }

    // Meeting point of the value wavefronts.  The hardware barrier would also wait for the index
    // wavefronts, so each value wavefront posts {step, its value} and reads the others' until all
    // carry this step; LDS keeps a wavefront's operations in order, so whoever sees the post also
    // sees what that wavefront wrote to the ring before it.  Two sets by step parity: a wavefront
    // can be at most one step ahead of the slowest, because it needs that one's post to go on.
    auto exchange_min = [&](unsigned long long (&box)[2][4], int par, int step, float val) {
        if (lane == 0)
            __hip_atomic_store(&box[par][wv], ((unsigned long long)(unsigned)step << 32) | (unsigned)__float_as_int(val),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        float m;
        bool all;
        int looks = 0;
        do {
            // all four posts in one batch of LDS reads (those of absent wavefronts are ignored)
            unsigned long long e[4];
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2)
                e[w2] = __hip_atomic_load(&box[par][w2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            m = INFINITY;
            all = true;
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) {
                const bool here = w2 < NWV;
                all = all && (!here || (int)(e[w2] >> 32) == step);
                m = mrf_min(m, here ? __int_as_float((int)(unsigned)e[w2]) : INFINITY);
            }
            all = __builtin_amdgcn_readfirstlane((int)all) != 0;
            // (the partners are a few instructions apart: look again at once, and at the clock now and then)
            if (!all && (++looks & 4095) == 0) mrf_wait_check(wait_block);
        } while (!all);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        return m;
    };

    float carry = 0.0f;
    int par = 0;
    int freed = 0;          // every step <= freed is finished by the index wavefronts (possibly stale view)
    for (int n0 = 1; n0 < len; n0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u], n0 - 1 + D + u);
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int nn = n0 + u;
            const bool past = nn >= len;
            const float wgt = wcur[u];
            const int slot = nn & (NR - 1);
            float *hb = &ring[slot][TW];

            // the slot was last used by step nn - NR
            int wait_turns = 0;
            while (__builtin_expect(!past && freed < nn - NR, 0)) {
                int lo = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&consumed[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
#pragma unroll
                for (int j = 1; j < NI; ++j) {
                    const int cj = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(&consumed[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                    lo = cj < lo ? cj : lo;
                }
                freed = lo + NI - 1;
                if (freed < nn - NR) mrf_wait_turn(wait_block, wait_turns);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");

            float v = cur[u][0];
            if (TRWP) {
                float mrm = 0.0f;
#pragma unroll
                for (int c = 1; c < RMAX; ++c) {
                    v = __builtin_fmaf(carry_at[c], carry, v);
                    v = __builtin_fmaf(use[c], cur[u][c], v);
                    mrm = __builtin_fmaf(is_rm[c], cur[u][c], mrm);
                }
                v = __builtin_fmaf(carry_at[RMAX], carry, v);
                v = rho * v;
                v = v - mrm;
            } else {
#pragma unroll
                for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[u][c], v);
                v = v + carry;
            }
            // (lanes past L rewrite the +inf their ring entries hold anyway: no divergence; what
            // they carry from node to node is never looked at)
            const float av = valid ? v : INFINITY;
            if (!past) hb[lam] = av;
            const float hloc = mrf_wave_min(av);
            // (written by every lane of the first value wavefront: no divergent branch in the step)
            if (wv == 0 && !past) ringw[slot] = wgt;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            const float hmin = exchange_min(hmx, par, nn, hloc);
            // every entry of the node is in the ring: let the index wavefronts have it
            if (wv == 0 && !past)
                __hip_atomic_store(&produced, nn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const bool wpos = __builtin_amdgcn_readfirstlane(__float_as_int(wgt)) >= 0;
            float tv;
            // (evaluated for every node, so that the usual case is straight-line code; replaced
            // below for a negative weight)
            {
                const float gmin = __builtin_fmaf(wgt, fT, hmin);
                // The two candidates at distance d share f(d), and a correctly rounded fma is
                // non-decreasing in its addend: the smaller of the two comes from the smaller h.
                float dl[TW];
                dl[0] = __builtin_fmaf(wgt, f[0], v);
#pragma unroll
                for (int d = 1; d < TW; ++d)
                    dl[d] = __builtin_fmaf(wgt, f[d], mrf_min(hb[lam - d], hb[lam + d]));
                float W = mrf_min(dl[0], gmin);
#pragma unroll
                for (int d = 1; d + 1 < TW; d += 2) W = mrf_min3(W, dl[d], dl[d + 1]);
                if ((TW & 1) == 0) W = mrf_min(W, dl[TW - 1]);
                tv = W;
            }
            if (__builtin_expect(!wpos, 0)) {
                float best = INFINITY;
                for (int mu = 0; mu < L; ++mu) {
                    int dist = mu > lam ? mu - lam : lam - mu;
                    dist = dist < TW ? dist : TW;
                    const float dlt = __builtin_fmaf(wgt, ftab[dist], hb[mu]);
                    if (dlt < best) best = dlt;
                }
                tv = best;
            }
            float tq = hmin;
            if (__builtin_expect(!(wpos && f0zero), 0)) {
                // general case: the minimum of the new message needs its own exchange
                const float tloc = mrf_wave_min(valid ? tv : INFINITY);
                tq = exchange_min(tmx, par, nn, tloc);
            }
            carry = tv - tq;
            par ^= 1;
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            wcur[u] = wnxt[u];
#pragma unroll
            for (int c = 0; c < RMAX; ++c) cur[u][c] = nxt[u][c];
        }
    }
}

// ---- dense sweep for few labels: several scanlines per wavefront ----------------------------
//
// For L <= 32 a wavefront with one scanline leaves most lanes idle.  Here a wavefront is cut
// into 64/SEG segments of SEG lanes (SEG = 16 or 32 >= L); each segment walks its own
// scanline, possibly of another direction and length than its neighbours, so everything
// that is wave-uniform in the other kernels (node addresses, weight, source flags) is
// per-lane here.  V(.,lambda) sits in SEG registers per lane, h is exchanged through a
// per-segment LDS row, the minimum over labels is a DPP row reduction (plus one swizzle
// for 32-lane segments) and q comes from the segment's slice of a ballot.
__device__ inline float mrf_segment_min21(float v, int lane)
{
    const bool up = mrf_seg21_upper(lane);
    float u = up ? v : INFINITY, lo = up ? INFINITY : v;
    u = mrf_min(u, mrf_dpp_f32<0xB1>(u));
    lo = mrf_min(lo, mrf_dpp_f32<0xB1>(lo));
    u = mrf_min(u, mrf_dpp_f32<0x4E>(u));
    lo = mrf_min(lo, mrf_dpp_f32<0x4E>(lo));
    u = mrf_min(u, mrf_dpp_f32<0x141>(u));
    lo = mrf_min(lo, mrf_dpp_f32<0x141>(lo));
    u = mrf_min(u, mrf_dpp_f32<0x140>(u));
    lo = mrf_min(lo, mrf_dpp_f32<0x140>(lo));
    // rows 1..3: lane 15 of the row before (its upper minimum) joins this row's lower minimum
    const float pu = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        __builtin_bit_cast(int, INFINITY), __builtin_bit_cast(int, u), 0x142 /* row_bcast:15 */, 0xE, 0xF, false));
    const float full = mrf_min(lo, pu);            // the whole segment's minimum, in rows 1..3 (segment = row - 1)
    // upper lanes fetch it from the first lane of the next row; lower lanes hold it already
    const int from = up ? ((lane & 48) + 16) & 63 : lane;
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(from << 2, __builtin_bit_cast(int, full)));
}

template <int SEG>
__device__ inline float mrf_segment_min(float v)
{
    if (SEG == 21) return mrf_segment_min21(v, (int)(threadIdx.x & 63));
    v = mrf_min(v, mrf_dpp_f32<0xB1>(v));
    v = mrf_min(v, mrf_dpp_f32<0x4E>(v));
    v = mrf_min(v, mrf_dpp_f32<0x141>(v));
    v = mrf_min(v, mrf_dpp_f32<0x140>(v));
    if (SEG == 32)   // partner row inside the 32-lane group: swizzle, xor lane id with 16
        v = mrf_min(v, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F)));
    return v;
}

// The same minimum for 32-lane segments without the trip through the LDS crossbar that the
// swizzle costs: five in-place DPP minima leave the minimum of lanes 0..31 in lane 31 and that of
// lanes 32..63 in lane 63; two v_readlane and a select hand them back.  For the value wavefront
// of latency-bound launches.  All 64 lanes must be active.
__device__ inline float mrf_segment_min32_regs(float v, int lane)
{
    float a, b;
    asm("s_nop 1\n\t"
        "v_min_f32_dpp %2, %2, %2 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %2, %2, %2 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %2, %2, %2 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %2, %2, %2 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %2, %2, %2 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_readlane_b32 %0, %2, 31\n\t"
        "v_readlane_b32 %1, %2, 63"
        : "=s"(a), "=s"(b), "+v"(v));
    return lane < 32 ? a : b;
}

// lowest lane of the caller's segment whose bit is set in a wavefront ballot, as a label
template <int SEG>
__device__ inline int mrf_segment_first(unsigned long long bal, int lane)
{
    if (SEG == 21) {
        const int sh = (lane / 21) * 21;
        return __ffs((int)((unsigned)(bal >> sh) & 0x1FFFFFu)) - 1;
    }
    const unsigned word = lane < 32 ? (unsigned)bal : (unsigned)(bal >> 32);
    const unsigned mine = SEG == 32 ? word : ((word >> (lane & 16)) & 0xFFFFu);
    return __ffs((int)mine) - 1;
}

// MU: source labels evaluated per node, L rounded up to a multiple of four (<= SEG, or 24 for the
// 21-lane segments, whose LDS rows are padded to 28 entries).
// IDX = 1, 2: that many further wavefronts per workgroup take the argmin tables and the stores (as in
// mrf_fwd_sweep_window_duo): the first computes values only and hands each node's h and
// weights over through a ring in LDS.  For launches that leave most issue slots idle; the host
// uses two, because an index wavefront has more to do per node than the value wavefront.
template <int SEG, int MU, int RMAX, int D, bool TRWP, int IDX>
__global__ void __launch_bounds__(64 * (1 + IDX))
mrf_fwd_sweep_packed(const MrfFwdParams P)
{
    static_assert(MU % 4 == 0 && (MU <= SEG || (SEG == 21 && MU == 24)), "source label count");
    constexpr int NSEG = 64 / SEG;                // (three segments of 21 lanes leave lane 63 idle)
    constexpr int NROW = SEG == 21 ? 4 : NSEG;    // LDS rows: the idle lane gets one of its own to scribble in
    constexpr int SEGP = SEG == 21 ? 28 : SEG + 4;   // row stride: 16-byte rows on different banks
    constexpr int NR = IDX ? 8 : 1;               // ring slots (IDX), else the one working row set
    static_assert(NR >= D || !IDX, "ring depth");
    __shared__ __align__(16) float hring[NR][NROW][SEGP];
    __shared__ float wring[NR][64];
    __shared__ int produced;
    __shared__ MrfWaitBlock wait_lds;             // for the waits below (mrf_wait_turn)
    __shared__ int consumed[2];                   // per index wavefront: last step finished
    const int L = P.g.L;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool index_wave = IDX && wave > 0;
    if (IDX && !index_wave) __builtin_amdgcn_s_setprio(3);      // the value wavefront goes first on a shared SIMD
    const int seg = lane / SEG, lam = lane % SEG;
    const bool valid = lam < L;
    const int lamc = valid ? lam : 0;
    const long long N = P.g.N;
    const long long total = P.blk_begin[P.r_count];
    const long long sl = (long long)blockIdx.x * NSEG + seg;
    const bool act_seg = sl < total && seg < NSEG;

    // per-lane description of the segment's scanline
    int r = P.r_first, nsc = 1, dh = 0, dw = 1, n_pre = 0, n_src = 0, rm_slot = -1;
    long long local = 0;
    float rho = 1.0f;
    int sdir[RMAX];
#pragma unroll
    for (int c = 0; c < RMAX; ++c) sdir[c] = 0;
    for (int ri = 0; ri < P.r_count; ++ri) {
        const int rr = P.r_first + ri;
        const bool mine = act_seg && sl >= P.blk_begin[ri] && sl < P.blk_begin[ri + 1];
        if (mine) {
            r = rr; local = sl - P.blk_begin[ri]; nsc = P.g.nscan[rr]; dh = P.g.dh[rr]; dw = P.g.dw[rr];
            rho = P.rho[rr]; n_pre = P.n_pre[rr]; n_src = P.n_src[rr]; rm_slot = P.rm_slot[rr];
#pragma unroll
            for (int c = 0; c + 1 < RMAX; ++c) sdir[c] = P.src_dir[rr][c];
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
    // Entry offsets walk along the scanline by additions: every lane has a scanline of its own, and a 64-bit
    // product per access and node costs four issue slots each.
    const long long stepL = nstep * L;
    const long long out0 = ((long long)r * N + head) * L + lam;      // entry of the first node in m_out / p
    const long long outq0 = (long long)r * N + head;                 // and in q

    const float *src[RMAX];
    float use[RMAX], carry_at[RMAX + 1], is_rm[RMAX];
    src[0] = P.unary + (size_t)P.unary_slab[r] * N * L;
    use[0] = 1.0f;
    is_rm[0] = 0.0f;
#pragma unroll
    for (int c = 1; c < RMAX; ++c) {
        src[c] = (c <= n_src) ? P.m_in + (size_t)sdir[c - 1] * N * L : src[0];
        use[c] = (c <= n_src) ? 1.0f : 0.0f;
        is_rm[c] = (c - 1 == rm_slot) ? 1.0f : 0.0f;
    }
#pragma unroll
    for (int c = 1; c <= RMAX; ++c) carry_at[c] = (c == n_pre + 1) ? 1.0f : 0.0f;

    float Vr[MU];
#pragma unroll
    for (int mu = 0; mu < MU; ++mu) Vr[mu] = (mu < L && valid) ? P.V[(size_t)mu * L + lam] : 0.0f;
    if (!index_wave) {
#pragma unroll
        for (int sl2 = 0; sl2 < NR; ++sl2) {
            hring[sl2][seg][lam] = INFINITY;      // entries mu >= L stay +inf: they never win
            if (lam < SEGP - SEG) hring[sl2][seg][SEG + lam] = INFINITY;
        }
        if (lane == 0) { produced = 0; consumed[0] = 1 - IDX; consumed[1] = 0; mrf_wait_init(&wait_lds, P.fault, P.spin_limit); }   // "finished" starts one turn before
    }
    const MrfWaitBlock *const wait_block = &wait_lds;
    __syncthreads();

    if ((!IDX || wave == 1) && act_seg && valid) {
        P.m_out[((size_t)r * N + head) * L + lam] = 0.0f;
        P.p[((size_t)r * N + head) * L + lam] = 0;
        if (lam == 0) P.q[(size_t)r * N + head] = 0;
    }

    // longest scanline of the wavefront bounds the loop
    int maxlen = 1;
#pragma unroll
    for (int sg = 0; sg < NSEG; ++sg) {
        const int l2 = __builtin_amdgcn_readlane(len, sg * SEG);
        maxlen = l2 > maxlen ? l2 : maxlen;
    }

    if (index_wave) {
        // ---- p, q and all stores, one node behind or more ----------------------------------
        // index wavefront jw takes steps 1 + jw, 1 + jw + IDX, ...
        const int jw = wave - 1;
        int seen = 0;
        long long io = out0 + (1 + jw) * stepL, iq = outq0 + (1 + jw) * nstep;
        const long long io_step = (IDX > 0 ? IDX : 1) * stepL, iq_step = (IDX > 0 ? IDX : 1) * nstep;
        for (int nn = 1 + jw; nn < maxlen; nn += (IDX > 0 ? IDX : 1), io += io_step, iq += iq_step) {
            int wait_turns = 0;
            while (seen < nn) {
                seen = __builtin_amdgcn_readfirstlane(
                    __hip_atomic_load(&produced, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                if (seen < nn) mrf_wait_turn(wait_block, wait_turns);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            const int slot = nn & (NR - 1);
            const bool act = act_seg && nn < len;
            const float wgt = wring[slot][lane];
            float dl[MU];
#pragma unroll
            for (int m4 = 0; m4 < MU; m4 += 4) {
                const float4 hv = *reinterpret_cast<const float4 *>(&hring[slot][seg][m4]);
                const float hq[4] = { hv.x, hv.y, hv.z, hv.w };
#pragma unroll
                for (int c = 0; c < 4; ++c) dl[m4 + c] = __builtin_fmaf(wgt, Vr[m4 + c], hq[c]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            if (lane == 0) __hip_atomic_store(&consumed[jw], nn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            float best = mrf_min(dl[0], dl[1]);
#pragma unroll
            for (int m = 2; m + 1 < MU; m += 2) best = mrf_min3(best, dl[m], dl[m + 1]);
            int bidx = MU - 1;
            mrf_static_for<MU / 4>([&](auto g4) {
                constexpr int m0 = MU - 4 - 4 * decltype(g4)::value;      // groups from the top down
                mrf_first_equal4<m0>(bidx, best, dl[m0], dl[m0 + 1], dl[m0 + 2], dl[m0 + 3]);
            });
            const float tv = valid ? best : INFINITY;
            const float tq = mrf_segment_min<SEG>(tv);
            const int qidx = mrf_segment_first<SEG>(__ballot(tv == tq), lane);
            if (act && valid) {
                P.m_out[io] = tv - tq;
                P.p[io] = (uint8_t)bidx;
                if (lam == 0) P.q[iq] = (uint8_t)qidx;
            }
        }
        return;
    }

    const float *wbase = P.w + (P.w_mul ? (size_t)r * N : 0);
    const int lastsrc = len >= 2 ? len - 2 : 0;
    float cur[D][RMAX], nxt[D][RMAX];
    float wcur[D], wnxt[D];
    // source nodes 0, 1, 2, ... in the order of the calls; past the end: reload the last one, never used
    int pf_n = 0;
    long long pf_off = head * L + lamc;
    long long pf_w = (len >= 2 ? head + nstep : head) * P.w_mul;
    const long long stepW = nstep * P.w_mul;
    auto prefetch = [&](float (&dst)[RMAX], float &wdst) {
#pragma unroll
        for (int c = 0; c < RMAX; ++c) dst[c] = src[c][pf_off];
        wdst = wbase[pf_w];
        const bool more = pf_n < lastsrc;
        pf_off += more ? stepL : 0;
        pf_w += more ? stepW : 0;
        ++pf_n;
    };
#pragma unroll
    for (int u = 0; u < D; ++u) prefetch(cur[u], wcur[u]);
    long long so = out0 + stepL, sq = outq0 + nstep;        // entries of node 1, the first one updated

    float carry = 0.0f;
    int freed = 0;          // every step <= freed has been read by the index wavefront (possibly stale view)
    for (int n0 = 1; n0 < maxlen; n0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) prefetch(nxt[u], wnxt[u]);
#pragma unroll
        for (int u = 0; u < D; ++u, so += stepL, sq += nstep) {
            const int nn = n0 + u;
            const bool act = act_seg && nn < len;       // this segment still has a node to update
            const float wgt = wcur[u];

            float v = cur[u][0];
            if (TRWP) {
                float mrm = 0.0f;
#pragma unroll
                for (int c = 1; c < RMAX; ++c) {
                    v = __builtin_fmaf(carry_at[c], carry, v);
                    v = __builtin_fmaf(use[c], cur[u][c], v);
                    mrm = __builtin_fmaf(is_rm[c], cur[u][c], mrm);
                }
                v = __builtin_fmaf(carry_at[RMAX], carry, v);
                v = rho * v;
                v = v - mrm;
            } else {
#pragma unroll
                for (int c = 1; c < RMAX; ++c) v = __builtin_fmaf(use[c], cur[u][c], v);
                v = v + carry;
            }
            const int slot = IDX ? (nn & (NR - 1)) : 0;
            if (IDX) {
                // the slot was last used by step nn - NR
                int wait_turns = 0;
                while (__builtin_expect(freed < nn - NR, 0)) {
                    // the index wavefronts take the steps in turn: behind the slowest one's last
                    // step, the others have finished theirs
                    int lo = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(&consumed[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                    if (IDX > 1) {
                        const int c1 = __builtin_amdgcn_readfirstlane(
                            __hip_atomic_load(&consumed[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                        lo = c1 < lo ? c1 : lo;
                    }
                    freed = lo + IDX - 1;
                    if (freed < nn - NR) mrf_wait_turn(wait_block, wait_turns);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                }
                wring[slot][lane] = wgt;
            }
            // (lanes past L rewrite the +inf their entries hold anyway: no divergence; what they
            // carry from node to node is never looked at)
            hring[slot][seg][lam] = valid ? v : INFINITY;
            mrf_wave_lds_fence();

            // all candidates, their minimum with three-operand minima, then the lowest index
            // that attains it (scanning downwards, so the lowest survives)
            float dl[MU];
#pragma unroll
            for (int m4 = 0; m4 < MU; m4 += 4) {
                const float4 hv = *reinterpret_cast<const float4 *>(&hring[slot][seg][m4]);
                const float hq[4] = { hv.x, hv.y, hv.z, hv.w };
#pragma unroll
                for (int c = 0; c < 4; ++c) dl[m4 + c] = __builtin_fmaf(wgt, Vr[m4 + c], hq[c]);
            }
            if (IDX) {
                // (LDS keeps a wavefront's operations in order: the counter lands behind the entries)
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                if (lane == 0) __hip_atomic_store(&produced, nn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else {
                mrf_wave_lds_fence();
            }
            float best = mrf_min(dl[0], dl[1]);
#pragma unroll
            for (int m = 2; m + 1 < MU; m += 2) best = mrf_min3(best, dl[m], dl[m + 1]);
            const float tv = valid ? best : INFINITY;
            const float tq = (IDX && SEG == 32) ? mrf_segment_min32_regs(tv, lane) : mrf_segment_min<SEG>(tv);
            carry = tv - tq;
            if (IDX) continue;                    // the index wavefront does the rest

            int bidx = MU - 1;
            mrf_static_for<MU / 4>([&](auto g4) {
                constexpr int m0 = MU - 4 - 4 * decltype(g4)::value;      // groups from the top down
                mrf_first_equal4<m0>(bidx, best, dl[m0], dl[m0 + 1], dl[m0 + 2], dl[m0 + 3]);
            });
            const int qidx = mrf_segment_first<SEG>(__ballot(tv == tq), lane);

            if (act && valid) {
                P.m_out[so] = carry;
                P.p[so] = (uint8_t)bidx;
                if (lam == 0) P.q[sq] = (uint8_t)qidx;
            }
        }
#pragma unroll
        for (int u = 0; u < D; ++u) {
            wcur[u] = wnxt[u];
#pragma unroll
            for (int c = 0; c < RMAX; ++c) cur[u][c] = nxt[u][c];
        }
    }
}
