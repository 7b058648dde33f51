/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.  Body of the oracle, included twice by
 * mrf_oracle.c: once with REAL=float (the precision the paper computes in; every
 * argmin decision is taken in it) and once with REAL=double (truth for finite
 * differences and for brute-force comparisons).
 *
 * Everything here is the paper's algorithms taken step by step, in the paper's
 * order and notation, with no blocking, fusion or reordering:
 *   Alg. 1  forward ISGMR      Alg. 2  forward TRWP
 *   Alg. 3  backprop ISGMR     Alg. 4  backprop TRWP   (Appendix A)
 *   Sec. 3.2  standard single-pass SGM (Eq. sgm_old, Eq. isgmr-aggregation-old), forward only
 * using the pairwise decomposition theta_{i-r,i}(mu,lambda) = theta_{i-r,i} V(mu,lambda)
 * (Sec. 5.1 "MRF model parameters", Appendix D.2) so that the gradients are those of
 * the edge weights (Eq. supp-gradient-edge) and of V (Eq. supp-gradient-smoothness).
 *
 * Layouts (row-major, last index fastest):
 *   unary, cost, grad_cost, grad_unary   [B][H][W][L]
 *   V, grad_V                            [L][L]   V[mu at i-r][lambda at i]
 *   w, grad_w                            [R][B][H][W]   entry (r,i) = theta_{i-r,i}
 *   messages                             [R][B][H][W][L]
 *   p                                    [K][R][B][H][W][L]  uint8
 *   q                                    [K][R][B][H][W]     uint8
 *   theta_e, grad_theta_e (optional)     [R][B][H][W][L][L]  entry (r,i,mu,lambda) =
 *                                        theta_{i-r,i}(mu,lambda): pairwise potentials given per
 *                                        edge as in Eq. isgmr / Eq. trwp, instead of w and V
 * A node whose predecessor i-r lies outside the grid is the first node of its
 * scanline: its message in direction r is 0 for ever and its p, q entries are 0.
 *
 * Parity status of the readings taken where the paper is silent is listed in the
 * header of mrf_oracle.c.
 */

#ifndef REAL
#error "define REAL, REAL_FMA and NAME() before including this file"
#endif

/* ---- one message update: Alg. 1 lines 6-13 / Alg. 2 lines 6-13 ------------------
 * h[mu]  : everything inside the min that does not depend on lambda
 * wgt    : edge weight theta_{i-r,i}
 * Te     : the edge's own table theta_{i-r,i}(mu,lambda) [L][L] where the problem gives
 *          pairwise potentials per edge (Eq. isgmr as written), else NULL and the
 *          potential is wgt * V(mu,lambda)
 * out    : normalised message (Eq. isgmr-norm), pidx[lambda] = argmin_mu (lowest
 *          index on ties), returns q = argmin_lambda (lowest index on ties).      */
static int NAME(node_update)(int L, const REAL *h, REAL wgt, const REAL *V, const REAL *Te,
                             REAL *out, uint8_t *pidx)
{
    for (int lam = 0; lam < L; ++lam) {
        REAL best = (REAL)INFINITY;
        int arg = 0;
        for (int mu = 0; mu < L; ++mu) {
            REAL delta = Te ? h[mu] + Te[(size_t)mu * L + lam]
                            : REAL_FMA(wgt, V[(size_t)mu * L + lam], h[mu]);
            if (delta < best) { best = delta; arg = mu; }
        }
        out[lam] = best;
        pidx[lam] = (uint8_t)arg;
    }
    int q = 0;
    for (int lam = 1; lam < L; ++lam)
        if (out[lam] < out[q]) q = lam;
    REAL mn = out[q];
    for (int lam = 0; lam < L; ++lam) out[lam] = out[lam] - mn;
    return q;
}

/* final costs and labels: Eq. isgmr-aggregation and Eq. disp */
static void NAME(aggregate)(const grid_t *g, const REAL *unary, const REAL *m,
                            REAL *cost, uint8_t *labels)
{
    const size_t N = grid_nodes(g);
    const int L = g->L;
    for (size_t i = 0; i < N; ++i) {
        for (int lam = 0; lam < L; ++lam) {
            REAL c = unary[i * L + lam];
            for (int d = 0; d < g->R; ++d) c = c + m[((size_t)d * N + i) * L + lam];
            cost[i * L + lam] = c;
        }
        if (labels) {
            int a = 0;
            for (int lam = 1; lam < L; ++lam)
                if (cost[i * L + lam] < cost[i * L + a]) a = lam;
            labels[i] = (uint8_t)a;
        }
    }
}

/* ================================ Alg. 1 ======================================= */
int NAME(mrfo_isgmr_forward)(int B, int H, int W, int L, int R, const int *dirs, int K,
                             const REAL *unary, const REAL *V, const REAL *w, REAL w_scalar,
                             const REAL *theta_e,
                             REAL *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                             REAL *messages)
{
    grid_t g;
    if (grid_init(&g, B, H, W, L, R, dirs, K)) return -1;
    const size_t N = grid_nodes(&g);
    REAL *m = (REAL *)calloc((size_t)R * N * L, sizeof(REAL));      /* m      <- 0 */
    REAL *mhat = (REAL *)calloc((size_t)R * N * L, sizeof(REAL));   /* m-hat  <- 0 */
    heads_t hd;
    memset(p, 0, (size_t)K * R * N * L);
    memset(q, 0, (size_t)K * R * N);

    for (int k = 0; k < K; ++k) {
        for (int r = 0; r < R; ++r) {
            const int rm = g.opp[r];
            heads_collect(&g, r, &hd);
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 4)
#endif
            for (long t = 0; t < (long)hd.n; ++t) {          /* scanlines: independent */
                REAL *h = (REAL *)malloc(sizeof(REAL) * L);
                int b = hd.b[t], y = hd.y[t], x = hd.x[t];
                for (;;) {                                   /* nodes: sequential */
                    int yn = y + g.dh[r], xn = x + g.dw[r];
                    if (!in_grid(&g, yn, xn)) break;
                    size_t j = node_index(&g, b, y, x), i = node_index(&g, b, yn, xn);
                    for (int mu = 0; mu < L; ++mu) {
                        /* Eq. isgmr's bracket without the pairwise term: the terms known from
                         * iteration k first (unary, then the other directions in index order),
                         * the running message of this iteration last */
                        REAL a = unary[j * L + mu];
                        for (int d = 0; d < R; ++d)
                            if (d != r && d != rm) a = a + m[((size_t)d * N + j) * L + mu];
                        a = a + mhat[((size_t)r * N + j) * L + mu];
                        h[mu] = a;
                    }
                    REAL wgt = w ? w[(size_t)r * N + i] : w_scalar;
                    const REAL *Te = theta_e ? theta_e + ((size_t)r * N + i) * L * L : NULL;
                    int qq = NAME(node_update)(L, h, wgt, V, Te, &mhat[((size_t)r * N + i) * L],
                                               &p[(((size_t)k * R + r) * N + i) * L]);
                    q[((size_t)k * R + r) * N + i] = (uint8_t)qq;
                    y = yn; x = xn;
                }
                free(h);
            }
            heads_free(&hd);
        }
        memcpy(m, mhat, sizeof(REAL) * (size_t)R * N * L);   /* m <- m-hat after the iteration */
    }
    NAME(aggregate)(&g, unary, m, cost, labels);
    if (messages) memcpy(messages, m, sizeof(REAL) * (size_t)R * N * L);
    free(m); free(mhat);
    return 0;
}

/* ==================== standard single-pass SGM (Sec. 3.2) ====================== *
 * The update in the form the SGM paper gives it, Eq. sgm_old: the message to node i holds
 * the node's own unary,
 *     m^r_i(lambda) = theta_i(lambda) + min_mu ( m^r_{i-r}(mu) + theta_{i-r,i}(mu,lambda) ),
 * one pass over every direction, and the final cost is the plain sum of the messages,
 * Eq. isgmr-aggregation-old (which counts every unary |R| times -- the over-counting that
 * the revised update removes).
 * Readings: the first node of a scanline has nothing before it, so its message is its
 * unary; every computed message is reparametrised by Eq. isgmr-norm (minimum over labels
 * subtracted, q = its lowest argmin), as the paper states for messages in general; ties
 * and the fused multiply-add as everywhere else.  p, q have the K = 1 layout.            */
int NAME(mrfo_sgm_standard_forward)(int B, int H, int W, int L, int R, const int *dirs,
                                    const REAL *unary, const REAL *V, const REAL *w, REAL w_scalar,
                                    REAL *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                                    REAL *messages)
{
    grid_t g;
    if (grid_init(&g, B, H, W, L, R, dirs, 1)) return -1;
    const size_t N = grid_nodes(&g);
    REAL *m = (REAL *)calloc((size_t)R * N * L, sizeof(REAL));
    REAL *t = (REAL *)malloc(sizeof(REAL) * L);
    heads_t hd;
    memset(p, 0, (size_t)R * N * L);
    memset(q, 0, (size_t)R * N);
    for (int r = 0; r < R; ++r) {
        heads_collect(&g, r, &hd);
        for (size_t s = 0; s < hd.n; ++s) {
            int b = hd.b[s], y = hd.y[s], x = hd.x[s];
            size_t j = node_index(&g, b, y, x);
            for (int lam = 0; lam < L; ++lam) m[((size_t)r * N + j) * L + lam] = unary[j * L + lam];
            for (;;) {
                int yn = y + g.dh[r], xn = x + g.dw[r];
                if (!in_grid(&g, yn, xn)) break;
                size_t i = node_index(&g, b, yn, xn);
                j = node_index(&g, b, y, x);
                REAL wgt = w ? w[(size_t)r * N + i] : w_scalar;
                const REAL *prev = &m[((size_t)r * N + j) * L];
                REAL *out = &m[((size_t)r * N + i) * L];
                for (int lam = 0; lam < L; ++lam) {
                    REAL best = (REAL)INFINITY;
                    int arg = 0;
                    for (int mu = 0; mu < L; ++mu) {
                        REAL delta = REAL_FMA(wgt, V[(size_t)mu * L + lam], prev[mu]);
                        if (delta < best) { best = delta; arg = mu; }
                    }
                    t[lam] = best;
                    p[((size_t)r * N + i) * L + lam] = (uint8_t)arg;
                }
                for (int lam = 0; lam < L; ++lam) t[lam] = unary[i * L + lam] + t[lam];
                int qq = 0;
                for (int lam = 1; lam < L; ++lam)
                    if (t[lam] < t[qq]) qq = lam;
                q[(size_t)r * N + i] = (uint8_t)qq;
                REAL mn = t[qq];
                for (int lam = 0; lam < L; ++lam) out[lam] = t[lam] - mn;
                y = yn; x = xn;
            }
        }
        heads_free(&hd);
    }
    for (size_t i = 0; i < N; ++i) {
        for (int lam = 0; lam < L; ++lam) {
            REAL c = (REAL)0;
            for (int d = 0; d < R; ++d) c = c + m[((size_t)d * N + i) * L + lam];
            cost[i * L + lam] = c;
        }
        if (labels) {
            int a = 0;
            for (int lam = 1; lam < L; ++lam)
                if (cost[i * L + lam] < cost[i * L + a]) a = lam;
            labels[i] = (uint8_t)a;
        }
    }
    if (messages) memcpy(messages, m, sizeof(REAL) * (size_t)R * N * L);
    free(m); free(t);
    return 0;
}

/* ================================ Alg. 2 ======================================= */
int NAME(mrfo_trwp_forward)(int B, int H, int W, int L, int R, const int *dirs, int K,
                            const REAL *unary, const REAL *V, const REAL *w, REAL w_scalar,
                            const REAL *rho, const REAL *rho_edge, const REAL *theta_e,
                            REAL *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                            REAL *messages)
{
    grid_t g;
    if (grid_init(&g, B, H, W, L, R, dirs, K)) return -1;
    const size_t N = grid_nodes(&g);
    REAL *m = (REAL *)calloc((size_t)R * N * L, sizeof(REAL));
    heads_t hd;
    memset(p, 0, (size_t)K * R * N * L);
    memset(q, 0, (size_t)K * R * N);

    for (int k = 0; k < K; ++k) {
        for (int r = 0; r < R; ++r) {                        /* directions: sequential */
            const int rm = g.opp[r];
            heads_collect(&g, r, &hd);
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 4)
#endif
            for (long t = 0; t < (long)hd.n; ++t) {
                REAL *h = (REAL *)malloc(sizeof(REAL) * L);
                int b = hd.b[t], y = hd.y[t], x = hd.x[t];
                for (;;) {
                    int yn = y + g.dh[r], xn = x + g.dw[r];
                    if (!in_grid(&g, yn, xn)) break;
                    size_t j = node_index(&g, b, y, x), i = node_index(&g, b, yn, xn);
                    for (int mu = 0; mu < L; ++mu) {
                        REAL s = unary[j * L + mu];
                        for (int d = 0; d < R; ++d) s = s + m[((size_t)d * N + j) * L + mu];
                        /* rho_{i-r,i} of Eq. trwp: per edge where an array is given (stored like
                         * the edge weight, at the node the edge arrives at), else per direction */
                        REAL a = (rho_edge ? rho_edge[(size_t)r * N + i] : rho[r]) * s;
                        if (rm >= 0) a = a - m[((size_t)rm * N + j) * L + mu];
                        h[mu] = a;
                    }
                    REAL wgt = w ? w[(size_t)r * N + i] : w_scalar;
                    const REAL *Te = theta_e ? theta_e + ((size_t)r * N + i) * L * L : NULL;
                    int qq = NAME(node_update)(L, h, wgt, V, Te, &m[((size_t)r * N + i) * L],
                                               &p[(((size_t)k * R + r) * N + i) * L]);
                    q[((size_t)k * R + r) * N + i] = (uint8_t)qq;
                    y = yn; x = xn;
                }
                free(h);
            }
            heads_free(&hd);
        }
    }
    NAME(aggregate)(&g, unary, m, cost, labels);
    if (messages) memcpy(messages, m, sizeof(REAL) * (size_t)R * N * L);
    free(m);
    return 0;
}

/* ---- backward of one message update (Alg. 3 lines 8-15 / Alg. 4 lines 6-13) ----
 * g[lambda] is the gradient of the normalised message at node i; it is modified in
 * place by the reparametrisation step (Eq. supp-isgmr-back-norm).  Also accumulates the
 * edge-weight gradient (Eq. supp-gradient-edge) and the V gradient
 * (Eq. supp-gradient-smoothness); neither carries rho (Alg. 4 line 12).  Where the
 * problem gives pairwise potentials per edge, gTe is the edge's gradient table and
 * receives g(lambda) at (p(lambda), lambda) (Eq. supp-gradient-pairwise).            */
static void NAME(norm_backward_and_pairwise)(int L, REAL *g, int qstar, const uint8_t *pidx,
                                             REAL wgt, const REAL *V, REAL *gw_entry, REAL *gV,
                                             REAL *gTe)
{
    REAL tot = (REAL)0;
    for (int lam = 0; lam < L; ++lam) tot = tot + g[lam];
    g[qstar] = g[qstar] - tot;
    if (gw_entry) {
        REAL acc = (REAL)0;
        for (int lam = 0; lam < L; ++lam) acc = acc + g[lam] * V[(size_t)pidx[lam] * L + lam];
        *gw_entry = *gw_entry + acc;
    }
    if (gV)
        for (int lam = 0; lam < L; ++lam)
            gV[(size_t)pidx[lam] * L + lam] = gV[(size_t)pidx[lam] * L + lam] + wgt * g[lam];
    if (gTe)
        for (int lam = 0; lam < L; ++lam)
            gTe[(size_t)pidx[lam] * L + lam] = gTe[(size_t)pidx[lam] * L + lam] + g[lam];
}

/* ================================ Alg. 3 ======================================= */
int NAME(mrfo_isgmr_backward)(int B, int H, int W, int L, int R, const int *dirs, int K,
                              const REAL *V, const REAL *w, REAL w_scalar,
                              const REAL *grad_cost, const uint8_t *p, const uint8_t *q,
                              REAL *grad_unary, REAL *grad_w, REAL *grad_V, REAL *grad_theta_e)
{
    grid_t g;
    if (grid_init(&g, B, H, W, L, R, dirs, K)) return -1;
    const size_t N = grid_nodes(&g), NL = N * (size_t)L;
    REAL *G = (REAL *)calloc((size_t)R * NL, sizeof(REAL));       /* grad of m      */
    REAL *Ghat = (REAL *)malloc(sizeof(REAL) * (size_t)R * NL);   /* grad of m-hat  */
    REAL *gl = (REAL *)malloc(sizeof(REAL) * L);
    heads_t hd;
    /* back Eq. isgmr-aggregation: every direction's message and the unary receive grad c */
    for (int r = 0; r < R; ++r) memcpy(Ghat + (size_t)r * NL, grad_cost, sizeof(REAL) * NL);
    memcpy(grad_unary, grad_cost, sizeof(REAL) * NL);
    if (grad_w) memset(grad_w, 0, sizeof(REAL) * (size_t)R * N);
    if (grad_V) memset(grad_V, 0, sizeof(REAL) * (size_t)L * L);
    if (grad_theta_e) memset(grad_theta_e, 0, sizeof(REAL) * (size_t)R * N * L * L);

    for (int k = K - 1; k >= 0; --k) {
        memset(G, 0, sizeof(REAL) * (size_t)R * NL);                      /* zero-out */
        for (int r = 0; r < R; ++r) {
            const int rm = g.opp[r];
            heads_collect(&g, r, &hd);
            for (size_t t = 0; t < hd.n; ++t) {
                /* walk to the last node of the scanline, then come back */
                int b = hd.b[t], y = hd.y[t], x = hd.x[t];
                while (in_grid(&g, y + g.dh[r], x + g.dw[r])) { y += g.dh[r]; x += g.dw[r]; }
                for (;;) {
                    int yp = y - g.dh[r], xp = x - g.dw[r];
                    if (!in_grid(&g, yp, xp)) break;        /* (y,x) is the first node */
                    size_t i = node_index(&g, b, y, x), j = node_index(&g, b, yp, xp);
                    const uint8_t *pidx = &p[(((size_t)k * R + r) * N + i) * L];
                    REAL wgt = w ? w[(size_t)r * N + i] : w_scalar;
                    for (int lam = 0; lam < L; ++lam) gl[lam] = Ghat[((size_t)r * N + i) * L + lam];
                    NAME(norm_backward_and_pairwise)(L, gl, q[((size_t)k * R + r) * N + i], pidx,
                                                     wgt, V, grad_w ? &grad_w[(size_t)r * N + i] : NULL,
                                                     grad_V,
                                                     grad_theta_e ? grad_theta_e + ((size_t)r * N + i) * L * L : NULL);
                    for (int lam = 0; lam < L; ++lam) {
                        int mu = pidx[lam];
                        grad_unary[j * L + mu] = grad_unary[j * L + mu] + gl[lam];
                        Ghat[((size_t)r * N + j) * L + mu] = Ghat[((size_t)r * N + j) * L + mu] + gl[lam];
                        for (int d = 0; d < R; ++d)
                            if (d != r && d != rm)
                                G[((size_t)d * N + j) * L + mu] = G[((size_t)d * N + j) * L + mu] + gl[lam];
                    }
                    y = yp; x = xp;
                }
            }
            heads_free(&hd);
        }
        /* Alg. 3 lines 16-18 read as: the consumed grad m-hat is dropped and the gradient
         * gathered for m (= m-hat of the previous iteration) takes its place.            */
        memcpy(Ghat, G, sizeof(REAL) * (size_t)R * NL);
    }
    free(G); free(Ghat); free(gl);
    return 0;
}

/* ================================ Alg. 4 ======================================= */
int NAME(mrfo_trwp_backward)(int B, int H, int W, int L, int R, const int *dirs, int K,
                             const REAL *V, const REAL *w, REAL w_scalar, const REAL *rho,
                             const REAL *rho_edge, const REAL *grad_cost, const uint8_t *p, const uint8_t *q,
                             REAL *grad_unary, REAL *grad_w, REAL *grad_V, REAL *grad_theta_e)
{
    grid_t g;
    if (grid_init(&g, B, H, W, L, R, dirs, K)) return -1;
    const size_t N = grid_nodes(&g), NL = N * (size_t)L;
    REAL *G = (REAL *)malloc(sizeof(REAL) * (size_t)R * NL);
    REAL *gl = (REAL *)malloc(sizeof(REAL) * L);
    heads_t hd;
    for (int r = 0; r < R; ++r) memcpy(G + (size_t)r * NL, grad_cost, sizeof(REAL) * NL);
    memcpy(grad_unary, grad_cost, sizeof(REAL) * NL);
    if (grad_w) memset(grad_w, 0, sizeof(REAL) * (size_t)R * N);
    if (grad_V) memset(grad_V, 0, sizeof(REAL) * (size_t)L * L);
    if (grad_theta_e) memset(grad_theta_e, 0, sizeof(REAL) * (size_t)R * N * L * L);

    for (int k = K - 1; k >= 0; --k) {
        for (int r = R - 1; r >= 0; --r) {       /* reverse of the forward direction order */
            const int rm = g.opp[r];
            heads_collect(&g, r, &hd);
            for (size_t t = 0; t < hd.n; ++t) {
                int b = hd.b[t], y = hd.y[t], x = hd.x[t];
                while (in_grid(&g, y + g.dh[r], x + g.dw[r])) { y += g.dh[r]; x += g.dw[r]; }
                for (;;) {
                    int yp = y - g.dh[r], xp = x - g.dw[r];
                    if (!in_grid(&g, yp, xp)) break;
                    size_t i = node_index(&g, b, y, x), j = node_index(&g, b, yp, xp);
                    const uint8_t *pidx = &p[(((size_t)k * R + r) * N + i) * L];
                    REAL wgt = w ? w[(size_t)r * N + i] : w_scalar;
                    for (int lam = 0; lam < L; ++lam) gl[lam] = G[((size_t)r * N + i) * L + lam];
                    NAME(norm_backward_and_pairwise)(L, gl, q[((size_t)k * R + r) * N + i], pidx,
                                                     wgt, V, grad_w ? &grad_w[(size_t)r * N + i] : NULL,
                                                     grad_V,
                                                     grad_theta_e ? grad_theta_e + ((size_t)r * N + i) * L * L : NULL);
                    for (int lam = 0; lam < L; ++lam) {
                        int mu = pidx[lam];
                        REAL sg = (rho_edge ? rho_edge[(size_t)r * N + i] : rho[r]) * gl[lam];
                        grad_unary[j * L + mu] = grad_unary[j * L + mu] + sg;
                        for (int d = 0; d < R; ++d)
                            G[((size_t)d * N + j) * L + mu] = G[((size_t)d * N + j) * L + mu] + sg;
                        if (rm >= 0)
                            G[((size_t)rm * N + j) * L + mu] = G[((size_t)rm * N + j) * L + mu] - gl[lam];
                    }
                    y = yp; x = xp;
                }
            }
            heads_free(&hd);
            memset(G + (size_t)r * NL, 0, sizeof(REAL) * NL);            /* zero-out */
        }
    }
    free(G); free(gl);
    return 0;
}
