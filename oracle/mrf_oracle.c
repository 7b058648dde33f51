/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C implementation of the min-sum message passing of
 * "Fast and Differentiable Message Passing on Pairwise Markov Random Fields":
 * forward ISGMR (Alg. 1), forward TRWP (Alg. 2), backprop ISGMR (Alg. 3), backprop
 * TRWP (Alg. 4).  It exists only to check the GPU library; it shares no code, header,
 * table or helper with it, and only tests, the smoke check and the bench's CPU
 * baseline may call it.
 *
 * Built twice from the same source: single-threaded (the oracle of record) and with
 * -fopenmp (forward scanlines of one direction in parallel -- they write disjoint
 * outputs, so results are bit-identical; used to make full-size parity affordable).
 *
 * Readings taken where the paper is silent or ambiguous:
 *  1. Ties in both argmins go to the lowest label (strict '<', ascending scan).
 *  2. fp evaluation order: the lambda-independent part h[mu] is summed left to right as
 *     written in mrf_oracle_impl.h (ISGMR: unary, then m-hat^r, then the other
 *     directions in index order; TRWP: unary, then all directions in index order, one
 *     multiplication by rho, one subtraction of m^{r-}); the pairwise term enters through
 *     a single fused multiply-add fma(theta_{i-r,i}, V(mu,lambda), h[mu]).
 *  3. First node of a scanline: message 0 for ever, p = q = 0, gradients reaching it
 *     are dropped (messages are initialised to 0, Alg. 1 line 1 / Alg. 2 line 1).
 *  4. TRWP sweeps the directions in the order of dirs[]; its backward pass sweeps them
 *     in the reverse order (needed by the in-place update, Sec. 4).
 *  5. Alg. 3 lines 16-18 are read as "grad m-hat <- grad m" (Appendix D.3 item 2).
 *  6. If the opposite direction r- is not in the direction set its term is absent.
 *  7. V is indexed V[mu at the previous node i-r][lambda at node i] for every direction.
 *  8. rho is one value per direction, or (optional array) one value per directed edge as Eq.
 *     trwp writes it; the edge weight and the per-edge rho of edge (i-r,i) in direction r
 *     are stored at node i.
 *  9. Gradients of theta_i, theta_{i-r,i} and V accumulate over all iterations,
 *     directions and nodes (Appendix D.3 item 1).
 * 10. Standard SGM (Eq. sgm_old): first node's message = its unary; computed messages are
 *     reparametrised by Eq. isgmr-norm like all others.
 * Pins (tests/test_oracle_*.py): brute-force min-marginals on chains and trees,
 * discounted brute force for TRWP with rho != 1, Viterbi for K = 1, the iteration-2 messages of
 * ISGMR on a loopy grid enumerated from those of iteration 1, standard SGM by scanline
 * enumeration with the node's own unary inside the minimum, invariants, central finite
 * differences of the double instantiation; tests/test_oracle_mutations.py plants mistakes in a
 * copy of this source and checks that the pins catch each.  Printed-value parity: unpinned (the
 * paper prints no worked numeric example).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MRFO_MAX_DIRS 16

typedef struct {
    int B, H, W, L, R, K;
    int dh[MRFO_MAX_DIRS], dw[MRFO_MAX_DIRS];
    int opp[MRFO_MAX_DIRS];  /* index of the opposite direction r-, or -1 */
} grid_t;

static int grid_init(grid_t *g, int B, int H, int W, int L, int R, const int *dirs, int K)
{
    if (B < 1 || H < 1 || W < 1 || L < 1 || L > 256 || R < 1 || R > MRFO_MAX_DIRS || K < 1)
        return -1;
    g->B = B; g->H = H; g->W = W; g->L = L; g->R = R; g->K = K;
    for (int r = 0; r < R; ++r) {
        g->dh[r] = dirs[2 * r];
        g->dw[r] = dirs[2 * r + 1];
        if (g->dh[r] == 0 && g->dw[r] == 0) return -1;
    }
    for (int r = 0; r < R; ++r) {
        g->opp[r] = -1;
        for (int d = 0; d < R; ++d) {
            if (d != r && g->dh[d] == g->dh[r] && g->dw[d] == g->dw[r]) return -1;
            if (g->dh[d] == -g->dh[r] && g->dw[d] == -g->dw[r]) g->opp[r] = d;
        }
    }
    return 0;
}

static size_t grid_nodes(const grid_t *g) { return (size_t)g->B * g->H * g->W; }
static int in_grid(const grid_t *g, int y, int x) { return y >= 0 && y < g->H && x >= 0 && x < g->W; }
static size_t node_index(const grid_t *g, int b, int y, int x)
{
    return ((size_t)b * g->H + y) * g->W + x;
}

/* first nodes of the scanlines of direction r: nodes whose predecessor is off the grid */
typedef struct { size_t n; int *b, *y, *x; } heads_t;

static void heads_collect(const grid_t *g, int r, heads_t *hd)
{
    size_t cap = grid_nodes(g);
    hd->n = 0;
    hd->b = (int *)malloc(sizeof(int) * cap);
    hd->y = (int *)malloc(sizeof(int) * cap);
    hd->x = (int *)malloc(sizeof(int) * cap);
    for (int b = 0; b < g->B; ++b)
        for (int y = 0; y < g->H; ++y)
            for (int x = 0; x < g->W; ++x)
                if (!in_grid(g, y - g->dh[r], x - g->dw[r])) {
                    hd->b[hd->n] = b; hd->y[hd->n] = y; hd->x[hd->n] = x; hd->n++;
                }
}

static void heads_free(heads_t *hd) { free(hd->b); free(hd->y); free(hd->x); }

/* number of scanlines of direction r (for tests of the first-node count, Eq. supp-wide) */
long mrfo_count_scanlines(int H, int W, int dh, int dw)
{
    int dirs[2] = { dh, dw };
    grid_t g;
    heads_t hd;
    if (grid_init(&g, 1, H, W, 1, 1, dirs, 1)) return -1;
    heads_collect(&g, 0, &hd);
    long n = (long)hd.n;
    heads_free(&hd);
    return n;
}

int mrfo_openmp_enabled(void)
{
#ifdef _OPENMP
    return 1;
#else
    return 0;
#endif
}

#define REAL float
#define REAL_FMA fmaf
#define NAME(x) x##_f32
#include "mrf_oracle_impl.h"
#undef REAL
#undef REAL_FMA
#undef NAME

#define REAL double
#define REAL_FMA fma
#define NAME(x) x##_f64
#include "mrf_oracle_impl.h"
#undef REAL
#undef REAL_FMA
#undef NAME
