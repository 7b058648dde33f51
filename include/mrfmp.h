/*
 * libmrfmp -- min-sum message passing on grid pairwise MRFs for AMD MI355X (gfx950).
 *
 * C ABI of the ISGMR and TRWP forward sweeps and their index-driven backward passes
 * ("Fast and Differentiable Message Passing on Pairwise Markov Random Fields",
 * Alg. 1-4).  Plain pointers and sizes only.
 *
 * Conventions shared by every entry point
 * ----------------------------------------
 *  - Pointers marked DEVICE are HIP device pointers on the current device; pointers
 *    marked HOST are ordinary host memory read during the call.
 *  - All tensors are dense, row-major, last index fastest:
 *        unary, cost, grad_cost, grad_unary   [B][H][W][L]   float
 *        pairwise, grad_pairwise              [L][L]         float  V[mu at i-r][lambda at i]
 *        edge_weight, grad_edge_weight        [R][B][H][W]   float  entry (r,i) = theta_{i-r,i}
 *        messages                             [R][B][H][W][L] float
 *        p                                    [K][R][B][H][W][L] uint8  (argmin over mu)
 *        q                                    [K][R][B][H][W]    uint8  (argmin over lambda)
 *        labels                               [B][H][W]      uint8
 *  - A node whose predecessor i-r is outside the grid is the first node of its scanline
 *    in direction r: its message is 0, its p and q entries are written as 0, its edge
 *    weight is never read and its edge-weight gradient is 0.
 *  - Ties in every argmin go to the lowest label.
 *  - Ownership: the caller owns every buffer, including the workspace; the library
 *    allocates no device memory and keeps no problem data between calls (the only state is
 *    the process-global settings of mrf_tune, mrf_set_sweep_events and the two report
 *    strings below).  Outputs are fully
 *    overwritten (gradients are assigned, not accumulated into what the caller passed).
 *  - Calls enqueue work on `hip_stream` (a hipStream_t, NULL = default stream) and return
 *    without synchronising.  Calls that share a workspace must be ordered by the caller.
 *  - Return value: MRF_OK (0) or a negative mrf_status.  Argument errors are detected
 *    before any GPU work is enqueued.  Nothing is printed and nothing aborts.
 *  - Inputs must be finite; NaN or infinity in unary, pairwise, edge_weight or grad_cost
 *    gives unspecified values (never out-of-bounds accesses: indices read from p and q
 *    are clamped to [0, L)).
 */
#ifndef MRFMP_H
#define MRFMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MRF_MAX_DIRECTIONS 16
#define MRF_MAX_LABELS 256

typedef enum {
    MRF_OK = 0,
    MRF_ERR_NULL_POINTER = -1,      /* a required pointer is NULL */
    MRF_ERR_BAD_SHAPE = -2,         /* B, H or W < 1, or a tensor would exceed 2^31-1 label vectors */
    MRF_ERR_BAD_LABELS = -3,        /* L outside [1, 256] (p, q are 8-bit, Sec. 4) */
    MRF_ERR_BAD_ITERATIONS = -4,    /* K < 1 */
    MRF_ERR_BAD_DIRECTIONS = -5,    /* R outside [1, 16], a zero step, or a repeated direction */
    MRF_ERR_WORKSPACE_TOO_SMALL = -6,
    MRF_ERR_BAD_PAIRWISE_KIND = -7, /* unknown pairwise_kind, trunc <= 0 for kinds 1-3, or scale < 0 for kinds 1, 2 */
    MRF_ERR_BAD_ALGORITHM = -8,     /* algo argument is neither MRF_ISGMR nor MRF_TRWP */
    MRF_ERR_HIP = -9,               /* a HIP runtime call or kernel launch failed */
    MRF_ERR_SCRATCH_LIMIT = -10,    /* the problem exceeds the fixed scratch of a no-allocation entry point */
    MRF_ERR_WAIT_EXPIRED = -11      /* reported by mrf_workspace_fault: a wait between wavefronts ran out */
} mrf_status;

enum { MRF_ISGMR = 0, MRF_TRWP = 1 };

/* pairwise_kind: a promise about the contents of `pairwise` that lets the forward pass
 * skip work; `pairwise` must still hold the full L x L table (it is what is read). */
enum {
    MRF_PAIRWISE_DENSE = 0,            /* no structure assumed */
    MRF_PAIRWISE_TRUNC_LINEAR = 1,     /* V(mu,lambda) = scale * min(|mu-lambda|, trunc)      */
    MRF_PAIRWISE_TRUNC_QUADRATIC = 2,  /* V(mu,lambda) = scale * min((mu-lambda)^2, trunc)    */
    MRF_PAIRWISE_DISTANCE = 3          /* V(mu,lambda) = f(|mu-lambda|), f(0) <= f(1) <= ..., constant for
                                          |mu-lambda| >= trunc: e.g. the three SGM penalties 0, P1, P2
                                          of Eq. vsgm with trunc = 2 (scale is not used)              */
};

/* The problem as the paper states it: energy parameters Theta = {theta_i, theta_ij} with
 * theta_{i-r,i}(mu,lambda) = theta_{i-r,i} V(mu,lambda) (Sec. 5.1), direction set R,
 * iteration count K, TRW coefficients rho (Eq. trwp). */
typedef struct {
    int32_t B, H, W, L;         /* batch, grid height, width, labels (1..256) */
    int32_t R;                  /* number of directions, 1..16 */
    const int32_t *dirs;        /* HOST  [R][2] steps (dh, dw); order = TRWP sweep order;
                                   r- is the entry (-dh,-dw) if present, else its term is absent */
    int32_t K;                  /* iterations >= 1 */
    const float *unary;         /* DEVICE [B][H][W][L]; forward only (may be NULL for backward) */
    const float *pairwise;      /* DEVICE [L][L] */
    const float *edge_weight;   /* DEVICE [R][B][H][W], or NULL => edge_weight_scalar on every edge */
    float edge_weight_scalar;
    const float *rho;           /* HOST  [R] rho_{i-r,i} per direction; TRWP only, ignored by ISGMR;
                                   may be NULL if rho_edge is given */
    int32_t pairwise_kind;      /* MRF_PAIRWISE_* */
    float trunc, scale;         /* parameters of kinds 1, 2 and 3 (trunc > 0) */
    const float *rho_edge;      /* DEVICE [R][B][H][W] or NULL: rho_{i-r,i} per directed edge as Eq. trwp
                                   writes it, entry (r,i) like edge_weight (first-node entries are never
                                   read); takes the place of rho[]; TRWP only.  Such problems run
                                   through the one-wavefront-per-scanline sweeps. */
    const float *pairwise_edge; /* DEVICE [R][B][H][W][L][L] or NULL: pairwise potentials given per edge,
                                   entry (r,i,mu,lambda) = theta_{i-r,i}(mu,lambda) as Eq. isgmr and Eq. trwp
                                   write them (tables of first nodes are never read).  Then pairwise (may be
                                   NULL), edge_weight and edge_weight_scalar are not used, L <= 64 and
                                   pairwise_kind = MRF_PAIRWISE_DENSE are required, and the backward entry
                                   points take grad_edge_weight = NULL and write to grad_pairwise, if given,
                                   the gradient of these tables, [R][B][H][W][L][L]
                                   (Eq. supp-gradient-pairwise; tables of first nodes get 0). */
    int32_t sgm_standard;       /* non-zero: standard single-pass SGM (Sec. 3.2, Eq. sgm_old and
                                   Eq. isgmr-aggregation-old) instead of the revised update: the message carries
                                   the node's own unary, m^r_i(lambda) = theta_i(lambda) + min_mu (m^r_{i-r}(mu) +
                                   theta_{i-r,i}(mu,lambda)), reparametrised by Eq. isgmr-norm (q is the argmin of
                                   this sum), the first node of a scanline holds its unary, and c_i = sum_r m^r_i.
                                   Forward only, through mrf_isgmr_forward with K = 1 (anything else, the backward
                                   entry points included, returns MRF_ERR_BAD_ALGORITHM); runs the dense sweep. */
} mrf_problem;

/* Bytes of DEVICE workspace (256-byte aligned base required) that the forward
 * (backward = 0) or backward (backward != 0) pass of `algo` needs for this problem;
 * 0 if the problem is invalid.  Pure host arithmetic.  The backward figure covers the
 * case that grad_pairwise is requested. */
size_t mrf_workspace_bytes(const mrf_problem *prob, int algo, int backward);

/* Checks a problem description the way the entry points do; no GPU work. */
int mrf_validate(const mrf_problem *prob, int algo);

/* Which forward kernel the sweeps of the second and later iterations get: 0 = the dense O(L^2)
 * sweep, w > 0 = the window sweep that evaluates 2w - 1 source labels per label (truncated models
 * whose truncation distance is at most 16 and below L; any direction set: with the default kernel-choice
 * rules an ISGMR sweep reads a single array from six directions on and at most seven message arrays
 * below that, a TRWP sweep up to fifteen).  Results are identical either way.  Negative mrf_status for
 * an invalid problem.  Host arithmetic. */
int mrf_forward_window(const mrf_problem *prob, int algo);

/* Forward propagation of ISGMR (Alg. 1; update Eq. isgmr, reparametrisation
 * Eq. isgmr-norm, final costs Eq. isgmr-aggregation, labelling Eq. disp).
 *   cost      DEVICE out, required
 *   labels    DEVICE out, may be NULL
 *   p, q      DEVICE out, required: the indices the backward pass replays (Sec. 4)
 *   messages  DEVICE out, may be NULL: final messages m of all directions */
int mrf_isgmr_forward(const mrf_problem *prob, float *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                      float *messages, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Forward propagation of TRWP (Alg. 2; update Eq. trwp).  Directions are swept one after
 * the other in the order of prob->dirs, messages are updated in place.  Same outputs. */
int mrf_trwp_forward(const mrf_problem *prob, float *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                     float *messages, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backpropagation of ISGMR (Alg. 3, Appendix A; gradients Eq. supp-gradient-unary,
 * supp-gradient-edge, supp-gradient-smoothness).
 *   grad_cost         DEVICE in,  dL/dc
 *   p, q              DEVICE in,  as written by mrf_isgmr_forward for the same problem
 *   grad_unary        DEVICE out, required
 *   grad_edge_weight  DEVICE out, may be NULL.  One value per directed edge; a caller that
 *                     stores theta_ij = theta_ji once adds the two directed entries itself.
 *   grad_pairwise     DEVICE out, may be NULL */
int mrf_isgmr_backward(const mrf_problem *prob, const float *grad_cost, const uint8_t *p, const uint8_t *q,
                       float *grad_unary, float *grad_edge_weight, float *grad_pairwise,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backpropagation of TRWP (Alg. 4, Appendix A).  Directions are swept in the reverse of
 * the forward order.  rho does not enter the pairwise gradients.  Same arguments. */
int mrf_trwp_backward(const mrf_problem *prob, const float *grad_cost, const uint8_t *p, const uint8_t *q,
                      float *grad_unary, float *grad_edge_weight, float *grad_pairwise,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* Scanline geometry used by the kernels ("tree parallelisation", Sec. 3.5 and Appendix C):
 * the scanlines of direction (dh,dw) are the maximal in-grid chains i, i+r, i+2r, ...
 * mrf_scanline_count returns how many there are in one H x W image (for |dh| = 1 this is
 * W + (H-1)|dw|, Eq. supp-wide); mrf_scanline_head gives the first node and the number of
 * nodes of scanline t in [0, count).  Host arithmetic, shared with the device code.
 * Returns MRF_OK or MRF_ERR_BAD_SHAPE / MRF_ERR_BAD_DIRECTIONS. */
int64_t mrf_scanline_count(int32_t H, int32_t W, int32_t dh, int32_t dw);
int mrf_scanline_head(int32_t H, int32_t W, int32_t dh, int32_t dw, int64_t t,
                      int32_t *y0, int32_t *x0, int32_t *len);

/* Energy of a labelling, Sec. 3.1 Eq. energy-function:
 *   energy[b] = sum_i theta_i(x_i) + sum over edges (i-r, i) of theta_{i-r,i} V(x_{i-r}, x_i)
 * for every batch image b.  The edge set holds every undirected neighbour pair once: the
 * edges of the first direction of each opposite pair in prob->dirs (and of every direction
 * without an opposite), with that direction's weights -- or, where prob->pairwise_edge is
 * given, with that direction's tables theta_{i-r,i}(x_{i-r}, x_i) (prob->pairwise may then be
 * NULL).  prob->K and prob->rho are not used.
 *   labels   DEVICE [B][H][W] uint8 (values >= L are read as L-1)
 *   energy   DEVICE [B] double, assigned
 *   workspace DEVICE, at least mrf_energy_workspace_bytes(prob), 256-byte aligned
 * Sums are formed in double in an order fixed by the launch shape.  Asynchronous on
 * hip_stream.  Returns MRF_OK or a negative MRF_ERR_* before any GPU work is issued. */
size_t mrf_energy_workspace_bytes(const mrf_problem *prob);
int mrf_energy(const mrf_problem *prob, const uint8_t *labels, double *energy, void *workspace,
               size_t workspace_bytes, void *hip_stream);

/* mrf_energy for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): same arguments and results without the
 * workspace.  The partial sums go to a device array inside the library (2 MiB per GPU the
 * library runs on, held until the process ends), which holds them for at most
 * MRF_ENERGY_NOALLOC_MAX_BATCH batch images: a larger prob->B returns MRF_ERR_SCRATCH_LIMIT
 * before any GPU work.  The call allocates nothing and frees nothing.  All calls on one GPU
 * share that array: calls that may overlap on one GPU (different streams, different threads)
 * race and must be ordered by the caller; calls on one stream are ordered by the stream. */
#define MRF_ENERGY_NOALLOC_MAX_BATCH 64
int mrf_energy_noalloc(const mrf_problem *prob, const uint8_t *labels, double *energy, void *hip_stream);

/* Loss head of the learning set-up (Appendix, Eqs. supp-isgmr-confidence,
 * supp-isgmr-regression, and the L1 loss named there): per pixel
 *   f(lambda) = exp(-c(lambda)) / sum_mu exp(-c(mu)),  d = sum_lambda lambda f(lambda),
 *   loss = (1/n) sum over counted pixels |d - target|,
 *   grad_cost(lambda) = d loss / d c(lambda) = sign(d - target)/n * (-f(lambda)) * (lambda - d)
 * (0 for pixels that do not count; sign(0) = 0), n = number of counted pixels.
 *   cost      DEVICE [n_pixels][L] float: the final costs c of a forward call
 *   target    DEVICE [n_pixels] float: real-valued ground-truth disparities
 *   mask      DEVICE [n_pixels] uint8 or NULL: non-zero = the pixel counts (NULL: all count)
 *   disparity DEVICE [n_pixels] float or NULL, assigned
 *   loss      DEVICE double, assigned
 *   grad_cost DEVICE [n_pixels][L] float or NULL, assigned: the grad_cost of mrf_*_backward
 *   workspace DEVICE, at least mrf_softmin_l1_workspace_bytes(), 256-byte aligned
 * Arithmetic in double, reproducible run to run.  Asynchronous on hip_stream. */
size_t mrf_softmin_l1_workspace_bytes(void);
int mrf_softmin_l1(int64_t n_pixels, int32_t L, const float *cost, const float *target, const uint8_t *mask,
                   float *disparity, double *loss, float *grad_cost, void *workspace, size_t workspace_bytes,
                   void *hip_stream);

/* The same head with the smooth L1 loss that Appendix D.1 names beside the standard one:
 *   per pixel l(x) = x^2 / (2 beta) for |x| < beta, |x| - beta / 2 otherwise, x = d - target
 * (the usual definition; the paper gives none), slope x / beta or sign(x) in grad_cost.
 * beta > 0 and finite, else MRF_ERR_BAD_PAIRWISE_KIND.  Same buffers and workspace as mrf_softmin_l1. */
int mrf_softmin_smooth_l1(int64_t n_pixels, int32_t L, const float *cost, const float *target, const uint8_t *mask,
                          float beta, float *disparity, double *loss, float *grad_cost, void *workspace,
                          size_t workspace_bytes, void *hip_stream);

/* Some sweep layouts spread a scanline over several wavefronts that hand nodes to each other
 * through rings in on-chip memory.  A wavefront that still finds itself waiting for another four
 * seconds after its workgroup started (sweeps take milliseconds) ends at once, those that wait for it
 * follow, and it raises a word in the first 256 bytes of the workspace, which every forward / backward call
 * clears when it starts.  This call waits for `hip_stream` to drain, reads that word and returns
 * MRF_OK, or MRF_ERR_WAIT_EXPIRED if the last call on this workspace was cut short (its outputs
 * are then incomplete; with correct kernels this never happens), or MRF_ERR_NULL_POINTER /
 * MRF_ERR_HIP.  Synchronous; workspace is the DEVICE pointer the call was given. */
int mrf_workspace_fault(const void *workspace, void *hip_stream);

/* Static text for a status code. */
const char *mrf_strerror(int status);

/* After a call returned MRF_ERR_HIP: which runtime call or launch failed and the runtime's
 * own text for the error ("" if none has failed yet).  Kept per calling thread; the
 * library owns the string. */
const char *mrf_last_error_detail(void);

/* Name of the kernel template that the most recent forward (backward = 0) or backward
 * (backward != 0) call launched for its last scanline sweep, "" before the first call: which
 * of the sweep layouts the launch-size rules picked.  For reports; kept per calling thread. */
const char *mrf_last_sweep_kernel(int backward);

/* The same launch in full: "name<template arguments> grid=G block=T", e.g.
 * "mrf_fwd_sweep_window<3,8,1,false,2> grid=9788 block=64" -- the instantiation a profiler
 * lists and the launch shape.  For reports and for tests that pin which instantiation a
 * benchmark shape gets; kept per calling thread, the library owns the string. */
const char *mrf_last_sweep_launch(int backward);

/* Profiling hook: while set (both non-NULL hipEvent_t handles), every forward or backward
 * call records `start_event` on its stream just before its first scanline-sweep launch and
 * `stop_event` just after its last one, so a caller can time the sweeps apart from the
 * surrounding element-wise kernels.  Pass NULL, NULL to clear.  Applies to the calls of the
 * thread that set it; the caller owns the events. */
int mrf_set_sweep_events(void *start_event, void *stop_event);

/* Tuning knobs for experiments; results never depend on them.  A setting applies to the calls of the
 * thread that made it (the library keeps these knobs, the hooks above and nothing else, per thread).
 *   knob 0: source labels per wavefront in the dense forward sweep (8, 12, 16, 24, 32, 48; 0 = heuristic)
 *   knob 1: non-zero = ignore pairwise_kind and always run the dense forward sweep
 *   knob 2: window sweep layout: 0 = by launch size, 1 = one wavefront per scanline,
 *           2 = one wavefront per 64 labels whenever L > 64
 *   knob 3: several scanlines per wavefront for L <= 32: 0 = by launch shape, 1 = never, 2 = always
 *   knob 4: window sweep with separate value and index wavefronts: 0 = by launch size, 1 = never,
 *           2 = whenever the window sweep applies (knob 2 = 2 takes precedence for L > 64)
 *   knob 5: index wavefronts per scanline in that sweep: 0 = by launch size, 1, 2
 *   knob 6: backward sweep with the node-to-node chain on its own wavefront: 0 = by launch size,
 *           1 = never, 2 = whenever it applies (grad_pairwise only for L <= 64)
 *   knob 7: helper wavefronts per scanline in that sweep: 0 = by launch size, 2, 4, 6, 8, 12
 *   knob 8: loader wavefront in front of the value wavefront (TRWP, window sweep, two index
 *           wavefronts): 0 = by launch size, 1 = never, 2 = whenever it applies
 *   knob 9: where knob 2 picks one wavefront per 64 labels, those wavefronts compute values only and
 *           index wavefronts of their own do the argmin tables and the stores: 0 = by launch size,
 *           1 = never, 2 = always
 *   knob 10: index wavefronts per scanline in that layout: 0 = default, 4, 8
 *   knob 11: two index wavefronts next to the value wavefront in the sweep of knob 3: 0 = by launch size,
 *           1 = never, 2 = always
 *   knob 12: in the sweep of knob 6, sum the lanes of the most popular scatter target in registers
 *           (truncated models): 0 = by launch shape, 1 = never, 2 = whenever V is not a dense table
 *   knob 13: three scanlines per wavefront (segments of 21 lanes) in the sweeps of knob 3 for 17..21 labels:
 *           0 = by launch size, 1 = never (two per wavefront), 2 = always
 *   knob 14: microseconds after the start of a workgroup beyond which a wavefront that still finds itself
 *           waiting for another gives up (see mrf_workspace_fault): 0 = default (4 s); 1 makes the
 *           multi-wavefront layouts give up almost at once (for tests of that path: every kernel still ends
 *           normally)
 *   knob 15: ISGMR backward with up to four directions, where the sweeps may read the other directions' scatter
 *           arrays themselves (one combine pass at the end) instead of a combine pass after every iteration:
 *           0 = for small problems (launch bound), 1 = never, 2 = always
 *   knob 16: dense forward sweep in which every wavefront owns 32 labels (loads, merge, normalisation and
 *           stores divided among the wavefronts) instead of doing that work for all labels (the layout knob 0
 *           tunes): 0 = for more than 96 labels, and for 65..96 labels where a sweep reads more than three message
 *           arrays or the launch has at least 4096 scanlines, 1 = never, 2 = for more than 64 labels
 *   knob 17: ISGMR forward in which one streaming pass per iteration sums the unary and the previous
 *           iteration's messages once per pair of opposite directions, so that every sweep reads one array
 *           instead of R - 1: 0 = from six directions on, 1 = never, 2 = always (more than one iteration)
 *   knob 18: backward sweep with grad_pairwise for 33..128 labels: the table accumulates in LDS, one per
 *           workgroup of eight wavefronts, instead of in a slot per wavefront in global memory: 0 = yes, 1 = no
 *   knob 19: grad_pairwise for 65..128 labels where the sweep of knob 6 runs one direction of up to 512 scanlines per launch (TRWP): its
 *           helpers store the gradient vector of every node and a streaming pass adds them into the table
 *           afterwards: 0 = yes, 1 = no (then another sweep accumulates the table itself)
 *   knob 20: backward sweep of knob 6 with two scanlines of up to 32 labels per workgroup (one direction per
 *           launch, TRWP): 0 = for 1,025 to 2,048 scanlines per launch, 1 = never, 2 = whenever it applies
 * Returns MRF_OK, or MRF_ERR_BAD_ALGORITHM for an unknown knob. */
int mrf_tune(int knob, int value);

/* Library version, e.g. "0.1.0". */
const char *mrf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MRFMP_H */
