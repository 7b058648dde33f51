// libmrfmp host side: argument checks, workspace layout and launch schedules of the
// ISGMR / TRWP forward and backward passes (Alg. 1-4).  Allocates nothing.
//
// One source, up to three translation units: compiled as it stands it holds everything; with
// -DMRF_PART=1 / 2 / 3 it holds the forward pass, the backward pass, or the entry points and
// the heads, so that the build can compile the three in parallel and link them.
#include "../../include/mrfmp.h"
#include "mrfmp_device.h"

#ifndef MRF_PART
#define MRF_PART 0
#endif
#define MRF_HAS_FWD (MRF_PART == 0 || MRF_PART == 1)
#define MRF_HAS_BWD (MRF_PART == 0 || MRF_PART == 2)
#define MRF_HAS_API (MRF_PART == 0 || MRF_PART == 3)

#if MRF_HAS_FWD
#include "mrfmp_fwd.h"
#endif
#if MRF_HAS_BWD
#include "mrfmp_bwd.h"
#endif
#if MRF_HAS_API
#include "mrfmp_head.h"
#endif

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

namespace mrf_host {

constexpr size_t kAlign = 256;
// wavefront-private V-gradient accumulators: many small ones (flushed from LDS once per
// wavefront) for few labels, fewer large ones (updated in place) otherwise
inline long long grad_slots(int L) { return L <= 32 ? 16384 : 1024; }

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

inline int check_problem(const mrf_problem *pr, int algo, bool forward)
{
    if (!pr) return MRF_ERR_NULL_POINTER;
    if (algo != MRF_ISGMR && algo != MRF_TRWP) return MRF_ERR_BAD_ALGORITHM;
    if (pr->B < 1 || pr->H < 1 || pr->W < 1) return MRF_ERR_BAD_SHAPE;
    if (pr->L < 1 || pr->L > MRF_MAX_LABELS) return MRF_ERR_BAD_LABELS;
    if (pr->K < 1) return MRF_ERR_BAD_ITERATIONS;
    // standard SGM is a single pass of the ISGMR sweeps without a backward pass of its own
    if (pr->sgm_standard && (algo != MRF_ISGMR || pr->K != 1 || pr->pairwise_edge)) return MRF_ERR_BAD_ALGORITHM;
    if (pr->R < 1 || pr->R > MRF_MAX_DIRECTIONS) return MRF_ERR_BAD_DIRECTIONS;
    if (!pr->dirs) return MRF_ERR_NULL_POINTER;
    for (int r = 0; r < pr->R; ++r) {
        const int dh = pr->dirs[2 * r], dw = pr->dirs[2 * r + 1];
        if (dh == 0 && dw == 0) return MRF_ERR_BAD_DIRECTIONS;
        for (int d = 0; d < r; ++d)
            if (pr->dirs[2 * d] == dh && pr->dirs[2 * d + 1] == dw) return MRF_ERR_BAD_DIRECTIONS;
    }
    const long long N = (long long)pr->B * pr->H * pr->W;
    if (N > 0x7fffffffLL) return MRF_ERR_BAD_SHAPE;
    if (!pr->pairwise && !pr->pairwise_edge) return MRF_ERR_NULL_POINTER;
    if (pr->pairwise_edge) {
        // one table per edge: few labels only, and no promise about V applies
        if (pr->L > 64) return MRF_ERR_BAD_LABELS;
        if (pr->pairwise_kind != MRF_PAIRWISE_DENSE) return MRF_ERR_BAD_PAIRWISE_KIND;
        if ((long long)pr->R * N * pr->L > 0x7fffffffLL) return MRF_ERR_BAD_SHAPE;
    }
    if (forward && !pr->unary) return MRF_ERR_NULL_POINTER;
    if (algo == MRF_TRWP && !pr->rho && !pr->rho_edge) return MRF_ERR_NULL_POINTER;
    if (pr->pairwise_kind != MRF_PAIRWISE_DENSE && pr->pairwise_kind != MRF_PAIRWISE_TRUNC_LINEAR &&
        pr->pairwise_kind != MRF_PAIRWISE_TRUNC_QUADRATIC && pr->pairwise_kind != MRF_PAIRWISE_DISTANCE)
        return MRF_ERR_BAD_PAIRWISE_KIND;
    if (pr->pairwise_kind != MRF_PAIRWISE_DENSE && !(pr->trunc > 0.0f)) return MRF_ERR_BAD_PAIRWISE_KIND;
    // the window sweeps need V non-decreasing in the label distance: a negative scale turns it round
    if ((pr->pairwise_kind == MRF_PAIRWISE_TRUNC_LINEAR || pr->pairwise_kind == MRF_PAIRWISE_TRUNC_QUADRATIC) &&
        !(pr->scale >= 0.0f)) return MRF_ERR_BAD_PAIRWISE_KIND;
    return MRF_OK;
}

inline void fill_geom(const mrf_problem *pr, MrfGeom &g)
{
    memset(&g, 0, sizeof(g));
    g.B = pr->B; g.H = pr->H; g.W = pr->W; g.L = pr->L; g.R = pr->R;
    g.N = (long long)pr->B * pr->H * pr->W;
    for (int r = 0; r < pr->R; ++r) {
        g.dh[r] = pr->dirs[2 * r];
        g.dw[r] = pr->dirs[2 * r + 1];
    }
    for (int r = 0; r < pr->R; ++r) {
        g.opp[r] = -1;
        for (int d = 0; d < pr->R; ++d)
            if (g.dh[d] == -g.dh[r] && g.dw[d] == -g.dw[r]) g.opp[r] = d;
        g.nscan[r] = (int)mrf_geom_scanlines(g.H, g.W, g.dh[r], g.dw[r]);
    }
}

inline size_t msg_bytes(const mrf_problem *pr)
{
    return align_up((size_t)pr->R * pr->B * pr->H * pr->W * pr->L * sizeof(float));
}

inline size_t gradv_bytes(const mrf_problem *pr)
{
    return align_up((size_t)grad_slots(pr->L) * pr->L * pr->L * sizeof(double));
}

// room for the node gradients that mrf_bwd_gv_from_g reads (65..128 labels)
inline size_t gstore_bytes(const mrf_problem *pr)
{
    if (pr->L <= 64 || pr->L > 128) return 0;
    return align_up((size_t)pr->B * pr->H * pr->W * pr->L * sizeof(double));
}

// ---- process-global state: defined in the translation unit of the entry points ----------
// tuning knobs (0 = heuristic)
#if MRF_HAS_API
#define MRF_G(decl, init) thread_local decl = init
#else
#define MRF_G(decl, init) extern thread_local decl
#endif
MRF_G(int g_tune_mch, 0);
MRF_G(int g_tune_no_window, 0);
MRF_G(int g_tune_split, 0);      // 0 auto, 1 never, 2 whenever L > 64
MRF_G(int g_tune_pack, 0);       // 0 auto, 1 never, 2 whenever L <= 32
MRF_G(int g_tune_duo, 0);        // 0 auto, 1 never, 2 whenever the window applies
MRF_G(int g_tune_duo_ni, 0);     // index wavefronts per scanline: 0 auto, 1, 2
MRF_G(int g_tune_loader, 0);     // loader wavefront in the window sweep: 0 auto, 1 never, 2 whenever possible
MRF_G(int g_tune_squad, 0);      // index wavefronts next to the split layout: 0 by launch size, 1 never, 2 always
MRF_G(int g_tune_squad_ni, 0);   // how many: 0 auto, 4, 8
MRF_G(int g_tune_pack3, 0);      // three scanlines per wavefront for 17..21 labels: 0 by launch size, 1 never, 2 always
MRF_G(int g_tune_isgmr_lazy, 0); // ISGMR backward without a combine pass per iteration (up to 4 directions): 0 auto, 1 never
MRF_G(int g_tune_isgmr_presum, 0); // ISGMR forward with the per-pair sums of the previous iteration formed once: 0 from six directions, 1 never, 2 always
MRF_G(int g_tune_chain_pk, 0);     // chain backward with two scanlines of up to 32 labels per workgroup: 0 = 1,025..2,048 scanlines of one direction, 1 never, 2 always
MRF_G(int g_tune_gv_apart, 0);     // V gradient of 65..128 labels by a streaming pass behind the chain backward sweep: 0 yes, 1 no
MRF_G(int g_tune_gv_tile, 0);      // V gradient of 33..128 labels in one LDS table per workgroup: 0 yes, 1 no (a slot per wavefront in global memory)
MRF_G(int g_tune_dense_sliced, 0); // dense sweep for more than 64 labels with a slice of the labels per wavefront: 0 yes, 1 no
MRF_G(int g_tune_spin_limit, 0); // turns a wait between wavefronts may take: 0 = default
MRF_G(int g_tune_pack_idx, 0);   // index wavefronts in the packed dense sweep: 0 by launch size, 1 never, 2 always
MRF_G(int g_tune_chain, 0);      // backward sweep with a chain wavefront: 0 auto, 1 never, 2 whenever possible
MRF_G(int g_tune_chain_hot, 0);  // its pre-reduction of the most popular scatter target: 0 auto, 1 never, 2 whenever V is no dense table
MRF_G(int g_tune_chain_ni, 0);   // its helpers per scanline: 0 auto, 2, 4, 6, 8
MRF_G(hipEvent_t g_ev_start, nullptr);
MRF_G(hipEvent_t g_ev_stop, nullptr);
#undef MRF_G
#if MRF_HAS_API
thread_local char g_error_detail[256] = "";
thread_local const char *g_last_sweep[2] = {"", ""};      // kernel of the last forward / backward sweep launch
thread_local char g_last_launch[2][160] = {"", ""};       // the same with template arguments and launch shape
#else
extern thread_local char g_error_detail[256];
extern thread_local const char *g_last_sweep[2];
extern thread_local char g_last_launch[2][160];
#endif

// records the kernel of a sweep launch: its name, and "name<template arguments> grid=.. block=.."
inline void note_launch(int backward, const char *name, long long grid, int block, const char *fmt, ...)
    __attribute__((format(printf, 5, 6)));
inline void note_launch(int backward, const char *name, long long grid, int block, const char *fmt, ...)
{
    g_last_sweep[backward] = name;
    char args[96];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(args, sizeof(args), fmt, ap);
    va_end(ap);
    snprintf(g_last_launch[backward], sizeof(g_last_launch[backward]), "%s<%s> grid=%lld block=%d", name, args, grid, block);
}

// Workspace header (the first 256 bytes): float [0] = the scalar edge weight, int at byte 128 = the
// fault word that a wait between wavefronts raises when it runs out (mrf_wait_again).
constexpr size_t kFaultOffset = 128;
// how long after its start a workgroup may still find one of its wavefronts waiting for another, in microseconds
// (sweeps take milliseconds)
constexpr int kSpinLimit = 4000000;
inline int spin_limit() { return g_tune_spin_limit > 0 ? g_tune_spin_limit : kSpinLimit; }
hipError_t init_header(void *workspace, float w_scalar, hipStream_t st);

// records which call failed and how, for mrf_last_error_detail
inline int hip_fail(hipError_t e, const char *what)
{
    snprintf(g_error_detail, sizeof(g_error_detail), "%s: %s", what, hipGetErrorString(e));
    return MRF_ERR_HIP;
}

inline void mark(hipEvent_t ev, hipStream_t st)
{
    if (g_ev_start && g_ev_stop) (void)hipEventRecord(ev, st);
}

// truncation distance that the forward pass rounds up to one of its window kernels, or 0
inline int window_width(const mrf_problem *pr)
{
    if (g_tune_no_window || pr->pairwise_kind == MRF_PAIRWISE_DENSE) return 0;
    double t = pr->trunc;
    if (pr->pairwise_kind == MRF_PAIRWISE_TRUNC_QUADRATIC) t = sqrt(t);
    if (!(t > 0.0) || t > 16.0) return 0;
    int ti = (int)ceil(t);
    if (ti < 1) ti = 1;
    if (ti >= pr->L) return 0;
    return ti <= 2 ? 2 : (ti <= 4 ? 4 : (ti <= 8 ? 8 : (ti <= 12 ? 12 : 16)));
}

// the three parts
hipError_t fill(float *dst, long long n, float v, hipStream_t st);
int run_forward(const mrf_problem *pr, int algo, float *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                float *messages, void *workspace, size_t workspace_bytes, void *hip_stream);
int run_backward(const mrf_problem *pr, int algo, const float *grad_cost, const uint8_t *p, const uint8_t *q,
                 float *grad_unary, float *grad_w, float *grad_V, void *workspace, size_t workspace_bytes,
                 void *hip_stream);

#if MRF_HAS_FWD
template <int LP, int MCH, int RMAX, int D>
hipError_t launch_fwd(const MrfFwdParams &P, int algo, long long blocks, hipStream_t st)
{
    note_launch(0, "mrf_fwd_sweep", blocks, 64 * P.NW, "%d,%d,%d,%d,%s", LP, MCH, RMAX, D, algo == MRF_TRWP ? "true" : "false");
    constexpr int NWMAX = (64 * LP + MCH - 1) / MCH;
    const size_t lds = (size_t)NWMAX * NWMAX * MCH * sizeof(float) +
                       (NWMAX > 1 ? (size_t)2 * NWMAX * 64 * LP * sizeof(float2) : 0);
    if (algo == MRF_TRWP)
        hipLaunchKernelGGL((mrf_fwd_sweep<LP, MCH, RMAX, D, true>), dim3((unsigned)blocks), dim3(64 * P.NW), lds, st, P);
    else
        hipLaunchKernelGGL((mrf_fwd_sweep<LP, MCH, RMAX, D, false>), dim3((unsigned)blocks), dim3(64 * P.NW), lds, st, P);
    return hipGetLastError();
}

template <int LP, int RMAX, int D>
hipError_t launch_fwd_sliced(const MrfFwdParams &P, int algo, long long blocks, hipStream_t st)
{
    note_launch(0, "mrf_fwd_sweep_sliced", blocks, 64 * P.NW, "%d,%d,%d,%s", LP, RMAX, D, algo == MRF_TRWP ? "true" : "false");
    if (algo == MRF_TRWP)
        hipLaunchKernelGGL((mrf_fwd_sweep_sliced<LP, RMAX, D, true>), dim3((unsigned)blocks), dim3(64 * P.NW), 0, st, P);
    else
        hipLaunchKernelGGL((mrf_fwd_sweep_sliced<LP, RMAX, D, false>), dim3((unsigned)blocks), dim3(64 * P.NW), 0, st, P);
    return hipGetLastError();
}

// source labels per wavefront: small enough that the slice of V fits in registers, large
// enough that at most 16 wavefronts share a node
// (33..64 labels: four wavefronts of 16 source labels while the launch leaves SIMD slots free, two of 32 from
// 2,048 scanlines on: 512 x 512, 64 labels, ISGMR 2.64 -> 2.02 ms; TRWP on 4 x 512 x 512 11.4 -> 8.2 ms, but on
// 1 x 512 x 512 4.5 against 5.2 ms)
int pick_mch(int L, int LP, bool many_sources, long long blocks)
{
    static const int allowed[4][5] = { {8, 16, 32, 0, 0}, {8, 12, 16, 24, 32}, {16, 24, 32, 48, 0}, {32, 0, 0, 0, 0} };
    int want = g_tune_mch;
    if (want <= 0) want = LP == 1 ? ((L <= 32 || blocks >= 2048) ? 32 : 16) : (LP == 2 ? 24 : 32);
    if (many_sources) want = (LP <= 2) ? (want < 16 ? 16 : (want == 24 || want == 12 ? 16 : want)) : 32;
    int best = 0;
    for (int i = 0; i < 5; ++i) {
        const int m = allowed[LP - 1][i];
        if (m == 0) continue;
        if (many_sources && m != 16 && m != 32) continue;
        if (best == 0 || mrf_iabs(m - want) < mrf_iabs(best - want)) best = m;
    }
    return best;
}

// pairwise potentials per edge (L <= 64): the table is fetched in two halves of ceil(L/2) rows
// (rounded up to a multiple of four)
hipError_t launch_edge(const MrfFwdParams &P, int algo, long long blocks, hipStream_t st)
{
    int ms = 0;
    for (int r = P.r_first; r < P.r_first + P.r_count; ++r)
        if (P.n_src[r] > ms) ms = P.n_src[r];
    const int rmax = (ms + 1 <= 4) ? 4 : ((ms + 1 <= 8) ? 8 : 16);
    const int L = P.g.L;
    note_launch(0, "mrf_fwd_sweep_edge", blocks, 64, "%d,%d,%s", (L + 7) / 8 * 4, rmax, algo == MRF_TRWP ? "true" : "false");
    if (L > 64) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(64);
#define MRF_E(half, rm) \
    if (L <= 2 * half && rmax == rm) { \
        if (algo == MRF_TRWP) hipLaunchKernelGGL((mrf_fwd_sweep_edge<half, rm, true>), grid, block, 0, st, P); \
        else hipLaunchKernelGGL((mrf_fwd_sweep_edge<half, rm, false>), grid, block, 0, st, P); \
        return hipGetLastError(); \
    }
#define MRF_EH(half) MRF_E(half, 4) MRF_E(half, 8) MRF_E(half, 16)
    MRF_EH(4) MRF_EH(8) MRF_EH(12) MRF_EH(16) MRF_EH(20) MRF_EH(24) MRF_EH(28) MRF_EH(32)
#undef MRF_EH
#undef MRF_E
    return hipErrorInvalidValue;
}

template <int LP, int RMAX, int D>
hipError_t launch_window(const MrfFwdParams &P, int algo, int tw, long long blocks, hipStream_t st)
{
    note_launch(0, "mrf_fwd_sweep_window", blocks, 64, "%d,%d,%d,%s,%d", LP, RMAX, D, algo == MRF_TRWP ? "true" : "false", tw);
#define MRF_W(twv) \
    if (tw == twv) { \
        if (algo == MRF_TRWP) hipLaunchKernelGGL((mrf_fwd_sweep_window<LP, RMAX, D, true, twv>), dim3((unsigned)blocks), dim3(64), 0, st, P); \
        else hipLaunchKernelGGL((mrf_fwd_sweep_window<LP, RMAX, D, false, twv>), dim3((unsigned)blocks), dim3(64), 0, st, P); \
        return hipGetLastError(); \
    }
    MRF_W(2) MRF_W(4) MRF_W(8) MRF_W(12) MRF_W(16)
#undef MRF_W
    return hipErrorInvalidValue;
}

// ISGMR sweeps that read one array only
template <int LP>
hipError_t launch_window_one(const MrfFwdParams &P, int tw, long long blocks, hipStream_t st)
{
    note_launch(0, "mrf_fwd_sweep_window", blocks, 64, "%d,1,4,false,%d", LP, tw);
#define MRF_W(twv) \
    if (tw == twv) { \
        hipLaunchKernelGGL((mrf_fwd_sweep_window<LP, 1, 4, false, twv>), dim3((unsigned)blocks), dim3(64), 0, st, P); \
        return hipGetLastError(); \
    }
    MRF_W(2) MRF_W(4) MRF_W(8) MRF_W(12) MRF_W(16)
#undef MRF_W
    return hipErrorInvalidValue;
}

// TRWP with nine to sixteen directions: up to fifteen message arrays per update
template <int LP>
hipError_t launch_window_many(const MrfFwdParams &P, int tw, long long blocks, hipStream_t st)
{
    // (prefetch two nodes deep where the registers allow: a node step otherwise waits a whole memory round trip)
    constexpr int D = LP <= 2 ? 2 : 1;
    note_launch(0, "mrf_fwd_sweep_window", blocks, 64, "%d,16,%d,true,%d", LP, D, tw);
#define MRF_W(twv) \
    if (tw == twv) { \
        hipLaunchKernelGGL((mrf_fwd_sweep_window<LP, 16, D, true, twv>), dim3((unsigned)blocks), dim3(64), 0, st, P); \
        return hipGetLastError(); \
    }
    MRF_W(2) MRF_W(4) MRF_W(8) MRF_W(12) MRF_W(16)
#undef MRF_W
    return hipErrorInvalidValue;
}

template <int LP, int RMAX, int D, int NI>
hipError_t launch_window_duo(const MrfFwdParams &P, int algo, int tw, long long blocks, hipStream_t st)
{
    note_launch(0, "mrf_fwd_sweep_window_duo", blocks, 64 * (1 + NI), "%d,%d,%d,%s,%d,%d,false", LP, RMAX, D,
                algo == MRF_TRWP ? "true" : "false", tw, NI);
#define MRF_W(twv) \
    if (tw == twv) { \
        if (algo == MRF_TRWP) hipLaunchKernelGGL((mrf_fwd_sweep_window_duo<LP, RMAX, D, true, twv, NI, false>), dim3((unsigned)blocks), dim3(64 * (1 + NI)), 0, st, P); \
        else hipLaunchKernelGGL((mrf_fwd_sweep_window_duo<LP, RMAX, D, false, twv, NI, false>), dim3((unsigned)blocks), dim3(64 * (1 + NI)), 0, st, P); \
        return hipGetLastError(); \
    }
    MRF_W(2) MRF_W(4) MRF_W(8) MRF_W(12) MRF_W(16)
#undef MRF_W
    return hipErrorInvalidValue;
}

// value + loader + two index wavefronts (TRWP, up to three other directions)
template <int LP>
hipError_t launch_window_loader(const MrfFwdParams &P, int tw, long long blocks, hipStream_t st)
{
    note_launch(0, "mrf_fwd_sweep_window_duo", blocks, 256, "%d,4,%d,true,%d,2,true", LP, (LP <= 2 ? 4 : 2), tw);
#define MRF_W(twv) \
    if (tw == twv) { \
        hipLaunchKernelGGL((mrf_fwd_sweep_window_duo<LP, 4, (LP <= 2 ? 4 : 2), true, twv, 2, true>), dim3((unsigned)blocks), dim3(256), 0, st, P); \
        return hipGetLastError(); \
    }
    MRF_W(2) MRF_W(4) MRF_W(8) MRF_W(12) MRF_W(16)
#undef MRF_W
    return hipErrorInvalidValue;
}

template <int RMAX, int D>
hipError_t launch_window_split(const MrfFwdParams &P, int algo, int tw, long long blocks, hipStream_t st)
{
    const unsigned threads = 64u * (unsigned)((P.g.L + 63) / 64);
    note_launch(0, "mrf_fwd_sweep_window_split", blocks, (int)threads, "%d,%d,%s,%d", RMAX, D, algo == MRF_TRWP ? "true" : "false", tw);
#define MRF_W(twv) \
    if (tw == twv) { \
        if (algo == MRF_TRWP) hipLaunchKernelGGL((mrf_fwd_sweep_window_split<RMAX, D, true, twv>), dim3((unsigned)blocks), dim3(threads), 0, st, P); \
        else hipLaunchKernelGGL((mrf_fwd_sweep_window_split<RMAX, D, false, twv>), dim3((unsigned)blocks), dim3(threads), 0, st, P); \
        return hipGetLastError(); \
    }
    MRF_W(2) MRF_W(8) MRF_W(16)
#undef MRF_W
    return hipErrorInvalidValue;
}

template <int RMAX, int D>
hipError_t launch_window_squad(const MrfFwdParams &P, int algo, int tw, int ni, long long blocks, hipStream_t st)
{
    const unsigned nwv = (unsigned)((P.g.L + 63) / 64);
    note_launch(0, "mrf_fwd_sweep_window_squad", blocks, (int)(64u * (nwv + ni)), "%d,%d,%s,%d,%d", RMAX, D,
                algo == MRF_TRWP ? "true" : "false", tw, ni);
#define MRF_W(twv, niv) \
    if (tw == twv && ni == niv) { \
        if (algo == MRF_TRWP) hipLaunchKernelGGL((mrf_fwd_sweep_window_squad<RMAX, D, true, twv, niv>), dim3((unsigned)blocks), dim3(64u * (nwv + niv)), 0, st, P); \
        else hipLaunchKernelGGL((mrf_fwd_sweep_window_squad<RMAX, D, false, twv, niv>), dim3((unsigned)blocks), dim3(64u * (nwv + niv)), 0, st, P); \
        return hipGetLastError(); \
    }
    MRF_W(2, 4) MRF_W(8, 4) MRF_W(16, 4) MRF_W(2, 8) MRF_W(8, 8) MRF_W(16, 8)
#undef MRF_W
    return hipErrorInvalidValue;
}

// Distance from which a truncated pairwise function is constant, or 0 if the window
// kernel does not apply (dense kind, no truncation inside the label range, wide window).

template <int SEG, int MU>
hipError_t launch_packed_mu(const MrfFwdParams &P, int algo, int rmax, long long scanlines, hipStream_t st)
{
    const unsigned blocks = (unsigned)((scanlines + 64 / SEG - 1) / (64 / SEG));
    // few wavefronts in the launch: further ones per workgroup for the argmin tables and the stores
    // (two of them: an index wavefront has more to do per node than the value wavefront)
    const bool idx = g_tune_pack_idx != 1 && (g_tune_pack_idx == 2 || blocks <= 1024);
    note_launch(0, "mrf_fwd_sweep_packed", blocks, idx ? 192 : 64, "%d,%d,%d,%d,%s,%d", SEG, MU, rmax, rmax == 4 ? 4 : (rmax == 8 ? 2 : 1),
                algo == MRF_TRWP ? "true" : "false", idx ? 2 : 0);
#define MRF_P(rm, d) \
    if (rmax == rm) { \
        if (idx) { \
            if (algo == MRF_TRWP) hipLaunchKernelGGL((mrf_fwd_sweep_packed<SEG, MU, rm, d, true, 2>), dim3(blocks), dim3(192), 0, st, P); \
            else hipLaunchKernelGGL((mrf_fwd_sweep_packed<SEG, MU, rm, d, false, 2>), dim3(blocks), dim3(192), 0, st, P); \
        } else { \
            if (algo == MRF_TRWP) hipLaunchKernelGGL((mrf_fwd_sweep_packed<SEG, MU, rm, d, true, 0>), dim3(blocks), dim3(64), 0, st, P); \
            else hipLaunchKernelGGL((mrf_fwd_sweep_packed<SEG, MU, rm, d, false, 0>), dim3(blocks), dim3(64), 0, st, P); \
        } \
        return hipGetLastError(); \
    }
    MRF_P(4, 4) MRF_P(8, 2) MRF_P(16, 1)
#undef MRF_P
    return hipErrorInvalidValue;
}

template <int SEG>
hipError_t launch_packed(const MrfFwdParams &P, int algo, int rmax, long long scanlines, hipStream_t st)
{
    // three scanlines of up to 21 labels per wavefront: always 24 source labels
    if constexpr (SEG == 21) {
        return launch_packed_mu<21, 24>(P, algo, rmax, scanlines, st);
    } else {
        // source labels per node: L rounded up to a multiple of four
        const int mu = (P.g.L + 3) / 4 * 4;
        if (mu <= SEG - 12) return launch_packed_mu<SEG, SEG - 12>(P, algo, rmax, scanlines, st);
        if (mu <= SEG - 8) return launch_packed_mu<SEG, SEG - 8>(P, algo, rmax, scanlines, st);
        if (mu <= SEG - 4) return launch_packed_mu<SEG, SEG - 4>(P, algo, rmax, scanlines, st);
        return launch_packed_mu<SEG, SEG>(P, algo, rmax, scanlines, st);
    }
}

hipError_t dispatch_fwd(MrfFwdParams &P, int algo, int tw, long long blocks, hipStream_t st)
{
    // few labels: several scanlines per wavefront (dense evaluation), unless the launch is so
    // small that it is latency bound and a truncated model can use the shorter window step
    // (up to 16 labels the window templates evaluate 15 candidates, no fewer than the dense step)
    if (P.Te) return launch_edge(P, algo, blocks, st);
    // (TRW coefficients per edge: the two one-wavefront-per-scanline sweeps read them)
    const bool generic = P.rho_e != nullptr;
    if (P.sgm_std) tw = 0;         // standard SGM: the dense sweep is the one that knows it
    if (!P.sgm_std && !generic && P.g.L <= 32 && g_tune_pack != 1 && (g_tune_pack == 2 || tw == 0 || blocks >= 1024 || P.g.L <= 16)) {
        int ms = 0;
        for (int r = P.r_first; r < P.r_first + P.r_count; ++r)
            if (P.n_src[r] > ms) ms = P.n_src[r];
        const int rmax = (ms + 1 <= 4) ? 4 : ((ms + 1 <= 8) ? 8 : 16);
        P.NW = 1;
        // 17..21 labels (the 21 classes of the segmentation shape): three scanlines per wavefront once the
        // launch has wavefronts to spare, else two (a latency-bound launch gains nothing from fewer wavefronts)
        if (P.g.L > 16 && P.g.L <= 21 && g_tune_pack3 != 1 && (g_tune_pack3 == 2 || blocks >= 3072))
            return launch_packed<21>(P, algo, rmax, blocks, st);
        return P.g.L <= 16 ? launch_packed<16>(P, algo, rmax, blocks, st) : launch_packed<32>(P, algo, rmax, blocks, st);
    }
    if (tw > 0) {
        const int LPw = (P.g.L + 63) / 64;
        int ms = 0;
        for (int r = P.r_first; r < P.r_first + P.r_count; ++r)
            if (P.n_src[r] > ms) ms = P.n_src[r];
        // few scanlines in the launch and many labels: spread each node step over one
        // wavefront per 64 labels
        // (wide windows over many labels only: otherwise the value/index pair below is faster)
        // (measured with four directions: window 16, 192 or 256 labels, ISGMR with 1,536 to 3,072 scanlines: 2.2
        // against 3.8 ms, 2.6 against 5.4 ms, 5.0 against 7.2 ms, 7.3 against 8.2 ms for the next best layout; window
        // 8, 192 or 256 labels: the value/index pair is ahead, TRWP 2.3 against 3.9 ms, ISGMR 1.3 against 1.6 ms)
        const int tws = tw == 4 ? 8 : (tw == 12 ? 16 : tw);      // (these two layouts exist for windows 2, 8 and 16: a wider window is as exact)
        const bool split = !generic && LPw > 1 && g_tune_split != 1 &&
                           (g_tune_split == 2 || (LPw >= 3 && tws >= 16 && blocks * LPw <= 16384));
        if (ms + 1 <= 8 && split && g_tune_squad != 1 && (g_tune_squad == 2 || blocks <= 512)) {
            // the value wavefronts of the split layout, with the index work on wavefronts of their own
            P.NW = LPw;
            const int ni = (g_tune_squad_ni == 4 || g_tune_squad_ni == 8) ? g_tune_squad_ni : 8;
            if (ms + 1 <= 4) return launch_window_squad<4, 4>(P, algo, tws, ni, blocks, st);
            return launch_window_squad<8, 2>(P, algo, tws, ni, blocks, st);
        }
        if (ms + 1 <= 8 && split) {
            P.NW = LPw;
            if (ms + 1 <= 4) return launch_window_split<4, 4>(P, algo, tws, blocks, st);
            return launch_window_split<8, 2>(P, algo, tws, blocks, st);
        }
        // few scanlines: a second wavefront per scanline takes the argmin tables and the
        // stores off the dependency chain
        // (its addressing wants a node step times L in 32 bits)
        bool step_fits = true;
        for (int r = P.r_first; r < P.r_first + P.r_count; ++r) {
            const long long st = ((long long)mrf_iabs(P.g.dh[r]) * P.g.W + mrf_iabs(P.g.dw[r])) * P.g.L;
            if (st > 0x7fffffffLL) step_fits = false;
        }
        // (a second wavefront per scanline pays while the scanlines alone leave SIMD slots free; measured on
        // square grids with four directions: ISGMR at 2,048 scanlines 1.41 ms with it against 1.52 ms without,
        // at 2,560 scanlines 2.74 against 2.21 ms with 96 labels but 1.27 against 1.37 ms with 40; TRWP at 2,048
        // scanlines 4.92 against 4.32 ms)
        const long long duo_max = algo == MRF_TRWP ? 1536 : (LPw == 1 ? 3072 : 2048);
        const bool duo = !generic && step_fits && g_tune_duo != 1 && (g_tune_duo == 2 || blocks <= duo_max);
        if (ms + 1 <= 8 && duo) {
            P.NW = 1;
            // two index wavefronts while the launch is far from filling the machine
            const int ni = g_tune_duo_ni ? g_tune_duo_ni : (blocks <= 1536 ? 2 : 1);
            // TRWP launches that leave SIMDs idle: a loader wavefront in front of the value wavefront
            if (algo == MRF_TRWP && ms + 1 <= 4 && ni == 2 && g_tune_loader != 1 &&
                (g_tune_loader == 2 || blocks <= 512)) {
                if (LPw == 1) return launch_window_loader<1>(P, tw, blocks, st);
                if (LPw == 2) return launch_window_loader<2>(P, tw, blocks, st);
                if (LPw == 3) return launch_window_loader<3>(P, tw, blocks, st);
                if (LPw == 4) return launch_window_loader<4>(P, tw, blocks, st);
            }
#define MRF_WCASE(lp) \
            if (LPw == lp && ms + 1 <= 4 && ni == 2) return launch_window_duo<lp, 4, (lp <= 2 ? 4 : 2), 2>(P, algo, tw, blocks, st); \
            if (LPw == lp && ms + 1 <= 4) return launch_window_duo<lp, 4, (lp <= 2 ? 4 : 2), 1>(P, algo, tw, blocks, st); \
            if (LPw == lp && ni == 2) return launch_window_duo<lp, 8, (lp <= 2 ? 2 : 1), 2>(P, algo, tw, blocks, st); \
            if (LPw == lp) return launch_window_duo<lp, 8, (lp <= 2 ? 2 : 1), 1>(P, algo, tw, blocks, st);
            MRF_WCASE(1) MRF_WCASE(2) MRF_WCASE(3) MRF_WCASE(4)
#undef MRF_WCASE
        }
        if (ms + 1 <= 8) {
            P.NW = 1;
            // (nothing but the start term to read: the first iteration of ISGMR, and its later ones after
            // mrf_isgmr_presum; a deeper prefetch fits in the registers the other sources would take)
#define MRF_WCASE(lp) \
            if (LPw == lp && ms == 0 && algo == MRF_ISGMR) return launch_window_one<lp>(P, tw, blocks, st);
            MRF_WCASE(1) MRF_WCASE(2) MRF_WCASE(3) MRF_WCASE(4)
#undef MRF_WCASE
#define MRF_WCASE(lp) \
            if (LPw == lp && ms + 1 <= 4) return launch_window<lp, 4, (lp <= 2 ? 4 : 2)>(P, algo, tw, blocks, st); \
            if (LPw == lp) return launch_window<lp, 8, (lp <= 2 ? 2 : 1)>(P, algo, tw, blocks, st);
            MRF_WCASE(1) MRF_WCASE(2) MRF_WCASE(3) MRF_WCASE(4)
#undef MRF_WCASE
        }
        if (algo == MRF_TRWP && ms + 1 <= 16) {
            P.NW = 1;
            if (LPw == 1) return launch_window_many<1>(P, tw, blocks, st);
            if (LPw == 2) return launch_window_many<2>(P, tw, blocks, st);
            if (LPw == 3) return launch_window_many<3>(P, tw, blocks, st);
            if (LPw == 4) return launch_window_many<4>(P, tw, blocks, st);
        }
    }
    const int L = P.g.L;
    const int LP = (L + 63) / 64;
    int max_src = 0;
    for (int r = P.r_first; r < P.r_first + P.r_count; ++r)
        if (P.n_src[r] > max_src) max_src = P.n_src[r];
    const int rmax = (max_src + 1 <= 4) ? 4 : ((max_src + 1 <= 8) ? 8 : 16);
    // more than 64 labels: every wavefront owns 32 of them (unless a tuning knob or a per-edge variant asks
    // for the sweep in which every wavefront does the O(L) work of the whole node)
    // (for 65..128 labels where the work outside the candidates is large: many source arrays, or a launch that
    // fills the machine several times over; else three wavefronts of 32 source labels are no faster than four
    // of 24: measured at 96 labels, 256 x 512, per iteration: TRWP with 8 directions 5.70 -> 4.01 ms, with 16
    // 15.1 -> 8.8 ms, ISGMR with 16 directions 4.12 -> 3.74 ms, but TRWP with 4 directions 1.81 -> 1.96 ms)
    // (from 97 labels on the other sweep needs five or six wavefronts of 24 source labels: 256 x 256, 128 labels,
    // ISGMR 3.80 -> 2.03 ms, TRWP 4.1 -> 3.8 ms; at 72 and 80 labels the two are level for ISGMR and this one is
    // behind for TRWP)
    if ((LP >= 3 || (LP == 2 && (g_tune_dense_sliced == 2 || rmax >= 8 || blocks >= 4096 || L > 96))) && !generic && !P.sgm_std && g_tune_mch == 0 && g_tune_dense_sliced != 1) {
        P.NW = (L + 31) / 32;
#define MRF_SCASE(lp) \
        if (LP == lp && rmax == 4) return launch_fwd_sliced<lp, 4, 4>(P, algo, blocks, st); \
        if (LP == lp && rmax == 8) return launch_fwd_sliced<lp, 8, 2>(P, algo, blocks, st); \
        if (LP == lp && rmax == 16) return launch_fwd_sliced<lp, 16, 1>(P, algo, blocks, st);
        MRF_SCASE(2) MRF_SCASE(3) MRF_SCASE(4)
#undef MRF_SCASE
    }
    const int mch = pick_mch(L, LP, rmax > 4, blocks);
    P.NW = (L + mch - 1) / mch;
    // prefetch depth: as deep as the register file allows next to the slice of V
#define MRF_CASE(lp, m) \
    if (LP == lp && mch == m && rmax == 4) return launch_fwd<lp, m, 4, (lp <= 2 ? 4 : 2)>(P, algo, blocks, st);
#define MRF_CASE_MANY(lp, m) \
    if (LP == lp && mch == m && rmax == 8) return launch_fwd<lp, m, 8, (lp <= 2 ? 2 : 1)>(P, algo, blocks, st); \
    if (LP == lp && mch == m && rmax == 16) return launch_fwd<lp, m, 16, 1>(P, algo, blocks, st);
    MRF_CASE(1, 8) MRF_CASE(1, 16) MRF_CASE(1, 32)
    MRF_CASE(2, 8) MRF_CASE(2, 12) MRF_CASE(2, 16) MRF_CASE(2, 24) MRF_CASE(2, 32)
    MRF_CASE(3, 16) MRF_CASE(3, 24) MRF_CASE(3, 32) MRF_CASE(3, 48)
    MRF_CASE(4, 32)
    MRF_CASE_MANY(1, 16) MRF_CASE_MANY(1, 32) MRF_CASE_MANY(2, 16) MRF_CASE_MANY(2, 32)
    MRF_CASE_MANY(3, 32) MRF_CASE_MANY(4, 32)
#undef MRF_CASE
#undef MRF_CASE_MANY
    return hipErrorInvalidValue;
}

// Which message arrays enter h at the previous node, in the order they are summed, for the
// sweep of direction r.  live: bit d set if array d holds data (else it is all zero and is
// skipped: adding 0 changes nothing).
void fill_sources(MrfFwdParams &P, int algo, int r, unsigned live)
{
    const int R = P.g.R, rm = P.g.opp[r];
    int n = 0, npre = 0, rmslot = -1;
    for (int d = 0; d < R; ++d) {
        if (d == r || !((live >> d) & 1u)) continue;
        if (algo == MRF_ISGMR && d == rm) continue;       // Eq. isgmr excludes r and r-
        if (algo == MRF_TRWP && d < r) ++npre;            // Eq. trwp sums all d in index order
        if (d == rm) rmslot = n;
        P.src_dir[r][n++] = (signed char)d;
    }
    P.n_pre[r] = (signed char)npre;
    P.n_src[r] = (signed char)n;
    P.rm_slot[r] = (signed char)rmslot;
}

hipError_t fill(float *dst, long long n, float v, hipStream_t st);

int run_forward(const mrf_problem *pr, int algo, float *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                float *messages, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_problem(pr, algo, true);
    if (rc != MRF_OK) return rc;
    if (!cost || !p || !q) return MRF_ERR_NULL_POINTER;
    const size_t need = mrf_workspace_bytes(pr, algo, 0);
    if (need > 0 && (!workspace || workspace_bytes < need)) return workspace ? MRF_ERR_WORKSPACE_TOO_SMALL : MRF_ERR_NULL_POINTER;
    hipStream_t st = (hipStream_t)hip_stream;

    MrfFwdParams P;
    memset(&P, 0, sizeof(P));
    fill_geom(pr, P.g);
    const long long N = P.g.N;
    const int R = pr->R, L = pr->L, K = pr->K;
    P.unary = pr->unary; P.V = pr->pairwise;
    for (int r = 0; r < R; ++r) P.rho[r] = (algo == MRF_TRWP && pr->rho) ? pr->rho[r] : 1.0f;
    P.rho_e = (algo == MRF_TRWP) ? pr->rho_edge : nullptr;
    P.Te = pr->pairwise_edge;
    P.sgm_std = pr->sgm_standard ? 1 : 0;

    // workspace: [scalars 256 B][messages A][messages B (ISGMR only)]
    float *scal = (float *)workspace;
    float *bufA = (float *)((char *)workspace + kAlign);
    float *bufB = (float *)((char *)workspace + kAlign + msg_bytes(pr));
    // header: the scalar weight (read through the same vector loads as per-edge weights) and the fault word
    { const hipError_t e_ = init_header(workspace, pr->edge_weight_scalar, st); if (e_ != hipSuccess) return hip_fail(e_, "init_header"); }
    P.fault = (int *)((char *)workspace + kFaultOffset);
    P.spin_limit = spin_limit();
    if (pr->edge_weight) { P.w = pr->edge_weight; P.w_mul = 1; }
    else { P.w = scal; P.w_mul = 0; }
    const size_t pk = (size_t)R * N * L, qk = (size_t)R * N;
    float *final_m = nullptr;
    const int tw = window_width(pr);

    mark(g_ev_start, st);
    if (algo == MRF_ISGMR) {
        // all directions of one iteration in one launch; messages ping-pong between two buffers
        P.r_first = 0; P.r_count = R;
        long long blocks = 0;
        for (int r = 0; r < R; ++r) { P.blk_begin[r] = blocks; blocks += (long long)pr->B * P.g.nscan[r]; }
        P.blk_begin[R] = blocks;
        // Six directions or more: one streaming pass per iteration sums what the previous iteration left at
        // every node, once per pair of opposite directions (mrf_isgmr_presum), and the sweeps read that one
        // array like a unary.  The messages of iteration k - 1 are dead once it has run, so the sweeps write
        // over them and the second buffer holds the sums.
        const long long NL = N * L;
        const bool presum = K > 1 && !pr->sgm_standard && g_tune_isgmr_presum != 1 && (g_tune_isgmr_presum == 2 || R >= 6);
        MrfPresumParams S;
        memset(&S, 0, sizeof(S));
        S.NL = NL; S.R = R; S.unary = pr->unary; S.m = bufA; S.out = bufB;
        for (int r = 0; r < R; ++r) S.opp[r] = P.g.opp[r];
        const bool svec = (NL % 4 == 0) && (((uintptr_t)pr->unary | (uintptr_t)bufA | (uintptr_t)bufB) % 16 == 0);
        long long sblocks = ((svec ? NL / 4 : NL) + 255) / 256;
        if (sblocks > 32768) sblocks = 32768;
        if (sblocks < 1) sblocks = 1;
        for (int k = 0; k < K; ++k) {
            if (presum) {
                P.m_in = bufA; P.m_out = bufA;
                P.unary = (k == 0) ? pr->unary : bufB;
                for (int r = 0; r < R; ++r) {
                    fill_sources(P, algo, r, 0u);
                    P.unary_slab[r] = (signed char)((k == 0) ? 0 : ((P.g.opp[r] >= 0 && P.g.opp[r] < r) ? P.g.opp[r] : r));
                }
                if (k > 0) {
                    const dim3 sg((unsigned)sblocks), sb(256);
                    if (R <= 8 && svec) hipLaunchKernelGGL((mrf_isgmr_presum<8, 4>), sg, sb, 0, st, S);
                    else if (R <= 8) hipLaunchKernelGGL((mrf_isgmr_presum<8, 1>), sg, sb, 0, st, S);
                    else if (svec) hipLaunchKernelGGL((mrf_isgmr_presum<16, 4>), sg, sb, 0, st, S);
                    else hipLaunchKernelGGL((mrf_isgmr_presum<16, 1>), sg, sb, 0, st, S);
                    { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "hipGetLastError"); }
                }
            } else {
                P.m_in = (k & 1) ? bufB : bufA;      // written by iteration k-1 (unused when k = 0)
                P.m_out = (k & 1) ? bufA : bufB;
                for (int r = 0; r < R; ++r) fill_sources(P, algo, r, k == 0 ? 0u : 0xffffffffu);
            }
            P.p = p + (size_t)k * pk;
            P.q = q + (size_t)k * qk;
            { const hipError_t e_ = dispatch_fwd(P, algo, tw, blocks, st); if (e_ != hipSuccess) return hip_fail(e_, "dispatch_fwd"); }
            if (presum && k > 0) {
                const size_t used = strlen(g_last_launch[0]);
                snprintf(g_last_launch[0] + used, sizeof(g_last_launch[0]) - used, " after mrf_isgmr_presum<%d,%d>", R <= 8 ? 8 : 16, svec ? 4 : 1);
            }
            final_m = P.m_out;
        }
    } else {
        // one launch per (iteration, direction); messages updated in place
        P.m_in = bufA; P.m_out = bufA;
        for (int k = 0; k < K; ++k) {
            for (int r = 0; r < R; ++r) {
                P.r_first = r; P.r_count = 1;
                P.blk_begin[0] = 0;
                const long long blocks = (long long)pr->B * P.g.nscan[r];
                P.blk_begin[1] = blocks;
                // in the first iteration the directions after r have not been written yet: they read as 0
                fill_sources(P, algo, r, k == 0 ? ((1u << r) - 1u) : 0xffffffffu);
                P.p = p + (size_t)k * pk;
                P.q = q + (size_t)k * qk;
                { const hipError_t e_ = dispatch_fwd(P, algo, tw, blocks, st); if (e_ != hipSuccess) return hip_fail(e_, "dispatch_fwd"); }
            }
        }
        final_m = bufA;
    }
    mark(g_ev_stop, st);

    MrfAggParams A;
    A.N = N; A.L = L; A.R = R; A.no_unary = pr->sgm_standard ? 1 : 0;
    A.unary = pr->unary; A.m = final_m; A.cost = cost; A.labels = labels;
    long long ablocks = (N + 3) / 4;
    if (ablocks > 65536) ablocks = 65536;
    if (R <= 4) hipLaunchKernelGGL(mrf_aggregate<4>, dim3((unsigned)ablocks), dim3(256), 0, st, A);
    else if (R <= 8) hipLaunchKernelGGL(mrf_aggregate<8>, dim3((unsigned)ablocks), dim3(256), 0, st, A);
    else hipLaunchKernelGGL(mrf_aggregate<16>, dim3((unsigned)ablocks), dim3(256), 0, st, A);
    { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "hipGetLastError"); }
    if (messages) {
        const hipError_t e_ = hipMemcpyAsync(messages, final_m, pk * sizeof(float), hipMemcpyDeviceToDevice, st);
        if (e_ != hipSuccess) return hip_fail(e_, "hipMemcpyAsync");
    }
    return MRF_OK;
}

#endif  // MRF_HAS_FWD

#if MRF_HAS_BWD
template <int LP, int NS, int D>
hipError_t launch_bwd(const MrfBwdParams &P, long long blocks, size_t lds, hipStream_t st)
{
    const dim3 grid((unsigned)blocks), block(64 * MRF_BWD_WAVES);
    const bool hot = !(P.rho_e || P.gE) && !(P.gw && P.v_mode == 0) && P.hot_label;
    const bool no_unary = hot && NS == 1 && P.unary_dir < 0;
    note_launch(1, "mrf_bwd_sweep", blocks, 64 * MRF_BWD_WAVES, "%d,%d,%d,%s,%s,%s%s", LP, NS, D,
                (P.gw && P.v_mode == 0) ? "true" : "false", hot ? "true" : "false",
                (P.rho_e || P.gE) ? "true" : "false", no_unary ? ",false" : "");
    if (P.rho_e && P.gw && P.v_mode == 0)
        hipLaunchKernelGGL((mrf_bwd_sweep<LP, NS, D, true, false, true>), grid, block, lds, st, P);
    else if (P.rho_e || P.gE)
        hipLaunchKernelGGL((mrf_bwd_sweep<LP, NS, D, false, false, true>), grid, block, lds, st, P);
    else if (P.gw && P.v_mode == 0)
        hipLaunchKernelGGL((mrf_bwd_sweep<LP, NS, D, true, false>), grid, block, lds, st, P);
    else if (no_unary) {
        if constexpr (NS == 1) {
            if (P.g.L == 64 * LP)
                hipLaunchKernelGGL((mrf_bwd_sweep<LP, NS, D, false, true, false, false, MRF_BWD_WAVES, true>), grid, block, lds, st, P);
            else
                hipLaunchKernelGGL((mrf_bwd_sweep<LP, NS, D, false, true, false, false>), grid, block, lds, st, P);
        }
    } else if (P.hot_label)
        hipLaunchKernelGGL((mrf_bwd_sweep<LP, NS, D, false, true>), grid, block, lds, st, P);
    else
        hipLaunchKernelGGL((mrf_bwd_sweep<LP, NS, D, false, false>), grid, block, lds, st, P);
    return hipGetLastError();
}

// The V gradient in one LDS table per workgroup of MRF_BWD_TILE_WAVES wavefronts (33..128 labels)
#define MRF_BWD_TILE_WAVES 8
template <int LP, int NS, int D>
hipError_t launch_bwd_tile(const MrfBwdParams &P, long long blocks, size_t lds, hipStream_t st)
{
    const dim3 grid((unsigned)blocks), block(64 * MRF_BWD_TILE_WAVES);
    const bool vg = P.gw && P.v_mode == 0;
    note_launch(1, "mrf_bwd_sweep", blocks, 64 * MRF_BWD_TILE_WAVES, "%d,%d,%d,%s,false,false,true,%d", LP, NS, D, vg ? "true" : "false",
                MRF_BWD_TILE_WAVES);
#define MRF_T_GO(...) \
    do { \
        if (lds > 64 * 1024) { \
            const hipError_t ea_ = hipFuncSetAttribute(reinterpret_cast<const void *>(&__VA_ARGS__), \
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (ea_ != hipSuccess) return ea_; \
        } \
        hipLaunchKernelGGL((__VA_ARGS__), grid, block, lds, st, P); \
    } while (0)
    if (vg) MRF_T_GO(mrf_bwd_sweep<LP, NS, D, true, false, false, true, MRF_BWD_TILE_WAVES>);
    else MRF_T_GO(mrf_bwd_sweep<LP, NS, D, false, false, false, true, MRF_BWD_TILE_WAVES>);
#undef MRF_T_GO
    return hipGetLastError();
}

template <int NS, int D>
hipError_t launch_bwd_split(const MrfBwdParams &P, long long blocks, size_t lds, hipStream_t st)
{
    const dim3 grid((unsigned)blocks), block(64u * (unsigned)((P.g.L + 63) / 64));
    note_launch(1, "mrf_bwd_sweep_split", blocks, (int)block.x, "%d,%d,%s", NS, D, (P.gw && P.v_mode == 0) ? "true" : "false");
    if (P.gw && P.v_mode == 0)
        hipLaunchKernelGGL((mrf_bwd_sweep_split<NS, D, true>), grid, block, lds, st, P);
    else
        hipLaunchKernelGGL((mrf_bwd_sweep_split<NS, D, false>), grid, block, lds, st, P);
    return hipGetLastError();
}

// LDS a workgroup of the chain sweep may take: the whole 160 KB of a compute unit when every
// compute unit gets at most one workgroup, half when two, else the 64 KB any launch may have.
inline size_t chain_lds_cap(long long scanlines)
{
    if (scanlines <= 256) return 156 * 1024;
    if (scanlines <= 512) return 78 * 1024;
    return 64 * 1024;
}

template <int LP, int NS, int D>
hipError_t launch_bwd_chain(const MrfBwdParams &P, int ni, bool vg, hipStream_t st)
{
    const dim3 grid((unsigned)P.total_scanlines);
    const bool gv = P.gV != nullptr;
    const bool gs = LP == 2 && P.gstore != nullptr;       // the helpers store the node gradients (V in LDS, no tables)
    if (gs) vg = false;
    note_launch(1, "mrf_bwd_sweep_chain", P.total_scanlines, 64 * (1 + ni), "%d,%d,%d,%d,%s,%s,%s", LP, NS, D, ni,
                (!(LP == 1 && gv) && vg) ? "true" : "false", ((LP == 1 && gv) || gs) ? "true" : "false",
                (!(LP == 1 && gv) && !gs && !vg && P.hot_label) ? "true" : "false");
    if (gv && (LP != 1 || P.total_scanlines * ni > grad_slots(P.g.L))) return hipErrorInvalidValue;
    const size_t lds = mrf_bwd_chain_lds_bytes(LP, ni, P.g.L, P.unary_dir >= 0, vg, gv || gs);
    if (lds > chain_lds_cap(P.total_scanlines)) return hipErrorInvalidValue;
    // (more than 64 KB of dynamic LDS has to be announced per kernel)
#define MRF_CH_GO(...) \
    do { \
        if (lds > 64 * 1024) { \
            const hipError_t ea_ = hipFuncSetAttribute(reinterpret_cast<const void *>(&__VA_ARGS__), \
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (ea_ != hipSuccess) return ea_; \
        } \
        hipLaunchKernelGGL((__VA_ARGS__), grid, dim3(64 * (1 + ni)), lds, st, P); \
    } while (0)
#define MRF_CH(n) \
    if (ni == n) { \
        if constexpr (LP == 1) { \
            if (gv) { \
                MRF_CH_GO(mrf_bwd_sweep_chain<LP, NS, D, n, false, true, false>); \
                return hipGetLastError(); \
            } \
        } \
        if constexpr (LP == 2) { \
            if (gs) { \
                MRF_CH_GO(mrf_bwd_sweep_chain<LP, NS, D, n, false, true, false>); \
                return hipGetLastError(); \
            } \
        } \
        if (vg) MRF_CH_GO(mrf_bwd_sweep_chain<LP, NS, D, n, true, false, false>); \
        else if (P.hot_label) MRF_CH_GO(mrf_bwd_sweep_chain<LP, NS, D, n, false, false, true>); \
        else MRF_CH_GO(mrf_bwd_sweep_chain<LP, NS, D, n, false, false, false>); \
        return hipGetLastError(); \
    }
    MRF_CH(2) MRF_CH(4) MRF_CH(6) MRF_CH(8) MRF_CH(12)
#undef MRF_CH
#undef MRF_CH_GO
    return hipErrorInvalidValue;
}

// two scanlines of up to 32 labels per workgroup: chain wavefront + ni helpers
template <int NS, int D>
hipError_t launch_bwd_chain_pk(const MrfBwdParams &P, int ni, hipStream_t st)
{
    const long long blocks = (P.total_scanlines + 1) / 2;
    const bool gv = P.gV != nullptr;
    note_launch(1, "mrf_bwd_sweep_chain_pk", blocks, 64 * (1 + ni), "%d,%d,%d,%s", NS, D, ni, gv ? "true" : "false");
    if (gv && blocks * 2 > grad_slots(P.g.L)) return hipErrorInvalidValue;
    const size_t lds = mrf_bwd_chain_pk_lds_bytes(ni, P.g.L, gv);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(64 * (1 + ni));
#define MRF_PK(n) \
    if (ni == n) { \
        if (gv) hipLaunchKernelGGL((mrf_bwd_sweep_chain_pk<NS, D, n, true>), grid, block, lds, st, P); \
        else hipLaunchKernelGGL((mrf_bwd_sweep_chain_pk<NS, D, n, false>), grid, block, lds, st, P); \
        return hipGetLastError(); \
    }
    MRF_PK(2) MRF_PK(4) MRF_PK(8)
#undef MRF_PK
    return hipErrorInvalidValue;
}

template <int SEG>
hipError_t launch_bwd_packed(const MrfBwdParams &P, int ns, hipStream_t st)
{
    constexpr int NSEG = 64 / SEG;
    const int L = P.g.L;
    long long blocks = (P.total_scanlines + NSEG - 1) / NSEG;
    if (P.gV && blocks > grad_slots(L) / NSEG) blocks = grad_slots(L) / NSEG;
    note_launch(1, "mrf_bwd_sweep_packed", blocks, 64, "%d,%d,%d", SEG, ns, ns <= 4 ? 4 : (ns == 8 ? 2 : 1));
    const size_t lds = sizeof(double) * (64 + (P.gV ? (size_t)NSEG * L * L : 0)) + sizeof(float) * (size_t)L * L;
    const dim3 grid((unsigned)blocks), block(64);
    if (ns == 1 && P.unary_dir < 0) hipLaunchKernelGGL((mrf_bwd_sweep_packed<SEG, 1, 4, false>), grid, block, lds, st, P);
    else if (ns == 1) hipLaunchKernelGGL((mrf_bwd_sweep_packed<SEG, 1, 4>), grid, block, lds, st, P);
    else if (ns == 4) hipLaunchKernelGGL((mrf_bwd_sweep_packed<SEG, 4, 4>), grid, block, lds, st, P);
    else if (ns == 8) hipLaunchKernelGGL((mrf_bwd_sweep_packed<SEG, 8, 2>), grid, block, lds, st, P);
    else hipLaunchKernelGGL((mrf_bwd_sweep_packed<SEG, 16, 1>), grid, block, lds, st, P);
    return hipGetLastError();
}

hipError_t dispatch_bwd(MrfBwdParams &P, int pairwise_kind, hipStream_t st)
{
    const int L = P.g.L;
    const int LP = (L + 63) / 64;
    long long blocks = (P.total_scanlines + MRF_BWD_WAVES - 1) / MRF_BWD_WAVES;
    if (P.gV && blocks > grad_slots(L) / MRF_BWD_WAVES) blocks = grad_slots(L) / MRF_BWD_WAVES;
    // LDS: scatter vectors, optional private V-gradient accumulators, optional copy of V
    P.gv_lds = (P.gV && L <= 32) ? 1 : 0;
    // truncated models scatter most labels to one target; pre-reducing it pays when LDS
    // conflicts, not instruction issue, bound the step
    P.hot_label = (pairwise_kind != MRF_PAIRWISE_DENSE && (L > 128 || P.total_scanlines > 1024)) ? 1 : 0;
    P.v_mode = 0;
    if (P.gw) {
        if ((size_t)L * L * sizeof(float) <= 40 * 1024) P.v_mode = 1;
        else if (pairwise_kind != MRF_PAIRWISE_DENSE) P.v_mode = 2;   // promise: V(mu,lambda) = V(0,|mu-lambda|)
    }
    const size_t lds = sizeof(double) * ((size_t)MRF_BWD_WAVES * 64 * LP + (P.gv_lds ? (size_t)MRF_BWD_WAVES * L * L : 0)) +
                       sizeof(float) * (P.v_mode == 1 ? (size_t)L * L : (P.v_mode == 2 ? (size_t)L : 0));
    int need = 0;
    for (int r = P.r_first; r < P.r_first + P.r_count; ++r)
        if (P.n_src[r] + (P.use_gc ? 1 : 0) > need) need = P.n_src[r] + (P.use_gc ? 1 : 0);
    const int ns = need <= 1 ? 1 : (need <= 4 ? 4 : (need <= 8 ? 8 : 16));
    // few scanlines: the node-to-node chain on a wavefront of its own, helpers around it
    // (its addressing wants a node step times L in 32 bits; with the V gradient, L <= 64, room in LDS and
    // a slot per helper)
    bool step_fits = true;
    for (int r = P.r_first; r < P.r_first + P.r_count; ++r) {
        const long long stp = ((long long)mrf_iabs(P.g.dh[r]) * P.g.W + mrf_iabs(P.g.dw[r])) * L;
        if (stp > 0x7fffffffLL) step_fits = false;
    }
    const bool gv_any = P.gV != nullptr;
    // 65..128 labels, one direction per launch: the chain layout has no room for V-gradient tables, so its
    // helpers store the node gradients and a streaming pass adds them up afterwards (mrf_bwd_gv_from_g)
    // (up to 512 scanlines per launch: beyond that the helpers' gathers from V in global memory hold the chain
    // layout back, 7.8 against 4.5 ms at 1,024 scanlines of 2 x 512 x 512 with 96 labels)
    const bool gv_apart = gv_any && LP == 2 && P.gstore_buf && P.r_count == 1 && !P.rho_e && !P.force_plain &&
                          P.total_scanlines <= 512 && g_tune_gv_apart != 1;
    const bool gv = gv_any && !gv_apart;      // the V gradient inside the sweep that runs
    // as many helpers as keep up with the chain while the machine and the LDS have room
    // (measured per launch shape at L = 96: 256 scanlines 165 / 121 / 98 / 90 us with 4 / 6 / 8 / 12
    // helpers; 512 scanlines, two workgroups per compute unit, 94 / 78 / 98 us with 4 / 6 / 8)
    int ni = g_tune_chain_ni ? g_tune_chain_ni
                             : (P.total_scanlines <= 256 ? 12
                                : (P.total_scanlines <= 512 ? (LP >= 2 ? 6 : 8) : (P.total_scanlines <= 1024 ? 6 : 4)));
    if (!g_tune_chain_ni && gv && P.total_scanlines > 384 && ni > 6) ni = 6;   // (the accumulators take LDS)
    const bool vg = P.gw && pairwise_kind == MRF_PAIRWISE_DENSE;
    // (LDS of the chain layout: with the node gradients stored apart it holds all of V, as with its own tables)
    const bool vg_lds = vg && !gv_apart, gv_lds = gv || gv_apart;
    while (ni > 2 && (mrf_bwd_chain_lds_bytes(LP, ni, L, P.unary_dir >= 0, vg_lds, gv_lds) > chain_lds_cap(P.total_scanlines) ||
                      (gv && P.total_scanlines * ni > grad_slots(L)))) ni = (ni == 12) ? 8 : ni - 2;
    // TRW coefficients or pairwise tables per edge: mrf_bwd_sweep handles them (and is the one
    // sweep that never touches V when no edge-weight gradient is asked for)
    const bool generic = P.rho_e != nullptr || P.force_plain;
    const bool chain_fits = !generic && step_fits && ns <= 8 && g_tune_chain != 1 &&
                            (!gv || (LP == 1 && P.total_scanlines * ni <= grad_slots(L))) &&
                            mrf_bwd_chain_lds_bytes(LP, ni, L, P.unary_dir >= 0, vg_lds, gv_lds) <= chain_lds_cap(P.total_scanlines);
    // (65..128 labels with several source arrays, TRWP: at 2,048 scanlines per launch the plain sweep is ahead,
    // 5.1 against 7.5 ms on 4 x 512 x 512 with 96 labels; at 1,024 the chain, 2.3 against 3.6 ms)
    // (more than 128 labels, one source array, ISGMR: at 1,536 scanlines the chain is ahead, 1.7 against 2.4 ms
    // with 192 labels, at 2,048 the plain sweep, 3.1 against 3.6 ms; several source arrays: level at 1,024)
    // (a launch of eight or more directions has many short diagonal scanlines: the chain stays ahead longer,
    // 0.80 against 1.04 ms at 2,876 scanlines of a 160 x 320 grid, 0.81 against 0.89 ms at 3,452 of 192 x 384)
    const long long chain_max = LP <= 2 ? ((LP == 2 && ns >= 4) ? 1536 : (P.r_count >= 8 ? 3584 : 2560)) : (ns == 1 ? 1536 : 512);
    const bool chain = chain_fits && (g_tune_chain == 2 || P.total_scanlines <= chain_max);
    // few labels, one direction per launch (TRWP), more scanlines than the chain layout takes one by one: two
    // scanlines per workgroup around a chain wavefront
    if (!generic && L <= 32 && P.r_count == 1 && ns <= 8 && g_tune_chain != 1 && g_tune_pack != 2 && g_tune_chain_pk != 1 &&
        (g_tune_chain_pk == 2 || (P.total_scanlines > 1024 && P.total_scanlines <= 2048))) {
        // (helpers: 4 x 512 x 512, 32 labels, 2,048 scanlines: 3.0 ms with four, 3.2 with eight, 3.5 ms for the packed
        // sweep; 3 x 512 x 512, 16 labels, 8 directions, 1,536 scanlines: 5.0 / 4.3 / 5.4 ms; the LDS of a compute unit,
        // which four such workgroups share, sets the pace)
        const int nip = (g_tune_chain_ni == 2 || g_tune_chain_ni == 4 || g_tune_chain_ni == 8) ? g_tune_chain_ni
                                                                                            : (P.total_scanlines <= 1536 ? 8 : 4);
        if (!(gv_any && (P.total_scanlines + 1) / 2 * 2 > grad_slots(L))) {
            if (ns == 1) return launch_bwd_chain_pk<1, 2>(P, nip, st);
            if (ns == 4) return launch_bwd_chain_pk<4, 2>(P, nip, st);
            return launch_bwd_chain_pk<8, 1>(P, nip, st);
        }
    }
    // few labels: several scanlines per wavefront, once there are enough of them
    if (!generic && L <= 32 && g_tune_pack != 1 && (g_tune_pack == 2 || P.total_scanlines >= 256) &&
        !(chain && g_tune_pack != 2 && (g_tune_chain == 2 || P.total_scanlines <= ((ns == 1 && !gv) ? 1536 : 1024))))
    {
        // three scanlines per wavefront: measured slower than two on the segmentation shape (the LDS
        // scatter, not instruction issue, bounds this sweep), so only on request
        if (L > 16 && L <= 21 && g_tune_pack3 == 2)
            return launch_bwd_packed<21>(P, ns, st);
        return L <= 16 ? launch_bwd_packed<16>(P, ns, st) : launch_bwd_packed<32>(P, ns, st);
    }
    if (chain) {
        // truncated models: the chain wavefront sums the lanes of the most popular scatter target
        // in registers
        // where LDS throughput, not the latency of the chain, bounds the launch
        P.hot_label = (pairwise_kind != MRF_PAIRWISE_DENSE && !gv && g_tune_chain_hot != 1 &&
                       (g_tune_chain_hot == 2 || L > 128 || P.total_scanlines > 1024)) ? 1 : 0;
        if (gv_apart) {
            double *const slots = P.gV;
            P.gV = nullptr; P.gstore = P.gstore_buf;
            hipError_t e = hipErrorInvalidValue;
            if (ns == 1) e = launch_bwd_chain<2, 1, 2>(P, ni, vg, st);
            else if (ns == 4) e = launch_bwd_chain<2, 4, 2>(P, ni, vg, st);
            else if (ns == 8) e = launch_bwd_chain<2, 8, 1>(P, ni, vg, st);
            P.gV = slots; P.gstore = nullptr;
            if (e != hipSuccess) return e;
            MrfGvParams G;
            G.N = P.g.N; G.L = L; G.g = P.gstore_buf;
            G.p = P.p + (size_t)P.r_first * P.g.N * L;
            G.w = P.w + (P.w_mul ? (size_t)P.r_first * P.g.N : 0); G.w_mul = P.w_mul;
            G.gV = slots;
            const size_t glds = sizeof(double) * (size_t)L * L;
            if (glds > 64 * 1024) {
                const hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void *>(&mrf_bwd_gv_from_g),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)glds);
                if (ea != hipSuccess) return ea;
            }
            hipLaunchKernelGGL(mrf_bwd_gv_from_g, dim3(256), dim3(512), glds, st, G);
            return hipGetLastError();
        }
#define MRF_CCASE(lp) \
        if (LP == lp && ns == 1) return launch_bwd_chain<lp, 1, 2>(P, ni, vg, st); \
        if (LP == lp && ns == 4) return launch_bwd_chain<lp, 4, (lp <= 2 ? 2 : 1)>(P, ni, vg, st); \
        if (LP == lp && ns == 8) return launch_bwd_chain<lp, 8, 1>(P, ni, vg, st);
        MRF_CCASE(1) MRF_CCASE(2) MRF_CCASE(3) MRF_CCASE(4)
#undef MRF_CCASE
    }
    // few scanlines and many labels: one wavefront per 64 labels
    const bool split = !generic && LP >= 3 && g_tune_split != 1 && ns <= 8 &&
                       (g_tune_split == 2 || ((P.total_scanlines < 1024 || (P.total_scanlines == 1024 && LP == 3)) && P.total_scanlines * LP <= 4096));
    if (split) {
        long long sblocks = P.total_scanlines;
        if (P.gV && sblocks > grad_slots(L)) sblocks = grad_slots(L);
        const size_t slds = sizeof(float) * (P.v_mode == 1 ? (size_t)L * L : (P.v_mode == 2 ? (size_t)L : 0));
        P.gv_lds = 0;
        if (ns == 1) return launch_bwd_split<1, 4>(P, sblocks, slds, st);
        if (ns == 4) return launch_bwd_split<4, 4>(P, sblocks, slds, st);
        return launch_bwd_split<8, 2>(P, sblocks, slds, st);
    }
    // the V gradient of 33..128 labels: one table in LDS per workgroup, more wavefronts per workgroup
    if (P.gV && !P.gv_lds && !(P.rho_e || P.gE) && LP <= 2 && g_tune_gv_tile != 1) {
        const size_t tlds = sizeof(double) * ((size_t)MRF_BWD_TILE_WAVES * 64 * LP + (size_t)L * L) +
                            sizeof(float) * (P.v_mode == 1 ? (size_t)L * L : (P.v_mode == 2 ? (size_t)L : 0));
        if (tlds <= 156 * 1024) {
            long long tblocks = (P.total_scanlines + MRF_BWD_TILE_WAVES - 1) / MRF_BWD_TILE_WAVES;
            if (tblocks > grad_slots(L)) tblocks = grad_slots(L);
            P.gv_lds = 2;
            P.hot_label = 0;
#define MRF_TCASE(lp) \
            if (LP == lp && ns == 1) return launch_bwd_tile<lp, 1, 4>(P, tblocks, tlds, st); \
            if (LP == lp && ns == 4) return launch_bwd_tile<lp, 4, 4>(P, tblocks, tlds, st); \
            if (LP == lp && ns == 8) return launch_bwd_tile<lp, 8, 2>(P, tblocks, tlds, st); \
            if (LP == lp && ns == 16) return launch_bwd_tile<lp, 16, 1>(P, tblocks, tlds, st);
            MRF_TCASE(1) MRF_TCASE(2)
#undef MRF_TCASE
        }
    }
#define MRF_BCASE(lp) \
    if (LP == lp && ns == 1) return launch_bwd<lp, 1, (lp >= 3 ? 2 : 4)>(P, blocks, lds, st); \
    if (LP == lp && ns == 4) return launch_bwd<lp, 4, (lp <= 2 ? 4 : 2)>(P, blocks, lds, st); \
    if (LP == lp && ns == 8) return launch_bwd<lp, 8, 2>(P, blocks, lds, st); \
    if (LP == lp && ns == 16) return launch_bwd<lp, 16, 1>(P, blocks, lds, st);
    MRF_BCASE(1) MRF_BCASE(2) MRF_BCASE(3) MRF_BCASE(4)
#undef MRF_BCASE
    return hipErrorInvalidValue;
}

hipError_t fill(float *dst, long long n, float v, hipStream_t st)
{
    long long blocks = (n + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(mrf_fill_f32, dim3((unsigned)blocks), dim3(256), 0, st, dst, n, v);
    return hipGetLastError();
}

hipError_t fill64(double *dst, long long n, hipStream_t st)
{
    long long blocks = (n + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(mrf_fill_f64, dim3((unsigned)blocks), dim3(256), 0, st, dst, n, 0.0);
    return hipGetLastError();
}

int run_backward(const mrf_problem *pr, int algo, const float *grad_cost, const uint8_t *p, const uint8_t *q,
                 float *grad_unary, float *grad_w, float *grad_V, void *workspace, size_t workspace_bytes,
                 void *hip_stream)
{
    if (pr && pr->sgm_standard) return MRF_ERR_BAD_ALGORITHM;    // (Alg. 3 differentiates the revised update only)
    int rc = check_problem(pr, algo, false);
    if (rc != MRF_OK) return rc;
    if (!grad_cost || !p || !q || !grad_unary) return MRF_ERR_NULL_POINTER;
    // pairwise potentials per edge: grad_V is their gradient [R][B][H][W][L][L]; there are no
    // edge weights to differentiate
    const bool edge_tables = pr->pairwise_edge != nullptr;
    if (edge_tables && grad_w) return MRF_ERR_BAD_PAIRWISE_KIND;
    const size_t need = mrf_workspace_bytes(pr, algo, 1);
    if (!workspace) return MRF_ERR_NULL_POINTER;
    if (workspace_bytes < need) return MRF_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;

    MrfBwdParams P;
    memset(&P, 0, sizeof(P));
    fill_geom(pr, P.g);
    const long long N = P.g.N;
    const int R = pr->R, L = pr->L, K = pr->K;
    const long long NL = N * L;
    P.V = pr->pairwise;
    P.gw = grad_w;
    P.gc = grad_cost;
    P.gunary = grad_unary;
    P.unary_dir = -1;
    P.rho_e = (algo == MRF_TRWP) ? pr->rho_edge : nullptr;
    const size_t pk = (size_t)R * N * L, qk = (size_t)R * N;

    // workspace: [scalars 256 B][buf0][buf1 (ISGMR only)][V-gradient slots][node gradients for mrf_bwd_gv_from_g (65..128 labels)]
    char *ws = (char *)workspace;
    float *scal = (float *)ws;
    float *buf0 = (float *)(ws + kAlign);                   // ISGMR: grad m-hat   TRWP: s per direction
    float *buf1 = (float *)(ws + kAlign + msg_bytes(pr));   // ISGMR: s per direction
    double *gvslots = (double *)(ws + kAlign + (algo == MRF_ISGMR ? 2 : 1) * msg_bytes(pr));
    { const hipError_t e_ = init_header(workspace, pr->edge_weight_scalar, st); if (e_ != hipSuccess) return hip_fail(e_, "init_header"); }
    P.fault = (int *)(ws + kFaultOffset);
    P.spin_limit = spin_limit();
    if (pr->edge_weight) { P.w = pr->edge_weight; P.w_mul = 1; }
    else { P.w = scal; P.w_mul = 0; }

    if (grad_w) {
        const hipError_t e_ = fill(grad_w, (long long)R * N, 0.0f, st);
        if (e_ != hipSuccess) return hip_fail(e_, "fill");
    }
    P.force_plain = edge_tables ? 1 : 0;
    if (edge_tables && grad_V) {
        P.gE = grad_V;
        { const hipError_t e_ = fill(grad_V, (long long)R * N * L * L, 0.0f, st); if (e_ != hipSuccess) return hip_fail(e_, "fill"); }
    } else if (grad_V) {
        P.gV = gvslots;
        if (gstore_bytes(pr) > 0) P.gstore_buf = (double *)((char *)gvslots + gradv_bytes(pr));
        { const hipError_t e_ = fill64(gvslots, grad_slots(L) * L * L, st); if (e_ != hipSuccess) return hip_fail(e_, "fill64"); }
    }

    mark(g_ev_start, st);
    if (algo == MRF_ISGMR) {
        P.r_first = 0; P.r_count = R;
        long long tot = 0;
        for (int r = 0; r < R; ++r) { P.blk_begin[r] = tot; tot += (long long)pr->B * P.g.nscan[r]; }
        P.blk_begin[R] = tot;
        P.total_scanlines = tot;
        P.S = buf1;
        for (int r = 0; r < R; ++r) {
            // one source: grad m-hat^r itself
            P.n_src[r] = 1; P.src_dir[r][0] = (signed char)r; P.coefG[r][0] = 1.0f; P.coefT[r][0] = 0.0f;
            P.carry_scale[r] = 1.0f;
        }
        MrfCombineParams C;
        memset(&C, 0, sizeof(C));
        C.NL = NL; C.R = R; C.skip_dir = -1;
        for (int r = 0; r < R; ++r) {
            C.opp[r] = P.g.opp[r];
            C.canon[r] = (P.g.opp[r] >= 0 && P.g.opp[r] < r) ? P.g.opp[r] : r;
        }
        C.S = buf1; C.gc = grad_cost; C.gunary = grad_unary;
        long long cblocks = (NL + 255) / 256;
        if (cblocks > 32768) cblocks = 32768;
        // four entries per thread where every array starts on a 16-byte boundary
        const bool cvec = (NL % 4 == 0) && (((uintptr_t)buf0 | (uintptr_t)buf1 | (uintptr_t)grad_cost | (uintptr_t)grad_unary) % 16 == 0);
        long long cblocks4 = (NL / 4 + 255) / 256;
        if (cblocks4 > 32768) cblocks4 = 32768;
        if (cblocks4 < 1) cblocks4 = 1;
        // Up to four directions: no combine pass between iterations.  The sweep of direction d in
        // iteration k reads what the other directions scattered in iteration k + 1 itself (grad m-hat^d =
        // sum over r not in {d, d-} of s^r: at most two arrays, against one array plus the combine's 2 R + 2
        // per node) and the sweep of direction 0 adds all of them, and its own s, to grad theta; one
        // combine pass at the end adds what the other directions scattered in the last sweep.  The s
        // arrays of two iterations alternate between the two buffers.
        // Pays only where the pass is bound by its launches (the combine passes are a third of them): on the
        // stereo and segmentation shapes the sweeps, which are bound by instruction issue and latency, lose
        // more on the extra arrays (2.29 against 1.80 ms, 4.05 against 3.76 ms) than the combine passes cost.
        const bool lazy = R <= 4 && g_tune_isgmr_lazy != 1 && (g_tune_isgmr_lazy == 2 || NL <= (1LL << 19));
        for (int k = K - 1; lazy && k >= 0; --k) {
            float *s_cur = ((K - 1 - k) & 1) ? buf0 : buf1, *s_prev = ((K - 1 - k) & 1) ? buf1 : buf0;
            P.S = s_cur;
            P.unary_dir = 0;
            P.unary_init = (k == K - 1);
            if (k == K - 1) {
                // back Eq. isgmr-aggregation: every direction's message, and theta, receive grad c
                P.src_base = grad_cost; P.src_stride = 0;
                for (int r = 0; r < R; ++r) { P.n_src[r] = 1; P.src_dir[r][0] = (signed char)r; P.coefG[r][0] = 1.0f; P.coefT[r][0] = 1.0f; }
            } else {
                P.src_base = s_prev; P.src_stride = NL;
                for (int d = 0; d < R; ++d) {
                    int n = 0;
                    for (int r = 0; r < R; ++r) {
                        if (r == d) continue;
                        const bool excluded = (r == P.g.opp[d]);          // Eq. isgmr leaves out r and r-
                        if (excluded && d != 0) continue;
                        P.src_dir[d][n] = (signed char)r;
                        P.coefG[d][n] = excluded ? 0.0f : 1.0f;
                        P.coefT[d][n] = 1.0f;                             // (grad theta: read by direction 0 only)
                        ++n;
                    }
                    P.n_src[d] = (signed char)n;
                }
            }
            P.p = p + (size_t)k * pk;
            P.q = q + (size_t)k * qk;
            { const hipError_t e_ = dispatch_bwd(P, pr->pairwise_kind, st); if (e_ != hipSuccess) return hip_fail(e_, "dispatch_bwd"); }
            if (k == 0) {
                C.S = s_cur; C.first = 0; C.ghat = nullptr; C.skip_dir = 0;
                const dim3 cg((unsigned)(cvec ? cblocks4 : cblocks)), cb(256);
                if (cvec) hipLaunchKernelGGL((mrf_isgmr_bwd_combine<4, 4>), cg, cb, 0, st, C);
                else hipLaunchKernelGGL((mrf_isgmr_bwd_combine<4, 1>), cg, cb, 0, st, C);
                { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "hipGetLastError"); }
            }
        }
        for (int k = K - 1; !lazy && k >= 0; --k) {
            if (k == K - 1) { P.src_base = grad_cost; P.src_stride = 0; }   // back Eq. isgmr-aggregation
            else { P.src_base = buf0; P.src_stride = NL; }
            // (grad m-hat of a direction and of its opposite are the same sum: one array serves both)
            for (int r = 0; r < R; ++r) P.src_dir[r][0] = (signed char)((k == K - 1) ? r : C.canon[r]);
            P.p = p + (size_t)k * pk;
            P.q = q + (size_t)k * qk;
            { const hipError_t e_ = dispatch_bwd(P, pr->pairwise_kind, st); if (e_ != hipSuccess) return hip_fail(e_, "dispatch_bwd"); }
            C.first = (k == K - 1);
            C.ghat = (k > 0) ? buf0 : nullptr;
            const dim3 cg((unsigned)(cvec ? cblocks4 : cblocks)), cb(256);
            if (R <= 4 && cvec) hipLaunchKernelGGL((mrf_isgmr_bwd_combine<4, 4>), cg, cb, 0, st, C);
            else if (R <= 4) hipLaunchKernelGGL((mrf_isgmr_bwd_combine<4, 1>), cg, cb, 0, st, C);
            else if (R <= 8 && cvec) hipLaunchKernelGGL((mrf_isgmr_bwd_combine<8, 4>), cg, cb, 0, st, C);
            else if (R <= 8) hipLaunchKernelGGL((mrf_isgmr_bwd_combine<8, 1>), cg, cb, 0, st, C);
            else if (cvec) hipLaunchKernelGGL((mrf_isgmr_bwd_combine<16, 4>), cg, cb, 0, st, C);
            else hipLaunchKernelGGL((mrf_isgmr_bwd_combine<16, 1>), cg, cb, 0, st, C);
            { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "hipGetLastError"); }
        }
    } else {
        P.S = buf0;
        P.src_base = buf0; P.src_stride = NL;
        P.unary_dir = 0;
        for (int k = K - 1; k >= 0; --k) {
            for (int d = R - 1; d >= 0; --d) {      // reverse of the forward direction order
                P.r_first = d; P.r_count = 1;
                P.blk_begin[0] = 0;
                P.total_scanlines = (long long)pr->B * P.g.nscan[d];
                P.blk_begin[1] = P.total_scanlines;
                // directions that swept since the last sweep of d: all others, except that in the
                // first processed iteration only those after d have swept at all
                int n = 0;
                for (int r = 0; r < R; ++r) {
                    if (r == d || (k == K - 1 && r < d)) continue;
                    P.src_dir[d][n] = (signed char)r;
                    const float rho_r = pr->rho ? pr->rho[r] : 1.0f;   // (not read when rho_edge is given)
                    P.coefG[d][n] = rho_r - (r == P.g.opp[d] ? 1.0f : 0.0f);
                    P.coefT[d][n] = rho_r;
                    ++n;
                }
                P.n_src[d] = (signed char)n;
                P.carry_scale[d] = pr->rho ? pr->rho[d] : 1.0f;
                P.use_gc = (k == K - 1);
                P.unary_init = (k == K - 1);
                P.p = p + (size_t)k * pk;
                P.q = q + (size_t)k * qk;
                { const hipError_t e_ = dispatch_bwd(P, pr->pairwise_kind, st); if (e_ != hipSuccess) return hip_fail(e_, "dispatch_bwd"); }
            }
        }
    }
    mark(g_ev_stop, st);
    if (grad_V && !edge_tables) {
        const long long n = (long long)L * L;
        const long long slots = grad_slots(L), chunk = 128;
        const unsigned eb = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(mrf_reduce_slot_chunks, dim3(eb, (unsigned)((slots + chunk - 1) / chunk)), dim3(256), 0, st,
                           gvslots, n, slots, chunk);
        { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "hipGetLastError"); }
        hipLaunchKernelGGL(mrf_reduce_slot_heads, dim3(eb), dim3(256), 0, st, (const double *)gvslots, grad_V, n, slots, chunk);
        { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "hipGetLastError"); }
    }
    return MRF_OK;
}

#endif  // MRF_HAS_BWD

}  // namespace mrf_host

#if MRF_HAS_API
namespace mrf_host {
hipError_t init_header(void *workspace, float w_scalar, hipStream_t st)
{
    hipLaunchKernelGGL(mrf_init_header, dim3(1), dim3(64), 0, st, (float *)workspace,
                       (int *)((char *)workspace + kFaultOffset), w_scalar);
    return hipGetLastError();
}
}  // namespace mrf_host

using namespace mrf_host;

extern "C" {

size_t mrf_workspace_bytes(const mrf_problem *prob, int algo, int backward)
{
    if (check_problem(prob, algo, false) != MRF_OK) return 0;
    if (!backward) return kAlign + (algo == MRF_ISGMR ? 2 : 1) * msg_bytes(prob);
    return kAlign + (algo == MRF_ISGMR ? 2 : 1) * msg_bytes(prob) + gradv_bytes(prob) + gstore_bytes(prob);
}

int mrf_validate(const mrf_problem *prob, int algo) { return check_problem(prob, algo, true); }

int mrf_forward_window(const mrf_problem *prob, int algo)
{
    const int rc = check_problem(prob, algo, false);
    if (rc != MRF_OK) return rc;
    // The window sweeps take up to fifteen message arrays next to the unary for TRWP (any direction set the
    // library accepts) and up to seven for ISGMR, whose sweeps read a single array from six directions on
    // (run_forward); count what an ISGMR launch of the later iterations reads with fewer directions.
    if (algo == MRF_ISGMR && !(prob->R >= 6 && prob->K > 1)) {
        int most = 0;
        for (int r = 0; r < prob->R; ++r) {
            bool has_opp = false;
            for (int d = 0; d < prob->R; ++d)
                if (prob->dirs[2 * d] == -prob->dirs[2 * r] && prob->dirs[2 * d + 1] == -prob->dirs[2 * r + 1]) has_opp = true;
            const int n = prob->R - 1 - (has_opp ? 1 : 0);
            if (n > most) most = n;
        }
        if (most + 1 > 8) return 0;
    }
    return window_width(prob);
}

int mrf_isgmr_forward(const mrf_problem *prob, float *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                      float *messages, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_forward(prob, MRF_ISGMR, cost, labels, p, q, messages, workspace, workspace_bytes, hip_stream);
}

int mrf_trwp_forward(const mrf_problem *prob, float *cost, uint8_t *labels, uint8_t *p, uint8_t *q,
                     float *messages, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_forward(prob, MRF_TRWP, cost, labels, p, q, messages, workspace, workspace_bytes, hip_stream);
}

int mrf_isgmr_backward(const mrf_problem *prob, const float *grad_cost, const uint8_t *p, const uint8_t *q,
                       float *grad_unary, float *grad_edge_weight, float *grad_pairwise,
                       void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_backward(prob, MRF_ISGMR, grad_cost, p, q, grad_unary, grad_edge_weight, grad_pairwise,
                        workspace, workspace_bytes, hip_stream);
}

int mrf_trwp_backward(const mrf_problem *prob, const float *grad_cost, const uint8_t *p, const uint8_t *q,
                      float *grad_unary, float *grad_edge_weight, float *grad_pairwise,
                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_backward(prob, MRF_TRWP, grad_cost, p, q, grad_unary, grad_edge_weight, grad_pairwise,
                        workspace, workspace_bytes, hip_stream);
}

int64_t mrf_scanline_count(int32_t H, int32_t W, int32_t dh, int32_t dw)
{
    if (H < 1 || W < 1) return MRF_ERR_BAD_SHAPE;
    if (dh == 0 && dw == 0) return MRF_ERR_BAD_DIRECTIONS;
    return mrf_geom_scanlines(H, W, dh, dw);
}

int mrf_scanline_head(int32_t H, int32_t W, int32_t dh, int32_t dw, int64_t t,
                      int32_t *y0, int32_t *x0, int32_t *len)
{
    if (!y0 || !x0 || !len) return MRF_ERR_NULL_POINTER;
    if (H < 1 || W < 1) return MRF_ERR_BAD_SHAPE;
    if (dh == 0 && dw == 0) return MRF_ERR_BAD_DIRECTIONS;
    if (t < 0 || t >= mrf_geom_scanlines(H, W, dh, dw)) return MRF_ERR_BAD_SHAPE;
    int a, b, c;
    mrf_geom_head(H, W, dh, dw, t, a, b, c);
    *y0 = a; *x0 = b; *len = c;
    return MRF_OK;
}

const char *mrf_strerror(int status)
{
    switch (status) {
    case MRF_OK: return "ok";
    case MRF_ERR_NULL_POINTER: return "a required pointer is NULL";
    case MRF_ERR_BAD_SHAPE: return "B, H, W must be >= 1 and B*H*W < 2^31";
    case MRF_ERR_BAD_LABELS: return "L must be in [1, 256]";
    case MRF_ERR_BAD_ITERATIONS: return "K must be >= 1";
    case MRF_ERR_BAD_DIRECTIONS: return "R must be in [1, 16], steps non-zero and distinct";
    case MRF_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than mrf_workspace_bytes()";
    case MRF_ERR_BAD_PAIRWISE_KIND: return "unknown pairwise_kind, invalid trunc or negative scale";
    case MRF_ERR_BAD_ALGORITHM: return "algo must be MRF_ISGMR or MRF_TRWP";
    case MRF_ERR_HIP: return "HIP runtime call or kernel launch failed";
    case MRF_ERR_WAIT_EXPIRED: return "a wait between wavefronts of a sweep ran out of its budget: the results of that call are incomplete";
    case MRF_ERR_SCRATCH_LIMIT: return "problem exceeds the fixed scratch of a no-allocation entry point (batch > 64)";
    default: return "unknown status";
    }
}

size_t mrf_energy_workspace_bytes(const mrf_problem *prob)
{
    if (check_problem(prob, MRF_ISGMR, false) != MRF_OK) return 0;
    return sizeof(double) * (size_t)prob->B * MRF_HEAD_BLOCKS;
}

// launches of mrf_energy on `partial`, which holds B * MRF_HEAD_BLOCKS doubles
static int energy_launch(const mrf_problem *prob, const uint8_t *labels, double *energy, double *partial,
                         hipStream_t st)
{
    MrfEnergyParams E;
    memset(&E, 0, sizeof(E));
    fill_geom(prob, E.g);
    E.unary = prob->unary; E.V = prob->pairwise; E.Te = prob->pairwise_edge; E.labels = labels;
    E.partial = partial;
    if (prob->edge_weight) { E.w = prob->edge_weight; E.w_mul = 1; }
    else { E.w = nullptr; E.w_mul = 0; }
    for (int r = 0; r < prob->R; ++r)
        if (E.g.opp[r] < 0 || r < E.g.opp[r]) E.edge_dir[E.n_edge_dir++] = r;
    const long long HW = (long long)prob->H * prob->W;
    long long blocks = (HW + 255) / 256;
    if (blocks > MRF_HEAD_BLOCKS) blocks = MRF_HEAD_BLOCKS;
    E.w_scalar = prob->edge_weight_scalar;
    hipLaunchKernelGGL(mrf_energy_partial, dim3((unsigned)blocks, (unsigned)prob->B), dim3(256), 0, st, E);
    { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "mrf_energy_partial"); }
    hipLaunchKernelGGL(mrf_sum_partials, dim3((unsigned)prob->B), dim3(64), 0, st, (const double *)E.partial, (int)blocks,
                       energy, (const long long *)nullptr);
    { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "mrf_sum_partials"); }
    return MRF_OK;
}

int mrf_energy(const mrf_problem *prob, const uint8_t *labels, double *energy, void *workspace,
               size_t workspace_bytes, void *hip_stream)
{
    const int rc = check_problem(prob, MRF_ISGMR, true);
    if (rc != MRF_OK) return rc;
    if (!labels || !energy || !workspace) return MRF_ERR_NULL_POINTER;
    if (workspace_bytes < mrf_energy_workspace_bytes(prob)) return MRF_ERR_WORKSPACE_TOO_SMALL;
    return energy_launch(prob, labels, energy, (double *)workspace, (hipStream_t)hip_stream);
}

// ---- mrf_energy for callers that cannot allocate: the partial sums live in a device array of the
// library's own.  Every GPU holds its own copy of the array at its own address; the name below is
// only the host-side handle of the symbol, so host code asks the runtime once per device where the
// copy lives and passes that pointer on.
static __device__ __align__(256) double mrf_energy_scratch[(size_t)MRF_ENERGY_NOALLOC_MAX_BATCH * MRF_HEAD_BLOCKS];
#define MRF_MAX_DEVICES 64
static double *g_energy_scratch_ptr[MRF_MAX_DEVICES];     // per device, set on the first call there

int mrf_energy_noalloc(const mrf_problem *prob, const uint8_t *labels, double *energy, void *hip_stream)
{
    const int rc = check_problem(prob, MRF_ISGMR, true);
    if (rc != MRF_OK) return rc;
    if (!labels || !energy) return MRF_ERR_NULL_POINTER;
    if (prob->B > MRF_ENERGY_NOALLOC_MAX_BATCH) return MRF_ERR_SCRATCH_LIMIT;
    int dev = -1;
    { const hipError_t e_ = hipGetDevice(&dev); if (e_ != hipSuccess) return hip_fail(e_, "hipGetDevice"); }
    if (dev < 0 || dev >= MRF_MAX_DEVICES) return MRF_ERR_SCRATCH_LIMIT;
    if (!g_energy_scratch_ptr[dev]) {
        double *ptr = nullptr;
        const hipError_t e_ = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(mrf_energy_scratch));
        if (e_ != hipSuccess || !ptr) return hip_fail(e_, "hipGetSymbolAddress(mrf_energy_scratch)");
        g_energy_scratch_ptr[dev] = ptr;
    }
    // (every partial sum the second kernel reads is written by the first: nothing has to start at zero)
    return energy_launch(prob, labels, energy, g_energy_scratch_ptr[dev], (hipStream_t)hip_stream);
}

size_t mrf_softmin_l1_workspace_bytes(void)
{
    return kAlign + (sizeof(double) + sizeof(long long)) * MRF_HEAD_BLOCKS;
}

static int softmin_loss(int64_t n_pixels, int32_t L, const float *cost, const float *target, const uint8_t *mask,
                        float *disparity, double *loss, float *grad_cost, double beta, void *workspace,
                        size_t workspace_bytes, void *hip_stream);

int mrf_softmin_l1(int64_t n_pixels, int32_t L, const float *cost, const float *target, const uint8_t *mask,
                   float *disparity, double *loss, float *grad_cost, void *workspace, size_t workspace_bytes,
                   void *hip_stream)
{
    return softmin_loss(n_pixels, L, cost, target, mask, disparity, loss, grad_cost, 0.0, workspace, workspace_bytes,
                        hip_stream);
}

int mrf_softmin_smooth_l1(int64_t n_pixels, int32_t L, const float *cost, const float *target, const uint8_t *mask,
                          float beta, float *disparity, double *loss, float *grad_cost, void *workspace,
                          size_t workspace_bytes, void *hip_stream)
{
    if (!(beta > 0.0f) || !(beta < INFINITY)) return MRF_ERR_BAD_PAIRWISE_KIND;
    return softmin_loss(n_pixels, L, cost, target, mask, disparity, loss, grad_cost, (double)beta, workspace,
                        workspace_bytes, hip_stream);
}

static int softmin_loss(int64_t n_pixels, int32_t L, const float *cost, const float *target, const uint8_t *mask,
                        float *disparity, double *loss, float *grad_cost, double beta, void *workspace,
                        size_t workspace_bytes, void *hip_stream)
{
    if (n_pixels < 1 || n_pixels > 0x7fffffffLL) return MRF_ERR_BAD_SHAPE;
    if (L < 1 || L > MRF_MAX_LABELS) return MRF_ERR_BAD_LABELS;
    if (!cost || !target || !loss || !workspace) return MRF_ERR_NULL_POINTER;
    if (workspace_bytes < mrf_softmin_l1_workspace_bytes()) return MRF_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    MrfLossParams Q;
    memset(&Q, 0, sizeof(Q));
    Q.N = n_pixels; Q.L = L; Q.cost = cost; Q.target = target; Q.mask = mask;
    Q.disparity = disparity; Q.grad_cost = grad_cost; Q.beta = beta;
    Q.count = (long long *)workspace;
    Q.partial = (double *)((char *)workspace + kAlign);
    Q.cpartial = (long long *)((char *)workspace + kAlign + sizeof(double) * MRF_HEAD_BLOCKS);
    if (mask) {
        long long cb = (n_pixels + 255) / 256;
        if (cb > MRF_HEAD_BLOCKS) cb = MRF_HEAD_BLOCKS;
        hipLaunchKernelGGL(mrf_count_mask_partial, dim3((unsigned)cb), dim3(256), 0, st, Q);
        hipLaunchKernelGGL(mrf_count_mask_final, dim3(1), dim3(64), 0, st, Q, (int)cb);
    } else {
        hipLaunchKernelGGL(mrf_set_i64, dim3(1), dim3(64), 0, st, Q.count, (long long)n_pixels);
    }
    { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "mrf_softmin_l1 count"); }
    long long blocks = (n_pixels + 3) / 4;
    if (blocks > MRF_HEAD_BLOCKS) blocks = MRF_HEAD_BLOCKS;
    hipLaunchKernelGGL(mrf_softmin_l1_kernel, dim3((unsigned)blocks), dim3(256), 0, st, Q);
    { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "mrf_softmin_l1_kernel"); }
    hipLaunchKernelGGL(mrf_sum_partials, dim3(1), dim3(64), 0, st, (const double *)Q.partial, (int)blocks, loss,
                       (const long long *)Q.count);
    { const hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return hip_fail(e_, "mrf_sum_partials"); }
    return MRF_OK;
}

// Which forward or backward call used this workspace last, did one of its waits between
// wavefronts run out?  Waits for the stream, then reads the fault word of the header.
int mrf_workspace_fault(const void *workspace, void *hip_stream)
{
    if (!workspace) return MRF_ERR_NULL_POINTER;
    hipStream_t st = (hipStream_t)hip_stream;
    { const hipError_t e_ = hipStreamSynchronize(st); if (e_ != hipSuccess) return hip_fail(e_, "hipStreamSynchronize"); }
    int word = 0;
    { const hipError_t e_ = hipMemcpy(&word, (const char *)workspace + kFaultOffset, sizeof(int), hipMemcpyDeviceToHost);
      if (e_ != hipSuccess) return hip_fail(e_, "hipMemcpy"); }
    return word != 0 ? MRF_ERR_WAIT_EXPIRED : MRF_OK;
}

const char *mrf_last_error_detail(void) { return g_error_detail; }

const char *mrf_last_sweep_kernel(int backward) { return g_last_sweep[backward ? 1 : 0]; }

const char *mrf_last_sweep_launch(int backward) { return g_last_launch[backward ? 1 : 0]; }

const char *mrf_version(void) { return "0.3.8"; }

int mrf_set_sweep_events(void *start_event, void *stop_event)
{
    g_ev_start = (hipEvent_t)start_event;
    g_ev_stop = (hipEvent_t)stop_event;
    return MRF_OK;
}

int mrf_tune(int knob, int value)
{
    if (knob == 0) { g_tune_mch = value; return MRF_OK; }
    if (knob == 1) { g_tune_no_window = value; return MRF_OK; }
    if (knob == 2) { g_tune_split = value; return MRF_OK; }
    if (knob == 3) { g_tune_pack = value; return MRF_OK; }
    if (knob == 4) { g_tune_duo = value; return MRF_OK; }
    if (knob == 5) { g_tune_duo_ni = (value == 1 || value == 2) ? value : 0; return MRF_OK; }
    if (knob == 6) { g_tune_chain = value; return MRF_OK; }
    if (knob == 12) { g_tune_chain_hot = value; return MRF_OK; }
    if (knob == 8) { g_tune_loader = value; return MRF_OK; }
    if (knob == 9) { g_tune_squad = value; return MRF_OK; }
    if (knob == 11) { g_tune_pack_idx = value; return MRF_OK; }
    if (knob == 10) { g_tune_squad_ni = value; return MRF_OK; }
    if (knob == 13) { g_tune_pack3 = value; return MRF_OK; }
    if (knob == 14) { g_tune_spin_limit = value > 0 ? value : 0; return MRF_OK; }
    if (knob == 15) { g_tune_isgmr_lazy = value; return MRF_OK; }
    if (knob == 16) { g_tune_dense_sliced = value; return MRF_OK; }
    if (knob == 17) { g_tune_isgmr_presum = value; return MRF_OK; }
    if (knob == 18) { g_tune_gv_tile = value; return MRF_OK; }
    if (knob == 19) { g_tune_gv_apart = value; return MRF_OK; }
    if (knob == 20) { g_tune_chain_pk = value; return MRF_OK; }
    if (knob == 7) { g_tune_chain_ni = (value == 2 || value == 4 || value == 6 || value == 8 || value == 12) ? value : 0; return MRF_OK; }
    return MRF_ERR_BAD_ALGORITHM;
}

}  // extern "C"
#endif  // MRF_HAS_API
