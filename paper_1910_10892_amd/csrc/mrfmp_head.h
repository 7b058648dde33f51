// The two heads around the message-passing path: the energy of a labelling
// (Sec. 3.1, Eq. energy-function) and the SoftMin disparity regression with an L1 loss
// (Appendix, Eqs. supp-isgmr-confidence, supp-isgmr-regression), whose derivative with
// respect to the final costs is what the backward passes (Alg. 3, 4) start from.
//
// Both stream over the grid once and are bound by HBM.  All sums are formed in double, in
// an order that depends only on the launch shape (per wavefront in node order, per
// workgroup in wavefront order, then over workgroups in index order), so results are
// reproducible run to run.
#pragma once

#include "mrfmp_device.h"

#define MRF_HEAD_BLOCKS 4096     // workgroups per batch image (energy) / per call (loss): partial sums kept

struct MrfEnergyParams {
    MrfGeom g;
    const float *unary;      // [B][H][W][L]
    const float *V;          // [L][L], V[x at i-r][x at i]
    const float *Te;         // [R][N][L][L] pairwise potentials per edge, or NULL: then w * V applies
    const float *w;          // [R][N], or NULL with w_mul == 0: w_scalar for every edge
    int w_mul;
    float w_scalar;
    const uint8_t *labels;   // [B][H][W]
    int edge_dir[MRF_MAXR];  // directions whose edges enter the energy: the first of every opposite pair
    int n_edge_dir;
    double *partial;         // [B][MRF_HEAD_BLOCKS]
};

// sum of a double over the workgroup in wavefront order; valid in thread 0
__device__ inline double mrf_block_sum_f64(double v, double *scratch)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    v = mrf_wave_sum_f64(v);
    if (lane == 0) scratch[wv] = v;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += scratch[w];
    __syncthreads();
    return t;
}

// grid (MRF_HEAD_BLOCKS, B): a thread per node of one image, grid-stride
__global__ void __launch_bounds__(256) mrf_energy_partial(const MrfEnergyParams P)
{
    __shared__ double scratch[4];
    const int b = blockIdx.y;
    const int H = P.g.H, W = P.g.W, L = P.g.L;
    const long long HW = (long long)H * W;
    double acc = 0.0;
    for (long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x; n < HW; n += (long long)gridDim.x * blockDim.x) {
        const int y = (int)(n / W), x = (int)(n - (long long)y * W);
        const long long i = (long long)b * HW + n;
        int xi = P.labels[i];
        xi = xi < L ? xi : L - 1;
        acc += (double)P.unary[(size_t)i * L + xi];
        for (int e = 0; e < P.n_edge_dir; ++e) {
            const int r = P.edge_dir[e];
            const int ys = y - P.g.dh[r], xs = x - P.g.dw[r];
            if (ys >= 0 && ys < H && xs >= 0 && xs < W) {
                int xj = P.labels[(long long)b * HW + (long long)ys * W + xs];
                xj = xj < L ? xj : L - 1;
                if (P.Te) {
                    // the edge's own table theta_{i-r,i}(x_{i-r}, x_i)
                    acc += (double)P.Te[(((size_t)r * P.g.N + i) * L + xj) * L + xi];
                } else {
                    const float wgt = P.w_mul ? P.w[(size_t)r * P.g.N + i] : P.w_scalar;
                    acc += (double)wgt * (double)P.V[(size_t)xj * L + xi];
                }
            }
        }
    }
    const double t = mrf_block_sum_f64(acc, scratch);
    if (threadIdx.x == 0) P.partial[(size_t)b * gridDim.x + blockIdx.x] = t;
}

// out[b] = scale * sum of partial[b][0..n) in index order; one workgroup per b.
// scale_from: if not NULL, scale = 1 / max(*scale_from, 1) (a count kept on the device)
__global__ void __launch_bounds__(64) mrf_sum_partials(const double *partial, int n, double *out, const long long *scale_from)
{
    const int b = blockIdx.x;
    double v = 0.0;
    for (int k = threadIdx.x; k < n; k += 64) v += partial[(size_t)b * n + k];
    v = mrf_wave_sum_f64(v);
    if (threadIdx.x == 0) {
        if (scale_from) {
            const long long c = *scale_from;
            v = v / (double)(c > 0 ? c : 1);
        }
        out[b] = v;
    }
}

// first 256 bytes of a sweep workspace: the scalar edge weight and the cleared fault word
__global__ void mrf_init_header(float *scalar, int *fault, float w)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { *scalar = w; *fault = 0; }
}

struct MrfLossParams {
    long long N;             // pixels
    int L;
    const float *cost;       // [N][L]
    const float *target;     // [N]
    const uint8_t *mask;     // [N] or NULL: non-zero = the pixel counts
    float *disparity;        // [N] or NULL
    float *grad_cost;        // [N][L] or NULL
    double *partial;         // [MRF_HEAD_BLOCKS] sums of |d - g|
    long long *count;        // number of counted pixels (written by mrf_count_mask, or N)
    long long *cpartial;     // [MRF_HEAD_BLOCKS]
    double beta;             // 0: standard L1; > 0: smooth L1 with this threshold
};

__global__ void mrf_set_i64(long long *dst, long long v)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = v;
}

__global__ void __launch_bounds__(256) mrf_count_mask_partial(const MrfLossParams P)
{
    __shared__ double scratch[4];
    double c = 0.0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < P.N; i += (long long)gridDim.x * blockDim.x)
        c += P.mask[i] != 0 ? 1.0 : 0.0;
    const double t = mrf_block_sum_f64(c, scratch);       // exact: integers below 2^53
    if (threadIdx.x == 0) P.cpartial[blockIdx.x] = (long long)t;
}

__global__ void __launch_bounds__(64) mrf_count_mask_final(const MrfLossParams P, int n)
{
    double v = 0.0;
    for (int k = threadIdx.x; k < n; k += 64) v += (double)P.cpartial[k];
    v = mrf_wave_sum_f64(v);
    if (threadIdx.x == 0) *P.count = (long long)v;
}

// One wavefront per pixel, lanes over labels (label = lane + 64 s).
//   f = exp(-(c - cmin)) / sum, d = sum_lambda lambda f(lambda),
//   d loss / d c(lambda) = sign(d - g) / n * (-f(lambda)) (lambda - d)
__global__ void __launch_bounds__(256) mrf_softmin_l1_kernel(const MrfLossParams P)
{
    __shared__ double scratch[4];
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long nwaves = (long long)gridDim.x * (blockDim.x >> 6);
    const int L = P.L;
    const long long cnt = *P.count;
    const double inv_n = 1.0 / (double)(cnt > 0 ? cnt : 1);
    double acc = 0.0;                    // this wavefront's sum of |d - g| (same value in every lane)
    for (long long i = wave; i < P.N; i += nwaves) {
        float c[4];
        float mn = INFINITY;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int lam = lane + 64 * s;
            c[s] = lam < L ? P.cost[(size_t)i * L + lam] : INFINITY;
            mn = fminf(mn, c[s]);
        }
        mn = mrf_wave_min(mn);
        double e[4], se = 0.0, sle = 0.0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int lam = lane + 64 * s;
            // (the exponential in single precision, about 1e-7 relative; the sums below in double)
            e[s] = lam < L ? (double)expf(mn - c[s]) : 0.0;
            se += e[s];
            sle += (double)lam * e[s];
        }
        se = mrf_wave_sum_f64(se);
        sle = mrf_wave_sum_f64(sle);
        const double d = sle / se;
        const double g = (double)P.target[i];
        const bool counts = P.mask ? P.mask[i] != 0 : true;
        const double diff = d - g;
        // per-pixel loss l(d - g) and its slope: |x| and sign(x), or for smooth L1 x^2 / (2 beta) and
        // x / beta inside |x| < beta, |x| - beta / 2 and sign(x) outside
        const bool small = P.beta > 0.0 && fabs(diff) < P.beta;
        if (counts) acc += small ? diff * diff / (2.0 * P.beta) : fabs(diff) - 0.5 * P.beta;
        if (lane == 0 && P.disparity) P.disparity[i] = (float)d;
        if (P.grad_cost) {
            const double sgn = counts ? (small ? diff / P.beta : (diff > 0.0 ? 1.0 : (diff < 0.0 ? -1.0 : 0.0))) : 0.0;
            const double k = sgn * inv_n / se;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int lam = lane + 64 * s;
                if (lam < L) P.grad_cost[(size_t)i * L + lam] = (float)(-k * e[s] * ((double)lam - d));
            }
        }
    }
    // acc is wave-uniform: add the wavefronts of the workgroup in order
    const int wv = threadIdx.x >> 6;
    if (lane == 0) scratch[wv] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += scratch[w];
        P.partial[blockIdx.x] = t;
    }
}
