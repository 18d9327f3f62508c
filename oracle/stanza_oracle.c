/*
 * CPU checker for the layer-separated training step: TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, definition-level C for every operation of one training iteration
 * with the CONV and FC layers trained on separate workers (paper: Sec. 3.2,
 * the training process with separated layers; update rule Eq. (1) of Sec. 2.1;
 * momentum SGD with weight decay per the experimental setup of Sec. 6.1).  The method reaches
 * exactly an ordinary mini-batch SGD step, so each function below is the plain
 * definition of its operation written as nested loops.  No blocking, no
 * vector intrinsics, no BLAS; OpenMP splits only the outermost independent loop.
 *
 * Storage type REAL is float (default) or double (-DREAL=double, used by the
 * finite-difference pins).  Every sum is accumulated in double and rounded once
 * on store.
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may use this
 * file.  It shares no code with the GPU library and is never a fallback for it.
 *
 * Layouts: activations NHWC, conv weights [K][R][S][C], FC weights [out][in].
 * Convolution is cross-correlation (no filter flip), zero padding, floor output
 * size.  Pool windows are clipped to the image (padding never wins the max);
 * the first maximum in row-major window order is the argmax; ReLU'(0) = 0.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif

typedef struct {
    int32_t N, H, W, C;      /* input batch, height, width, channels */
    int32_t K, R, S;         /* output channels, filter height, width */
    int32_t stride_h, stride_w, pad_h, pad_w;
} oconv_t;

typedef struct {
    int32_t N, H, W, C;
    int32_t win_h, win_w, stride_h, stride_w, pad_h, pad_w;
    int32_t relu;
} opool_t;

static inline int out_dim(int h, int win, int stride, int pad) { return (h + 2 * pad - win) / stride + 1; }

int oracle_real_bytes(void) { return (int)sizeof(REAL); }

/* number of OpenMP threads the loops below will use */
int oracle_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- convolution
 * Forward pass of a CONV layer (Sec. 3.1: each filter is slid over the input):
 *   Y[n,p,q,k] = b[k] + sum_{r,s,c} X[n, p*sh - ph + r, q*sw - pw + s, c] * Wt[k,r,s,c]
 * terms outside the image are zero; optional ReLU on store. */
void oracle_conv_fwd(const oconv_t *d, const REAL *x, const REAL *w, const REAL *bias, int relu, REAL *y)
{
    const int Ho = out_dim(d->H, d->R, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->S, d->stride_w, d->pad_w);
    const long rows = (long)d->N * Ho;
#pragma omp parallel for schedule(static)
    for (long np = 0; np < rows; ++np) {
        const int n = (int)(np / Ho), p = (int)(np % Ho);
        for (int q = 0; q < Wo; ++q)
            for (int k = 0; k < d->K; ++k) {
                double acc = bias ? (double)bias[k] : 0.0;
                for (int r = 0; r < d->R; ++r) {
                    const int h = p * d->stride_h - d->pad_h + r;
                    if (h < 0 || h >= d->H) continue;
                    for (int s = 0; s < d->S; ++s) {
                        const int ww = q * d->stride_w - d->pad_w + s;
                        if (ww < 0 || ww >= d->W) continue;
                        const REAL *xp = x + (((size_t)n * d->H + h) * d->W + ww) * d->C;
                        const REAL *wp = w + (((size_t)k * d->R + r) * d->S + s) * d->C;
                        for (int c = 0; c < d->C; ++c) acc += (double)xp[c] * (double)wp[c];
                    }
                }
                if (relu && acc < 0.0) acc = 0.0;
                y[(((size_t)n * Ho + p) * Wo + q) * d->K + k] = (REAL)acc;
            }
    }
}

/* One forward output element, for sampled checks on tensors too large to do whole. */
double oracle_conv_fwd_at(const oconv_t *d, const REAL *x, const REAL *w, const REAL *bias, int relu,
                          int n, int p, int q, int k)
{
    double acc = bias ? (double)bias[k] : 0.0;
    for (int r = 0; r < d->R; ++r) {
        const int h = p * d->stride_h - d->pad_h + r;
        if (h < 0 || h >= d->H) continue;
        for (int s = 0; s < d->S; ++s) {
            const int ww = q * d->stride_w - d->pad_w + s;
            if (ww < 0 || ww >= d->W) continue;
            const REAL *xp = x + (((size_t)n * d->H + h) * d->W + ww) * d->C;
            const REAL *wp = w + (((size_t)k * d->R + r) * d->S + s) * d->C;
            for (int c = 0; c < d->C; ++c) acc += (double)xp[c] * (double)wp[c];
        }
    }
    if (relu && acc < 0.0) acc = 0.0;
    return acc;
}

/* Gradient of the loss w.r.t. the layer input (backpropagation through a CONV layer,
 * Sec. 3.2): dX[n,h,w,c] = sum over (k,r,s) with p*sh - ph + r == h, q*sw - pw + s == w
 * of dY[n,p,q,k] * Wt[k,r,s,c]. */
static double bwd_data_at(const oconv_t *d, const REAL *dy, const REAL *w, int Ho, int Wo, int n, int h, int ww, int c)
{
    double acc = 0.0;
    for (int r = 0; r < d->R; ++r) {
        const int hp = h + d->pad_h - r;
        if (hp < 0 || hp % d->stride_h) continue;
        const int p = hp / d->stride_h;
        if (p >= Ho) continue;
        for (int s = 0; s < d->S; ++s) {
            const int wq = ww + d->pad_w - s;
            if (wq < 0 || wq % d->stride_w) continue;
            const int q = wq / d->stride_w;
            if (q >= Wo) continue;
            const REAL *dyp = dy + (((size_t)n * Ho + p) * Wo + q) * d->K;
            for (int k = 0; k < d->K; ++k)
                acc += (double)dyp[k] * (double)w[(((size_t)k * d->R + r) * d->S + s) * d->C + c];
        }
    }
    return acc;
}

void oracle_conv_bwd_data(const oconv_t *d, const REAL *dy, const REAL *w, REAL *dx)
{
    const int Ho = out_dim(d->H, d->R, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->S, d->stride_w, d->pad_w);
    const long rows = (long)d->N * d->H;
#pragma omp parallel for schedule(static)
    for (long nh = 0; nh < rows; ++nh) {
        const int n = (int)(nh / d->H), h = (int)(nh % d->H);
        for (int ww = 0; ww < d->W; ++ww)
            for (int c = 0; c < d->C; ++c)
                dx[(((size_t)n * d->H + h) * d->W + ww) * d->C + c] = (REAL)bwd_data_at(d, dy, w, Ho, Wo, n, h, ww, c);
    }
}

double oracle_conv_bwd_data_at(const oconv_t *d, const REAL *dy, const REAL *w, int n, int h, int ww, int c)
{
    const int Ho = out_dim(d->H, d->R, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->S, d->stride_w, d->pad_w);
    return bwd_data_at(d, dy, w, Ho, Wo, n, h, ww, c);
}

/* Gradient w.r.t. the filter and the bias (the conv gradients of Sec. 3.2; part of T_c in Sec. 4.2.1):
 *   dW[k,r,s,c] = sum_{n,p,q} dY[n,p,q,k] * X[n, p*sh - ph + r, q*sw - pw + s, c]
 *   db[k]       = sum_{n,p,q} dY[n,p,q,k] */
static double bwd_weight_at(const oconv_t *d, const REAL *x, const REAL *dy, int Ho, int Wo, int k, int r, int s, int c)
{
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n)
        for (int p = 0; p < Ho; ++p) {
            const int h = p * d->stride_h - d->pad_h + r;
            if (h < 0 || h >= d->H) continue;
            for (int q = 0; q < Wo; ++q) {
                const int ww = q * d->stride_w - d->pad_w + s;
                if (ww < 0 || ww >= d->W) continue;
                acc += (double)dy[(((size_t)n * Ho + p) * Wo + q) * d->K + k] *
                       (double)x[(((size_t)n * d->H + h) * d->W + ww) * d->C + c];
            }
        }
    return acc;
}

void oracle_conv_bwd_weight(const oconv_t *d, const REAL *x, const REAL *dy, REAL *dw, REAL *dbias)
{
    const int Ho = out_dim(d->H, d->R, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->S, d->stride_w, d->pad_w);
    const long taps = (long)d->K * d->R * d->S;
#pragma omp parallel for schedule(dynamic, 1)
    for (long krs = 0; krs < taps; ++krs) {
        const int k = (int)(krs / (d->R * d->S)), r = (int)((krs / d->S) % d->R), s = (int)(krs % d->S);
        for (int c = 0; c < d->C; ++c)
            dw[(size_t)krs * d->C + c] = (REAL)bwd_weight_at(d, x, dy, Ho, Wo, k, r, s, c);
    }
    if (dbias) {
        const size_t M = (size_t)d->N * Ho * Wo;
#pragma omp parallel for schedule(static)
        for (int k = 0; k < d->K; ++k) {
            double acc = 0.0;
            for (size_t m = 0; m < M; ++m) acc += (double)dy[m * d->K + k];
            dbias[k] = (REAL)acc;
        }
    }
}

double oracle_conv_bwd_weight_at(const oconv_t *d, const REAL *x, const REAL *dy, int k, int r, int s, int c)
{
    const int Ho = out_dim(d->H, d->R, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->S, d->stride_w, d->pad_w);
    return bwd_weight_at(d, x, dy, Ho, Wo, k, r, s, c);
}

double oracle_colsum_at(const REAL *a, size_t rows, size_t cols, size_t j)
{
    double acc = 0.0;
    for (size_t i = 0; i < rows; ++i) acc += (double)a[i * cols + j];
    return acc;
}

/* Backward of an element-wise ReLU whose output was y: dz = dy where y > 0, else 0. */
void oracle_relu_bwd(size_t numel, const REAL *dy, const REAL *y, REAL *dz)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < numel; ++i) dz[i] = y[i] > (REAL)0 ? dy[i] : (REAL)0;
}

/* ------------------------------------------------------------------ max-pool
 * The pooling layer that follows the last CONV layer stays on the CONV worker
 * (Sec. 3.2, note on the split point); it has no parameters (Fig. 3 caption).
 *   P[n,p,q,c] = max over the window (clipped to the image), then max(.,0) if relu;
 *   argmax = i*win_w + j of the first maximum in row-major (i,j) order. */
void oracle_pool_relu_fwd(const opool_t *d, const REAL *x, REAL *y, uint8_t *argmax)
{
    const int Ho = out_dim(d->H, d->win_h, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->win_w, d->stride_w, d->pad_w);
    const long rows = (long)d->N * Ho;
#pragma omp parallel for schedule(static)
    for (long np = 0; np < rows; ++np) {
        const int n = (int)(np / Ho), p = (int)(np % Ho);
        for (int q = 0; q < Wo; ++q)
            for (int c = 0; c < d->C; ++c) {
                int found = 0, best_idx = 0;
                REAL best = 0;
                for (int i = 0; i < d->win_h; ++i) {
                    const int h = p * d->stride_h - d->pad_h + i;
                    if (h < 0 || h >= d->H) continue;
                    for (int j = 0; j < d->win_w; ++j) {
                        const int ww = q * d->stride_w - d->pad_w + j;
                        if (ww < 0 || ww >= d->W) continue;
                        const REAL v = x[(((size_t)n * d->H + h) * d->W + ww) * d->C + c];
                        if (!found || v > best) { best = v; best_idx = i * d->win_w + j; found = 1; }
                    }
                }
                const size_t o = (((size_t)n * Ho + p) * Wo + q) * d->C + c;
                y[o] = (d->relu && best < (REAL)0) ? (REAL)0 : best;
                if (argmax) argmax[o] = (uint8_t)best_idx;
            }
    }
}

/* dX[n,h,w,c] = sum over the windows (p,q) covering (h,w) whose argmax is (h,w)
 * of dP[n,p,q,c], gated by P > 0 when the ReLU was fused. */
void oracle_pool_relu_bwd(const opool_t *d, const REAL *dy, const REAL *y, const uint8_t *argmax, REAL *dx)
{
    const int Ho = out_dim(d->H, d->win_h, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->win_w, d->stride_w, d->pad_w);
    const long rows = (long)d->N * d->H;
#pragma omp parallel for schedule(static)
    for (long nh = 0; nh < rows; ++nh) {
        const int n = (int)(nh / d->H), h = (int)(nh % d->H);
        for (int ww = 0; ww < d->W; ++ww)
            for (int c = 0; c < d->C; ++c) {
                double acc = 0.0;
                for (int i = 0; i < d->win_h; ++i) {
                    const int hp = h + d->pad_h - i;
                    if (hp < 0 || hp % d->stride_h) continue;
                    const int p = hp / d->stride_h;
                    if (p >= Ho) continue;
                    for (int j = 0; j < d->win_w; ++j) {
                        const int wq = ww + d->pad_w - j;
                        if (wq < 0 || wq % d->stride_w) continue;
                        const int q = wq / d->stride_w;
                        if (q >= Wo) continue;
                        const size_t o = (((size_t)n * Ho + p) * Wo + q) * d->C + c;
                        if (argmax[o] != (uint8_t)(i * d->win_w + j)) continue;
                        if (d->relu && !(y[o] > (REAL)0)) continue;
                        acc += (double)dy[o];
                    }
                }
                dx[(((size_t)n * d->H + h) * d->W + ww) * d->C + c] = (REAL)acc;
            }
    }
}

/* ------------------------------------------- residual add and global average
 * (needed by the residual-network-shaped workload only; plain definitions) */
void oracle_add_relu_fwd(size_t numel, const REAL *a, const REAL *b, REAL *o)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < numel; ++i) {
        const double s = (double)a[i] + (double)b[i];
        o[i] = (REAL)(s > 0.0 ? s : 0.0);
    }
}

void oracle_gap_fwd(int N, int HW, int C, const REAL *x, REAL *f)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int i = 0; i < HW; ++i) acc += (double)x[((size_t)n * HW + i) * C + c];
            f[(size_t)n * C + c] = (REAL)(acc / (double)HW);
        }
}

void oracle_gap_bwd(int N, int HW, int C, const REAL *df, REAL *dx)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i)
            for (int c = 0; c < C; ++c)
                dx[((size_t)n * HW + i) * C + c] = (REAL)((double)df[(size_t)n * C + c] / (double)HW);
}

/* ------------------------------------------------------------------ FC layers
 * Every output unit of an FC layer reads every output of the layer before it
 * (Sec. 3.1):  Z[i,o] = b[o] + sum_j A[i,j] * Wt[o,j], optional ReLU. */
void oracle_fc_fwd(int n, int in, int out, const REAL *a, const REAL *w, const REAL *b, int relu, REAL *z)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (int o = 0; o < out; ++o) {
            double acc = b ? (double)b[o] : 0.0;
            for (int j = 0; j < in; ++j) acc += (double)a[(size_t)i * in + j] * (double)w[(size_t)o * in + j];
            if (relu && acc < 0.0) acc = 0.0;
            z[(size_t)i * out + o] = (REAL)acc;
        }
}

double oracle_fc_fwd_at(int in, const REAL *a_row, const REAL *w_row, const REAL *b, int o, int relu)
{
    double acc = b ? (double)b[o] : 0.0;
    for (int j = 0; j < in; ++j) acc += (double)a_row[j] * (double)w_row[j];
    return (relu && acc < 0.0) ? 0.0 : acc;
}

/* dW[o,j] = sum_i dZ[i,o] A[i,j];  db[o] = sum_i dZ[i,o];  dA[i,j] = sum_o dZ[i,o] Wt[o,j] */
void oracle_fc_bwd(int n, int in, int out, const REAL *a, const REAL *w, const REAL *dz,
                   REAL *dw, REAL *db, REAL *da)
{
#pragma omp parallel for schedule(static)
    for (int o = 0; o < out; ++o) {
        double sb = 0.0;
        for (int i = 0; i < n; ++i) sb += (double)dz[(size_t)i * out + o];
        db[o] = (REAL)sb;
        for (int j = 0; j < in; ++j) {
            double acc = 0.0;
            for (int i = 0; i < n; ++i) acc += (double)dz[(size_t)i * out + o] * (double)a[(size_t)i * in + j];
            dw[(size_t)o * in + j] = (REAL)acc;
        }
    }
    if (da) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < in; ++j) {
                double acc = 0.0;
                for (int o = 0; o < out; ++o) acc += (double)dz[(size_t)i * out + o] * (double)w[(size_t)o * in + j];
                da[(size_t)i * in + j] = (REAL)acc;
            }
    }
}

/* ------------------------------------------------------------- softmax + loss
 * The FC stack ends in a softmax classifier (Sec. 3.1); the loss is the mean
 * cross-entropy over the n samples of the global batch, which is what puts the
 * 1/n of Eq. (1) into every gradient:
 *   loss = (1/n) sum_i [ log sum_j exp(z_ij) - z_i[y_i] ]
 *   dZ_ij = (softmax(z_i)_j - [j == y_i]) / n ;  pred_i = lowest index of the row max. */
double oracle_softmax_ce(int n, int classes, const REAL *z, const int32_t *labels, REAL *dz, int32_t *pred)
{
    double total = 0.0;
    for (int i = 0; i < n; ++i) {
        const REAL *zi = z + (size_t)i * classes;
        int arg = 0;
        for (int j = 1; j < classes; ++j)
            if (zi[j] > zi[arg]) arg = j;
        const double zmax = (double)zi[arg];
        double denom = 0.0;
        for (int j = 0; j < classes; ++j) denom += exp((double)zi[j] - zmax);
        total += log(denom) + zmax - (double)zi[labels[i]];
        if (dz)
            for (int j = 0; j < classes; ++j) {
                const double sm = exp((double)zi[j] - zmax) / denom;
                dz[(size_t)i * classes + j] = (REAL)((sm - (j == labels[i] ? 1.0 : 0.0)) / (double)n);
            }
        if (pred) pred[i] = arg;
    }
    return total / (double)n;
}

/* One of several FC workers (Sec. 4.1.3: each FC worker serves an equal share of
 * the CONV workers and keeps a complete set of FC layers; their gradients are
 * all-reduced afterwards).  The loss is still the mean over the GLOBAL batch of
 * Eq. (1), so a worker that holds n_local of the n_global rows contributes
 *   loss_part = (1/n_global) sum_{local i} [ log sum_j exp(z_ij) - z_i[y_i] ]
 *   dZ_ij     = (softmax(z_i)_j - [j == y_i]) / n_global
 * and the parts add up to the single-worker quantities. */
double oracle_softmax_ce_part(int n_local, int n_global, int classes, const REAL *z, const int32_t *labels, REAL *dz,
                              int32_t *pred)
{
    double total = 0.0;
    for (int i = 0; i < n_local; ++i) {
        const REAL *zi = z + (size_t)i * classes;
        int arg = 0;
        for (int j = 1; j < classes; ++j)
            if (zi[j] > zi[arg]) arg = j;
        const double zmax = (double)zi[arg];
        double denom = 0.0;
        for (int j = 0; j < classes; ++j) denom += exp((double)zi[j] - zmax);
        total += log(denom) + zmax - (double)zi[labels[i]];
        if (dz)
            for (int j = 0; j < classes; ++j) {
                const double sm = exp((double)zi[j] - zmax) / denom;
                dz[(size_t)i * classes + j] = (REAL)((sm - (j == labels[i] ? 1.0 : 0.0)) / (double)n_global);
            }
        if (pred) pred[i] = arg;
    }
    return total / (double)n_global;
}

/* -------------------------------------------------------------- average pool
 * The pooling branch of the Inception blocks (the paper trains Inception-V3, Sec. 6.1,
 * without describing its layers): the mean over the part of the window that lies inside
 * the image (padding is not counted), and its transpose for the backward pass:
 *   y[n,p,q,c]  = (1/cnt(p,q)) sum over valid (i,j) of x[n, p*s-pad+i, q*s-pad+j, c]
 *   dx[n,h,w,c] = sum over windows (p,q) containing (h,w) of dy[n,p,q,c] / cnt(p,q) */
void oracle_avgpool_fwd(const opool_t *d, const REAL *x, REAL *y)
{
    const int Ho = out_dim(d->H, d->win_h, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->win_w, d->stride_w, d->pad_w);
#pragma omp parallel for schedule(static)
    for (int np = 0; np < d->N * Ho; ++np) {
        const int n = np / Ho, p = np % Ho;
        for (int q = 0; q < Wo; ++q)
            for (int c = 0; c < d->C; ++c) {
                double s = 0.0;
                int cnt = 0;
                for (int i = 0; i < d->win_h; ++i)
                    for (int j = 0; j < d->win_w; ++j) {
                        const int h = p * d->stride_h - d->pad_h + i, w = q * d->stride_w - d->pad_w + j;
                        if (h < 0 || h >= d->H || w < 0 || w >= d->W) continue;
                        s += (double)x[(((size_t)n * d->H + h) * d->W + w) * d->C + c];
                        ++cnt;
                    }
                y[(((size_t)n * Ho + p) * Wo + q) * d->C + c] = (REAL)(s / (double)cnt);
            }
    }
}

void oracle_avgpool_bwd(const opool_t *d, const REAL *dy, REAL *dx)
{
    const int Ho = out_dim(d->H, d->win_h, d->stride_h, d->pad_h), Wo = out_dim(d->W, d->win_w, d->stride_w, d->pad_w);
#pragma omp parallel for schedule(static)
    for (int nh = 0; nh < d->N * d->H; ++nh) {
        const int n = nh / d->H, h = nh % d->H;
        for (int w = 0; w < d->W; ++w)
            for (int c = 0; c < d->C; ++c) {
                double s = 0.0;
                for (int p = 0; p < Ho; ++p)
                    for (int q = 0; q < Wo; ++q) {
                        const int h0 = p * d->stride_h - d->pad_h, w0 = q * d->stride_w - d->pad_w;
                        if (h < h0 || h >= h0 + d->win_h || w < w0 || w >= w0 + d->win_w) continue;
                        int cnt = 0;   /* valid elements of window (p,q) */
                        for (int i = 0; i < d->win_h; ++i)
                            for (int j = 0; j < d->win_w; ++j)
                                if (h0 + i >= 0 && h0 + i < d->H && w0 + j >= 0 && w0 + j < d->W) ++cnt;
                        s += (double)dy[(((size_t)n * Ho + p) * Wo + q) * d->C + c] / (double)cnt;
                    }
                dx[(((size_t)n * d->H + h) * d->W + w) * d->C + c] = (REAL)s;
            }
    }
}

/* -------------------------------------------------------------- batch normalisation
 * The residual networks of the paper's table of models (Sec. 6.1) carry a
 * normalisation layer after every convolution; the paper never discusses it, so the
 * transform is taken as published (training mode): over the M = N*H*W rows of an
 * NHWC tensor viewed as [M][C], per channel c
 *   mean_c = (1/M) sum_m x[m,c]          var_c = (1/M) sum_m (x[m,c] - mean_c)^2   (biased)
 *   istd_c = 1 / sqrt(var_c + eps)       xhat  = (x - mean_c) * istd_c
 *   y[m,c] = gamma_c * xhat[m,c] + beta_c,  then max(.,0) if relu
 * Each CONV worker normalises over its OWN batch (no exchange of statistics between
 * workers); running averages, when given, move by
 *   run_mean <- (1-mom) run_mean + mom mean,   run_var <- (1-mom) run_var + mom var M/(M-1). */
void oracle_bn_fwd(size_t rows, int C, const REAL *x, const REAL *gamma, const REAL *beta, double eps, int relu,
                   REAL *y, REAL *mean_out, REAL *istd_out, REAL *run_mean, REAL *run_var, double mom)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (size_t m = 0; m < rows; ++m) s += (double)x[m * C + c];
        const double mean = s / (double)rows;
        double q = 0.0;
        for (size_t m = 0; m < rows; ++m) {
            const double d = (double)x[m * C + c] - mean;
            q += d * d;
        }
        const double var = q / (double)rows;
        const double istd = 1.0 / sqrt(var + eps);
        for (size_t m = 0; m < rows; ++m) {
            double v = (double)gamma[c] * (((double)x[m * C + c] - mean) * istd) + (double)beta[c];
            if (relu && v < 0.0) v = 0.0;
            y[m * C + c] = (REAL)v;
        }
        if (mean_out) mean_out[c] = (REAL)mean;
        if (istd_out) istd_out[c] = (REAL)istd;
        if (run_mean) run_mean[c] = (REAL)((1.0 - mom) * (double)run_mean[c] + mom * mean);
        if (run_var) run_var[c] = (REAL)((1.0 - mom) * (double)run_var[c] + mom * (rows > 1 ? q / (double)(rows - 1) : var));
    }
}

/* Backward of the transform above for the gradient dy of its (pre-ReLU) output; a fused
 * ReLU is undone by the caller with oracle_relu_bwd first.  With xhat as above:
 *   dbeta_c = sum_m dy[m,c]     dgamma_c = sum_m dy[m,c] xhat[m,c]
 *   dx[m,c] = gamma_c istd_c ( dy[m,c] - dbeta_c / M - xhat[m,c] dgamma_c / M )
 * (the mean and the variance both depend on every x of the channel). */
void oracle_bn_bwd(size_t rows, int C, const REAL *x, const REAL *dy, const REAL *gamma, const REAL *mean, const REAL *istd,
                   REAL *dx, REAL *dgamma, REAL *dbeta)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        const double mu = (double)mean[c], is = (double)istd[c];
        double sb = 0.0, sg = 0.0;
        for (size_t m = 0; m < rows; ++m) {
            const double g = (double)dy[m * C + c];
            sb += g;
            sg += g * (((double)x[m * C + c] - mu) * is);
        }
        for (size_t m = 0; m < rows; ++m) {
            const double xh = ((double)x[m * C + c] - mu) * is;
            dx[m * C + c] = (REAL)((double)gamma[c] * is * ((double)dy[m * C + c] - sb / (double)rows - xh * sg / (double)rows));
        }
        dgamma[c] = (REAL)sg;
        dbeta[c] = (REAL)sb;
    }
}

/* -------------------------------------------------------------- optimiser
 * Momentum SGD with weight decay (Sec. 6.1), in the form of the software stack
 * the paper ran:  g' = g + wd*w ;  v <- m*v + g' ;  w <- w - lr*v. */
void oracle_sgd_momentum(size_t numel, REAL *w, REAL *v, const REAL *g, double lr, double momentum, double wd)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < numel; ++i) {
        const double gi = (double)g[i] + wd * (double)w[i];
        const double vi = momentum * (double)v[i] + gi;
        v[i] = (REAL)vi;
        w[i] = (REAL)((double)w[i] - lr * vi);
    }
}

/* Server-side aggregation (Sec. 2.2: servers aggregate the gradients from all
 * workers and perform the global update; Sec. 3.2: CONV workers exchange their
 * gradients to obtain the sum over all samples of the batch):
 *   g = scale * sum_{k<K} g_k, accumulated in shard order, then the update above. */
void oracle_ps_aggregate(size_t numel, REAL *w, REAL *v, const REAL *const *grads, int K,
                         double scale, double lr, double momentum, double wd)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < numel; ++i) {
        double s = 0.0;
        for (int k = 0; k < K; ++k) s += (double)grads[k][i];
        const double gi = scale * s + wd * (double)w[i];
        const double vi = momentum * (double)v[i] + gi;
        v[i] = (REAL)vi;
        w[i] = (REAL)((double)w[i] - lr * vi);
    }
}
