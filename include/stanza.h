/*
 * stanza.h — C ABI of the MI355X (gfx950) library for one GPU's share of a training
 * iteration with the CONV and FC layers trained on separate workers.
 *
 * The calls follow the paper's training process with layer separation (Sec. 3.2 and
 * Fig. 5): a CONV worker runs its conv stack forward (stanza_conv_fwd, stanza_pool_relu_fwd)
 * and hands the activations after the last pooling layer to the FC worker
 * ("push_activation" in the API table of Sec. 5); the FC worker runs stanza_fc_step over
 * the row-concatenated activations of all K workers, returns the gradient of those
 * activations ("pull_fc") and updates the FC parameters; every CONV worker continues
 * backpropagation (stanza_pool_relu_bwd, stanza_conv_bwd_weight, stanza_conv_bwd_data);
 * the K workers' conv gradients are summed and applied by stanza_ps_aggregate
 * ("pull_grad" plus the optimiser step; over the whole model it is the server-side
 * aggregation of the parameter-server iteration of Sec. 2.2).
 *
 * Conventions, valid for every entry point unless it says otherwise
 *   - Pointers are DEVICE pointers unless the name starts with host_; descriptor structs
 *     are read on the host during the call and may be freed after it returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue kernel launches and return: nothing synchronises, nothing is copied by the runtime, so every
 *     call may be recorded in a stream capture.  Scalar results stay in device memory.
 *   - The caller owns every buffer, workspace included.  The library allocates no memory, on
 *     the device or the host, and keeps no state between calls.
 *   - Layouts: activations NHWC ([N][H][W][C], C fastest); conv weights [K][R][S][C];
 *     FC weights [out][in]; features [n][A] with A the NHWC flattening (h*W + w)*C + c of
 *     the last pooled map, worker k owning rows k*B .. (k+1)*B-1.
 *   - Convolution is cross-correlation with zero padding and floor output size
 *     Ho = (H + 2*pad_h - R)/stride_h + 1.  Pool windows are clipped to the image.
 *   - Element type: float32 everywhere for STANZA_F32.  For STANZA_BF16 the tensors x, w, y,
 *     dy, dx of the conv calls are bfloat16 (products accumulate in float32); bias, dw, dbias
 *     and everything in fc_step / ps_aggregate stay float32.
 *   - Every tensor must have fewer than 2^31 elements and a 16-byte aligned base pointer.  float32 tensors of 2 GiB and more
 *     are gathered element by element (correct, slower); the bfloat16 conv calls refuse them (STANZA_EUNSUPPORTED).
 *   - Return value: STANZA_OK (0) or a negative stanza_status.  Errors are decided before
 *     any launch (nothing has been written) except STANZA_EHIP, which reports a launch
 *     failure.  No C++ exception crosses this boundary.
 *   - Not checkable on the host and therefore preconditions: labels in [0, classes), finite
 *     inputs, no aliasing between inputs and outputs other than the documented in-place
 *     parameters.
 */
#ifndef STANZA_H
#define STANZA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    STANZA_OK = 0,
    STANZA_EINVAL = -1,       /* a size, stride, pad or count is out of range */
    STANZA_ENULL = -2,        /* a required pointer is NULL */
    STANZA_EALIGN = -3,       /* a pointer is not 16-byte aligned */
    STANZA_EUNSUPPORTED = -4, /* dtype / shape combination this build has no kernel for */
    STANZA_EWORKSPACE = -5,   /* ws_bytes is smaller than the matching *_workspace_bytes() */
    STANZA_EHIP = -6,         /* the HIP runtime reported an error at launch */
    STANZA_ECAPACITY = -7     /* the input is larger than the fixed capacity of an entry point that allocates nothing */
} stanza_status;

typedef enum { STANZA_F32 = 0, STANZA_BF16 = 1 } stanza_dtype;

enum {
    STANZA_CONV_BIAS = 1u,   /* fwd: add bias[k];  bwd_weight: also produce dbias */
    STANZA_CONV_RELU = 2u,   /* fwd: y = max(y, 0);  bwd_*: dy is gated by [y > 0] when y is given */
    STANZA_CONV_ACCUM = 4u,  /* bwd_data: dx += result instead of dx = result (residual joins) */
    STANZA_CONV_NINE_TAP = 8u /* bwd_weight (and its workspace query), float32 3x3 stride-1 pad-1 layers: take the kernel that keeps all */
                             /* nine taps in one workgroup wherever it can run, also where the library would choose the implicit GEMM */
                             /* (small or odd-sized images); same result up to summation order.  Ignored elsewhere. */
};
enum { STANZA_POOL_RELU = 1u };

/* One CONV layer (Sec. 3.1).  x: [N][H][W][C], w: [K][R][S][C], y: [N][Ho][Wo][K]. */
typedef struct {
    int32_t N, H, W, C;
    int32_t K, R, S;
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t dtype;           /* stanza_dtype */
    uint32_t flags;          /* STANZA_CONV_* */
} stanza_conv_desc;

/* Max-pool window over x: [N][H][W][C] -> y: [N][Ho][Wo][C]; requires pad < win, win_h*win_w <= 255. */
typedef struct {
    int32_t N, H, W, C;
    int32_t win_h, win_w, stride_h, stride_w, pad_h, pad_w;
    uint32_t flags;          /* STANZA_POOL_RELU: y = max(pool, 0), backward gated by [y > 0] */
} stanza_pool_desc;

/* The FC worker's stack: host_dims = {A, hidden_1, ..., classes} (n_layers + 1 entries), ReLU
 * between layers and none after the last; n_samples = K*B rows of features. */
typedef struct {
    int32_t n_layers;
    const int32_t *host_dims;
    int32_t n_samples;
    float lr, momentum, weight_decay;
    float dropout_p;          /* 0: none; otherwise every hidden layer's ReLU output passes through stanza_dropout with */
    uint64_t dropout_seed;    /* this seed and stream_id = (dropout_step << 8) | index of the layer (0-based), so that */
    uint64_t dropout_step;    /* layers and iterations draw different masks; dropout_step < 2^56 */
    int32_t compute_dtype;    /* STANZA_F32, or STANZA_BF16: the hidden layers' GEMMs read bfloat16 copies of the features, */
                              /* activations, gradients and weights (products accumulate in float32); the last layer, the */
                              /* loss, all parameters, momentum buffers, gradients written out and dfeats stay float32. */
                              /* Needs every width but the last to be a multiple of 8.  Dropout then acts on the bfloat16 */
                              /* activations: same masks, kept units scaled in float32 and rounded once. */
} stanza_fc_desc;

const char *stanza_strerror(int status);
int stanza_version(void);

/* ---- CONV worker: forward pass of one layer of its conv stack (Sec. 3.1, Sec. 3.2)
 *   y[n,p,q,k] = bias[k] + sum_{r,s,c} x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c] * w[k,r,s,c]
 * followed by max(.,0) with STANZA_CONV_RELU.  bias (float32 [K]) is required iff STANZA_CONV_BIAS.
 * which: 0 forward, 1 backward-data, 2 backward-weight.  For forward and backward-data the workspace is OPTIONAL:
 * with ws == NULL (or fewer bytes than stanza_conv_workspace_bytes reports) every output tile is computed by one
 * workgroup; with it, the tiles of the last, partly filled round of workgroups (all tiles when there are few) are cut
 * into reduction slices that are added in a fixed order by a second kernel, so that all compute units finish together.
 * Results are run-to-run identical either way; the two ways differ in the last bits (summation order). */
size_t stanza_conv_workspace_bytes(const stanza_conv_desc *desc, int which);
int stanza_conv_fwd(const stanza_conv_desc *desc, const void *x, const void *w, const float *bias,
                    void *y, void *ws, size_t ws_bytes, void *stream);
/* The same with a residual join in the epilogue (the residual networks of the paper's table of models, Sec. 6.1; the join itself
 * is not described there: the published one):  y = conv(x, w) + bias + res, then max(.,0) with STANZA_CONV_RELU, i.e. the
 * convolution followed by stanza_add_relu_fwd without the intermediate tensor.  res: [N,Ho,Wo,K] of the dtype of y, 16-byte
 * aligned, must not overlap y; required (NULL is STANZA_ENULL).  The backward pass of the join is stanza_add_relu_bwd on y as
 * before; the convolution's own backward calls then take that gradient ungated. */
int stanza_conv_fwd_res(const stanza_conv_desc *desc, const void *x, const void *w, const float *bias, const void *res,
                        void *y, void *ws, size_t ws_bytes, void *stream);

/* ---- CONV worker: backpropagation to the layer input, run once the FC worker has handed back the gradient of the
 * worker's activations (Sec. 3.2):
 *   dx[n,h,w,c] = sum_{k,r,s} g[n,(h+pad_h-r)/stride_h,(w+pad_w-s)/stride_w,k] * w[k,r,s,c]
 * over the taps where both divisions are exact and in range, with g = dy, or dy*[y>0] when
 * STANZA_CONV_RELU is set and y (the forward output) is not NULL.
 * x_mask (optional, same shape as dx): the result is multiplied by [x_mask > 0] on store, which is the
 * backward of the ReLU that produced this layer's input.  STANZA_CONV_ACCUM adds the result to the
 * existing dx before masking. */
int stanza_conv_bwd_data(const stanza_conv_desc *desc, const void *dy, const void *y, const void *w,
                         const void *x_mask, void *dx, void *ws, size_t ws_bytes, void *stream);

/* ---- CONV worker: filter and bias gradients (part of the conv compute time T_c of Sec. 4.2.1)
 *   dw[k,r,s,c] = sum_{n,p,q} g[n,p,q,k] * x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c]
 *   dbias[k]    = sum_{n,p,q} g[n,p,q,k]           (written iff STANZA_CONV_BIAS; then dbias != NULL)
 * g as above.  dw, dbias are float32 and overwritten.  The long reduction is split over workgroups
 * and the partial sums are added in a fixed order (results are run-to-run identical); ws must hold
 * stanza_conv_workspace_bytes(desc, 2) bytes. */
int stanza_conv_bwd_weight(const stanza_conv_desc *desc, const void *x, const void *dy, const void *y,
                           float *dw, float *dbias, void *ws, size_t ws_bytes, void *stream);

/* ---- Max-pool (+ReLU), kept on the CONV worker so that fewer activations cross to the FC worker
 * (Sec. 3.2, note on the split point).
 *   y[n,p,q,c] = max over the clipped window of x, then max(.,0) with STANZA_POOL_RELU
 *   argmax[n,p,q,c] = i*win_w + j of the first maximum in row-major window order (uint8)
 * backward: dx[n,h,w,c] = sum of dy over the windows whose argmax is (h,w), gated by [y > 0] with
 * STANZA_POOL_RELU.  dtype: STANZA_F32 or STANZA_BF16 for x, y, dy, dx. */
int stanza_pool_relu_fwd(const stanza_pool_desc *desc, int32_t dtype, const void *x, void *y, uint8_t *argmax, void *stream);
int stanza_pool_relu_bwd(const stanza_pool_desc *desc, int32_t dtype, const void *dy, const void *y,
                         const uint8_t *argmax, void *dx, void *stream);

/* ---- Residual join and global average pool of the residual-network-shaped workload (the paper trains
 * such a network, Sec. 6.1 table of models, without describing these layers: plain definitions).
 *   add_relu_fwd: o = max(a + b, 0);  add_relu_bwd: dz = dout * [o > 0] (the gradient of both a and b)
 *   gap_fwd: f[n,c] = mean_{h,w} x[n,h,w,c];  gap_bwd: dx[n,h,w,c] = df[n,c] / (H*W)
 * dtype: STANZA_F32, or STANZA_BF16 for a, b, o, dout, dz (numel % 8 == 0) and for x / dx of the global average pool
 * (f and df, the features handed to the FC worker and their gradient, are always float32). */
int stanza_add_relu_fwd(int64_t numel, int32_t dtype, const void *a, const void *b, void *o, void *stream);
int stanza_add_relu_bwd(int64_t numel, int32_t dtype, const void *dout, const void *o, void *dz, void *stream);
int stanza_gap_fwd(int32_t N, int32_t HW, int32_t C, int32_t dtype, const void *x, float *f, void *stream);
int stanza_gap_bwd(int32_t N, int32_t HW, int32_t C, int32_t dtype, const float *df, void *dx, void *stream);

/* ---- Average-pool branch and channel concatenation of the Inception blocks (the paper trains Inception-V3, Sec. 6.1,
 * without describing its layers: plain definitions).  The average pool takes dtype = STANZA_F32 or STANZA_BF16 (then
 * C % 8 == 0; sums in float32, one rounding at the store); the copy moves 4-byte elements, so a bfloat16 tensor is copied as
 * pairs (even lengths and offsets).
 *   avgpool_fwd: y[n,p,q,c] = mean of x over the part of the window inside the image (padding is not counted);
 *   avgpool_bwd: dx[n,h,w,c] = sum over the windows (p,q) containing (h,w) of dy[n,p,q,c] / (valid elements of (p,q)).
 *   desc as for the max-pool (flags ignored; any window size; every window must reach the image).
 *   copy2d: dst[r*dst_ld + j] = src[r*src_ld + j] for r < rows, j < cols (lengths in floats): with src a branch's
 *   [rows][cols] output and dst = wide + channel offset, dst_ld = the wide tensor's channels, it writes one slice of a
 *   concatenation; with the roles swapped it cuts the slice of the gradient back out.  src, dst 4-byte aligned (16-byte
 *   accesses are used when pointers, cols and both lds allow); rows*ld < 2^31; ld < cols is STANZA_EINVAL. */
int stanza_avgpool_fwd(const stanza_pool_desc *desc, int32_t dtype, const void *x, void *y, void *stream);
int stanza_avgpool_bwd(const stanza_pool_desc *desc, int32_t dtype, const void *dy, void *dx, void *stream);
int stanza_copy2d(int64_t rows, int32_t cols, const float *src, int64_t src_ld, float *dst, int64_t dst_ld, void *stream);

/* ---- Batch normalisation in training mode, on the CONV worker (the residual networks of the paper's table of models,
 * Sec. 6.1, carry one after every convolution; the paper does not describe the layer, so the published transform is
 * used, and every worker takes the statistics over its OWN batch: nothing is exchanged between workers).
 * x, y, dy, dx are [rows][C] (an NHWC tensor with rows = N*H*W), float32 or bfloat16 (then C % 8 == 0); gamma, beta,
 * the statistics and the parameter gradients are float32 [C].
 *   fwd   mean_c = (1/rows) sum_m x[m,c];  var_c = (1/rows) sum_m (x[m,c] - mean_c)^2;  istd_c = 1/sqrt(var_c + eps)
 *         y[m,c] = ((x[m,c] - mean_c) * s_c) + beta_c  with  s_c = gamma_c istd_c  (each operation rounded to float32
 *         on its own), then max(.,0) when relu != 0.  save_mean and save_istd receive the statistics.
 *         running_mean / running_var (both optional, NULL to skip) move by r <- (1 - momentum) r + momentum * stat, the
 *         variance entering with the factor rows/(rows-1).
 *   bwd   g = dy, or dy * [((x - mean_c) s_c) + beta_c > 0] when relu != 0 (the sign of the forward output, recomputed from x with the
 *         same float32 operations, so y is not an argument);  xhat = (x - mean_c) istd_c
 *         dbeta_c = sum_m g[m,c];  dgamma_c = sum_m g[m,c] xhat[m,c]
 *         dx[m,c] = s_c (g[m,c] - dbeta_c/rows - xhat[m,c] dgamma_c/rows)
 *         save_mean / save_istd are the forward call's outputs; dgamma, dbeta are overwritten.
 * Sums over rows are taken per workgroup and then over workgroups in a fixed order (run-to-run identical results).
 * ws must hold stanza_bn_workspace_bytes(rows, C, dtype) bytes (0 is returned for invalid arguments).
 * Errors: rows < 1, C < 1, rows*C >= 2^31, eps <= 0, momentum outside [0,1] -> STANZA_EINVAL; bfloat16 with C % 8 != 0 or
 * an unknown dtype -> STANZA_EUNSUPPORTED; NULL, alignment and workspace errors as elsewhere. */
size_t stanza_bn_workspace_bytes(int64_t rows, int32_t C, int32_t dtype);
int stanza_bn_fwd(int64_t rows, int32_t C, int32_t dtype, float eps, int32_t relu, const void *x, const float *gamma,
                  const float *beta, void *y, float *save_mean, float *save_istd, float *running_mean, float *running_var,
                  float momentum, void *ws, size_t ws_bytes, void *stream);
/* Forward with a residual join fused in (the residual blocks of the published networks end in normalisation, join, ReLU):
 *   y = bn(x) + res, then max(.,0) when relu != 0; res [rows][C] of the dtype of x, 16-byte aligned, not overlapping y, required.
 * Statistics and running averages as in stanza_bn_fwd.  Backward: stanza_add_relu_bwd on y, then stanza_bn_bwd with relu = 0. */
int stanza_bn_fwd_res(int64_t rows, int32_t C, int32_t dtype, float eps, int32_t relu, const void *x, const float *gamma,
                      const float *beta, const void *res, void *y, float *save_mean, float *save_istd, float *running_mean,
                      float *running_var, float momentum, void *ws, size_t ws_bytes, void *stream);
/* A convolution followed by a normalisation layer (every convolution of the residual and Inception networks of the paper's table
 * of models, Sec. 6.1; the fusion is not in the paper): the convolution's epilogue leaves per-tile column sums of its output in
 * `stats`, and the normalisation layer takes mean and variance from them instead of reading the tensor once more (two passes over
 * the tensor instead of three).
 *   stanza_conv_fwd_stats  = stanza_conv_fwd (same arguments, same y) that also fills stats; float32 only, K % 4 == 0 and no
 *       STANZA_CONV_RELU (otherwise STANZA_EUNSUPPORTED).  stats: device memory of stanza_conv_stats_bytes(desc) bytes (0 for
 *       a descriptor this call does not take), 16-byte aligned, contents opaque (a header, then per tile and column the sums of
 *       (y - k) and (y - k)^2 about the tile's first row k); fewer bytes -> STANZA_EWORKSPACE.
 *   stanza_bn_fwd_stats    = stanza_bn_fwd / stanza_bn_fwd_res (res != NULL: y = bn(x) + res before the ReLU) for float32 x
 *       = the y of that convolution call (rows = N*Ho*Wo, C = K; C % 4 == 0), with stats as that call left it; needs no workspace.
 *       The variance is the shifted two-sum form of stanza_bn_fwd about one row of the data, summed in a fixed order; mean and
 *       1/std agree with stanza_bn_fwd to rounding.  A stats buffer that was not written for this [rows][C] matrix, or is
 *       shorter than its own header says, gives NaN statistics (detected on the device: no error code). */
size_t stanza_conv_stats_bytes(const stanza_conv_desc *desc);
int stanza_conv_fwd_stats(const stanza_conv_desc *desc, const void *x, const void *w, const float *bias, void *y, void *stats,
                          size_t stats_bytes, void *ws, size_t ws_bytes, void *stream);
int stanza_bn_fwd_stats(int64_t rows, int32_t C, float eps, int32_t relu, const void *x, const void *stats, size_t stats_bytes,
                        const float *gamma, const float *beta, const void *res, void *y, float *save_mean, float *save_istd,
                        float *running_mean, float *running_var, float momentum, void *stream);
int stanza_bn_bwd(int64_t rows, int32_t C, int32_t dtype, int32_t relu, const void *x, const void *dy, const float *gamma,
                  const float *beta, const float *save_mean, const float *save_istd, void *dx, float *dgamma, float *dbeta,
                  void *ws, size_t ws_bytes, void *stream);

/* float32 -> bfloat16 (round to nearest even) and back, for feeding the STANZA_BF16 conv path from
 * float32 master weights and images.  Any element-aligned pointers; 16-byte-aligned ones take the vector path.
 * Errors: numel < 1 or beyond 2^43 -> STANZA_EINVAL; NULL -> STANZA_ENULL. */
int stanza_cast_f32_to_bf16(int64_t numel, const float *src, void *dst, void *stream);
int stanza_cast_bf16_to_f32(int64_t numel, const void *src, float *dst, void *stream);
/* The same cast over many tensors in one launch (a CONV worker's per-step bfloat16 copies of all its master filters).
 *   stanza_cast_plan writes a table of the n tensors (host_numel[t] elements from host_src[t] to host_dst[t]; device pointers, 16-byte
 *   aligned, held in host arrays) into ws (stanza_cast_workspace_bytes(n) bytes, caller-owned).  The table travels inside the
 *   arguments of small fill launches on `stream` (one per 480 table words): the call only enqueues, the host arrays may be freed
 *   when it returns, and it may be recorded in a stream capture like every other call;
 *   stanza_cast_f32_to_bf16_planned then converts all of them, any number of times, with the same n and host_numel.
 * Errors: n < 1, a tensor with numel < 1 -> STANZA_EINVAL; NULL / alignment / workspace size as elsewhere. */
size_t stanza_cast_workspace_bytes(int32_t n_tensors);
int stanza_cast_plan(int32_t n_tensors, const int64_t *host_numel, const float *const *host_src, void *const *host_dst, void *ws,
                     size_t ws_bytes, void *stream);
int stanza_cast_f32_to_bf16_planned(int32_t n_tensors, const int64_t *host_numel, const void *ws, size_t ws_bytes, void *stream);

/* ---- FC worker step (Sec. 3.2: the FC worker collects the activations of all workers, continues the
 * forward pass to the loss, backpropagates through the FC layers down to the gradient of the received
 * activations, sends those gradients back and updates the FC parameters).
 *   forward   Z_l = A_{l-1} W_l^T + b_l, A_l = max(Z_l, 0) for l < n_layers, A_0 = feats
 *   loss      (1/n) sum_i [logsumexp(Z_L[i,:]) - Z_L[i, labels[i]]]   (mean over the GLOBAL batch n, which
 *             is what makes the sum of the workers' conv gradients the whole-batch gradient, Eq. 1)
 *   pred[i]   lowest index of the maximum of Z_L[i,:]
 *   backward  dZ_L = (softmax(Z_L) - onehot)/n; db_l = column sums of dZ_l; dW_l = dZ_l^T A_{l-1};
 *             dA_{l-1} = (dZ_l W_l) * [A_{l-1} > 0], all with the weights as they were BEFORE this call;
 *             dfeats = dZ_1 W_1 (no gate)
 *   update    for every W_l, b_l:  g += weight_decay*p;  v = momentum*v + g;  p -= lr*v   (Sec. 6.1)
 * With desc->dropout_p > 0:  A_l = dropout(max(Z_l, 0)) for l < n_layers, and dA_{l-1} passes back through the same mask
 * and scale before the ReLU gate (stanza_dropout below; the caller advances desc->dropout_step every iteration).
 * host_W, host_b, host_vW, host_vb: host arrays of n_layers device pointers; parameters and momentum
 * buffers are updated in place.  dfeats [n][A] and loss (1 float) are outputs; pred [n] may be NULL.
 * ws must hold stanza_fc_workspace_bytes(desc) bytes. */
size_t stanza_fc_workspace_bytes(const stanza_fc_desc *desc);
int stanza_fc_step(const stanza_fc_desc *desc, const float *feats, const int32_t *labels,
                   float *const *host_W, float *const *host_b, float *const *host_vW, float *const *host_vb,
                   float *dfeats, float *loss, int32_t *pred, void *ws, size_t ws_bytes, void *stream);

/* ---- Seeded dropout (the FC layers of the AlexNet- and VGG-shaped models of Sec. 6.1 are trained with it; the paper does
 * not describe it, so the published inverted form is used):  y[i] = keep_i ? x[i] / (1 - p) : 0, float32, x == y allowed.
 * keep_i is drawn from the counter-based Philox-4x32 generator with ten rounds (Salmon, Moraes, Dror, Shaw, SC 2011):
 * element i takes word (i mod 4) of the block with counter words (i/4 low, i/4 high, stream_id low, stream_id high) and key
 * words (seed low, seed high), and is kept iff the word is >= floor(p * 2^32).  The operation is its own transpose: the
 * backward pass is the same call on the gradient.  Nothing is stored between the two.
 * Errors: numel < 1 or >= 2^31, p outside [0, 1) -> STANZA_EINVAL; NULL / alignment as elsewhere. */
int stanza_dropout(int64_t numel, float p, uint64_t seed, uint64_t stream_id, const float *x, float *y, void *stream);

/* ---- One of several FC workers (Sec. 4.1.3: the CONV workers are divided evenly among the FC workers, every FC worker holds
 * its own full copy of the FC layers, and the FC workers then exchange their gradients by the same recursive doubling).  The same forward / loss / backward as stanza_fc_step over this worker's n_samples rows, except that
 *   - the loss is still the mean over the GLOBAL batch of n_global >= n_samples rows (Eq. 1): loss_part =
 *     (1/n_global) sum over this worker's rows, dZ_L = (softmax - onehot)/n_global, so that the workers' parts add up;
 *   - nothing is updated: dW_l and db_l are written to host_gW[l] ([out][in]) and host_gb[l] ([out]), float32, for
 *     stanza_ps_aggregate_ordered over the FC workers' gradient sets (STANZA_SUM_RECURSIVE_DOUBLING for the paper's order).
 * desc->lr, momentum, weight_decay are ignored.  n_global < n_samples is STANZA_EINVAL; other errors, workspace size and
 * ownership as for stanza_fc_step. */
int stanza_fc_grads(const stanza_fc_desc *desc, int32_t n_global, const float *feats, const int32_t *labels,
                    float *const *host_W, float *const *host_b, float *const *host_gW, float *const *host_gb,
                    float *dfeats, float *loss_part, int32_t *pred, void *ws, size_t ws_bytes, void *stream);

/* ---- Gradient aggregation and update (Sec. 3.2: the CONV workers combine their gradients into the gradient of the
 * whole batch, sum_x grad l(x, w_conv), and update their replicas; Sec. 2.2: the servers add up the workers' gradients
 * and apply the update).  Per tensor t and element i:
 *   g = scale * (g_0[i] + g_1[i] + ... + g_{K-1}[i]) + weight_decay * w[i]   (shards added in index order)
 *   v[i] = momentum * v[i] + g;   w[i] -= lr * v[i]
 * host_numel [n_tensors]; host_w, host_v [n_tensors] device pointers (updated in place);
 * host_grads [K * n_tensors] device pointers, shard-major: host_grads[k*n_tensors + t].
 * One launch covers all tensors.  ws receives the pointer table (stanza_ps_workspace_bytes(n_tensors, K) bytes).  The
 * table travels inside the arguments of small fill launches on `stream`, one per 480 table words (n_tensors*(K + 4) + 1
 * words in all: two launches for a 26-tensor set at K = 16), which precede the aggregation launch on the same stream:
 * nothing is allocated, no copy is issued and nothing waits, the host arrays may be freed when the call returns, and the
 * call may be recorded in a stream capture.
 * stanza_ps_plan writes the table only.  stanza_ps_aggregate_planned runs the aggregation launch on a table a previous
 * stanza_ps_plan / stanza_ps_aggregate put into ws (same n_tensors, host_numel, K), for callers whose buffers stay put
 * from one iteration to the next. */
size_t stanza_ps_workspace_bytes(int32_t n_tensors, int32_t K);
int stanza_ps_plan(int32_t n_tensors, const int64_t *host_numel, float *const *host_w, float *const *host_v,
                   const float *const *host_grads, int32_t K, void *ws, size_t ws_bytes, void *stream);
int stanza_ps_aggregate_planned(int32_t n_tensors, const int64_t *host_numel, int32_t K, float scale, float lr,
                                float momentum, float weight_decay, const void *ws, size_t ws_bytes, void *stream);
int stanza_ps_aggregate(int32_t n_tensors, const int64_t *host_numel, float *const *host_w, float *const *host_v,
                        const float *const *host_grads, int32_t K, float scale, float lr, float momentum,
                        float weight_decay, void *ws, size_t ws_bytes, void *stream);

/* ---- The same aggregation with the shards added in the order of the paper's all-reduce (Sec. 4.1.2, recursive
 * doubling): in round i = 1, 2, ... worker j adds to its own partial sum the partial sum of worker j xor 2^(i-1), so
 * after log2 K rounds every worker holds the balanced pairwise tree ((g_0+g_1)+(g_2+g_3))+((g_4+g_5)+(g_6+g_7))...
 * Addition being commutative, every worker holds the same bits (the property the paper chose the schedule for),
 * and on one GPU one tree gives them all.  When K is not a power of two, P = 2^floor(log2 K) workers take part: the
 * surplus worker P + i first sends its gradient to worker i (i < K - P), which adds it to its own before round 1; the
 * paper picks the surplus workers and their partners at random, this library takes the last K - P workers and
 * partners them with the first K - P.  The final round that returns the result to the surplus workers is a copy.
 * order: STANZA_SUM_INDEX_ORDER gives exactly stanza_ps_aggregate / stanza_ps_aggregate_planned.
 * Errors and ownership as above; an unknown order is STANZA_EINVAL. */
typedef enum { STANZA_SUM_INDEX_ORDER = 0, STANZA_SUM_RECURSIVE_DOUBLING = 1 } stanza_sum_order;
int stanza_ps_aggregate_ordered_planned(int32_t order, int32_t n_tensors, const int64_t *host_numel, int32_t K, float scale,
                                        float lr, float momentum, float weight_decay, const void *ws, size_t ws_bytes,
                                        void *stream);
int stanza_ps_aggregate_ordered(int32_t order, int32_t n_tensors, const int64_t *host_numel, float *const *host_w,
                                float *const *host_v, const float *const *host_grads, int32_t K, float scale, float lr,
                                float momentum, float weight_decay, void *ws, size_t ws_bytes, void *stream);

/* ---- The same aggregation for callers that cannot allocate: code recorded under HIP graph capture, tight serving or training
 * loops, and harnesses that forbid hipMalloc, which therefore have no workspace to pass.  Arguments and arithmetic are those of
 * stanza_ps_aggregate_ordered without ws / ws_bytes; the pointer table goes to a fixed array inside the library's device image
 * (256 KiB on every GPU the library runs on, held until the process ends) instead of a caller-owned workspace.
 *   - Capacity: n_tensors * (K + 4) + 1 <= 32768 table words (e.g. 1638 tensors at K = 16); beyond that STANZA_ECAPACITY and
 *     nothing is launched.  Other errors as for stanza_ps_aggregate_ordered.
 *   - The call allocates nothing on host or device and only enqueues launches on `stream`.  The first call on a device
 *     looks up that device's address of the array (no stream work; make it before a stream capture begins).
 *   - Every call on a GPU shares that GPU's array and rewrites the table whole, so nothing needs clearing between calls,
 *     but two calls that overlap on one GPU (different streams, or different threads) race on it: serialise them. */
int stanza_ps_aggregate_static(int32_t order, int32_t n_tensors, const int64_t *host_numel, float *const *host_w,
                               float *const *host_v, const float *const *host_grads, int32_t K, float scale, float lr,
                               float momentum, float weight_decay, void *stream);

/* ---- Performance model and node assignment (host arithmetic only; Sec. 4.2 and Sec. 7.1).  Times in seconds,
 * bandwidth in bit/s per node, every transferred value is 32 bits wide.
 *   rounds(n_c)          = log2 n_c when n_c is a power of two, floor(log2 n_c) + 2 otherwise (recursive doubling with
 *                          the extra send/return rounds for the surplus workers, Sec. 4.1.2); 0 for n_c = 1
 *   t_s(n_c, n_f)        = T_c + (n_c/n_f) T_f + 2 n_c A K / (n_f B) + P_c rounds(n_c) / B            (Eqs. 2-3)
 *   throughput_s         = n_c K / t_s                                                             (Eq. 4)
 *   assignment           = argmax over n_c + n_f = N, n_c, n_f >= 1 of throughput_s, by exhaustive search   (Eq. 5)
 *   t_ps(n_w, n_s)       = 2 n_w P / (n_s B) + T_ps ;  throughput_ps = n_w K / t_ps                  (Eqs. 6-7)
 * T_c, T_f: single-worker CONV time and FC time for ONE conv worker's activations (measured, e.g. by bench.py);
 * A: activations per sample handed to the FC worker; K: per-node batch; P_c, P: parameter counts.
 * The time functions return a negative value on invalid arguments (counts < 1, non-positive bandwidth). */
typedef struct {
    double T_c, T_f;          /* seconds */
    double A, K, P_c;         /* activations per sample, per-node batch, conv parameters */
    double bandwidth_bits;    /* per-node bandwidth, bit/s */
} stanza_model_params;

int32_t stanza_model_allreduce_rounds(int32_t n_c);
double stanza_model_stanza_time(const stanza_model_params *m, int32_t n_c, int32_t n_f);
double stanza_model_stanza_throughput(const stanza_model_params *m, int32_t n_c, int32_t n_f);
int stanza_model_assign(const stanza_model_params *m, int32_t N, int32_t *n_c, int32_t *n_f, double *throughput);
double stanza_model_ps_time(double P, double T_ps, int32_t n_w, int32_t n_s, double bandwidth_bits);
double stanza_model_ps_throughput(double P, double T_ps, double K, int32_t n_w, int32_t n_s, double bandwidth_bits);

#ifdef __cplusplus
}
#endif
#endif /* STANZA_H */
