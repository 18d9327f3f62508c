// FC-worker step (paper Sec. 3.2): forward over the concatenated activations of all CONV workers,
// mean softmax cross-entropy over the global batch, backpropagation through the FC layers down to the
// gradient of the received activations, and the momentum-SGD update (Sec. 6.1) of every FC parameter.
//
// The three GEMMs of a layer are launches of the implicit-GEMM engine with a 1x1 "image":
//   forward    Z  = A W^T + b        FWD        (N=n, H=W=1, C=in,  K=out)
//   to input   dA = dZ W             BWD_DATA   gated by [A > 0] on store
//   to weights dW = dZ^T A           BWD_WEIGHT with the update fused into the tile store, so the
//                                    gradient matrix never goes to memory
// dA is always issued before the update of the same layer's W, so it sees the pre-update weights.
#include "internal.h"

namespace stanza {

// One wavefront per row: max / argmax (lowest index wins ties), sum of exponentials, then the gradient
// (softmax - onehot)/n and the row's loss term  log(sum) + max - z[label].
__global__ __launch_bounds__(256) void softmax_ce_kernel(int n, int n_global, int classes, const float *__restrict__ z,
                                                         const int32_t *__restrict__ labels, float *__restrict__ dz,
                                                         float *__restrict__ row_loss, int32_t *__restrict__ pred)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const float *zr = z + (size_t)row * classes;
    float best = -INFINITY;
    int bidx = 0x7fffffff;
    for (int j = lane; j < classes; j += 64) {
        const float v = zr[j];
        if (v > best) { best = v; bidx = j; }   // ascending j per lane: first maximum kept
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ob = __shfl_xor(best, off);
        const int oi = __shfl_xor(bidx, off);
        if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
    }
    float sum = 0.f;
    for (int j = lane; j < classes; j += 64) sum += expf(zr[j] - best);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    const int label = labels[row];
    const float inv = 1.f / sum, invn = 1.f / (float)n_global;
    float *dr = dz + (size_t)row * classes;
    for (int j = lane; j < classes; j += 64) {
        const float sm = expf(zr[j] - best) * inv;
        dr[j] = (sm - (j == label ? 1.f : 0.f)) * invn;
    }
    if (lane == 0) {
        const float zl = ((unsigned)label < (unsigned)classes) ? zr[label] : NAN;
        row_loss[row] = logf(sum) + best - zl;
        if (pred) pred[row] = bidx;
    }
}

// Sum of the n row losses divided by n_global (the mean when the worker holds the whole batch), in a fixed order.
__global__ __launch_bounds__(256) void mean_loss_kernel(int n, int n_global, const float *__restrict__ row_loss, float *__restrict__ loss)
{
    __shared__ float red[256];
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) s += row_loss[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = red[0] / (float)n_global;
}

// Seeded dropout of hidden activations (the FC layers of the paper's AlexNet- and VGG-shaped models, Sec. 6.1, are trained
// with it; the paper does not describe the operation, so the published inverted form is used).  The mask comes from the
// counter-based Philox-4x32 generator with ten rounds (Salmon et al., SC 2011): element i takes word i mod 4 of the
// block whose counter is (i / 4, stream) under the key `seed`, and is kept iff that word is >= thr = floor(p * 2^32).
// Nothing is stored: the backward pass draws the same words again.
struct PhiloxKey {
    uint32_t k0, k1, s0, s1;   // seed (low, high), stream (low, high)
};

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// y[i] = keep_i ? x[i] * scale : 0 (x == y allowed).  One thread per generator block of four elements.
__global__ __launch_bounds__(256) void dropout_kernel(size_t numel, uint32_t thr, float scale, PhiloxKey key, const float *x, float *y)
{
    const size_t blk = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t i0 = blk * 4;
    if (i0 >= numel) return;
    uint32_t r[4];
    philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), key.s0, key.s1, key.k0, key.k1, r);
    if (i0 + 4 <= numel) {
        const float4 v = *reinterpret_cast<const float4 *>(x + i0);
        float4 o;
        o.x = r[0] >= thr ? v.x * scale : 0.f;
        o.y = r[1] >= thr ? v.y * scale : 0.f;
        o.z = r[2] >= thr ? v.z * scale : 0.f;
        o.w = r[3] >= thr ? v.w * scale : 0.f;
        *reinterpret_cast<float4 *>(y + i0) = o;
    } else {
        for (int e = 0; i0 + e < numel; ++e) y[i0 + e] = r[e] >= thr ? x[i0 + e] * scale : 0.f;
    }
}

__global__ __launch_bounds__(256) void scale_kernel(size_t numel, float scale, float *y)
{
    const size_t i0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 + 4 <= numel) {
        float4 v = *reinterpret_cast<float4 *>(y + i0);
        v.x *= scale; v.y *= scale; v.z *= scale; v.w *= scale;
        *reinterpret_cast<float4 *>(y + i0) = v;
    } else {
        for (size_t i = i0; i < numel; ++i) y[i] *= scale;
    }
}

// bfloat16 forms for the hidden layers kept in bf16: the same generator blocks (element i takes word i % 4 of block i / 4), two
// blocks = 8 elements = one 16-byte vector per thread; kept elements are scaled in float32 and rounded once.  numel % 8 == 0.
__device__ __forceinline__ uint32_t bf16_scale_pair(uint32_t pair, float s_lo, float s_hi)
{
    auto one = [](uint32_t h, float s) -> uint32_t {
        uint32_t u = __float_as_uint(__uint_as_float(h << 16) * s);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
        u += 0x7fffu + ((u >> 16) & 1u);
        return u >> 16;
    };
    return one(pair & 0xffffu, s_lo) | (one(pair >> 16, s_hi) << 16);
}
__global__ __launch_bounds__(256) void dropout_bf16_kernel(size_t numel, uint32_t thr, float scale, PhiloxKey key, uint4 *y)
{
    const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (v * 8 >= numel) return;
    uint32_t r0[4], r1[4];
    philox4x32_10((uint32_t)(2 * v), (uint32_t)((2 * v) >> 32), key.s0, key.s1, key.k0, key.k1, r0);
    philox4x32_10((uint32_t)(2 * v + 1), (uint32_t)((2 * v + 1) >> 32), key.s0, key.s1, key.k0, key.k1, r1);
    float sc[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        sc[e] = r0[e] >= thr ? scale : 0.f;
        sc[4 + e] = r1[e] >= thr ? scale : 0.f;
    }
    uint4 x = y[v];
    x.x = bf16_scale_pair(x.x, sc[0], sc[1]);
    x.y = bf16_scale_pair(x.y, sc[2], sc[3]);
    x.z = bf16_scale_pair(x.z, sc[4], sc[5]);
    x.w = bf16_scale_pair(x.w, sc[6], sc[7]);
    y[v] = x;
}
__global__ __launch_bounds__(256) void scale_bf16_kernel(size_t numel, float scale, uint4 *y)
{
    const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (v * 8 >= numel) return;
    uint4 x = y[v];
    x.x = bf16_scale_pair(x.x, scale, scale);
    x.y = bf16_scale_pair(x.y, scale, scale);
    x.z = bf16_scale_pair(x.z, scale, scale);
    x.w = bf16_scale_pair(x.w, scale, scale);
    y[v] = x;
}

// Momentum-SGD update from a gradient in memory (the bf16 hidden layers: their filter-gradient kernel has no fused update).
__global__ __launch_bounds__(256) void sgd_update_kernel(size_t numel, float *__restrict__ w, float *__restrict__ v, const float *__restrict__ g,
                                                         float lr, float mom, float wd)
{
    const size_t i0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 + 4 <= numel) {
        float4 ww = *reinterpret_cast<float4 *>(w + i0), vv = *reinterpret_cast<float4 *>(v + i0);
        const float4 gg = *reinterpret_cast<const float4 *>(g + i0);
        vv.x = mom * vv.x + (gg.x + wd * ww.x); ww.x -= lr * vv.x;
        vv.y = mom * vv.y + (gg.y + wd * ww.y); ww.y -= lr * vv.y;
        vv.z = mom * vv.z + (gg.z + wd * ww.z); ww.z -= lr * vv.z;
        vv.w = mom * vv.w + (gg.w + wd * ww.w); ww.w -= lr * vv.w;
        *reinterpret_cast<float4 *>(v + i0) = vv;
        *reinterpret_cast<float4 *>(w + i0) = ww;
    } else {
        for (size_t i = i0; i < numel; ++i) {
            const float vel = mom * v[i] + (g[i] + wd * w[i]);
            v[i] = vel;
            w[i] -= lr * vel;
        }
    }
}

static bool dropout_valid(float p) { return p >= 0.f && p < 1.f; }
static uint32_t dropout_threshold(float p) { return (uint32_t)((double)p * 4294967296.0); }
static PhiloxKey dropout_key(uint64_t seed, uint64_t stream_id)
{
    return PhiloxKey{(uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)stream_id, (uint32_t)(stream_id >> 32)};
}

struct FcLayout {
    size_t act_off[32];   // float offset of A_l (l = 1..L) in the workspace
    size_t dz_off[2];     // two gradient buffers of n * max_width floats
    size_t row_loss_off;
    size_t db_off;        // column-sum scratch: colsum_blocks(n) * max_width
    size_t partial_off;   // reduction-slice sums of the forward / input-gradient GEMMs that are cut (largest of them)
    size_t partial_floats;
    // bf16 hidden layers (compute_dtype == STANZA_BF16), offsets in floats like the rest:
    size_t a16_off[32];   // bf16 A_l, l = 0 .. L-1 (n * dims[l] halves)
    size_t w16_off[32];   // bf16 copy of W_l, l = 1 .. L-1
    size_t dz16_off[2];   // two bf16 gradient buffers of n * max_width halves
    size_t dfeats16_off;  // bf16 gradient of the features before it is widened
    size_t dw_off;        // float32 weight gradient of one hidden layer (the largest)
    size_t dbh_off;       // float32 bias gradient of one hidden layer
    size_t wgrad_off;     // workspace of the bf16 filter-gradient calls
    size_t wgrad_bytes;
    size_t floats;
};

static stanza_conv_desc fc_conv_desc(int n, int in, int out, int dtype, uint32_t flags)
{
    return stanza_conv_desc{n, 1, 1, in, out, 1, 1, 1, 1, 0, 0, dtype, flags};
}

static int fc_layout(const stanza_fc_desc *d, FcLayout *lay)
{
    if (!d || !d->host_dims) return STANZA_ENULL;
    if (d->n_layers <= 0 || d->n_layers > 30 || d->n_samples <= 0) return STANZA_EINVAL;
    size_t off = 0;
    int maxw = 0;
    for (int l = 0; l <= d->n_layers; ++l) {
        const int w = d->host_dims[l];
        if (w <= 0 || (int64_t)w * d->n_samples >= (int64_t(1) << 31)) return STANZA_EINVAL;
        if (l > 0) {
            if ((int64_t)w * d->host_dims[l - 1] >= (int64_t(1) << 31)) return STANZA_EINVAL;
            lay->act_off[l] = off;
            off += (round256((size_t)d->n_samples * w * 4)) / 4;
            maxw = max(maxw, w);
        }
    }
    const size_t dzf = round256((size_t)d->n_samples * maxw * 4) / 4;
    lay->dz_off[0] = off; off += dzf;
    lay->dz_off[1] = off; off += dzf;
    lay->row_loss_off = off; off += round256((size_t)d->n_samples * 4) / 4;
    lay->db_off = off; off += round256((size_t)colsum_blocks(d->n_samples) * maxw * 4) / 4;
    size_t pf = 0;
    for (int l = 1; l <= d->n_layers; ++l) {
        pf = max(pf, igemm_partial_floats(MODE_FWD, d->n_samples, d->host_dims[l], d->host_dims[l - 1]));
        pf = max(pf, igemm_partial_floats(MODE_BWD_DATA, d->n_samples, d->host_dims[l - 1], d->host_dims[l]));
    }
    lay->partial_off = off; lay->partial_floats = pf; off += round256(pf * 4) / 4;
    if (d->compute_dtype == STANZA_BF16) {
        const int L = d->n_layers, n = d->n_samples;
        size_t dwf = 0;
        int maxh = 0;
        lay->wgrad_bytes = 0;
        // Everything the nested bfloat16 convolution calls could refuse is refused here, before the first launch: widths that are
        // not multiples of 8, and operands of 2 GiB and more (those calls address them with 32-bit byte offsets).
        for (int l = 0; l < L; ++l) {
            if (d->host_dims[l] % 8) return STANZA_EUNSUPPORTED;
            if ((int64_t)n * d->host_dims[l] * 2 >= (int64_t(1) << 31)) return STANZA_EUNSUPPORTED;
            if (l > 0 && (int64_t)d->host_dims[l] * d->host_dims[l - 1] * 2 >= (int64_t(1) << 31)) return STANZA_EUNSUPPORTED;
            lay->a16_off[l] = off; off += round256((size_t)n * d->host_dims[l] * 2) / 4;
        }
        for (int l = 1; l < L; ++l) {
            const int in = d->host_dims[l - 1], out = d->host_dims[l];
            lay->w16_off[l] = off; off += round256((size_t)out * in * 2) / 4;
            dwf = max(dwf, (size_t)out * in);
            maxh = max(maxh, max(in, out));
            const stanza_conv_desc cd = fc_conv_desc(n, in, out, STANZA_BF16, STANZA_CONV_BIAS);
            lay->wgrad_bytes = max(lay->wgrad_bytes, stanza_conv_workspace_bytes(&cd, 2));
        }
        const size_t dz16f = round256((size_t)n * max(maxh, 8) * 2) / 4;
        lay->dz16_off[0] = off; off += dz16f;
        lay->dz16_off[1] = off; off += dz16f;
        lay->dfeats16_off = off; off += round256((size_t)n * d->host_dims[0] * 2) / 4;
        lay->dw_off = off; off += round256(dwf * 4) / 4;
        lay->dbh_off = off; off += round256((size_t)max(maxh, 8) * 4) / 4;
        lay->wgrad_off = off; off += round256(lay->wgrad_bytes) / 4;
    } else if (d->compute_dtype != STANZA_F32) {
        return STANZA_EUNSUPPORTED;
    }
    lay->floats = off;
    return STANZA_OK;
}

static ConvGeo fc_geo(int n, int in, int out) { return ConvGeo{n, 1, 1, in, out, 1, 1, 1, 1, 0, 0, 1, 1}; }

}  // namespace stanza

using namespace stanza;

extern "C" size_t stanza_fc_workspace_bytes(const stanza_fc_desc *desc)
{
    FcLayout lay;
    if (fc_layout(desc, &lay) != STANZA_OK) return 0;
    return lay.floats * 4;
}

// Shared body of stanza_fc_step (update fused, gW == nullptr) and stanza_fc_grads (gradients written to gW / gb, no
// update, loss and gradient normalised by n_global).
static int fc_run(const stanza_fc_desc *desc, int n_global, const float *feats, const int32_t *labels, float *const *host_W,
                  float *const *host_b, float *const *host_vW, float *const *host_vb, float *const *host_gW, float *const *host_gb,
                  float *dfeats, float *loss, int32_t *pred, void *ws, size_t ws_bytes, void *stream)
{
    const bool fused = host_gW == nullptr;
    FcLayout lay;
    int rc = fc_layout(desc, &lay);
    if (rc) return rc;
    if (n_global < desc->n_samples) return STANZA_EINVAL;
    if (!dropout_valid(desc->dropout_p) || desc->dropout_step >= (uint64_t(1) << 56)) return STANZA_EINVAL;
    if (!feats || !labels || !host_W || !host_b || !dfeats || !loss || !ws) return STANZA_ENULL;
    if (fused ? (!host_vW || !host_vb) : !host_gb) return STANZA_ENULL;
    if (ws_bytes < lay.floats * 4) return STANZA_EWORKSPACE;
    if (!aligned16(feats) || !aligned16(dfeats) || !aligned16(ws)) return STANZA_EALIGN;
    const int L = desc->n_layers, n = desc->n_samples;
    const int32_t *dims = desc->host_dims;
    for (int l = 0; l < L; ++l) {
        if (!host_W[l] || !host_b[l]) return STANZA_ENULL;
        if (fused ? (!host_vW[l] || !host_vb[l]) : (!host_gW[l] || !host_gb[l])) return STANZA_ENULL;
        if (!aligned16(host_W[l]) || !aligned16(host_b[l]) || !aligned16(fused ? host_vW[l] : host_gW[l]) ||
            !aligned16(fused ? host_vb[l] : host_gb[l]))
            return STANZA_EALIGN;
    }
    hipStream_t st = (hipStream_t)stream;
    float *base = (float *)ws;
    const bool half = desc->compute_dtype == STANZA_BF16;   // hidden layers in bf16, the last layer and the loss in float32
    const bool drop = desc->dropout_p > 0.f;
    const uint32_t drop_thr = dropout_threshold(desc->dropout_p);
    const float drop_scale = 1.f / (1.f - desc->dropout_p);
    auto act = [&](int l) -> const float * { return l == 0 ? feats : base + lay.act_off[l]; };

    // forward
    auto a16 = [&](int l) -> void * { return base + lay.a16_off[l]; };
    auto w16 = [&](int l) -> void * { return base + lay.w16_off[l]; };
    if (half) {
        if ((rc = stanza_cast_f32_to_bf16((int64_t)n * dims[0], feats, a16(0), stream))) return rc;
        for (int l = 1; l < L; ++l) {
            const stanza_conv_desc cd = fc_conv_desc(n, dims[l - 1], dims[l], STANZA_BF16, STANZA_CONV_BIAS | STANZA_CONV_RELU);
            if ((rc = stanza_cast_f32_to_bf16((int64_t)dims[l] * dims[l - 1], host_W[l - 1], w16(l), stream))) return rc;   // this step's copy
            if ((rc = stanza_conv_fwd(&cd, a16(l - 1), w16(l), host_b[l - 1], a16(l), nullptr, 0, stream))) return rc;
            if (drop) {    // the next layer, the float32 copy for the last layer and the backward pass see the dropped activations
                const size_t numel = (size_t)n * dims[l];
                hipLaunchKernelGGL(dropout_bf16_kernel, dim3((unsigned)cdiv64(numel / 8, 256)), dim3(256), 0, st, numel, drop_thr, drop_scale,
                                   dropout_key(desc->dropout_seed, (desc->dropout_step << 8) | (uint64_t)(l - 1)), (uint4 *)a16(l));
                if ((rc = launch_status())) return rc;
            }
        }
        if (L > 1 && (rc = stanza_cast_bf16_to_f32((int64_t)n * dims[L - 1], a16(L - 1), base + lay.act_off[L - 1], stream))) return rc;
    }
    for (int l = half ? L : 1; l <= L; ++l) {
        GemmParams p{};
        p.g = fc_geo(n, dims[l - 1], dims[l]);
        p.a = act(l - 1);
        p.b = host_W[l - 1];
        p.bias = host_b[l - 1];
        p.out = base + lay.act_off[l];
        p.M = n; p.Nn = dims[l]; p.Kd = dims[l - 1];
        p.flags = EPI_BIAS | (l < L ? EPI_RELU : 0u);
        if ((rc = launch_igemm(MODE_FWD, p, 1, base + lay.partial_off, lay.partial_floats, st))) return rc;
        if (drop && l < L) {   // hidden layer: the next layer (and the backward pass) sees the dropped activations
            const size_t numel = (size_t)n * dims[l];
            hipLaunchKernelGGL(dropout_kernel, dim3((unsigned)cdiv64(cdiv64(numel, 4), 256)), dim3(256), 0, st, numel, drop_thr, drop_scale,
                               dropout_key(desc->dropout_seed, (desc->dropout_step << 8) | (uint64_t)(l - 1)), p.out, p.out);
            if ((rc = launch_status())) return rc;
        }
    }
    // loss and its gradient
    float *dz = base + lay.dz_off[0], *dz_next = base + lay.dz_off[1];
    float *row_loss = base + lay.row_loss_off;
    hipLaunchKernelGGL(softmax_ce_kernel, dim3(cdiv(n, 4)), dim3(256), 0, st, n, n_global, dims[L], act(L), labels, dz, row_loss, pred);
    if ((rc = launch_status())) return rc;
    hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(256), 0, st, n, n_global, row_loss, loss);
    if ((rc = launch_status())) return rc;
    // backward (+ update), last layer first
    const int dbb = colsum_blocks(n);
    for (int l = L; l >= 1; --l) {
        const int in = dims[l - 1], out = dims[l];
        if (half && l < L) {
            // hidden layer in bf16: dz arrives as float32 from the last layer (l == L-1) or as bf16 from the layer above
            void *dz16 = base + lay.dz16_off[(L - 1 - l) & 1], *dz16_next = base + lay.dz16_off[(L - l) & 1];
            if (l == L - 1 && (rc = stanza_cast_f32_to_bf16((int64_t)n * out, dz, dz16, stream))) return rc;
            const stanza_conv_desc cd = fc_conv_desc(n, in, out, STANZA_BF16, STANZA_CONV_BIAS);
            void *dx16 = l == 1 ? (void *)(base + lay.dfeats16_off) : dz16_next;
            if ((rc = stanza_conv_bwd_data(&cd, dz16, nullptr, w16(l), l == 1 ? nullptr : a16(l - 1), dx16, nullptr, 0, stream))) return rc;
            if (drop && l > 1) {   // the gate used the dropped activations (see the float32 path below): the kept units' scale remains
                const size_t numel = (size_t)n * in;
                hipLaunchKernelGGL(scale_bf16_kernel, dim3((unsigned)cdiv64(numel / 8, 256)), dim3(256), 0, st, numel, drop_scale, (uint4 *)dx16);
                if ((rc = launch_status())) return rc;
            }
            if (l == 1 && (rc = stanza_cast_bf16_to_f32((int64_t)n * in, dx16, dfeats, stream))) return rc;
            float *dw = fused ? base + lay.dw_off : host_gW[l - 1];
            float *db = fused ? base + lay.dbh_off : host_gb[l - 1];
            if ((rc = stanza_conv_bwd_weight(&cd, a16(l - 1), dz16, nullptr, dw, db, base + lay.wgrad_off, lay.wgrad_bytes, stream))) return rc;
            if (fused) {
                const size_t nw = (size_t)out * in;
                hipLaunchKernelGGL(sgd_update_kernel, dim3((unsigned)cdiv64(cdiv64(nw, 4), 256)), dim3(256), 0, st, nw, host_W[l - 1], host_vW[l - 1],
                                   (const float *)dw, desc->lr, desc->momentum, desc->weight_decay);
                hipLaunchKernelGGL(sgd_update_kernel, dim3((unsigned)cdiv64(cdiv64(out, 4), 256)), dim3(256), 0, st, (size_t)out, host_b[l - 1], host_vb[l - 1],
                                   (const float *)db, desc->lr, desc->momentum, desc->weight_decay);
                if ((rc = launch_status())) return rc;
            }
            continue;
        }
        {   // gradient of the layer input, with the weights as they still are
            GemmParams p{};
            p.g = fc_geo(n, in, out);
            p.a = dz;
            p.b = host_W[l - 1];
            p.out = (l == 1) ? dfeats : dz_next;
            p.xmask = (l == 1) ? nullptr : act(l - 1);
            p.M = n; p.Nn = in; p.Kd = out;
            p.flags = p.xmask ? EPI_XMASK : 0u;
            if ((rc = launch_igemm(MODE_BWD_DATA, p, 1, base + lay.partial_off, lay.partial_floats, st))) return rc;
            if (drop && l > 1) {
                // the gate [A > 0] above used the dropped activations, so dropped units are zero already (ReLU and mask
                // in one test); what remains of the mask's backward is the scale of the kept units
                const size_t numel = (size_t)n * in;
                hipLaunchKernelGGL(scale_kernel, dim3((unsigned)cdiv64(cdiv64(numel, 4), 256)), dim3(256), 0, st, numel, drop_scale, dz_next);
                if ((rc = launch_status())) return rc;
            }
        }
        {   // weight gradient: fused with the update, or written out
            GemmParams p{};
            p.g = fc_geo(n, in, out);
            p.a = dz;
            p.b = act(l - 1);
            p.M = out; p.Nn = in; p.Kd = n;
            if (fused) {
                p.flags = EPI_SGD;
                p.sgd_w = host_W[l - 1]; p.sgd_v = host_vW[l - 1];
                p.lr = desc->lr; p.mom = desc->momentum; p.wd = desc->weight_decay;
            } else {
                p.out = host_gW[l - 1];
            }
            if ((rc = launch_igemm(MODE_BWD_WEIGHT, p, 1, nullptr, 0, st))) return rc;
        }
        if (fused)
            rc = launch_colsum(dz, nullptr, n, out, base + lay.db_off, dbb, nullptr, host_b[l - 1], host_vb[l - 1], desc->lr,
                               desc->momentum, desc->weight_decay, st);
        else
            rc = launch_colsum(dz, nullptr, n, out, base + lay.db_off, dbb, host_gb[l - 1], nullptr, nullptr, 0.f, 0.f, 0.f, st);
        if (rc) return rc;
        float *tmp = dz; dz = dz_next; dz_next = tmp;
    }
    return STANZA_OK;
}

extern "C" int stanza_fc_step(const stanza_fc_desc *desc, const float *feats, const int32_t *labels, float *const *host_W,
                              float *const *host_b, float *const *host_vW, float *const *host_vb, float *dfeats, float *loss,
                              int32_t *pred, void *ws, size_t ws_bytes, void *stream)
{
    if (!desc) return STANZA_ENULL;
    return fc_run(desc, desc->n_samples, feats, labels, host_W, host_b, host_vW, host_vb, nullptr, nullptr, dfeats, loss, pred, ws,
                  ws_bytes, stream);
}

extern "C" int stanza_fc_grads(const stanza_fc_desc *desc, int32_t n_global, const float *feats, const int32_t *labels,
                               float *const *host_W, float *const *host_b, float *const *host_gW, float *const *host_gb,
                               float *dfeats, float *loss_part, int32_t *pred, void *ws, size_t ws_bytes, void *stream)
{
    if (!desc) return STANZA_ENULL;
    if (!host_gW) return STANZA_ENULL;
    return fc_run(desc, n_global, feats, labels, host_W, host_b, nullptr, nullptr, host_gW, host_gb, dfeats, loss_part, pred, ws,
                  ws_bytes, stream);
}

extern "C" int stanza_dropout(int64_t numel, float p, uint64_t seed, uint64_t stream_id, const float *x, float *y, void *stream)
{
    if (numel < 1 || numel >= (int64_t(1) << 31) || !dropout_valid(p)) return STANZA_EINVAL;
    if (!x || !y) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(y)) return STANZA_EALIGN;
    hipLaunchKernelGGL(dropout_kernel, dim3((unsigned)cdiv64(cdiv64(numel, 4), 256)), dim3(256), 0, (hipStream_t)stream, (size_t)numel,
                       dropout_threshold(p), 1.f / (1.f - p), dropout_key(seed, stream_id), x, y);
    return launch_status();
}
