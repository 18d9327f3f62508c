// Branch-and-join pieces of the Inception blocks (the paper trains Inception-V3, Sec. 6.1, without describing its
// layers: plain definitions): the average-pool branch and the channel concatenation / split, written as a strided
// two-dimensional copy between [rows][channels] matrices.  All HBM-bound: one thread per pixel and 16-byte channel
// vector, every byte moved once.
#include "internal.h"

namespace stanza {

struct AvgGeo {
    int N, H, W, C, wh, ww, sh, sw, ph, pw, Ho, Wo;
};

// Number of window positions of output index p that fall inside [0, extent).
__device__ __forceinline__ int avg_valid(int p, int stride, int pad, int win, int extent)
{
    const int lo = p * stride - pad;
    return min(lo + win, extent) - max(lo, 0);
}

// y[n,p,q,:] = mean over the valid part of the window.  One thread per output pixel and VW channels.
template <int VW>
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const AvgGeo g, const float *__restrict__ x, float *__restrict__ y, size_t total)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cv = g.C / VW;
    const int c = (int)(idx % cv);
    size_t t = idx / cv;
    const int q = (int)(t % g.Wo); t /= g.Wo;
    const int p = (int)(t % g.Ho);
    const int n = (int)(t / g.Ho);
    const int h0 = p * g.sh - g.ph, w0 = q * g.sw - g.pw;
    float acc[VW];
#pragma unroll
    for (int e = 0; e < VW; ++e) acc[e] = 0.f;
    for (int i = max(h0, 0); i < min(h0 + g.wh, g.H); ++i)
        for (int j = max(w0, 0); j < min(w0 + g.ww, g.W); ++j) {
            const float *src = x + ((((size_t)n * g.H + i) * g.W + j) * cv + c) * VW;
            if constexpr (VW == 4) {
                const float4 v = *reinterpret_cast<const float4 *>(src);
                acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
            } else {
                acc[0] += src[0];
            }
        }
    const float inv = 1.f / (float)(avg_valid(p, g.sh, g.ph, g.wh, g.H) * avg_valid(q, g.sw, g.pw, g.ww, g.W));
    float *dst = y + idx * VW;
    if constexpr (VW == 4) *reinterpret_cast<float4 *>(dst) = make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
    else dst[0] = acc[0] * inv;
}

// dx[n,h,w,:] = sum over the windows (p,q) that contain (h,w) of dy[n,p,q,:] / valid(p,q).  One thread per input pixel.
template <int VW>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const AvgGeo g, const float *__restrict__ dy, float *__restrict__ dx, size_t total)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cv = g.C / VW;
    const int c = (int)(idx % cv);
    size_t t = idx / cv;
    const int w = (int)(t % g.W); t /= g.W;
    const int h = (int)(t % g.H);
    const int n = (int)(t / g.H);
    // p*sh - ph <= h <= p*sh - ph + wh - 1
    const int p_lo = max((h + g.ph - g.wh + g.sh) / g.sh, 0), p_hi = min((h + g.ph) / g.sh, g.Ho - 1);
    const int q_lo = max((w + g.pw - g.ww + g.sw) / g.sw, 0), q_hi = min((w + g.pw) / g.sw, g.Wo - 1);
    float acc[VW];
#pragma unroll
    for (int e = 0; e < VW; ++e) acc[e] = 0.f;
    for (int p = p_lo; p <= p_hi; ++p) {
        const int nh = avg_valid(p, g.sh, g.ph, g.wh, g.H);
        for (int q = q_lo; q <= q_hi; ++q) {
            const float inv = 1.f / (float)(nh * avg_valid(q, g.sw, g.pw, g.ww, g.W));
            const float *src = dy + ((((size_t)n * g.Ho + p) * g.Wo + q) * cv + c) * VW;
            if constexpr (VW == 4) {
                const float4 v = *reinterpret_cast<const float4 *>(src);
                acc[0] = fmaf(v.x, inv, acc[0]); acc[1] = fmaf(v.y, inv, acc[1]);
                acc[2] = fmaf(v.z, inv, acc[2]); acc[3] = fmaf(v.w, inv, acc[3]);
            } else {
                acc[0] = fmaf(src[0], inv, acc[0]);
            }
        }
    }
    float *dst = dx + idx * VW;
    if constexpr (VW == 4) *reinterpret_cast<float4 *>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    else dst[0] = acc[0];
}

// bfloat16 forms of the two kernels above: 8 channels (16 bytes) per thread, sums in float32, one rounding at the store.
__device__ __forceinline__ float bf16_up(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint32_t bf16_down(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ void acc8(float (&acc)[8], const uint4 &v, float scale)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        acc[2 * e] = fmaf(bf16_up(w[e] & 0xffffu), scale, acc[2 * e]);
        acc[2 * e + 1] = fmaf(bf16_up(w[e] >> 16), scale, acc[2 * e + 1]);
    }
}
__device__ __forceinline__ uint4 pack8(const float (&a)[8], float scale)
{
    return make_uint4(bf16_down(a[0] * scale) | (bf16_down(a[1] * scale) << 16), bf16_down(a[2] * scale) | (bf16_down(a[3] * scale) << 16),
                      bf16_down(a[4] * scale) | (bf16_down(a[5] * scale) << 16), bf16_down(a[6] * scale) | (bf16_down(a[7] * scale) << 16));
}

__global__ __launch_bounds__(256) void avgpool_fwd_bf16_kernel(const AvgGeo g, const uint4 *__restrict__ x, uint4 *__restrict__ y, size_t total)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cv = g.C / 8;
    const int c = (int)(idx % cv);
    size_t t = idx / cv;
    const int q = (int)(t % g.Wo); t /= g.Wo;
    const int p = (int)(t % g.Ho);
    const int n = (int)(t / g.Ho);
    const int h0 = p * g.sh - g.ph, w0 = q * g.sw - g.pw;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int i = max(h0, 0); i < min(h0 + g.wh, g.H); ++i)
        for (int j = max(w0, 0); j < min(w0 + g.ww, g.W); ++j) acc8(acc, x[(((size_t)n * g.H + i) * g.W + j) * cv + c], 1.f);
    y[idx] = pack8(acc, 1.f / (float)(avg_valid(p, g.sh, g.ph, g.wh, g.H) * avg_valid(q, g.sw, g.pw, g.ww, g.W)));
}

__global__ __launch_bounds__(256) void avgpool_bwd_bf16_kernel(const AvgGeo g, const uint4 *__restrict__ dy, uint4 *__restrict__ dx, size_t total)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cv = g.C / 8;
    const int c = (int)(idx % cv);
    size_t t = idx / cv;
    const int w = (int)(t % g.W); t /= g.W;
    const int h = (int)(t % g.H);
    const int n = (int)(t / g.H);
    const int p_lo = max((h + g.ph - g.wh + g.sh) / g.sh, 0), p_hi = min((h + g.ph) / g.sh, g.Ho - 1);
    const int q_lo = max((w + g.pw - g.ww + g.sw) / g.sw, 0), q_hi = min((w + g.pw) / g.sw, g.Wo - 1);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int p = p_lo; p <= p_hi; ++p) {
        const int nh = avg_valid(p, g.sh, g.ph, g.wh, g.H);
        for (int q = q_lo; q <= q_hi; ++q)
            acc8(acc, dy[(((size_t)n * g.Ho + p) * g.Wo + q) * cv + c], 1.f / (float)(nh * avg_valid(q, g.sw, g.pw, g.ww, g.W)));
    }
    dx[idx] = pack8(acc, 1.f);
}

// dst[r*dst_ld + j] = src[r*src_ld + j], j < cols (all in elements of VW floats).
template <int VW>
__global__ __launch_bounds__(256) void copy2d_kernel(size_t total, int cols, size_t src_ld, size_t dst_ld, const float *__restrict__ src,
                                                     float *__restrict__ dst)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const size_t r = idx / cols;
    const int j = (int)(idx - r * cols);
    if constexpr (VW == 4)
        reinterpret_cast<float4 *>(dst)[r * dst_ld + j] = reinterpret_cast<const float4 *>(src)[r * src_ld + j];
    else
        dst[r * dst_ld + j] = src[r * src_ld + j];
}

static int avg_geometry(const stanza_pool_desc *d, AvgGeo *g)
{
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->win_h <= 0 || d->win_w <= 0) return STANZA_EINVAL;
    if (d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0) return STANZA_EINVAL;
    if (d->pad_h >= d->win_h || d->pad_w >= d->win_w) return STANZA_EINVAL;
    if (d->H + 2 * d->pad_h < d->win_h || d->W + 2 * d->pad_w < d->win_w) return STANZA_EINVAL;
    const int Ho = (d->H + 2 * d->pad_h - d->win_h) / d->stride_h + 1;
    const int Wo = (d->W + 2 * d->pad_w - d->win_w) / d->stride_w + 1;
    // every window must reach at least one pixel of the image (its mean is over the valid part)
    if ((Ho - 1) * d->stride_h - d->pad_h >= d->H || (Wo - 1) * d->stride_w - d->pad_w >= d->W) return STANZA_EINVAL;
    if ((int64_t)d->N * d->H * d->W * d->C >= (int64_t(1) << 31)) return STANZA_EINVAL;
    *g = AvgGeo{d->N, d->H, d->W, d->C, d->win_h, d->win_w, d->stride_h, d->stride_w, d->pad_h, d->pad_w, Ho, Wo};
    return STANZA_OK;
}

}  // namespace stanza

using namespace stanza;

extern "C" int stanza_avgpool_fwd(const stanza_pool_desc *desc, int32_t dtype, const void *x, void *y, void *stream)
{
    if (!desc) return STANZA_ENULL;
    AvgGeo g;
    int rc = avg_geometry(desc, &g);
    if (rc) return rc;
    if (dtype != STANZA_F32 && !(dtype == STANZA_BF16 && g.C % 8 == 0)) return STANZA_EUNSUPPORTED;
    if (!x || !y) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(y)) return STANZA_EALIGN;
    const size_t outs = (size_t)g.N * g.Ho * g.Wo * g.C;
    if (dtype == STANZA_BF16) {
        hipLaunchKernelGGL(avgpool_fwd_bf16_kernel, dim3((unsigned)cdiv64(outs / 8, 256)), dim3(256), 0, (hipStream_t)stream, g, (const uint4 *)x, (uint4 *)y,
                           outs / 8);
        return launch_status();
    }
    if (g.C % 4 == 0)
        hipLaunchKernelGGL(avgpool_fwd_kernel<4>, dim3((unsigned)cdiv64(outs / 4, 256)), dim3(256), 0, (hipStream_t)stream, g, (const float *)x, (float *)y, outs / 4);
    else
        hipLaunchKernelGGL(avgpool_fwd_kernel<1>, dim3((unsigned)cdiv64(outs, 256)), dim3(256), 0, (hipStream_t)stream, g, (const float *)x, (float *)y, outs);
    return launch_status();
}

extern "C" int stanza_avgpool_bwd(const stanza_pool_desc *desc, int32_t dtype, const void *dy, void *dx, void *stream)
{
    if (!desc) return STANZA_ENULL;
    AvgGeo g;
    int rc = avg_geometry(desc, &g);
    if (rc) return rc;
    if (dtype != STANZA_F32 && !(dtype == STANZA_BF16 && g.C % 8 == 0)) return STANZA_EUNSUPPORTED;
    if (!dy || !dx) return STANZA_ENULL;
    if (!aligned16(dy) || !aligned16(dx)) return STANZA_EALIGN;
    const size_t ins = (size_t)g.N * g.H * g.W * g.C;
    if (dtype == STANZA_BF16) {
        hipLaunchKernelGGL(avgpool_bwd_bf16_kernel, dim3((unsigned)cdiv64(ins / 8, 256)), dim3(256), 0, (hipStream_t)stream, g, (const uint4 *)dy, (uint4 *)dx,
                           ins / 8);
        return launch_status();
    }
    if (g.C % 4 == 0)
        hipLaunchKernelGGL(avgpool_bwd_kernel<4>, dim3((unsigned)cdiv64(ins / 4, 256)), dim3(256), 0, (hipStream_t)stream, g, (const float *)dy, (float *)dx, ins / 4);
    else
        hipLaunchKernelGGL(avgpool_bwd_kernel<1>, dim3((unsigned)cdiv64(ins, 256)), dim3(256), 0, (hipStream_t)stream, g, (const float *)dy, (float *)dx, ins);
    return launch_status();
}

extern "C" int stanza_copy2d(int64_t rows, int32_t cols, const float *src, int64_t src_ld, float *dst, int64_t dst_ld, void *stream)
{
    if (rows < 1 || cols < 1 || src_ld < cols || dst_ld < cols) return STANZA_EINVAL;
    if (rows * src_ld >= (int64_t(1) << 31) || rows * dst_ld >= (int64_t(1) << 31)) return STANZA_EINVAL;
    if (!src || !dst) return STANZA_ENULL;
    if ((reinterpret_cast<uintptr_t>(src) & 3u) || (reinterpret_cast<uintptr_t>(dst) & 3u)) return STANZA_EALIGN;
    const bool vec = cols % 4 == 0 && src_ld % 4 == 0 && dst_ld % 4 == 0 && aligned16(src) && aligned16(dst);
    if (vec) {
        const size_t total = (size_t)rows * (cols / 4);
        hipLaunchKernelGGL(copy2d_kernel<4>, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, (hipStream_t)stream, total, cols / 4, (size_t)src_ld / 4,
                           (size_t)dst_ld / 4, src, dst);
    } else {
        const size_t total = (size_t)rows * cols;
        hipLaunchKernelGGL(copy2d_kernel<1>, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, (hipStream_t)stream, total, cols, (size_t)src_ld, (size_t)dst_ld,
                           src, dst);
    }
    return launch_status();
}
