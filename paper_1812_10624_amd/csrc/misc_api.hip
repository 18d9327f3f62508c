// HBM-bound entry points: max-pool(+ReLU) forward/backward kept on the CONV worker (paper Sec. 3.2,
// note on the split point), the residual join and global average pool of the residual-network-shaped
// workload, bf16 casts, and the gradient aggregation + momentum-SGD update (Sec. 3.2: the CONV workers combine
// their gradients and update their replicas of the conv parameters; Sec. 2.2: server-side aggregation).  Every kernel moves each byte once with 16-byte accesses along the contiguous axis.
#include "internal.h"

#include <mutex>

namespace stanza {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}


// ------------------------------------------------------------------ max-pool (+ReLU)
struct PoolGeo {
    int N, H, W, C, wh, ww, sh, sw, ph, pw, Ho, Wo, relu;
};

// One thread per output pixel and group of VW channels.
template <int VW>
__global__ __launch_bounds__(256) void pool_fwd_kernel(const PoolGeo g, const float *__restrict__ x, float *__restrict__ y,
                                                       uint8_t *__restrict__ argmax, size_t total)
{
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= total) return;
    const int CV = g.C / VW;
    const int cv = (int)(id % CV);
    size_t pix = id / CV;
    const int q = (int)(pix % g.Wo);
    pix /= g.Wo;
    const int pp = (int)(pix % g.Ho);
    const int n = (int)(pix / g.Ho);
    float best[VW];
    int bidx[VW];
    bool found = false;
    for (int i = 0; i < g.wh; ++i) {
        const int h = pp * g.sh - g.ph + i;
        if ((unsigned)h >= (unsigned)g.H) continue;
        for (int j = 0; j < g.ww; ++j) {
            const int w = q * g.sw - g.pw + j;
            if ((unsigned)w >= (unsigned)g.W) continue;
            const float *src = x + (((size_t)n * g.H + h) * g.W + w) * g.C + cv * VW;
            float v[VW];
            if constexpr (VW == 4) {
                const float4 t = *reinterpret_cast<const float4 *>(src);
                v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
            } else {
                v[0] = src[0];
            }
#pragma unroll
            for (int e = 0; e < VW; ++e)
                if (!found || v[e] > best[e]) { best[e] = v[e]; bidx[e] = i * g.ww + j; }
            found = true;
        }
    }
    const size_t o = id * VW;
#pragma unroll
    for (int e = 0; e < VW; ++e)
        if (g.relu && best[e] < 0.f) best[e] = 0.f;
    if constexpr (VW == 4) {
        *reinterpret_cast<float4 *>(y + o) = make_float4(best[0], best[1], best[2], best[3]);
        if (argmax)
            *reinterpret_cast<uint32_t *>(argmax + o) =
                (uint32_t)bidx[0] | ((uint32_t)bidx[1] << 8) | ((uint32_t)bidx[2] << 16) | ((uint32_t)bidx[3] << 24);
    } else {
        y[o] = best[0];
        if (argmax) argmax[o] = (uint8_t)bidx[0];
    }
}

// One thread per input pixel and group of VW channels: gather over the windows that cover it.
template <int VW>
__global__ __launch_bounds__(256) void pool_bwd_kernel(const PoolGeo g, const float *__restrict__ dy, const float *__restrict__ y,
                                                       const uint8_t *__restrict__ argmax, float *__restrict__ dx, size_t total)
{
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= total) return;
    const int CV = g.C / VW;
    const int cv = (int)(id % CV);
    size_t pix = id / CV;
    const int w = (int)(pix % g.W);
    pix /= g.W;
    const int h = (int)(pix % g.H);
    const int n = (int)(pix / g.H);
    float acc[VW];
#pragma unroll
    for (int e = 0; e < VW; ++e) acc[e] = 0.f;
    for (int i = 0; i < g.wh; ++i) {
        const int hp = h + g.ph - i;
        if (hp < 0) break;
        const int pp = hp / g.sh;
        if (pp * g.sh != hp || pp >= g.Ho) continue;
        for (int j = 0; j < g.ww; ++j) {
            const int wq = w + g.pw - j;
            if (wq < 0) break;
            const int q = wq / g.sw;
            if (q * g.sw != wq || q >= g.Wo) continue;
            const size_t o = (((size_t)n * g.Ho + pp) * g.Wo + q) * g.C + cv * VW;
            const uint32_t code = (uint32_t)(i * g.ww + j);
            if constexpr (VW == 4) {
                const uint32_t am = *reinterpret_cast<const uint32_t *>(argmax + o);
                const float4 d = *reinterpret_cast<const float4 *>(dy + o);
                float4 yy = make_float4(1.f, 1.f, 1.f, 1.f);
                if (g.relu) yy = *reinterpret_cast<const float4 *>(y + o);
                if ((am & 255u) == code && yy.x > 0.f) acc[0] += d.x;
                if (((am >> 8) & 255u) == code && yy.y > 0.f) acc[1] += d.y;
                if (((am >> 16) & 255u) == code && yy.z > 0.f) acc[2] += d.z;
                if ((am >> 24) == code && yy.w > 0.f) acc[3] += d.w;
            } else {
                if (argmax[o] == code && (!g.relu || y[o] > 0.f)) acc[0] += dy[o];
            }
        }
    }
    const size_t o = id * VW;
    if constexpr (VW == 4)
        *reinterpret_cast<float4 *>(dx + o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    else
        dx[o] = acc[0];
}

// bfloat16 variants: 8 channels (16 bytes) per thread; bf16 -> f32 is exact, so the comparison is done in float
__device__ __forceinline__ float h2f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__global__ __launch_bounds__(256) void pool_fwd_bf16_kernel(const PoolGeo g, const uint16_t *__restrict__ x, uint16_t *__restrict__ y,
                                                            uint8_t *__restrict__ argmax, size_t total)
{
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= total) return;
    const int CV = g.C / 8;
    const int cv = (int)(id % CV);
    size_t pix = id / CV;
    const int q = (int)(pix % g.Wo);
    pix /= g.Wo;
    const int pp = (int)(pix % g.Ho);
    const int n = (int)(pix / g.Ho);
    uint16_t best[8];
    int bidx[8];
    bool found = false;
    for (int i = 0; i < g.wh; ++i) {
        const int h = pp * g.sh - g.ph + i;
        if ((unsigned)h >= (unsigned)g.H) continue;
        for (int j = 0; j < g.ww; ++j) {
            const int w = q * g.sw - g.pw + j;
            if ((unsigned)w >= (unsigned)g.W) continue;
            const uint4 tv = *reinterpret_cast<const uint4 *>(x + (((size_t)n * g.H + h) * g.W + w) * g.C + cv * 8);
            const uint16_t *v = reinterpret_cast<const uint16_t *>(&tv);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (!found || h2f(v[e]) > h2f(best[e])) { best[e] = v[e]; bidx[e] = i * g.ww + j; }
            found = true;
        }
    }
    const size_t o = id * 8;
    uint4 outv;
    uint16_t *ov = reinterpret_cast<uint16_t *>(&outv);
    uint32_t am[2] = {0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        ov[e] = (g.relu && h2f(best[e]) < 0.f) ? (uint16_t)0 : best[e];
        am[e >> 2] |= (uint32_t)bidx[e] << (8 * (e & 3));
    }
    *reinterpret_cast<uint4 *>(y + o) = outv;
    if (argmax) *reinterpret_cast<uint2 *>(argmax + o) = make_uint2(am[0], am[1]);
}

__global__ __launch_bounds__(256) void pool_bwd_bf16_kernel(const PoolGeo g, const uint16_t *__restrict__ dy, const uint16_t *__restrict__ y,
                                                            const uint8_t *__restrict__ argmax, uint16_t *__restrict__ dx, size_t total)
{
    const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= total) return;
    const int CV = g.C / 8;
    const int cv = (int)(id % CV);
    size_t pix = id / CV;
    const int w = (int)(pix % g.W);
    pix /= g.W;
    const int h = (int)(pix % g.H);
    const int n = (int)(pix / g.H);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int i = 0; i < g.wh; ++i) {
        const int hp = h + g.ph - i;
        if (hp < 0) break;
        const int pp = hp / g.sh;
        if (pp * g.sh != hp || pp >= g.Ho) continue;
        for (int j = 0; j < g.ww; ++j) {
            const int wq = w + g.pw - j;
            if (wq < 0) break;
            const int q = wq / g.sw;
            if (q * g.sw != wq || q >= g.Wo) continue;
            const size_t o = (((size_t)n * g.Ho + pp) * g.Wo + q) * g.C + cv * 8;
            const uint32_t code = (uint32_t)(i * g.ww + j);
            const uint2 am = *reinterpret_cast<const uint2 *>(argmax + o);
            const uint4 dv = *reinterpret_cast<const uint4 *>(dy + o);
            const uint16_t *d = reinterpret_cast<const uint16_t *>(&dv);
            uint4 yv = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);   // 1.0: no gate
            if (g.relu) yv = *reinterpret_cast<const uint4 *>(y + o);
            const uint16_t *yy = reinterpret_cast<const uint16_t *>(&yv);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t a = ((e < 4 ? am.x : am.y) >> (8 * (e & 3))) & 255u;
                if (a == code && h2f(yy[e]) > 0.f) acc[e] += h2f(d[e]);
            }
        }
    }
    uint4 outv;
    uint16_t *ov = reinterpret_cast<uint16_t *>(&outv);
#pragma unroll
    for (int e = 0; e < 8; ++e) ov[e] = f32_to_bf16_rne(acc[e]);
    *reinterpret_cast<uint4 *>(dx + id * 8) = outv;
}

// ---- non-overlapping windows (window == stride, no padding, image a whole number of windows: every pool of the
// VGG-16-shaped and tiny stacks).  One thread per OUTPUT pixel and 16-byte channel vector, in both directions: forward reads
// its window, backward reads dy / y / argmax once and writes the window's input pixels (the gather form above reads them once
// per input pixel, four times for a 2x2 window).  grid = (vectors of an output row / 256, N*Ho); 32-bit index arithmetic, one
// multiply-shift division per thread; every access is non-temporal (each byte is touched once).
typedef unsigned int pool_u4 __attribute__((ext_vector_type(4)));
template <bool BF16>
__global__ __launch_bounds__(256) void pool_fwd_tiled_kernel(const PoolGeo g, FastDiv fd_cv, const void *__restrict__ xv, void *__restrict__ yv,
                                                             uint8_t *__restrict__ argmax)
{
    constexpr int VW = BF16 ? 8 : 4;
    const int CV = g.C / VW;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= g.Wo * CV) return;
    const int q = fdiv(idx, fd_cv), cv = idx - q * CV;
    const int np = blockIdx.y, n = np / g.Ho, pp = np - n * g.Ho;
    const pool_u4 *x = reinterpret_cast<const pool_u4 *>(xv);
    float best[VW];
    uint32_t braw[VW];
    int bidx[VW];
    for (int i = 0; i < g.wh; ++i) {
        for (int j = 0; j < g.ww; ++j) {
            const size_t off = (((size_t)n * g.H + pp * g.sh + i) * g.W + q * g.sw + j) * CV + cv;
            const pool_u4 t = __builtin_nontemporal_load(x + off);
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const uint32_t raw = BF16 ? ((t[e >> 1] >> (16 * (e & 1))) & 0xffffu) : t[e];
                const float v = BF16 ? __uint_as_float(raw << 16) : __uint_as_float(raw);
                if ((i == 0 && j == 0) || v > best[e]) { best[e] = v; braw[e] = raw; bidx[e] = i * g.ww + j; }
            }
        }
    }
    const size_t o = ((size_t)np * g.Wo + q) * CV + cv;      // in 16-byte vectors
    pool_u4 out = {0u, 0u, 0u, 0u};
    uint32_t am[2] = {0u, 0u};
#pragma unroll
    for (int e = 0; e < VW; ++e) {
        const uint32_t raw = (g.relu && best[e] < 0.f) ? 0u : braw[e];
        if (BF16) out[e >> 1] |= raw << (16 * (e & 1)); else out[e] = raw;
        am[e >> 2] |= (uint32_t)bidx[e] << (8 * (e & 3));
    }
    __builtin_nontemporal_store(out, reinterpret_cast<pool_u4 *>(yv) + o);
    if (argmax) {
        if (BF16) *reinterpret_cast<uint2 *>(argmax + o * 8) = make_uint2(am[0], am[1]);
        else *reinterpret_cast<uint32_t *>(argmax + o * 4) = am[0];
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void pool_bwd_tiled_kernel(const PoolGeo g, FastDiv fd_cv, const void *__restrict__ dyv, const void *__restrict__ yv,
                                                             const uint8_t *__restrict__ argmax, void *__restrict__ dxv)
{
    constexpr int VW = BF16 ? 8 : 4;
    const int CV = g.C / VW;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= g.Wo * CV) return;
    const int q = fdiv(idx, fd_cv), cv = idx - q * CV;
    const int np = blockIdx.y, n = np / g.Ho, pp = np - n * g.Ho;
    const size_t o = ((size_t)np * g.Wo + q) * CV + cv;
    const pool_u4 d = __builtin_nontemporal_load(reinterpret_cast<const pool_u4 *>(dyv) + o);
    pool_u4 gate = d;
    if (g.relu) {
        const pool_u4 yy = __builtin_nontemporal_load(reinterpret_cast<const pool_u4 *>(yv) + o);
        // keep dy where y > 0: a positive finite float / bfloat16 has a non-zero pattern with the sign bit clear
#pragma unroll
        for (int e = 0; e < VW; ++e) {
            if (BF16) {
                const uint32_t h = (yy[e >> 1] >> (16 * (e & 1))) & 0xffffu;
                if (h == 0u || (h & 0x8000u)) gate[e >> 1] &= ~(0xffffu << (16 * (e & 1)));
            } else {
                if (!(__uint_as_float(yy[e]) > 0.f)) gate[e] = 0u;
            }
        }
    }
    uint32_t am[2];
    if (BF16) { const uint2 a = *reinterpret_cast<const uint2 *>(argmax + o * 8); am[0] = a.x; am[1] = a.y; }
    else { am[0] = *reinterpret_cast<const uint32_t *>(argmax + o * 4); am[1] = 0u; }
    pool_u4 *dx = reinterpret_cast<pool_u4 *>(dxv);
    for (int i = 0; i < g.wh; ++i) {
        for (int j = 0; j < g.ww; ++j) {
            const uint32_t code = (uint32_t)(i * g.ww + j);
            pool_u4 out = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const bool hit = ((am[e >> 2] >> (8 * (e & 3))) & 255u) == code;
                if (BF16) out[e >> 1] |= hit ? (gate[e >> 1] & (0xffffu << (16 * (e & 1)))) : 0u;
                else out[e] = hit ? gate[e] : 0u;
            }
            const size_t off = (((size_t)n * g.H + pp * g.sh + i) * g.W + q * g.sw + j) * CV + cv;
            __builtin_nontemporal_store(out, dx + off);
        }
    }
}

static bool pool_is_tiled(const PoolGeo &g, int vw)
{
    return g.wh == g.sh && g.ww == g.sw && g.ph == 0 && g.pw == 0 && g.H % g.wh == 0 && g.W % g.ww == 0 && g.C % vw == 0 &&
           (int64_t)g.N * g.Ho <= 65535;      // rows of the output ride on gridDim.y
}

static int pool_geometry(const stanza_pool_desc *d, PoolGeo *g)
{
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->win_h <= 0 || d->win_w <= 0) return STANZA_EINVAL;
    if (d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0) return STANZA_EINVAL;
    if (d->pad_h >= d->win_h || d->pad_w >= d->win_w || d->win_h * d->win_w > 255) return STANZA_EINVAL;
    if (d->H + 2 * d->pad_h < d->win_h || d->W + 2 * d->pad_w < d->win_w) return STANZA_EINVAL;
    const int Ho = (d->H + 2 * d->pad_h - d->win_h) / d->stride_h + 1;
    const int Wo = (d->W + 2 * d->pad_w - d->win_w) / d->stride_w + 1;
    // every window must reach at least one pixel of the image (clipped windows are never empty)
    if ((Ho - 1) * d->stride_h - d->pad_h >= d->H || (Wo - 1) * d->stride_w - d->pad_w >= d->W) return STANZA_EINVAL;
    if ((int64_t)d->N * d->H * d->W * d->C >= (int64_t(1) << 31)) return STANZA_EINVAL;
    *g = PoolGeo{d->N, d->H, d->W, d->C, d->win_h, d->win_w, d->stride_h, d->stride_w, d->pad_h, d->pad_w, Ho, Wo,
                 (d->flags & STANZA_POOL_RELU) ? 1 : 0};
    return STANZA_OK;
}

// ------------------------------------------------------------------ residual join, global average pool
__global__ __launch_bounds__(256) void add_relu_fwd_kernel(size_t n4, size_t numel, const float *__restrict__ a, const float *__restrict__ b,
                                                           float *__restrict__ o)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) {
        const float4 x = reinterpret_cast<const float4 *>(a)[i], y = reinterpret_cast<const float4 *>(b)[i];
        reinterpret_cast<float4 *>(o)[i] =
            make_float4(fmaxf(x.x + y.x, 0.f), fmaxf(x.y + y.y, 0.f), fmaxf(x.z + y.z, 0.f), fmaxf(x.w + y.w, 0.f));
    } else if (i == n4) {
        for (size_t j = n4 * 4; j < numel; ++j) o[j] = fmaxf(a[j] + b[j], 0.f);
    }
}

__global__ __launch_bounds__(256) void add_relu_bwd_kernel(size_t n4, size_t numel, const float *__restrict__ dout,
                                                           const float *__restrict__ o, float *__restrict__ dz)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) {
        const float4 d = reinterpret_cast<const float4 *>(dout)[i], y = reinterpret_cast<const float4 *>(o)[i];
        reinterpret_cast<float4 *>(dz)[i] = gate4(d, y);
    } else if (i == n4) {
        for (size_t j = n4 * 4; j < numel; ++j) dz[j] = o[j] > 0.f ? dout[j] : 0.f;
    }
}

__global__ void gap_fwd_kernel(int N, int HW, int C, const float *__restrict__ x, float *__restrict__ f)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x, n = blockIdx.y;
    if (c >= C) return;
    float s = 0.f;
    for (int i = 0; i < HW; ++i) s += x[((size_t)n * HW + i) * C + c];
    f[(size_t)n * C + c] = s / (float)HW;
}

__global__ void gap_bwd_kernel(size_t total, int HW, int C, const float *__restrict__ df, float *__restrict__ dx)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % C);
    const size_t n = i / ((size_t)HW * C);
    dx[i] = df[n * C + c] / (float)HW;
}

// bf16 forms (numel % 8 == 0: channel counts of a bf16 stack are multiples of 8): 8 elements per thread, float32 arithmetic,
// one rounding on store.
__global__ __launch_bounds__(256) void add_relu_fwd_bf16_kernel(size_t n8, const uint4 *__restrict__ a, const uint4 *__restrict__ b, uint4 *__restrict__ o)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const uint4 x = a[i], y = b[i];
    const uint32_t *px = reinterpret_cast<const uint32_t *>(&x), *py = reinterpret_cast<const uint32_t *>(&y);
    uint4 r;
    uint32_t *pr = reinterpret_cast<uint32_t *>(&r);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float lo = fmaxf(__uint_as_float(px[w] << 16) + __uint_as_float(py[w] << 16), 0.f);
        const float hi = fmaxf(__uint_as_float(px[w] & 0xffff0000u) + __uint_as_float(py[w] & 0xffff0000u), 0.f);
        pr[w] = (uint32_t)f32_to_bf16_rne(lo) | ((uint32_t)f32_to_bf16_rne(hi) << 16);
    }
    o[i] = r;
}

__global__ __launch_bounds__(256) void add_relu_bwd_bf16_kernel(size_t n8, const uint4 *__restrict__ dout, const uint4 *__restrict__ o, uint4 *__restrict__ dz)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    uint4 d = dout[i];
    const uint4 y = o[i];
    uint32_t *pd = reinterpret_cast<uint32_t *>(&d);
    const uint32_t *py = reinterpret_cast<const uint32_t *>(&y);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        // o = max(.,0) is never negative: an element is positive iff its bits are non-zero (and not -0)
        const uint32_t lo = (py[w] & 0x7fffu) != 0 && !(py[w] & 0x8000u) ? 0x0000ffffu : 0u;
        const uint32_t hi = (py[w] & 0x7fff0000u) != 0 && !(py[w] & 0x80000000u) ? 0xffff0000u : 0u;
        pd[w] &= lo | hi;
    }
    dz[i] = d;
}

__global__ void gap_fwd_bf16_kernel(int N, int HW, int C, const uint16_t *__restrict__ x, float *__restrict__ f)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x, n = blockIdx.y;
    if (c >= C) return;
    float s = 0.f;
    for (int i = 0; i < HW; ++i) s += __uint_as_float((uint32_t)x[((size_t)n * HW + i) * C + c] << 16);
    f[(size_t)n * C + c] = s / (float)HW;
}

__global__ void gap_bwd_bf16_kernel(size_t total, int HW, int C, const float *__restrict__ df, uint16_t *__restrict__ dx)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % C);
    const size_t n = i / ((size_t)HW * C);
    dx[i] = f32_to_bf16_rne(df[n * C + c] / (float)HW);
}

// ------------------------------------------------------------------ bf16 casts
// A workgroup converts one block of CAST_CHUNK elements.  A full block of 16-byte-aligned tensors: 16 elements per thread as two
// runs of 8 (four 16-byte loads and two 16-byte stores, or the reverse), every access of a wavefront contiguous.  The last block
// of a tensor, and tensors that are not 16-byte aligned: element by element.
constexpr int CAST_CHUNK = 4096;
__device__ __forceinline__ void cast_block_f32_bf16(const float *__restrict__ s, uint16_t *__restrict__ d, int64_t left, bool vec)
{
    if (vec && left >= CAST_CHUNK) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int e0 = h * 2048 + threadIdx.x * 8;
            const float4 a = *reinterpret_cast<const float4 *>(s + e0), b = *reinterpret_cast<const float4 *>(s + e0 + 4);
            uint4 o;
            o.x = (uint32_t)f32_to_bf16_rne(a.x) | ((uint32_t)f32_to_bf16_rne(a.y) << 16);
            o.y = (uint32_t)f32_to_bf16_rne(a.z) | ((uint32_t)f32_to_bf16_rne(a.w) << 16);
            o.z = (uint32_t)f32_to_bf16_rne(b.x) | ((uint32_t)f32_to_bf16_rne(b.y) << 16);
            o.w = (uint32_t)f32_to_bf16_rne(b.z) | ((uint32_t)f32_to_bf16_rne(b.w) << 16);
            *reinterpret_cast<uint4 *>(d + e0) = o;
        }
    } else {
        const int n = (int)(left < CAST_CHUNK ? left : CAST_CHUNK);
        for (int i = threadIdx.x; i < n; i += 256) d[i] = f32_to_bf16_rne(s[i]);
    }
}

__global__ __launch_bounds__(256) void cast_f32_bf16_kernel(size_t numel, const float *__restrict__ src, uint16_t *__restrict__ dst, int vec)
{
    const size_t base = (size_t)blockIdx.x * CAST_CHUNK;
    cast_block_f32_bf16(src + base, dst + base, (int64_t)(numel - base), vec != 0);
}

__global__ __launch_bounds__(256) void cast_bf16_f32_kernel(size_t numel, const uint16_t *__restrict__ src, float *__restrict__ dst, int vec)
{
    const size_t base = (size_t)blockIdx.x * CAST_CHUNK;
    const uint16_t *__restrict__ s = src + base;
    float *__restrict__ d = dst + base;
    const size_t left = numel - base;
    if (vec && left >= CAST_CHUNK) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int e0 = h * 2048 + threadIdx.x * 8;
            const uint4 v = *reinterpret_cast<const uint4 *>(s + e0);
            *reinterpret_cast<float4 *>(d + e0) = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                                                              __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
            *reinterpret_cast<float4 *>(d + e0 + 4) = make_float4(__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xffff0000u),
                                                                  __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xffff0000u));
        }
    } else {
        const int n = (int)(left < CAST_CHUNK ? left : CAST_CHUNK);
        for (int i = threadIdx.x; i < n; i += 256) d[i] = __uint_as_float((uint32_t)s[i] << 16);
    }
}

// A small table of 8-byte words (element counts and device pointers) reaches device memory INSIDE kernel arguments: the launch
// copies them into its argument buffer, so the host arrays may be freed when the call returns, nothing is allocated or staged
// on the host, no copy engine is involved and nothing waits; under stream capture the words become part of the graph node.
// A table longer than one launch's argument space goes out in several launches, in order, on the same stream.
constexpr int FILL_WORDS = 480;            // 3,840 bytes of the 4 KB a launch may carry
struct FillChunk {
    uint64_t w[FILL_WORDS];
};

__global__ __launch_bounds__(256) void table_fill_kernel(uint64_t *__restrict__ dst, int count, const FillChunk c)
{
    for (int i = threadIdx.x; i < count; i += 256) dst[i] = c.w[i];
}

class TableWriter {
public:
    TableWriter(void *dst, hipStream_t st) : dst_((uint64_t *)dst), st_(st) {}
    void push(uint64_t word)
    {
        chunk_.w[n_++] = word;
        if (n_ == FILL_WORDS) flush();
    }
    void push_ptr(const void *ptr) { push((uint64_t)reinterpret_cast<uintptr_t>(ptr)); }
    void flush()
    {
        if (n_ == 0) return;
        hipLaunchKernelGGL(table_fill_kernel, dim3(1), dim3(256), 0, st_, dst_, n_, chunk_);
        dst_ += n_;
        n_ = 0;
    }

private:
    uint64_t *dst_;
    hipStream_t st_;
    int n_ = 0;
    FillChunk chunk_;
};

// Many tensors in one launch (the per-step bf16 copies of all master filters of a CONV worker: one launch instead of one per
// layer).  Table in device memory, built by stanza_cast_plan:
//   int64 chunk_prefix[n + 1]   exclusive prefix of per-tensor block counts (CAST_CHUNK elements each)
//   int64 numel[n];  const float *src[n];  uint16 *dst[n]          (16-byte aligned: checked by stanza_cast_plan)
__global__ __launch_bounds__(256) void cast_f32_bf16_multi_kernel(const void *ws, int n)
{
    const int64_t *prefix = (const int64_t *)ws;
    const int64_t *numel = prefix + (n + 1);
    const float *const *src = (const float *const *)(numel + n);
    uint16_t *const *dst = (uint16_t *const *)(src + n);
    const int64_t chunk = blockIdx.x;
    int lo = 0, hi = n;                      // largest t with prefix[t] <= chunk
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (prefix[mid] <= chunk) lo = mid; else hi = mid;
    }
    const int64_t base = (chunk - prefix[lo]) * CAST_CHUNK;
    cast_block_f32_bf16(src[lo] + base, dst[lo] + base, numel[lo] - base, true);
}

// ------------------------------------------------------------------ aggregation + momentum SGD
// Table in device memory (built by stanza_ps_plan):
//   int64 chunk_prefix[n_tensors + 1]   exclusive prefix of per-tensor chunk counts (PS_CHUNK elements each)
//   int64 numel[n_tensors]
//   float* w[n_tensors], v[n_tensors]
//   const float* grads[K * n_tensors]   shard-major
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
#ifndef STANZA_PS_CHUNK
#define STANZA_PS_CHUNK 4096
#endif
// Every access of the full-chunk path is a 16-byte buffer load / store with the non-temporal bit: each byte is touched
// once per call, so nothing is worth keeping in L2.  Measured on a 123.6 M-parameter set at K = 16: plain global
// loads and stores 5.2 TB/s, non-temporal global loads 5.5, non-temporal buffer loads and stores 6.0.
constexpr int PS_NT = 2;   // cache-policy operand of the buffer intrinsics: bit 1 = nt
__device__ __forceinline__ __amdgpu_buffer_rsrc_t ps_rsrc(const float *ptr)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(ptr), 0, STANZA_PS_CHUNK * 4, 0x00020000);
}
#ifndef STANZA_PS_THREADS
#define STANZA_PS_THREADS 128
#endif
// 128 threads x 8 vectors move the same 16 KB per stream and workgroup as 256 x 4 did, 1.5 % faster on the 123.6 M-parameter
// set at K = 16 (0.695 -> 0.707 of the HBM peak; 64 x 16 the same; any other chunk size, with either shape, is slower)
constexpr int PS_T = STANZA_PS_THREADS;    // threads per workgroup
constexpr int PS_CHUNK = STANZA_PS_CHUNK;  // elements per workgroup: PS_T threads x PS_CHUNK/(4 PS_T) vectors of 4

struct PsTable {
    const int64_t *prefix;
    const int64_t *numel;
    float *const *w;
    float *const *v;
    const float *const *grads;
};

__host__ __device__ inline PsTable ps_table_at(const void *ws, int n_tensors)
{
    const char *b = (const char *)ws;
    PsTable t;
    t.prefix = (const int64_t *)b;
    t.numel = t.prefix + (n_tensors + 1);
    t.w = (float *const *)(t.numel + n_tensors);
    t.v = t.w + n_tensors;
    t.grads = (const float *const *)(t.v + n_tensors);
    return t;
}

// Order in which the K shards are added.  Index order: ((g_0 + g_1) + g_2) + ...  Recursive doubling (Sec. 4.1.2): the
// sum every worker holds after the all-reduce in which, in round i, worker j adds what worker j xor 2^(i-1) holds to its
// own: a balanced pairwise tree over the P = 2^floor(log2 K) workers that take part, ((g_0+g_1)+(g_2+g_3))+..., where
// worker i < K - P has first added the gradient that surplus worker P + i sent it.  Floating-point addition is
// commutative, so all workers hold the same bits, and one tree gives them.
enum { PS_ORDER_INDEX = 0, PS_ORDER_RD = 1 };

// Balanced tree over leaves [LO, LO + N) with compile-time shape; leaf(k, out) loads shard k.
template <int LO, int N, int P, int R, class V, class Leaf>
__device__ __forceinline__ void ps_tree(Leaf &leaf, V &out)
{
    if constexpr (N == 1) {
        leaf(LO, out);
        if constexpr (LO < R) {
            V extra;
            leaf(P + LO, extra);
            out += extra;
        }
    } else {
        ps_tree<LO, N / 2, P, R>(leaf, out);
        V right;
        ps_tree<LO + N / 2, N / 2, P, R>(leaf, right);
        out += right;
    }
}

constexpr int ps_floor_pow2(int k) { int p = 1; while (p * 2 <= k) p *= 2; return p; }

// Sum of the K shards in the requested order.  V: a value type with += (a float or a pack of vectors).
template <int KFIX, int ORDER, class V, class Leaf>
__device__ __forceinline__ void ps_shard_sum(int K, Leaf &leaf, V &out)
{
    if constexpr (ORDER == PS_ORDER_INDEX) {
        const int kk = KFIX > 0 ? KFIX : K;
        leaf(0, out);
#pragma unroll
        for (int k = 1; k < kk; ++k) {
            V x;
            leaf(k, x);
            out += x;
        }
    } else if constexpr (KFIX > 0) {
        constexpr int P = ps_floor_pow2(KFIX);
        ps_tree<0, P, P, KFIX - P>(leaf, out);
    } else {
        // run-time K: leaves enter a binary counter of partial sums (slot l holds the sum of a finished block of 2^l
        // leaves); all slot indices are compile-time so the slots stay in registers.
        constexpr int LEVELS = 13;   // K <= 4096
        int P = 1, m = 0;
        while (P * 2 <= K) { P *= 2; ++m; }
        const int R = K - P;
        V slot[LEVELS];
        for (int i = 0; i < P; ++i) {
            V x;
            leaf(i, x);
            if (i < R) {
                V extra;
                leaf(P + i, extra);
                x += extra;
            }
            bool placed = false;
#pragma unroll
            for (int l = 0; l < LEVELS; ++l) {
                if (!placed) {
                    if ((i >> l) & 1) { V left = slot[l]; left += x; x = left; }
                    else { slot[l] = x; placed = true; }
                }
            }
        }
#pragma unroll
        for (int l = 0; l < LEVELS; ++l)
            if (l == m) out = slot[l];
    }
}

template <int U>
struct PsPack {
    v4f x[U];
    __device__ __forceinline__ PsPack &operator+=(const PsPack &o)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] += o.x[u];
        return *this;
    }
};

template <int KFIX, int ORDER>
__global__ __launch_bounds__(PS_T) void ps_aggregate_kernel(const void *ws, int n_tensors, int K, float scale, float lr, float mom, float wd)
{
    const PsTable tb = ps_table_at(ws, n_tensors);
    const int64_t chunk = blockIdx.x;
    // Tensor of this chunk: largest t with prefix[t] <= chunk.  Up to 64 tensors (a CNN's conv or FC parameter set) the
    // lanes of a wavefront test one prefix each and count: one memory latency before the shard loads can be issued instead
    // of the log2(n) dependent ones of a binary search.
    int t;
    if (n_tensors <= 64) {
        const int lane = threadIdx.x & 63;
        const bool le = lane < n_tensors && tb.prefix[lane] <= chunk;
        t = __popcll(__ballot(le)) - 1;
    } else {
        int lo = 0, hi = n_tensors;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tb.prefix[mid] <= chunk) lo = mid; else hi = mid;
        }
        t = lo;
    }
    const int64_t numel = tb.numel[t];
    const int64_t base = (chunk - tb.prefix[t]) * PS_CHUNK;
    float *__restrict__ w = tb.w[t];
    float *__restrict__ v = tb.v[t];
    const float *const *gp = tb.grads + t;   // shard k at gp[k * n_tensors]
    constexpr int U = PS_CHUNK / (4 * PS_T);   // vectors per thread; all of their loads are issued before any store
    if (base + PS_CHUNK <= numel) {
        // One buffer descriptor per stream, based at this workgroup's chunk (wavefront-uniform), so tensors of any size
        // are addressed with a 32-bit in-chunk offset.
        const uint32_t off = threadIdx.x * 16u;
        auto leaf = [&](int k, PsPack<U> &out) {
            const __amdgpu_buffer_rsrc_t rg = ps_rsrc(gp[(size_t)k * n_tensors] + base);
#pragma unroll
            for (int u = 0; u < U; ++u) out.x[u] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rg, off + u * (PS_T * 16u), 0, PS_NT));
        };
        PsPack<U> s;
        ps_shard_sum<KFIX, ORDER>(K, leaf, s);
        v4f wv[U], vv[U];
        const __amdgpu_buffer_rsrc_t rw = ps_rsrc(w + base), rv = ps_rsrc(v + base);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            wv[u] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rw, off + u * (PS_T * 16u), 0, PS_NT));
            vv[u] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rv, off + u * (PS_T * 16u), 0, PS_NT));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            v4f a = vv[u], b = wv[u];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a[e] = mom * a[e] + (scale * s.x[u][e] + wd * b[e]);
                b[e] -= lr * a[e];
            }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, a), rv, off + u * (PS_T * 16u), 0, PS_NT);
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, b), rw, off + u * (PS_T * 16u), 0, PS_NT);
        }
    } else {
        // ragged last chunk of a tensor: scalar, same summation order
        for (int64_t j = base + threadIdx.x; j < numel; j += PS_T) {
            auto leaf = [&](int k, float &out) { out = gp[(size_t)k * n_tensors][j]; };
            float sum;
            ps_shard_sum<0, ORDER>(K, leaf, sum);
            const float wj = w[j];
            const float vel = mom * v[j] + (scale * sum + wd * wj);
            v[j] = vel;
            w[j] = wj - lr * vel;
        }
    }
}

}  // namespace stanza

using namespace stanza;

extern "C" const char *stanza_strerror(int status)
{
    switch (status) {
    case STANZA_OK: return "ok";
    case STANZA_EINVAL: return "invalid size, stride, pad or count";
    case STANZA_ENULL: return "required pointer is NULL";
    case STANZA_EALIGN: return "pointer is not 16-byte aligned";
    case STANZA_EUNSUPPORTED: return "unsupported dtype or shape";
    case STANZA_EWORKSPACE: return "workspace too small";
    case STANZA_EHIP: return "HIP runtime error at launch";
    case STANZA_ECAPACITY: return "input exceeds the fixed capacity of an entry point that allocates nothing";
    }
    return "unknown status";
}

extern "C" int stanza_version(void) { return 100; }

extern "C" int stanza_pool_relu_fwd(const stanza_pool_desc *desc, int32_t dtype, const void *x, void *y, uint8_t *argmax, void *stream)
{
    if (!desc) return STANZA_ENULL;
    PoolGeo g;
    int rc = pool_geometry(desc, &g);
    if (rc) return rc;
    if (dtype != STANZA_F32 && !(dtype == STANZA_BF16 && g.C % 8 == 0)) return STANZA_EUNSUPPORTED;
    if (!x || !y) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(y) || (reinterpret_cast<uintptr_t>(argmax) & 7u)) return STANZA_EALIGN;
    hipStream_t st = (hipStream_t)stream;
    const size_t outs = (size_t)g.N * g.Ho * g.Wo * g.C;
    if (pool_is_tiled(g, dtype == STANZA_BF16 ? 8 : 4)) {
        const int cv = g.C / (dtype == STANZA_BF16 ? 8 : 4);
        const dim3 grid((unsigned)cdiv(g.Wo * cv, 256), (unsigned)(g.N * g.Ho));
        if (dtype == STANZA_BF16)
            hipLaunchKernelGGL(pool_fwd_tiled_kernel<true>, grid, dim3(256), 0, st, g, make_fastdiv(cv), x, y, argmax);
        else
            hipLaunchKernelGGL(pool_fwd_tiled_kernel<false>, grid, dim3(256), 0, st, g, make_fastdiv(cv), x, y, argmax);
        return launch_status();
    }
    if (dtype == STANZA_BF16) {
        const size_t total = outs / 8;
        hipLaunchKernelGGL(pool_fwd_bf16_kernel, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, st, g, (const uint16_t *)x, (uint16_t *)y, argmax, total);
        return launch_status();
    }
    if (g.C % 4 == 0) {
        const size_t total = outs / 4;
        hipLaunchKernelGGL(pool_fwd_kernel<4>, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, st, g, (const float *)x, (float *)y, argmax, total);
    } else {
        hipLaunchKernelGGL(pool_fwd_kernel<1>, dim3((unsigned)cdiv64(outs, 256)), dim3(256), 0, st, g, (const float *)x, (float *)y, argmax, outs);
    }
    return launch_status();
}

extern "C" int stanza_pool_relu_bwd(const stanza_pool_desc *desc, int32_t dtype, const void *dy, const void *y, const uint8_t *argmax,
                                    void *dx, void *stream)
{
    if (!desc) return STANZA_ENULL;
    PoolGeo g;
    int rc = pool_geometry(desc, &g);
    if (rc) return rc;
    if (dtype != STANZA_F32 && !(dtype == STANZA_BF16 && g.C % 8 == 0)) return STANZA_EUNSUPPORTED;
    if (!dy || !argmax || !dx || (g.relu && !y)) return STANZA_ENULL;
    if (!aligned16(dy) || !aligned16(dx) || !aligned16(y) || (reinterpret_cast<uintptr_t>(argmax) & 7u)) return STANZA_EALIGN;
    hipStream_t st = (hipStream_t)stream;
    const size_t ins = (size_t)g.N * g.H * g.W * g.C;
    if (pool_is_tiled(g, dtype == STANZA_BF16 ? 8 : 4)) {
        const int cv = g.C / (dtype == STANZA_BF16 ? 8 : 4);
        const dim3 grid((unsigned)cdiv(g.Wo * cv, 256), (unsigned)(g.N * g.Ho));
        if (dtype == STANZA_BF16)
            hipLaunchKernelGGL(pool_bwd_tiled_kernel<true>, grid, dim3(256), 0, st, g, make_fastdiv(cv), dy, y, argmax, dx);
        else
            hipLaunchKernelGGL(pool_bwd_tiled_kernel<false>, grid, dim3(256), 0, st, g, make_fastdiv(cv), dy, y, argmax, dx);
        return launch_status();
    }
    if (dtype == STANZA_BF16) {
        const size_t total = ins / 8;
        hipLaunchKernelGGL(pool_bwd_bf16_kernel, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, st, g, (const uint16_t *)dy, (const uint16_t *)y, argmax,
                           (uint16_t *)dx, total);
        return launch_status();
    }
    if (g.C % 4 == 0) {
        const size_t total = ins / 4;
        hipLaunchKernelGGL(pool_bwd_kernel<4>, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, st, g, (const float *)dy, (const float *)y, argmax,
                           (float *)dx, total);
    } else {
        hipLaunchKernelGGL(pool_bwd_kernel<1>, dim3((unsigned)cdiv64(ins, 256)), dim3(256), 0, st, g, (const float *)dy, (const float *)y, argmax,
                           (float *)dx, ins);
    }
    return launch_status();
}

static int ew_check(int64_t numel, int32_t dtype, const void *a, const void *b, const void *c)
{
    if (numel <= 0 || numel >= (int64_t(1) << 31)) return STANZA_EINVAL;
    if (dtype != STANZA_F32 && !(dtype == STANZA_BF16 && numel % 8 == 0)) return STANZA_EUNSUPPORTED;
    if (!a || !b || !c) return STANZA_ENULL;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return STANZA_EALIGN;
    return STANZA_OK;
}

extern "C" int stanza_add_relu_fwd(int64_t numel, int32_t dtype, const void *a, const void *b, void *o, void *stream)
{
    int rc = ew_check(numel, dtype, a, b, o);
    if (rc) return rc;
    if (dtype == STANZA_BF16) {
        const size_t n8 = (size_t)numel / 8;
        hipLaunchKernelGGL(add_relu_fwd_bf16_kernel, dim3((unsigned)cdiv64(n8, 256)), dim3(256), 0, (hipStream_t)stream, n8, (const uint4 *)a,
                           (const uint4 *)b, (uint4 *)o);
        return launch_status();
    }
    const size_t n4 = (size_t)numel / 4;
    hipLaunchKernelGGL(add_relu_fwd_kernel, dim3((unsigned)cdiv64(n4 + 1, 256)), dim3(256), 0, (hipStream_t)stream, n4, (size_t)numel,
                       (const float *)a, (const float *)b, (float *)o);
    return launch_status();
}

extern "C" int stanza_add_relu_bwd(int64_t numel, int32_t dtype, const void *dout, const void *o, void *dz, void *stream)
{
    int rc = ew_check(numel, dtype, dout, o, dz);
    if (rc) return rc;
    if (dtype == STANZA_BF16) {
        const size_t n8 = (size_t)numel / 8;
        hipLaunchKernelGGL(add_relu_bwd_bf16_kernel, dim3((unsigned)cdiv64(n8, 256)), dim3(256), 0, (hipStream_t)stream, n8, (const uint4 *)dout,
                           (const uint4 *)o, (uint4 *)dz);
        return launch_status();
    }
    const size_t n4 = (size_t)numel / 4;
    hipLaunchKernelGGL(add_relu_bwd_kernel, dim3((unsigned)cdiv64(n4 + 1, 256)), dim3(256), 0, (hipStream_t)stream, n4, (size_t)numel,
                       (const float *)dout, (const float *)o, (float *)dz);
    return launch_status();
}

extern "C" int stanza_gap_fwd(int32_t N, int32_t HW, int32_t C, int32_t dtype, const void *x, float *f, void *stream)
{
    if (N <= 0 || HW <= 0 || C <= 0 || (int64_t)N * HW * C >= (int64_t(1) << 31)) return STANZA_EINVAL;
    if (dtype != STANZA_F32 && dtype != STANZA_BF16) return STANZA_EUNSUPPORTED;
    if (!x || !f) return STANZA_ENULL;
    if (dtype == STANZA_BF16)
        hipLaunchKernelGGL(gap_fwd_bf16_kernel, dim3(cdiv(C, 256), N), dim3(256), 0, (hipStream_t)stream, N, HW, C, (const uint16_t *)x, f);
    else
        hipLaunchKernelGGL(gap_fwd_kernel, dim3(cdiv(C, 256), N), dim3(256), 0, (hipStream_t)stream, N, HW, C, (const float *)x, f);
    return launch_status();
}

extern "C" int stanza_gap_bwd(int32_t N, int32_t HW, int32_t C, int32_t dtype, const float *df, void *dx, void *stream)
{
    if (N <= 0 || HW <= 0 || C <= 0 || (int64_t)N * HW * C >= (int64_t(1) << 31)) return STANZA_EINVAL;
    if (dtype != STANZA_F32 && dtype != STANZA_BF16) return STANZA_EUNSUPPORTED;
    if (!df || !dx) return STANZA_ENULL;
    const size_t total = (size_t)N * HW * C;
    if (dtype == STANZA_BF16)
        hipLaunchKernelGGL(gap_bwd_bf16_kernel, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, (hipStream_t)stream, total, HW, C, df, (uint16_t *)dx);
    else
        hipLaunchKernelGGL(gap_bwd_kernel, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, (hipStream_t)stream, total, HW, C, df, (float *)dx);
    return launch_status();
}

extern "C" int stanza_cast_f32_to_bf16(int64_t numel, const float *src, void *dst, void *stream)
{
    if (numel <= 0) return STANZA_EINVAL;
    if (!src || !dst) return STANZA_ENULL;
    if (cdiv64(numel, CAST_CHUNK) >= (int64_t(1) << 31)) return STANZA_EINVAL;
    hipLaunchKernelGGL(cast_f32_bf16_kernel, dim3((unsigned)cdiv64(numel, CAST_CHUNK)), dim3(256), 0, (hipStream_t)stream, (size_t)numel, src,
                       (uint16_t *)dst, (int)(aligned16(src) && aligned16(dst)));
    return launch_status();
}

extern "C" int stanza_cast_bf16_to_f32(int64_t numel, const void *src, float *dst, void *stream)
{
    if (numel <= 0) return STANZA_EINVAL;
    if (!src || !dst) return STANZA_ENULL;
    if (cdiv64(numel, CAST_CHUNK) >= (int64_t(1) << 31)) return STANZA_EINVAL;
    hipLaunchKernelGGL(cast_bf16_f32_kernel, dim3((unsigned)cdiv64(numel, CAST_CHUNK)), dim3(256), 0, (hipStream_t)stream, (size_t)numel,
                       (const uint16_t *)src, dst, (int)(aligned16(src) && aligned16(dst)));
    return launch_status();
}

extern "C" size_t stanza_cast_workspace_bytes(int32_t n_tensors)
{
    if (n_tensors <= 0) return 0;
    return round256(sizeof(int64_t) * (2 * (size_t)n_tensors + 1) + sizeof(void *) * 2 * (size_t)n_tensors);
}

extern "C" int stanza_cast_plan(int32_t n_tensors, const int64_t *host_numel, const float *const *host_src, void *const *host_dst, void *ws,
                                size_t ws_bytes, void *stream)
{
    if (n_tensors <= 0 || n_tensors > (1 << 20)) return STANZA_EINVAL;
    if (!host_numel || !host_src || !host_dst || !ws) return STANZA_ENULL;
    const size_t need = stanza_cast_workspace_bytes(n_tensors);
    if (ws_bytes < need) return STANZA_EWORKSPACE;
    if (!aligned16(ws)) return STANZA_EALIGN;
    int64_t acc = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (host_numel[t] <= 0) return STANZA_EINVAL;
        if (!host_src[t] || !host_dst[t]) return STANZA_ENULL;
        if (!aligned16(host_src[t]) || !aligned16(host_dst[t])) return STANZA_EALIGN;
        acc += cdiv64(host_numel[t], CAST_CHUNK);
    }
    if (acc >= (int64_t(1) << 31)) return STANZA_EINVAL;
    // table layout: prefix[n + 1], numel[n], src[n], dst[n]
    TableWriter tw(ws, (hipStream_t)stream);
    acc = 0;
    for (int t = 0; t < n_tensors; ++t) {
        tw.push((uint64_t)acc);
        acc += cdiv64(host_numel[t], CAST_CHUNK);
    }
    tw.push((uint64_t)acc);
    for (int t = 0; t < n_tensors; ++t) tw.push((uint64_t)host_numel[t]);
    for (int t = 0; t < n_tensors; ++t) tw.push_ptr(host_src[t]);
    for (int t = 0; t < n_tensors; ++t) tw.push_ptr(host_dst[t]);
    tw.flush();
    return launch_status();
}

extern "C" int stanza_cast_f32_to_bf16_planned(int32_t n_tensors, const int64_t *host_numel, const void *ws, size_t ws_bytes, void *stream)
{
    if (n_tensors <= 0) return STANZA_EINVAL;
    if (!host_numel || !ws) return STANZA_ENULL;
    if (ws_bytes < stanza_cast_workspace_bytes(n_tensors)) return STANZA_EWORKSPACE;
    int64_t total = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (host_numel[t] <= 0) return STANZA_EINVAL;
        total += cdiv64(host_numel[t], CAST_CHUNK);
    }
    if (total >= (int64_t(1) << 31)) return STANZA_EINVAL;
    hipLaunchKernelGGL(cast_f32_bf16_multi_kernel, dim3((unsigned)total), dim3(256), 0, (hipStream_t)stream, ws, n_tensors);
    return launch_status();
}

// ------------------------------------------------------------------ ps_aggregate host side
extern "C" size_t stanza_ps_workspace_bytes(int32_t n_tensors, int32_t K)
{
    if (n_tensors <= 0 || K <= 0) return 0;
    return round256(sizeof(int64_t) * (2 * (size_t)n_tensors + 1) + sizeof(void *) * ((size_t)n_tensors * (2 + (size_t)K)));
}

static int ps_total_chunks(int32_t n_tensors, const int64_t *host_numel, int64_t *total)
{
    int64_t acc = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (host_numel[t] <= 0) return STANZA_EINVAL;
        acc += cdiv64(host_numel[t], PS_CHUNK);
    }
    if (acc >= (int64_t(1) << 31)) return STANZA_EINVAL;
    *total = acc;
    return STANZA_OK;
}

// The table of ps_aggregate_kernel (prefix[n + 1], numel[n], w[n], v[n], grads[K * n]) written to `table` by launches on `st`.
static void ps_write_table(int32_t n_tensors, const int64_t *host_numel, float *const *host_w, float *const *host_v,
                           const float *const *host_grads, int32_t K, void *table, hipStream_t st)
{
    TableWriter tw(table, st);
    int64_t acc = 0;
    for (int t = 0; t < n_tensors; ++t) {
        tw.push((uint64_t)acc);
        acc += cdiv64(host_numel[t], PS_CHUNK);
    }
    tw.push((uint64_t)acc);
    for (int t = 0; t < n_tensors; ++t) tw.push((uint64_t)host_numel[t]);
    for (int t = 0; t < n_tensors; ++t) tw.push_ptr(host_w[t]);
    for (int t = 0; t < n_tensors; ++t) tw.push_ptr(host_v[t]);
    for (size_t i = 0; i < (size_t)K * n_tensors; ++i) tw.push_ptr(host_grads[i]);
    tw.flush();
}

extern "C" int stanza_ps_plan(int32_t n_tensors, const int64_t *host_numel, float *const *host_w, float *const *host_v,
                              const float *const *host_grads, int32_t K, void *ws, size_t ws_bytes, void *stream)
{
    if (n_tensors <= 0 || K <= 0 || n_tensors > (1 << 20) || K > 4096) return STANZA_EINVAL;
    if (!host_numel || !host_w || !host_v || !host_grads || !ws) return STANZA_ENULL;
    const size_t need = stanza_ps_workspace_bytes(n_tensors, K);
    if (ws_bytes < need) return STANZA_EWORKSPACE;
    if (!aligned16(ws)) return STANZA_EALIGN;
    int64_t total;
    int rc = ps_total_chunks(n_tensors, host_numel, &total);
    if (rc) return rc;
    for (int t = 0; t < n_tensors; ++t) {
        if (!host_w[t] || !host_v[t]) return STANZA_ENULL;
        if (!aligned16(host_w[t]) || !aligned16(host_v[t])) return STANZA_EALIGN;
        for (int k = 0; k < K; ++k) {
            const float *gp = host_grads[(size_t)k * n_tensors + t];
            if (!gp) return STANZA_ENULL;
            if (!aligned16(gp)) return STANZA_EALIGN;
        }
    }
    ps_write_table(n_tensors, host_numel, host_w, host_v, host_grads, K, ws, (hipStream_t)stream);
    return launch_status();
}

template <int ORDER>
static void ps_launch(int32_t K, dim3 grid, hipStream_t st, const void *ws, int32_t n_tensors, float scale, float lr, float momentum, float weight_decay)
{
    const dim3 block(PS_T);
    switch (K) {
    case 2: hipLaunchKernelGGL((ps_aggregate_kernel<2, ORDER>), grid, block, 0, st, ws, n_tensors, K, scale, lr, momentum, weight_decay); break;
    case 4: hipLaunchKernelGGL((ps_aggregate_kernel<4, ORDER>), grid, block, 0, st, ws, n_tensors, K, scale, lr, momentum, weight_decay); break;
    case 8: hipLaunchKernelGGL((ps_aggregate_kernel<8, ORDER>), grid, block, 0, st, ws, n_tensors, K, scale, lr, momentum, weight_decay); break;
    case 16: hipLaunchKernelGGL((ps_aggregate_kernel<16, ORDER>), grid, block, 0, st, ws, n_tensors, K, scale, lr, momentum, weight_decay); break;
    default: hipLaunchKernelGGL((ps_aggregate_kernel<0, ORDER>), grid, block, 0, st, ws, n_tensors, K, scale, lr, momentum, weight_decay); break;
    }
}

extern "C" int stanza_ps_aggregate_ordered_planned(int32_t order, int32_t n_tensors, const int64_t *host_numel, int32_t K, float scale, float lr,
                                                   float momentum, float weight_decay, const void *ws, size_t ws_bytes, void *stream)
{
    if (n_tensors <= 0 || K <= 0 || K > 4096) return STANZA_EINVAL;
    if (order != STANZA_SUM_INDEX_ORDER && order != STANZA_SUM_RECURSIVE_DOUBLING) return STANZA_EINVAL;
    if (!host_numel || !ws) return STANZA_ENULL;
    if (ws_bytes < stanza_ps_workspace_bytes(n_tensors, K)) return STANZA_EWORKSPACE;
    int64_t total;
    int rc = ps_total_chunks(n_tensors, host_numel, &total);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)total);
    if (order == STANZA_SUM_RECURSIVE_DOUBLING) ps_launch<PS_ORDER_RD>(K, grid, st, ws, n_tensors, scale, lr, momentum, weight_decay);
    else ps_launch<PS_ORDER_INDEX>(K, grid, st, ws, n_tensors, scale, lr, momentum, weight_decay);
    return launch_status();
}

extern "C" int stanza_ps_aggregate_planned(int32_t n_tensors, const int64_t *host_numel, int32_t K, float scale, float lr, float momentum,
                                           float weight_decay, const void *ws, size_t ws_bytes, void *stream)
{
    return stanza_ps_aggregate_ordered_planned(STANZA_SUM_INDEX_ORDER, n_tensors, host_numel, K, scale, lr, momentum, weight_decay, ws, ws_bytes, stream);
}

extern "C" int stanza_ps_aggregate_ordered(int32_t order, int32_t n_tensors, const int64_t *host_numel, float *const *host_w, float *const *host_v,
                                           const float *const *host_grads, int32_t K, float scale, float lr, float momentum, float weight_decay,
                                           void *ws, size_t ws_bytes, void *stream)
{
    if (order != STANZA_SUM_INDEX_ORDER && order != STANZA_SUM_RECURSIVE_DOUBLING) return STANZA_EINVAL;
    int rc = stanza_ps_plan(n_tensors, host_numel, host_w, host_v, host_grads, K, ws, ws_bytes, stream);
    if (rc) return rc;
    return stanza_ps_aggregate_ordered_planned(order, n_tensors, host_numel, K, scale, lr, momentum, weight_decay, ws, ws_bytes, stream);
}

extern "C" int stanza_ps_aggregate(int32_t n_tensors, const int64_t *host_numel, float *const *host_w, float *const *host_v,
                                   const float *const *host_grads, int32_t K, float scale, float lr, float momentum, float weight_decay,
                                   void *ws, size_t ws_bytes, void *stream)
{
    return stanza_ps_aggregate_ordered(STANZA_SUM_INDEX_ORDER, n_tensors, host_numel, host_w, host_v, host_grads, K, scale, lr, momentum,
                                       weight_decay, ws, ws_bytes, stream);
}

// ------------------------------------------------------------------ aggregation without a workspace
// For callers that cannot allocate device memory and so have no workspace to hand over: the pointer table lives in a fixed array
// of this library's device image.  Each GPU holds its own copy of the array at its own address; host code never uses the
// array's name as an address, only the pointer that hipGetSymbolAddress returned for the current device.
constexpr int PS_STATIC_WORDS = 32768;          // 256 KiB per GPU, held until the process ends
static __device__ __align__(256) unsigned long long scratch[PS_STATIC_WORDS];

constexpr int PS_STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[PS_STATIC_MAX_DEVICES];   // per device: device address of `scratch`, resolved on first use

static int ps_static_table(void **table)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return STANZA_EHIP;
    if (dev < 0 || dev >= PS_STATIC_MAX_DEVICES) return STANZA_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return STANZA_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *table = g_scratch_ptr[dev];
    return STANZA_OK;
}

extern "C" int stanza_ps_aggregate_static(int32_t order, int32_t n_tensors, const int64_t *host_numel, float *const *host_w,
                                          float *const *host_v, const float *const *host_grads, int32_t K, float scale, float lr,
                                          float momentum, float weight_decay, void *stream)
{
    if (order != STANZA_SUM_INDEX_ORDER && order != STANZA_SUM_RECURSIVE_DOUBLING) return STANZA_EINVAL;
    if (n_tensors <= 0 || K <= 0 || K > 4096) return STANZA_EINVAL;
    if ((int64_t)n_tensors * ((int64_t)K + 4) + 1 > PS_STATIC_WORDS) return STANZA_ECAPACITY;
    void *table = nullptr;
    int rc = ps_static_table(&table);
    if (rc) return rc;
    const size_t bytes = (size_t)PS_STATIC_WORDS * sizeof(unsigned long long);
    // Validation and the table launches are those of the workspace form; the table is rewritten whole by every call, so
    // nothing of the previous call's contents is read.
    rc = stanza_ps_plan(n_tensors, host_numel, host_w, host_v, host_grads, K, table, bytes, stream);
    if (rc) return rc;
    return stanza_ps_aggregate_ordered_planned(order, n_tensors, host_numel, K, scale, lr, momentum, weight_decay, table, bytes, stream);
}
