// Batch normalisation (training mode) on the CONV worker, for the residual networks of the paper's table of models
// (Sec. 6.1), which carry a normalisation layer after every convolution.  The paper does not describe the layer;
// the transform is the published one, with the statistics taken over the worker's own batch.
//
// An NHWC tensor is a [rows][C] matrix with the channel contiguous, so every kernel here is a column-wise pass over a
// row-major matrix, bound by HBM: a thread owns one 16-byte channel vector and walks down the rows, a workgroup of 256
// threads covers TX vectors of a row and TY = 256 / TX consecutive rows per pass (one contiguous stretch of memory when
// the row fits), and a grid of row slabs x column blocks covers the matrix.  Reductions over rows are done per thread,
// then over the workgroup's TY rows through LDS, then over the slabs by a small second kernel, each in a fixed order:
// results are run-to-run identical.
//   forward   stats pass (read x) -> finalise (mean, 1/std, running averages) -> apply pass (read x, write y)
//   backward  reduce pass (read x, dy) -> finalise (dgamma, dbeta) -> apply pass (read x, dy, write dx)
// A fused ReLU is undone in the backward passes by recomputing the sign of the forward output from x (the same
// float32 expression, operation by operation, as the forward apply pass), so y is never read back.
#include "internal.h"

namespace stanza {

struct BnGeo {
    int rows, C, cv;       // cv: channel vectors per row
    int TX, TY;            // threads across a row, rows per pass (TX * TY <= 256)
    int rows_per_slab;     // rows of one blockIdx.x
};

typedef unsigned int bn_u4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t bn_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// VW consecutive channels starting at vector index `vec` (in units of VW elements).
template <int VW, bool BF16, bool NT>
__device__ __forceinline__ void bn_load(const void *base, size_t vec, float (&v)[VW])
{
    if constexpr (VW == 1) {
        v[0] = reinterpret_cast<const float *>(base)[vec];
    } else {
        const bn_u4 *p = reinterpret_cast<const bn_u4 *>(base) + vec;
        const bn_u4 t = NT ? __builtin_nontemporal_load(p) : *p;
#pragma unroll
        for (int e = 0; e < VW; ++e)
            v[e] = BF16 ? __uint_as_float(((t[e >> 1] >> (16 * (e & 1))) & 0xffffu) << 16) : __uint_as_float(t[e]);
    }
}

template <int VW, bool BF16>
__device__ __forceinline__ void bn_store(void *base, size_t vec, const float (&v)[VW])
{
    if constexpr (VW == 1) {
        reinterpret_cast<float *>(base)[vec] = v[0];
    } else {
        bn_u4 t = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < VW; ++e) {
            if (BF16) t[e >> 1] |= bn_bf16_rne(v[e]) << (16 * (e & 1));
            else t[e] = __float_as_uint(v[e]);
        }
        __builtin_nontemporal_store(t, reinterpret_cast<bn_u4 *>(base) + vec);
    }
}

// Forward output before the ReLU, ((x - mean) * s) + beta with s = gamma * istd, written out operation by operation (no
// contraction into a fused multiply-add) so that the forward pass and the sign test of the backward passes take the same
// roundings.  Subtracting the mean first keeps the result accurate for channels whose mean is large against their spread.
__device__ __forceinline__ float bn_affine(float x, float mean, float sc, float beta)
{
#pragma clang fp contract(off)
    const float d = x - mean;
    const float t = d * sc;
    return t + beta;
}
__device__ __forceinline__ float bn_scale(float gamma, float istd) { return gamma * istd; }
__device__ __forceinline__ float bn_xhat(float x, float mean, float istd) { return (x - mean) * istd; }

// Per-thread sums over the rows r0 + ty, r0 + ty + TY, ... of its slab, four rows in flight, then the workgroup's TY
// rows in row order through LDS.  BWD = false: a = sum (x - k), b = sum (x - k)^2 with k = x[0][c] (a shift inside the
// data's range keeps the variance free of cancellation).  BWD = true: a = sum g, b = sum g * xhat with
// g = dy * [forward output > 0] (relu) or dy.  partial: [slab][2][C].
template <int VW, bool BF16, bool BWD>
__global__ __launch_bounds__(256) void bn_reduce_kernel(const BnGeo g, const void *__restrict__ xv, const void *__restrict__ dyv,
                                                        const float *__restrict__ gamma, const float *__restrict__ beta,
                                                        const float *__restrict__ mean, const float *__restrict__ istd, int relu,
                                                        float *__restrict__ partial)
{
    __shared__ float red[256 * 2 * VW];
    const int ty = threadIdx.x / g.TX, tx = threadIdx.x - ty * g.TX;
    const int col = blockIdx.y * g.TX + tx;
    const bool active = ty < g.TY && col < g.cv;
    float a[VW], b[VW], k[VW], is[VW], sc[VW], sh[VW];
#pragma unroll
    for (int e = 0; e < VW; ++e) a[e] = b[e] = k[e] = is[e] = sc[e] = sh[e] = 0.f;
    if (active) {
        if (BWD) {
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int c = col * VW + e;
                k[e] = mean[c];
                is[e] = istd[c];
                sc[e] = bn_scale(gamma[c], is[e]);
                sh[e] = beta[c];
            }
        } else {
            bn_load<VW, BF16, false>(xv, (size_t)col, k);
        }
        const int r0 = blockIdx.x * g.rows_per_slab;
        const int r1 = min(r0 + g.rows_per_slab, g.rows);
        auto take = [&](const float (&x)[VW], const float (&dy)[VW]) {
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                if (BWD) {
                    const float gr = (relu && !(bn_affine(x[e], k[e], sc[e], sh[e]) > 0.f)) ? 0.f : dy[e];
                    const float xh = bn_xhat(x[e], k[e], is[e]);
                    a[e] += gr;
                    b[e] = fmaf(gr, xh, b[e]);
                } else {
                    const float d = x[e] - k[e];
                    a[e] += d;
                    b[e] = fmaf(d, d, b[e]);
                }
            }
        };
        int r = r0 + ty;
        for (; r + 3 * g.TY < r1; r += 4 * g.TY) {
            float x[4][VW], dy[4][VW];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const size_t vec = (size_t)(r + u * g.TY) * g.cv + col;
                bn_load<VW, BF16, false>(xv, vec, x[u]);
                if (BWD) bn_load<VW, BF16, false>(dyv, vec, dy[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) take(x[u], BWD ? dy[u] : x[u]);
        }
        for (; r < r1; r += g.TY) {
            float x[VW], dy[VW];
            const size_t vec = (size_t)r * g.cv + col;
            bn_load<VW, BF16, false>(xv, vec, x);
            if (BWD) bn_load<VW, BF16, false>(dyv, vec, dy);
            take(x, BWD ? dy : x);
        }
    }
#pragma unroll
    for (int e = 0; e < VW; ++e) {
        red[threadIdx.x * 2 * VW + e] = a[e];
        red[threadIdx.x * 2 * VW + VW + e] = b[e];
    }
    __syncthreads();
    if (ty == 0 && col < g.cv) {
        for (int t = 1; t < g.TY; ++t) {
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                a[e] += red[(t * g.TX + tx) * 2 * VW + e];
                b[e] += red[(t * g.TX + tx) * 2 * VW + VW + e];
            }
        }
        float *out = partial + (size_t)blockIdx.x * 2 * g.C + (size_t)col * VW;
#pragma unroll
        for (int e = 0; e < VW; ++e) {
            out[e] = a[e];
            out[g.C + e] = b[e];
        }
    }
}

// Sums the slabs' partial sums per channel: a workgroup takes 8 channels x 32 interleaved groups of slabs (eight loads in
// flight per thread: the pass is bound by latency, not by bytes), each group in slab order, then the groups in group order.
// BWD = false: mean, 1/std and (when given) the running averages.  BWD = true: out_a = dbeta, out_b = dgamma.
constexpr int BN_FIN_CH = 8, BN_FIN_LANES = 32;
template <bool BWD, bool BF16>
__global__ __launch_bounds__(256) void bn_finalize_kernel(int C, int slabs, int rows, const float *__restrict__ partial,
                                                          const void *__restrict__ x_row0, float eps, float *__restrict__ out_a,
                                                          float *__restrict__ out_b, float *__restrict__ run_mean,
                                                          float *__restrict__ run_var, float mom)
{
    __shared__ float red[BN_FIN_LANES][BN_FIN_CH][2];
    const int cl = threadIdx.x % BN_FIN_CH, lane = threadIdx.x / BN_FIN_CH;
    const int c = blockIdx.x * BN_FIN_CH + cl;
    float a = 0.f, b = 0.f;
    if (c < C) {
        int s = lane;
        for (; s + 7 * BN_FIN_LANES < slabs; s += 8 * BN_FIN_LANES) {
            float va[8], vb[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                va[u] = partial[(size_t)(s + u * BN_FIN_LANES) * 2 * C + c];
                vb[u] = partial[(size_t)(s + u * BN_FIN_LANES) * 2 * C + C + c];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                a += va[u];
                b += vb[u];
            }
        }
        for (; s < slabs; s += BN_FIN_LANES) {
            a += partial[(size_t)s * 2 * C + c];
            b += partial[(size_t)s * 2 * C + C + c];
        }
    }
    red[lane][cl][0] = a;
    red[lane][cl][1] = b;
    __syncthreads();
    if (lane != 0 || c >= C) return;
    for (int t = 1; t < BN_FIN_LANES; ++t) {
        a += red[t][cl][0];
        b += red[t][cl][1];
    }
    if (BWD) {
        out_a[c] = a;
        out_b[c] = b;
        return;
    }
    const float k = BF16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(x_row0)[c] << 16)
                         : reinterpret_cast<const float *>(x_row0)[c];
    const float inv = 1.f / (float)rows;
    const float m1 = a * inv;
    const float var = fmaxf(fmaf(-m1, m1, b * inv), 0.f);
    const float mu = k + m1;
    out_a[c] = mu;
    out_b[c] = 1.f / sqrtf(var + eps);
    if (run_mean) run_mean[c] = (1.f - mom) * run_mean[c] + mom * mu;
    if (run_var) run_var[c] = (1.f - mom) * run_var[c] + mom * (rows > 1 ? var * ((float)rows / (float)(rows - 1)) : var);
}

// Mean and 1/std from the column statistics that a forward convolution left behind (StatsHeader in igemm.h): per entry and
// column the sums of (y - k) and (y - k)^2 about the entry's own first row k.  Re-based on one shift per column, kref = k of the
// column's first entry, an entry of n rows contributes  n d + a  and  b + d (2 a + n d)  with d = k - kref  (the expansion of
// sum (y - kref) and sum (y - kref)^2 over its rows), so the result is the shifted two-sum variance that the statistics pass
// computes, in a fixed order: a workgroup takes CH columns x 256 / CH lanes, a lane every (256 / CH)-th entry in entry order (four
// entries in flight: the pass is bound by latency), then the lanes by halving.  CH = 1 for the tall matrices of the first stages
// (a thousand and more entries per column), 16 for the short ones.  A header that does not describe this matrix or does not fit
// the buffer gives NaN.
template <int CH>
__global__ __launch_bounds__(256) void bn_finalize_tiles_kernel(int C, int rows, const float *__restrict__ stats, size_t stats_floats, float eps,
                                                                float *__restrict__ out_mean, float *__restrict__ out_istd,
                                                                float *__restrict__ run_mean, float *__restrict__ run_var, float mom)
{
    constexpr int LANES = 256 / CH;
    __shared__ float red[LANES][CH][2];
    const StatsHeader h = *reinterpret_cast<const StatsHeader *>(stats);
    const int cl = threadIdx.x % CH, lane = threadIdx.x / CH;
    const int c = blockIdx.x * CH + cl;
    bool ok = h.magic == STATS_MAGIC && h.M == rows && h.Nn == C && (h.bm == 64 || h.bm == 128 || h.bm == 256) && (h.bn == 64 || h.bn == 128);
    int sub = 1, rows_sub = 1;
    if (ok) {
        sub = h.bm * h.bn / 1024;
        rows_sub = 1024 / h.bn;
        const long long tiles = (long long)h.tilesM * h.tilesN;
        ok = h.tilesM == (rows + h.bm - 1) / h.bm && h.tilesN == (C + h.bn - 1) / h.bn && h.dp_tiles >= 0 && h.dp_tiles <= tiles &&
             (unsigned long long)STATS_HEADER_FLOATS + ((unsigned long long)h.dp_tiles + (unsigned long long)(tiles - h.dp_tiles) * sub) * 3ull * h.bn <=
                 (unsigned long long)stats_floats;
    }
    if (!ok) {
        if (lane == 0 && c < C) out_mean[c] = out_istd[c] = __uint_as_float(0x7fc00000u);
        return;
    }
    float s1 = 0.f, s2 = 0.f, kref = 0.f;
    if (c < C) {
        const int bn = h.bn, tile_n = c / bn;
        const float *col = stats + STATS_HEADER_FLOATS + (c - tile_n * bn);
        const size_t estride = (size_t)3 * bn;
        // tile rows of this column whose tile is computed whole: tile_m * tilesN + tile_n < dp_tiles
        const int mdp = h.dp_tiles > tile_n ? min(h.tilesM, (h.dp_tiles - tile_n + h.tilesN - 1) / h.tilesN) : 0;
        auto entry_of = [&](int tile_m, int s) -> size_t {
            const int tile = tile_m * h.tilesN + tile_n;
            return tile < h.dp_tiles ? (size_t)tile : (size_t)h.dp_tiles + (size_t)(tile - h.dp_tiles) * sub + s;
        };
        kref = col[entry_of(0, 0) * estride + 2 * bn];
        auto take = [&](int n, float a, float b, float k) {
            const float d = k - kref, nf = (float)n;
            s1 += fmaf(nf, d, a);
            s2 += fmaf(d, fmaf(nf, d, 2.f * a), b);
        };
        for (int tm = lane; tm < mdp; tm += 4 * LANES) {
            float a[4], b[4], k[4];
            int n[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int tmu = tm + u * LANES;
                n[u] = tmu < mdp ? min(h.bm, rows - tmu * h.bm) : 0;
                if (n[u] > 0) {
                    const float *q = col + entry_of(tmu, 0) * estride;
                    a[u] = q[0]; b[u] = q[bn]; k[u] = q[2 * bn];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (n[u] > 0) take(n[u], a[u], b[u], k[u]);
        }
        const int split_entries = (h.tilesM - mdp) * sub;
        for (int j = lane; j < split_entries; j += 4 * LANES) {
            float a[4], b[4], k[4];
            int n[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ju = j + u * LANES;
                n[u] = 0;
                if (ju < split_entries) {
                    const int tm = mdp + ju / sub, sidx = ju % sub;
                    n[u] = min(rows_sub, rows - tm * h.bm - sidx * rows_sub);
                    if (n[u] > 0) {
                        const float *q = col + entry_of(tm, sidx) * estride;
                        a[u] = q[0]; b[u] = q[bn]; k[u] = q[2 * bn];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (n[u] > 0) take(n[u], a[u], b[u], k[u]);
        }
    }
    red[lane][cl][0] = s1;
    red[lane][cl][1] = s2;
    __syncthreads();
#pragma unroll
    for (int half = LANES / 2; half > 0; half >>= 1) {
        if (lane < half) {
            red[lane][cl][0] += red[lane + half][cl][0];
            red[lane][cl][1] += red[lane + half][cl][1];
        }
        __syncthreads();
    }
    if (lane != 0 || c >= C) return;
    s1 = red[0][cl][0];
    s2 = red[0][cl][1];
    const float inv = 1.f / (float)rows;
    const float m1 = s1 * inv;
    const float var = fmaxf(fmaf(-m1, m1, s2 * inv), 0.f);
    const float mu = kref + m1;
    out_mean[c] = mu;
    out_istd[c] = 1.f / sqrtf(var + eps);
    if (run_mean) run_mean[c] = (1.f - mom) * run_mean[c] + mom * mu;
    if (run_var) run_var[c] = (1.f - mom) * run_var[c] + mom * (rows > 1 ? var * ((float)rows / (float)(rows - 1)) : var);
}

// BWD = false: y = gamma * xhat + beta (+ReLU); with dyv != nullptr it holds a residual tensor that is added before the ReLU (a
// residual join fused into the layer: y = max(bn(x) + res, 0)).  BWD = true: dx = gamma istd (g - dbeta/M - xhat dgamma/M).
template <int VW, bool BF16, bool BWD>
__global__ __launch_bounds__(256) void bn_apply_kernel(const BnGeo g, const void *__restrict__ xv, const void *__restrict__ dyv,
                                                       const float *__restrict__ gamma, const float *__restrict__ beta,
                                                       const float *__restrict__ mean, const float *__restrict__ istd,
                                                       const float *__restrict__ dgamma, const float *__restrict__ dbeta, int relu,
                                                       void *__restrict__ outv)
{
    const int ty = threadIdx.x / g.TX, tx = threadIdx.x - ty * g.TX;
    const int col = blockIdx.y * g.TX + tx;
    if (ty >= g.TY || col >= g.cv) return;
    float mu[VW], is[VW], sc[VW], sh[VW], c1[VW], c2[VW];
    const float inv = 1.f / (float)g.rows;
#pragma unroll
    for (int e = 0; e < VW; ++e) {
        const int c = col * VW + e;
        mu[e] = mean[c];
        is[e] = istd[c];
        sc[e] = bn_scale(gamma[c], is[e]);
        sh[e] = beta[c];
        c1[e] = BWD ? dbeta[c] * inv : 0.f;
        c2[e] = BWD ? dgamma[c] * inv : 0.f;
    }
    const int r0 = blockIdx.x * g.rows_per_slab;
    const int r1 = min(r0 + g.rows_per_slab, g.rows);
    const bool with_res = !BWD && dyv != nullptr;
    auto emit = [&](size_t vec, const float (&x)[VW], const float (&dy)[VW]) {
        float o[VW];
#pragma unroll
        for (int e = 0; e < VW; ++e) {
            const float yv = bn_affine(x[e], mu[e], sc[e], sh[e]);
            if (BWD) {
                const float gr = (relu && !(yv > 0.f)) ? 0.f : dy[e];
                const float xh = bn_xhat(x[e], mu[e], is[e]);
                o[e] = sc[e] * fmaf(-xh, c2[e], gr - c1[e]);
            } else {
                const float z = with_res ? yv + dy[e] : yv;
                o[e] = (relu && !(z > 0.f)) ? 0.f : z;
            }
        }
        bn_store<VW, BF16>(outv, vec, o);
    };
    int r = r0 + ty;
    for (; r + 3 * g.TY < r1; r += 4 * g.TY) {
        float x[4][VW], dy[4][VW];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t vec = (size_t)(r + u * g.TY) * g.cv + col;
            bn_load<VW, BF16, true>(xv, vec, x[u]);
            if (BWD || with_res) bn_load<VW, BF16, true>(dyv, vec, dy[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) emit((size_t)(r + u * g.TY) * g.cv + col, x[u], (BWD || with_res) ? dy[u] : x[u]);
    }
    for (; r < r1; r += g.TY) {
        float x[VW], dy[VW];
        const size_t vec = (size_t)r * g.cv + col;
        bn_load<VW, BF16, true>(xv, vec, x);
        if (BWD || with_res) bn_load<VW, BF16, true>(dyv, vec, dy);
        emit(vec, x, (BWD || with_res) ? dy : x);
    }
}

// ------------------------------------------------------------------ host side
struct BnPlan {
    BnGeo reduce, apply;
    int vw, col_blocks, slabs, slabs_apply;
    size_t ws_floats;
};

static int bn_plan(int64_t rows, int32_t C, int32_t dtype, BnPlan *p)
{
    if (rows < 1 || C < 1 || rows * (int64_t)C >= (int64_t(1) << 31)) return STANZA_EINVAL;
    if (dtype != STANZA_F32 && dtype != STANZA_BF16) return STANZA_EUNSUPPORTED;
    if (dtype == STANZA_BF16 && C % 8 != 0) return STANZA_EUNSUPPORTED;
    p->vw = dtype == STANZA_BF16 ? 8 : (C % 4 == 0 ? 4 : 1);
    BnGeo g;
    g.rows = (int)rows;
    g.C = C;
    g.cv = C / p->vw;
    g.TX = g.cv < 256 ? g.cv : 256;
    g.TY = 256 / g.TX;
    p->col_blocks = cdiv(g.cv, g.TX);
    // reduction passes: about 1024 workgroups, each with at least eight passes over its TY rows
    const int64_t wanted = cdiv64(rows, (int64_t)g.TY * 8);
    const int64_t cap = 1024 / p->col_blocks > 0 ? 1024 / p->col_blocks : 1;
    p->slabs = (int)(wanted < 1 ? 1 : (wanted > cap ? cap : wanted));
    g.rows_per_slab = (int)cdiv64(rows, p->slabs);
    p->slabs = (int)cdiv64(rows, g.rows_per_slab);
    p->reduce = g;
    // element-wise passes: four passes per workgroup
    g.rows_per_slab = g.TY * 4;
    p->slabs_apply = (int)cdiv64(rows, g.rows_per_slab);
    p->apply = g;
    p->ws_floats = (size_t)p->slabs * 2 * C;
    return STANZA_OK;
}

template <bool BWD>
static void bn_launch_reduce(const BnPlan &p, int dtype, hipStream_t st, const void *x, const void *dy, const float *gamma, const float *beta,
                             const float *mean, const float *istd, int relu, float *partial)
{
    const dim3 grid((unsigned)p.slabs, (unsigned)p.col_blocks);
    if (dtype == STANZA_BF16)
        hipLaunchKernelGGL((bn_reduce_kernel<8, true, BWD>), grid, dim3(256), 0, st, p.reduce, x, dy, gamma, beta, mean, istd, relu, partial);
    else if (p.vw == 4)
        hipLaunchKernelGGL((bn_reduce_kernel<4, false, BWD>), grid, dim3(256), 0, st, p.reduce, x, dy, gamma, beta, mean, istd, relu, partial);
    else
        hipLaunchKernelGGL((bn_reduce_kernel<1, false, BWD>), grid, dim3(256), 0, st, p.reduce, x, dy, gamma, beta, mean, istd, relu, partial);
}

template <bool BWD>
static void bn_launch_apply(const BnPlan &p, int dtype, hipStream_t st, const void *x, const void *dy, const float *gamma, const float *beta,
                            const float *mean, const float *istd, const float *dgamma, const float *dbeta, int relu, void *out)
{
    const dim3 grid((unsigned)p.slabs_apply, (unsigned)p.col_blocks);
    if (dtype == STANZA_BF16)
        hipLaunchKernelGGL((bn_apply_kernel<8, true, BWD>), grid, dim3(256), 0, st, p.apply, x, dy, gamma, beta, mean, istd, dgamma, dbeta, relu, out);
    else if (p.vw == 4)
        hipLaunchKernelGGL((bn_apply_kernel<4, false, BWD>), grid, dim3(256), 0, st, p.apply, x, dy, gamma, beta, mean, istd, dgamma, dbeta, relu, out);
    else
        hipLaunchKernelGGL((bn_apply_kernel<1, false, BWD>), grid, dim3(256), 0, st, p.apply, x, dy, gamma, beta, mean, istd, dgamma, dbeta, relu, out);
}

}  // namespace stanza

using namespace stanza;

extern "C" size_t stanza_bn_workspace_bytes(int64_t rows, int32_t C, int32_t dtype)
{
    BnPlan p;
    if (bn_plan(rows, C, dtype, &p)) return 0;
    return round256(p.ws_floats * sizeof(float));
}

static int bn_fwd_any(int64_t rows, int32_t C, int32_t dtype, float eps, int32_t relu, const void *x, const float *gamma,
                      const float *beta, const void *res, bool want_res, void *y, float *save_mean, float *save_istd, float *running_mean,
                      float *running_var, float momentum, void *ws, size_t ws_bytes, void *stream)
{
    BnPlan p;
    int rc = bn_plan(rows, C, dtype, &p);
    if (rc) return rc;
    if (!(eps > 0.f) || !(momentum >= 0.f && momentum <= 1.f)) return STANZA_EINVAL;
    if (!x || !gamma || !beta || !y || !save_mean || !save_istd || !ws || (want_res && !res)) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(y) || !aligned16(ws) || !aligned16(res)) return STANZA_EALIGN;
    if (ws_bytes < p.ws_floats * sizeof(float)) return STANZA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float *partial = reinterpret_cast<float *>(ws);
    bn_launch_reduce<false>(p, dtype, st, x, nullptr, nullptr, nullptr, nullptr, nullptr, 0, partial);
    if (dtype == STANZA_BF16)
        hipLaunchKernelGGL((bn_finalize_kernel<false, true>), dim3((unsigned)cdiv(C, BN_FIN_CH)), dim3(256), 0, st, C, p.slabs, (int)rows, partial, x, eps,
                           save_mean, save_istd, running_mean, running_var, momentum);
    else
        hipLaunchKernelGGL((bn_finalize_kernel<false, false>), dim3((unsigned)cdiv(C, BN_FIN_CH)), dim3(256), 0, st, C, p.slabs, (int)rows, partial, x, eps,
                           save_mean, save_istd, running_mean, running_var, momentum);
    bn_launch_apply<false>(p, dtype, st, x, want_res ? res : nullptr, gamma, beta, save_mean, save_istd, nullptr, nullptr, relu ? 1 : 0, y);
    return launch_status();
}

extern "C" int stanza_bn_fwd(int64_t rows, int32_t C, int32_t dtype, float eps, int32_t relu, const void *x, const float *gamma,
                             const float *beta, void *y, float *save_mean, float *save_istd, float *running_mean, float *running_var,
                             float momentum, void *ws, size_t ws_bytes, void *stream)
{
    return bn_fwd_any(rows, C, dtype, eps, relu, x, gamma, beta, nullptr, false, y, save_mean, save_istd, running_mean, running_var, momentum, ws,
                      ws_bytes, stream);
}

extern "C" int stanza_bn_fwd_res(int64_t rows, int32_t C, int32_t dtype, float eps, int32_t relu, const void *x, const float *gamma,
                                 const float *beta, const void *res, void *y, float *save_mean, float *save_istd, float *running_mean,
                                 float *running_var, float momentum, void *ws, size_t ws_bytes, void *stream)
{
    return bn_fwd_any(rows, C, dtype, eps, relu, x, gamma, beta, res, true, y, save_mean, save_istd, running_mean, running_var, momentum, ws,
                      ws_bytes, stream);
}

extern "C" int stanza_bn_fwd_stats(int64_t rows, int32_t C, float eps, int32_t relu, const void *x, const void *stats, size_t stats_bytes,
                                   const float *gamma, const float *beta, const void *res, void *y, float *save_mean, float *save_istd,
                                   float *running_mean, float *running_var, float momentum, void *stream)
{
    BnPlan p;
    int rc = bn_plan(rows, C, STANZA_F32, &p);
    if (rc) return rc;
    if (C % 4 != 0) return STANZA_EUNSUPPORTED;
    if (!(eps > 0.f) || !(momentum >= 0.f && momentum <= 1.f)) return STANZA_EINVAL;
    if (!x || !stats || !gamma || !beta || !y || !save_mean || !save_istd) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(y) || !aligned16(stats) || !aligned16(res)) return STANZA_EALIGN;
    if (stats_bytes < STATS_HEADER_FLOATS * sizeof(float)) return STANZA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    // lanes per column by the number of entries a column has (a tile has 64 to 256 rows)
    const float *sf = (const float *)stats;
    const size_t sfl = stats_bytes / sizeof(float);
    if (rows >= 32768)
        hipLaunchKernelGGL(bn_finalize_tiles_kernel<1>, dim3((unsigned)C), dim3(256), 0, st, C, (int)rows, sf, sfl, eps, save_mean, save_istd,
                           running_mean, running_var, momentum);
    else if (rows >= 4096)
        hipLaunchKernelGGL(bn_finalize_tiles_kernel<4>, dim3((unsigned)cdiv(C, 4)), dim3(256), 0, st, C, (int)rows, sf, sfl, eps, save_mean,
                           save_istd, running_mean, running_var, momentum);
    else
        hipLaunchKernelGGL(bn_finalize_tiles_kernel<16>, dim3((unsigned)cdiv(C, 16)), dim3(256), 0, st, C, (int)rows, sf, sfl, eps, save_mean,
                           save_istd, running_mean, running_var, momentum);
    bn_launch_apply<false>(p, STANZA_F32, st, x, res, gamma, beta, save_mean, save_istd, nullptr, nullptr, relu ? 1 : 0, y);
    return launch_status();
}

extern "C" int stanza_bn_bwd(int64_t rows, int32_t C, int32_t dtype, int32_t relu, const void *x, const void *dy, const float *gamma,
                             const float *beta, const float *save_mean, const float *save_istd, void *dx, float *dgamma, float *dbeta,
                             void *ws, size_t ws_bytes, void *stream)
{
    BnPlan p;
    int rc = bn_plan(rows, C, dtype, &p);
    if (rc) return rc;
    if (!x || !dy || !gamma || !beta || !save_mean || !save_istd || !dx || !dgamma || !dbeta || !ws) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(ws)) return STANZA_EALIGN;
    if (ws_bytes < p.ws_floats * sizeof(float)) return STANZA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float *partial = reinterpret_cast<float *>(ws);
    bn_launch_reduce<true>(p, dtype, st, x, dy, gamma, beta, save_mean, save_istd, relu ? 1 : 0, partial);
    hipLaunchKernelGGL((bn_finalize_kernel<true, false>), dim3((unsigned)cdiv(C, BN_FIN_CH)), dim3(256), 0, st, C, p.slabs, (int)rows, partial, nullptr, 0.f,
                       dbeta, dgamma, nullptr, nullptr, 0.f);
    bn_launch_apply<true>(p, dtype, st, x, dy, gamma, beta, save_mean, save_istd, dgamma, dbeta, relu ? 1 : 0, dx);
    return launch_status();
}
