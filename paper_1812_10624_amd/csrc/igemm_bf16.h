// bf16-in / fp32-accumulate variant of the implicit-GEMM engine (same three gather modes and the same
// GemmParams as igemm.h; see there for the index conventions).  x, w, y, dy, dx are bfloat16; products are
// accumulated in float32 by v_mfma_f32_32x32x16_bf16; bias, filter gradients and bias gradients are float32.
//
// One MFMA lane supplies 8 consecutive reduction elements of one tile row, so both LDS tiles are stored
// row-major with the reduction contiguous ([BM][BK+8] bf16, 80-byte rows: 16-byte operand reads of 8
// consecutive rows cover all 32 banks).  Operands whose reduction is contiguous in memory go global -> register
// -> LDS as 16-byte vectors; operands whose row index is contiguous (w in BWD_DATA, dy and x in BWD_WEIGHT)
// are transposed element by element on the LDS store.
#pragma once
#include "igemm.h"

namespace stanza {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int BKH = 32;        // reduction depth of one LDS stage (bf16 elements)
constexpr int LDKH = BKH + 8;  // LDS row stride in elements

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ bool bf16_pos(uint16_t h) { return h != 0 && !(h & 0x8000u); }   // h > 0 (finite inputs)
__device__ __forceinline__ uint16_t h8at(const uint4 &v, int e) { return reinterpret_cast<const uint16_t *>(&v)[e]; }
__device__ __forceinline__ uint4 ldg16(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
// keep element e of v where the matching element of m is > 0
__device__ __forceinline__ uint4 gate8(uint4 v, uint4 m)
{
    uint32_t *pv = reinterpret_cast<uint32_t *>(&v);
    const uint32_t *pm = reinterpret_cast<const uint32_t *>(&m);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t lo = bf16_pos((uint16_t)(pm[w] & 0xffffu)) ? 0x0000ffffu : 0u;
        const uint32_t hi = bf16_pos((uint16_t)(pm[w] >> 16)) ? 0xffff0000u : 0u;
        pv[w] &= (lo | hi);
    }
    return v;
}

template <int MODE, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(NTHREADS) void igemm_bf16_kernel(const GemmParams p)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BM % 64 == 0 && BN % 64 == 0, "loader granularity");
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int AV = BM / 64, BV = BN / 64;            // 16-byte vectors (8 elements) per thread per stage
    constexpr int KS = BKH / 16;                         // MFMA k-steps per stage

    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM][LDKH];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN][LDKH];

    const int per_xcd = gridDim.x >> 3;
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= p.tiles * p.splits) return;
    const int split = L / p.tiles, tile = L - split * p.tiles;
    const int tile_n = tile % p.tilesN, tile_m = tile / p.tilesN;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const ConvGeo &g = p.g;
    const uint16_t *pa = reinterpret_cast<const uint16_t *>(p.a);
    const uint16_t *pb = reinterpret_cast<const uint16_t *>(p.b);
    const uint16_t *pmask = reinterpret_cast<const uint16_t *>(p.amask);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wave_m = wave / WN, wave_n = wave % WN;

    int kbeg = 0, kend = p.Kd;
    if (MODE == MODE_BWD_WEIGHT) {
        kbeg = split * p.chunks_per_split * BKH;
        kend = min(p.Kd, kbeg + p.chunks_per_split * BKH);
    }
    const int nchunks = (kend - kbeg + BKH - 1) / BKH;
    const bool amask = (p.flags & LOAD_AMASK) != 0;

    // reduction-contiguous fetch: thread -> vector kq (8 elements) of 4 along the stage, rows row0 + 64*i
    const int kq = t & 3, row0 = t >> 2;
    // row-contiguous fetch: thread -> vector c8 along the tile edge, reduction rows kr0 + RP*i
    constexpr int A_F8 = BM / 8, A_RP = NTHREADS / A_F8;
    constexpr int B_F8 = BN / 8, B_RP = NTHREADS / B_F8;

    int a_hb[AV], a_wb[AV], a_base[AV];
    int bw_r = 0, bw_s = 0, bw_c = 0;
    if (MODE == MODE_FWD) {
        const int HoWo = g.Ho * g.Wo;
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int m = m0 + row0 + 64 * i;
            if (m < p.M) {
                const int n = m / HoWo, pq = m - n * HoWo, pp = pq / g.Wo, q = pq - pp * g.Wo;
                a_hb[i] = pp * g.sh - g.ph;
                a_wb[i] = q * g.sw - g.pw;
                a_base[i] = n * g.H * g.W * g.C;
            } else {
                a_hb[i] = -(1 << 28); a_wb[i] = 0; a_base[i] = 0;
            }
        }
    } else if (MODE == MODE_BWD_DATA) {
        const int HW = g.H * g.W;
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int m = m0 + row0 + 64 * i;
            if (m < p.M) {
                const int n = m / HW, hw = m - n * HW, h = hw / g.W, w = hw - h * g.W;
                a_hb[i] = h + g.ph;
                a_wb[i] = w + g.pw;
                a_base[i] = n * g.Ho * g.Wo * g.K;
            } else {
                a_hb[i] = -(1 << 28); a_wb[i] = 0; a_base[i] = 0;
            }
        }
    } else {
        const int j = n0 + (t % B_F8) * 8;           // C % 8 == 0: the 8 columns share one tap
        bw_c = j % g.C;
        const int rs = j / g.C;
        bw_s = rs % g.S;
        bw_r = rs / g.S;
    }

    const bool tap_minor = MODE != MODE_BWD_WEIGHT && (p.flags & ORDER_TAP_MINOR);
    auto stage_k = [&](int ch) -> int {
        if (!tap_minor) return kbeg + ch * BKH;
        const int cblk = fdiv(ch, p.fd_rs), tap = ch - cblk * (g.R * g.S);
        return tap * (MODE == MODE_FWD ? g.C : g.K) + cblk * BKH;
    };

    uint4 ra[AV], rb[BV], rg[AV];
    unsigned oka = 0, okb = 0;
    const bool want_db = MODE == MODE_BWD_WEIGHT && (p.flags & EPI_DBIAS) && tile_n == 0;
    float dbacc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) dbacc[e] = 0.f;

    auto fetch_a = [&](int ch, int i) {
        const int kchunk = stage_k(ch);
        int off;
        bool ok;
        if (MODE == MODE_FWD || MODE == MODE_BWD_DATA) {
            const int CC = (MODE == MODE_FWD) ? g.C : g.K;
            const int kk = kchunk + kq * 8;
            const int rs = fdiv(kk, MODE == MODE_FWD ? p.fd_c : p.fd_k), cc = kk - rs * CC;
            const int ar = fdiv(rs, p.fd_s), as = rs - ar * g.S;
            if (MODE == MODE_FWD) {
                const int h = a_hb[i] + ar, w = a_wb[i] + as;
                ok = kk < p.Kd && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
                off = a_base[i] + (h * g.W + w) * g.C + cc;
            } else {
                int pp, q;
                ok = strided_src(a_hb[i] - ar, g.sh, g.Ho, pp);
                ok = strided_src(a_wb[i] - as, g.sw, g.Wo, q) && ok && kk < p.Kd;
                off = a_base[i] + (pp * g.Wo + q) * g.K + cc;
            }
        } else {
            const int col = m0 + (t % A_F8) * 8;
            const int pix = kchunk + t / A_F8 + A_RP * i;
            ok = pix < kend && col < p.M;
            off = pix * g.K + col;
        }
        off = ok ? off : 0;
        ra[i] = ldg16(pa + off);
        if (MODE != MODE_FWD && amask) rg[i] = ldg16(pmask + off);
        oka |= (unsigned)ok << i;
    };

    auto fetch_b = [&](int ch, int i) {
        const int kchunk = stage_k(ch);
        int off;
        bool ok;
        if (MODE == MODE_FWD) {
            const int j = n0 + row0 + 64 * i;
            const int kk = kchunk + kq * 8;
            ok = j < p.Nn && kk < p.Kd;
            off = j * p.Kd + kk;
        } else if (MODE == MODE_BWD_DATA) {
            const int col = n0 + (t % B_F8) * 8;
            const int kk = kchunk + t / B_F8 + B_RP * i;
            const int rs = fdiv(kk, p.fd_k), bk = kk - rs * g.K;
            const int br = fdiv(rs, p.fd_s), bs = rs - br * g.S;
            ok = kk < p.Kd && col < p.Nn;
            off = ((bk * g.R + br) * g.S + bs) * g.C + col;
        } else {
            const int col = n0 + (t % B_F8) * 8;
            const int pix = kchunk + t / B_F8 + B_RP * i;
            const int img = fdiv(pix, p.fd_howo), pq = pix - img * (g.Ho * g.Wo);
            const int pp = fdiv(pq, p.fd_wo), q = pq - pp * g.Wo;
            const int h = pp * g.sh - g.ph + bw_r, w = q * g.sw - g.pw + bw_s;
            ok = pix < kend && col < p.Nn && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
            off = ((img * g.H + h) * g.W + w) * g.C + bw_c;
        }
        rb[i] = ldg16(pb + (ok ? off : 0));
        okb |= (unsigned)ok << i;
    };

    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            uint4 v = ra[i];
            if (MODE != MODE_FWD && amask) v = gate8(v, rg[i]);
            if (!((oka >> i) & 1u)) v = make_uint4(0u, 0u, 0u, 0u);
            if (MODE == MODE_BWD_WEIGHT) {
                const int kr = t / A_F8 + A_RP * i, c8 = (t % A_F8) * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    As[buf][c8 + e][kr] = h8at(v, e);
                    if (want_db) dbacc[e] += bf16_to_f32(h8at(v, e));
                }
            } else {
                *reinterpret_cast<uint4 *>(&As[buf][row0 + 64 * i][kq * 8]) = v;
            }
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            uint4 v = rb[i];
            if (!((okb >> i) & 1u)) v = make_uint4(0u, 0u, 0u, 0u);
            if (MODE == MODE_FWD) {
                *reinterpret_cast<uint4 *>(&Bs[buf][row0 + 64 * i][kq * 8]) = v;
            } else {
                const int kr = t / B_F8 + B_RP * i, c8 = (t % B_F8) * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e) Bs[buf][c8 + e][kr] = h8at(v, e);
            }
        }
        oka = 0;
        okb = 0;
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#pragma unroll
    for (int i = 0; i < AV; ++i) fetch_a(0, i);
#pragma unroll
    for (int i = 0; i < BV; ++i) fetch_b(0, i);
    stash(0);
    __syncthreads();

    const int lrow = lane & 31, lk = lane >> 5;
    for (int ch = 0; ch < nchunks; ++ch) {
        const int buf = ch & 1;
#pragma unroll
        for (int i = 0; i < AV; ++i) fetch_a(ch + 1, i);
#pragma unroll
        for (int i = 0; i < BV; ++i) fetch_b(ch + 1, i);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                av[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&As[buf][wave_m * WTM + i * 32 + lrow][ks * 16 + lk * 8]));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bv[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&Bs[buf][wave_n * WTN + j * 32 + lrow][ks * 16 + lk * 8]));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        stash(buf ^ 1);
        __syncthreads();
    }

    if (MODE == MODE_BWD_WEIGHT && want_db) {
        // threads t, t + A_F8, ... hold partial sums of the same 8 channels: add them in thread order through LDS
        float *red = reinterpret_cast<float *>(&As[0][0][0]);
#pragma unroll
        for (int e = 0; e < 8; ++e) red[(t / A_F8) * BM + (t % A_F8) * 8 + e] = dbacc[e];
        __syncthreads();
        if (t < BM && m0 + t < p.M) {
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < A_RP; ++r) s += red[r * BM + t];
            p.dbias[(size_t)split * p.dbias_stride + m0 + t] = s;
        }
    }

    // epilogue: accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 tile
    uint16_t *outh = reinterpret_cast<uint16_t *>(p.out);
    const uint16_t *xm = reinterpret_cast<const uint16_t *>(p.xmask);
    const size_t split_off = (MODE == MODE_BWD_WEIGHT) ? (size_t)split * p.M * p.Nn : 0;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wave_n * WTN + j * 32 + lrow;
        if (col >= p.Nn) continue;
        float bias = 0.f;
        if (MODE == MODE_FWD && (p.flags & EPI_BIAS)) bias = p.bias[col];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wave_m * WTM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                if (row >= p.M) continue;
                const size_t o = (size_t)row * p.Nn + col;
                float v = acc[i][j][r];
                if (MODE == MODE_FWD) {
                    v += bias;
                    if (p.flags & EPI_RELU) v = fmaxf(v, 0.f);
                    outh[o] = f32_to_bf16(v);
                } else if (MODE == MODE_BWD_DATA) {
                    if (p.flags & EPI_ACCUM) v += bf16_to_f32(outh[o]);
                    if (p.flags & EPI_XMASK) v = bf16_pos(xm[o]) ? v : 0.f;
                    outh[o] = f32_to_bf16(v);
                } else {
                    p.out[split_off + o] = v;
                }
            }
        }
    }
}

}  // namespace stanza
