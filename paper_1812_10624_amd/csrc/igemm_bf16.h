// bf16-in / fp32-accumulate variant of the implicit-GEMM engine (same three gather modes and the same
// GemmParams as igemm.h; see there for the index conventions).  x, w, y, dy, dx are bfloat16; products are
// accumulated in float32 by v_mfma_f32_32x32x16_bf16; bias, filter gradients and bias gradients are float32.
//
// One MFMA lane supplies 8 consecutive reduction elements of one tile row.  Every operand goes global -> register
// -> LDS as 16-byte vectors in the order it has in memory, and nothing is transposed element by element:
//   * an operand whose reduction index is contiguous in memory (x and w in FWD, dy in BWD_DATA) is kept ROW-MAJOR
//     in LDS, [rows][BKH+8], and a lane reads its 8 elements with one 16-byte read;
//   * an operand whose row/column index is contiguous (w in BWD_DATA, dy and x in BWD_WEIGHT) is kept
//     REDUCTION-MAJOR, [BKH][rows+32], and is read with the gfx950 LDS transpose read (ds_read_b64_tr_b16): within
//     each group of 16 lanes, lane s points at 4 consecutive row elements of reduction row s/4, chunk s%4, and the
//     hardware hands lane i the 4 reduction elements of row i.  Two such reads give the lane its 8 elements.
//     (Lane layout checked on the device against a tile holding its own indices.)
// Fetches are buffer loads (a masked lane gets an out-of-range offset and the hardware returns zero), issued two
// stages ahead of their use: the registers of stage s+2 are loaded while stage s is multiplied and stage s+1 is
// written to LDS.  bf16 outputs leave through LDS so that every global store is a 16-byte vector of a full row
// segment; for that the MFMA operands are swapped (the accumulators hold the transposed tile, 4 consecutive output
// columns per lane).
#pragma once
#include "igemm.h"
#include <type_traits>

namespace stanza {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
constexpr int BKH = 64;        // reduction depth of one LDS stage (bf16 elements); also the filter-gradient slice unit
constexpr int KPAD = 32;       // row pad of a reduction-major tile: row stride = 64 bytes mod 256, so the four reduction rows
                               // a 16-lane group reads land on four different 64-byte bank groups

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
// Two floats rounded to nearest even and packed, through the hardware conversion (v_cvt_pk_bf16_f32): the same bits as
// f32_to_bf16 for every finite input, in one instruction instead of eight and without the branch around the NaN case (the
// epilogue converts 64 values per lane: written out it was 1,100 vector and 600 scalar instructions per tile and wavefront, as
// many as 18 stages of the main loop).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bool bf16_pos(uint16_t h) { return h != 0 && !(h & 0x8000u); }   // h > 0 (finite inputs)
__device__ __forceinline__ uint16_t h8at(const uint4 &v, int e) { return reinterpret_cast<const uint16_t *>(&v)[e]; }
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
__device__ __forceinline__ uint4 bload16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0));
}
// 4 consecutive reduction elements of this lane's row out of a reduction-major LDS tile (see the header comment)
__device__ __forceinline__ s16x4 lds_tr4(const uint16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
}

// AMASK: dy is gated by [y > 0] as it is read (a second fetch per A vector); without it the registers allow fetching two
// stages ahead.
template <int MODE, int BM, int BN, int WM, int WN, bool FAST, bool AMASK>
__device__ __forceinline__ void igemm_bf16_body(const GemmParams p)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BM % 64 == 0 && BN % 64 == 0, "loader granularity");
    constexpr int WTM = BM / WM, WTN = BN / WN;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && WTM <= 128, "MFMA granularity");
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int KS = BKH / 16;                         // MFMA k-steps per stage
    constexpr bool A_KMAJ = MODE == MODE_BWD_WEIGHT, B_KMAJ = MODE != MODE_FWD;
    constexpr bool SWAP = MODE != MODE_BWD_WEIGHT;       // bf16 output: accumulate the transposed tile
    constexpr int LDR = BKH + 8;                         // row-major tile: elements per row (144 bytes: conflict-free 16-byte reads)
    constexpr int LDAK = BM + KPAD, LDBK = BN + KPAD;    // reduction-major tiles: elements per reduction row
    constexpr int A_ELEMS = A_KMAJ ? BKH * LDAK : BM * LDR;
    constexpr int B_ELEMS = B_KMAJ ? BKH * LDBK : BN * LDR;
    constexpr int STAGE = A_ELEMS + B_ELEMS;
    constexpr int CROWS = BM < 128 ? BM : 128;           // output rows staged per epilogue pass
    constexpr int LDC = BN + 8;
    constexpr int C_ELEMS = SWAP ? CROWS * LDC : 0;
    constexpr int SMEM = 2 * STAGE > C_ELEMS ? 2 * STAGE : C_ELEMS;
    __shared__ __attribute__((aligned(16))) uint16_t smem[SMEM];

    // 16-byte vectors per thread per stage and their thread mapping
    constexpr int KQ = BKH / 8, RPP = NTHREADS / KQ;     // row-major fetch: vector kq along the stage, rows row0 + RPP*i
    constexpr int A_F8 = BM / 8, A_RP = NTHREADS / A_F8; // reduction-major fetch: vector c8 along the tile edge, rows kr0 + RP*i
    constexpr int B_F8 = BN / 8, B_RP = NTHREADS / B_F8;
    constexpr int AV = BM * BKH / 8 / NTHREADS, BV = BN * BKH / 8 / NTHREADS;
    static_assert(AV >= 1 && BV >= 1, "tile too small for the loader");

    const int per_xcd = gridDim.x >> 3;
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= p.tiles * p.splits) return;
    const int split = L / p.tiles, tile = L - split * p.tiles;
    const int tile_n = tile % p.tilesN, tile_m = tile / p.tilesN;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const ConvGeo &g = p.g;
    // taps the reduction runs over: all of them, or those of the stride class (BWD_DATA)
    const int tapS = MODE == MODE_BWD_DATA ? p.sub.Sc : g.S;
    const int tapRS = MODE == MODE_BWD_DATA ? p.sub.Rc * p.sub.Sc : g.R * g.S;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wave_m = wave / WN, wave_n = wave % WN;

    int kbeg = 0, kend = p.Kd;
    if (MODE == MODE_BWD_WEIGHT) {
        kbeg = split * p.chunks_per_split * BKH;
        kend = min(p.Kd, kbeg + p.chunks_per_split * BKH);
    }
    const int nchunks = (kend - kbeg + BKH - 1) / BKH;
    constexpr bool amask = AMASK;

    const int kq = t % KQ, row0 = t / KQ;
    int a_hb[AV], a_wb[AV], a_base[AV], a_row[AV], b_row[BV];
    int bw_r = 0, bw_s = 0, bw_c = 0;
    if (MODE == MODE_FWD) {
        const int HoWo = g.Ho * g.Wo;
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int m = m0 + row0 + RPP * i;
            if (m < p.M) {
                const int n = fdiv(m, p.fd_howo), pq = m - n * HoWo, pp = fdiv(pq, p.fd_wo), q = pq - pp * g.Wo;
                a_hb[i] = pp * g.sh - g.ph;
                a_wb[i] = q * g.sw - g.pw;
                a_base[i] = n * g.H * g.W * g.C;
            } else {
                a_hb[i] = -(1 << 28); a_wb[i] = 0; a_base[i] = 0;
            }
            a_row[i] = m < p.M ? a_base[i] + (a_hb[i] * g.W + a_wb[i]) * g.C + kq * 8 : 0;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) b_row[i] = (n0 + row0 + RPP * i) * p.Kd + kq * 8;
    } else if (MODE == MODE_BWD_DATA) {
        const int HW = p.sub.Hc * p.sub.Wc;      // rows are the pixels of one stride class (igemm.h, StrideClass)
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int m = m0 + row0 + RPP * i;
            if (m < p.M) {
                const int n = fdiv(m, p.fd_hcwc), hw = m - n * HW, ci = fdiv(hw, p.fd_wc), cj = hw - ci * p.sub.Wc;
                a_hb[i] = ci + p.sub.pa;
                a_wb[i] = cj + p.sub.qb;
                a_base[i] = n * g.Ho * g.Wo * g.K;
            } else {
                a_hb[i] = -(1 << 28); a_wb[i] = 0; a_base[i] = 0;
            }
            a_row[i] = m < p.M ? a_base[i] + (a_hb[i] * g.Wo + a_wb[i]) * g.K + kq * 8 : 0;   // source pixel of tap (0,0) of the class
        }
#pragma unroll
        for (int i = 0; i < BV; ++i)   // w[k][r][s][c] at k = this thread's reduction row, tap (0,0), its 8 columns
            b_row[i] = (t / B_F8 + B_RP * i) * (g.R * g.S * g.C) + n0 + (t % B_F8) * 8;
    } else {
        const int j = n0 + (t % B_F8) * 8;           // C % 8 == 0: the 8 columns share one tap
        const int rs = fdiv(j, p.fd_c);
        bw_c = j - rs * g.C;
        bw_r = fdiv(rs, p.fd_s);                     // >= R when j >= Nn: the column predicate covers it
        bw_s = rs - bw_r * g.S;
#pragma unroll
        for (int i = 0; i < AV; ++i) { a_hb[i] = a_wb[i] = a_base[i] = a_row[i] = 0; }
#pragma unroll
        for (int i = 0; i < BV; ++i) b_row[i] = 0;
    }

    // FAST path state (see fetch): tap validity mask per A row, static validity per B vector, running stage position
    // (the host takes this path for at most 32 taps)
    uint32_t a_mask[AV];
    uint32_t b_oob[BV];          // 0, or OOB_OFF for a B vector beyond the column range
    int f_cblk = 0, f_tap = 0, f_ar = 0, f_as = 0;
    if (FAST) {
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            // bit (ar * tapS + as) = row tap ar inside the image AND column tap as inside it: the column bits once, then one
            // shifted copy per valid row tap (R + S steps instead of R * S)
            uint32_t cb = 0;
            for (int as = 0; as < tapS; ++as)
                cb |= (uint32_t)(MODE == MODE_FWD ? (unsigned)(a_wb[i] + as) < (unsigned)g.W : (unsigned)(a_wb[i] - as) < (unsigned)g.Wo) << as;
            uint32_t mk = 0;
            for (int ar = 0, sh = 0; sh < tapRS; ++ar, sh += tapS) {
                const bool ok = MODE == MODE_FWD ? (unsigned)(a_hb[i] + ar) < (unsigned)g.H : (unsigned)(a_hb[i] - ar) < (unsigned)g.Ho;
                mk |= ok ? cb << sh : 0u;
            }
            a_mask[i] = mk;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) b_oob[i] = (MODE == MODE_FWD ? (n0 + row0 + RPP * i < p.Nn) : (n0 + (t % B_F8) * 8 < p.Nn)) ? 0u : OOB_OFF;
    }

    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(p.a, p.a_bytes);
    const __amdgpu_buffer_rsrc_t rsrc_g = make_rsrc(p.amask ? p.amask : p.a, p.a_bytes);
    const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(p.b, p.b_bytes);

    // two register sets: set (s & 1) holds stage s from its fetch until it is written to LDS; one set when the gate vectors
    // take the registers of the second
    constexpr bool PREFETCH2 = !AMASK && (FAST || MODE == MODE_BWD_WEIGHT);   // (the per-element address arithmetic of the general
                                                                             // forward / backward-data path needs the registers)
    uint4 ra[PREFETCH2 ? 2 : 1][AV], rb[PREFETCH2 ? 2 : 1][BV], rg[PREFETCH2 ? 2 : 1][AV];
    const bool want_db = MODE == MODE_BWD_WEIGHT && (p.flags & EPI_DBIAS) && tile_n == 0;
    float dbacc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) dbacc[e] = 0.f;

    // Issue part `part` of `nparts` of the global loads of stage `ch` into register set `set` (vector i belongs to part
    // i % nparts; the running state of the fast path moves on with the last part).  Stages past the end are fetched fully masked.
    auto fetch = [&](int ch, auto set_c, int part, int nparts) {
        constexpr int set = decltype(set_c)::value;
        const bool kok = ch < nchunks;
        if (FAST) {
            // channel-block-major, tap-minor visiting order: the taps of one channel block re-read the same image rows.
            // Stages are fetched in ascending order, so (channel block, tap row, tap column) is a running scalar state, a
            // row's tap validity is one bit of its precomputed mask, and an address is its precomputed row offset plus a scalar.
            int sa, sb;      // wavefront-uniform byte offsets of this stage
            if (MODE == MODE_FWD) {
                sa = ((f_ar * g.W + f_as) * g.C + f_cblk * BKH) * 2;
                sb = (f_tap * g.C + f_cblk * BKH) * 2;
            } else {
                sa = (f_cblk * BKH - (f_ar * g.Wo + f_as) * g.K) * 2;
                const int wtap = (p.sub.r0 + f_ar * g.sh) * g.S + p.sub.s0 + f_as * g.sw;    // the filter tap this class tap stands for
                sb = ((f_cblk * BKH * (g.R * g.S) + wtap) * g.C) * 2;
            }
            // A masked lane gets bit 31 of its offset set (any such offset is past the end of the buffer, whose size is below
            // 2 GiB, so the load returns zero); written as arithmetic on purpose: selects here made the compiler wrap every
            // load in its own branch, which cut the loop into pieces it could not schedule across.
            const uint32_t koff = kok ? 0u : OOB_OFF;
#pragma unroll
            for (int i = 0; i < AV; ++i) {
                if (i % nparts != part) continue;
                const uint32_t bo = (uint32_t)(a_row[i] * 2 + sa) | koff | ((~(a_mask[i] >> f_tap) & 1u) << 31);
                ra[set][i] = bload16(rsrc_a, bo);
                if (MODE == MODE_BWD_DATA && amask) rg[set][i] = bload16(rsrc_g, bo);
            }
#pragma unroll
            for (int i = 0; i < BV; ++i) {
                if (i % nparts != part) continue;
                rb[set][i] = bload16(rsrc_b, (uint32_t)(b_row[i] * 2 + sb) | koff | b_oob[i]);
            }
            if (part != nparts - 1) return;
            ++f_tap;
            ++f_as;
            const int wrap_s = f_as == tapS, wrap_t = f_tap == tapRS;
            f_as = wrap_s ? 0 : f_as;
            f_ar += wrap_s;
            f_as = wrap_t ? 0 : f_as;
            f_ar = wrap_t ? 0 : f_ar;
            f_tap = wrap_t ? 0 : f_tap;
            f_cblk += wrap_t;
            return;
        }
        const int kchunk = kbeg + ch * BKH;
#pragma unroll
        // (validity as 0 / 1 integers combined with &, and masked lanes by setting bit 31 of the offset: see the fast path)
        for (int i = 0; i < AV; ++i) {
            if (i % nparts != part) continue;
            int off;
            uint32_t ok;
            if (MODE == MODE_FWD || MODE == MODE_BWD_DATA) {
                const int CC = (MODE == MODE_FWD) ? g.C : g.K;
                const int kk = kchunk + kq * 8;
                const int rs = fdiv(kk, MODE == MODE_FWD ? p.fd_c : p.fd_k), cc = kk - rs * CC;
                const int ar = fdiv(rs, p.fd_s), as = rs - ar * tapS;
                if (MODE == MODE_FWD) {
                    const int h = a_hb[i] + ar, w = a_wb[i] + as;
                    ok = (uint32_t)(kk < p.Kd) & (uint32_t)((unsigned)h < (unsigned)g.H) & (uint32_t)((unsigned)w < (unsigned)g.W);
                    off = a_base[i] + (h * g.W + w) * g.C + cc;
                } else {
                    const int pp = a_hb[i] - ar, q = a_wb[i] - as;
                    ok = (uint32_t)(kk < p.Kd) & (uint32_t)((unsigned)pp < (unsigned)g.Ho) & (uint32_t)((unsigned)q < (unsigned)g.Wo);
                    off = a_base[i] + (pp * g.Wo + q) * g.K + cc;
                }
            } else {
                const int col = m0 + (t % A_F8) * 8;
                const int pix = kchunk + t / A_F8 + A_RP * i;
                ok = (uint32_t)(pix < kend) & (uint32_t)(col < p.M);
                off = pix * g.K + col;
            }
            const uint32_t bo = ((uint32_t)off * 2u & 0x7fffffffu) | ((ok ^ 1u) << 31);
            ra[set][i] = bload16(rsrc_a, bo);
            if (MODE != MODE_FWD && amask) rg[set][i] = bload16(rsrc_g, bo);
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            if (i % nparts != part) continue;
            int off;
            uint32_t ok;
            if (MODE == MODE_FWD) {
                const int j = n0 + row0 + RPP * i;
                const int kk = kchunk + kq * 8;
                ok = (uint32_t)(j < p.Nn) & (uint32_t)(kk < p.Kd);
                off = j * p.Kd + kk;
            } else if (MODE == MODE_BWD_DATA) {
                const int col = n0 + (t % B_F8) * 8;
                const int kk = kchunk + t / B_F8 + B_RP * i;
                const int rs = fdiv(kk, p.fd_k), bk = kk - rs * g.K;
                const int tr = fdiv(rs, p.fd_s), ts = rs - tr * tapS;
                const int br = p.sub.r0 + tr * g.sh, bs = p.sub.s0 + ts * g.sw;
                ok = (uint32_t)(kk < p.Kd) & (uint32_t)(col < p.Nn);
                off = ((bk * g.R + br) * g.S + bs) * g.C + col;
            } else {
                const int col = n0 + (t % B_F8) * 8;
                const int pix = kchunk + t / B_F8 + B_RP * i;
                const int img = fdiv(pix, p.fd_howo), pq = pix - img * (g.Ho * g.Wo);
                const int pp = fdiv(pq, p.fd_wo), q = pq - pp * g.Wo;
                const int h = pp * g.sh - g.ph + bw_r, w = q * g.sw - g.pw + bw_s;
                ok = (uint32_t)(pix < kend) & (uint32_t)(col < p.Nn) & (uint32_t)((unsigned)h < (unsigned)g.H) & (uint32_t)((unsigned)w < (unsigned)g.W);
                off = ((img * g.H + h) * g.W + w) * g.C + bw_c;
            }
            rb[set][i] = bload16(rsrc_b, ((uint32_t)off * 2u & 0x7fffffffu) | ((ok ^ 1u) << 31));
        }
    };

    // Gate and write part `part` of `nparts` of register set `set` into LDS buffer `buf` (vector v of the AV + BV vectors
    // belongs to part v * nparts / (AV + BV)).
    auto stash = [&](auto set_c, int buf, int part, int nparts) {
        constexpr int set = decltype(set_c)::value;
        uint16_t *As = smem + buf * STAGE, *Bs = As + A_ELEMS;
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            if (i * nparts / (AV + BV) != part) continue;
            uint4 v = ra[set][i];
            if (MODE != MODE_FWD && amask) v = gate8(v, rg[set][i]);
            if (A_KMAJ) {
                *reinterpret_cast<uint4 *>(&As[(t / A_F8 + A_RP * i) * LDAK + (t % A_F8) * 8]) = v;
                ra[set][i] = v;      // the gated vector, for the bias-gradient sums below
            } else {
                *reinterpret_cast<uint4 *>(&As[(row0 + RPP * i) * LDR + kq * 8]) = v;
            }
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            if ((AV + i) * nparts / (AV + BV) != part) continue;
            if (B_KMAJ) *reinterpret_cast<uint4 *>(&Bs[(t / B_F8 + B_RP * i) * LDBK + (t % B_F8) * 8]) = rb[set][i];
            else *reinterpret_cast<uint4 *>(&Bs[(row0 + RPP * i) * LDR + kq * 8]) = rb[set][i];
        }
        if (A_KMAJ && want_db && part == nparts - 1) {      // one workgroup-uniform branch per stage, after the stores
#pragma unroll
            for (int i = 0; i < AV; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) dbacc[e] += bf16_to_f32(h8at(ra[set][i], e));
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int lrow = lane & 31, lk = lane >> 5;
    // transpose-read lane roles: 16-lane group G covers tile rows 16*(G&1).. and reduction rows 8*(G>>1)..
    const int tr_m = 16 * ((lane >> 4) & 1) + 4 * (lane & 3), tr_k = 8 * (lane >> 5) + ((lane >> 2) & 3);

    // MFMA operands of one k-step, two register slots: slot (ks & 1) is multiplied while the other is being read.
    bf16x8 av[2][TM], bv[2][TN];
    auto load_ops = [&](int buf, int ks, auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
        const uint16_t *As = smem + buf * STAGE, *Bs = As + A_ELEMS;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (A_KMAJ) {
                const uint16_t *q = &As[(ks * 16 + tr_k) * LDAK + wave_m * WTM + i * 32 + tr_m];
                const s16x4 lo = lds_tr4(q), hi = lds_tr4(q + 4 * LDAK);
                av[slot][i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            } else {
                av[slot][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&As[(wave_m * WTM + i * 32 + lrow) * LDR + ks * 16 + lk * 8]));
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (B_KMAJ) {
                const uint16_t *q = &Bs[(ks * 16 + tr_k) * LDBK + wave_n * WTN + j * 32 + tr_m];
                const s16x4 lo = lds_tr4(q), hi = lds_tr4(q + 4 * LDBK);
                bv[slot][j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            } else {
                bv[slot][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&Bs[(wave_n * WTN + j * 32 + lrow) * LDR + ks * 16 + lk * 8]));
            }
        }
    };
    auto mfma = [&](auto slot_c, int i, int j) {
        constexpr int slot = decltype(slot_c)::value;
        acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[slot][j], av[slot][i], acc[i][j], 0, 0, 0)
                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[slot][i], bv[slot][j], acc[i][j], 0, 0, 0);
    };

    constexpr std::integral_constant<int, 0> S0{};
    constexpr std::integral_constant<int, 1> S1{};
    static_assert(KS % 2 == 0 && KS >= 4, "operand slots alternate by k-step and a stage ends on slot 1");
    // One stage = KS k-steps.  K-step ks: read the operands of k-step ks + 1 (of the NEXT stage's k-step 0 in the last one), then
    // its MFMAs with a slice of the global fetch after the first and a slice of the LDS writes of the next stage after the
    // second.  The LDS writes end with k-step KS - 2, whose MFMAs are followed by the stage's one barrier: after it the next
    // stage's buffer is complete (so its k-step 0 can be read under the last k-step's MFMAs) and nobody reads the buffer that
    // the stage after it will overwrite (a stage's last LDS reads are issued before its barrier).
    auto stage = [&](int ch, auto par_c) {
        constexpr int par = decltype(par_c)::value;
        constexpr std::integral_constant<int, PREFETCH2 ? par : 0> set_f{};          // fetch target
        constexpr std::integral_constant<int, PREFETCH2 ? (par ^ 1) : 0> set_s{};    // register set written to LDS
        const int fch = ch + (PREFETCH2 ? 2 : 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks < KS - 1) {
                if (ks & 1) load_ops(par, ks + 1, S0); else load_ops(par, ks + 1, S1);
            } else {
                load_ops(par ^ 1, 0, S0);
            }
            __builtin_amdgcn_sched_barrier(0);
            int n = 0;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (ks & 1) mfma(S1, i, j); else mfma(S0, i, j);
                    __builtin_amdgcn_sched_barrier(0);
                    if (n == 0) {
                        // two register sets: the fetch is spread over the k-steps; one set: all of it first, its LDS writes last
                        if (PREFETCH2) fetch(fch, set_f, ks, KS);
                        else if (ks == 0) fetch(fch, set_f, 0, 1);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (n == (TM * TN > 1 ? 1 : 0)) {
                        if (PREFETCH2) { if (ks < KS - 1) stash(set_s, par ^ 1, ks, KS - 1); }
                        else if (ks == KS - 2) stash(set_s, par ^ 1, 0, 1);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    ++n;
                }
            if (ks == KS - 2) {
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // A stage left to the compiler's own schedule: used when a wavefront has fewer than four MFMAs per k-step (64-row or
    // 64-column tiles), too few to cover a k-step's reads one step ahead; there the pinned order above is the slower one.
    auto compute = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            load_ops(buf, ks, S0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mfma(S0, i, j);
        }
    };

    fetch(0, S0, 0, 1);
    stash(S0, 0, 0, 1);
    if constexpr (PREFETCH2) fetch(1, S1, 0, 1);
    __syncthreads();
    if constexpr (TM * TN >= 4) {
        load_ops(0, 0, S0);
        __builtin_amdgcn_sched_barrier(0);
        for (int ch = 0; ch < nchunks; ch += 2) {
            stage(ch, S0);
            if (ch + 1 >= nchunks) break;
            stage(ch + 1, S1);
        }
    } else if constexpr (PREFETCH2) {
        for (int ch = 0; ch < nchunks; ch += 2) {
            fetch(ch + 2, S0, 0, 1);
            compute(0);
            stash(S1, 1, 0, 1);
            __syncthreads();
            if (ch + 1 >= nchunks) break;
            fetch(ch + 3, S1, 0, 1);
            compute(1);
            stash(S0, 0, 0, 1);
            __syncthreads();
        }
    } else {
        for (int ch = 0; ch < nchunks; ++ch) {
            fetch(ch + 1, S0, 0, 1);
            compute(ch & 1);
            stash(S0, (ch + 1) & 1, 0, 1);
            __syncthreads();
        }
    }

    if (MODE == MODE_BWD_WEIGHT && want_db) {
        // threads t, t + A_F8, ... hold partial sums of the same 8 channels: add them in thread order through LDS
        __syncthreads();
        float *red = reinterpret_cast<float *>(smem);
        static_assert(A_RP * BM * 4 <= SMEM * 2, "bias-gradient scratch fits in the stage buffers");
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

    if (!SWAP) {
        // float32 tile (filter gradient or a reduction slice of it): register r of lane l is row 8*(r/4) + 4*(l/32) + r%4,
        // column l%32 of its 32x32 tile
        const size_t split_off = (size_t)split * p.M * p.Nn;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wave_n * WTN + j * 32 + lrow;
            if (col >= p.Nn) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + wave_m * WTM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                    if (row < p.M) p.out[split_off + (size_t)row * p.Nn + col] = acc[i][j][r];
                }
            }
        }
        return;
    }

    // bf16 tile.  Operands were swapped, so register r of lane l is output row l%32, column 8*(r/4) + 4*(l/32) + r%4 of its
    // 32x32 tile: 4 consecutive columns per register quad.  Bias and ReLU are applied here, the tile is staged in LDS
    // (CROWS rows at a time), and read back as 16-byte row vectors for the accumulate / mask / store.
    uint16_t *outh = reinterpret_cast<uint16_t *>(p.out);
    const uint16_t *xm = reinterpret_cast<const uint16_t *>(p.xmask);
    constexpr int CH8 = BN / 8, ROWS_PER_PASS = NTHREADS / CH8;
    // element offset of (row, col) in the output: dense rows, or the scattered pixels of a stride class
    auto out_index = [&](int row, int col) -> size_t {
        if (MODE == MODE_BWD_DATA && (p.flags & OUT_STRIDED)) {
            const int n = fdiv(row, p.fd_hcwc), hw = row - n * (p.sub.Hc * p.sub.Wc);
            const int ci = fdiv(hw, p.fd_wc), cj = hw - ci * p.sub.Wc;
            return ((size_t)(n * g.H + p.sub.h0 + ci * g.sh) * g.W + p.sub.w0 + cj * g.sw) * g.C + col;
        }
        return (size_t)row * p.Nn + col;
    };
    // What the staging reads from global memory is loaded in clusters before it starts (the bias of this lane's columns once, the
    // residual or the previous gradient of a whole staging pass together): one load after the other, each waited for where it is
    // used, was 8 to 24 memory round trips in a row per tile, as long as the whole main loop of a 64-deep reduction.
    float4 bias4[TN][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) bias4[j][q4] = zero4();
    if (MODE == MODE_FWD && (p.flags & EPI_BIAS)) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int col_l = wave_n * WTN + j * 32 + 8 * q4 + 4 * lk;
                if (n0 + col_l < p.Nn) bias4[j][q4] = ldg4(p.bias + n0 + col_l);
            }
    }
    const bool want_add = MODE == MODE_FWD ? (p.flags & EPI_RESIDUAL) != 0 : MODE == MODE_BWD_DATA ? (p.flags & EPI_ACCUM) != 0 : false;
#pragma unroll
    for (int half = 0; half < BM / CROWS; ++half) {
        __syncthreads();
        if ((wave_m * WTM) / CROWS == half) {
            uint2 add2[TN][4][TM];
            if (want_add) {
                // FWD: the shortcut's bf16 tensor of a residual join (added in float32, before the ReLU and the one rounding);
                // BWD_DATA: the previous gradient (residual joins only)
                const uint16_t *src = MODE == MODE_FWD ? reinterpret_cast<const uint16_t *>(p.res) : outh;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                        for (int i = 0; i < TM; ++i) {
                            const int col = n0 + wave_n * WTN + j * 32 + 8 * q4 + 4 * lk, row = m0 + wave_m * WTM + i * 32 + lrow;
                            add2[j][q4][i] = (row < p.M && col < p.Nn) ? *reinterpret_cast<const uint2 *>(src + out_index(row, col)) : make_uint2(0u, 0u);
                        }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int col_l = wave_n * WTN + j * 32 + 8 * q4 + 4 * lk;
                    const float4 bias = bias4[j][q4];
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const int row_l = wave_m * WTM + i * 32 + lrow - half * CROWS;
                        float v0 = acc[i][j][4 * q4 + 0] + bias.x, v1 = acc[i][j][4 * q4 + 1] + bias.y;
                        float v2 = acc[i][j][4 * q4 + 2] + bias.z, v3 = acc[i][j][4 * q4 + 3] + bias.w;
                        if (want_add) {
                            const uint2 rr = add2[j][q4][i];
                            v0 += bf16_to_f32((uint16_t)(rr.x & 0xffffu)); v1 += bf16_to_f32((uint16_t)(rr.x >> 16));
                            v2 += bf16_to_f32((uint16_t)(rr.y & 0xffffu)); v3 += bf16_to_f32((uint16_t)(rr.y >> 16));
                        }
                        if (MODE == MODE_FWD && (p.flags & EPI_RELU)) {
                            v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f);
                        }
                        *reinterpret_cast<uint2 *>(&smem[row_l * LDC + col_l]) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
                    }
                }
            }
        }
        __syncthreads();
        // The masks of up to eight passes are loaded before the first of their stores: loads and stores share one counter and
        // return out of order with respect to each other, so a load waited for with stores in flight waits for those stores too
        // (pass by pass, every pass cost a round trip to memory).  The accumulators are dead by now: the registers are there.
        constexpr int PASSES = CROWS / ROWS_PER_PASS, PG = PASSES < 8 ? PASSES : 8;
        static_assert(PASSES % PG == 0, "pass groups");
        const int c8 = (t % CH8) * 8, col = n0 + c8;
        const bool want_m = MODE == MODE_BWD_DATA && (p.flags & EPI_XMASK);
#pragma unroll
        for (int grp = 0; grp < PASSES / PG; ++grp) {
            uint4 pre_m[PG];
            if (want_m) {
#pragma unroll
                for (int q = 0; q < PG; ++q) {
                    const int row = m0 + half * CROWS + (grp * PG + q) * ROWS_PER_PASS + t / CH8;
                    pre_m[q] = (row < p.M && col < p.Nn) ? *reinterpret_cast<const uint4 *>(xm + out_index(row, col)) : make_uint4(0u, 0u, 0u, 0u);
                }
            }
#pragma unroll
            for (int q = 0; q < PG; ++q) {
                const int row_l = (grp * PG + q) * ROWS_PER_PASS + t / CH8;
                const int row = m0 + half * CROWS + row_l;
                if (row >= p.M || col >= p.Nn) continue;
                uint4 v = *reinterpret_cast<const uint4 *>(&smem[row_l * LDC + c8]);
                if (want_m) v = gate8(v, pre_m[q]);
                *reinterpret_cast<uint4 *>(outh + out_index(row, col)) = v;
            }
        }
    }
}

template <int MODE, int BM, int BN, int WM, int WN, bool FAST, bool AMASK>
__global__ __launch_bounds__(NTHREADS, 2) void igemm_bf16_kernel(const GemmParams p)
{
    igemm_bf16_body<MODE, BM, BN, WM, WN, FAST, AMASK>(p);
}

// The stride classes of a strided layer's data gradient in one launch (see igemm_classes_kernel): blockIdx.y = class.
template <int BM, int BN, int WM, int WN, bool FAST, bool AMASK>
__global__ __launch_bounds__(NTHREADS, 2) void igemm_bf16_classes_kernel(const GemmClasses P)
{
    igemm_bf16_body<MODE_BWD_DATA, BM, BN, WM, WN, FAST, AMASK>(P.q[blockIdx.y]);
}

}  // namespace stanza
