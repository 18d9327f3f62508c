// Implicit-GEMM engine for gfx950: one LDS-tiled, MFMA (v_mfma_f32_32x32x2_f32) main loop with
// three operand-gather modes that cover the convolution forward pass and its two adjoints
// (paper Sec. 3.2: CONV worker forward and backpropagation) and, with H = W = R = S = 1, the FC
// worker's three GEMMs.
//
//   FWD         C[m=(n,p,q)][j=k]       = sum_{(r,s,c)} x[n,p*sh-ph+r,q*sw-pw+s,c] * w[k,r,s,c]
//   BWD_DATA    C[m=(n,h,w)][j=c]       = sum_{(r,s,k)} dy[n,(h+ph-r)/sh,(w+pw-s)/sw,k] * w[k,r,s,c]
//   BWD_WEIGHT  C[m=k][j=(r,s,c)]       = sum_{(n,p,q)} dy[n,p,q,k] * x[n,p*sh-ph+r,q*sw-pw+s,c]
//
// An operand whose reduction index is contiguous in memory (x and w in FWD, dy in BWD_DATA) is fetched as
// 16-byte vectors along the reduction and kept row-major in LDS; an operand whose GEMM row/column index is
// contiguous (w in BWD_DATA, dy and x in BWD_WEIGHT) is fetched as 16-byte vectors along the tile edge and
// kept reduction-major.  Out-of-image taps, ragged tile edges and the reduction tail are predicated loads
// that yield zero; nothing is padded in memory.
//
// Work items.  A launch holds `dp_tiles` whole output tiles followed by `split_tiles` tiles whose reduction
// is cut into `splits` slices (every tile for BWD_WEIGHT with a long reduction; for FWD / BWD_DATA only the
// last few tiles, so that the final partial round of workgroups is made of short items and the CUs finish
// together).  A slice item writes its raw accumulators to a workspace; a second kernel adds the slices in
// slice order and applies the epilogue.  Which tiles are sliced depends on the shape alone.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stanza {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;         // reduction depth of one LDS stage
constexpr int NTHREADS = 256;  // 4 wavefronts
constexpr int KQ = BK / 4;     // 16-byte vectors along the reduction per tile row
constexpr int PAD_V = 4;  // row pad of a tile written as 16-byte vectors (keeps rows 16-byte aligned)

enum { MODE_FWD = 0, MODE_BWD_DATA = 1, MODE_BWD_WEIGHT = 2 };

enum : uint32_t {
    EPI_BIAS = 1u,     // FWD: + bias[j]
    EPI_RELU = 2u,     // FWD: max(.,0)
    EPI_RESIDUAL = 512u,   // FWD: + res[row][col] (a residual join: the shortcut's tensor, same shape as the output) before the ReLU
    EPI_ACCUM = 4u,    // BWD_DATA: += previous contents
    EPI_XMASK = 8u,    // BWD_DATA: * [xmask > 0]
    EPI_SGD = 16u,     // BWD_WEIGHT: fused momentum-SGD update of sgd_w / sgd_v with the tile as gradient
    LOAD_AMASK = 32u,  // BWD_*: dy is gated by [amask > 0] as it is read
    EPI_DBIAS = 64u,   // BWD_WEIGHT: column-tile-0 workgroups also sum dy over their reduction slice (bias gradient)
    OUT_STRIDED = 256u,     // BWD_DATA: the rows of this launch are one stride class of a strided layer (scattered dx pixels)
    ORDER_TAP_MINOR = 128u, // FWD / BWD_DATA: visit the reduction channel-block-major, tap-minor (needs channels % BK == 0)
    EPI_STATS = 1024u       // FWD (Nn % 4 == 0, no ReLU / residual): also write per-tile column sums of the output, see StatsHeader
};

// Column statistics of a forward output, written by the epilogue so that a normalisation layer that follows need not read the
// tensor once more to get them.  The buffer starts with this header (8 words), then one entry of [3][bn] floats per whole tile
// (entry index = tile index, tile = tile_m * tilesN + tile_n) and, for a tile that was cut into reduction slices, one entry per
// 1024 / bn of its rows (entry index = dp_tiles + (tile - dp_tiles) * (bm * bn / 1024) + row block), written by the fix-up
// kernel.  An entry holds, for each of the tile's columns: sum (y - k), sum (y - k)^2 and k, where k is the entry's first row
// (a shift inside the data's range, so that the squares do not cancel).  The row count of an entry follows from the header.
struct StatsHeader {
    int magic, tilesM, tilesN, dp_tiles, bm, bn, M, Nn;
};
constexpr int STATS_MAGIC = 0x53544154;
constexpr int STATS_HEADER_FLOATS = 8;

struct ConvGeo {
    int N, H, W, C, K, R, S, sh, sw, ph, pw, Ho, Wo;
};

// Division of a non-negative 31-bit value by a launch-time constant: q = (n * mul) >> sh  (exact for n < 2^31).
struct FastDiv {
    uint32_t mul, sh;
};
__host__ inline FastDiv make_fastdiv(uint32_t d)
{
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    FastDiv f;
    f.mul = (uint32_t)(((1ull << (31 + l)) / d) + 1);
    f.sh = 31 + l;
    return f;
}
__device__ __forceinline__ int fdiv(int n, FastDiv f) { return (int)(((uint64_t)(uint32_t)n * f.mul) >> f.sh); }

// BWD_DATA works on one stride class of the input pixels at a time: the pixels (h0 + i*sh, w0 + j*sw), 0 <= i < Hc, 0 <= j < Wc,
// all of which receive contributions from the same taps (r0 + tr*sh, s0 + ts*sw), 0 <= tr < Rc, 0 <= ts < Sc, namely from the
// output pixels (pa + i - tr, qb + j - ts).  Within a class the adjoint is a unit-stride problem and no tap is ever skipped
// for a stride mismatch.  A unit-stride layer is the single class h0 = w0 = r0 = s0 = 0, Hc = H, Wc = W, Rc = R, Sc = S,
// pa = pad_h, qb = pad_w.
struct StrideClass {
    int h0, w0, Hc, Wc, pa, qb, r0, s0, Rc, Sc;
};

struct GemmParams {
    ConvGeo g;
    StrideClass sub;      // BWD_DATA only
    FastDiv fd_c, fd_k, fd_s, fd_howo, fd_wo, fd_rs;   // divisors C, K, S, Ho*Wo, Wo, R*S (BWD_DATA: Sc and Rc*Sc of the class)
    FastDiv fd_hcwc, fd_wc;                            // BWD_DATA epilogue of a strided layer: Hc*Wc, Wc
    const float *a;       // FWD: x      BWD_DATA: dy   BWD_WEIGHT: dy
    const float *amask;   // BWD_*: forward output y gating dy, or nullptr
    const float *b;       // FWD: w      BWD_DATA: w    BWD_WEIGHT: x
    float *out;           // FWD: y      BWD_DATA: dx   BWD_WEIGHT: dw or split partials [split][M*Nn]
    const float *bias;    // FWD
    const float *xmask;   // BWD_DATA
    float *dbias;         // EPI_DBIAS: [M] or split partials (stride dbias_stride floats per slice)
    size_t dbias_stride;
    float *sgd_w, *sgd_v; // EPI_SGD
    const float *res;     // EPI_RESIDUAL (element type of the output)
    float *stats;         // EPI_STATS: header + entries
    float lr, mom, wd;
    int M, Nn, Kd;        // GEMM extents (Kd = full reduction length)
    int tilesM, tilesN, tiles;
    int dp_tiles;         // tiles [0, dp_tiles) are computed whole by one workgroup each
    int split_tiles;      // tiles [dp_tiles, tiles) are cut into `splits` reduction slices
    int splits;
    int chunks_per_split; // reduction stages (of BK) per slice
    float *partial;       // FWD / BWD_DATA slice items: raw accumulators, [slice * split_tiles + tile - dp_tiles][BM*BN]
    uint32_t flags;
    uint32_t a_bytes, b_bytes;   // extent of the a / b tensors (vector fetch paths address them as 32-bit buffer offsets)
};

__device__ __forceinline__ float4 ldg4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 zero4() { return make_float4(0.f, 0.f, 0.f, 0.f); }
// Branch-free predicated vector load: masked lanes read the (always valid) base address and get zero.
__device__ __forceinline__ float4 ldg4_if(const float *base, int off, bool ok)
{
    const float4 v = ldg4(base + (ok ? off : 0));
    return make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
}
// Vector fetches go through buffer loads: a lane whose element is padding, beyond a ragged edge or past the end of the
// reduction is given the offset OOB_OFF, which lies outside the buffer, and the hardware returns zero for it.  That
// replaces a pointer select, a 64-bit address computation and four data selects per vector.
constexpr uint32_t OOB_OFF = 0x80000000u;   // tensors on this path are at most 2 GiB
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *ptr, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(ptr), 0, bytes, 0x00020000);
}
__device__ __forceinline__ float4 bload4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0));
}
__device__ __forceinline__ float &f4at(float4 &v, int e) { return reinterpret_cast<float *>(&v)[e]; }
__device__ __forceinline__ float4 gate4(float4 v, float4 m)
{
    return make_float4(m.x > 0.f ? v.x : 0.f, m.y > 0.f ? v.y : 0.f, m.z > 0.f ? v.z : 0.f, m.w > 0.f ? v.w : 0.f);
}

// FAST (FWD / BWD_DATA with both vector paths, channel count a multiple of BK): a stage lies
// inside one filter tap, so the tap is wavefront-uniform (scalar registers) and a row's address is a precomputed row
// offset plus a scalar; no per-thread division or multiplication is left in the main loop.
// The workgroup's whole program; p lives in the kernel's argument segment (igemm_kernel: the argument itself;
// igemm_classes_kernel: one of several parameter sets, picked by blockIdx.y).
template <int MODE, int BM, int BN, int WM, int WN, bool VECA, bool VECB, bool FAST>
__device__ __forceinline__ void igemm_body(const GemmParams p)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BM % 64 == 0 && BN % 64 == 0, "loader granularity");
    constexpr int WTM = BM / WM, WTN = BN / WN;          // wavefront tile
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "MFMA granularity");
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int RPP = NTHREADS / KQ;                   // tile rows covered by one pass of a reduction-contiguous fetch
    constexpr int AV = BM * BK / 1024, BV = BN * BK / 1024;  // 16-byte vectors per thread per stage
    // LDS layouts.  An operand whose reduction index is contiguous in memory (x and w in FWD, dy in BWD_DATA) is kept
    // ROW-MAJOR, [rows][BK] with the 16-byte vectors of a row swizzled (see kq_sw): the fetched vector is stored as it is,
    // and a lane reads 4 consecutive reduction elements of its row with one 16-byte read, which feed 4 MFMAs.  Lanes 0-31 take elements 8g..8g+3 and lanes 32-63 elements 8g+4..8g+7 of reduction group g, so MFMA j of
    // the group multiplies the element pair (8g+j, 8g+4+j): a permutation of the reduction that both operands follow.
    // An operand whose row/column index is contiguous (w in BWD_DATA, dy and x in BWD_WEIGHT) is kept
    // REDUCTION-MAJOR, [BK][rows+4], stored as 16-byte vectors and read as scalars (conflict-free 128-byte rows).
    constexpr bool A_ROWK = MODE != MODE_BWD_WEIGHT, B_ROWK = MODE == MODE_FWD;
    constexpr int LDK = BK;      // unpadded 64-byte rows; the four 16-byte vectors of a row are XOR-swizzled (see kq_sw)
    constexpr int LDA = BM + PAD_V, LDB = BN + PAD_V;
    constexpr int A_FLOATS = A_ROWK ? BM * LDK : BK * LDA, B_FLOATS = B_ROWK ? BN * LDK : BK * LDB;
    // one block: [A stage 0][A stage 1][B stage 0][B stage 1]; the epilogue reuses it to stage CROWS output rows at a time
    constexpr int SMEM_FLOATS = 2 * (A_FLOATS + B_FLOATS);
    static_assert(SMEM_FLOATS >= 32 * BN, "room for 32 staged output rows");
    // output rows staged per epilogue pass: as many as the stage buffers hold (fewer barriers, more stores in flight)
    constexpr int CROWS = BM * BN <= SMEM_FLOATS ? BM : (BM / 2) * BN <= SMEM_FLOATS ? BM / 2 : (BM / 4) * BN <= SMEM_FLOATS && BM / 4 >= 32 ? BM / 4 : 32;
    static_assert(CROWS % 32 == 0 && BM % CROWS == 0 && CROWS * BN <= SMEM_FLOATS, "staged rows");
    __shared__ __attribute__((aligned(16))) float smem[SMEM_FLOATS];
    auto AsBuf = [&](int buf) -> float * { return smem + buf * A_FLOATS; };
    auto BsBuf = [&](int buf) -> float * { return smem + 2 * A_FLOATS + buf * B_FLOATS; };

    // Workgroup -> (reduction slice, tile).  Consecutive workgroup ids land on different XCDs (round robin over
    // 8), so give each XCD one contiguous run of work items: neighbours in M share their input halo and the
    // whole weight panel in that XCD's L2, and for BWD_WEIGHT all column tiles of one reduction slice (which
    // read the same dy rows and the same pixels of x, shifted by a tap) run side by side on one XCD.
    // The whole tiles come first in launch order and the slice items last, each group spread over the XCDs.
    const int grid_a = ((p.dp_tiles + 7) >> 3) << 3;
    const bool sliced = (int)blockIdx.x >= grid_a;
    const int bid = sliced ? blockIdx.x - grid_a : blockIdx.x;
    const int per_xcd = (sliced ? gridDim.x - grid_a : grid_a) >> 3;
    const int L = (bid & 7) * per_xcd + (bid >> 3);
    if (L >= (sliced ? p.split_tiles * p.splits : p.dp_tiles)) return;
    const int split = sliced ? L / p.split_tiles : 0;
    const int tile = sliced ? p.dp_tiles + (L - split * p.split_tiles) : L;
    const int tile_n = tile % p.tilesN, tile_m = tile / p.tilesN;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const ConvGeo &g = p.g;
    // taps the reduction runs over: all of them, or those of the stride class (BWD_DATA)
    const int tapS = MODE == MODE_BWD_DATA ? p.sub.Sc : g.S;
    const int tapRS = MODE == MODE_BWD_DATA ? p.sub.Rc * p.sub.Sc : g.R * g.S;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wave_m = wave / WN, wave_n = wave % WN;

    // reduction stages [ch_beg, ch_end) of this work item
    const int all_chunks = (p.Kd + BK - 1) / BK;
    const int ch_beg = sliced ? split * p.chunks_per_split : 0;
    const int ch_end = sliced ? min(all_chunks, ch_beg + p.chunks_per_split) : all_chunks;
    const int kend = min(p.Kd, ch_end * BK);
    const bool amask = (p.flags & LOAD_AMASK) != 0;

    // ------------------------------------------------------------------ loader state
    // "KC" loaders (reduction contiguous in memory): thread -> vector kq of 4 along the reduction, rows row0 + 64*i.
    const int kq = t % KQ, row0 = t / KQ;
    // Row-major LDS tiles: vector v of row r sits at position v ^ ((r >> 1) & 3) ^ ((r >> 3) & 3).  A group of 8 consecutive
    // lanes over 32 banks, or of 16 over 64, then touches every bank once both when a stage is written (consecutive rows x 4
    // vectors) and when operands are read (consecutive rows, one vector each), without padding the rows.  (The LDS
    // bank-conflict counter reads 4 cycles per 16-byte operand read with this layout and with padded 80-byte rows alike.)
    const int kq_sw = kq ^ ((row0 >> 1) & 3) ^ ((row0 >> 3) & 3);      // rows row0 + 64*i share the swizzle
    // "MC" loaders (row/column index contiguous): thread -> vector c4 along the tile edge, reduction rows kr0 + RP*i.
    constexpr int A_F4 = BM / 4, A_RP = NTHREADS / A_F4;
    constexpr int B_F4 = BN / 4, B_RP = NTHREADS / B_F4;

    // A operand state
    int a_hb[AV], a_wb[AV];          // FWD: p*sh-ph, q*sw-pw      BWD_DATA: h+ph, w+pw
    int a_base[AV];                  // element offset of the image (FWD: n*H*W*C, BWD_DATA: n*Ho*Wo*K)
    int a_row[AV];                   // FAST: element offset of the row's tap-(0,0) source pixel (may be out of the image)
    int b_row[BV];                   // FAST: element offset of this thread's B vector at stage 0
    // B operand state
    int bw_r[4], bw_s[4], bw_c[4];   // BWD_WEIGHT: fixed (r,s,c) of this thread's 4 columns

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
            a_row[i] = m < p.M ? a_base[i] + (a_hb[i] * g.W + a_wb[i]) * g.C + kq * 4 : 0;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) b_row[i] = (n0 + row0 + RPP * i) * p.Kd + kq * 4;
    } else if (MODE == MODE_BWD_DATA) {
        const int HW = p.sub.Hc * p.sub.Wc;
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
            a_row[i] = m < p.M ? a_base[i] + (a_hb[i] * g.Wo + a_wb[i]) * g.K + kq * 4 : 0;   // source pixel of tap (0,0) of the class
        }
#pragma unroll
        for (int i = 0; i < BV; ++i)   // w[k][r][s][c] at k = reduction row of this thread, tap (0,0), its 4 columns
            b_row[i] = (t / (BN / 4) + (NTHREADS / (BN / 4)) * i) * (g.R * g.S * g.C) + n0 + (t % (BN / 4)) * 4;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = n0 + (t % B_F4) * 4 + e;
            const int rs = fdiv(j, p.fd_c);
            bw_c[e] = j - rs * g.C;
            bw_r[e] = fdiv(rs, p.fd_s);         // >= R when j >= Nn: the column predicate below covers it
            bw_s[e] = rs - bw_r[e] * g.S;
        }
    }

    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(p.a, p.a_bytes);
    const __amdgpu_buffer_rsrc_t rsrc_g = make_rsrc(p.amask ? p.amask : p.a, p.a_bytes);
    const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(p.b, p.b_bytes);

    // Stage registers: loaded vectors (vector paths: already zero where masked, see OOB_OFF) and optional ReLU-gate
    // vectors; the gate is applied when the stage is written to LDS, so that nothing waits on a global load before
    // the MFMAs of the current stage.
    float4 ra[AV], rb[BV], rg[AV];
    const bool want_db = MODE == MODE_BWD_WEIGHT && (p.flags & EPI_DBIAS) && tile_n == 0;
    float4 dbacc = zero4();   // bias gradient: running sum of this thread's dy vectors (4 channels, its reduction rows)

    // Reduction offset of stage `ch`.  The reduction index of FWD / BWD_DATA is (tap, channel); when the channel
    // count is a multiple of BK a stage stays inside one tap, and the stages are visited channel-block-major,
    // tap-minor: the R*S taps of one 64-byte channel block re-read the same few image rows back to back, so they
    // hit in L2 instead of going out to the fabric once per tap.  Any visiting order gives the same sum up to
    // rounding; this one is fixed by the shape alone.
    const bool tap_minor = MODE != MODE_BWD_WEIGHT && (FAST || (p.flags & ORDER_TAP_MINOR));
    auto stage_k = [&](int ch) -> int {
        if (!tap_minor) return ch * BK;
        const int cblk = fdiv(ch, p.fd_rs), tap = ch - cblk * tapRS;
        return tap * (MODE == MODE_FWD ? g.C : g.K) + cblk * BK;
    };

    // Issue the global loads of A vector i of stage `ch`.  Stages past the end are fetched too, fully masked.
    auto fetch_a = [&](int ch, int i) {
        if (FAST) {
            // wavefront-uniform: channel block and tap of the stage
            const int cblk = fdiv(ch, p.fd_rs), tap = ch - cblk * tapRS;
            const int ar = fdiv(tap, p.fd_s), as = tap - ar * tapS;
            const bool kok = ch < ch_end;
            int off;
            bool ok;
            if (MODE == MODE_FWD) {
                ok = kok && (unsigned)(a_hb[i] + ar) < (unsigned)g.H && (unsigned)(a_wb[i] + as) < (unsigned)g.W;
                off = a_row[i] + ((ar * g.W + as) * g.C + cblk * BK);
            } else {
                ok = kok && (unsigned)(a_hb[i] - ar) < (unsigned)g.Ho && (unsigned)(a_wb[i] - as) < (unsigned)g.Wo;
                off = a_row[i] + (cblk * BK - (ar * g.Wo + as) * g.K);
            }
            const uint32_t bo = ok ? (uint32_t)off * 4u : OOB_OFF;
            ra[i] = bload4(rsrc_a, bo);
            if (MODE == MODE_BWD_DATA && amask) rg[i] = bload4(rsrc_g, bo);
            return;
        }
        const int kchunk = stage_k(ch);
        if (MODE == MODE_FWD || MODE == MODE_BWD_DATA) {
            const int CC = (MODE == MODE_FWD) ? g.C : g.K;
            if (VECA) {
                const int kk = kchunk + kq * 4;
                const int rs = fdiv(kk, MODE == MODE_FWD ? p.fd_c : p.fd_k), cc = kk - rs * CC;
                const int ar = fdiv(rs, p.fd_s), as = rs - ar * tapS;
                int off;
                bool ok;
                if (MODE == MODE_FWD) {
                    const int h = a_hb[i] + ar, w = a_wb[i] + as;
                    ok = kk < p.Kd && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
                    off = a_base[i] + (h * g.W + w) * g.C + cc;
                } else {
                    const int pp = a_hb[i] - ar, q = a_wb[i] - as;
                    ok = kk < p.Kd && (unsigned)pp < (unsigned)g.Ho && (unsigned)q < (unsigned)g.Wo;
                    off = a_base[i] + (pp * g.Wo + q) * g.K + cc;
                }
                const uint32_t bo = ok ? (uint32_t)off * 4u : OOB_OFF;
                ra[i] = bload4(rsrc_a, bo);
                if (MODE == MODE_BWD_DATA && amask) rg[i] = bload4(rsrc_g, bo);
            } else {
                float4 v = zero4();
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int kk = kchunk + kq * 4 + e;
                    const int c = kk % CC, rs = kk / CC, s = rs % tapS, r = rs / tapS;
                    int off;
                    bool ok;
                    if (MODE == MODE_FWD) {
                        const int h = a_hb[i] + r, w = a_wb[i] + s;
                        ok = kk < p.Kd && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
                        off = a_base[i] + (h * g.W + w) * g.C + c;
                    } else {
                        const int pp = a_hb[i] - r, q = a_wb[i] - s;
                        ok = kk < p.Kd && (unsigned)pp < (unsigned)g.Ho && (unsigned)q < (unsigned)g.Wo;
                        off = a_base[i] + (pp * g.Wo + q) * g.K + c;
                    }
                    if (ok) {
                        float x = p.a[off];
                        if (MODE == MODE_BWD_DATA && amask) x = p.amask[off] > 0.f ? x : 0.f;
                        f4at(v, e) = x;
                    }
                }
                ra[i] = v;
                rg[i] = make_float4(1.f, 1.f, 1.f, 1.f);
            }
        } else {  // BWD_WEIGHT A: dy viewed as [pixel][K], row m = output channel
            const int col = m0 + (t % A_F4) * 4;
            const int pix = kchunk + t / A_F4 + A_RP * i;
            if (VECA) {
                const bool ok = pix < kend && col < p.M;
                const uint32_t bo = ok ? (uint32_t)(pix * g.K + col) * 4u : OOB_OFF;
                ra[i] = bload4(rsrc_a, bo);
                if (amask) rg[i] = bload4(rsrc_g, bo);
            } else {
                float4 v = zero4();
                if (pix < kend) {
                    const int off = pix * g.K + col;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < p.M) {
                            float x = p.a[off + e];
                            if (amask) x = p.amask[off + e] > 0.f ? x : 0.f;
                            f4at(v, e) = x;
                        }
                }
                ra[i] = v;
                rg[i] = make_float4(1.f, 1.f, 1.f, 1.f);
            }
        }
    };

    auto fetch_b = [&](int ch, int i) {
        if (FAST) {
            const int cblk = fdiv(ch, p.fd_rs), tap = ch - cblk * tapRS;
            bool ok = ch < ch_end;
            int off;
            if (MODE == MODE_FWD) {
                ok = ok && n0 + row0 + RPP * i < p.Nn;
                off = b_row[i] + (tap * g.C + cblk * BK);
            } else {
                ok = ok && n0 + (t % B_F4) * 4 < p.Nn;
                const int tr = fdiv(tap, p.fd_s), ts = tap - tr * tapS;
                const int wtap = (p.sub.r0 + tr * g.sh) * g.S + p.sub.s0 + ts * g.sw;    // the filter tap this class tap stands for
                off = b_row[i] + (cblk * BK * (g.R * g.S) + wtap) * g.C;
            }
            rb[i] = bload4(rsrc_b, ok ? (uint32_t)off * 4u : OOB_OFF);
            return;
        }
        const int kchunk = stage_k(ch);
        if (MODE == MODE_FWD) {  // w as [Nn][Kd], reduction contiguous
            const int j = n0 + row0 + RPP * i;
            const int kk = kchunk + kq * 4;
            if (VECB) {
                const bool ok = j < p.Nn && kk < p.Kd;
                rb[i] = bload4(rsrc_b, ok ? (uint32_t)(j * p.Kd + kk) * 4u : OOB_OFF);
            } else {
                float4 v = zero4();
                if (j < p.Nn) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (kk + e < p.Kd) f4at(v, e) = p.b[j * p.Kd + kk + e];
                }
                rb[i] = v;
            }
        } else if (MODE == MODE_BWD_DATA) {  // w[k][r][s][c]: column j = c contiguous, row (r,s,k)
            const int col = n0 + (t % B_F4) * 4;
            const int kk = kchunk + t / B_F4 + B_RP * i;
            const int rs = fdiv(kk, p.fd_k), bk = kk - rs * g.K;
            const int tr = fdiv(rs, p.fd_s), ts = rs - tr * tapS;
            const int br = p.sub.r0 + tr * g.sh, bs = p.sub.s0 + ts * g.sw;
            const int off = ((bk * g.R + br) * g.S + bs) * g.C + col;
            if (VECB) {
                const bool ok = kk < p.Kd && col < p.Nn;
                rb[i] = bload4(rsrc_b, ok ? (uint32_t)off * 4u : OOB_OFF);
            } else {
                float4 v = zero4();
                if (kk < p.Kd) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < p.Nn) f4at(v, e) = p.b[off + e];
                }
                rb[i] = v;
            }
        } else {  // BWD_WEIGHT B: x gathered at (pixel row, column (r,s,c))
            const int col = n0 + (t % B_F4) * 4;
            const int pix = kchunk + t / B_F4 + B_RP * i;
            const int img = fdiv(pix, p.fd_howo), pq = pix - img * (g.Ho * g.Wo);
            const int pp = fdiv(pq, p.fd_wo), q = pq - pp * g.Wo;
            const int hb = pp * g.sh - g.ph, wb = q * g.sw - g.pw;
            const int ib = img * g.H;
            if (VECB) {
                const int h = hb + bw_r[0], w = wb + bw_s[0];
                const bool ok = pix < kend && col < p.Nn && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
                rb[i] = bload4(rsrc_b, ok ? (uint32_t)(((ib + h) * g.W + w) * g.C + bw_c[0]) * 4u : OOB_OFF);
            } else {
                float4 v = zero4();
                if (pix < kend) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int h = hb + bw_r[e], w = wb + bw_s[e];
                        if (col + e < p.Nn && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W)
                            f4at(v, e) = p.b[((ib + h) * g.W + w) * g.C + bw_c[e]];
                    }
                }
                rb[i] = v;
            }
        }
    };

    // Gate and write the fetched stage into LDS buffer `buf`.
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            float4 v = ra[i];
            if (MODE != MODE_FWD && amask) v = gate4(v, rg[i]);
            if (MODE == MODE_BWD_WEIGHT) {
                *reinterpret_cast<float4 *>(&AsBuf(buf)[(t / A_F4 + A_RP * i) * LDA + (t % A_F4) * 4]) = v;
                if (want_db) { dbacc.x += v.x; dbacc.y += v.y; dbacc.z += v.z; dbacc.w += v.w; }
            } else {
                *reinterpret_cast<float4 *>(&AsBuf(buf)[(row0 + RPP * i) * LDK + kq_sw * 4]) = v;
            }
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            if (MODE == MODE_FWD) {
                *reinterpret_cast<float4 *>(&BsBuf(buf)[(row0 + RPP * i) * LDK + kq_sw * 4]) = rb[i];
            } else {
                *reinterpret_cast<float4 *>(&BsBuf(buf)[(t / B_F4 + B_RP * i) * LDB + (t % B_F4) * 4]) = rb[i];
            }
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#pragma unroll
    for (int i = 0; i < AV; ++i) fetch_a(ch_beg, i);
#pragma unroll
    for (int i = 0; i < BV; ++i) fetch_b(ch_beg, i);
    stash(0);
    __syncthreads();

    const int lrow = lane & 31, lk = lane >> 5;
    const int rd_sw = ((lrow >> 1) & 3) ^ ((lrow >> 3) & 3);   // tile rows of a lane differ by multiples of 32
    constexpr int KS = BK / 2;                      // MFMA k-steps per stage
    static_assert(AV + BV <= KS, "one fetch slot per k-step");
    for (int ch = ch_beg; ch < ch_end; ++ch) {
        const int buf = (ch - ch_beg) & 1;
        // Per k-step: (1) LDS reads of the NEXT k-step's operands, (2) this k-step's MFMAs, (3) one slice of the
        // next stage's global fetch (address arithmetic + load issue), which executes in the shadow of the MFMAs.
        // The scheduling barriers pin this order.
        // Operand registers for one reduction group (8 elements = 4 k-steps): row-major operands arrive as one float4
        // per 32-row tile and group, reduction-major operands as one scalar per tile and k-step (double-buffered so that
        // the LDS read of k-step ks+1 is in flight during the MFMAs of k-step ks).
        float4 a4[2][TM], b4[2][TN];
        float a1[2][TM], b1[2][TN];
        auto read_group = [&](int gi, int slot) {
            if (A_ROWK) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a4[slot][i] = *reinterpret_cast<const float4 *>(&AsBuf(buf)[(wave_m * WTM + i * 32 + lrow) * LDK + ((gi * 2 + lk) ^ rd_sw) * 4]);
            }
            if (B_ROWK) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b4[slot][j] = *reinterpret_cast<const float4 *>(&BsBuf(buf)[(wave_n * WTN + j * 32 + lrow) * LDK + ((gi * 2 + lk) ^ rd_sw) * 4]);
            }
        };
        // reduction row that lane half lk multiplies in k-step ks: pairs (8g+j, 8g+4+j) when a row-major operand fixes
        // the order, (2ks, 2ks+1) otherwise
        auto krow = [&](int ks) -> int { return (A_ROWK || B_ROWK) ? (ks >> 2) * 8 + lk * 4 + (ks & 3) : ks * 2 + lk; };
        // A reduction-major operand gives lane lrow the TM (TN) CONSECUTIVE rows TM*lrow + i of its wavefront tile, one per
        // MFMA tile i, so that one 8-byte read serves two tiles; the epilogue maps accumulators back the same way.
        auto read_scalar = [&](int ks, int slot) {
            if (!A_ROWK) {
                const float *src = &AsBuf(buf)[krow(ks) * LDA + wave_m * WTM + TM * lrow];
                if constexpr (TM == 2) {
                    const float2 v = *reinterpret_cast<const float2 *>(src);
                    a1[slot][0] = v.x; a1[slot][1] = v.y;
                } else {
#pragma unroll
                    for (int i = 0; i < TM; ++i) a1[slot][i] = src[i];
                }
            }
            if (!B_ROWK) {
                const float *src = &BsBuf(buf)[krow(ks) * LDB + wave_n * WTN + TN * lrow];
                if constexpr (TN == 2) {
                    const float2 v = *reinterpret_cast<const float2 *>(src);
                    b1[slot][0] = v.x; b1[slot][1] = v.y;
                } else {
#pragma unroll
                    for (int j = 0; j < TN; ++j) b1[slot][j] = src[j];
                }
            }
        };
        read_group(0, 0);
        read_scalar(0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1, gi = ks >> 2, e = ks & 3, gs = gi & 1;
            if (e == 0 && (gi + 1) * 4 < KS) read_group(gi + 1, gs ^ 1);
            if (ks + 1 < KS) read_scalar(ks + 1, nxt);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const float av = A_ROWK ? f4at(a4[gs][i], e) : a1[cur][i];
                    const float bv = B_ROWK ? f4at(b4[gs][j], e) : b1[cur][j];
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                }
            if (ks < AV) fetch_a(ch + 1, ks);
            else if (ks < AV + BV) fetch_b(ch + 1, ks - AV);
            __builtin_amdgcn_sched_barrier(0);
        }
        stash(buf ^ 1);
        __syncthreads();
    }

    if (MODE == MODE_BWD_WEIGHT && want_db) {
        // The A_RP threads t, t + A_F4, ... hold partial sums of the same 4 channels: add them in thread order
        // through LDS (the last stage barrier has passed, the tiles are free).
        float *red = smem;
        *reinterpret_cast<float4 *>(&red[(t / A_F4) * LDA + (t % A_F4) * 4]) = dbacc;
        __syncthreads();
        if (t < BM && m0 + t < p.M) {
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < A_RP; ++r) s += red[r * LDA + t];
            p.dbias[(size_t)split * p.dbias_stride + m0 + t] = s;
        }
    }

    // ------------------------------------------------------------------ epilogue
    // Accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 tile.
    // With a reduction-major operand, MFMA row (column) index x of tile i stands for row (column) TM*x + i (TN*x + i) of the
    // wavefront tile, see read_scalar.
    auto wrow = [&](int i, int x) -> int { return A_ROWK ? i * 32 + x : TM * x + i; };
    auto wcol = [&](int j, int x) -> int { return B_ROWK ? j * 32 + x : TN * x + j; };
    const size_t split_off = (MODE == MODE_BWD_WEIGHT && !(p.flags & EPI_SGD)) ? (size_t)split * p.M * p.Nn : 0;
    if (MODE != MODE_BWD_WEIGHT && sliced) {
        // raw accumulators of this slice, tile-local [BM][BN]; the fix-up kernel adds the slices and applies the epilogue
        float *dst = p.partial + (size_t)L * (BM * BN);
        if constexpr (!B_ROWK && TN == 2) {
            // a lane's two column tiles are neighbouring columns: one 8-byte store, whole rows per instruction
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    *reinterpret_cast<float2 *>(&dst[(wave_m * WTM + wrow(i, 8 * (r >> 2) + 4 * lk + (r & 3))) * BN + wave_n * WTN + 2 * lrow]) =
                        make_float2(acc[i][0][r], acc[i][1][r]);
            return;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    dst[(wave_m * WTM + wrow(i, 8 * (r >> 2) + 4 * lk + (r & 3))) * BN + wave_n * WTN + wcol(j, lrow)] = acc[i][j][r];
        return;
    }
    // element offset of (row, col) in the output: dense rows, or the scattered pixels of a stride class
    auto out_index = [&](int row, int col) -> size_t {
        if (MODE == MODE_BWD_DATA && (p.flags & OUT_STRIDED)) {
            const int n = fdiv(row, p.fd_hcwc), hw = row - n * (p.sub.Hc * p.sub.Wc);
            const int ci = fdiv(hw, p.fd_wc), cj = hw - ci * p.sub.Wc;
            return ((size_t)(n * g.H + p.sub.h0 + ci * g.sh) * g.W + p.sub.w0 + cj * g.sw) * g.C + col;
        }
        return (size_t)row * p.Nn + col;
    };
    if (MODE != MODE_BWD_WEIGHT && (p.Nn & 3) == 0) {
        // Output rows are whole 16-byte vectors: stage the tile in LDS CROWS rows at a time and let every thread move float4s of
        // full row segments (bias / ReLU, or accumulate / mask, on the vectors).  One scalar store per accumulator register
        // (64 per thread, plus as many mask and accumulate loads in BWD_DATA) cost 9 % of a 64-channel 3x3 layer and a quarter
        // of a 1x1 layer with 64 input channels.
        constexpr int CH4 = BN / 4, ROWS_PASS = NTHREADS / CH4;
        float *Cs = smem;
        // EPI_STATS: a thread meets the same 4 columns in every pass, so it keeps their sums about the tile's first row
        const bool stats = MODE == MODE_FWD && (p.flags & EPI_STATS);
        float4 sk = zero4(), sa = zero4(), sb = zero4();
        if (stats && blockIdx.x == 0 && t == 0) {
            StatsHeader h{STATS_MAGIC, p.tilesM, p.tilesN, p.dp_tiles, BM, BN, p.M, p.Nn};
            *reinterpret_cast<StatsHeader *>(p.stats) = h;
        }
        // a thread meets the same 4 columns in every pass: their bias is loaded once, before any store
        float4 bias4 = zero4();
        if (MODE == MODE_FWD && (p.flags & EPI_BIAS) && n0 + (t % CH4) * 4 < p.Nn) bias4 = ldg4(p.bias + n0 + (t % CH4) * 4);
#pragma unroll
        for (int chunk = 0; chunk < BM / CROWS; ++chunk) {
            __syncthreads();       // the stage buffers (first chunk) or the previous chunk have been read by everyone
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int tile_row = wave_m * WTM + i * 32;          // rows of MFMA tile i are 32 consecutive tile rows here
                if (tile_row / CROWS != chunk) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        Cs[(tile_row % CROWS + 8 * (r >> 2) + 4 * lk + (r & 3)) * BN + wave_n * WTN + wcol(j, lrow)] = acc[i][j][r];
            }
            __syncthreads();
            // What the epilogue reads from global memory (residual, previous gradient, mask) is folded into the staged tile
            // first, every thread on the elements it will store, and the stores follow in a loop of their own.  Loads and stores
            // share one counter and return out of order with respect to each other, so a load that is waited for while stores
            // are in flight waits for every one of those stores: with load and store in the same pass, each pass cost a full
            // round trip to memory (32 per 128x128 tile).
            constexpr int PASSES = CROWS / ROWS_PASS;
            const int c4 = (t % CH4) * 4, col = n0 + c4;
            const bool want_a = MODE == MODE_FWD ? (p.flags & EPI_RESIDUAL) != 0 : (p.flags & EPI_ACCUM) != 0;
            const bool want_m = MODE == MODE_BWD_DATA && (p.flags & EPI_XMASK);
            // (one sweep per operand, its loads issued together: 4 * PASSES registers, which the staged accumulators left free)
            auto fold = [&](const float *src, auto op) {
                float4 g4[PASSES];
#pragma unroll
                for (int pass = 0; pass < PASSES; ++pass) {
                    const int row = m0 + chunk * CROWS + pass * ROWS_PASS + t / CH4;
                    g4[pass] = (row < p.M && col < p.Nn) ? ldg4(src + out_index(row, col)) : zero4();
                }
#pragma unroll
                for (int pass = 0; pass < PASSES; ++pass) {
                    const int row_l = pass * ROWS_PASS + t / CH4;
                    float4 *c = reinterpret_cast<float4 *>(&Cs[row_l * BN + c4]);
                    *c = op(*c, g4[pass]);      // (rows past the end: staged, never stored)
                }
            };
            if (want_a) {
                if (MODE == MODE_FWD)        // (bias before the residual)
                    fold(p.res, [&](float4 v, float4 a) { return make_float4(v.x + bias4.x + a.x, v.y + bias4.y + a.y, v.z + bias4.z + a.z, v.w + bias4.w + a.w); });
                else
                    fold(p.out, [&](float4 v, float4 a) { return make_float4(v.x + a.x, v.y + a.y, v.z + a.z, v.w + a.w); });
            }
            if (want_m) fold(p.xmask, [&](float4 v, float4 m) { return gate4(v, m); });
            const float4 bias_now = (MODE == MODE_FWD && !want_a) ? bias4 : zero4();
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) {
                const int row_l = pass * ROWS_PASS + t / CH4;
                const int row = m0 + chunk * CROWS + row_l;
                if (row >= p.M || col >= p.Nn) continue;
                float4 v = *reinterpret_cast<const float4 *>(&Cs[row_l * BN + c4]);
                if (MODE == MODE_FWD) {
                    v.x += bias_now.x; v.y += bias_now.y; v.z += bias_now.z; v.w += bias_now.w;
                    if (stats) {       // (never together with a residual: conv_fwd_any)
                        if (chunk == 0 && pass == 0) {       // the tile's first row (always inside the matrix), with the bias
                            sk = *reinterpret_cast<const float4 *>(&Cs[c4]);
                            sk.x += bias4.x; sk.y += bias4.y; sk.z += bias4.z; sk.w += bias4.w;
                        }
                        const float4 d = make_float4(v.x - sk.x, v.y - sk.y, v.z - sk.z, v.w - sk.w);
                        sa.x += d.x; sa.y += d.y; sa.z += d.z; sa.w += d.w;
                        sb.x = fmaf(d.x, d.x, sb.x); sb.y = fmaf(d.y, d.y, sb.y); sb.z = fmaf(d.z, d.z, sb.z); sb.w = fmaf(d.w, d.w, sb.w);
                    }
                    if (p.flags & EPI_RELU) v = make_float4(fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f));
                }
                *reinterpret_cast<float4 *>(p.out + out_index(row, col)) = v;
            }
        }
        if (stats) {
            // the ROWS_PASS threads of a column group, in row order; layout [ROWS_PASS][2][BN] then the shifts [BN]
            static_assert((2 * ROWS_PASS + 1) * BN <= SMEM_FLOATS, "room for the column sums");
            __syncthreads();
            const int rp = t / CH4, c4 = (t % CH4) * 4;
            *reinterpret_cast<float4 *>(&Cs[(2 * rp) * BN + c4]) = sa;
            *reinterpret_cast<float4 *>(&Cs[(2 * rp + 1) * BN + c4]) = sb;
            if (rp == 0) *reinterpret_cast<float4 *>(&Cs[2 * ROWS_PASS * BN + c4]) = sk;
            __syncthreads();
            if (t < BN && n0 + t < p.Nn) {
                float a = 0.f, b = 0.f;
#pragma unroll
                for (int r = 0; r < ROWS_PASS; ++r) {
                    a += Cs[(2 * r) * BN + t];
                    b += Cs[(2 * r + 1) * BN + t];
                }
                float *e = p.stats + STATS_HEADER_FLOATS + (size_t)tile * (3 * BN);
                e[t] = a;
                e[BN + t] = b;
                e[2 * BN + t] = Cs[2 * ROWS_PASS * BN + t];
            }
        }
        return;
    }
    if constexpr (MODE == MODE_BWD_WEIGHT && TN == 2) {
        // A lane's two column tiles are the neighbouring columns 2*lrow, 2*lrow + 1: with an even row length they leave as one
        // 8-byte store (whole 256-byte row segments per instruction instead of every other float twice).
        const int col = n0 + wave_n * WTN + 2 * lrow;
        if ((p.Nn & 1) == 0) {
            if (col >= p.Nn) return;
            if (p.flags & EPI_SGD) {
                // fused momentum update: the parameters and velocities of SG rows are loaded before the first of their stores
                // (a load waited for with stores in flight waits for those stores as well: row by row, every row cost a round
                // trip to memory, 32 per tile)
                constexpr int SG = 8;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
#pragma unroll
                    for (int r0 = 0; r0 < 16; r0 += SG) {
                        float2 w[SG], vel[SG];
#pragma unroll
                        for (int q = 0; q < SG; ++q) {
                            const int r = r0 + q, row = m0 + wave_m * WTM + wrow(i, 8 * (r >> 2) + 4 * lk + (r & 3));
                            const size_t o = (size_t)min(row, p.M - 1) * p.Nn + col;
                            w[q] = *reinterpret_cast<const float2 *>(p.sgd_w + o);
                            vel[q] = *reinterpret_cast<const float2 *>(p.sgd_v + o);
                        }
#pragma unroll
                        for (int q = 0; q < SG; ++q) {
                            const int r = r0 + q, row = m0 + wave_m * WTM + wrow(i, 8 * (r >> 2) + 4 * lk + (r & 3));
                            if (row >= p.M) continue;
                            const size_t o = (size_t)row * p.Nn + col;
                            const float2 v = make_float2(acc[i][0][r], acc[i][1][r]);
                            float2 ve = vel[q];
                            ve.x = p.mom * ve.x + (v.x + p.wd * w[q].x);
                            ve.y = p.mom * ve.y + (v.y + p.wd * w[q].y);
                            *reinterpret_cast<float2 *>(p.sgd_v + o) = ve;
                            *reinterpret_cast<float2 *>(p.sgd_w + o) = make_float2(w[q].x - p.lr * ve.x, w[q].y - p.lr * ve.y);
                        }
                    }
                }
                return;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + wave_m * WTM + wrow(i, 8 * (r >> 2) + 4 * lk + (r & 3));
                    if (row >= p.M) continue;
                    const size_t o = (size_t)row * p.Nn + col;
                    *reinterpret_cast<float2 *>(p.out + split_off + o) = make_float2(acc[i][0][r], acc[i][1][r]);
                }
            }
            return;
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wave_n * WTN + wcol(j, lrow);
        if (col >= p.Nn) continue;
        float bias = 0.f;
        if (MODE == MODE_FWD && (p.flags & EPI_BIAS)) bias = p.bias[col];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wave_m * WTM + wrow(i, 8 * (r >> 2) + 4 * lk + (r & 3));
                if (row >= p.M) continue;
                const size_t o = out_index(row, col);
                float v = acc[i][j][r];
                if (MODE == MODE_FWD) {
                    v += bias;
                    if (p.flags & EPI_RESIDUAL) v += p.res[o];
                    if (p.flags & EPI_RELU) v = fmaxf(v, 0.f);
                    p.out[o] = v;
                } else if (MODE == MODE_BWD_DATA) {
                    if (p.flags & EPI_ACCUM) v += p.out[o];
                    if (p.flags & EPI_XMASK) v = p.xmask[o] > 0.f ? v : 0.f;
                    p.out[o] = v;
                } else {
                    if (p.flags & EPI_SGD) {
                        const float w = p.sgd_w[o];
                        const float gg = v + p.wd * w;
                        const float vel = p.mom * p.sgd_v[o] + gg;
                        p.sgd_v[o] = vel;
                        p.sgd_w[o] = w - p.lr * vel;
                    } else {
                        p.out[split_off + o] = v;
                    }
                }
            }
        }
    }
}

template <int MODE, int BM, int BN, int WM, int WN, bool VECA, bool VECB, bool FAST = false>
// register cap: 128 (four workgroups per CU) for the vector-fetch variants of the 128-row tiles; the scalar-gather variants
// (3-channel first layers) need more and spill under it
__global__ __launch_bounds__(NTHREADS, (BM >= 256 ? 3 : (VECA && VECB) ? 4 : 2)) void igemm_kernel(const GemmParams p)
{
    igemm_body<MODE, BM, BN, WM, WN, VECA, VECB, FAST>(p);
}

// Several independent GEMMs of one shape family in one launch: the stride classes of a strided layer's data gradient (each
// class gathers its own taps into its own, disjoint, pixels of dx).  One class by itself is a few dozen to a few hundred
// tiles; launched one after the other they left most CUs idle.  blockIdx.y = class, blockIdx.x = its work items (workgroups
// past a class's last tile leave at once).
constexpr int MAX_CLASSES = 4;
struct GemmClasses { GemmParams q[MAX_CLASSES]; };

template <int BM, int BN, int WM, int WN, bool VECA, bool VECB, bool FAST>
__global__ __launch_bounds__(NTHREADS, (BM >= 256 ? 3 : (VECA && VECB) ? 4 : 2)) void igemm_classes_kernel(const GemmClasses P)
{
    igemm_body<MODE_BWD_DATA, BM, BN, WM, WN, VECA, VECB, FAST>(P.q[blockIdx.y]);
}

}  // namespace stanza
