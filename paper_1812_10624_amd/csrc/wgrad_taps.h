// Filter gradient of a 3x3, stride-1, pad-1 convolution with all nine taps fused (paper Sec. 3.2: the CONV worker's
// backpropagation; part of T_c of Sec. 4.2.1):
//   dW[k][r][s][c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p-1+r, q-1+s, c]
// The implicit-GEMM engine treats (r,s,c) as the GEMM's column index, so every column tile (one or two taps) streams the
// whole of dy and its own shifted view of x again: nine times the operand traffic when the tiles of a slice do not keep
// step in L2.  Here a workgroup owns 64 output channels x 64 input channels and ALL NINE taps (9 x 64 x 64 accumulators,
// 144 registers per lane), so that a stretch of dy and the rows of x around it are staged in LDS once and multiplied
// nine times, each tap reading the same LDS rows at a shifted pixel.
//
// Stage = RP output rows x SW output pixels of one image (RP = 1 and SW <= 30 for wide images; RP > 1 for images of 14
// pixels and fewer).  dy of a stage is laid out as RP rows of XW = SW + 2 (rounded up to even) pixel slots, the extra
// slots of a row holding zeros: a pixel's slot j then finds its tap (r,s) operand at slot j + r*XW + s of the x window,
// which has the same row length, and an MFMA k-step (two consecutive slots) never straddles a row.
// x lives in a ring of NR = 2*RP + 4 rows of XW pixels: a stage reads RP + 2 consecutive ring rows (image rows p0-1 ..
// p0+RP, columns q0-1 .. q0+XW-2, zeros outside the image); going down a column strip, the next stage reuses the last
// two and fetches RP new rows, so x is read once (plus the two-column overlap of neighbouring strips).
// A pixel row of 64 channels is stored with its two 32-channel halves swapped when the pixel's slot is odd: the two
// half-wavefronts of an MFMA operand read (two consecutive pixels, 32 channels each) then fall on different banks.
#pragma once
#include "igemm.h"

namespace stanza {

#ifndef TAPS_NOFENCE
#define TAPS_FENCE __builtin_amdgcn_sched_barrier(0)
#else
#define TAPS_FENCE
#endif

constexpr int TAPS_XSLOTS = 186;   // pixel slots of the x ring (NR * XW <= 186: ring + dy stages stay under 64 KB, two workgroups per CU)
constexpr int TAPS_J = 32;         // pixel slots of one dy stage (RP * XW <= 32)
constexpr int TAPS_T = 64;         // channels per tile, both ways

struct TapsParams {
    const float *dy, *amask, *x;   // amask: forward output gating dy ([amask > 0]) in the GATED kernel
    float *out;             // dW, or the slices' partial sums [slice][K][3][3][C]
    float *dbias;           // db, or the slices' partial sums [slice][K]; nullptr when not wanted
    int N, H, W, C, K;
    int SW, XW, RP, NR, KS; // strip width, slots per row, rows per stage, ring rows, MFMA k-steps per stage
    int strips, rowblocks;  // column strips and row blocks per image
    int tiles_c, tiles;     // tiles = ceil(K/64) * tiles_c
    int slices, stages_per_item, total_stages;
    FastDiv fd_xw, fd_rowblocks, fd_strips, fd_tiles, fd_tiles_c;
    uint32_t dy_bytes, x_bytes;
};

// XWC, RPC: the stage geometry as compile-time constants (the k-steps of a stage are then unrolled, every LDS operand read is
// a per-stage base register plus an immediate offset, and the waits between the reads of k-step ks+1 and the MFMAs of
// k-step ks are exact); 0, 0: any geometry, taken from p at run time.
template <bool GATED, int XWC, int RPC>
__global__ __launch_bounds__(256, 2) void wgrad_taps_kernel(const TapsParams p)
{
    // two zero pixels behind the ring: the last k-step of a row reads up to two slots past its end (times dy = 0)
    __shared__ __attribute__((aligned(16))) float xL[(TAPS_XSLOTS + 2) * TAPS_T];
    __shared__ __attribute__((aligned(16))) float dyL[2 * TAPS_J * TAPS_T];

    // Work item -> (pixel slice, channel tile).  Every XCD gets one contiguous run of items, tile fastest: the tiles of a
    // slice, which read the same dy rows and the same x rows (other channels), run side by side on one XCD's L2.
    const int per_xcd = gridDim.x >> 3;
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= p.tiles * p.slices) return;
    const int slice = fdiv(L, p.fd_tiles), tile = L - slice * p.tiles;
    const int tk = fdiv(tile, p.fd_tiles_c), tc = tile - tk * p.tiles_c;
    const int k0 = tk * TAPS_T, c0 = tc * TAPS_T;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, lrow = lane & 31, lk = lane >> 5;
    const int wk = wave >> 1, wc = wave & 1;       // this wavefront's 32 output channels x 32 input channels
    const int g4 = (t & 15) * 4;                   // loader: 4 channels of the 64-wide tile, pixel slots (t >> 4) + 16*i
    const int XW = XWC > 0 ? XWC : p.XW, RP = XWC > 0 ? RPC : p.RP, NR = 2 * RP + 4, W = p.W, H = p.H;

    // zero the ring once: slots that no load ever writes (behind a short last stage) must hold finite values
    for (int i = t; i < (TAPS_XSLOTS + 2) * TAPS_T / 4; i += 256) reinterpret_cast<float4 *>(xL)[i] = zero4();

    // ---- loader constants of this thread
    // dy: slot j = (t >> 4) + 16*i  ->  (row jr, column jc) of the stage
    int dy_off[2], dy_rc[2];
    // x, new rows of the next stage: pixel f = (t >> 4) + 16*i of RP x XW;  x, top two rows (new column strip): f of 2 x XW
    int xn_off[2], xn_rc[2], xt_off[4], xt_rc[4];
    const bool kch = k0 + g4 < p.K, cch = c0 + g4 < p.C;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int f = (t >> 4) + 16 * i;
        const int row = fdiv(f, p.fd_xw), col = f - row * XW;
        if (i < 2) {
            dy_rc[i] = (kch && row < RP && col < p.SW) ? (row | (col << 8)) : -1;
            dy_off[i] = (row * W + col) * p.K + k0 + g4;
            xn_rc[i] = (cch && row < RP) ? (row | (col << 8)) : -1;
            xn_off[i] = ((1 + row) * W + col - 1) * p.C + c0 + g4;
        }
        xt_rc[i] = (cch && row < 2) ? (row | (col << 8)) : -1;
        xt_off[i] = ((row - 1) * W + col - 1) * p.C + c0 + g4;
    }
    const __amdgpu_buffer_rsrc_t rs_dy = make_rsrc(p.dy, p.dy_bytes), rs_m = make_rsrc(GATED ? p.amask : p.dy, p.dy_bytes);
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.x, p.x_bytes);

    // ---- stages of this item: ids [sid, send), (image, strip, row block) with the row block fastest
    int sid = slice * p.stages_per_item;
    const int send = min(p.total_stages, sid + p.stages_per_item);
    int rb, strip, n;
    {
        const int q = fdiv(sid, p.fd_rowblocks);
        rb = sid - q * p.rowblocks;
        n = fdiv(q, p.fd_strips);
        strip = q - n * p.strips;
    }

    float4 r_dy[2], r_m[2], r_xn[2], r_xt[4];
    // issue the loads of the stage at (n, rb, strip); top: also the two rows above its first new row
    auto fetch = [&](int n_, int rb_, int strip_, bool live, bool top) {
        const int p0 = rb_ * RP, q0 = strip_ * p.SW;
        const int pix0 = (n_ * H + p0) * W + q0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = dy_rc[i] & 255, col = dy_rc[i] >> 8;
            const bool ok = live && dy_rc[i] >= 0 && p0 + row < H && q0 + col < W;
            const uint32_t bo = ok ? (uint32_t)(pix0 * p.K + dy_off[i]) * 4u : OOB_OFF;
            r_dy[i] = bload4(rs_dy, bo);
            if (GATED) r_m[i] = bload4(rs_m, bo);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = xn_rc[i] & 255, col = xn_rc[i] >> 8;
            const bool ok = live && xn_rc[i] >= 0 && p0 + 1 + row < H && (unsigned)(q0 - 1 + col) < (unsigned)W;
            r_xn[i] = bload4(rs_x, ok ? (uint32_t)(pix0 * p.C + xn_off[i]) * 4u : OOB_OFF);
        }
        if (top) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = xt_rc[i] & 255, col = xt_rc[i] >> 8;
                const bool ok = live && xt_rc[i] >= 0 && (unsigned)(p0 - 1 + row) < (unsigned)H && (unsigned)(q0 - 1 + col) < (unsigned)W;
                r_xt[i] = bload4(rs_x, ok ? (uint32_t)(pix0 * p.C + xt_off[i]) * 4u : OOB_OFF);
            }
        }
    };
    const bool want_db = p.dbias != nullptr && tc == 0;
    float4 dbacc = zero4();
    // write the fetched stage into dy buffer `buf` and the ring rows of the window whose first row sits in ring slot `head`
    auto stash = [&](int buf, int head, bool top) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float4 v = r_dy[i];
            if (GATED) v = gate4(v, r_m[i]);
            const int j = (t >> 4) + 16 * i;
            *reinterpret_cast<float4 *>(&dyL[(buf * TAPS_J + j) * TAPS_T + (g4 ^ ((j & 1) << 5))]) = v;
            if (want_db) { dbacc.x += v.x; dbacc.y += v.y; dbacc.z += v.z; dbacc.w += v.w; }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (xn_rc[i] < 0) continue;
            const int row = xn_rc[i] & 255, col = xn_rc[i] >> 8;
            int slot = head + 2 + row;
            slot -= slot >= NR ? NR : 0;
            *reinterpret_cast<float4 *>(&xL[(slot * XW + col) * TAPS_T + (g4 ^ ((col & 1) << 5))]) = r_xn[i];
        }
        if (top) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (xt_rc[i] < 0) continue;
                const int row = xt_rc[i] & 255, col = xt_rc[i] >> 8;
                int slot = head + row;
                slot -= slot >= NR ? NR : 0;
                *reinterpret_cast<float4 *>(&xL[(slot * XW + col) * TAPS_T + (g4 ^ ((col & 1) << 5))]) = r_xt[i];
            }
        }
    };

    f32x16 acc[9];
#pragma unroll
    for (int i = 0; i < 9; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    int head = 0, buf = 0;
    fetch(n, rb, strip, sid < send, true);
    __syncthreads();            // the zero fill is complete
    stash(0, 0, true);
    __syncthreads();

    // operand addresses inside a pixel row: channel of this lane, halves swapped for odd pixels
    const int a_lane = lk * TAPS_T + ((wk * 32 + lrow) ^ (lk << 5));
    const int b_even = lk * TAPS_T + ((wc * 32 + lrow) ^ (lk << 5));          // taps s = 0, 2: pixel parity = lk
    const int b_odd = lk * TAPS_T + ((wc * 32 + lrow) ^ ((lk ^ 1) << 5));     // tap s = 1
    const int KS = p.KS;

    for (; sid < send; ++sid) {
        // next stage and how its window relates to this one
        int rb2 = rb + 1, strip2 = strip, n2 = n;
        if (rb2 == p.rowblocks) {
            rb2 = 0;
            if (++strip2 == p.strips) { strip2 = 0; ++n2; }
        }
        const bool live2 = sid + 1 < send, top2 = rb2 == 0;
        fetch(n2, rb2, strip2, live2, top2);

        const float *dyB = dyL + buf * (TAPS_J * TAPS_T);
        float a[2], b[2][9];
        auto mfma9 = [&](int set) {
#pragma unroll
            for (int i = 0; i < 9; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[set], b[set][i], acc[i], 0, 0, 0);
        };
        if constexpr (XWC > 0) {
            constexpr int KSC = RPC * XWC / 2 - 1;
            // ring rows of the window: one base per row and pixel parity, everything else is an immediate offset
            const float *row_even[RPC + 2], *row_odd[RPC + 2];
#pragma unroll
            for (int wr = 0; wr < RPC + 2; ++wr) {
                int slot = head + wr;
                slot -= slot >= NR ? NR : 0;
                row_even[wr] = xL + slot * (XWC * TAPS_T) + b_even;
                row_odd[wr] = xL + slot * (XWC * TAPS_T) + TAPS_T + b_odd;
            }
            const float *dyA = dyB + a_lane;
            auto read = [&](int ks, int set) {      // ks is a constant after unrolling
                const int jr = (2 * ks) / XWC, jcb = 2 * ks - jr * XWC;
                a[set] = dyA[ks * (2 * TAPS_T)];
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    b[set][r * 3 + 0] = row_even[jr + r][jcb * TAPS_T];
                    b[set][r * 3 + 1] = row_odd[jr + r][jcb * TAPS_T];
                    b[set][r * 3 + 2] = row_even[jr + r][(jcb + 2) * TAPS_T];
                }
            };
            read(0, 0);
#pragma unroll
            for (int ks = 0; ks < KSC; ++ks) {
                if (ks + 1 < KSC) read(ks + 1, (ks + 1) & 1);
                TAPS_FENCE;
                mfma9(ks & 1);
                TAPS_FENCE;
            }
        } else {
            auto read = [&](int ks, int jr, int jcb, int set) {
                a[set] = dyB[ks * (2 * TAPS_T) + a_lane];
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    int slot = head + jr + r;
                    slot -= slot >= NR ? NR : 0;
                    const float *row = xL + (slot * XW + jcb) * TAPS_T;
                    b[set][r * 3 + 0] = row[b_even];
                    b[set][r * 3 + 1] = row[TAPS_T + b_odd];
                    b[set][r * 3 + 2] = row[2 * TAPS_T + b_even];
                }
            };
            int jr = 0, jcb = 0;
            auto advance = [&]() {
                jcb += 2;
                if (jcb >= XW) { jcb -= XW; ++jr; }
            };
            read(0, 0, 0, 0);
            for (int ks = 0; ks < KS; ks += 2) {
                advance();
                if (ks + 1 < KS) read(ks + 1, jr, jcb, 1);
                TAPS_FENCE;
                mfma9(0);
                TAPS_FENCE;
                if (ks + 1 < KS) {
                    advance();
                    if (ks + 2 < KS) read(ks + 2, jr, jcb, 0);
                    TAPS_FENCE;
                    mfma9(1);
                    TAPS_FENCE;
                }
            }
        }

        const int head2 = top2 ? head + RP + 2 : head + RP;
        head = head2 - (head2 >= NR ? NR : 0);
        buf ^= 1;
        if (live2) stash(buf, head, top2);
        __syncthreads();
        rb = rb2; strip = strip2; n = n2;
    }

    // ---- bias gradient: threads t, t + 16, ... hold partial sums of the same 4 channels; add them in thread order
    if (want_db) {
        float *red = dyL;
        *reinterpret_cast<float4 *>(&red[(t >> 4) * TAPS_T + g4]) = dbacc;
        __syncthreads();
        if (t < TAPS_T && k0 + t < p.K) {
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) s += red[r * TAPS_T + t];
            p.dbias[(size_t)slice * p.K + k0 + t] = s;
        }
    }

    // ---- epilogue: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 tile
    const int c = c0 + wc * 32 + lrow;
    if (c >= p.C) return;
    float *dst = p.out + (size_t)slice * p.K * 9 * p.C;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int k = k0 + wk * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        if (k >= p.K) continue;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) dst[((size_t)k * 9 + tap) * p.C + c] = acc[tap][r];
    }
}


// ---------------------------------------------------------------------------------------------------------------------
// The same filter gradient for an image layer: C = 4 input channels (3 padded to 4), 3x3, stride 1, pad 1.  With so few
// channels the layer is bound by the one pass over dy (its arithmetic is 2*27 flops per dy element), and the generic tiles
// spend their time on loader arithmetic for operands that are mostly padding.  Here the GEMM's column index is (tap, c):
// 36 columns, three 16-wide MFMA tiles (v_mfma_f32_16x16x4_f32; the twelve columns beyond 36 read zeros).  A workgroup owns
// 64 output channels (16 per wavefront) and walks over row segments of up to 56 output pixels: dy of the segment (56 x 64
// floats) and the three image rows around it (58 pixels x 4 channels each) are staged in LDS, double-buffered; a k-step is
// 4 pixels: one dy read, three window reads (each lane at its own tap's shift), three MFMAs, all at immediate offsets.
constexpr int C4_SW = 56;                 // output pixels per stage
constexpr int C4_XW = C4_SW + 2;          // window pixels per row
constexpr int C4_KS = C4_SW / 4;          // k-steps per stage
constexpr int C4_WIN = 3 * C4_XW * 4;     // floats of one window
constexpr int C4_ZERO = C4_KS * 16 + 16;  // zero floats behind it (columns 36..47)

struct TapsC4Params {
    const float *dy, *amask, *x;   // x: [N,H,W,4]
    float *out, *dbias;            // dW [K][3][3][4] or the slices' partial sums; db or its partial sums (nullptr: not wanted)
    int N, H, W, K;
    int SW, strips;                // strip width (<= 56) and strips per row
    int tiles, slices, stages_per_item, total_stages;
    FastDiv fd_h, fd_strips, fd_tiles;
    uint32_t dy_bytes, x_bytes;
};

template <bool GATED>
__global__ __launch_bounds__(256, 4) void wgrad_taps_c4_kernel(const TapsC4Params p)
{
    __shared__ __attribute__((aligned(16))) float dyL[2 * C4_SW * TAPS_T];
    __shared__ __attribute__((aligned(16))) float xW[2 * (C4_WIN + C4_ZERO)];

    const int per_xcd = gridDim.x >> 3;
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= p.tiles * p.slices) return;
    const int slice = fdiv(L, p.fd_tiles), tk = L - slice * p.tiles;
    const int k0 = tk * TAPS_T;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, l16 = lane & 15, lq = lane >> 4;
    const int g4 = (t & 15) * 4;
    const int W = p.W, H = p.H, K = p.K;

    for (int i = t; i < 2 * (C4_WIN + C4_ZERO); i += 256) xW[i] = 0.f;     // the zero columns stay zero; the windows are rewritten

    // stages [sid, send): (image, strip, row) with the row fastest
    int sid = slice * p.stages_per_item;
    const int send = min(p.total_stages, sid + p.stages_per_item);
    int row, strip, n;
    {
        const int q = fdiv(sid, p.fd_h);
        row = sid - q * H;
        n = fdiv(q, p.fd_strips);
        strip = q - n * p.strips;
    }
    const __amdgpu_buffer_rsrc_t rs_dy = make_rsrc(p.dy, p.dy_bytes), rs_m = make_rsrc(GATED ? p.amask : p.dy, p.dy_bytes);
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.x, p.x_bytes);
    const bool kch = k0 + g4 < K;
    const int wrow = t / C4_XW, wcol = t - wrow * C4_XW;      // window loader: thread -> (row 0..2, pixel), t < 3 * XW

    float4 r_dy[4], r_m[4], r_x;
    auto fetch = [&](int n_, int row_, int strip_, bool live) {
        const int q0 = strip_ * p.SW;
        const int pix0 = (n_ * H + row_) * W + q0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int px = (t >> 4) + 16 * i;
            const bool ok = live && kch && px < p.SW && q0 + px < W;
            const uint32_t bo = ok ? (uint32_t)((pix0 + px) * K + k0 + g4) * 4u : OOB_OFF;
            r_dy[i] = bload4(rs_dy, bo);
            if (GATED) r_m[i] = bload4(rs_m, bo);
        }
        const int h = row_ - 1 + wrow, w = q0 - 1 + wcol;
        const bool okx = live && t < 3 * C4_XW && (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
        r_x = bload4(rs_x, okx ? (uint32_t)(((n_ * H + h) * W + w) * 4) * 4u : OOB_OFF);
    };
    const bool want_db = p.dbias != nullptr;
    float4 dbacc = zero4();
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int px = (t >> 4) + 16 * i;
            if (px >= C4_SW) continue;
            float4 v = r_dy[i];
            if (GATED) v = gate4(v, r_m[i]);
            // the 16-channel quarters of a pixel row are rotated by the pixel's position in its group of four: the four
            // pixels of a k-step then lie in four different quarters of the banks
            *reinterpret_cast<float4 *>(&dyL[(buf * C4_SW + px) * TAPS_T + (g4 ^ ((px & 3) << 4))]) = v;
            if (want_db) { dbacc.x += v.x; dbacc.y += v.y; dbacc.z += v.z; dbacc.w += v.w; }
        }
        if (t < 3 * C4_XW) *reinterpret_cast<float4 *>(&xW[buf * (C4_WIN + C4_ZERO) + t * 4]) = r_x;
    };

    typedef float f32x4 __attribute__((ext_vector_type(4)));
    f32x4 acc[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // operand offsets of this lane (floats): dy at pixel lq of the k-step, channel 16*wave + l16;
    // window column j = 16*nt + l16 = (tap, c): pixel lq + s of row r, or the zero area for j >= 36
    const int a_off = lq * TAPS_T + ((wave * 16 + l16) ^ (lq << 4));
    int b_off[3];
#pragma unroll
    for (int nt = 0; nt < 3; ++nt) {
        const int j = nt * 16 + l16, tap = j >> 2, c = j & 3, r = tap / 3, s = tap - r * 3;
        b_off[nt] = tap < 9 ? (r * C4_XW + s + lq) * 4 + c : C4_WIN + lq * 4 + c;
    }

    int buf = 0;
    fetch(n, row, strip, sid < send);
    __syncthreads();
    stash(0);
    __syncthreads();
    for (; sid < send; ++sid) {
        int row2 = row + 1, strip2 = strip, n2 = n;
        if (row2 == H) {
            row2 = 0;
            if (++strip2 == p.strips) { strip2 = 0; ++n2; }
        }
        const bool live2 = sid + 1 < send;
        fetch(n2, row2, strip2, live2);
        const float *dyA = dyL + buf * (C4_SW * TAPS_T) + a_off;
        const float *xB = xW + buf * (C4_WIN + C4_ZERO);
        float a[2], b[2][3];
        auto read = [&](int ks, int set) {
            a[set] = dyA[ks * (4 * TAPS_T)];
#pragma unroll
            for (int nt = 0; nt < 3; ++nt) b[set][nt] = xB[b_off[nt] + ks * 16];
        };
        read(0, 0);
#pragma unroll
        for (int ks = 0; ks < C4_KS; ++ks) {
            if (ks + 1 < C4_KS) read(ks + 1, (ks + 1) & 1);
            TAPS_FENCE;
#pragma unroll
            for (int nt = 0; nt < 3; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ks & 1], b[ks & 1][nt], acc[nt], 0, 0, 0);
            TAPS_FENCE;
        }
        buf ^= 1;
        if (live2) stash(buf);
        __syncthreads();
        row = row2; strip = strip2; n = n2;
    }

    if (want_db) {
        float *red = dyL;
        *reinterpret_cast<float4 *>(&red[(t >> 4) * TAPS_T + g4]) = dbacc;
        __syncthreads();
        if (t < TAPS_T && k0 + t < K) {
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) s += red[r * TAPS_T + t];
            p.dbias[(size_t)slice * K + k0 + t] = s;
        }
    }
    // accumulator register r of lane l: row 4*(l/16) + r, column l%16 of a 16x16 tile
    float *dst = p.out + (size_t)slice * K * 36;
#pragma unroll
    for (int nt = 0; nt < 3; ++nt) {
        const int j = nt * 16 + l16;
        if (j >= 36) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int k = k0 + wave * 16 + 4 * lq + r;
            if (k < K) dst[(size_t)k * 36 + j] = acc[nt][r];
        }
    }
}


// ---------------------------------------------------------------------------------------------------------------------
// Forward pass of the same image layer (C = 4, 3x3, stride 1, pad 1): y[pix][k] = bias[k] + sum_{tap,c} x[pix (+) tap][c] w[k][tap][c].
// The layer writes 16 output floats for every input float: it is bound by the one pass over y.  A k-step of
// v_mfma_f32_16x16x4_f32 is exactly one tap (4 channels), so the filter is nine registers per 16 output channels and
// lives in registers for the whole kernel; the image window (6 rows x 34 pixels x 4 channels for a stage of 4 rows x 32
// output pixels) is the only operand staged in LDS.  Each wavefront owns one output row of the stage (two groups of 16
// pixels) x 64 output channels: 72 MFMAs, then bias / ReLU, and the tile leaves through a private LDS patch as 16-byte
// vectors of whole pixel rows (1 KB contiguous per store instruction).
constexpr int F4_ROWS = 4, F4_COLS = 32;                       // output pixels of a stage
constexpr int F4_WR = F4_ROWS + 2, F4_WC = F4_COLS + 2;        // window
constexpr int F4_WIN = F4_WR * F4_WC * 4;                      // floats
constexpr int F4_LDC = TAPS_T + 4;                             // row stride of the output patch (floats)

struct FwdC4Params {
    const float *x, *w, *bias;     // x [N,H,W,4], w [K][3][3][4], bias [K] or nullptr
    float *y;                      // [N,H,W,K]
    int N, H, W, K;
    int strips, rowblocks;         // per image
    int tiles, slices, stages_per_item, total_stages;
    FastDiv fd_rowblocks, fd_strips, fd_tiles;
    uint32_t x_bytes;
};

template <bool RELU>
__global__ __launch_bounds__(256, 4) void fwd_c4_kernel(const FwdC4Params p)
{
    __shared__ __attribute__((aligned(16))) float xW[2 * F4_WIN];
    __shared__ __attribute__((aligned(16))) float patch[4 * 16 * F4_LDC];

    const int per_xcd = gridDim.x >> 3;
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= p.tiles * p.slices) return;
    const int slice = fdiv(L, p.fd_tiles), tk = L - slice * p.tiles;
    const int k0 = tk * TAPS_T;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, l16 = lane & 15, lq = lane >> 4;
    const int W = p.W, H = p.H, K = p.K;

    // the filter: b[kt][tap] = w[k0 + 16*kt + l16][tap][c = lq]
    float b[4][9];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
        const int k = k0 + kt * 16 + l16;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) b[kt][tap] = k < K ? p.w[((size_t)k * 9 + tap) * 4 + lq] : 0.f;
    }
    float bias4[4];      // this lane's 4 consecutive output channels in the store phase
#pragma unroll
    for (int e = 0; e < 4; ++e) bias4[e] = (p.bias && k0 + l16 * 4 + e < K) ? p.bias[k0 + l16 * 4 + e] : 0.f;

    int sid = slice * p.stages_per_item;
    const int send = min(p.total_stages, sid + p.stages_per_item);
    int rb, strip, n;
    {
        const int q = fdiv(sid, p.fd_rowblocks);
        rb = sid - q * p.rowblocks;
        n = fdiv(q, p.fd_strips);
        strip = q - n * p.strips;
    }
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.x, p.x_bytes);
    const int wrow = t / F4_WC, wcol = t - wrow * F4_WC;          // window loader, t < F4_WR * F4_WC
    float4 r_x;
    auto fetch = [&](int n_, int rb_, int strip_, bool live) {
        const int h = rb_ * F4_ROWS - 1 + wrow, w = strip_ * F4_COLS - 1 + wcol;
        const bool ok = live && t < F4_WR * F4_WC && (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
        r_x = bload4(rs_x, ok ? (uint32_t)(((n_ * H + h) * W + w) * 4) * 4u : OOB_OFF);
    };
    auto stash = [&](int buf) {
        if (t < F4_WR * F4_WC) *reinterpret_cast<float4 *>(&xW[buf * F4_WIN + t * 4]) = r_x;
    };

    typedef float f32x4 __attribute__((ext_vector_type(4)));
    // A operand of pixel group g (16 pixels of this wavefront's row), tap (r,s): window[(wave + r)][16*g + l16 + s][c = lq]
    const int a_off = (wave * F4_WC + l16) * 4 + lq;
    float *mine = patch + wave * (16 * F4_LDC);

    int buf = 0;
    fetch(n, rb, strip, sid < send);
    stash(0);
    // Every load issued so far (the filter registers among them) is waited for here, once.  Loads and stores share one counter
    // and return out of order with respect to each other, so a load that is waited for while stores are in flight waits for
    // every one of those stores: left pending into the loop, the first use of a filter register waited in every iteration for
    // all stores of the previous stage.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (; sid < send; ++sid) {
        int rb2 = rb + 1, strip2 = strip, n2 = n;
        if (rb2 == p.rowblocks) {
            rb2 = 0;
            if (++strip2 == p.strips) { strip2 = 0; ++n2; }
        }
        const bool live2 = sid + 1 < send;
        fetch(n2, rb2, strip2, live2);
        __builtin_amdgcn_sched_barrier(0);      // (the load is issued here, a stage of MFMAs ahead of its use)
        const float *win = xW + buf * F4_WIN + a_off;
        f32x4 acc[2][4];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) acc[g][kt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                const float a = win[((tap / 3) * F4_WC + 16 * g + tap % 3) * 4];
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) acc[g][kt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[kt][tap], acc[g][kt], 0, 0, 0);
            }
        // The next window goes to LDS BEFORE this stage's stores are issued (same reason as above): the stores in flight at this
        // wait are those of the previous stage, a whole stage of MFMAs old.  The other window buffer is free: its last readers
        // passed the barrier that ended the previous stage.
        if (live2) stash(buf ^ 1);
        // accumulator register r of lane l: pixel 4*(l/16) + r, channel 16*kt + l%16.  Through this wavefront's LDS patch the
        // tile turns into whole pixel rows: lane l then holds 4 consecutive channels (4*(l%16) ..) of pixel l/16 + 4*j.
        const int prow = rb * F4_ROWS + wave;
#pragma unroll
        for (int g = 0; g < 2; ++g) {
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) mine[(4 * lq + r) * F4_LDC + kt * 16 + l16] = acc[g][kt][r];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int px = lq + 4 * j;
                float4 v = *reinterpret_cast<const float4 *>(&mine[px * F4_LDC + l16 * 4]);
                v.x += bias4[0]; v.y += bias4[1]; v.z += bias4[2]; v.w += bias4[3];
                if (RELU) v = make_float4(fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f));
                const int q = strip * F4_COLS + 16 * g + px;
                if (prow < H && q < W && k0 + l16 * 4 < K)
                    *reinterpret_cast<float4 *>(p.y + ((size_t)(n * H + prow) * W + q) * K + k0 + l16 * 4) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        buf ^= 1;
        __syncthreads();
        rb = rb2; strip = strip2; n = n2;
    }
}

}  // namespace stanza
