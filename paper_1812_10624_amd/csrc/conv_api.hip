// CONV-worker entry points: forward, backward-data, backward-weight (paper Sec. 3.2), all three as
// launches of the implicit-GEMM engine in igemm.h, plus the two small fixed-order reductions the
// filter gradient needs (split partial sums, bias-gradient column sums).
#include "internal.h"
#include "igemm_bf16.h"

namespace stanza {

int conv_geometry(const stanza_conv_desc *d, ConvGeo *g)
{
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0) return STANZA_EINVAL;
    if (d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0) return STANZA_EINVAL;
    if (d->pad_h >= d->R || d->pad_w >= d->S) return STANZA_EINVAL;
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return STANZA_EINVAL;
    const int Ho = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1;
    const int Wo = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    const int64_t lim = (int64_t(1) << 31) - 1;
    if ((int64_t)d->N * d->H * d->W * d->C > lim || (int64_t)d->N * Ho * Wo * d->K > lim ||
        (int64_t)d->K * d->R * d->S * d->C > lim)
        return STANZA_EINVAL;
    *g = ConvGeo{d->N, d->H, d->W, d->C, d->K, d->R, d->S, d->stride_h, d->stride_w, d->pad_h, d->pad_w, Ho, Wo};
    return STANZA_OK;
}

// BWD_DATA: the stride class the rows of a launch stand for.  A caller that leaves p.sub unset gets the single class of a
// unit-stride layer; the divisors of the tap decode follow the class.
static int prepare_stride_class(GemmParams &p, int bk)
{
    const ConvGeo &g = p.g;
    if (p.sub.Hc == 0) {
        if (g.sh != 1 || g.sw != 1) return STANZA_EINVAL;
        p.sub = StrideClass{0, 0, g.H, g.W, g.ph, g.pw, 0, 0, g.R, g.S};
    }
    p.fd_s = make_fastdiv(max(1, p.sub.Sc));
    p.fd_rs = make_fastdiv(max(1, p.sub.Rc * p.sub.Sc));
    p.fd_hcwc = make_fastdiv(p.sub.Hc * p.sub.Wc);
    p.fd_wc = make_fastdiv(p.sub.Wc);
    if (p.sub.Rc * p.sub.Sc > 1 && g.K % bk == 0) p.flags |= ORDER_TAP_MINOR;
    return STANZA_OK;
}

// ------------------------------------------------------------------ tile choice, work-item plan and launch
constexpr int CUS = 256;   // compute units of the MI355X this library is written for

enum TileShape { T256x64, T128x64, T64x64, T64x128, T128x128 };
struct ShapeDim { int bm, bn; };
static ShapeDim shape_dim(TileShape s)
{
    switch (s) {
    case T256x64: return {256, 64};
    case T128x64: return {128, 64};
    case T64x64: return {64, 64};
    case T64x128: return {64, 128};
    default: return {128, 128};
    }
}

// Tall tiles while they still give every CU a couple of workgroups; 64-wide when the GEMM is narrow.
// can_slice: the launch may cut tiles into reduction slices, so a small tile count is no reason to shrink the tile.
static TileShape pick_shape(int mode, int M, int Nn, int Kd, int splits, bool can_slice)
{
    const int want = 512;
    if (mode != MODE_BWD_WEIGHT && M > 64) {
        // Short reductions (the 1x1 layers of the residual and Inception stacks): a tile's fill and drain are not amortised by its
        // few stages; what hides them is more resident workgroups, i.e. smaller tiles.  Measured over those stacks' layers at
        // batch 32-64: 64x64 tiles 7-30 % faster than 256x64 / 128x64 for Nn <= 64 and Kd <= 288, 64x128 tiles 6-16 % faster than
        // 128x128 for Kd <= 64 (with Kd = 576 and beyond the larger tiles win again).
        if (Nn <= 64 && Kd <= 288 && cdiv(M, 64) >= want) return T64x64;
        if (Nn % 128 == 0 && Kd <= 64 && (int64_t)cdiv(M, 64) * (Nn / 128) >= want) return T64x128;
        // Fewer than two 128x128 tiles per CU, and a reduction too short for cutting every tile into slices to pay (the slices'
        // raw sums are written and read back): take the largest tile of which there are at least two per CU, so that only the
        // tiles of its last, partly filled round are cut.  Measured 11-17 % faster on the 28x28x128, 14x14x1024->512 and
        // 7x7x512->2048 layers of the residual stacks; from Kd = 2304 on the 128x128 tiles with every tile cut win, and so they do
        // on the 512-row GEMMs of the FC worker (its last layer's data gradient: 60 against 50 us).
        if (M >= 1024 && Nn > 64 && Kd <= 1536 && (int64_t)cdiv(M, 128) * cdiv(Nn, 128) < want) {
            if (Nn % 128 == 0 && (int64_t)cdiv(M, 64) * (Nn / 128) >= want) return T64x128;
            if ((int64_t)cdiv(M, 128) * cdiv(Nn, 64) >= want) return T128x64;
            if ((int64_t)cdiv(M, 64) * cdiv(Nn, 64) >= want) return T64x64;
        }
    }
    if (mode != MODE_BWD_WEIGHT && Nn > 64 && M > 64) {
        // Column padding: a 128-wide tile over Nn = 160 or 192 columns multiplies a quarter to a third of zeros.  64-wide tiles pad
        // less and run at about 0.88 of the 128-wide tile's rate per useful flop (1.5 LDS reads per MFMA instead of 1).
        const double eff128 = (double)Nn / (cdiv(Nn, 128) * 128), eff64 = 0.88 * (double)Nn / (cdiv(Nn, 64) * 64);
        if (eff64 > eff128 && (can_slice || (int64_t)cdiv(M, 128) * cdiv(Nn, 64) * splits >= want)) return T128x64;
    }
    if (can_slice && M > 64 && Nn > 64) return T128x128;
    if (Nn <= 64) {
        if (mode != MODE_BWD_WEIGHT && (int64_t)cdiv(M, 256) * splits >= want) return T256x64;
        if ((int64_t)cdiv(M, 128) * splits >= want) return T128x64;
        return T64x64;
    }
    if (M <= 64 || (int64_t)cdiv(M, 128) * cdiv(Nn, 128) * splits < want) {
        if (M <= 64 || (int64_t)cdiv(M, 64) * cdiv(Nn, 128) * splits < want * 2) return T64x128;
    }
    return T128x128;
}

// How one GEMM is cut into work items.
struct GemmPlan {
    TileShape shape;
    int tilesM, tilesN, tiles;
    int dp_tiles;          // tiles computed whole by one workgroup
    int split_tiles;       // the last tiles, each cut into `splits` reduction slices
    int splits;
    int chunks_per_split;  // reduction stages (of BK) per slice
    size_t partial_floats; // FWD / BWD_DATA slice sums: split_tiles * splits * bm * bn
};

// FWD / BWD_DATA.  Workgroups are handed to the 256 CUs as slots free up, so a launch of T equal tiles takes
// ceil(T / 256) tile-times and the last round leaves CUs idle unless T is a multiple of 256 (a 14x14x512 layer at batch 64
// is 3.06 rounds of 64x128 tiles).  The tiles of that last round are cut into s reduction slices, s chosen to minimise
//   ceil(tail * s / 256) / s  +  s * (tail / 256) * io  +  launch
// in tile-times, where io = (write + read of one slice's raw tile at a CU's share of the HBM rate) / (one tile's MFMA time)
// = 123 / Kd.  When the whole launch is less than two rounds every tile is sliced, which also gives each CU the two to three
// resident workgroups the main loop needs to hide its LDS and barrier latencies.
static GemmPlan plan_gemm(int mode, int M, int Nn, int Kd, int bw_splits, bool may_slice)
{
    GemmPlan pl{};
    pl.shape = pick_shape(mode, M, Nn, Kd, mode == MODE_BWD_WEIGHT ? bw_splits : 1, mode != MODE_BWD_WEIGHT && may_slice && cdiv(Kd, BK) >= 16);
    const ShapeDim sd = shape_dim(pl.shape);
    pl.tilesM = cdiv(M, sd.bm);
    pl.tilesN = cdiv(Nn, sd.bn);
    pl.tiles = pl.tilesM * pl.tilesN;
    const int chunks = cdiv(Kd, BK);
    pl.dp_tiles = pl.tiles;
    pl.splits = 1;
    pl.chunks_per_split = chunks;
    if (mode == MODE_BWD_WEIGHT) {
        if (bw_splits > 1) {
            pl.dp_tiles = 0;
            pl.split_tiles = pl.tiles;
            pl.chunks_per_split = cdiv(chunks, bw_splits);
            pl.splits = cdiv(chunks, pl.chunks_per_split);
        }
        return pl;
    }
    if (!may_slice || chunks < 16) return pl;
    const int full = pl.tiles / CUS;
    int tail = pl.tiles % CUS;
    double base = 1.0;                      // cost of the unsliced tail round
    if (pl.tiles < 2 * CUS) {
        tail = pl.tiles;
        base = cdiv(pl.tiles, CUS) / (pl.tiles < 2 * CUS ? 0.75 : 1.0);   // a CU with a single resident workgroup idles on latencies
    } else if (tail == 0 || full >= 16) {
        return pl;
    }
    const double io = 123.0 / Kd;
    int best_s = 1;
    double best = base;
    for (int s = 2; s <= 16 && chunks / s >= 4; ++s) {
        const int64_t items = (int64_t)tail * s;
        double c = (double)cdiv64(items, CUS) / s;
        if (pl.tiles < 2 * CUS && items < 2 * CUS) c /= 0.75;
        c += s * ((double)tail / CUS) * io + 0.02;
        if (c < best * 0.97) { best = c; best_s = s; }
    }
    if (best_s > 1) {
        pl.split_tiles = tail;
        pl.dp_tiles = pl.tiles - tail;
        pl.chunks_per_split = cdiv(chunks, best_s);
        pl.splits = cdiv(chunks, pl.chunks_per_split);
        pl.partial_floats = (size_t)pl.split_tiles * pl.splits * sd.bm * sd.bn;
    }
    return pl;
}

// Floats of the column-statistics buffer of a forward GEMM (header + entries), for whichever of the two plans the launch takes.
size_t igemm_stats_floats(int M, int Nn, int Kd)
{
    if (M <= 0 || Nn <= 0 || Kd <= 0) return 0;
    size_t most = 0;
    for (int may = 0; may < 2; ++may) {
        const GemmPlan pl = plan_gemm(MODE_FWD, M, Nn, Kd, 1, may != 0);
        const ShapeDim sd = shape_dim(pl.shape);
        const size_t entries = (size_t)pl.dp_tiles + (size_t)pl.split_tiles * (sd.bm * sd.bn / 1024);
        const size_t fl = entries * 3 * sd.bn;
        if (fl > most) most = fl;
    }
    return STATS_HEADER_FLOATS + most;
}

size_t igemm_partial_floats(int mode, int M, int Nn, int Kd)
{
    if (mode == MODE_BWD_WEIGHT || M <= 0 || Nn <= 0 || Kd <= 0) return 0;
    return plan_gemm(mode, M, Nn, Kd, 1, true).partial_floats;
}

// Adds the reduction slices of every sliced tile in slice order and applies the epilogue of the main kernel.
// grid = (split_tiles, bm*bn / 1024); a thread owns 4 consecutive columns of one row and keeps four slice loads in flight
// (one load per dependent add made a tile of 8 slices cost 8 memory latencies: 14 us per launch on the 1x1 layers).
__global__ __launch_bounds__(256) void slice_fixup_kernel(const GemmParams p, int mode, int bm, int bn)
{
    __shared__ float4 sv[256];
    const int ti = blockIdx.x, tile = p.dp_tiles + ti;
    const int tile_n = tile % p.tilesN, tile_m = tile / p.tilesN;
    const int q4 = bn / 4;
    const size_t tile_floats = (size_t)bm * bn;
    const int idx = blockIdx.y * 256 + threadIdx.x;
    const int row_l = idx / q4, col_l = (idx - row_l * q4) * 4;
    const int row = tile_m * bm + row_l, col = tile_n * bn + col_l;
    const bool stats = mode == MODE_FWD && (p.flags & EPI_STATS);
    const bool valid = row < p.M && col < p.Nn;
    if (!valid && !stats) return;
    float4 acc = zero4();
    if (valid) {
        const float *src = p.partial + (size_t)ti * tile_floats + (size_t)row_l * bn + col_l;
        const size_t slice_stride = (size_t)p.split_tiles * tile_floats;
        auto add = [&](const float4 &v) { acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w; };
        int sl = 0;
        for (; sl + 4 <= p.splits; sl += 4) {
            const float4 v0 = ldg4(src + sl * slice_stride), v1 = ldg4(src + (sl + 1) * slice_stride);
            const float4 v2 = ldg4(src + (sl + 2) * slice_stride), v3 = ldg4(src + (sl + 3) * slice_stride);
            add(v0); add(v1); add(v2); add(v3);
        }
        for (; sl < p.splits; ++sl) add(ldg4(src + sl * slice_stride));
        const size_t o = (size_t)row * p.Nn + col;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (col + e >= p.Nn) break;
            float v = f4at(acc, e);
            if (mode == MODE_FWD) {
                if (p.flags & EPI_BIAS) v += p.bias[col + e];
                if (p.flags & EPI_RESIDUAL) v += p.res[o + e];
                if (p.flags & EPI_RELU) v = fmaxf(v, 0.f);
            } else {
                if (p.flags & EPI_ACCUM) v += p.out[o + e];
                if (p.flags & EPI_XMASK) v = p.xmask[o + e] > 0.f ? v : 0.f;
            }
            p.out[o + e] = v;
            f4at(acc, e) = v;
        }
    }
    if (!stats) return;
    // EPI_STATS (Nn % 4 == 0): the block's 1024 / bn rows are one entry; the first q4 threads walk down their 4 columns in row order
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        StatsHeader h{STATS_MAGIC, p.tilesM, p.tilesN, p.dp_tiles, bm, bn, p.M, p.Nn};
        *reinterpret_cast<StatsHeader *>(p.stats) = h;
    }
    sv[threadIdx.x] = acc;
    __syncthreads();
    const int rows_blk = 256 / q4;
    const int r_first = tile_m * bm + (int)blockIdx.y * rows_blk;
    const int n_rows = min(rows_blk, p.M - r_first);
    if ((int)threadIdx.x >= q4 || n_rows <= 0 || tile_n * bn + (int)threadIdx.x * 4 >= p.Nn) return;
    const float4 k = sv[threadIdx.x];
    float4 a = zero4(), b = zero4();
    for (int r = 0; r < n_rows; ++r) {
        const float4 v = sv[r * q4 + threadIdx.x];
        const float4 d = make_float4(v.x - k.x, v.y - k.y, v.z - k.z, v.w - k.w);
        a.x += d.x; a.y += d.y; a.z += d.z; a.w += d.w;
        b.x = fmaf(d.x, d.x, b.x); b.y = fmaf(d.y, d.y, b.y); b.z = fmaf(d.z, d.z, b.z); b.w = fmaf(d.w, d.w, b.w);
    }
    const int sub = bm * bn / 1024;
    float *e = p.stats + STATS_HEADER_FLOATS + ((size_t)p.dp_tiles + (size_t)ti * sub + blockIdx.y) * (3 * bn) + threadIdx.x * 4;
    *reinterpret_cast<float4 *>(e) = a;
    *reinterpret_cast<float4 *>(e + bn) = b;
    *reinterpret_cast<float4 *>(e + 2 * bn) = k;
}

template <int MODE, int BM, int BN, int WM, int WN>
static int launch_tile(GemmParams &p, const GemmPlan &pl, bool veca, bool vecb, hipStream_t st)
{
    p.tilesM = pl.tilesM;
    p.tilesN = pl.tilesN;
    p.tiles = pl.tiles;
    p.dp_tiles = pl.dp_tiles;
    p.split_tiles = pl.split_tiles;
    p.splits = pl.splits;
    p.chunks_per_split = pl.chunks_per_split;
    dim3 grid((unsigned)(cdiv(pl.dp_tiles, 8) * 8 + cdiv(pl.split_tiles * pl.splits, 8) * 8));
    const ConvGeo &g = p.g;
    const bool fast = veca && vecb &&
                      ((MODE == MODE_FWD && g.C % BK == 0) || (MODE == MODE_BWD_DATA && g.K % BK == 0));
    if (MODE != MODE_BWD_WEIGHT && fast)
        hipLaunchKernelGGL((igemm_kernel<MODE, BM, BN, WM, WN, true, true, MODE != MODE_BWD_WEIGHT>), grid, dim3(NTHREADS), 0, st, p);
    else if (veca && vecb)
        hipLaunchKernelGGL((igemm_kernel<MODE, BM, BN, WM, WN, true, true>), grid, dim3(NTHREADS), 0, st, p);
    else if (MODE == MODE_BWD_WEIGHT && veca)   // first layer: dy is vectorisable, the 3-channel image is not
        hipLaunchKernelGGL((igemm_kernel<MODE, BM, BN, WM, WN, true, false>), grid, dim3(NTHREADS), 0, st, p);
    else
        hipLaunchKernelGGL((igemm_kernel<MODE, BM, BN, WM, WN, false, false>), grid, dim3(NTHREADS), 0, st, p);
    int rc = launch_status();
    if (rc || MODE == MODE_BWD_WEIGHT || pl.split_tiles == 0) return rc;
    hipLaunchKernelGGL(slice_fixup_kernel, dim3(pl.split_tiles, BM * BN / 1024), dim3(256), 0, st, p, MODE, BM, BN);
    return launch_status();
}

template <int MODE>
static int launch_mode(GemmParams &p, const GemmPlan &pl, bool veca, bool vecb, hipStream_t st)
{
    switch (pl.shape) {
    case T256x64:
        if constexpr (MODE != MODE_BWD_WEIGHT) return launch_tile<MODE, 256, 64, 4, 1>(p, pl, veca, vecb, st);
        return STANZA_EINVAL;
    case T128x64: return launch_tile<MODE, 128, 64, 2, 2>(p, pl, veca, vecb, st);
    case T64x64: return launch_tile<MODE, 64, 64, 2, 2>(p, pl, veca, vecb, st);
    case T64x128: return launch_tile<MODE, 64, 128, 2, 2>(p, pl, veca, vecb, st);
    default: return launch_tile<MODE, 128, 128, 2, 2>(p, pl, veca, vecb, st);
    }
}

int launch_igemm(int mode, GemmParams &p, int bw_splits, float *partial, size_t partial_floats, hipStream_t st)
{
    const ConvGeo &g = p.g;
    // Kd == 0: a stride class of BWD_DATA that no tap reaches (the result is zero, the epilogue still runs)
    if (p.M <= 0 || p.Nn <= 0 || p.Kd < 0 || (p.Kd == 0 && mode != MODE_BWD_DATA) || bw_splits <= 0) return STANZA_EINVAL;
    if (p.flags & OUT_STRIDED) partial = nullptr;      // the fix-up kernel writes dense rows only
    GemmPlan pl = plan_gemm(mode, p.M, p.Nn, p.Kd, bw_splits, partial != nullptr);
    if (pl.partial_floats > partial_floats) pl = plan_gemm(mode, p.M, p.Nn, p.Kd, bw_splits, false);
    p.partial = partial;
    p.fd_c = make_fastdiv(g.C);
    p.fd_k = make_fastdiv(g.K);
    p.fd_s = make_fastdiv(g.S);
    p.fd_howo = make_fastdiv(g.Ho * g.Wo);
    p.fd_wo = make_fastdiv(g.Wo);
    p.fd_rs = make_fastdiv(g.R * g.S);
    if (g.R * g.S > 1 && mode == MODE_FWD && g.C % BK == 0) p.flags |= ORDER_TAP_MINOR;
    if (mode == MODE_BWD_DATA) {
        const int rc = prepare_stride_class(p, BK);
        if (rc) return rc;
    }
    // extents of the two gathered tensors; the vector fetch paths address them with 32-bit byte offsets below 2 GiB
    const int64_t xb = (int64_t)g.N * g.H * g.W * g.C * 4, yb = (int64_t)g.N * g.Ho * g.Wo * g.K * 4, wb = (int64_t)g.K * g.R * g.S * g.C * 4;
    const int64_t ab = mode == MODE_FWD ? xb : yb, bb = mode == MODE_BWD_WEIGHT ? xb : wb;
    const int64_t lim = int64_t(1) << 31;
    p.a_bytes = (uint32_t)(ab < lim ? ab : 0);
    p.b_bytes = (uint32_t)(bb < lim ? bb : 0);
    const bool small_a = ab < lim, small_b = bb < lim;
    switch (mode) {
    case MODE_FWD: return launch_mode<MODE_FWD>(p, pl, g.C % 4 == 0 && small_a && small_b, g.C % 4 == 0 && small_a && small_b, st);
    case MODE_BWD_DATA: return launch_mode<MODE_BWD_DATA>(p, pl, g.K % 4 == 0 && small_a, g.C % 4 == 0 && small_b, st);
    case MODE_BWD_WEIGHT: return launch_mode<MODE_BWD_WEIGHT>(p, pl, g.K % 4 == 0 && small_a, g.C % 4 == 0 && small_b, st);
    }
    return STANZA_EINVAL;
}

// The stride classes of a strided layer's data gradient (n <= MAX_CLASSES parameter sets that differ in their class geometry,
// row count and reduction length) as ONE launch: one tile shape for all of them, chosen for their tiles together; no tile is cut
// into reduction slices (the classes together fill the CUs, and their rows are scattered pixels).
template <int BM, int BN, int WM, int WN>
static int launch_classes_tile(GemmClasses &P, int n, bool vec, hipStream_t st)
{
    int most = 0;
    for (int i = 0; i < n; ++i) {
        GemmParams &q = P.q[i];
        q.tilesM = cdiv(q.M, BM);
        q.tilesN = cdiv(q.Nn, BN);
        q.tiles = q.dp_tiles = q.tilesM * q.tilesN;
        q.split_tiles = 0;
        q.splits = 1;
        q.chunks_per_split = cdiv(q.Kd, BK);
        most = max(most, q.tiles);
    }
    const dim3 grid((unsigned)(cdiv(most, 8) * 8), (unsigned)n);
    const bool fast = vec && P.q[0].g.K % BK == 0;
    if (fast) hipLaunchKernelGGL((igemm_classes_kernel<BM, BN, WM, WN, true, true, true>), grid, dim3(NTHREADS), 0, st, P);
    else if (vec) hipLaunchKernelGGL((igemm_classes_kernel<BM, BN, WM, WN, true, true, false>), grid, dim3(NTHREADS), 0, st, P);
    else hipLaunchKernelGGL((igemm_classes_kernel<BM, BN, WM, WN, false, false, false>), grid, dim3(NTHREADS), 0, st, P);
    return launch_status();
}

static int launch_igemm_classes(GemmClasses &P, int n, hipStream_t st)
{
    if (n < 1 || n > MAX_CLASSES) return STANZA_EINVAL;
    const ConvGeo &g = P.q[0].g;
    const int64_t yb = (int64_t)g.N * g.Ho * g.Wo * g.K * 4, wb = (int64_t)g.K * g.R * g.S * g.C * 4, lim = int64_t(1) << 31;
    int64_t rows = 0;
    int kd_max = 0;
    for (int i = 0; i < n; ++i) {
        GemmParams &q = P.q[i];
        if (q.M <= 0 || q.Nn <= 0 || q.Kd < 0) return STANZA_EINVAL;
        q.partial = nullptr;
        q.fd_c = make_fastdiv(g.C);
        q.fd_k = make_fastdiv(g.K);
        q.fd_howo = make_fastdiv(g.Ho * g.Wo);
        q.fd_wo = make_fastdiv(g.Wo);
        const int rc = prepare_stride_class(q, BK);
        if (rc) return rc;
        q.a_bytes = (uint32_t)(yb < lim ? yb : 0);
        q.b_bytes = (uint32_t)(wb < lim ? wb : 0);
        rows += q.M;
        kd_max = max(kd_max, q.Kd);
    }
    const bool vec = g.K % 4 == 0 && g.C % 4 == 0 && yb < lim && wb < lim;
    switch (pick_shape(MODE_BWD_DATA, (int)(rows < INT32_MAX ? rows : INT32_MAX), P.q[0].Nn, kd_max, 1, false)) {
    case T256x64: return launch_classes_tile<256, 64, 4, 1>(P, n, vec, st);
    case T128x64: return launch_classes_tile<128, 64, 2, 2>(P, n, vec, st);
    case T64x64: return launch_classes_tile<64, 64, 2, 2>(P, n, vec, st);
    case T64x128: return launch_classes_tile<64, 128, 2, 2>(P, n, vec, st);
    default: return launch_classes_tile<128, 128, 2, 2>(P, n, vec, st);
    }
}

// ------------------------------------------------------------------ bf16-in path
template <int MODE, int BM, int BN, int WM, int WN>
static int launch_tile_bf16(GemmParams &p, int splits, hipStream_t st)
{
    p.tilesM = cdiv(p.M, BM);
    p.tilesN = cdiv(p.Nn, BN);
    p.tiles = p.tilesM * p.tilesN;
    p.splits = splits;
    dim3 grid((unsigned)(cdiv(p.tiles * splits, 8) * 8));
    const ConvGeo &g = p.g;
    // a stage that stays inside one filter tap: wavefront-uniform tap decode, no per-thread division in the main loop
    const bool fast = g.R * g.S <= 32 && ((MODE == MODE_FWD && g.C % BKH == 0) || (MODE == MODE_BWD_DATA && g.K % BKH == 0));
    const bool gated = MODE != MODE_FWD && (p.flags & LOAD_AMASK);
    constexpr bool CAN_FAST = MODE != MODE_BWD_WEIGHT, CAN_GATE = MODE != MODE_FWD;
    if (fast && !gated)
        hipLaunchKernelGGL((igemm_bf16_kernel<MODE, BM, BN, WM, WN, CAN_FAST, false>), grid, dim3(NTHREADS), 0, st, p);
    else if (fast)
        hipLaunchKernelGGL((igemm_bf16_kernel<MODE, BM, BN, WM, WN, CAN_FAST, CAN_GATE>), grid, dim3(NTHREADS), 0, st, p);
    else if (!gated)
        hipLaunchKernelGGL((igemm_bf16_kernel<MODE, BM, BN, WM, WN, false, false>), grid, dim3(NTHREADS), 0, st, p);
    else
        hipLaunchKernelGGL((igemm_bf16_kernel<MODE, BM, BN, WM, WN, false, CAN_GATE>), grid, dim3(NTHREADS), 0, st, p);
    return launch_status();
}

template <int MODE>
static int launch_mode_bf16(GemmParams &p, int splits, hipStream_t st)
{
    if (p.Nn <= 64) {
        // short reductions: more, smaller workgroups hide a tile's fill and drain (1x1 layers of the residual stacks, 64 columns:
        // 64x64 tiles 6-19 % faster than 128x64; with Kd = 576 at 224x224 the 128x64 tiles win)
        if (MODE != MODE_BWD_WEIGHT && p.Kd <= 288) return launch_tile_bf16<MODE, 64, 64, 2, 2>(p, splits, st);
        if ((int64_t)cdiv(p.M, 128) * splits >= 512) return launch_tile_bf16<MODE, 128, 64, 2, 2>(p, splits, st);
        return launch_tile_bf16<MODE, 64, 64, 2, 2>(p, splits, st);
    }
    // 128x128 tiles from 160 work items on (measured: with 196 to 507 items, the 14x14 and 28x28 layers at batch 64, they are 5-28 %
    // faster than twice as many 64x128 tiles; with 100 items, the 7x7 layers, the 64x128 tiles are 20 % faster)
    if (p.M <= 64 || (int64_t)cdiv(p.M, 128) * cdiv(p.Nn, 128) * splits < 160) {
        // ... and under 160 items 64x64 tiles beat 64x128 by 16-29 % on the 17x17 and 8x8 layers of the Inception stack (reductions
        // up to 2880 deep; at 4608 the 64x128 tiles are 5 % ahead)
        if (MODE != MODE_BWD_WEIGHT && p.M > 64 && p.Kd <= 3072) return launch_tile_bf16<MODE, 64, 64, 2, 2>(p, splits, st);
        return launch_tile_bf16<MODE, 64, 128, 2, 2>(p, splits, st);
    }
    // a column count that fills at most half of its last 128-wide tile (160, 192, 288, 320): 64-wide tiles multiply a quarter to a
    // third fewer zeros (17-25 % faster on those layers of the Inception stack)
    if (MODE != MODE_BWD_WEIGHT && p.Nn % 128 != 0 && p.Nn % 128 <= 64) return launch_tile_bf16<MODE, 128, 64, 2, 2>(p, splits, st);
    return launch_tile_bf16<MODE, 128, 128, 2, 2>(p, splits, st);
}

// bf16 form of launch_igemm_classes: the tile shape by the rules of launch_mode_bf16, applied to the classes' tiles together
template <int BM, int BN, int WM, int WN>
static int launch_classes_tile_bf16(GemmClasses &P, int n, hipStream_t st)
{
    int most = 0;
    for (int i = 0; i < n; ++i) {
        GemmParams &q = P.q[i];
        q.tilesM = cdiv(q.M, BM);
        q.tilesN = cdiv(q.Nn, BN);
        q.tiles = q.tilesM * q.tilesN;
        q.splits = 1;
        most = max(most, q.tiles);
    }
    const dim3 grid((unsigned)(cdiv(most, 8) * 8), (unsigned)n);
    const ConvGeo &g = P.q[0].g;
    const bool fast = g.R * g.S <= 32 && g.K % BKH == 0;
    const bool gated = P.q[0].flags & LOAD_AMASK;
    if (fast && !gated) hipLaunchKernelGGL((igemm_bf16_classes_kernel<BM, BN, WM, WN, true, false>), grid, dim3(NTHREADS), 0, st, P);
    else if (fast) hipLaunchKernelGGL((igemm_bf16_classes_kernel<BM, BN, WM, WN, true, true>), grid, dim3(NTHREADS), 0, st, P);
    else if (!gated) hipLaunchKernelGGL((igemm_bf16_classes_kernel<BM, BN, WM, WN, false, false>), grid, dim3(NTHREADS), 0, st, P);
    else hipLaunchKernelGGL((igemm_bf16_classes_kernel<BM, BN, WM, WN, false, true>), grid, dim3(NTHREADS), 0, st, P);
    return launch_status();
}

static int launch_igemm_bf16_classes(GemmClasses &P, int n, hipStream_t st)
{
    if (n < 1 || n > MAX_CLASSES) return STANZA_EINVAL;
    const ConvGeo &g = P.q[0].g;
    if (g.C % 8 || g.K % 8) return STANZA_EUNSUPPORTED;
    const int64_t yb = (int64_t)g.N * g.Ho * g.Wo * g.K * 2, wb = (int64_t)g.K * g.R * g.S * g.C * 2;
    if (yb >= (int64_t(1) << 31) || wb >= (int64_t(1) << 31)) return STANZA_EUNSUPPORTED;
    int64_t items128 = 0, items64 = 0;
    int kd_max = 0, m_max = 0;
    const int Nn = P.q[0].Nn;
    for (int i = 0; i < n; ++i) {
        GemmParams &q = P.q[i];
        if (q.M <= 0 || q.Nn <= 0 || q.Kd < 0) return STANZA_EINVAL;
        q.fd_c = make_fastdiv(g.C);
        q.fd_k = make_fastdiv(g.K);
        q.fd_howo = make_fastdiv(g.Ho * g.Wo);
        q.fd_wo = make_fastdiv(g.Wo);
        const int rc = prepare_stride_class(q, BKH);
        if (rc) return rc;
        q.a_bytes = (uint32_t)yb;
        q.b_bytes = (uint32_t)wb;
        items128 += (int64_t)cdiv(q.M, 128) * cdiv(Nn, 128);
        items64 += cdiv(q.M, 128);
        kd_max = max(kd_max, q.Kd);
        m_max = max(m_max, q.M);
    }
    // (the rules of launch_mode_bf16 for MODE_BWD_DATA, with the classes' work items added up)
    if (Nn <= 64) {
        if (kd_max <= 288) return launch_classes_tile_bf16<64, 64, 2, 2>(P, n, st);
        if (items64 >= 512) return launch_classes_tile_bf16<128, 64, 2, 2>(P, n, st);
        return launch_classes_tile_bf16<64, 64, 2, 2>(P, n, st);
    }
    if (m_max <= 64 || items128 < 160) {
        if (m_max > 64 && kd_max <= 3072) return launch_classes_tile_bf16<64, 64, 2, 2>(P, n, st);
        return launch_classes_tile_bf16<64, 128, 2, 2>(P, n, st);
    }
    if (Nn % 128 != 0 && Nn % 128 <= 64) return launch_classes_tile_bf16<128, 64, 2, 2>(P, n, st);
    return launch_classes_tile_bf16<128, 128, 2, 2>(P, n, st);
}

int launch_igemm_bf16(int mode, GemmParams &p, int splits, hipStream_t st)
{
    const ConvGeo &g = p.g;
    if (p.M <= 0 || p.Nn <= 0 || p.Kd < 0 || (p.Kd == 0 && mode != MODE_BWD_DATA) || splits <= 0) return STANZA_EINVAL;
    if (g.C % 8 || g.K % 8) return STANZA_EUNSUPPORTED;
    p.fd_c = make_fastdiv(g.C);
    p.fd_k = make_fastdiv(g.K);
    p.fd_s = make_fastdiv(g.S);
    p.fd_howo = make_fastdiv(g.Ho * g.Wo);
    p.fd_wo = make_fastdiv(g.Wo);
    p.fd_rs = make_fastdiv(g.R * g.S);
    if (mode == MODE_BWD_DATA) {
        const int rc = prepare_stride_class(p, BKH);
        if (rc) return rc;
    }
    // the gathered tensors are addressed with 32-bit byte offsets below 2 GiB (an offset of 2 GiB marks a masked lane)
    const int64_t xb = (int64_t)g.N * g.H * g.W * g.C * 2, yb = (int64_t)g.N * g.Ho * g.Wo * g.K * 2, wb = (int64_t)g.K * g.R * g.S * g.C * 2;
    const int64_t ab = mode == MODE_FWD ? xb : yb, bb = mode == MODE_BWD_WEIGHT ? xb : wb;
    if (ab >= (int64_t(1) << 31) || bb >= (int64_t(1) << 31)) return STANZA_EUNSUPPORTED;
    p.a_bytes = (uint32_t)ab;
    p.b_bytes = (uint32_t)bb;
    switch (mode) {
    case MODE_FWD: return launch_mode_bf16<MODE_FWD>(p, 1, st);
    case MODE_BWD_DATA: return launch_mode_bf16<MODE_BWD_DATA>(p, 1, st);
    case MODE_BWD_WEIGHT: return launch_mode_bf16<MODE_BWD_WEIGHT>(p, splits, st);
    }
    return STANZA_EINVAL;
}

// ------------------------------------------------------------------ fixed-order reductions
// out[i] = sum over slices of partial[slice][i]; likewise the second segment (bias gradient).  Output i is shared by LANES
// threads: thread l adds the slices l, l + LANES, ... in ascending order (four loads in flight) and the LANES sums are added in
// lane order through LDS.  A short output with hundreds of slices (a 1x1 filter gradient) would otherwise be one
// long dependent chain per thread on a handful of workgroups.
template <int LANES>
__global__ __launch_bounds__(256) void split_reduce_kernel(const float *__restrict__ partial, int splits, size_t numel, float *__restrict__ out,
                                                           const float *__restrict__ partial2, size_t numel2, float *__restrict__ out2)
{
    constexpr int OUTS = 256 / LANES;          // outputs per workgroup (consecutive: coalesced rows of every slice)
    __shared__ float red[LANES][OUTS];
    const int ol = threadIdx.x % OUTS, lane = threadIdx.x / OUTS;
    size_t i = (size_t)blockIdx.x * OUTS + ol;
    const float *src = partial;
    float *dst = out;
    size_t n = numel;
    bool live = true;
    if (i >= numel) {
        i -= numel;
        src = partial2; dst = out2; n = numel2;
        live = i < numel2;
    }
    float s = 0.f;
    if (live) {
        int k = lane;
        for (; k + 3 * LANES < splits; k += 4 * LANES) {
            const float v0 = src[(size_t)k * n + i], v1 = src[(size_t)(k + LANES) * n + i];
            const float v2 = src[(size_t)(k + 2 * LANES) * n + i], v3 = src[(size_t)(k + 3 * LANES) * n + i];
            s += v0; s += v1; s += v2; s += v3;
        }
        for (; k < splits; k += LANES) s += src[(size_t)k * n + i];
    }
    if (LANES == 1) {
        if (live) dst[i] = s;
        return;
    }
    red[lane][ol] = s;
    __syncthreads();
    if (lane == 0 && live) {
        for (int l = 1; l < LANES; ++l) s += red[l][ol];
        dst[i] = s;
    }
}

int launch_split_reduce(const float *partial, int splits, size_t numel, float *out, const float *partial2, size_t numel2, float *out2,
                        hipStream_t st)
{
    // enough threads to fill the GPU: more lanes per output the shorter the output and the more slices there are
    const size_t total = numel + numel2;
    const int lanes = (splits >= 64 && total < (size_t(1) << 18)) ? 16 : (splits >= 16 && total < (size_t(1) << 20)) ? 4 : 1;
    if (lanes == 16)
        hipLaunchKernelGGL(split_reduce_kernel<16>, dim3((unsigned)cdiv64(total, 16)), dim3(256), 0, st, partial, splits, numel, out, partial2, numel2, out2);
    else if (lanes == 4)
        hipLaunchKernelGGL(split_reduce_kernel<4>, dim3((unsigned)cdiv64(total, 64)), dim3(256), 0, st, partial, splits, numel, out, partial2, numel2, out2);
    else
        hipLaunchKernelGGL(split_reduce_kernel<1>, dim3((unsigned)cdiv64(total, 256)), dim3(256), 0, st, partial, splits, numel, out, partial2, numel2, out2);
    return launch_status();
}

// pass 1: workgroup (bx, by) sums rows [bx*rows_per, (bx+1)*rows_per) of columns by*64 .. by*64+63;
// wavefront w takes every 4th row, lanes take consecutive columns (256-byte row segments).
__global__ __launch_bounds__(256) void colsum_pass1(const float *__restrict__ a, const float *__restrict__ mask, int rows, int cols,
                                                    int rows_per, float *__restrict__ scratch)
{
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = blockIdx.y * 64 + lane;
    const int rbeg = blockIdx.x * rows_per, rend = min(rows, rbeg + rows_per);
    float s = 0.f;
    if (col < cols) {
        for (int r = rbeg + wave; r < rend; r += 4) {
            const size_t o = (size_t)r * cols + col;
            float v = a[o];
            if (mask) v = mask[o] > 0.f ? v : 0.f;
            s += v;
        }
    }
    red[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && col < cols) scratch[(size_t)blockIdx.x * cols + col] = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

__global__ void colsum_pass2(const float *__restrict__ scratch, int blocks, int cols, float *__restrict__ out,
                             float *__restrict__ sgd_p, float *__restrict__ sgd_v, float lr, float mom, float wd)
{
    const int col = blockIdx.x * blockDim.x + threadIdx.x;
    if (col >= cols) return;
    float s = 0.f;
    for (int b = 0; b < blocks; ++b) s += scratch[(size_t)b * cols + col];
    if (sgd_p) {
        const float w = sgd_p[col];
        const float vel = mom * sgd_v[col] + (s + wd * w);
        sgd_v[col] = vel;
        sgd_p[col] = w - lr * vel;
    } else {
        out[col] = s;
    }
}

int colsum_blocks(int rows) { return max(1, min(64, cdiv(rows, 64))); }

int launch_colsum(const float *a, const float *mask, int rows, int cols, float *scratch, int blocks, float *out,
                  float *sgd_p, float *sgd_v, float lr, float mom, float wd, hipStream_t st)
{
    const int rows_per = cdiv(rows, blocks);
    hipLaunchKernelGGL(colsum_pass1, dim3(blocks, cdiv(cols, 64)), dim3(256), 0, st, a, mask, rows, cols, rows_per, scratch);
    int rc = launch_status();
    if (rc) return rc;
    hipLaunchKernelGGL(colsum_pass2, dim3(cdiv(cols, 256)), dim3(256), 0, st, scratch, blocks, cols, out, sgd_p, sgd_v, lr, mom, wd);
    return launch_status();
}

// The nine-tap kernel takes float32 3x3 / stride 1 / pad 1 layers whose channel counts fill most of a 64 x 64 tile.
// Strip width SW <= 28 output pixels; a stage is RP rows of XW = SW + 2 (even) pixel slots, RP > 1 only when one strip
// spans the image; limits: RP * XW <= 32 slots per stage, (2 RP + 4) * XW <= 186 slots in the ring of x rows.
bool plan_wgrad_taps(const ConvGeo &g, TapsParams *tp)
{
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1) return false;
    if (g.C % 4 || g.K % 4 || g.C < 48 || g.K < 48) return false;
    const int64_t lim = int64_t(1) << 31;
    if ((int64_t)g.N * g.H * g.W * g.C * 4 >= lim || (int64_t)g.N * g.H * g.W * g.K * 4 >= lim) return false;
    TapsParams t{};
    t.N = g.N; t.H = g.H; t.W = g.W; t.C = g.C; t.K = g.K;
    t.strips = cdiv(g.W, 28);
    t.SW = cdiv(g.W, t.strips);
    t.XW = (t.SW + 2 + 1) & ~1;
    t.RP = 1;
    if (t.strips == 1) {
        t.RP = max(1, min(TAPS_J / t.XW, g.H));
        while (t.RP > 1 && (2 * t.RP + 4) * t.XW > TAPS_XSLOTS) --t.RP;
    }
    if (t.RP * t.XW > TAPS_J || (2 * t.RP + 4) * t.XW > TAPS_XSLOTS) return false;
    t.NR = 2 * t.RP + 4;
    t.KS = t.RP * t.XW / 2 - 1;
    t.rowblocks = cdiv(g.H, t.RP);
    t.total_stages = g.N * t.strips * t.rowblocks;
    t.tiles_c = cdiv(g.C, TAPS_T);
    t.tiles = cdiv(g.K, TAPS_T) * t.tiles_c;
    // one round of resident workgroups (two per CU: 144 accumulator registers per lane), slices of at least 4 stages
    int slices = max(1, 2 * CUS / t.tiles);
    slices = max(1, min(slices, t.total_stages / 4));
    t.stages_per_item = cdiv(t.total_stages, slices);
    t.slices = cdiv(t.total_stages, t.stages_per_item);
    t.fd_xw = make_fastdiv(t.XW);
    t.fd_rowblocks = make_fastdiv(t.rowblocks);
    t.fd_strips = make_fastdiv(t.strips);
    t.fd_tiles = make_fastdiv(t.tiles);
    t.fd_tiles_c = make_fastdiv(t.tiles_c);
    t.dy_bytes = (uint32_t)((int64_t)g.N * g.H * g.W * g.K * 4);
    t.x_bytes = (uint32_t)((int64_t)g.N * g.H * g.W * g.C * 4);
    *tp = t;
    return true;
}

// The image-layer form: 4 input channels (an RGB image padded to 4), any width (strips of at most 56 pixels).
bool plan_wgrad_taps_c4(const ConvGeo &g, TapsC4Params *tp)
{
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1 || g.C != 4 || g.K % 4) return false;
    const int64_t lim = int64_t(1) << 31;
    if ((int64_t)g.N * g.H * g.W * g.K * 4 >= lim) return false;
    TapsC4Params t{};
    t.N = g.N; t.H = g.H; t.W = g.W; t.K = g.K;
    t.strips = cdiv(g.W, C4_SW);
    t.SW = cdiv(g.W, t.strips);
    t.total_stages = g.N * t.strips * g.H;
    t.tiles = cdiv(g.K, TAPS_T);
    int slices = max(1, 4 * CUS / t.tiles);          // four resident workgroups per CU
    slices = max(1, min(slices, t.total_stages / 4));
    t.stages_per_item = cdiv(t.total_stages, slices);
    t.slices = cdiv(t.total_stages, t.stages_per_item);
    t.fd_h = make_fastdiv(g.H);
    t.fd_strips = make_fastdiv(t.strips);
    t.fd_tiles = make_fastdiv(t.tiles);
    t.dy_bytes = (uint32_t)((int64_t)g.N * g.H * g.W * g.K * 4);
    t.x_bytes = (uint32_t)((int64_t)g.N * g.H * g.W * 4 * 4);
    *tp = t;
    return true;
}

// Forward pass of an image layer (4 input channels, 3x3, stride 1, pad 1): the kernel that keeps the filter in registers.
bool plan_fwd_c4(const ConvGeo &g, FwdC4Params *fp)
{
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1 || g.C != 4 || g.K % 4) return false;
    if ((int64_t)g.N * g.H * g.W * 16 >= (int64_t(1) << 31)) return false;
    FwdC4Params f{};
    f.N = g.N; f.H = g.H; f.W = g.W; f.K = g.K;
    f.strips = cdiv(g.W, F4_COLS);
    f.rowblocks = cdiv(g.H, F4_ROWS);
    f.total_stages = g.N * f.strips * f.rowblocks;
    f.tiles = cdiv(g.K, TAPS_T);
    int slices = max(1, 4 * CUS / f.tiles);          // one round of four resident workgroups per CU (two rounds: 2 % slower)
    slices = max(1, min(slices, f.total_stages / 4));
    f.stages_per_item = cdiv(f.total_stages, slices);
    f.slices = cdiv(f.total_stages, f.stages_per_item);
    f.fd_rowblocks = make_fastdiv(f.rowblocks);
    f.fd_strips = make_fastdiv(f.strips);
    f.fd_tiles = make_fastdiv(f.tiles);
    f.x_bytes = (uint32_t)((int64_t)g.N * g.H * g.W * 16);
    *fp = f;
    return true;
}

// The stage geometries of the 224- to 28-pixel-wide, the 14- and the 7-pixel-wide layers have kernels of their own with
// the geometry compiled in; anything else runs the kernel that reads it from the parameters.
template <bool GATED>
static void launch_wgrad_taps_g(const TapsParams &tp, dim3 grid, hipStream_t st)
{
    if (tp.XW == 30 && tp.RP == 1) hipLaunchKernelGGL((wgrad_taps_kernel<GATED, 30, 1>), grid, dim3(256), 0, st, tp);
    else if (tp.XW == 16 && tp.RP == 2) hipLaunchKernelGGL((wgrad_taps_kernel<GATED, 16, 2>), grid, dim3(256), 0, st, tp);
    else if (tp.XW == 10 && tp.RP == 3) hipLaunchKernelGGL((wgrad_taps_kernel<GATED, 10, 3>), grid, dim3(256), 0, st, tp);
    else hipLaunchKernelGGL((wgrad_taps_kernel<GATED, 0, 0>), grid, dim3(256), 0, st, tp);
}
static void launch_wgrad_taps(const TapsParams &tp, dim3 grid, hipStream_t st)
{
    if (tp.amask) launch_wgrad_taps_g<true>(tp, grid, st);
    else launch_wgrad_taps_g<false>(tp, grid, st);
}

// Whether the nine-tap kernel is the faster choice for a layer it can handle.  Its MFMAs run over whole stages of pixel slots and
// whole 64x64 (k, c) tiles, so what it gains by fetching each operand once it loses where the slots or the tiles are partly empty:
// 7x7 and 8x8 images (stages of three rows, 54-71 % filled: the implicit GEMM is 10-31 % faster there), 13x13 (75 %: 7 %
// faster), 35 pixels wide with 96 channels (49 %: 28 %).  From 80 % on (14, 28, 56, 112, 224 pixels wide with channel counts that
// are multiples of 64: 87-93 %) the nine-tap kernel wins.
static bool taps_pays(const ConvGeo &g, const TapsParams &t)
{
    const double slots = (double)g.W / (t.strips * t.XW) * g.H / (double)(t.rowblocks * t.RP);
    const double tiles = (double)g.K / (cdiv(g.K, TAPS_T) * TAPS_T) * g.C / (double)(t.tiles_c * TAPS_T);
    return slots * tiles >= 0.8;
}

WgradPlan plan_wgrad(const ConvGeo &g, bool want_bias, int bk, bool force_taps)
{
    WgradPlan pl{};
    TapsParams tp;
    TapsC4Params tp4;
    const bool nine = bk == BK && plan_wgrad_taps(g, &tp) && (force_taps || taps_pays(g, tp));
    const bool nine4 = bk == BK && !nine && plan_wgrad_taps_c4(g, &tp4);
    if (nine || nine4) {
        pl.taps = nine ? 1 : 2;
        pl.splits = nine ? tp.slices : tp4.slices;
        pl.chunks_per_split = nine ? tp.stages_per_item : tp4.stages_per_item;
        pl.partial_floats = pl.splits > 1 ? (size_t)pl.splits * g.K * 9 * g.C : 0;
        pl.db_floats = (want_bias && pl.splits > 1) ? (size_t)pl.splits * g.K : 0;
        pl.bytes = round256(pl.partial_floats * 4) + round256(pl.db_floats * 4);
        return pl;
    }
    const int M = g.K, Nn = g.R * g.S * g.C;
    const int64_t red = (int64_t)g.N * g.Ho * g.Wo;
    const int chunks = (int)cdiv64(red, bk);
    const int bm = M <= 64 ? 64 : 128, bn = Nn <= 64 ? 64 : 128;
    const int tiles = cdiv(M, bm) * cdiv(Nn, bn);
    // A whole number of rounds of workgroups and never a few items more: 1026 items on 256 CUs take as long as 1280.  Both kernels
    // keep four workgroups resident per CU and run best as exactly one such round (measured over the VGG-16-shaped layers, 2 to
    // 12 items per CU: five is slower than four, eight equals it at twice the partial sums).
    const int resident = 4 * CUS;
    int splits = resident / tiles;
    // ... unless that leaves a slice 16 stages or fewer (1x1 filters on small maps): a slice's partial tile, written and read
    // back, then costs as much as its MFMAs, and two items per CU with slices twice as long are faster (7 to 10 % on the 1x1
    // layers of the residual stacks at 7x7 to 28x28)
    if (splits > 1 && cdiv(chunks, splits) <= 16) splits = max(1, resident / 2 / tiles);
    splits = max(1, min(splits, chunks / 8));
    pl.chunks_per_split = cdiv(chunks, splits);
    pl.splits = cdiv(chunks, pl.chunks_per_split);
    pl.partial_floats = pl.splits > 1 ? (size_t)pl.splits * M * Nn : 0;
    pl.db_floats = (want_bias && pl.splits > 1) ? (size_t)pl.splits * g.K : 0;
    pl.bytes = round256(pl.partial_floats * 4) + round256(pl.db_floats * 4);
    return pl;
}

}  // namespace stanza

using namespace stanza;

extern "C" size_t stanza_conv_workspace_bytes(const stanza_conv_desc *desc, int which)
{
    ConvGeo g;
    if (!desc || which < 0 || which > 2 || conv_geometry(desc, &g) != STANZA_OK) return 0;
    if (which == 2)
        return plan_wgrad(g, (desc->flags & STANZA_CONV_BIAS) != 0, desc->dtype == STANZA_BF16 ? BKH : BK, (desc->flags & STANZA_CONV_NINE_TAP) != 0).bytes;
    if (desc->dtype != STANZA_F32) return 0;
    const size_t fl = which == 0 ? igemm_partial_floats(MODE_FWD, g.N * g.Ho * g.Wo, g.K, g.R * g.S * g.C)
                                 : igemm_partial_floats(MODE_BWD_DATA, g.N * g.H * g.W, g.C, g.R * g.S * g.K);
    return round256(fl * 4);
}

// float32 always; bfloat16 when both channel counts are multiples of 8 (one 16-byte vector stays inside a tap)
static int check_dtype(const stanza_conv_desc *d)
{
    if (d->dtype == STANZA_F32) return STANZA_OK;
    if (d->dtype == STANZA_BF16 && d->C % 8 == 0 && d->K % 8 == 0) return STANZA_OK;
    return STANZA_EUNSUPPORTED;
}

// ws / ws_bytes: the optional slice workspace of a float32 forward or backward-data call
static int launch_any(const stanza_conv_desc *d, int mode, GemmParams &p, int splits, void *ws, size_t ws_bytes, hipStream_t st)
{
    if (d->dtype == STANZA_BF16) return launch_igemm_bf16(mode, p, splits, st);
    if (mode == MODE_BWD_WEIGHT) return launch_igemm(mode, p, splits, nullptr, 0, st);
    return launch_igemm(mode, p, 1, (float *)ws, ws ? ws_bytes / 4 : 0, st);
}

static int launch_classes(const stanza_conv_desc *d, GemmClasses &P, int n, hipStream_t st)
{
    return d->dtype == STANZA_BF16 ? launch_igemm_bf16_classes(P, n, st) : launch_igemm_classes(P, n, st);
}

static int conv_fwd_any(const stanza_conv_desc *desc, const void *x, const void *w, const float *bias, const void *res, bool want_res, void *y,
                        void *ws, size_t ws_bytes, void *stream, float *stats = nullptr)
{
    if (!desc) return STANZA_ENULL;
    GemmParams p{};
    int rc = conv_geometry(desc, &p.g);
    if (rc) return rc;
    if ((rc = check_dtype(desc))) return rc;
    const bool has_bias = desc->flags & STANZA_CONV_BIAS;
    if (!x || !w || !y || (has_bias && !bias) || (want_res && !res)) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(bias) || !aligned16(ws) || !aligned16(res)) return STANZA_EALIGN;
    FwdC4Params f4;
    if (desc->dtype == STANZA_F32 && !want_res && !stats && plan_fwd_c4(p.g, &f4)) {
        f4.x = (const float *)x;
        f4.w = (const float *)w;
        f4.bias = has_bias ? bias : nullptr;
        f4.y = (float *)y;
        const dim3 grid((unsigned)(cdiv(f4.tiles * f4.slices, 8) * 8));
        if (desc->flags & STANZA_CONV_RELU) hipLaunchKernelGGL(fwd_c4_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, f4);
        else hipLaunchKernelGGL(fwd_c4_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, f4);
        return launch_status();
    }
    p.a = (const float *)x;
    p.b = (const float *)w;
    p.out = (float *)y;
    p.bias = bias;
    p.res = (const float *)res;
    p.M = p.g.N * p.g.Ho * p.g.Wo;
    p.Nn = p.g.K;
    p.Kd = p.g.R * p.g.S * p.g.C;
    p.flags = (has_bias ? EPI_BIAS : 0u) | ((desc->flags & STANZA_CONV_RELU) ? EPI_RELU : 0u) | (want_res ? EPI_RESIDUAL : 0u) |
              (stats ? EPI_STATS : 0u);
    p.stats = stats;
    return launch_any(desc, MODE_FWD, p, 1, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" size_t stanza_conv_stats_bytes(const stanza_conv_desc *desc)
{
    ConvGeo g;
    if (!desc || conv_geometry(desc, &g) || desc->dtype != STANZA_F32 || g.K % 4 != 0 || (desc->flags & STANZA_CONV_RELU)) return 0;
    return round256(igemm_stats_floats(g.N * g.Ho * g.Wo, g.K, g.R * g.S * g.C) * sizeof(float));
}

extern "C" int stanza_conv_fwd_stats(const stanza_conv_desc *desc, const void *x, const void *w, const float *bias, void *y, void *stats,
                                     size_t stats_bytes, void *ws, size_t ws_bytes, void *stream)
{
    if (!desc) return STANZA_ENULL;
    const size_t need = stanza_conv_stats_bytes(desc);
    if (need == 0) {
        ConvGeo g;
        const int rc = conv_geometry(desc, &g);
        return rc ? rc : STANZA_EUNSUPPORTED;       // float32, output channels a multiple of 4, no fused ReLU
    }
    if (!stats) return STANZA_ENULL;
    if (!aligned16(stats)) return STANZA_EALIGN;
    if (stats_bytes < need) return STANZA_EWORKSPACE;
    return conv_fwd_any(desc, x, w, bias, nullptr, false, y, ws, ws_bytes, stream, (float *)stats);
}

extern "C" int stanza_conv_fwd(const stanza_conv_desc *desc, const void *x, const void *w, const float *bias, void *y,
                               void *ws, size_t ws_bytes, void *stream)
{
    return conv_fwd_any(desc, x, w, bias, nullptr, false, y, ws, ws_bytes, stream);
}

extern "C" int stanza_conv_fwd_res(const stanza_conv_desc *desc, const void *x, const void *w, const float *bias, const void *res,
                                   void *y, void *ws, size_t ws_bytes, void *stream)
{
    return conv_fwd_any(desc, x, w, bias, res, true, y, ws, ws_bytes, stream);
}

extern "C" int stanza_conv_bwd_data(const stanza_conv_desc *desc, const void *dy, const void *y, const void *w,
                                    const void *x_mask, void *dx, void *ws, size_t ws_bytes, void *stream)
{
    if (!desc) return STANZA_ENULL;
    GemmParams p{};
    int rc = conv_geometry(desc, &p.g);
    if (rc) return rc;
    if ((rc = check_dtype(desc))) return rc;
    if (!dy || !w || !dx) return STANZA_ENULL;
    if (!aligned16(dy) || !aligned16(w) || !aligned16(dx) || !aligned16(y) || !aligned16(x_mask) || !aligned16(ws)) return STANZA_EALIGN;
    p.a = (const float *)dy;
    p.amask = (desc->flags & STANZA_CONV_RELU) ? (const float *)y : nullptr;
    p.b = (const float *)w;
    p.out = (float *)dx;
    p.xmask = (const float *)x_mask;
    p.Nn = p.g.C;
    p.flags = ((desc->flags & STANZA_CONV_ACCUM) ? EPI_ACCUM : 0u) | (x_mask ? EPI_XMASK : 0u) | (p.amask ? LOAD_AMASK : 0u);
    const ConvGeo &g = p.g;
    if (g.sh == 1 && g.sw == 1) {
        p.M = g.N * g.H * g.W;
        p.Kd = g.R * g.S * g.K;
        return launch_any(desc, MODE_BWD_DATA, p, 1, ws, ws_bytes, (hipStream_t)stream);
    }
    // Strided layer: one launch per stride class (a, b) = ((h + pad_h) mod stride_h, (w + pad_w) mod stride_w) of the input
    // pixels.  A pixel of class (a, b) only receives the taps r = a, a + stride_h, ..., s = b, b + stride_w, ...; gathering them
    // class by class multiplies no zeros (a 3x3 stride-2 layer has classes of 4, 2, 2 and 1 taps instead of 9 taps of which
    // three quarters miss).  The classes write disjoint pixels and together cover dx.
    // Up to MAX_CLASSES classes go out as one launch.
    GemmClasses P;
    int n = 0;
    for (int a = 0; a < g.sh; ++a) {
        for (int b = 0; b < g.sw; ++b) {
            GemmParams q = p;
            StrideClass &c = q.sub;
            c.h0 = ((a - g.ph) % g.sh + g.sh) % g.sh;
            c.w0 = ((b - g.pw) % g.sw + g.sw) % g.sw;
            if (c.h0 >= g.H || c.w0 >= g.W) continue;
            c.Hc = (g.H - c.h0 + g.sh - 1) / g.sh;
            c.Wc = (g.W - c.w0 + g.sw - 1) / g.sw;
            c.pa = (c.h0 + g.ph - a) / g.sh;
            c.qb = (c.w0 + g.pw - b) / g.sw;
            c.r0 = a;
            c.s0 = b;
            c.Rc = a < g.R ? (g.R - a + g.sh - 1) / g.sh : 0;
            c.Sc = b < g.S ? (g.S - b + g.sw - 1) / g.sw : 0;
            if (c.Rc == 0 || c.Sc == 0) c.Rc = c.Sc = 0;
            q.M = g.N * c.Hc * c.Wc;
            q.Kd = c.Rc * c.Sc * g.K;
            q.flags |= OUT_STRIDED;
            P.q[n++] = q;
            if (n == MAX_CLASSES) {
                if ((rc = launch_classes(desc, P, n, (hipStream_t)stream))) return rc;
                n = 0;
            }
        }
    }
    if (n > 0 && (rc = launch_classes(desc, P, n, (hipStream_t)stream))) return rc;
    return STANZA_OK;
}

extern "C" int stanza_conv_bwd_weight(const stanza_conv_desc *desc, const void *x, const void *dy, const void *y, float *dw,
                                      float *dbias, void *ws, size_t ws_bytes, void *stream)
{
    if (!desc) return STANZA_ENULL;
    GemmParams p{};
    int rc = conv_geometry(desc, &p.g);
    if (rc) return rc;
    if ((rc = check_dtype(desc))) return rc;
    const bool want_bias = desc->flags & STANZA_CONV_BIAS;
    if (!x || !dy || !dw || (want_bias && !dbias)) return STANZA_ENULL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dw) || !aligned16(y) || !aligned16(ws)) return STANZA_EALIGN;
    const WgradPlan pl = plan_wgrad(p.g, want_bias, desc->dtype == STANZA_BF16 ? BKH : BK, (desc->flags & STANZA_CONV_NINE_TAP) != 0);
    if (pl.bytes > 0 && (!ws || ws_bytes < pl.bytes)) return ws ? STANZA_EWORKSPACE : STANZA_ENULL;
    hipStream_t st = (hipStream_t)stream;
    float *partial = (float *)ws;
    float *dbscratch = (float *)((char *)ws + round256(pl.partial_floats * 4));
    if (pl.taps == 2) {
        TapsC4Params tp;
        if (!plan_wgrad_taps_c4(p.g, &tp)) return STANZA_EINVAL;
        tp.dy = (const float *)dy;
        tp.amask = (desc->flags & STANZA_CONV_RELU) ? (const float *)y : nullptr;
        tp.x = (const float *)x;
        tp.out = pl.splits > 1 ? partial : dw;
        tp.dbias = want_bias ? (pl.splits > 1 ? dbscratch : dbias) : nullptr;
        const dim3 grid((unsigned)(cdiv(tp.tiles * tp.slices, 8) * 8));
        if (tp.amask) hipLaunchKernelGGL(wgrad_taps_c4_kernel<true>, grid, dim3(256), 0, st, tp);
        else hipLaunchKernelGGL(wgrad_taps_c4_kernel<false>, grid, dim3(256), 0, st, tp);
        if ((rc = launch_status())) return rc;
        if (pl.splits > 1)
            rc = launch_split_reduce(partial, pl.splits, (size_t)p.g.K * 36, dw, dbscratch, want_bias ? (size_t)p.g.K : 0, dbias, st);
        return rc;
    }
    if (pl.taps) {
        TapsParams tp;
        if (!plan_wgrad_taps(p.g, &tp)) return STANZA_EINVAL;
        tp.dy = (const float *)dy;
        tp.amask = (desc->flags & STANZA_CONV_RELU) ? (const float *)y : nullptr;
        tp.x = (const float *)x;
        tp.out = pl.splits > 1 ? partial : dw;
        tp.dbias = want_bias ? (pl.splits > 1 ? dbscratch : dbias) : nullptr;
        const dim3 grid((unsigned)(cdiv(tp.tiles * tp.slices, 8) * 8));
        launch_wgrad_taps(tp, grid, st);
        if ((rc = launch_status())) return rc;
        if (pl.splits > 1)
            rc = launch_split_reduce(partial, pl.splits, (size_t)p.g.K * 9 * p.g.C, dw, dbscratch, want_bias ? (size_t)p.g.K : 0, dbias, st);
        return rc;
    }
    p.a = (const float *)dy;
    p.amask = (desc->flags & STANZA_CONV_RELU) ? (const float *)y : nullptr;
    p.b = (const float *)x;
    p.M = p.g.K;
    p.Nn = p.g.R * p.g.S * p.g.C;
    p.Kd = p.g.N * p.g.Ho * p.g.Wo;
    p.chunks_per_split = pl.chunks_per_split;
    p.flags = (p.amask ? LOAD_AMASK : 0u) | (want_bias ? EPI_DBIAS : 0u);
    p.out = pl.splits > 1 ? partial : dw;
    p.dbias = pl.splits > 1 ? dbscratch : dbias;
    p.dbias_stride = p.g.K;
    rc = launch_any(desc, MODE_BWD_WEIGHT, p, pl.splits, nullptr, 0, st);
    if (rc) return rc;
    if (pl.splits > 1)
        rc = launch_split_reduce(partial, pl.splits, (size_t)p.M * p.Nn, dw, dbscratch, want_bias ? (size_t)p.g.K : 0, dbias, st);
    return rc;
}
