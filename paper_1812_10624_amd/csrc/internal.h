// Host-side helpers shared by the translation units of libstanza (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/stanza.h"
#include "igemm.h"
#include "wgrad_taps.h"

namespace stanza {

inline int cdiv(int a, int b) { return (a + b - 1) / b; }
inline int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t b) { return (b + 255) & ~size_t(255); }

inline int hip_status(hipError_t e) { return e == hipSuccess ? STANZA_OK : STANZA_EHIP; }
inline int launch_status() { return hip_status(hipGetLastError()); }

// Validates a conv descriptor and fills the kernel-side geometry.
int conv_geometry(const stanza_conv_desc *d, ConvGeo *g);

// How the filter-gradient reduction is cut into workgroups; the same plan sizes the workspace and drives
// the launch, so the two can never disagree.
struct WgradPlan {
    int taps;              // float32 3x3 stride-1 pad-1 layers: 1 = the kernel that keeps all nine taps in one workgroup, 2 = its
                           // image-layer form for 4 input channels (wgrad_taps.h); 0 = the implicit-GEMM engine
    int splits;            // reduction slices (blockIdx.y); for taps: pixel slices
    int chunks_per_split;  // BK-deep stages per slice; for taps: stages per slice
    size_t partial_floats; // splits * K * R*S*C when splits > 1, else 0
    size_t db_floats;      // splits * K bias-gradient partials when splits > 1 and a bias gradient is wanted
    size_t bytes;
};
WgradPlan plan_wgrad(const ConvGeo &g, bool want_bias, int bk, bool force_taps);   // bk: reduction depth of one LDS stage; force_taps:
                                                                                    // the nine-tap kernel wherever it can run
// Stage geometry and work split of the nine-tap filter-gradient kernel; false when the layer is not one it handles.
bool plan_wgrad_taps(const ConvGeo &g, TapsParams *tp);
bool plan_wgrad_taps_c4(const ConvGeo &g, TapsC4Params *tp);
bool plan_fwd_c4(const ConvGeo &g, FwdC4Params *fp);

// Launch the implicit GEMM in `mode` over p (M, Nn, Kd, pointers and flags already set); picks the tile shape and fills
// the tile counts.  bw_splits: reduction slices of every tile, MODE_BWD_WEIGHT only (1 otherwise).
// FWD / BWD_DATA: when `partial` holds at least igemm_partial_floats(mode, M, Nn, Kd) floats, the tiles of the last,
// partly filled round of workgroups (or all tiles, when there are few) are cut into reduction slices whose raw sums go to
// `partial`, and a second kernel adds the slices in slice order and applies the epilogue; with partial == nullptr
// every tile is computed whole by one workgroup.  The cut depends on the GEMM extents alone.
int launch_igemm(int mode, GemmParams &p, int bw_splits, float *partial, size_t partial_floats, hipStream_t st);
size_t igemm_partial_floats(int mode, int M, int Nn, int Kd);
int launch_igemm_bf16(int mode, GemmParams &p, int splits, hipStream_t st);

// out[i] = sum_s partial[s*numel + i] in a fixed order (1, 4 or 16 interleaved groups of slices, each ascending, then the
// groups in order: the grouping depends on the sizes alone); likewise out2 from partial2 (numel2 may be 0).
int launch_split_reduce(const float *partial, int splits, size_t numel, float *out, const float *partial2, size_t numel2, float *out2,
                        hipStream_t st);

// Column sums of a [rows][cols] matrix (optionally gated by mask > 0) in two fixed-order passes.
// scratch: blocks*cols floats.  With sgd_p != nullptr the sums are used as the gradient of a fused
// momentum-SGD update of sgd_p / sgd_v instead of being written to out.
int colsum_blocks(int rows);
int launch_colsum(const float *a, const float *mask, int rows, int cols, float *scratch, int blocks, float *out,
                  float *sgd_p, float *sgd_v, float lr, float mom, float wd, hipStream_t st);

}  // namespace stanza
