// Internal launch interface between the C-ABI layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "contraction.h"

namespace onnxhip {

// Workgroup tiles of the contraction kernel (rows x columns x K step, wavefront grid):
//   TILE_64          64 x  64 x 16 (K < 512) or x 32, 2x2 wavefronts  -- outputs with many tiles
//   TILE_64_SLICED   64 x  64 x 32, 2x2 wavefronts x 2 K slices      -- few tiles, long K
//   TILE_128        128 x 128 x 16, 4x4 wavefronts  -- outputs of about 256 or 512 such tiles
//   TILE_256        256 x 256 x 16, 4x4 wavefronts  -- large products, one workgroup per CU
//   TILE_32_SLICED   32 x  32 x 64, 1 wavefront x 4 K slices          -- very few outputs (batch 1), long K
enum TileShape { TILE_64 = 0, TILE_64_SLICED = 1, TILE_128 = 2, TILE_256 = 3, TILE_32_SLICED = 4, TILE_COUNT };

// Picks the tile with the lowest estimated time for an M x N x K product repeated nz times.
// `narrow_ok`: the operand loaders of this call exist for the 32-wide tile (all but the gather loader).
int pick_tile(int64_t M, int64_t N, int64_t K, int64_t nz, bool narrow_ok = true);

// Scratch memory for split-K partial tiles: the buffer handed over through onnx_set_workspace,
// or the library's own fixed array for the entry point that may not allocate.  Every launcher
// receives the one its call uses as an argument.
struct Workspace {
    float* partial;
    int64_t partial_floats;
};
// A consistent copy of what onnx_set_workspace last stored.
Workspace workspace();

// Stores `message` as the calling thread's last error (what onnx_last_error returns) and hands
// `status` back.
int report_error(int status, const char* message);
// printf-style form of the same.
int fail_with(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// byte ranges [a, a+na) and [b, b+nb) intersect
inline bool overlaps(const void* a, int64_t na, const void* b, int64_t nb) {
    if (!a || !b || na <= 0 || nb <= 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

// What the calling thread's most recent contraction / LDS-patch / 16-bit Gemm launch was: the
// kernel family and the template instance.  onnx_last_launch formats it; the tests use it to
// show that a case reaches the instance it is meant to cover.
struct LaunchRecord {
    const char* family;      // "contraction", "conv_window", "gemm_lp"
    int bm, bn, bk, wm, wn, ks;
    int akind, bkind, avec, bvec;
    int npb;                 // conv_window: patch passes; gemm_lp: 1 = fp16, 2 = bf16, +2 when Y is 16-bit
    int ksplit, tail_tiles, tail_split;
};
void record_launch(const LaunchRecord& r);

// How many ways to split the K walk of `tiles` workgroup tiles of `tile_elems` outputs and `nk`
// K steps each, so that the 256 CUs are evenly loaded and hold enough workgroups to overlap each
// other's waits; 1 when the workspace cannot hold it.
// `overhead` is a workgroup's fixed cost (prologue, epilogue) in units of one K step.
int pick_split(int64_t tiles, int nk, int64_t tile_elems, double overhead, const Workspace& ws);

// Fills tiles_m / tiles_n of `p` for the chosen tile and enqueues the kernel instance for
// (akind, bkind) with 16-byte (vec 4) or 4-byte (vec 1) global loads per operand.
// nz = number of z-slices (grid.z).
hipError_t launch_contraction(ContractionParams& p, int akind, int bkind, int avec, int bvec, int tile,
                              int nz, const Workspace& ws, hipStream_t stream);

// Contraction on 16-bit operands (in_type: 1 = IEEE half, 2 = bfloat16; out_type: 0 = fp32, else
// in_type) in any operand layout (lp_generic.hip): akind KC / RC, bkind KC / RC / IM2COL.  `p` is
// filled as for launch_contraction, with strides and offsets counted in elements.
hipError_t launch_lp_generic(ContractionParams& p, int akind, int bkind, int nz, int in_type, int out_type,
                             hipStream_t stream);

// The tuned 16-bit kernel (gemm_lp.h): A K-contiguous, B K-contiguous or row-contiguous, wide
// loads.  lp_tuned_fits returns 0 when `p` (filled as for launch_lp_generic) does not meet its
// alignment and 32-bit-offset conditions, else the chunk width for B (8, or 4 for a
// row-contiguous B whose rows are only 8-byte aligned) to pass on to launch_lp_tuned.  `ws`: where
// the shares of a split K range may be parked (outputs with few tiles), or {nullptr, 0}.
int lp_tuned_fits(const ContractionParams& p, int akind, int bkind, int nz);
hipError_t launch_lp_tuned(ContractionParams& p, int bkind, int bvec, int nz, int in_type, int out_type, const Workspace& ws,
                           hipStream_t stream);

// Convolution through an LDS-resident input patch (conv_window.h).  `p` must be filled as for
// the IM2COL contraction (A = filters, B = input, ic geometry, K = Cg*kH*kW).  Returns false
// when no instance fits this shape (the caller then uses the generic path); otherwise
// enqueues the kernel and stores the launch status in *status.
bool launch_conv_window(ContractionParams& p, int kH, int kW, int OH, int OW, int Cg, int nz,
                        const Workspace& ws, hipStream_t stream, hipError_t* status);

// The same for 16-bit tensors (conv_window_lp.hip): 3x3 windows, input channels per group a multiple
// of 16, and either a workspace that holds a rewritten copy of the filter bank (p.M * nz * Cg * 9
// 16-bit values) or p.A already rewritten by launch_lp_filter_taps (filters_in_tap_order; 16-byte
// aligned).  in_type / out_type as for launch_lp_generic.
bool launch_conv_window_lp(ContractionParams& p, int kH, int kW, int OH, int OW, int Cg, int nz, int in_type, int out_type,
                           bool filters_in_tap_order, const Workspace& ws, hipStream_t stream, hipError_t* status);
// W [rows][Cg][3][3] -> packed [rows][Cg/16][9][16] (16-bit values; Cg a multiple of 16).
hipError_t launch_lp_filter_taps(const void* W, void* packed, int64_t rows, int Cg, hipStream_t stream);

// Layout passes ahead of a 1x1 convolution on 16-bit tensors (lp_layout.hip): the positions a strided
// convolution reads, copied into a dense [planes][OH][OW] tensor, and [N][C][P] rewritten as [N][P][C].
hipError_t launch_lp_subsample(const void* X, void* Xs, int64_t planes, int H, int W, int OH, int OW, int sH, int sW,
                               hipStream_t stream);
hipError_t launch_lp_planes_to_rows(const void* X, void* Xt, int N, int C, int P, hipStream_t stream);

struct WindowGeom {
    int N, C, H, W, OH, OW;
    int kH, kW, sH, sW, pT, pL, pB, pR, dH, dW;
};

// Convolution with the filters held in registers by persistent workgroups (conv_resident.hip):
// few input channels, large window (the 7x7 stride-2 stem of ResNet50).  group must be 1.
// Returns false when no instance fits this shape; otherwise enqueues and stores the launch
// status in *status.
bool launch_conv_resident(const float* X, const float* W, const float* B, const float* residual, float* Y,
                          const WindowGeom& g, int M, int Cg, int relu, hipStream_t stream, hipError_t* status);

// The 7x7 stride-2 convolution on 3 channels into 64 feature maps with pads of 3 (ResNet50's stem) on 16-bit tensors
// (conv_stem_lp.hip).  Returns false for every other shape (the caller then uses the general kernel); otherwise
// enqueues the kernel and stores the launch status in *status.  in_type / out_type as for launch_lp_generic.
bool launch_conv_stem_lp(const void* X, const void* W, const float* B, void* Y, const WindowGeom& g, int M, int Cg, int group,
                         bool has_residual, int relu, int in_type, int out_type, hipStream_t stream, hipError_t* status);

// Direct (one thread per output) convolution for shapes the matrix cores cannot use well:
// depthwise and other tiny-K / tiny-M groups.
hipError_t launch_conv_direct(const float* X, const float* W, const float* B, const float* residual,
                              float* Y, const WindowGeom& g, int M, int Cg, int group, int relu,
                              hipStream_t stream);
hipError_t launch_maxpool(const float* X, float* Y, int64_t* indices, const WindowGeom& g,
                          hipStream_t stream);
hipError_t launch_avgpool(const float* X, float* Y, const WindowGeom& g, int count_include_pad,
                          hipStream_t stream);
hipError_t launch_global_avgpool(const float* X, float* Y, int64_t planes, int HW, hipStream_t stream);
// The pools on 16-bit tensors (window_lp.hip); `type` is ONNX_F16 / ONNX_BF16, N*C*OH*OW < 2^31.
hipError_t launch_maxpool_lp(const void* X, void* Y, const WindowGeom& g, int type, hipStream_t stream);
hipError_t launch_avgpool_lp(const void* X, void* Y, const WindowGeom& g, int count_include_pad, int type, hipStream_t stream);
hipError_t launch_global_avgpool_lp(const void* X, void* Y, int64_t planes, int HW, int type, hipStream_t stream);
hipError_t launch_leakyrelu_lp(const void* X, void* Y, int64_t count, float alpha, int type, hipStream_t stream);

}  // namespace onnxhip
