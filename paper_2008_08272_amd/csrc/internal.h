// Internal launch interface between the C-ABI layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "contraction.h"

namespace onnxhip {

// Workgroup tiles of the contraction kernel (rows x columns x K step, wavefront grid):
//   TILE_64   64 x  64 x 16 (K < 1024) or x 32, 2x2 wavefronts  -- small problems
//   TILE_128 128 x 128 x 16, 4x2 wavefronts  -- the general case
//   TILE_256 256 x 256 x 16, 4x4 wavefronts  -- large products, one workgroup per CU
enum TileShape { TILE_64 = 0, TILE_128 = 1, TILE_256 = 2, TILE_COUNT };

// Picks the tile with the lowest estimated time for an M x N output repeated nz times.
int pick_tile(int64_t M, int64_t N, int64_t nz);

// Scratch memory for split-K partial tiles, handed over by the caller through onnx_set_workspace.
struct Workspace {
    float* partial;
    int64_t partial_floats;
};
const Workspace& workspace();

// Stores `message` as the calling thread's last error (what onnx_last_error returns) and hands
// `status` back; for the entry points that live outside the main C-ABI translation unit.
int report_error(int status, const char* message);

// How many ways to split the K walk of `tiles` workgroup tiles of `tile_elems` outputs and `nk`
// K steps each, so that the 256 CUs are evenly loaded and hold enough workgroups to overlap each
// other's waits; 1 when the workspace cannot hold it.
// `overhead` is a workgroup's fixed cost (prologue, epilogue) in units of one K step.
int pick_split(int64_t tiles, int nk, int64_t tile_elems, double overhead);

// Fills tiles_m / tiles_n of `p` for the chosen tile and enqueues the kernel instance for
// (akind, bkind, vec).  nz = number of z-slices (grid.z).
hipError_t launch_contraction(ContractionParams& p, int akind, int bkind, int vec, int tile,
                              int nz, hipStream_t stream);

// Convolution through an LDS-resident input patch (conv_window.h).  `p` must be filled as for
// the IM2COL contraction (A = filters, B = input, ic geometry, K = Cg*kH*kW).  Returns false
// when no instance fits this shape (the caller then uses the generic path); otherwise
// enqueues the kernel and stores the launch status in *status.
bool launch_conv_window(ContractionParams& p, int kH, int kW, int OH, int OW, int Cg, int nz,
                        hipStream_t stream, hipError_t* status);

struct WindowGeom {
    int N, C, H, W, OH, OW;
    int kH, kW, sH, sW, pT, pL, pB, pR, dH, dW;
};

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

}  // namespace onnxhip
