// Layout passes ahead of a 1x1 convolution on 16-bit tensors, so that shapes the tuned contraction
// kernel (gemm_lp.h) cannot read directly still run through it instead of through the general kernel:
//   * a strided 1x1 convolution reads every sH-th row and sW-th column of the input: the positions
//     it reads are copied into a dense [N][C][OH][OW] tensor, of which the convolution is pointwise;
//   * a pointwise convolution whose planes are not a multiple of 4 positions long (7 x 7 = 49) has
//     no aligned chunks of columns to load: its input is rewritten as [N][H*W][C], a K-contiguous
//     B matrix with one row per (image, position), the layout the kernel reads best.
// Both copies live in the caller's workspace for the duration of the call and move a small fraction
// of what the convolution itself moves.
#include "gemm_lp.h"
#include "internal.h"

namespace onnxhip {

namespace {

// Xs[plane][oh][ow] = X[plane][oh * sH][ow * sW]
__global__ __launch_bounds__(256) void lp_subsample_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Xs, uint32_t total,
                                                          FastDiv OW, FastDiv OH, int HW, int W, int sH, int sW) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    uint32_t q, ow, plane, oh;
    OW.divmod(idx, q, ow);
    OH.divmod(q, plane, oh);
    Xs[idx] = X[(int64_t)plane * HW + (int)oh * sH * W + (int)ow * sW];
}

// Xt[n][p][c] = X[n][c][p] for one image per blockIdx.z, 64 x 64 tiles through LDS: reads run
// along p, writes along c.
__global__ __launch_bounds__(256) void lp_planes_to_rows_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Xt, int C, int P) {
    __shared__ uint16_t tile[64][64 + 2];
    const int64_t image = (int64_t)blockIdx.z * C * P;
    const int c0 = blockIdx.y * 64, p0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int c = c0 + ty * 16 + r, p = p0 + tx;
        tile[ty * 16 + r][tx] = (c < C && p < P) ? X[image + (int64_t)c * P + p] : (uint16_t)0;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int p = p0 + ty * 16 + r, c = c0 + tx;
        if (p < P && c < C) Xt[image + (int64_t)p * C + c] = tile[tx][ty * 16 + r];
    }
}

}  // namespace

hipError_t launch_lp_subsample(const void* X, void* Xs, int64_t planes, int H, int W, int OH, int OW, int sH, int sW,
                               hipStream_t stream) {
    const int64_t total = planes * OH * OW;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(lp_subsample_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const uint16_t*>(X), static_cast<uint16_t*>(Xs), (uint32_t)total, FastDiv::make((uint32_t)OW),
                       FastDiv::make((uint32_t)OH), H * W, W, sH, sW);
    return hipGetLastError();
}

hipError_t launch_lp_planes_to_rows(const void* X, void* Xt, int N, int C, int P, hipStream_t stream) {
    if (N > 65535 || (C + 63) / 64 > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(lp_planes_to_rows_kernel, dim3((unsigned)((P + 63) / 64), (unsigned)((C + 63) / 64), (unsigned)N), dim3(256), 0,
                       stream, static_cast<const uint16_t*>(X), static_cast<uint16_t*>(Xt), C, P);
    return hipGetLastError();
}

}  // namespace onnxhip
