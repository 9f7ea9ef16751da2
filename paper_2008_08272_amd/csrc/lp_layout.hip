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

// Xs[plane][oh][ow] = X[plane][oh * sH][ow * sW]: VEC neighbouring outputs of one row per thread, their loads requested
// together and stored as one word of 2 * VEC bytes (OW a multiple of VEC, Xs aligned to it).
template <int VEC>
__global__ __launch_bounds__(256) void lp_subsample_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Xs, uint32_t groups,
                                                          FastDiv OWG, FastDiv OH, int HW, int W, int sH, int sW) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= groups) return;
    uint32_t q, og, plane, oh;
    OWG.divmod(idx, q, og);                      // OWG divides by the groups per output row
    OH.divmod(q, plane, oh);
    const uint16_t* row = X + (int64_t)plane * HW + (int)oh * sH * W + (int)og * VEC * sW;
    uint32_t v[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] = row[k * sW];
    if constexpr (VEC == 4) {
        typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
        const uintx2 out = {v[0] | (v[1] << 16), v[2] | (v[3] << 16)};
        *reinterpret_cast<uintx2*>(Xs + (int64_t)idx * 4) = out;
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<uint32_t*>(Xs + (int64_t)idx * 2) = v[0] | (v[1] << 16);
    } else {
        Xs[idx] = (uint16_t)v[0];
    }
}

// Xt[n][p][c] = X[n][c][p] for one image per blockIdx.z, 64 x 64 tiles through LDS: reads run
// along p, writes along c.  All sixteen loads of a thread are requested before the first LDS store (an index past the
// tensor reads the last row / column instead; what it reads is never stored), and all LDS reads before the first store.
__global__ __launch_bounds__(256) void lp_planes_to_rows_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Xt, int C, int P) {
    __shared__ uint16_t tile[64][64 + 2];
    const int64_t image = (int64_t)blockIdx.z * C * P;
    const int c0 = blockIdx.y * 64, p0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    uint16_t v[16];
    {
        const int p = min(p0 + tx, P - 1);
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = X[image + (int64_t)min(c0 + ty * 16 + r, C - 1) * P + p];
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) tile[ty * 16 + r][tx] = v[r];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] = tile[tx][ty * 16 + r];
    const int c = c0 + tx;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int p = p0 + ty * 16 + r;
        if (p < P && c < C) Xt[image + (int64_t)p * C + c] = v[r];
    }
}

}  // namespace

hipError_t launch_lp_subsample(const void* X, void* Xs, int64_t planes, int H, int W, int OH, int OW, int sH, int sW,
                               hipStream_t stream) {
    const int64_t total = planes * OH * OW;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* xs = static_cast<uint16_t*>(Xs);
    const uintptr_t a = reinterpret_cast<uintptr_t>(Xs);
    const int vec = (OW % 4 == 0 && a % 8 == 0) ? 4 : (OW % 2 == 0 && a % 4 == 0) ? 2 : 1;
    const uint32_t groups = (uint32_t)(total / vec);
    const dim3 grid((groups + 255u) / 256u), block(256);
    const FastDiv owg = FastDiv::make((uint32_t)(OW / vec)), oh = FastDiv::make((uint32_t)OH);
    if (vec == 4) hipLaunchKernelGGL(lp_subsample_kernel<4>, grid, block, 0, stream, x, xs, groups, owg, oh, H * W, W, sH, sW);
    else if (vec == 2) hipLaunchKernelGGL(lp_subsample_kernel<2>, grid, block, 0, stream, x, xs, groups, owg, oh, H * W, W, sH, sW);
    else hipLaunchKernelGGL(lp_subsample_kernel<1>, grid, block, 0, stream, x, xs, groups, owg, oh, H * W, W, sH, sW);
    return hipGetLastError();
}

hipError_t launch_lp_planes_to_rows(const void* X, void* Xt, int N, int C, int P, hipStream_t stream) {
    if (N > 65535 || (C + 63) / 64 > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(lp_planes_to_rows_kernel, dim3((unsigned)((P + 63) / 64), (unsigned)((C + 63) / 64), (unsigned)N), dim3(256), 0,
                       stream, static_cast<const uint16_t*>(X), static_cast<uint16_t*>(Xt), C, P);
    return hipGetLastError();
}

}  // namespace onnxhip
