// Sliding-window kernels that do not use the matrix cores: direct convolution for depthwise /
// tiny groups, MaxPool, AveragePool and GlobalAveragePool (Section 4.1 of the paper lists
// convolution and pooling among the supported operators).  All are bandwidth- or
// latency-bound: one thread per output element, lanes running along the contiguous output
// width so that loads and stores of a wavefront fall into few cache lines.
#include "internal.h"

namespace onnxhip {

struct OutIndex {
    FastDiv ow, oh, c;      // divisors OW, OH, and channels (M for conv, C for pools)
};

__device__ inline void split_output(const OutIndex& d, uint32_t idx, uint32_t& n, uint32_t& c,
                                    uint32_t& oh, uint32_t& ow) {
    uint32_t t;
    d.ow.divmod(idx, t, ow);
    d.oh.divmod(t, t, oh);
    d.c.divmod(t, n, c);
}

// Outputs are numbered below 2^31 per launch; larger tensors are covered by grid.y chunks of
// whole images so that 32-bit index arithmetic stays valid inside a chunk.
__global__ __launch_bounds__(256) void conv_direct_kernel(const float* __restrict__ X,
                                                          const float* __restrict__ Wt,
                                                          const float* __restrict__ B,
                                                          const float* __restrict__ residual,
                                                          float* __restrict__ Y, WindowGeom g, int M,
                                                          int Cg, int Mg, int relu, OutIndex d,
                                                          uint32_t per_image, int images_per_chunk) {
    const int img0 = blockIdx.y * images_per_chunk;
    const int nimg = min(images_per_chunk, g.N - img0);
    const uint32_t total = per_image * (uint32_t)nimg;
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    uint32_t n, m, oh, ow;
    split_output(d, idx, n, m, oh, ow);
    const int grp = (int)m / Mg;
    const int ih0 = (int)oh * g.sH - g.pT, iw0 = (int)ow * g.sW - g.pL;
    const float* xn = X + ((int64_t)(img0 + n) * g.C + (int64_t)grp * Cg) * g.H * g.W;
    const float* wm = Wt + (int64_t)m * Cg * g.kH * g.kW;
    float acc = 0.f;
    for (int c = 0; c < Cg; ++c) {
        const float* xc = xn + (int64_t)c * g.H * g.W;
        const float* wc = wm + c * g.kH * g.kW;
        for (int kh = 0; kh < g.kH; ++kh) {
            const int ih = ih0 + kh * g.dH;
            if (ih < 0 || ih >= g.H) continue;
            for (int kw = 0; kw < g.kW; ++kw) {
                const int iw = iw0 + kw * g.dW;
                if (iw < 0 || iw >= g.W) continue;
                acc = fmaf(xc[ih * g.W + iw], wc[kh * g.kW + kw], acc);
            }
        }
    }
    const int64_t o = (int64_t)img0 * per_image + idx;
    if (B) acc += B[m];
    if (residual) acc += residual[o];
    if (relu) acc = acc > 0.f ? acc : 0.f;
    Y[o] = acc;
}

__global__ __launch_bounds__(256) void maxpool_kernel(const float* __restrict__ X,
                                                      float* __restrict__ Y,
                                                      int64_t* __restrict__ indices, WindowGeom g,
                                                      OutIndex d, uint32_t per_image,
                                                      int images_per_chunk) {
    const int img0 = blockIdx.y * images_per_chunk;
    const int nimg = min(images_per_chunk, g.N - img0);
    const uint32_t total = per_image * (uint32_t)nimg;
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    uint32_t n, c, oh, ow;
    split_output(d, idx, n, c, oh, ow);
    const int ih0 = (int)oh * g.sH - g.pT, iw0 = (int)ow * g.sW - g.pL;
    const int64_t plane = ((int64_t)(img0 + n) * g.C + c) * g.H * g.W;
    const float* xc = X + plane;
    // scan kh outer, kw inner; a later tap wins only when strictly greater (first maximum)
    bool found = false;
    float best = 0.f;
    int best_off = 0;
    for (int kh = 0; kh < g.kH; ++kh) {
        const int ih = ih0 + kh * g.dH;
        if (ih < 0 || ih >= g.H) continue;
        for (int kw = 0; kw < g.kW; ++kw) {
            const int iw = iw0 + kw * g.dW;
            if (iw < 0 || iw >= g.W) continue;
            const float v = xc[ih * g.W + iw];
            if (!found || v > best) { best = v; best_off = ih * g.W + iw; found = true; }
        }
    }
    const int64_t o = (int64_t)img0 * per_image + idx;
    Y[o] = best;
    if (indices) indices[o] = plane + best_off;
}

__global__ __launch_bounds__(256) void avgpool_kernel(const float* __restrict__ X,
                                                      float* __restrict__ Y, WindowGeom g,
                                                      int count_include_pad, OutIndex d,
                                                      uint32_t per_image, int images_per_chunk) {
    const int img0 = blockIdx.y * images_per_chunk;
    const int nimg = min(images_per_chunk, g.N - img0);
    const uint32_t total = per_image * (uint32_t)nimg;
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    uint32_t n, c, oh, ow;
    split_output(d, idx, n, c, oh, ow);
    const int ih0 = (int)oh * g.sH - g.pT, iw0 = (int)ow * g.sW - g.pL;
    const float* xc = X + ((int64_t)(img0 + n) * g.C + c) * g.H * g.W;
    float acc = 0.f;
    int cnt = 0, cnt_padded = 0;
    for (int kh = 0; kh < g.kH; ++kh) {
        const int ih = ih0 + kh;
        if (ih >= g.H + g.pB) continue;
        for (int kw = 0; kw < g.kW; ++kw) {
            const int iw = iw0 + kw;
            if (iw >= g.W + g.pR) continue;
            ++cnt_padded;
            if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
            acc += xc[ih * g.W + iw];
            ++cnt;
        }
    }
    const float div = (float)(count_include_pad ? cnt_padded : cnt);
    Y[(int64_t)img0 * per_image + idx] = acc / div;
}

// One wavefront per (n, c) plane: lanes stride over the H*W contiguous values, partial sums
// meet in a butterfly of cross-lane moves, lane 0 stores the mean.
__global__ __launch_bounds__(256) void global_avgpool_kernel(const float* __restrict__ X,
                                                             float* __restrict__ Y, int64_t planes,
                                                             int HW) {
    const int lane = threadIdx.x & 63;
    const int64_t plane = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (plane >= planes) return;
    const float* xp = X + plane * HW;
    float acc = 0.f;
    for (int i = lane; i < HW; i += 64) acc += xp[i];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) Y[plane] = acc / (float)HW;
}

static inline void chunking(int N, uint64_t per_image, int& images_per_chunk, unsigned& chunks,
                            unsigned& blocks) {
    const uint64_t limit = 1ull << 30;
    uint64_t ipc = per_image ? limit / per_image : (uint64_t)N;
    if (ipc < 1) ipc = 1;
    if (ipc > (uint64_t)N) ipc = (uint64_t)N;
    images_per_chunk = (int)ipc;
    chunks = (unsigned)((N + ipc - 1) / ipc);
    blocks = (unsigned)((per_image * ipc + 255) / 256);
}

static inline OutIndex out_index(int OW, int OH, int C) {
    OutIndex d;
    d.ow = FastDiv::make((uint32_t)OW);
    d.oh = FastDiv::make((uint32_t)OH);
    d.c = FastDiv::make((uint32_t)C);
    return d;
}

hipError_t launch_conv_direct(const float* X, const float* W, const float* B, const float* residual,
                              float* Y, const WindowGeom& g, int M, int Cg, int group, int relu,
                              hipStream_t stream) {
    const uint64_t per_image = (uint64_t)M * g.OH * g.OW;
    if (per_image >= (1ull << 30)) return hipErrorInvalidValue;
    int ipc; unsigned chunks, blocks;
    chunking(g.N, per_image, ipc, chunks, blocks);
    hipLaunchKernelGGL(conv_direct_kernel, dim3(blocks, chunks), dim3(256), 0, stream, X, W, B, residual,
                       Y, g, M, Cg, M / group, relu, out_index(g.OW, g.OH, M), (uint32_t)per_image, ipc);
    return hipGetLastError();
}

hipError_t launch_maxpool(const float* X, float* Y, int64_t* indices, const WindowGeom& g,
                          hipStream_t stream) {
    const uint64_t per_image = (uint64_t)g.C * g.OH * g.OW;
    if (per_image >= (1ull << 30)) return hipErrorInvalidValue;
    int ipc; unsigned chunks, blocks;
    chunking(g.N, per_image, ipc, chunks, blocks);
    hipLaunchKernelGGL(maxpool_kernel, dim3(blocks, chunks), dim3(256), 0, stream, X, Y, indices, g,
                       out_index(g.OW, g.OH, g.C), (uint32_t)per_image, ipc);
    return hipGetLastError();
}

hipError_t launch_avgpool(const float* X, float* Y, const WindowGeom& g, int count_include_pad,
                          hipStream_t stream) {
    const uint64_t per_image = (uint64_t)g.C * g.OH * g.OW;
    if (per_image >= (1ull << 30)) return hipErrorInvalidValue;
    int ipc; unsigned chunks, blocks;
    chunking(g.N, per_image, ipc, chunks, blocks);
    hipLaunchKernelGGL(avgpool_kernel, dim3(blocks, chunks), dim3(256), 0, stream, X, Y, g,
                       count_include_pad, out_index(g.OW, g.OH, g.C), (uint32_t)per_image, ipc);
    return hipGetLastError();
}

hipError_t launch_global_avgpool(const float* X, float* Y, int64_t planes, int HW, hipStream_t stream) {
    const int64_t blocks = (planes + 3) / 4;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(global_avgpool_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, X, Y, planes, HW);
    return hipGetLastError();
}

}  // namespace onnxhip
