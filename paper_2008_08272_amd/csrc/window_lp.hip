// MaxPool / AveragePool / GlobalAveragePool and LeakyRelu on 16-bit tensors (IEEE half or bfloat16): what a
// network whose contractions run on 16-bit inputs (gemm_lp.h, conv_window_lp.hip) needs between
// them so that its activations never leave the 16-bit type.  Same ONNX semantics as the fp32
// pools (Section 4.1 of the paper lists pooling among the supported operators): the maximum is
// one of the inputs and is stored with its bits unchanged; an average is summed in fp32 in scan
// order, divided, and rounded to the type once.  Bandwidth-bound and small next to the
// convolutions: one thread per output element (one wavefront per plane for the global average).
#include "gemm_lp.h"
#include "internal.h"

namespace onnxhip {

namespace {

struct PoolIndex {
    FastDiv OW, OH;
};

template <int DT>
__global__ __launch_bounds__(256) void maxpool_lp_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, WindowGeom g,
                                                        PoolIndex d, uint32_t total) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    uint32_t q, ow, plane, oh;
    d.OW.divmod(idx, q, ow);
    d.OH.divmod(q, plane, oh);
    const int ih0 = (int)oh * g.sH - g.pT, iw0 = (int)ow * g.sW - g.pL;
    const uint16_t* xc = X + (int64_t)plane * g.H * g.W;
    // scan kh outer, kw inner; a later tap wins only when strictly greater (first maximum)
    bool found = false;
    float best = 0.f;
    uint16_t best_bits = 0;
    for (int kh = 0; kh < g.kH; ++kh) {
        const int ih = ih0 + kh * g.dH;
        if (ih < 0 || ih >= g.H) continue;
        for (int kw = 0; kw < g.kW; ++kw) {
            const int iw = iw0 + kw * g.dW;
            if (iw < 0 || iw >= g.W) continue;
            const uint16_t bits = xc[ih * g.W + iw];
            const float v = from_lp<DT>(bits);
            if (!found || v > best) { best = v; best_bits = bits; found = true; }
        }
    }
    Y[idx] = best_bits;
}

// MaxPool with 3 columns per window, horizontal stride 2 and left pad 1 (ResNet-50's pool behind the stem) on
// rows of even length: a thread computes the outputs (ow, ow + 1) for even ow.  Their windows cover the input
// columns 2*ow - 1 .. 2*ow + 3, which lie in three 4-byte aligned pairs starting at column 2*ow - 2: three loads
// per input row for two outputs instead of six 2-byte ones.  Same scan order and first-maximum rule as above.
template <int DT>
__global__ __launch_bounds__(256) void maxpool_lp_pairs_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, WindowGeom g,
                                                              PoolIndex d, uint32_t total_pairs) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;            // (plane, oh, pair of output columns)
    if (idx >= total_pairs) return;
    uint32_t q, op, plane, oh;
    d.OW.divmod(idx, q, op);                                         // d.OW divides by the pairs per output row
    d.OH.divmod(q, plane, oh);
    const int ow = 2 * (int)op;
    const int ih0 = (int)oh * g.sH - g.pT;
    const uint16_t* xc = X + (int64_t)plane * g.H * g.W;
    bool found[2] = {false, false};
    float best[2] = {0.f, 0.f};
    uint16_t best_bits[2] = {0, 0};
    auto offer = [&](int o, uint32_t bits) {
        const float v = from_lp<DT>(bits);
        if (!found[o] || v > best[o]) { best[o] = v; best_bits[o] = (uint16_t)bits; found[o] = true; }
    };
    for (int kh = 0; kh < g.kH; ++kh) {
        const int ih = ih0 + kh * g.dH;
        if (ih < 0 || ih >= g.H) continue;
        const uint32_t* row = reinterpret_cast<const uint32_t*>(xc + ih * g.W);      // W even, X 4-byte aligned
        const int c0 = 2 * ow - 2;                                                   // even; pairs at c0, c0 + 2, c0 + 4
        const uint32_t p0 = c0 >= 0 ? row[c0 >> 1] : 0u;
        const uint32_t p1 = row[(c0 + 2) >> 1];                                      // columns 2*ow, 2*ow + 1: always inside
        const uint32_t p2 = c0 + 4 < g.W ? row[(c0 + 4) >> 1] : 0u;
        // output ow: columns 2*ow - 1, 2*ow, 2*ow + 1; output ow + 1: columns 2*ow + 1, 2*ow + 2, 2*ow + 3
        if (c0 >= 0) offer(0, p0 >> 16);
        offer(0, p1 & 0xffffu);
        offer(0, p1 >> 16);
        offer(1, p1 >> 16);
        if (c0 + 4 < g.W) { offer(1, p2 & 0xffffu); offer(1, p2 >> 16); }
    }
    const int64_t o = ((int64_t)plane * g.OH + oh) * g.OW + ow;
    Y[o] = best_bits[0];
    if (ow + 1 < g.OW) Y[o + 1] = best_bits[1];
}

// The same windows on rows whose length is a multiple of 8 with exactly W / 2 outputs: a thread computes four
// neighbouring outputs of one output row from one 16-byte load per input row (columns 8c .. 8c + 7) and the
// column left of it (a 2-byte load that hits the cache line of the previous thread's load), and stores them as one
// 8-byte word.  Output 4c + j reads columns 8c + 2j - 1 .. 8c + 2j + 1; same scan order and
// first-maximum rule as above.
template <int DT>
__global__ __launch_bounds__(256) void maxpool_lp_quads_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, WindowGeom g,
                                                              PoolIndex d, uint32_t total_quads) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;            // (plane, oh, group of four output columns)
    if (idx >= total_quads) return;
    uint32_t q, c, plane, oh;
    d.OW.divmod(idx, q, c);                                          // d.OW divides by the groups per output row
    d.OH.divmod(q, plane, oh);
    const int ih0 = (int)oh * g.sH - g.pT;
    const uint16_t* xc = X + (int64_t)plane * g.H * g.W;
    bool found[4] = {false, false, false, false};
    float best[4] = {0.f, 0.f, 0.f, 0.f};
    uint32_t best_bits[4] = {0, 0, 0, 0};
    auto offer = [&](int o, uint32_t bits) {
        const float v = from_lp<DT>(bits);
        if (!found[o] || v > best[o]) { best[o] = v; best_bits[o] = bits; found[o] = true; }
    };
    // one input row's eight columns and the column left of them, in scan order
    auto offer_row = [&](const uintx4& v, uint32_t left) {
        if (c > 0) offer(0, left);
        uint32_t e[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) { e[2 * k] = v[k] & 0xffffu; e[2 * k + 1] = v[k] >> 16; }
        offer(0, e[0]);
        offer(0, e[1]);
#pragma unroll
        for (int j = 1; j < 4; ++j) {
            offer(j, e[2 * j - 1]);
            offer(j, e[2 * j]);
            offer(j, e[2 * j + 1]);
        }
    };
    // W a multiple of 8 and X 16-byte aligned: every load below is aligned and inside its row
    if (g.kH == 3) {
        // all six loads of the three rows requested before the first comparison (a row outside the image reads row 0
        // instead and is skipped afterwards)
        uintx4 v[3];
        uint32_t left[3];
        bool inside[3];
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const int ih = ih0 + kh * g.dH;
            inside[kh] = ih >= 0 && ih < g.H;
            const uint16_t* row = xc + (inside[kh] ? ih : 0) * g.W + 8 * (int)c;
            v[kh] = *reinterpret_cast<const uintx4*>(row);
            left[kh] = c > 0 ? row[-1] : 0u;
        }
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
            if (inside[kh]) offer_row(v[kh], left[kh]);
    } else {
        for (int kh = 0; kh < g.kH; ++kh) {
            const int ih = ih0 + kh * g.dH;
            if (ih < 0 || ih >= g.H) continue;
            const uint16_t* row = xc + ih * g.W + 8 * (int)c;
            offer_row(*reinterpret_cast<const uintx4*>(row), c > 0 ? row[-1] : 0u);
        }
    }
    typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
    const uintx2 out = {best_bits[0] | (best_bits[1] << 16), best_bits[2] | (best_bits[3] << 16)};
    *reinterpret_cast<uintx2*>(Y + ((int64_t)plane * g.OH + oh) * g.OW + 4 * (int)c) = out;
}

template <int DT>
__global__ __launch_bounds__(256) void avgpool_lp_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, WindowGeom g,
                                                        int count_include_pad, PoolIndex d, uint32_t total) {
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    uint32_t q, ow, plane, oh;
    d.OW.divmod(idx, q, ow);
    d.OH.divmod(q, plane, oh);
    const int ih0 = (int)oh * g.sH - g.pT, iw0 = (int)ow * g.sW - g.pL;
    const uint16_t* xc = X + (int64_t)plane * g.H * g.W;
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
            acc += from_lp<DT>(xc[ih * g.W + iw]);
            ++cnt;
        }
    }
    Y[idx] = to_lp<DT>(acc / (float)(count_include_pad ? cnt_padded : cnt));
}

// One wavefront per (n, c) plane: lanes stride over the H*W contiguous values, the partial sums
// meet in a butterfly of cross-lane moves, lane 0 stores the mean.
template <int DT>
__global__ __launch_bounds__(256) void global_avgpool_lp_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y,
                                                               int64_t planes, int HW) {
    const int lane = threadIdx.x & 63;
    const int64_t plane = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (plane >= planes) return;
    const uint16_t* xp = X + plane * HW;
    float acc = 0.f;
    for (int i = lane; i < HW; i += 64) acc += from_lp<DT>(xp[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) Y[plane] = to_lp<DT>(acc / (float)HW);
}

// Planes of at most 64 values (the 7 x 7 planes in front of a classifier): a wavefront takes eight neighbouring
// planes, one value per lane and plane, all eight loads requested together; the same butterfly per plane (the
// same order of additions as above), lanes 0..7 store the eight means.
template <int DT>
__global__ __launch_bounds__(256) void global_avgpool_lp_small_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y,
                                                                     int64_t planes, int HW) {
    const int lane = threadIdx.x & 63;
    const int64_t first = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 8;
    if (first >= planes) return;
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int64_t plane = first + k < planes ? first + k : planes - 1;
        acc[k] = lane < HW ? from_lp<DT>(X[plane * HW + lane]) : 0.f;
    }
    float mine = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) acc[k] += __shfl_xor(acc[k], off, 64);
        if (lane == k) mine = acc[k];
    }
    if (lane < 8 && first + lane < planes) Y[first + lane] = to_lp<DT>(mine / (float)HW);
}

// LeakyRelu (Section 3.1 of the paper: its operator definition lists F16 among the element types; Relu is
// alpha = 0): y = x for x >= 0, alpha * x otherwise, the product rounded to fp32 and then to the type.
// VEC = 8: one 16-byte load and store per thread; VEC = 1: any alignment and the tail.
template <int DT, int VEC>
__global__ __launch_bounds__(256) void leakyrelu_lp_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int64_t count,
                                                          float alpha) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (i >= count) return;
    auto one = [&](uint32_t bits) -> uint32_t {
        const float x = from_lp<DT>(bits);
        return x >= 0.f ? bits : to_lp<DT>(alpha * x);           // x >= 0 (and -0 only through the product) keeps its bits; NaN goes through the product
    };
    if constexpr (VEC == 8) {
        const uintx4 v = *reinterpret_cast<const uintx4*>(X + i);
        uintx4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = one(v[k] & 0xffffu) | (one(v[k] >> 16) << 16);
        *reinterpret_cast<uintx4*>(Y + i) = o;
    } else {
        Y[i] = (uint16_t)one(X[i]);
    }
}

}  // namespace

hipError_t launch_leakyrelu_lp(const void* X, void* Y, int64_t count, float alpha, int type, hipStream_t stream) {
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* y = static_cast<uint16_t*>(Y);
    const bool wide = count % 8 == 0 && ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(Y)) & 15u) == 0;
    const int64_t threads = wide ? count / 8 : count;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(256);
    if (type == LP_BF16) {
        if (wide) hipLaunchKernelGGL((leakyrelu_lp_kernel<LP_BF16, 8>), grid, block, 0, stream, x, y, count, alpha);
        else hipLaunchKernelGGL((leakyrelu_lp_kernel<LP_BF16, 1>), grid, block, 0, stream, x, y, count, alpha);
    } else {
        if (wide) hipLaunchKernelGGL((leakyrelu_lp_kernel<LP_F16, 8>), grid, block, 0, stream, x, y, count, alpha);
        else hipLaunchKernelGGL((leakyrelu_lp_kernel<LP_F16, 1>), grid, block, 0, stream, x, y, count, alpha);
    }
    return hipGetLastError();
}

// X, Y: 16-bit tensors of `type` (LP_F16 / LP_BF16).  The caller has checked that N*C*OH*OW < 2^31.
hipError_t launch_maxpool_lp(const void* X, void* Y, const WindowGeom& g, int type, hipStream_t stream) {
    const uint32_t total = (uint32_t)((int64_t)g.N * g.C * g.OH * g.OW);
    const PoolIndex d = {FastDiv::make((uint32_t)g.OW), FastDiv::make((uint32_t)g.OH)};
    const dim3 grid((total + 255u) / 256u), block(256);
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* y = static_cast<uint16_t*>(Y);
    // pairs of outputs from 4-byte loads: the window of output ow + 1 must end inside the pair at column 2*ow + 2, and the
    // last output's middle pair inside the row
    // four outputs per thread from 16-byte loads: rows a multiple of 8 long with W / 2 outputs each
    if (g.kW == 3 && g.sW == 2 && g.dW == 1 && g.pL == 1 && g.W % 8 == 0 && 2 * g.OW == g.W && (reinterpret_cast<uintptr_t>(X) & 15u) == 0 &&
        (reinterpret_cast<uintptr_t>(Y) & 7u) == 0) {
        const int quads_per_row = g.OW / 4;
        const uint32_t total_quads = (uint32_t)((int64_t)g.N * g.C * g.OH * quads_per_row);
        const PoolIndex dq = {FastDiv::make((uint32_t)quads_per_row), FastDiv::make((uint32_t)g.OH)};
        const dim3 qgrid((total_quads + 255u) / 256u);
        if (type == LP_BF16) hipLaunchKernelGGL(maxpool_lp_quads_kernel<LP_BF16>, qgrid, block, 0, stream, x, y, g, dq, total_quads);
        else hipLaunchKernelGGL(maxpool_lp_quads_kernel<LP_F16>, qgrid, block, 0, stream, x, y, g, dq, total_quads);
        return hipGetLastError();
    }
    if (g.kW == 3 && g.sW == 2 && g.dW == 1 && g.pL == 1 && g.W % 2 == 0 && 2 * g.OW <= g.W && (reinterpret_cast<uintptr_t>(X) & 3u) == 0) {
        const int pairs_per_row = (g.OW + 1) / 2;
        const uint32_t total_pairs = (uint32_t)((int64_t)g.N * g.C * g.OH * pairs_per_row);
        const PoolIndex dp = {FastDiv::make((uint32_t)pairs_per_row), FastDiv::make((uint32_t)g.OH)};
        const dim3 pgrid((total_pairs + 255u) / 256u);
        if (type == LP_BF16) hipLaunchKernelGGL(maxpool_lp_pairs_kernel<LP_BF16>, pgrid, block, 0, stream, x, y, g, dp, total_pairs);
        else hipLaunchKernelGGL(maxpool_lp_pairs_kernel<LP_F16>, pgrid, block, 0, stream, x, y, g, dp, total_pairs);
        return hipGetLastError();
    }
    if (type == LP_BF16) hipLaunchKernelGGL(maxpool_lp_kernel<LP_BF16>, grid, block, 0, stream, x, y, g, d, total);
    else hipLaunchKernelGGL(maxpool_lp_kernel<LP_F16>, grid, block, 0, stream, x, y, g, d, total);
    return hipGetLastError();
}

hipError_t launch_avgpool_lp(const void* X, void* Y, const WindowGeom& g, int count_include_pad, int type, hipStream_t stream) {
    const uint32_t total = (uint32_t)((int64_t)g.N * g.C * g.OH * g.OW);
    const PoolIndex d = {FastDiv::make((uint32_t)g.OW), FastDiv::make((uint32_t)g.OH)};
    const dim3 grid((total + 255u) / 256u), block(256);
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* y = static_cast<uint16_t*>(Y);
    if (type == LP_BF16) hipLaunchKernelGGL(avgpool_lp_kernel<LP_BF16>, grid, block, 0, stream, x, y, g, count_include_pad, d, total);
    else hipLaunchKernelGGL(avgpool_lp_kernel<LP_F16>, grid, block, 0, stream, x, y, g, count_include_pad, d, total);
    return hipGetLastError();
}

hipError_t launch_global_avgpool_lp(const void* X, void* Y, int64_t planes, int HW, int type, hipStream_t stream) {
    const int64_t blocks = (planes + 3) / 4;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* y = static_cast<uint16_t*>(Y);
    if (HW <= 64 && planes >= 64) {
        const dim3 grid((unsigned)((planes + 31) / 32)), block(256);
        if (type == LP_BF16) hipLaunchKernelGGL(global_avgpool_lp_small_kernel<LP_BF16>, grid, block, 0, stream, x, y, planes, HW);
        else hipLaunchKernelGGL(global_avgpool_lp_small_kernel<LP_F16>, grid, block, 0, stream, x, y, planes, HW);
        return hipGetLastError();
    }
    if (type == LP_BF16) hipLaunchKernelGGL(global_avgpool_lp_kernel<LP_BF16>, dim3((unsigned)blocks), dim3(256), 0, stream, x, y, planes, HW);
    else hipLaunchKernelGGL(global_avgpool_lp_kernel<LP_F16>, dim3((unsigned)blocks), dim3(256), 0, stream, x, y, planes, HW);
    return hipGetLastError();
}

}  // namespace onnxhip
