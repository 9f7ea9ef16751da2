// Sliding-window kernels that do not use the matrix cores: direct convolution for depthwise /
// tiny groups, MaxPool, AveragePool and GlobalAveragePool (Section 4.1 of the paper lists
// convolution and pooling among the supported operators).  All are bandwidth- or
// latency-bound.  The generic kernels use one thread per output element, lanes running along
// the contiguous output width; 3x3 convolutions and 2x2 / 3x3 max pools go through the
// plane-tile kernels further down, which stage the input in LDS.
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

// ---- row-strip variants -------------------------------------------------------------------
// One wavefront owns R consecutive output rows x 64 consecutive output columns of one (image,
// channel) plane, one column per lane.  It issues every load the strip needs up front (the
// ROWS_IN input rows it touches x KW taps per lane: neighbouring lanes and neighbouring taps
// hit the same cache lines, so memory sees each line once) and then only does arithmetic on
// registers: nothing waits on LDS or on a barrier, and a CU keeps several hundred independent
// loads in flight, which is what a bandwidth-bound kernel needs.  Vertical stride and
// dilation are template arguments so that the input row of every (output row, kh) is a
// register known at compile time; everything horizontal is plain address arithmetic.
struct StripMap {
    FastDiv chunks, strips;   // column chunks per row, strips per plane
    uint32_t waves;           // planes * strips * chunks
};

__device__ inline __amdgpu_buffer_rsrc_t plane_rsrc(const float* plane, int HW) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(plane), 0, HW * 4, 0x00020000);
}

// SHUF (KW = 3, horizontal stride and dilation 1, left pad 1, W <= 64 so that one wavefront spans
// a row): each lane loads only the input value above its own column; the taps to the left and
// right are the neighbouring lanes' values (zero outside the image).
template <int KH, int KW, int S, int D, int R, bool SHUF>
__global__ __launch_bounds__(256) void conv_rows_kernel(const float* __restrict__ X,
                                                        const float* __restrict__ Wt,
                                                        const float* __restrict__ B,
                                                        const float* __restrict__ residual,
                                                        float* __restrict__ Y, WindowGeom g, int M, int Cg,
                                                        int Mg, int relu, StripMap sm) {
    constexpr int ROWS_IN = (R - 1) * S + (KH - 1) * D + 1;
    constexpr uint32_t OUT = 0x80000000u;             // offset the buffer range check rejects
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * 4u + (threadIdx.x >> 6));
    if (wave >= sm.waves) return;
    const int lane = threadIdx.x & 63;
    uint32_t rest, chunk, pm, strip;
    sm.chunks.divmod(wave, rest, chunk);
    sm.strips.divmod(rest, pm, strip);                // pm = n*M + m
    const int n = (int)pm / M, m = (int)pm % M;
    const int grp = m / Mg;
    const int oh0 = (int)strip * R;
    const int ow = (int)chunk * 64 + lane;
    const int ih0 = oh0 * S - g.pT;
    uint32_t voff[KW];
#pragma unroll
    for (int kw = 0; kw < KW; ++kw) {
        const int iw = ow * g.sW - g.pL + kw * g.dW;
        voff[kw] = (ow < g.OW && (unsigned)iw < (unsigned)g.W) ? (uint32_t)iw * 4u : OUT;
    }
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    const int HW = g.H * g.W;
    const float* wm = Wt + (int64_t)m * Cg * KH * KW;
    for (int c = 0; c < Cg; ++c) {
        const __amdgpu_buffer_rsrc_t rs = plane_rsrc(X + ((int64_t)n * g.C + grp * Cg + c) * HW, HW);
        float x[ROWS_IN][KW];
        if (SHUF) {
            const uint32_t centre = ow < g.W ? (uint32_t)ow * 4u : OUT;
            float v[ROWS_IN];
#pragma unroll
            for (int i = 0; i < ROWS_IN; ++i) {
                const int ih = ih0 + i;
                const bool row_ok = (unsigned)ih < (unsigned)g.H;      // uniform
                v[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                           rs, (int)(row_ok ? centre : OUT), row_ok ? ih * g.W * 4 : 0, 0));
            }
#pragma unroll
            for (int i = 0; i < ROWS_IN; ++i) {
                const float left = __shfl_up(v[i], 1, 64), right = __shfl_down(v[i], 1, 64);
                x[i][0] = lane > 0 ? left : 0.f;
                x[i][KW / 2] = v[i];
                x[i][KW - 1] = lane < 63 ? right : 0.f;                 // lanes at and beyond W loaded zeros
            }
        } else {
#pragma unroll
            for (int i = 0; i < ROWS_IN; ++i) {
                const int ih = ih0 + i;
                const bool row_ok = (unsigned)ih < (unsigned)g.H;      // uniform
#pragma unroll
                for (int kw = 0; kw < KW; ++kw)
                    x[i][kw] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                   rs, (int)(row_ok ? voff[kw] : OUT), row_ok ? ih * g.W * 4 : 0, 0));
            }
        }
        float w[KH * KW];                                              // uniform: scalar loads
#pragma unroll
        for (int i = 0; i < KH * KW; ++i) w[i] = wm[c * KH * KW + i];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                for (int kw = 0; kw < KW; ++kw) acc[r] = fmaf(x[r * S + kh * D][kw], w[kh * KW + kw], acc[r]);
    }
    if (ow >= g.OW) return;
    const float bias = B ? B[m] : 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int oh = oh0 + r;
        if (oh < g.OH) {
            const int64_t o = ((int64_t)pm * g.OH + oh) * g.OW + ow;
            float v = acc[r] + bias;
            if (residual) v += residual[o];
            if (relu) v = v > 0.f ? v : 0.f;
            Y[o] = v;
        }
    }
}

// MaxPool on the same wavefront-per-strip scheme (vertical dilation 1).  Taps outside the image
// never take part; taps are visited kh outer, kw inner and a later tap replaces the running
// maximum only when strictly greater, so Indices reports the first maximum.
// PAIR (horizontal stride 2, dilation 1, left pad KW - 2, even W, one column chunk per row): the
// taps at input columns 2*ow and 2*ow + 1 come from one 8-byte load per lane, which makes the
// wavefront's load one contiguous 512-byte run instead of three runs of every other element;
// for KW = 3 the tap at 2*ow - 1 is the left neighbour lane's second value.
template <int KH, int KW, int S, int R, bool IDX, bool PAIR>
__global__ __launch_bounds__(256) void maxpool_rows_kernel(const float* __restrict__ X, float* __restrict__ Y,
                                                           int64_t* __restrict__ indices, WindowGeom g,
                                                           StripMap sm) {
    constexpr int ROWS_IN = (R - 1) * S + KH;
    constexpr uint32_t OUT = 0x80000000u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * 4u + (threadIdx.x >> 6));
    if (wave >= sm.waves) return;
    const int lane = threadIdx.x & 63;
    uint32_t rest, chunk, pc, strip;
    sm.chunks.divmod(wave, rest, chunk);
    sm.strips.divmod(rest, pc, strip);                // pc = n*C + c
    const int oh0 = (int)strip * R;
    const int ow = (int)chunk * 64 + lane;
    const int ih0 = oh0 * S - g.pT;
    const int iw0 = ow * g.sW - g.pL;
    uint32_t voff[KW];
    bool col_ok[KW];
#pragma unroll
    for (int kw = 0; kw < KW; ++kw) {
        const int iw = iw0 + kw * g.dW;
        col_ok[kw] = ow < g.OW && (unsigned)iw < (unsigned)g.W;
        voff[kw] = col_ok[kw] ? (uint32_t)iw * 4u : OUT;
    }
    const int HW = g.H * g.W;
    const int64_t plane_abs = (int64_t)pc * HW;
    const __amdgpu_buffer_rsrc_t rs = plane_rsrc(X + plane_abs, HW);
    float x[ROWS_IN][KW];
    if (PAIR) {
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        const uint32_t pair_off = (ow < g.OW && 2 * ow + 1 < g.W) ? (uint32_t)(2 * ow) * 4u : OUT;
        floatx2 v[ROWS_IN];
#pragma unroll
        for (int i = 0; i < ROWS_IN; ++i) {
            const int ih = ih0 + i;
            const bool row_ok = (unsigned)ih < (unsigned)g.H;          // uniform
            v[i] = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(
                       rs, (int)(row_ok ? pair_off : OUT), row_ok ? ih * g.W * 4 : 0, 0));
        }
#pragma unroll
        for (int i = 0; i < ROWS_IN; ++i) {
            x[i][KW - 2] = v[i].x;
            x[i][KW - 1] = v[i].y;
            if (KW == 3) x[i][0] = __shfl_up(v[i].y, 1, 64);           // lane 0 has ow = 0: its left tap is padding
        }
    } else {
#pragma unroll
        for (int i = 0; i < ROWS_IN; ++i) {
            const int ih = ih0 + i;
            const bool row_ok = (unsigned)ih < (unsigned)g.H;          // uniform
#pragma unroll
            for (int kw = 0; kw < KW; ++kw)
                x[i][kw] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                               rs, (int)(row_ok ? voff[kw] : OUT), row_ok ? ih * g.W * 4 : 0, 0));
        }
    }
    if (ow >= g.OW) return;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int oh = oh0 + r;
        if (oh >= g.OH) break;
        float best = -__builtin_inff();
        bool found = false;
        int bh = 0, bw = 0;
#pragma unroll
        for (int kh = 0; kh < KH; ++kh) {
            const bool row_ok = (unsigned)(ih0 + r * S + kh) < (unsigned)g.H;
#pragma unroll
            for (int kw = 0; kw < KW; ++kw) {
                const float v = x[r * S + kh][kw];
                const bool take = row_ok && col_ok[kw] && (!found || v > best);
                best = take ? v : best;
                if (IDX) {
                    bh = take ? kh : bh;
                    bw = take ? kw : bw;
                }
                found = found || take;
            }
        }
        const int64_t o = ((int64_t)pc * g.OH + oh) * g.OW + ow;
        Y[o] = best;
        if (IDX) indices[o] = plane_abs + (int64_t)(ih0 + r * S + bh) * g.W + (iw0 + bw * g.dW);
    }
}

static inline bool strip_map(const WindowGeom& g, int64_t planes, int R, StripMap& sm) {
    const int64_t chunks = (g.OW + 63) / 64, strips = (g.OH + R - 1) / R;
    const int64_t waves = planes * strips * chunks;
    if (g.OW < 1 || g.OH < 1 || (int64_t)g.H * g.W * 4 >= (1LL << 31) || waves >= (1LL << 31)) return false;
    sm.chunks = FastDiv::make((uint32_t)chunks);
    sm.strips = FastDiv::make((uint32_t)strips);
    sm.waves = (uint32_t)waves;
    return true;
}

template <int S, int D>
static hipError_t launch_conv_rows(const float* X, const float* W, const float* B, const float* residual,
                                   float* Y, const WindowGeom& g, int M, int Cg, int group, int relu,
                                   const StripMap& sm, hipStream_t stream) {
    // one load per row instead of three when a wavefront spans the whole row (see SHUF)
    if (g.sW == 1 && g.dW == 1 && g.pL == 1 && g.W <= 64 && g.OW <= 64)
        hipLaunchKernelGGL((conv_rows_kernel<3, 3, S, D, 8, true>), dim3((sm.waves + 3) / 4), dim3(256), 0, stream, X, W,
                           B, residual, Y, g, M, Cg, M / group, relu, sm);
    else
        hipLaunchKernelGGL((conv_rows_kernel<3, 3, S, D, 8, false>), dim3((sm.waves + 3) / 4), dim3(256), 0, stream, X,
                           W, B, residual, Y, g, M, Cg, M / group, relu, sm);
    return hipGetLastError();
}

// ---- plane-tile variants ------------------------------------------------------------------
// A workgroup owns a strip of output rows of one (image, channel) plane.  It copies the input
// rows the strip needs into LDS with fully coalesced loads (every input element is read from
// memory once, padding is materialised in LDS: 0 for convolution, -inf for MaxPool), then each
// thread produces outputs from LDS, lanes along the output width.  The filter taps of a
// convolution are uniform for the workgroup and come from scalar loads.
constexpr int PLANE_LDS_FLOATS = 6144;          // 24 KiB
constexpr uint32_t kOutOfRange = 0x80000000u;

struct PlaneTiling {
    int toh, row_tiles;       // output rows per strip, strips per plane
    int rows_in, lw;          // input rows per strip, LDS row length = W + pL + pR
    FastDiv lwd, owd, rtd;    // divisors: lw, OW, row_tiles
};

// Copies input rows [ih_first, ih_first + rows_in) x columns [-pL, W + pR) of one plane into LDS.
__device__ inline void plane_fill(float* lds, const float* plane, const WindowGeom& g, const PlaneTiling& t,
                                  int ih_first, float pad) {
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(plane), 0,
                                                                       g.H * g.W * 4, 0x00020000);
    const int total = t.rows_in * t.lw;
    for (int e = threadIdx.x; e < total; e += 256) {
        uint32_t row, x;
        t.lwd.divmod((uint32_t)e, row, x);
        const int ih = ih_first + (int)row, iw = (int)x - g.pL;
        const bool ok = (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
        const float v = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                            r, ok ? (ih * g.W + iw) * 4 : (int)kOutOfRange, 0, 0));
        lds[e] = ok ? v : pad;
    }
}

template <int KH, int KW>
__global__ __launch_bounds__(256) void conv_plane_kernel(const float* __restrict__ X,
                                                         const float* __restrict__ Wt,
                                                         const float* __restrict__ B,
                                                         const float* __restrict__ residual,
                                                         float* __restrict__ Y, WindowGeom g, int M, int Cg,
                                                         int Mg, int relu, PlaneTiling t) {
    __shared__ float lds[PLANE_LDS_FLOATS];
    uint32_t pm, rt;
    t.rtd.divmod(blockIdx.x, pm, rt);                  // pm = n*M + m
    const int n = (int)pm / M, m = (int)pm % M;
    const int grp = m / Mg;
    const int oh0 = (int)rt * t.toh;
    const int nrows = min(t.toh, g.OH - oh0);
    const int ih_first = oh0 * g.sH - g.pT;
    const int nout = nrows * g.OW;
    constexpr int MAXO = 12;                           // outputs per thread held in registers
    float acc[MAXO];
#pragma unroll
    for (int i = 0; i < MAXO; ++i) acc[i] = 0.f;
    const float* wm = Wt + (int64_t)m * Cg * KH * KW;
    for (int c = 0; c < Cg; ++c) {
        const float* plane = X + ((int64_t)n * g.C + grp * Cg + c) * g.H * g.W;
        if (c) __syncthreads();
        plane_fill(lds, plane, g, t, ih_first, 0.f);
        float w[KH * KW];                              // uniform: scalar loads
#pragma unroll
        for (int i = 0; i < KH * KW; ++i) w[i] = wm[c * KH * KW + i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < MAXO; ++i) {
            const int idx = threadIdx.x + i * 256;
            if (idx < nout) {
                uint32_t r, ow;
                t.owd.divmod((uint32_t)idx, r, ow);
                const float* p = lds + ((int)r * g.sH) * t.lw + (int)ow * g.sW;
                float a = acc[i];
#pragma unroll
                for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                    for (int kw = 0; kw < KW; ++kw) a = fmaf(p[kh * g.dH * t.lw + kw * g.dW], w[kh * KW + kw], a);
                acc[i] = a;
            }
        }
    }
    const float bias = B ? B[m] : 0.f;
    const int64_t o0 = ((int64_t)pm * g.OH + oh0) * g.OW;
#pragma unroll
    for (int i = 0; i < MAXO; ++i) {
        const int idx = threadIdx.x + i * 256;
        if (idx < nout) {
            float v = acc[i] + bias;
            if (residual) v += residual[o0 + idx];
            if (relu) v = v > 0.f ? v : 0.f;
            Y[o0 + idx] = v;
        }
    }
}

template <int KH, int KW, bool IDX>
__global__ __launch_bounds__(256) void maxpool_plane_kernel(const float* __restrict__ X, float* __restrict__ Y,
                                                            int64_t* __restrict__ indices, WindowGeom g,
                                                            PlaneTiling t) {
    __shared__ float lds[PLANE_LDS_FLOATS];
    uint32_t pc, rt;
    t.rtd.divmod(blockIdx.x, pc, rt);                  // pc = n*C + c
    const int oh0 = (int)rt * t.toh;
    const int nrows = min(t.toh, g.OH - oh0);
    const int ih_first = oh0 * g.sH - g.pT;
    const int64_t plane_abs = (int64_t)pc * g.H * g.W;
    plane_fill(lds, X + plane_abs, g, t, ih_first, -__builtin_inff());
    __syncthreads();
    const int nout = nrows * g.OW;
    const int64_t o0 = ((int64_t)pc * g.OH + oh0) * g.OW;
    for (int idx = threadIdx.x; idx < nout; idx += 256) {
        uint32_t r, ow;
        t.owd.divmod((uint32_t)idx, r, ow);
        const int lr = (int)r * g.sH, lc = (int)ow * g.sW;        // window origin in LDS coordinates
        const float* p = lds + lr * t.lw + lc;
        // Padding holds -inf and can never replace the running maximum; the scan starts from
        // the first tap inside the image so that an all -inf window still reports that tap.
        // Taps are visited kh outer, kw inner and replace on strict >, i.e. first maximum wins.
        float best = -__builtin_inff();
        int bh = 0, bw = 0;
        if (IDX) {
            const int ih0 = ih_first + lr, iw0 = lc - g.pL;
            bh = ih0 < 0 ? (-ih0 + g.dH - 1) / g.dH : 0;
            bw = iw0 < 0 ? (-iw0 + g.dW - 1) / g.dW : 0;
        }
#pragma unroll
        for (int kh = 0; kh < KH; ++kh)
#pragma unroll
            for (int kw = 0; kw < KW; ++kw) {
                const float v = p[kh * g.dH * t.lw + kw * g.dW];
                if (IDX) {
                    const bool take = v > best;
                    bh = take ? kh : bh;
                    bw = take ? kw : bw;
                }
                best = fmaxf(best, v);
            }
        Y[o0 + idx] = best;
        if (IDX) {
            const int ih = ih_first + lr + bh * g.dH, iw = lc - g.pL + bw * g.dW;
            indices[o0 + idx] = plane_abs + (int64_t)ih * g.W + iw;
        }
    }
}

// Strip height such that the input rows of a strip fit the LDS tile; false if not even one
// output row fits or the strip would exceed what a thread holds in registers.
static inline bool plane_tiling(const WindowGeom& g, int64_t planes, int max_out_per_thread, PlaneTiling& t) {
    const int64_t lw = (int64_t)g.W + g.pL + g.pR;
    const int64_t eh = (int64_t)(g.kH - 1) * g.dH + 1, ew = (int64_t)(g.kW - 1) * g.dW + 1;
    if (lw * eh > PLANE_LDS_FLOATS || g.OW < 1 || g.OH < 1) return false;
    if ((int64_t)(g.OW - 1) * g.sW + ew > lw) return false;        // windows stay inside the padded row
    if ((int64_t)g.H * g.W * 4 >= (1LL << 31)) return false;
    int64_t toh = (PLANE_LDS_FLOATS / lw - eh) / g.sH + 1;
    if (toh > g.OH) toh = g.OH;
    if (max_out_per_thread > 0) {
        const int64_t by_regs = (int64_t)max_out_per_thread * 256 / g.OW;
        if (by_regs < 1) return false;
        if (toh > by_regs) toh = by_regs;
    }
    // enough strips to occupy the chip when there are few planes
    while (toh > 1 && planes * ((g.OH + toh - 1) / toh) < 2048) toh = (toh + 1) / 2;
    t.toh = (int)toh;
    t.row_tiles = (int)((g.OH + toh - 1) / toh);
    t.rows_in = (int)((toh - 1) * g.sH + eh);
    t.lw = (int)lw;
    if ((int64_t)t.rows_in * lw > PLANE_LDS_FLOATS) return false;
    if (planes * t.row_tiles > 0x7fffffffLL) return false;
    t.lwd = FastDiv::make((uint32_t)lw);
    t.owd = FastDiv::make((uint32_t)g.OW);
    t.rtd = FastDiv::make((uint32_t)t.row_tiles);
    return true;
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
    if (g.kH == 3 && g.kW == 3) {
        StripMap sm;
        if (strip_map(g, (int64_t)g.N * M, 8, sm)) {
            if (g.sH == 1 && g.dH == 1) return launch_conv_rows<1, 1>(X, W, B, residual, Y, g, M, Cg, group, relu, sm, stream);
            if (g.sH == 2 && g.dH == 1) return launch_conv_rows<2, 1>(X, W, B, residual, Y, g, M, Cg, group, relu, sm, stream);
            if (g.sH == 1 && g.dH == 2) return launch_conv_rows<1, 2>(X, W, B, residual, Y, g, M, Cg, group, relu, sm, stream);
        }
        PlaneTiling t;
        if (plane_tiling(g, (int64_t)g.N * M, 12, t)) {
            hipLaunchKernelGGL((conv_plane_kernel<3, 3>), dim3((unsigned)((int64_t)g.N * M * t.row_tiles)), dim3(256), 0,
                               stream, X, W, B, residual, Y, g, M, Cg, M / group, relu, t);
            return hipGetLastError();
        }
    }
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
    const int shape = g.kH != g.kW ? 0 : g.kH == 3 ? 3 : g.kH == 2 ? 2 : 0;
    StripMap sm;
    if (shape && g.dH == 1 && g.sH == 2 && strip_map(g, (int64_t)g.N * g.C, 4, sm)) {
        const dim3 grid((sm.waves + 3) / 4), block(256);
        // 8-byte loads of column pairs: every row of every plane starts 8-byte aligned, the pair
        // (2*ow, 2*ow + 1) holds the window's last two taps, and the lane to the left holds the first
        const bool pair = g.sW == 2 && g.dW == 1 && g.pL == shape - 2 && g.W % 2 == 0 && g.OW <= 64 &&
                          (reinterpret_cast<uintptr_t>(X) & 7u) == 0;
#define ONNXHIP_POOL(K_, P_)                                                                                       \
    if (indices) hipLaunchKernelGGL((maxpool_rows_kernel<K_, K_, 2, 4, true, P_>), grid, block, 0, stream, X, Y, indices, g, sm); \
    else hipLaunchKernelGGL((maxpool_rows_kernel<K_, K_, 2, 4, false, P_>), grid, block, 0, stream, X, Y, indices, g, sm);
        if (shape == 3) { if (pair) { ONNXHIP_POOL(3, true) } else { ONNXHIP_POOL(3, false) } }
        else { if (pair) { ONNXHIP_POOL(2, true) } else { ONNXHIP_POOL(2, false) } }
#undef ONNXHIP_POOL
        return hipGetLastError();
    }
    PlaneTiling t;
    if (shape && plane_tiling(g, (int64_t)g.N * g.C, 0, t)) {
        const dim3 grid((unsigned)((int64_t)g.N * g.C * t.row_tiles)), block(256);
#define ONNXHIP_POOL(K_)                                                                                          \
    if (indices) hipLaunchKernelGGL((maxpool_plane_kernel<K_, K_, true>), grid, block, 0, stream, X, Y, indices, g, t); \
    else hipLaunchKernelGGL((maxpool_plane_kernel<K_, K_, false>), grid, block, 0, stream, X, Y, indices, g, t);
        if (shape == 3) { ONNXHIP_POOL(3) } else { ONNXHIP_POOL(2) }
#undef ONNXHIP_POOL
        return hipGetLastError();
    }
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
