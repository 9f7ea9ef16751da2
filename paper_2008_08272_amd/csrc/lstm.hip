// ONNX LSTM (named among the supported operators in Section 4.1 of the paper).  The input
// projection of the whole sequence (x_t W' + Wb + Rb for every t) is one Gemm through the
// contraction kernels; every time step is then ONE launch of lstm_step_kernel, which forms
// h R' on the matrix cores, adds the projection, applies the gates and writes the new state:
// both directions of a bidirectional LSTM go into the same launch.
#include <stdio.h>

#include <type_traits>

#include "../../include/onnxhip.h"
#include "internal.h"

using namespace onnxhip;

namespace {

#define fail(st, ...) static_cast<onnx_status>(fail_with((st), __VA_ARGS__))

__device__ inline float sigmoidf(float v) { return 1.0f / (1.0f + expf(-v)); }

// bias[k] = Wb[k] + Rb[k] for the 4H gate rows (zeros without B)
__global__ __launch_bounds__(256) void lstm_bias_kernel(const float* __restrict__ B, float* __restrict__ bias, int n4h) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n4h) bias[i] = B ? B[i] + B[n4h + i] : 0.f;
}

// dst = src, or zeros without src
__global__ __launch_bounds__(256) void lstm_state_kernel(const float* __restrict__ src, float* __restrict__ dst, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = src ? src[i] : 0.f;
}

// One time step of up to two directions.
struct LstmStep {
    const float* hprev[2];    // [batch, H]
    float* hnext[2];          // [batch, H]
    float* c[2];              // [batch, H], updated in place
    const float* R[2];        // [4H, H], gate blocks i, o, f, c
    const float* G[2];        // [batch, 4H]: this step's slice of the input projection (biases included)
    float* y[2];              // this step's slot of Y, or NULL
    float* y_h[2];            // final-state outputs (last step only), or NULL
    float* y_c[2];
    int batch, H;
    int KW;                   // k per wavefront: a multiple of 8, 4 * KW >= H
};

// A workgroup owns 32 batch rows x 8 hidden units: the 32 columns of its MFMAs are the 4 gates of
// those units (column 8 g + u is row g*H + u0 + u of R).  Its four wavefronts split the reduction
// over k: wavefront w takes k in [w*KW, (w+1)*KW), in blocks of 128.  A wavefront stages its own
// block of h rows and R rows in its own part of LDS with coalesced loads (a row's 128 k are 32
// lanes x 16 bytes; VEC = 1: 4-byte loads, for H not a multiple of 4 or unaligned pointers) and
// reads the MFMA operands back from there, lanes 0-31 feeding the first 64 k of the block and lanes
// 32-63 the second: no barrier until the four partial 32 x 32 sums meet in LDS, after which thread
// (b, u) applies the gates for its batch row and unit.
template <int VEC>
__global__ __launch_bounds__(256) void lstm_step_kernel(const LstmStep p) {
    constexpr int KB = 128;                             // k per block
    constexpr int PITCH = KB + 4;                       // LDS row pitch: 16-byte reads of 8 neighbouring rows hit disjoint banks
    __shared__ __attribute__((aligned(16))) float stage[4][2][32 * PITCH];   // per wavefront: h rows, R rows
    const int d = blockIdx.z, u0 = blockIdx.x * 8, b0 = blockIdx.y * 32;
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 31, h2 = lane >> 5;
    const int H = p.H;
    const __amdgpu_buffer_rsrc_t ra = tile_rsrc(p.hprev[d]);
    const __amdgpu_buffer_rsrc_t rb = tile_rsrc(p.R[d]);
    float* sa = stage[wave][0];
    float* sb = stage[wave][1];

    // what the gate phase will need from memory is requested now, so that it arrives during the MFMAs
    const int gb = t & 31, gu = t >> 5;                 // this thread's batch row and unit in the gate phase
    const bool g_ok = b0 + gb < p.batch && u0 + gu < H;
    const int idx = (b0 + gb) * H + u0 + gu;
    float pre[4] = {0.f, 0.f, 0.f, 0.f}, c_old = 0.f;
    if (g_ok) {
        const float* g_row = p.G[d] + (int64_t)(b0 + gb) * 4 * H + u0 + gu;
#pragma unroll
        for (int g = 0; g < 4; ++g) pre[g] = g_row[(int64_t)g * H];
        c_old = p.c[d][idx];
    }

    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    for (int kb = 0; kb < p.KW; kb += KB) {
        const int k0 = wave * p.KW + kb;                // first k of this block
        const int klen = min(KB, p.KW - kb);            // a multiple of 8
        // ---- stage: pass j brings rows 2j and 2j+1 (lanes 0-31 / 32-63), 4 k per lane
        floatx4 va[16], vb[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int row = 2 * j + h2, k = k0 + 4 * li;
            const int arow = b0 + row;
            const int brow = (row >> 3) * H + u0 + (row & 7);          // gate row/8, unit row%8
            const bool k_in = 4 * li < klen;
            const bool a_ok = k_in && arow < p.batch, b_ok = k_in && u0 + (row & 7) < H;
            if (VEC == 4) {
                va[j] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(ra, (a_ok && k < H) ? (arow * H + k) * 4 : (int)OOB, 0, 0));
                vb[j] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rb, (b_ok && k < H) ? (brow * H + k) * 4 : (int)OOB, 0, 0));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    va[j][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ra, (a_ok && k + e < H) ? (arow * H + k + e) * 4 : (int)OOB, 0, 0));
                    vb[j][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, (b_ok && k + e < H) ? (brow * H + k + e) * 4 : (int)OOB, 0, 0));
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            *reinterpret_cast<floatx4*>(sa + (2 * j + h2) * PITCH + 4 * li) = va[j];
            *reinterpret_cast<floatx4*>(sb + (2 * j + h2) * PITCH + 4 * li) = vb[j];
        }
        // ---- MFMAs: this lane's row, its half of the block, 4 k per 16-byte read (the LDS queue of a
        // wavefront is served in order, so these reads see the stores above)
        const int half = klen / 2;
        floatx4 fa[KB / 8], fb[KB / 8];                  // all of the block's fragments first, then its MFMAs
#pragma unroll
        for (int q = 0; q < KB / 8; ++q) {
            const int off = 4 * q < half ? h2 * half + 4 * q : 0;      // past a short block: any staged value, multiplied by nothing
            fa[q] = *reinterpret_cast<const floatx4*>(sa + li * PITCH + off);
            fb[q] = *reinterpret_cast<const floatx4*>(sb + li * PITCH + off);
        }
#pragma unroll
        for (int q = 0; q < KB / 8; ++q) {
            if (4 * q < half) {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[q][e], fb[q][e], acc, 0, 0, 0);
            }
        }
    }
    __shared__ float red[4][16][64];
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[r];
    __syncthreads();

    // ---- gates: thread (gb, gu); accumulator element (row, col) sits in register 4*(row/8) + row%4 of lane col + 32*((row%8)/4)
    if (!g_ok) return;
    const int reg = 4 * (gb >> 3) + (gb & 3), lhalf = 32 * ((gb & 7) >> 2);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int l = 8 * g + gu + lhalf;
        pre[g] += (red[0][reg][l] + red[1][reg][l]) + (red[2][reg][l] + red[3][reg][l]);
    }
    const float gi = sigmoidf(pre[0]), go = sigmoidf(pre[1]), gf = sigmoidf(pre[2]), gc = tanhf(pre[3]);
    const float cn = gf * c_old + gi * gc;
    const float hn = go * tanhf(cn);
    p.c[d][idx] = cn;
    p.hnext[d][idx] = hn;
    if (p.y[d]) p.y[d][idx] = hn;
    if (p.y_h[d]) p.y_h[d][idx] = hn;
    if (p.y_c[d]) p.y_c[d][idx] = cn;
}

// scratch layout per direction (floats): G [seq*batch*4H], P [batch*4H], h [2][batch*H], c [batch*H], bias [4H]
int64_t scratch_floats_per_direction(int64_t seq, int64_t batch, int64_t H) {
    auto up = [](int64_t v) { return (v + 63) / 64 * 64; };      // keep every block 256-byte aligned
    return up(seq * batch * 4 * H) + up(batch * 4 * H) + 2 * up(batch * H) + up(batch * H) + up(4 * H);
}

}  // namespace

extern "C" {

size_t onnx_lstm_scratch_bytes(const int64_t x_dims[3], int64_t hidden_size, int direction) {
    if (!x_dims || hidden_size < 1 || x_dims[0] < 0 || x_dims[1] < 0) return 0;
    const int dirs = direction == ONNX_LSTM_BIDIRECTIONAL ? 2 : 1;
    return (size_t)(dirs * scratch_floats_per_direction(x_dims[0], x_dims[1], hidden_size) * 4);
}

onnx_status onnx_lstm(const float* X, const int64_t x_dims[3], const float* W, const float* R, const float* B,
                      const float* initial_h, const float* initial_c, int64_t hidden_size, int direction, float* Y,
                      float* Y_h, float* Y_c, void* scratch, size_t scratch_bytes, void* stream) {
    if (!x_dims) return fail(ONNX_ERR_NULL, "lstm: NULL dims array");
    if (direction != ONNX_LSTM_FORWARD && direction != ONNX_LSTM_REVERSE && direction != ONNX_LSTM_BIDIRECTIONAL)
        return fail(ONNX_ERR_ATTR, "lstm: direction must be forward (0), reverse (1) or bidirectional (2)");
    const int64_t seq = x_dims[0], batch = x_dims[1], in = x_dims[2], H = hidden_size;
    if (seq < 0 || batch < 0 || in < 0) return fail(ONNX_ERR_SHAPE, "lstm: negative dimension");
    if (H < 1) return fail(ONNX_ERR_ATTR, "lstm: hidden_size must be at least 1");
    const int dirs = direction == ONNX_LSTM_BIDIRECTIONAL ? 2 : 1;
    if (batch == 0) return ONNX_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t ns = dirs * batch * H * 4;
    if (batch * 4 * H * 4 >= (1LL << 31) || seq * batch > 0x7fffffffLL || in > 0x7fffffffLL || 4 * H * H * 4 >= (1LL << 31))
        return fail(ONNX_ERR_UNSUPPORTED, "lstm: an extent exceeds the 32-bit offsets of the kernels");
    if (seq == 0) {
        // no step: the final states are the initial ones
        if (overlaps(Y_h, ns, initial_h, ns) || overlaps(Y_c, ns, initial_c, ns) || overlaps(Y_h, ns, Y_c, ns))
            return fail(ONNX_ERR_ALIAS, "lstm: an output overlaps an input");
        const int n = (int)(dirs * batch * H);
        if (Y_h) hipLaunchKernelGGL(lstm_state_kernel, dim3((n + 255) / 256), dim3(256), 0, s, initial_h, Y_h, n);
        if (Y_c) hipLaunchKernelGGL(lstm_state_kernel, dim3((n + 255) / 256), dim3(256), 0, s, initial_c, Y_c, n);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return fail(ONNX_ERR_DEVICE, "lstm: %s", hipGetErrorString(e0));
        return ONNX_OK;
    }
    if (!X || !W || !R) return fail(ONNX_ERR_NULL, "lstm: X, W and R must not be NULL");
    if (!Y && !Y_h && !Y_c) return fail(ONNX_ERR_NULL, "lstm: at least one of Y, Y_h, Y_c must be given");
    const size_t need = onnx_lstm_scratch_bytes(x_dims, H, direction);
    if (!scratch) return fail(ONNX_ERR_NULL, "lstm: scratch must not be NULL (%zu bytes are needed)", need);
    if (scratch_bytes < need)
        return fail(ONNX_ERR_ATTR, "lstm: %zu bytes of scratch are needed (onnx_lstm_scratch_bytes), %zu given", need, scratch_bytes);
    if ((reinterpret_cast<uintptr_t>(scratch) & 255u) != 0) return fail(ONNX_ERR_ATTR, "lstm: scratch must be 256-byte aligned");
    const int64_t ny = seq * dirs * batch * H * 4;
    const void* ins[] = {X, W, R, B, initial_h, initial_c};
    const int64_t in_bytes[] = {seq * batch * in * 4, dirs * 4 * H * in * 4, dirs * 4 * H * H * 4, dirs * 8 * H * 4, ns, ns};
    for (int i = 0; i < 6; ++i)
        if (overlaps(Y, ny, ins[i], in_bytes[i]) || overlaps(Y_h, ns, ins[i], in_bytes[i]) || overlaps(Y_c, ns, ins[i], in_bytes[i]) ||
            overlaps(scratch, (int64_t)need, ins[i], in_bytes[i]))
            return fail(ONNX_ERR_ALIAS, "lstm: an output or the scratch overlaps an input");
    if (overlaps(scratch, (int64_t)need, Y, ny) || overlaps(scratch, (int64_t)need, Y_h, ns) || overlaps(scratch, (int64_t)need, Y_c, ns))
        return fail(ONNX_ERR_ALIAS, "lstm: the scratch overlaps an output");
    // what the input projection's Gemm will ask of its operands (rows of X, W and of its result within 32-bit tile
    // offsets), checked here so that nothing has been enqueued when it is refused
    const int64_t span = (1LL << 31) - 64;
    if ((256 * in + in) * 4 >= span || (256 * 4 * H + 4 * H) * 4 >= span)
        return fail(ONNX_ERR_UNSUPPORTED, "lstm: input_size or hidden_size too large for the projection Gemm's 32-bit tile offsets");

    auto up = [](int64_t v) { return (v + 63) / 64 * 64; };
    const int64_t per_dir = scratch_floats_per_direction(seq, batch, H);
    const int n4h = (int)(4 * H), nbh = (int)(batch * H);
    float* Gd[2] = {nullptr, nullptr};
    float* hbuf[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};
    float* cbuf[2] = {nullptr, nullptr};
    for (int d = 0; d < dirs; ++d) {
        float* G = static_cast<float*>(scratch) + d * per_dir;
        float* P = G + up(seq * batch * 4 * H);          // (kept in the layout; the fused step kernel needs no staging of its own)
        float* hbuf0 = P + up(batch * 4 * H);
        float* hbuf1 = hbuf0 + up(batch * H);
        float* c = hbuf1 + up(batch * H);
        float* bias = c + up(batch * H);
        Gd[d] = G; hbuf[d][0] = hbuf0; hbuf[d][1] = hbuf1; cbuf[d] = c;
        const float* Wd = W + (int64_t)d * 4 * H * in;
        hipLaunchKernelGGL(lstm_bias_kernel, dim3((n4h + 255) / 256), dim3(256), 0, s, B ? B + (int64_t)d * 8 * H : nullptr, bias, n4h);
        hipLaunchKernelGGL(lstm_state_kernel, dim3((nbh + 255) / 256), dim3(256), 0, s,
                           initial_h ? initial_h + (int64_t)d * nbh : nullptr, hbuf0, nbh);
        hipLaunchKernelGGL(lstm_state_kernel, dim3((nbh + 255) / 256), dim3(256), 0, s,
                           initial_c ? initial_c + (int64_t)d * nbh : nullptr, c, nbh);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(ONNX_ERR_DEVICE, "lstm: %s", hipGetErrorString(e));
        // G = X [seq*batch, in] * W_d' + (Wb + Rb): the input projection of every time step at once
        const int64_t xd[2] = {seq * batch, in}, wd[2] = {4 * H, in}, bd[2] = {1, 4 * H}, gd[2] = {seq * batch, 4 * H};
        const onnx_status st = onnx_gemm(X, xd, Wd, wd, bias, bd, 2, 1.0f, 1.0f, 0, 1, ONNX_ACT_NONE, G, gd, stream);
        if (st != ONNX_OK) return st;
    }
    LstmStep p;
    p.batch = (int)batch; p.H = (int)H;
    p.KW = (int)(((H + 3) / 4 + 7) / 8 * 8);
    const bool vec = H % 4 == 0 && aligned16(R);
    const dim3 grid((unsigned)((H + 7) / 8), (unsigned)((batch + 31) / 32), (unsigned)dirs);
    if (grid.y > 65535u) return fail(ONNX_ERR_UNSUPPORTED, "lstm: batch above 2^21");
    for (int64_t step = 0; step < seq; ++step) {
        const bool last = step == seq - 1;
        for (int d = 0; d < 2; ++d) {
            const int dd = d < dirs ? d : 0;
            const bool backwards = direction == ONNX_LSTM_REVERSE || dd == 1;
            const int64_t t = backwards ? seq - 1 - step : step;
            p.hprev[d] = hbuf[dd][step & 1];
            p.hnext[d] = hbuf[dd][(step & 1) ^ 1];
            p.c[d] = cbuf[dd];
            p.R[d] = R + (int64_t)dd * 4 * H * H;
            p.G[d] = Gd[dd] + t * batch * 4 * H;
            p.y[d] = Y ? Y + ((t * dirs + dd) * batch) * H : nullptr;
            p.y_h[d] = last && Y_h ? Y_h + (int64_t)dd * nbh : nullptr;
            p.y_c[d] = last && Y_c ? Y_c + (int64_t)dd * nbh : nullptr;
        }
        if (vec) hipLaunchKernelGGL(lstm_step_kernel<4>, grid, dim3(256), 0, s, p);
        else hipLaunchKernelGGL(lstm_step_kernel<1>, grid, dim3(256), 0, s, p);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ONNX_ERR_DEVICE, "lstm: %s", hipGetErrorString(e));
    return ONNX_OK;
}

}  // extern "C"
