// ONNX LSTM (named among the supported operators in Section 4.1 of the paper): the input
// projection of the whole sequence is one Gemm, every time step is one small Gemm on the hidden
// state plus one element-wise cell kernel.  All arithmetic of the products runs in the
// contraction kernels (through onnx_gemm); this file adds the cell kernel, the bias and state
// preparation kernels and the sequencing.
#include <stdio.h>

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

// One time step of one direction.  P [batch, 4H] holds the gate pre-activations in the order
// i, o, f, c.  c is updated in place, h_out receives the new hidden state, and so do y (the
// slot of this step in Y) and the final-state outputs when they are wanted.
__global__ __launch_bounds__(256) void lstm_cell_kernel(const float* __restrict__ P, float* __restrict__ c,
                                                        float* __restrict__ h_out, float* __restrict__ y,
                                                        float* __restrict__ y_h, float* __restrict__ y_c, int batch,
                                                        int H) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= batch * H) return;
    const int b = idx / H, j = idx - b * H;
    const float* p = P + (int64_t)b * 4 * H + j;
    const float gi = sigmoidf(p[0]), go = sigmoidf(p[H]), gf = sigmoidf(p[2 * H]), gc = tanhf(p[3 * H]);
    const float cn = gf * c[idx] + gi * gc;
    const float hn = go * tanhf(cn);
    c[idx] = cn;
    h_out[idx] = hn;
    if (y) y[idx] = hn;
    if (y_h) y_h[idx] = hn;
    if (y_c) y_c[idx] = cn;
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
    if (seq * batch == 0) return ONNX_OK;
    if (batch * 4 * H > 0x7fffffffLL || seq * batch > 0x7fffffffLL || in > 0x7fffffffLL)
        return fail(ONNX_ERR_UNSUPPORTED, "lstm: extent above 2^31-1");
    if (!X || !W || !R) return fail(ONNX_ERR_NULL, "lstm: X, W and R must not be NULL");
    if (!Y && !Y_h && !Y_c) return fail(ONNX_ERR_NULL, "lstm: at least one of Y, Y_h, Y_c must be given");
    const size_t need = onnx_lstm_scratch_bytes(x_dims, H, direction);
    if (!scratch || scratch_bytes < need)
        return fail(ONNX_ERR_NULL, "lstm: %zu bytes of scratch are needed (onnx_lstm_scratch_bytes), %zu given", need,
                    scratch ? scratch_bytes : (size_t)0);
    if ((reinterpret_cast<uintptr_t>(scratch) & 255u) != 0) return fail(ONNX_ERR_ATTR, "lstm: scratch must be 256-byte aligned");
    const int64_t ny = seq * dirs * batch * H * 4, ns = dirs * batch * H * 4;
    const void* ins[] = {X, W, R, B, initial_h, initial_c};
    const int64_t in_bytes[] = {seq * batch * in * 4, dirs * 4 * H * in * 4, dirs * 4 * H * H * 4, dirs * 8 * H * 4, ns, ns};
    for (int i = 0; i < 6; ++i)
        if (overlaps(Y, ny, ins[i], in_bytes[i]) || overlaps(Y_h, ns, ins[i], in_bytes[i]) || overlaps(Y_c, ns, ins[i], in_bytes[i]) ||
            overlaps(scratch, (int64_t)need, ins[i], in_bytes[i]))
            return fail(ONNX_ERR_ALIAS, "lstm: an output or the scratch overlaps an input");
    if (overlaps(scratch, (int64_t)need, Y, ny) || overlaps(scratch, (int64_t)need, Y_h, ns) || overlaps(scratch, (int64_t)need, Y_c, ns))
        return fail(ONNX_ERR_ALIAS, "lstm: the scratch overlaps an output");

    hipStream_t s = static_cast<hipStream_t>(stream);
    auto up = [](int64_t v) { return (v + 63) / 64 * 64; };
    const int64_t per_dir = scratch_floats_per_direction(seq, batch, H);
    const int n4h = (int)(4 * H), nbh = (int)(batch * H);
    for (int d = 0; d < dirs; ++d) {
        float* G = static_cast<float*>(scratch) + d * per_dir;
        float* P = G + up(seq * batch * 4 * H);
        float* hbuf0 = P + up(batch * 4 * H);
        float* hbuf1 = hbuf0 + up(batch * H);
        float* c = hbuf1 + up(batch * H);
        float* bias = c + up(batch * H);
        const float* Wd = W + (int64_t)d * 4 * H * in;
        const float* Rd = R + (int64_t)d * 4 * H * H;
        hipLaunchKernelGGL(lstm_bias_kernel, dim3((n4h + 255) / 256), dim3(256), 0, s, B ? B + (int64_t)d * 8 * H : nullptr, bias, n4h);
        hipLaunchKernelGGL(lstm_state_kernel, dim3((nbh + 255) / 256), dim3(256), 0, s,
                           initial_h ? initial_h + (int64_t)d * nbh : nullptr, hbuf0, nbh);
        hipLaunchKernelGGL(lstm_state_kernel, dim3((nbh + 255) / 256), dim3(256), 0, s,
                           initial_c ? initial_c + (int64_t)d * nbh : nullptr, c, nbh);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(ONNX_ERR_DEVICE, "lstm: %s", hipGetErrorString(e));
        // G = X [seq*batch, in] * W_d' + (Wb + Rb): the input projection of every time step at once
        const int64_t xd[2] = {seq * batch, in}, wd[2] = {4 * H, in}, bd[2] = {1, 4 * H}, gd[2] = {seq * batch, 4 * H};
        onnx_status st = onnx_gemm(X, xd, Wd, wd, bias, bd, 2, 1.0f, 1.0f, 0, 1, ONNX_ACT_NONE, G, gd, stream);
        if (st != ONNX_OK) return st;
        const bool backwards = direction == ONNX_LSTM_REVERSE || d == 1;
        const int64_t hd[2] = {batch, H}, rd[2] = {4 * H, H}, pd[2] = {batch, 4 * H};
        float* hprev = hbuf0;
        float* hnext = hbuf1;
        for (int64_t step = 0; step < seq; ++step) {
            const int64_t t = backwards ? seq - 1 - step : step;
            // P = h * R_d' + G_t
            st = onnx_gemm(hprev, hd, Rd, rd, G + t * batch * 4 * H, pd, 2, 1.0f, 1.0f, 0, 1, ONNX_ACT_NONE, P, pd, stream);
            if (st != ONNX_OK) return st;
            const bool last = step == seq - 1;
            hipLaunchKernelGGL(lstm_cell_kernel, dim3((nbh + 255) / 256), dim3(256), 0, s, P, c, hnext,
                               Y ? Y + ((t * dirs + d) * batch) * H : nullptr, last && Y_h ? Y_h + (int64_t)d * nbh : nullptr,
                               last && Y_c ? Y_c + (int64_t)d * nbh : nullptr, (int)batch, (int)H);
            float* tmp = hprev; hprev = hnext; hnext = tmp;
        }
        e = hipGetLastError();
        if (e != hipSuccess) return fail(ONNX_ERR_DEVICE, "lstm: %s", hipGetErrorString(e));
    }
    return ONNX_OK;
}

}  // extern "C"
