// Contractions on 16-bit inputs in any operand layout: the kernel behind the cases of onnx_gemm_lp,
// onnx_matmul_lp and onnx_conv_lp that the tuned kernel (gemm_lp.h) does not take: a transposed A,
// K not a multiple of 8, rows of a row-contiguous B that are not a multiple of 4 long, unaligned
// operands, and every convolution whose input has to be gathered (anything but 1x1 / stride 1 /
// no padding).
// The paper's operator definitions admit 16-bit floating-point tensors (Section 3.1); Conv,
// MatMul and Gemm keep their ONNX semantics, products are exact in fp32 and summed in fp32
// accumulators (v_mfma_f32_32x32x16_{f16,bf16}).
//
// The 16-bit MFMA wants, from both operands, 8 consecutive k per lane.  Operands that are not
// K-contiguous in memory (Gemm's transA = 1 or transB = 0, MatMul's B, the input of every
// convolution) are therefore transposed on their way into LDS: this kernel loads 16-bit
// elements one by one with coalesced 2-byte loads along whichever index is contiguous in
// memory (rows for a row-contiguous operand and for the gathered convolution input, k
// otherwise) and stores them into LDS as [row][k], where a lane's 8 k are one 16-byte read.
// Tile 64 x 64 x 32, four wavefronts of 32 x 32, one LDS buffer, no split-K: a plain, general
// path.
#include "gemm_lp.h"
#include "internal.h"

namespace onnxhip {

namespace {

constexpr int GB = 64;             // tile rows and columns
constexpr int GK = 32;             // K step
constexpr int GPITCH = GK + 8;     // LDS row pitch in 16-bit values (80 bytes: 16-byte aligned rows)

// Element loader of one operand tile (64 rows x 32 k), 256 threads, 8 values per thread and step.
template <int KIND, bool IS_B>
struct LpElementLoader {
    const uint16_t* base;          // operand of this z-slice
    int64_t off[8];                // KC: element offset of (row_i, k = lane k) at k0 = 0; RC: of (row, k_i); IM2COL: window origin
    bool ok[8];
    int kk, rr;                    // this thread's k (KC) or row (RC / IM2COL) within the tile, and the other index's start
    int K, ld;
    int ih0, iw0;
    bool col_ok;

    __device__ inline void init(const uint16_t* p, int64_t ld_, int row0, int rows_total, int K_, const ContractionParams& cp) {
        base = p; K = K_; ld = (int)ld_;
        const int t = threadIdx.x;
        ih0 = iw0 = 0; col_ok = true;
        if (KIND == LOAD_KC) {
            kk = t % GK; rr = t / GK;                       // rows rr + 8 i
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = row0 + rr + 8 * i;
                ok[i] = row < rows_total;
                off[i] = (int64_t)row * ld_ + kk;
            }
        } else {
            rr = t % GB; kk = t / GB;                       // k = kk + 4 i
            const int j = row0 + rr;
            col_ok = j < rows_total;
            const uint32_t jj = col_ok ? (uint32_t)j : (uint32_t)row0;
            int64_t col_off = jj;
            if (IS_B && cp.col_images) {
                uint32_t n, px;
                cp.colP.divmod(jj, n, px);
                if (KIND == LOAD_IM2COL) {
                    uint32_t oh, ow;
                    cp.ic.OW.divmod(px, oh, ow);
                    ih0 = (int)oh * cp.ic.sH - cp.ic.pT;
                    iw0 = (int)ow * cp.ic.sW - cp.ic.pL;
                    col_off = (int64_t)n * cp.ic.image_stride + (int64_t)ih0 * cp.ic.W + iw0;
                } else {
                    col_off = (int64_t)n * cp.b_img + px;
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                ok[i] = col_ok;
                off[i] = col_off + (KIND == LOAD_IM2COL ? 0 : (int64_t)(kk + 4 * i) * ld_);
            }
        }
    }

    // the 8 values of the K step that starts at k0
    __device__ inline void fetch(int k0, const ContractionParams& cp, uint16_t v[8]) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (KIND == LOAD_KC) {
                v[i] = (ok[i] && k0 + kk < K) ? base[off[i] + k0] : (uint16_t)0;
            } else if (KIND == LOAD_RC) {
                v[i] = (ok[i] && k0 + kk + 4 * i < K) ? base[off[i] + (int64_t)k0 * ld] : (uint16_t)0;
            } else {
                const uint32_t k = (uint32_t)(k0 + kk + 4 * i);
                uint32_t c, rem, kh, kw;
                cp.ic.kHW.divmod(k, c, rem);
                cp.ic.kW.divmod(rem, kh, kw);
                const int dh = (int)kh * cp.ic.dH, dw = (int)kw * cp.ic.dW;
                const int ih = ih0 + dh, iw = iw0 + dw;
                const bool good = ok[i] && (int)k < K && (unsigned)ih < (unsigned)cp.ic.H && (unsigned)iw < (unsigned)cp.ic.W;
                v[i] = good ? base[off[i] + ((int64_t)c * cp.ic.H + dh) * cp.ic.W + dw] : (uint16_t)0;
            }
        }
    }

    __device__ inline void commit(uint16_t* lds, const uint16_t v[8]) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (KIND == LOAD_KC) lds[(rr + 8 * i) * GPITCH + kk] = v[i];
            else lds[rr * GPITCH + kk + 4 * i] = v[i];
        }
    }
};

template <int DT, bool LP_OUT, int AKIND, int BKIND>
__global__ __launch_bounds__(256) void lp_generic_kernel(const ContractionParams cp) {
    __shared__ __attribute__((aligned(16))) uint16_t lds_a[GB * GPITCH];
    __shared__ __attribute__((aligned(16))) uint16_t lds_b[GB * GPITCH];

    const int zslice = blockIdx.y * gridDim.z + blockIdx.z;
    if (zslice >= cp.nz) return;
    const int tile_m = blockIdx.x / cp.tiles_n, tile_n = blockIdx.x % cp.tiles_n;
    const int m0 = tile_m * GB, n0 = tile_n * GB;
    int64_t a_off, b_off;
    slice_offsets(cp, zslice, a_off, b_off);

    LpElementLoader<AKIND, false> la;
    LpElementLoader<BKIND, true> lb;
    la.init(reinterpret_cast<const uint16_t*>(cp.A) + a_off, cp.a_ld, m0, cp.M, cp.K, cp);
    lb.init(reinterpret_cast<const uint16_t*>(cp.B) + b_off, cp.b_ld, n0, cp.N, cp.K, cp);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, h = lane >> 5;
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    const int nk = (cp.K + GK - 1) / GK;
    for (int kt = 0; kt < nk; ++kt) {
        uint16_t va[8], vb[8];
        la.fetch(kt * GK, cp, va);
        lb.fetch(kt * GK, cp, vb);
        __syncthreads();                                    // the previous step's fragments have been read
        la.commit(lds_a, va);
        lb.commit(lds_b, vb);
        __syncthreads();
#pragma unroll
        for (int g = 0; g < GK / 16; ++g) {
            const floatx4 fa = *reinterpret_cast<const floatx4*>(lds_a + (wm * 32 + li) * GPITCH + g * 16 + h * 8);
            const floatx4 fb = *reinterpret_cast<const floatx4*>(lds_b + (wn * 32 + li) * GPITCH + g * 16 + h * 8);
            acc = mfma16<DT>(fa, fb, acc);
        }
    }

    // ---- epilogue: alpha*acc + beta*bias (+ residual), Relu, store as fp32 or rounded to the input type
    const int col = n0 + wn * 32 + li;
    if (col >= cp.N) return;
    int64_t col_off = col;
    if (cp.col_images) {
        uint32_t n, px;
        cp.colP.divmod((uint32_t)col, n, px);
        col_off = (int64_t)n * cp.y_img + px;
    }
    const int64_t zi = zslice;
    const int mode = cp.bias ? cp.bias_mode : BIAS_NONE;
    const float* bias = cp.bias ? cp.bias + zi * cp.bias_zs : nullptr;
    const float col_bias = mode == BIAS_COL ? cp.beta * bias[(int64_t)col * cp.bias_cs] : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 32 + 8 * (r / 4) + 4 * h + r % 4;
        if (row >= cp.M) continue;
        const int64_t o = zi * cp.y_zs + (int64_t)row * cp.y_rs + col_off;
        float add = col_bias;
        if (mode == BIAS_ROW) add = cp.beta * bias[row];
        if (mode == BIAS_FULL) add = cp.beta * bias[(int64_t)row * cp.N + col];
        float v = fmaf(cp.alpha, acc[r], add);
        if (cp.residual) {
            if (LP_OUT) {
                const uint16_t rv = reinterpret_cast<const uint16_t*>(cp.residual)[o];
                v += DT == LP_F16 ? (float)__builtin_bit_cast(_Float16, rv) : __builtin_bit_cast(float, (uint32_t)rv << 16);
            } else {
                v += cp.residual[o];
            }
        }
        if (cp.relu) v = fmaxf(v, 0.f);
        if (LP_OUT) reinterpret_cast<uint16_t*>(cp.Y)[o] = to_lp<DT>(v);
        else cp.Y[o] = v;
    }
}

template <int DT, bool LP_OUT>
hipError_t launch_kinds(const ContractionParams& p, int akind, int bkind, dim3 grid, hipStream_t stream) {
#define ONNXHIP_LP_CASE(AK, BKK)                                                                            \
    if (akind == AK && bkind == BKK) {                                                                      \
        hipLaunchKernelGGL((lp_generic_kernel<DT, LP_OUT, AK, BKK>), grid, dim3(256), 0, stream, p);        \
        return hipGetLastError();                                                                           \
    }
    ONNXHIP_LP_CASE(LOAD_KC, LOAD_KC)
    ONNXHIP_LP_CASE(LOAD_KC, LOAD_RC)
    ONNXHIP_LP_CASE(LOAD_RC, LOAD_KC)
    ONNXHIP_LP_CASE(LOAD_RC, LOAD_RC)
    ONNXHIP_LP_CASE(LOAD_KC, LOAD_IM2COL)
#undef ONNXHIP_LP_CASE
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_lp_generic(ContractionParams& p, int akind, int bkind, int nz, int in_type, int out_type,
                             hipStream_t stream) {
    p.tiles_m = (p.M + GB - 1) / GB;
    p.tiles_n = (p.N + GB - 1) / GB;
    p.nz = nz;
    p.ksplit = 1;
    p.ws_partial = nullptr;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    p.tail_begin = (int)tiles;
    p.tail_split = 1;
    const unsigned gz = nz < 32768 ? (unsigned)nz : 32768u;
    const unsigned gy = ((unsigned)nz + gz - 1) / gz;
    if (gy > 65535u) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles, gy, gz);
    const bool lp_out = out_type != 0;
    record_launch(LaunchRecord{"lp_generic", GB, GB, GK, 2, 2, 1, akind, bkind, 1, 1, in_type + (lp_out ? 2 : 0), 1, 0, 1});
    if (in_type == LP_F16) return lp_out ? launch_kinds<LP_F16, true>(p, akind, bkind, grid, stream) : launch_kinds<LP_F16, false>(p, akind, bkind, grid, stream);
    return lp_out ? launch_kinds<LP_BF16, true>(p, akind, bkind, grid, stream) : launch_kinds<LP_BF16, false>(p, akind, bkind, grid, stream);
}

}  // namespace onnxhip
