// A whole small model as one launch: onnx_chain.  The paper compiles a model into a single entry
// function (Section 3) and reports the MNIST network as its small example (Section 4.2: two
// convolutions with Relu, two max pools, a matrix product with bias).  For such a model one
// launch per operator costs more than the arithmetic: five launches of a few microseconds each
// for under a million multiply-adds.  Here one workgroup of 16 wavefronts runs the chain for one
// image with everything on chip:
//   * at the start every weight and bias of the chain and the image are fetched into LDS in one
//     go (wavefronts take 64-float chunks of the list of tensors; all loads of a thread are
//     issued before the first is used), so global-memory latency is paid once;
//   * activations ping-pong between two LDS buffers.  A buffer that feeds a Conv is laid out with
//     that Conv's zero padding around every plane, so the Conv needs no bounds checks;
//   * Conv is an implicit GEMM on the matrix cores (v_mfma_f32_16x16x4_f32): a wavefront owns 16
//     output channels x 16 output positions, lane (j, kk) supplies filter value W[m0+j][k0+kk] and
//     input value in[origin(pos j) + offset(k0+kk)], offset(k) = c*plane + kh*dH*pitch + kw*dW
//     from a table built per Conv;
//   * pools are one thread per output over the LDS buffer, Gemm one wavefront per output column
//     with a cross-lane sum.
// Operator semantics are those of onnx_conv / onnx_maxpool / onnx_avgpool / onnx_gemm.
#include "internal.h"
#include "../../include/onnxhip.h"

namespace onnxhip {

namespace {

constexpr int CHAIN_THREADS = 1024;
constexpr int CHAIN_WAVES = CHAIN_THREADS / 64;
constexpr int ACT_MAX = ONNX_CHAIN_MAX_ACTIVATION;
constexpr int ARENA_MAX = ONNX_CHAIN_MAX_WEIGHTS;
constexpr int KOFF_MAX = ONNX_CHAIN_MAX_CONV_K;
constexpr int MAX_OPS = ONNX_CHAIN_MAX_OPS;
constexpr int MAX_COPIES = 2 * MAX_OPS + 1;
constexpr int STAGE_BATCH = 8;            // chunks a wavefront has in flight

// One tensor staged into LDS: `count` floats read contiguously from src, stored as rows of
// `row` floats, `pitch` apart, `rows` rows per plane, planes `plane` apart, from float offset dst.
struct ChainCopy {
    const float* src;
    int count, chunk0;       // chunk0: index of this tensor's first 64-float chunk in the whole list
    int dst, pitch, plane;
    int per_image;           // src advances by count per image (the input tensor)
    int mode;                // 0: stored contiguously, 1: rows of one plane, 2: rows and planes, 3: transposed (element x of row r at dst + x*pitch + r)
    FastDiv row, rows;
};

struct ChainOp {
    int kind, act;
    int C, H, W;                                   // input
    int in_pitch, in_plane, in_off;                // element (c,h,w) of the input buffer: in_off + c*in_plane + h*in_pitch + w
    int M, OH, OW;                                 // output (Gemm: M outputs, OH = OW = 1)
    int out_pitch, out_plane, out_off, out_zero;   // same for the output buffer; out_zero: floats to clear first (0: no padding)
    int kH, kW, sH, sW, pT, pL, pB, pR, dH, dW;
    int K, Kp;                                     // Conv: C*kH*kW and the LDS pitch of a filter row; Gemm: C*H*W
    int w_off, b_off;                              // LDS offsets of weights and bias (b_off < 0: no bias)
    int transB, cip;
    int interior;                                  // pools: every window lies inside the input
    int direct;                                    // Conv: at most 8 output channels and a short K: one thread per position
    float alpha, beta;
    float* Y;                                      // NULL or [images][M][OH][OW]
    int y_img;
    FastDiv dOW, dOHW, dkHW, dkW;
};

struct ChainParams {
    int n_ops, n_copies, total_chunks, in_zero;
    ChainOp ops[MAX_OPS];
    ChainCopy copies[MAX_COPIES];
};

typedef float floatx4v __attribute__((ext_vector_type(4)));

// What a Conv of the chain needs to know, all of it the same for every lane.
struct ConvSite {
    const float* in;         // input buffer, laid out with this Conv's padding
    float* out;              // output buffer
    float* yimg;             // NULL or this image's result in device memory
    const float* w;          // filter rows in LDS, Kp apart
    const float* bias;       // NULL or [M] in LDS
    const int* koff;         // input offset of every k
    FastDiv dOW;
    int M, P, K, Kp, sH, sW, in_pitch, out_off, out_plane, out_pitch, relu;
};

// Items (16 output channels x G tiles of 16 positions) wave, wave + 16, ... of one Conv.  The K walk
// takes 16 k per trip (four MFMAs per tile); lane (j, kk) owns the four consecutive k 16*trip + 4*kk
// + u, u = 0..3, of every trip: its filter values and its input offsets are one 16-byte LDS read
// each.  The reads of trip t+1 (filter values, and input values at the offsets fetched during
// trip t-1) are issued before the MFMAs of trip t.  Filter rows and the offset table are padded to
// whole trips; what lies beyond K is masked out of both operands.
typedef int intx4v __attribute__((ext_vector_type(4)));

template <int G>
__device__ inline void conv_items(const ConvSite& c, int wave, int lane, int tiles_p, int mblocks) {
    const int j = lane & 15, kk = lane >> 4;
    const int groups = (tiles_p + G - 1) / G;
    const int K = c.K, ntrip = (K + 15) >> 4;
    int mb = 0, gp = wave;                                  // item = mb * groups + gp
    while (gp >= groups) { gp -= groups; ++mb; }
    while (mb < mblocks) {
        int base[G], opos[G], pos[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            pos[g] = (gp * G + g) * 16 + j;
            uint32_t oh, ow;
            c.dOW.divmod((uint32_t)(pos[g] < c.P ? pos[g] : c.P - 1), oh, ow);
            base[g] = (int)oh * c.sH * c.in_pitch + (int)ow * c.sW;
            opos[g] = (int)oh * c.out_pitch + (int)ow;
        }
        const int m = mb * 16 + j;
        const float* ap = c.w + (m < c.M ? m : c.M - 1) * c.Kp + 4 * kk;
        const int* kp = c.koff + 4 * kk;
        const bool a_row = m < c.M;
        floatx4v acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = floatx4v{0.f, 0.f, 0.f, 0.f};

        // Register sets 0 and 1 take turns: while the MFMAs of one trip read set s, the reads of the
        // next trip fill set 1 - s.  Only the last trip can reach beyond K and is masked.
        floatx4v a[2];
        intx4v ko[2];
        float b[2][G][4];
        auto fetch_ab = [&](int s, int trip, const intx4v& off) {
            a[s] = *reinterpret_cast<const floatx4v*>(ap + 16 * trip);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int g = 0; g < G; ++g) b[s][g][u] = c.in[base[g] + off[u]];
        };
        auto fetch_ko = [&](int s, int trip) { ko[s] = *reinterpret_cast<const intx4v*>(kp + 16 * trip); };
        auto mfmas = [&](int s) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float av = a_row ? a[s][u] : 0.f;
#pragma unroll
                for (int g = 0; g < G; ++g) acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, b[s][g][u], acc[g], 0, 0, 0);
            }
        };
        fetch_ko(0, 0);
        fetch_ab(0, 0, ko[0]);
        if (ntrip > 1) fetch_ko(1, 1);
        int trip = 0;
        // two trips per round; set 0 holds the operands of trip `trip`, ko[1] the offsets of trip + 1
        for (; trip + 2 < ntrip; trip += 2) {
            fetch_ab(1, trip + 1, ko[1]);
            fetch_ko(0, trip + 2);
            mfmas(0);
            fetch_ab(0, trip + 2, ko[0]);
            if (trip + 3 < ntrip) fetch_ko(1, trip + 3);
            mfmas(1);
        }
        // one or two trips are left: `trip` (in set 0) and possibly trip + 1; the last one is masked
        int last = 0;
        if (trip + 1 < ntrip) {
            fetch_ab(1, trip + 1, ko[1]);
            mfmas(0);
            last = 1;
        }
        {
            const int kin = K - 4 * kk - 16 * (ntrip - 1);      // this lane's k of the last trip that lie below K
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float av = (a_row && u < kin) ? (last ? a[1][u] : a[0][u]) : 0.f;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float bv = u < kin ? (last ? b[1][g][u] : b[0][g][u]) : 0.f;
                    acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[g], 0, 0, 0);
                }
            }
        }
        // results: lane (j, kk) holds channels mb*16 + 4*kk + r, r = 0..3, of position j of each tile
        const int mch0 = mb * 16 + 4 * kk;
        float bias[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) bias[r] = (c.bias && mch0 + r < c.M) ? c.bias[mch0 + r] : 0.f;
        float* orow = c.out + c.out_off + mch0 * c.out_plane;
        float* yrow = c.yimg ? c.yimg + mch0 * c.P : nullptr;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (pos[g] < c.P) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (mch0 + r < c.M) {
                        float v = acc[g][r] + bias[r];
                        if (c.relu) v = fmaxf(v, 0.f);
                        orow[r * c.out_plane + opos[g]] = v;
                        if (yrow) yrow[r * c.P + pos[g]] = v;
                    }
                }
            }
        }
        gp += CHAIN_WAVES;
        while (gp >= groups) { gp -= groups; ++mb; }
    }
}

// A Conv with at most 8 output channels and a short reduction: the matrix-core path would leave half
// of every MFMA empty and spend its time in set-up and epilogue.  One thread per output position
// instead: per k one input value, the k-th column of the filter matrix (stored [k][8] in LDS: two
// 16-byte reads that every lane shares) and 8 FMAs.
__device__ inline void conv_direct8(const ConvSite& c, int t) {
    for (int pos = t; pos < c.P; pos += CHAIN_THREADS) {
        uint32_t oh, ow;
        c.dOW.divmod((uint32_t)pos, oh, ow);
        const float* bp = c.in + (int)oh * c.sH * c.in_pitch + (int)ow * c.sW;
        float acc[8];
#pragma unroll
        for (int m = 0; m < 8; ++m) acc[m] = 0.f;
        auto tap = [&](int k, int off) {
            const float x = bp[off];
            const floatx4v w0 = *reinterpret_cast<const floatx4v*>(c.w + 8 * k);
            const floatx4v w1 = *reinterpret_cast<const floatx4v*>(c.w + 8 * k + 4);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                acc[m] = fmaf(w0[m], x, acc[m]);
                acc[4 + m] = fmaf(w1[m], x, acc[4 + m]);
            }
        };
        int k = 0;
        for (; k + 4 <= c.K; k += 4) {
            const intx4v off = *reinterpret_cast<const intx4v*>(c.koff + k);
#pragma unroll
            for (int u = 0; u < 4; ++u) tap(k + u, off[u]);
        }
        for (; k < c.K; ++k) tap(k, c.koff[k]);
        float* o = c.out + c.out_off + (int)oh * c.out_pitch + (int)ow;
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            if (m < c.M) {
                float v = acc[m] + (c.bias ? c.bias[m] : 0.f);
                if (c.relu) v = fmaxf(v, 0.f);
                o[m * c.out_plane] = v;
                if (c.yimg) c.yimg[m * c.P + pos] = v;
            }
        }
    }
}

__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Sum of a value over the 64 lanes, the same in every lane, without LDS traffic: rotations inside
// each row of 16 lanes (DPP row_ror 8, 4, 2, 1), then the four row totals through scalar registers.
__device__ inline float wave_sum(float v) {
#define ONNXHIP_ROW_ROR(n) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + (n), 0xf, 0xf, false))
    ONNXHIP_ROW_ROR(8);
    ONNXHIP_ROW_ROR(4);
    ONNXHIP_ROW_ROR(2);
    ONNXHIP_ROW_ROR(1);
#undef ONNXHIP_ROW_ROR
    const int b = __builtin_bit_cast(int, v);
    return (__builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0)) + __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16))) +
           (__builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32)) + __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48)));
}

// The argument block is read once, by all threads together, into LDS: it is a few KB that the
// scalar unit would otherwise fetch line by line, one memory latency after the other, as the
// chain walks through its descriptors.
__global__ __launch_bounds__(CHAIN_THREADS) void chain_kernel(const ChainParams) {
    __shared__ __attribute__((aligned(16))) float lds[2 * ACT_MAX + ARENA_MAX];
    __shared__ __attribute__((aligned(16))) int koff[KOFF_MAX];
    __shared__ __attribute__((aligned(16))) ChainParams sp;

    const int t = threadIdx.x, lane = t & 63;
    const int wave = uni(t >> 6);
    const int image = blockIdx.x;
    {
        typedef const __attribute__((address_space(4))) uint32_t* KernargPtr;
        KernargPtr kp = (KernargPtr)__builtin_amdgcn_kernarg_segment_ptr();
        uint32_t* d = reinterpret_cast<uint32_t*>(&sp);
        for (int i = t; i < (int)(sizeof(ChainParams) / 4); i += CHAIN_THREADS) d[i] = kp[i];
    }
    __syncthreads();

    // ---- stage the weights, the biases and the image
    const int total_chunks = uni(sp.total_chunks), n_copies = uni(sp.n_copies), in_zero = uni(sp.in_zero);
    // lane i knows where tensor i starts in the chunk list: the tensor of chunk q is the number of
    // lanes whose tensor starts at or before q, minus one
    const int my_chunk0 = lane < n_copies ? sp.copies[lane].chunk0 : 0x7fffffff;
    for (int q0 = 0; q0 < total_chunks; q0 += CHAIN_WAVES * STAGE_BATCH) {
        float v[STAGE_BATCH];
        int d[STAGE_BATCH];
#pragma unroll
        for (int u = 0; u < STAGE_BATCH; ++u) {
            const int q = q0 + wave + CHAIN_WAVES * u;           // the same for the whole wavefront
            d[u] = -1;
            v[u] = 0.f;
            if (q < total_chunks) {
                const int s = __builtin_popcountll(__ballot(my_chunk0 <= q)) - 1;
                const ChainCopy& c = sp.copies[s];
                const int e = (q - c.chunk0) * 64 + lane;
                if (e < c.count) {
                    const float* src = c.src + (c.per_image ? (int64_t)image * c.count : 0);
                    v[u] = src[e];
                    const int mode = uni(c.mode);
                    if (mode == 0) {
                        d[u] = c.dst + e;
                    } else {
                        uint32_t r, x, pl = 0, h;
                        c.row.divmod((uint32_t)e, r, x);
                        h = r;
                        if (mode == 2) c.rows.divmod(r, pl, h);
                        d[u] = mode == 3 ? c.dst + (int)x * c.pitch + (int)r : c.dst + (int)pl * c.plane + (int)h * c.pitch + (int)x;
                    }
                }
            }
        }
        if (q0 == 0) {
            for (int i = t; i < in_zero; i += CHAIN_THREADS) lds[i] = 0.f;
            __syncthreads();
        }
#pragma unroll
        for (int u = 0; u < STAGE_BATCH; ++u)
            if (d[u] >= 0) lds[d[u]] = v[u];
    }
    __syncthreads();

    const float* arena = lds + 2 * ACT_MAX;
    const int n_ops = uni(sp.n_ops);
    for (int o = 0; o < n_ops; ++o) {
        const ChainOp& op = sp.ops[o];
        const int kind = uni(op.kind), relu = uni(op.act) == ONNX_ACT_RELU;
        const int M = uni(op.M), OW = uni(op.OW), P = uni(op.OH) * OW, K = uni(op.K);
        const int in_pitch = uni(op.in_pitch), in_plane = uni(op.in_plane), in_off = uni(op.in_off);
        const int out_pitch = uni(op.out_pitch), out_plane = uni(op.out_plane), out_off = uni(op.out_off);
        const int out_zero = uni(op.out_zero), w_off = uni(op.w_off), b_off = uni(op.b_off);
        const int sH = uni(op.sH), sW = uni(op.sW), dH = uni(op.dH), dW = uni(op.dW);
        const FastDiv dOW = op.dOW;
        const float* in = lds + (o & 1) * ACT_MAX;
        float* out = lds + ((o + 1) & 1) * ACT_MAX;
        float* yimg = op.Y ? op.Y + (int64_t)image * op.y_img : nullptr;

        for (int i = t; i < out_zero; i += CHAIN_THREADS) out[i] = 0.f;
        if (kind == ONNX_CHAIN_CONV) {
            const FastDiv dkHW = op.dkHW, dkW = op.dkW;
            const int K16 = (K + 15) & ~15;
            for (int k = t; k < K16; k += CHAIN_THREADS) {
                const uint32_t kc = (uint32_t)(k < K ? k : K - 1);
                uint32_t c, rem, kh, kw;
                dkHW.divmod(kc, c, rem);
                dkW.divmod(rem, kh, kw);
                koff[k] = (int)c * in_plane + (int)kh * dH * in_pitch + (int)kw * dW;
            }
        }
        if (out_zero > 0 || kind == ONNX_CHAIN_CONV) __syncthreads();

        if (kind == ONNX_CHAIN_CONV) {
            const int Kp = uni(op.Kp);
            const int tiles_p = (P + 15) >> 4, mblocks = (M + 15) >> 4;
            const ConvSite cs{in, out, yimg, arena + w_off, b_off >= 0 ? arena + b_off : nullptr, koff, dOW,
                              M, P, K, Kp, sH, sW, in_pitch, out_off, out_plane, out_pitch, relu};
            // position tiles per item: as many as still leave an item for every wavefront
            if (uni(op.direct)) conv_direct8(cs, t);
            else if (tiles_p * mblocks >= 4 * CHAIN_WAVES - 15) conv_items<4>(cs, wave, lane, tiles_p, mblocks);
            else if (tiles_p * mblocks >= 2 * CHAIN_WAVES - 7) conv_items<2>(cs, wave, lane, tiles_p, mblocks);
            else conv_items<1>(cs, wave, lane, tiles_p, mblocks);
        } else if (kind == ONNX_CHAIN_MAXPOOL || kind == ONNX_CHAIN_AVGPOOL) {
            const FastDiv dOHW = op.dOHW;
            const int H = uni(op.H), W = uni(op.W), kH = uni(op.kH), kW = uni(op.kW);
            const int pT = uni(op.pT), pL = uni(op.pL), pB = uni(op.pB), pR = uni(op.pR), cip = uni(op.cip);
            const int interior = uni(op.interior);
            for (int e = t; e < M * P; e += CHAIN_THREADS) {
                uint32_t c, rem, oh, ow;
                dOHW.divmod((uint32_t)e, c, rem);
                dOW.divmod(rem, oh, ow);
                const int ih0 = (int)oh * sH - pT, iw0 = (int)ow * sW - pL;
                const float* xc = in + in_off + (int)c * in_plane;
                float v;
                if (interior) {                                 // no tap can fall outside: no checks, no counting
                    const float* x0 = xc + ih0 * in_pitch + iw0;
                    float acc = kind == ONNX_CHAIN_MAXPOOL ? x0[0] : 0.f;
                    for (int kh = 0; kh < kH; ++kh) {
                        const float* xr = x0 + kh * dH * in_pitch;
                        for (int kw = 0; kw < kW; ++kw) {
                            const float x = xr[kw * dW];
                            if (kind == ONNX_CHAIN_MAXPOOL) acc = x > acc ? x : acc;
                            else acc += x;
                        }
                    }
                    v = kind == ONNX_CHAIN_MAXPOOL ? acc : acc / (float)(kH * kW);
                } else
                if (kind == ONNX_CHAIN_MAXPOOL) {
                    bool found = false;
                    float best = 0.f;
                    for (int kh = 0; kh < kH; ++kh) {
                        const int ih = ih0 + kh * dH;
                        if (ih < 0 || ih >= H) continue;
                        for (int kw = 0; kw < kW; ++kw) {
                            const int iw = iw0 + kw * dW;
                            if (iw < 0 || iw >= W) continue;
                            const float x = xc[ih * in_pitch + iw];
                            if (!found || x > best) { best = x; found = true; }
                        }
                    }
                    v = best;
                } else {
                    float acc = 0.f;
                    int cnt = 0, cnt_padded = 0;
                    for (int kh = 0; kh < kH; ++kh) {
                        const int ih = ih0 + kh;
                        if (ih >= H + pB) continue;
                        for (int kw = 0; kw < kW; ++kw) {
                            const int iw = iw0 + kw;
                            if (iw >= W + pR) continue;
                            ++cnt_padded;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            acc += xc[ih * in_pitch + iw];
                            ++cnt;
                        }
                    }
                    v = acc / (float)(cip ? cnt_padded : cnt);
                }
                out[out_off + (int)c * out_plane + (int)oh * out_pitch + (int)ow] = v;
                if (yimg) yimg[e] = v;
            }
        } else {  // ONNX_CHAIN_GEMM: the input buffer is the plain row-major [C][H][W] = one row of K values
            const float* wt = arena + w_off;
            const int transB = uni(op.transB);
            const float alpha = op.alpha, beta = op.beta;
            for (int nn = wave; nn < M; nn += CHAIN_WAVES) {
                float acc = 0.f;
                for (int k = lane; k < K; k += 64)
                    acc = fmaf(in[in_off + k], transB ? wt[nn * K + k] : wt[k * M + nn], acc);
                acc = wave_sum(acc);
                if (lane == 0) {
                    float v = alpha * acc;
                    if (b_off >= 0) v = fmaf(beta, arena[b_off + nn], v);
                    if (relu) v = fmaxf(v, 0.f);
                    out[out_off + nn * out_plane] = v;
                    if (yimg) yimg[nn] = v;
                }
            }
        }
        __syncthreads();
    }
}

#define fail(st, ...) static_cast<onnx_status>(fail_with((st), __VA_ARGS__))

// pads a consumer wants around each plane of its input buffer: a Conv's own, nothing otherwise
void consumer_pads(const onnx_chain_op* ops, int n_ops, int o, int64_t pads[4]) {
    for (int i = 0; i < 4; ++i) pads[i] = 0;
    if (o < n_ops && ops[o].kind == ONNX_CHAIN_CONV)
        for (int i = 0; i < 4; ++i) pads[i] = ops[o].pads[i];
}

}  // namespace

}  // namespace onnxhip

using namespace onnxhip;

extern "C" onnx_status onnx_chain(const onnx_chain_op* ops, int n_ops, const float* X, const int64_t x_dims[4],
                                  void* stream) {
    if (!ops || !x_dims) return fail(ONNX_ERR_NULL, "chain: ops or x_dims is NULL");
    if (n_ops < 1 || n_ops > MAX_OPS)
        return fail(ONNX_ERR_UNSUPPORTED, "chain: %d operators (1..%d are supported)", n_ops, MAX_OPS);
    for (int i = 0; i < 4; ++i)
        if (x_dims[i] < 0) return fail(ONNX_ERR_SHAPE, "chain: x_dims[%d] is negative", i);
    const int64_t images = x_dims[0];
    ChainParams p;
    p.n_ops = n_ops;
    p.n_copies = 0;
    int64_t dims[4] = {images, x_dims[1], x_dims[2], x_dims[3]};
    int64_t arena = 0, chunks = 0;
    bool empty = images == 0;

    // ---- walk the chain: shapes, buffer layouts, what goes where in LDS
    int64_t lay[4];
    consumer_pads(ops, n_ops, 0, lay);
    auto padded_size = [](const int64_t d[4], const int64_t pd[4]) {
        return d[1] * (d[2] + pd[0] + pd[2]) * (d[3] + pd[1] + pd[3]);
    };
    if (padded_size(dims, lay) > ACT_MAX || dims[1] * dims[2] * dims[3] <= 0)
        return dims[1] * dims[2] * dims[3] <= 0
                   ? fail(ONNX_ERR_SHAPE, "chain: the input has no elements per image")
                   : fail(ONNX_ERR_UNSUPPORTED, "chain: the input (with the first Conv's padding) exceeds %d floats", ACT_MAX);
    auto add_copy = [&](const float* src, int64_t count, int64_t dst, int64_t row, int64_t pitch, int64_t rows,
                        int64_t plane, int per_image) {
        ChainCopy& c = p.copies[p.n_copies++];
        c.src = src; c.count = (int)count; c.chunk0 = (int)chunks; c.dst = (int)dst;
        c.pitch = (int)pitch; c.plane = (int)plane; c.per_image = per_image;
        c.row = FastDiv::make((uint32_t)row); c.rows = FastDiv::make((uint32_t)rows);
        const bool one_plane = rows * row >= count;
        c.mode = (row >= count || (pitch == row && (one_plane || plane == rows * row))) ? 0 : (one_plane ? 1 : 2);
        chunks += (count + 63) / 64;
    };
    {
        const int64_t pitch = dims[3] + lay[1] + lay[3], plane = (dims[2] + lay[0] + lay[2]) * pitch;
        if (!X) return fail(ONNX_ERR_NULL, "chain: X is NULL");
        add_copy(X, dims[1] * dims[2] * dims[3], lay[0] * pitch + lay[1], dims[3], pitch, dims[2], plane, 1);
        p.in_zero = (lay[0] | lay[1] | lay[2] | lay[3]) ? (int)(dims[1] * plane) : 0;
    }
    for (int o = 0; o < n_ops; ++o) {
        const onnx_chain_op& s = ops[o];
        ChainOp& op = p.ops[o];
        op.kind = s.kind; op.act = s.act;
        if (s.act != ONNX_ACT_NONE && s.act != ONNX_ACT_RELU) return fail(ONNX_ERR_ATTR, "chain: op %d: unknown activation %d", o, s.act);
        op.C = (int)dims[1]; op.H = (int)dims[2]; op.W = (int)dims[3];
        op.in_pitch = (int)(dims[3] + lay[1] + lay[3]);
        op.in_plane = (int)((dims[2] + lay[0] + lay[2]) * op.in_pitch);
        op.in_off = (int)(lay[0] * op.in_pitch + lay[1]);
        op.w_off = 0; op.b_off = -1; op.K = 0; op.Kp = 0; op.transB = 0; op.cip = 0; op.interior = 0; op.direct = 0; op.alpha = 1.f; op.beta = 1.f;
        op.kH = op.kW = op.sH = op.sW = op.dH = op.dW = 1; op.pT = op.pL = op.pB = op.pR = 0;
        int64_t yd[4] = {images, 0, 1, 1};
        if (s.kind == ONNX_CHAIN_CONV) {
            if (!s.W) return fail(ONNX_ERR_NULL, "chain: op %d (Conv): W is NULL", o);
            const int64_t wd[4] = {s.outputs, dims[1], s.kernel[0], s.kernel[1]};
            if (s.outputs < 1 || s.kernel[0] < 1 || s.kernel[1] < 1)
                return fail(ONNX_ERR_ATTR, "chain: op %d (Conv): outputs and kernel must be positive", o);
            const onnx_status st = onnx_conv_infer(dims, wd, s.pads, s.strides, s.dilations, 1, yd);
            if (st != ONNX_OK) return st;
            const int64_t K = dims[1] * s.kernel[0] * s.kernel[1];
            if (K > KOFF_MAX) return fail(ONNX_ERR_UNSUPPORTED, "chain: op %d (Conv): C*kH*kW = %lld exceeds %d", o, (long long)K, KOFF_MAX);
            // a filter row in LDS: whole trips of 16 k plus 4, so that rows start 16-byte aligned and the
            // 16-byte reads of 16 consecutive rows fall on different banks
            op.K = (int)K; op.Kp = (int)(((K + 15) & ~(int64_t)15) + 4);
            arena = (arena + 3) & ~(int64_t)3;
            op.kH = (int)s.kernel[0]; op.kW = (int)s.kernel[1]; op.sH = (int)s.strides[0]; op.sW = (int)s.strides[1];
            op.dH = (int)s.dilations[0]; op.dW = (int)s.dilations[1];
            op.pT = (int)s.pads[0]; op.pL = (int)s.pads[1]; op.pB = (int)s.pads[2]; op.pR = (int)s.pads[3];
            op.w_off = (int)arena;
            // few output channels, short K: the one-thread-per-position form, filters stored [k][8]
            // (when that takes no more LDS than the rows would)
            op.direct = s.outputs <= 8 && K <= 256 && 8 * K <= s.outputs * op.Kp;
            if (arena + s.outputs * op.Kp <= ARENA_MAX) {
                if (op.direct) {
                    add_copy(s.W, s.outputs * K, 2 * ACT_MAX + arena, K, 8, s.outputs, 0, 0);
                    p.copies[p.n_copies - 1].mode = 3;
                } else {
                    add_copy(s.W, s.outputs * K, 2 * ACT_MAX + arena, K, op.Kp, s.outputs, 0, 0);
                }
            }
            arena += s.outputs * op.Kp;
        } else if (s.kind == ONNX_CHAIN_MAXPOOL || s.kind == ONNX_CHAIN_AVGPOOL) {
            const bool global = s.kind == ONNX_CHAIN_AVGPOOL && s.kernel[0] == 0 && s.kernel[1] == 0;
            const int64_t kernel[2] = {global ? dims[2] : s.kernel[0], global ? dims[3] : s.kernel[1]};
            const int64_t zero4[4] = {0, 0, 0, 0}, one2[2] = {1, 1};
            const int64_t* dil = s.kind == ONNX_CHAIN_MAXPOOL ? s.dilations : one2;
            const onnx_status st = onnx_pool_infer(dims, kernel, global ? zero4 : s.pads, global ? one2 : s.strides, dil,
                                                   global ? 0 : s.ceil_mode, yd);
            if (st != ONNX_OK) return st;
            op.kH = (int)kernel[0]; op.kW = (int)kernel[1];
            if (!global) {
                op.sH = (int)s.strides[0]; op.sW = (int)s.strides[1];
                op.pT = (int)s.pads[0]; op.pL = (int)s.pads[1]; op.pB = (int)s.pads[2]; op.pR = (int)s.pads[3];
            }
            op.dH = (int)dil[0]; op.dW = (int)dil[1];
            op.cip = s.count_include_pad != 0;
            op.interior = op.pT == 0 && op.pL == 0 && yd[2] > 0 && yd[3] > 0 &&
                          (yd[2] - 1) * op.sH + (int64_t)(op.kH - 1) * op.dH < dims[2] &&
                          (yd[3] - 1) * op.sW + (int64_t)(op.kW - 1) * op.dW < dims[3];
        } else if (s.kind == ONNX_CHAIN_GEMM) {
            if (!s.W) return fail(ONNX_ERR_NULL, "chain: op %d (Gemm): W is NULL", o);
            if (s.outputs < 1) return fail(ONNX_ERR_ATTR, "chain: op %d (Gemm): outputs must be positive", o);
            const int64_t K = dims[1] * dims[2] * dims[3];
            yd[1] = s.outputs;
            op.K = (int)K; op.transB = s.transB != 0; op.alpha = s.alpha; op.beta = s.beta;
            op.w_off = (int)arena;
            if (arena + K * s.outputs <= ARENA_MAX)
                add_copy(s.W, K * s.outputs, 2 * ACT_MAX + arena, K * s.outputs, 0, 1, 0, 0);
            arena += K * s.outputs;
        } else {
            return fail(ONNX_ERR_ATTR, "chain: op %d: unknown kind %d", o, s.kind);
        }
        if (s.B && (s.kind == ONNX_CHAIN_CONV || s.kind == ONNX_CHAIN_GEMM)) {
            op.b_off = (int)arena;
            if (arena + s.outputs <= ARENA_MAX)
                add_copy(s.B, s.outputs, 2 * ACT_MAX + arena, s.outputs, 0, 1, 0, 0);
            arena += s.outputs;
        }
        if (arena > ARENA_MAX)
            return fail(ONNX_ERR_UNSUPPORTED, "chain: weights and biases up to op %d need %lld floats of LDS, %d are there", o,
                        (long long)arena, ARENA_MAX);
        if (yd[1] * yd[2] * yd[3] <= 0) empty = true;
        // the output buffer, laid out for its consumer
        consumer_pads(ops, n_ops, o + 1, lay);
        if (padded_size(yd, lay) > ACT_MAX)
            return fail(ONNX_ERR_UNSUPPORTED, "chain: the result of op %d (with its consumer's padding) exceeds %d floats", o, ACT_MAX);
        op.M = (int)yd[1]; op.OH = (int)yd[2]; op.OW = (int)yd[3];
        op.out_pitch = (int)(yd[3] + lay[1] + lay[3]);
        op.out_plane = (int)((yd[2] + lay[0] + lay[2]) * op.out_pitch);
        op.out_off = (int)(lay[0] * op.out_pitch + lay[1]);
        op.out_zero = (lay[0] | lay[1] | lay[2] | lay[3]) ? (int)(yd[1] * op.out_plane) : 0;
        op.Y = s.Y; op.y_img = (int)(yd[1] * yd[2] * yd[3]);
        if (o == n_ops - 1 && !s.Y && !empty) return fail(ONNX_ERR_NULL, "chain: the last operator's Y is NULL");
        op.dOW = FastDiv::make((uint32_t)(yd[3] > 0 ? yd[3] : 1));
        op.dOHW = FastDiv::make((uint32_t)(yd[2] * yd[3] > 0 ? yd[2] * yd[3] : 1));
        op.dkHW = FastDiv::make((uint32_t)(op.kH * op.kW));
        op.dkW = FastDiv::make((uint32_t)op.kW);
        for (int i = 0; i < 4; ++i) dims[i] = yd[i];
    }
    if (images > 0x7fffffffLL) return fail(ONNX_ERR_UNSUPPORTED, "chain: more than 2^31-1 images");
    if (empty) return ONNX_OK;
    // no result may overlap the input, a weight, a bias or another result
    const int64_t x_bytes = images * x_dims[1] * x_dims[2] * x_dims[3] * 4;
    for (int o = 0; o < n_ops; ++o) {
        if (!p.ops[o].Y) continue;
        const int64_t y_bytes = images * p.ops[o].y_img * 4;
        if (overlaps(p.ops[o].Y, y_bytes, X, x_bytes)) return fail(ONNX_ERR_ALIAS, "chain: the result of op %d overlaps X", o);
        for (int c = 1; c < p.n_copies; ++c)
            if (overlaps(p.ops[o].Y, y_bytes, p.copies[c].src, (int64_t)p.copies[c].count * 4))
                return fail(ONNX_ERR_ALIAS, "chain: the result of op %d overlaps a weight or bias", o);
        for (int q = 0; q < o; ++q)
            if (p.ops[q].Y && overlaps(p.ops[o].Y, y_bytes, p.ops[q].Y, images * p.ops[q].y_img * 4))
                return fail(ONNX_ERR_ALIAS, "chain: the results of ops %d and %d overlap", q, o);
    }
    p.total_chunks = (int)chunks;
    hipLaunchKernelGGL(chain_kernel, dim3((unsigned)images), dim3(CHAIN_THREADS), 0, static_cast<hipStream_t>(stream), p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ONNX_ERR_DEVICE, "chain: %s", hipGetErrorString(e));
    return ONNX_OK;
}
