// Tiled fp32 contraction on the gfx950 matrix cores.
//
// One kernel template computes, per z-slice,   Y[i, j] = epilogue( sum_k A(i,k) * B(k,j) )
// for ONNX Gemm, MatMul and Conv (the operators of Sections 3.4 and 4.1 of the paper; the
// convolution is evaluated as the product of the filter matrix [M x Cg*kH*kW] with the
// never-materialised matrix of input patches [Cg*kH*kW x N*OH*OW]).
//
// Work decomposition: a workgroup of 4 wavefronts owns a BM x BN tile of Y and walks K in
// steps of 16.  Each step stages an A tile and a B tile in LDS (double buffered: global
// loads for step t+1 are issued before the MFMAs of step t and written to the other buffer
// after them, one barrier per step).  Each wavefront owns a (BM/WM) x (BN/WN) sub-tile as
// a grid of 32x32 accumulators fed by v_mfma_f32_32x32x2_f32.
//
// Operand kinds (how a tile is fetched and how it sits in LDS):
//   KC      k is the contiguous index in memory (Gemm A, Gemm B with transB, conv filters).
//           LDS holds [row][16+4]; a lane reads 4 consecutive k with one 16-byte read.
//   RC      the row (i or j) is the contiguous index (Gemm A with transA, Gemm B, the input
//           of a 1x1 stride-1 unpadded conv).  LDS holds [k][rows+8]; lanes read along rows.
//   IM2COL  B only: element (k, j) is gathered from the NCHW input with pads, strides,
//           dilations and group resolved in the address computation.  LDS as RC.
// Because both operands of one MFMA must carry the same k, and a KC lane holds 4 consecutive
// k, the 8 k of a half-step are dealt as  k = 4*(lane/32) + s  to MFMA number s = 0..3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace onnxhip {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int BK = 16;
constexpr int NTHREADS = 256;
constexpr int LDK = BK + 4;          // row stride of a KC tile in LDS (floats)
constexpr int RC_PAD = 8;            // extra floats per k-row of an RC tile
constexpr int MAX_BATCH_DIMS = 6;
constexpr int NUM_XCD = 8;

enum { LOAD_KC = 0, LOAD_RC = 1, LOAD_IM2COL = 2 };

// Unsigned division by a run-time constant d >= 1 for numerators below 2^31:
// with s = floor(log2 d) and m = floor(2^(32+s)/d) + 1,  n / d == (n*m) >> (32+s).
// (m would need 33 bits when d is a power of two; those divide by shifting.)
struct FastDiv {
    uint32_t m, s, d, pow2;
    __host__ __device__ static FastDiv make(uint32_t d) {
        FastDiv f;
        f.d = d;
        uint32_t s = 0;
        while ((2u << s) <= d && s < 31) ++s;      // s = floor(log2 d)
        f.s = s;
        f.pow2 = ((d & (d - 1)) == 0) ? 1u : 0u;
        f.m = f.pow2 ? 0u : (uint32_t)((((uint64_t)1 << (32 + s)) / d) + 1);
        return f;
    }
    __host__ __device__ inline uint32_t div(uint32_t n) const {
        const uint32_t hi = (uint32_t)(((uint64_t)n * m) >> 32);
        return pow2 ? (n >> s) : (hi >> s);
    }
    __host__ __device__ inline void divmod(uint32_t n, uint32_t& q, uint32_t& r) const {
        q = div(n);
        r = n - q * d;
    }
};

struct Im2colGeom {
    int C, H, W;             // channels of the whole image, input height and width
    int sH, sW, pT, pL, dH, dW;
    FastDiv kHW, kW, P, OW;  // divisors: kH*kW, kW, OH*OW, OW
    int64_t image_stride;    // C*H*W
};

struct ContractionParams {
    const float* A;
    const float* B;
    float* Y;
    const float* bias;       // NULL or addressed  bias[z*bias_zs + i*bias_rs + j*bias_cs]
    const float* residual;   // NULL or laid out exactly like Y
    int M, N, K;             // extents of one z-slice
    int64_t a_ld, b_ld;      // KC: stride between rows; RC: stride between consecutive k
    int nbd;                 // z decomposes over bdim[0..nbd) (row-major), offsets below
    int bdim[MAX_BATCH_DIMS];
    int64_t a_bs[MAX_BATCH_DIMS], b_bs[MAX_BATCH_DIMS];
    int64_t y_zs, bias_zs;   // per-z offsets of Y (and residual) and of bias
    int64_t y_rs;            // stride between rows i of Y
    // With col_images set (conv) column j of B / Y is (image, pixel) = (j / colP, j % colP):
    // its offset is (j / colP) * img + j % colP with img = y_img for Y, b_img for an RC B.
    int col_images;
    FastDiv colP;
    int64_t y_img, b_img;
    float alpha, beta;
    int64_t bias_rs, bias_cs;
    int relu;
    int tiles_m, tiles_n;
    int nz;                  // number of z-slices; slice = blockIdx.y * gridDim.z + blockIdx.z
    Im2colGeom ic;
};

// ------------------------------------------------------------------------------------------
// Tile loader: global -> registers -> LDS for a ROWS x 16 tile.
template <int KIND, int VEC, int ROWS>
struct TileLoader {
    static constexpr bool kc = (KIND == LOAD_KC);
    // threads along the fast axis of a pass and rows/k covered per pass
    static constexpr int FAST = kc ? (BK / VEC) : (ROWS / VEC);
    static constexpr int SLOW_PER_PASS = NTHREADS / FAST;
    static constexpr int SLOW = kc ? ROWS : BK;
    static constexpr int NLOAD = (SLOW + SLOW_PER_PASS - 1) / SLOW_PER_PASS;
    static constexpr int LDR = ROWS + RC_PAD;
    static constexpr int LDS_FLOATS = kc ? ROWS * LDK : BK * LDR;
    static_assert(SLOW % SLOW_PER_PASS == 0 || SLOW < SLOW_PER_PASS, "tile/loader mismatch");

    float reg[NLOAD * VEC];
    int fast, slow0;            // this thread's coordinates within a pass
    bool active;                // false when SLOW < SLOW_PER_PASS leaves the thread idle
    // KC: per-pass row validity is recomputed (cheap); RC/IM2COL: one column per thread
    int64_t col_off;            // RC: offset of this thread's first column; IM2COL: image base
    bool col_ok;
    int ih0, iw0;               // IM2COL: top-left input coordinate of the column's window
    const float* base;
    int64_t ld;
    int rows_total, row0, K;

    // `images`: the row index is a column of B that splits into (image, pixel) through cp.colP.
    __device__ inline void init(const float* p, int64_t ld_, int row0_, int rows_total_, int K_,
                                bool images, const ContractionParams& cp) {
        base = p; ld = ld_; row0 = row0_; rows_total = rows_total_; K = K_;
        const int t = threadIdx.x;
        fast = t % FAST;
        slow0 = t / FAST;
        if (FAST % 64 == 0) slow0 = __builtin_amdgcn_readfirstlane(slow0);   // uniform per wavefront
        active = slow0 < SLOW;
        col_off = 0; col_ok = true; ih0 = 0; iw0 = 0;
        if (!kc) {
            const int j = row0 + fast * VEC;
            col_ok = j < rows_total;
            const uint32_t jj = col_ok ? (uint32_t)j : 0u;
            if (KIND == LOAD_RC) {
                if (images) {
                    uint32_t n, px;
                    cp.colP.divmod(jj, n, px);
                    col_off = (int64_t)n * cp.b_img + px;
                } else {
                    col_off = jj;
                }
            } else {
                uint32_t n, px, oh, ow;
                cp.colP.divmod(jj, n, px);
                cp.ic.OW.divmod(px, oh, ow);
                ih0 = (int)oh * cp.ic.sH - cp.ic.pT;
                iw0 = (int)ow * cp.ic.sW - cp.ic.pL;
                col_off = (int64_t)n * cp.ic.image_stride + (int64_t)ih0 * cp.ic.W + iw0;
            }
        }
    }

    // Issue the global loads of the tile whose first k is k0.
    __device__ inline void fetch(int k0, const ContractionParams& cp) {
#pragma unroll
        for (int p = 0; p < NLOAD; ++p) {
            const int slow = slow0 + p * SLOW_PER_PASS;
            if (kc) {
                const int row = row0 + slow;
                const int k = k0 + fast * VEC;
                const bool ok = active && row < rows_total && k < K;
                const float* src = base + (int64_t)row * ld + k;
                if (VEC == 4) {
                    floatx4 v = {0.f, 0.f, 0.f, 0.f};
                    if (ok) v = *reinterpret_cast<const floatx4*>(src);
                    reg[p * 4 + 0] = v.x; reg[p * 4 + 1] = v.y; reg[p * 4 + 2] = v.z; reg[p * 4 + 3] = v.w;
                } else {
                    reg[p] = ok ? *src : 0.f;
                }
            } else if (KIND == LOAD_RC) {
                const int k = k0 + slow;
                const bool ok = active && col_ok && k < K;
                const float* src = base + col_off + (int64_t)k * ld;
                if (VEC == 4) {
                    floatx4 v = {0.f, 0.f, 0.f, 0.f};
                    if (ok) v = *reinterpret_cast<const floatx4*>(src);
                    reg[p * 4 + 0] = v.x; reg[p * 4 + 1] = v.y; reg[p * 4 + 2] = v.z; reg[p * 4 + 3] = v.w;
                } else {
                    reg[p] = ok ? *src : 0.f;
                }
            } else {
                // k -> (c, kh, kw); the same for every lane of a wavefront
                const uint32_t k = (uint32_t)(k0 + slow);
                uint32_t c, rem, kh, kw;
                cp.ic.kHW.divmod(k, c, rem);
                cp.ic.kW.divmod(rem, kh, kw);
                const int dh = (int)kh * cp.ic.dH, dw = (int)kw * cp.ic.dW;
                const int ih = ih0 + dh, iw = iw0 + dw;
                const bool ok = active && col_ok && (int)k < K && ih >= 0 && ih < cp.ic.H && iw >= 0 &&
                                iw < cp.ic.W;
                const int64_t off = col_off + ((int64_t)c * cp.ic.H + dh) * cp.ic.W + dw;
                reg[p] = ok ? base[off] : 0.f;
            }
        }
    }

    // Write the fetched tile into an LDS buffer.
    __device__ inline void commit(float* lds) const {
        if (!active) return;
#pragma unroll
        for (int p = 0; p < NLOAD; ++p) {
            const int slow = slow0 + p * SLOW_PER_PASS;
            if (kc) {
                float* dst = lds + slow * LDK + fast * VEC;
                if (VEC == 4) {
                    floatx4 v = {reg[p * 4 + 0], reg[p * 4 + 1], reg[p * 4 + 2], reg[p * 4 + 3]};
                    *reinterpret_cast<floatx4*>(dst) = v;
                } else {
                    *dst = reg[p];
                }
            } else {
                float* dst = lds + slow * LDR + fast * VEC;
                if (VEC == 4) {
                    floatx4 v = {reg[p * 4 + 0], reg[p * 4 + 1], reg[p * 4 + 2], reg[p * 4 + 3]};
                    *reinterpret_cast<floatx4*>(dst) = v;
                } else {
                    *dst = reg[p];
                }
            }
        }
    }

    // The 4 values (MFMA steps s = 0..3) this lane feeds for tile-row `row`, half-step g.
    __device__ static inline void frag(const float* lds, int row, int g, int h, float out[4]) {
        if (kc) {
            const floatx4 v = *reinterpret_cast<const floatx4*>(lds + row * LDK + g * 8 + h * 4);
            out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) out[s] = lds[(g * 8 + h * 4 + s) * LDR + row];
        }
    }
};

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of logical
// tile numbers so that tiles sharing A rows / B columns meet in the same L2.
__device__ inline int xcd_contiguous(int bid, int nblocks) {
    const int xcd = bid % NUM_XCD, local = bid / NUM_XCD;
    const int per = nblocks / NUM_XCD, rem = nblocks % NUM_XCD;
    return xcd < rem ? xcd * (per + 1) + local : rem * (per + 1) + (xcd - rem) * per + local;
}

template <int BM, int BN, int WM, int WN, int AKIND, int BKIND, int VEC>
__global__ __launch_bounds__(NTHREADS) void contraction_kernel(const ContractionParams cp) {
    static_assert(WM * WN * 64 == NTHREADS, "four wavefronts per workgroup");
    constexpr int WTM = BM / WM, WTN = BN / WN;     // wavefront sub-tile
    constexpr int TM = WTM / 32, TN = WTN / 32;     // 32x32 accumulators per wavefront
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "sub-tile of 32x32 blocks");
    constexpr int BVEC = (BKIND == LOAD_IM2COL) ? 1 : VEC;
    using ALoader = TileLoader<AKIND, VEC, BM>;
    using BLoader = TileLoader<BKIND, BVEC, BN>;

    __shared__ __attribute__((aligned(16))) float lds_a[2][ALoader::LDS_FLOATS];
    __shared__ __attribute__((aligned(16))) float lds_b[2][BLoader::LDS_FLOATS];

    // ---- which tile, which z-slice
    const int ntiles = cp.tiles_m * cp.tiles_n;
    const int logical = xcd_contiguous(blockIdx.x, ntiles);
    constexpr int GROUP = 8;                        // tile rows swept together
    const int per_group = GROUP * cp.tiles_n;
    const int grp = logical / per_group;
    const int first_m = grp * GROUP;
    const int rows_here = min(cp.tiles_m - first_m, GROUP);
    const int in_grp = logical - grp * per_group;
    const int tile_m = first_m + in_grp % rows_here;
    const int tile_n = in_grp / rows_here;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int zslice = blockIdx.y * gridDim.z + blockIdx.z;
    if (zslice >= cp.nz) return;                    // uniform for the whole workgroup
    int64_t a_off = 0, b_off = 0;
    {
        int z = zslice;
        for (int d = cp.nbd - 1; d >= 0; --d) {
            const int idx = z % cp.bdim[d];
            z /= cp.bdim[d];
            a_off += idx * cp.a_bs[d];
            b_off += idx * cp.b_bs[d];
        }
    }
    const int64_t zi = zslice;

    ALoader la;
    BLoader lb;
    la.init(cp.A + a_off, cp.a_ld, m0, cp.M, cp.K, false, cp);
    lb.init(cp.B + b_off, cp.b_ld, n0, cp.N, cp.K, cp.col_images != 0, cp);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, h = lane >> 5;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (cp.K + BK - 1) / BK;
    la.fetch(0, cp);
    lb.fetch(0, cp);
    la.commit(lds_a[0]);
    lb.commit(lds_b[0]);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            la.fetch((kt + 1) * BK, cp);
            lb.fetch((kt + 1) * BK, cp);
        }
        const float* sa = lds_a[cur];
        const float* sb = lds_b[cur];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            float fa[TM][4], fb[TN][4];
#pragma unroll
            for (int i = 0; i < TM; ++i) ALoader::frag(sa, wm * WTM + i * 32 + li, g, h, fa[i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) BLoader::frag(sb, wn * WTN + j * 32 + li, g, h, fb[j]);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][s], fb[j][s], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            la.commit(lds_a[cur ^ 1]);
            lb.commit(lds_b[cur ^ 1]);
        }
        __syncthreads();
    }

    // ---- epilogue: alpha*acc + beta*bias (+ residual), Relu, store.
    // Accumulator register r of a 32x32 block holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
    float* yz = cp.Y + zi * cp.y_zs;
    const float* rz = cp.residual ? cp.residual + zi * cp.y_zs : nullptr;
    const float* bz = cp.bias ? cp.bias + zi * cp.bias_zs : nullptr;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WTN + j * 32 + li;
        if (col >= cp.N) continue;
        int64_t coff = col;
        if (cp.col_images) {
            uint32_t n, px;
            cp.colP.divmod((uint32_t)col, n, px);
            coff = (int64_t)n * cp.y_img + px;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (row >= cp.M) continue;
                float v = cp.alpha * acc[i][j][r];
                if (bz) v += cp.beta * bz[row * cp.bias_rs + col * cp.bias_cs];
                const int64_t o = (int64_t)row * cp.y_rs + coff;
                if (rz) v += rz[o];
                if (cp.relu) v = v > 0.f ? v : 0.f;
                yz[o] = v;
            }
        }
    }
}

}  // namespace onnxhip
