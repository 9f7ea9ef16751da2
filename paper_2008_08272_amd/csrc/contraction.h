// Tiled fp32 contraction on the gfx950 matrix cores.
//
// One kernel template computes, per z-slice,   Y[i, j] = epilogue( sum_k A(i,k) * B(k,j) )
// for ONNX Gemm, MatMul and Conv (the operators of Sections 3.4 and 4.1 of the paper; the
// convolution is evaluated as the product of the filter matrix [M x Cg*kH*kW] with the
// never-materialised matrix of input patches [Cg*kH*kW x N*OH*OW]).
//
// Work decomposition: a workgroup of WM x WN wavefronts owns a BM x BN tile of Y and walks K
// in steps of BK.  Each step stages an A tile and a B tile in LDS (two buffers, one barrier per
// step; global loads run one or two steps ahead through staging registers, and the LDS reads
// of the fragments needed next are issued in between the MFMAs of the fragments in use).
// Each wavefront owns a (BM/WM) x (BN/WN) sub-tile as a grid of 32x32 accumulators fed by
// v_mfma_f32_32x32x2_f32.
//
// Operand kinds (how a tile is fetched and how it sits in LDS):
//   KC      k is the contiguous index in memory (Gemm A, Gemm B with transB, conv filters).
//           LDS holds [row][BK+4]; a lane reads 4 consecutive k with one 16-byte read.
//   RC      the row (i or j) is the contiguous index (Gemm A with transA, Gemm B, the input
//           of a 1x1 stride-1 unpadded conv).  LDS holds [k][rows+8]; lanes read along rows.
//   IM2COL  B only: element (k, j) is gathered from the NCHW input with pads, strides,
//           dilations and group resolved in the address computation.  LDS as RC.
//   RCS     B only: the input of a strided, unpadded 1x1 convolution.  As RC, except that
//           column j (an output pixel) sits at input pixel (oh*sH, ow*sW), so neighbouring
//           columns are not neighbours in memory and are fetched one value at a time; a k row
//           is still one plane further, so no per-element address arithmetic is needed.
// Because both operands of one MFMA must carry the same k, and a KC lane holds 4 consecutive
// k, the 8 k of a half-step are dealt as  k = 4*(lane/32) + s  to MFMA number s = 0..3.
//
// Global loads go through buffer resources (see OOB below): a lane whose element lies
// outside the operand gets 0 from the hardware range check, so the loop body has no divergent
// branch and no select, and loads, LDS traffic and MFMAs can be scheduled around each other.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace onnxhip {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int RC_PAD = 8;            // extra floats per k-row of an RC tile
constexpr int KC_PAD = 4;            // extra floats per row of a KC tile
constexpr int MAX_BATCH_DIMS = 6;
constexpr int NUM_XCD = 8;

enum { LOAD_KC = 0, LOAD_RC = 1, LOAD_IM2COL = 2, LOAD_RCS = 3 };
enum { BIAS_NONE = 0, BIAS_ROW = 1, BIAS_COL = 2, BIAS_FULL = 3 };

// Unsigned division by a run-time constant d >= 1 for numerators below 2^31:
// with s = floor(log2 d) and m = floor(2^(32+s)/d) + 1,  n / d == (n*m) >> (32+s).
// (m would need 33 bits when d is a power of two; those divide by shifting, selected with a
// mask rather than a branch so that the code stays straight-line.)
struct FastDiv {
    uint32_t m, s, d, pow2_mask;
    __host__ __device__ static FastDiv make(uint32_t d) {
        FastDiv f;
        f.d = d;
        uint32_t s = 0;
        while ((2u << s) <= d && s < 31) ++s;      // s = floor(log2 d)
        f.s = s;
        const bool pow2 = (d & (d - 1)) == 0;
        f.pow2_mask = pow2 ? 0xffffffffu : 0u;
        f.m = pow2 ? 0u : (uint32_t)((((uint64_t)1 << (32 + s)) / d) + 1);
        return f;
    }
    __host__ __device__ inline uint32_t div(uint32_t n) const {
        const uint32_t hi = (uint32_t)(((uint64_t)n * m) >> 32);
        return ((hi & ~pow2_mask) | (n & pow2_mask)) >> s;
    }
    __host__ __device__ inline void divmod(uint32_t n, uint32_t& q, uint32_t& r) const {
        q = div(n);
        r = n - q * d;
    }
};

struct Im2colGeom {
    int C, H, W;             // channels of the whole image, input height and width
    int sH, sW, pT, pL, dH, dW;
    FastDiv kHW, kW, OW;     // divisors: kH*kW, kW, OW
    int image_stride;        // C*H*W
    // LDS-patch convolution (conv_window.h) only:
    int OH, Cg;              // output height, input channels per group
    int E, IPR;              // window extent (kH-1)*dH+1; patch rows of one whole image (OH-1)*sH+E
    int PC, plane;           // patch columns (OW-1)*sW+(kW-1)*dW+1; floats per channel = patch rows * PC
    FastDiv OHd, PCd, planed, IPRd;
};

struct ContractionParams {
    const float* A;
    const float* B;
    float* Y;
    const float* bias;       // NULL or the epilogue's additive operand, see bias_mode
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
    // How `bias` is laid out against the M x N output: BIAS_ROW one value per row i (conv bias,
    // Gemm C of shape {M,1}), BIAS_COL one per column j with element stride bias_cs (Gemm C of
    // shape {N} / {1,N}; stride 0 for a scalar), BIAS_FULL an M x N matrix laid out like Y.
    int bias_mode;
    int bias_cs;
    int relu;
    int tiles_m, tiles_n;
    int nz;                  // number of z-slices
    // Split-K: grid.y = ksplit * (z overflow factor).  Workgroup (tile, split) sums its share of
    // the K steps; with ksplit > 1 it parks the partial tile in ws_partial and a second kernel
    // (splitk_finish_kernel) adds the partials in split order and runs the epilogue.
    int ksplit;
    float* ws_partial;
    // Tail split (ksplit == 1, nz == 1 only): blocks [0, tail_begin) compute whole tiles; the
    // remaining tiles_m*tiles_n - tail_begin tiles, which would keep only a few CUs busy at the
    // end of the launch, are each shared by tail_split blocks that follow in the same grid and
    // are finished by a splitk_finish_kernel over just those tiles.  tail_begin equals the tile
    // count when there is no tail.
    int tail_begin, tail_split;
    Im2colGeom ic;
};

// Buffer addressing: every operand tile is read through a buffer resource whose base is the
// tile's first element and whose extent is 2^31 bytes.  Lanes address it with 32-bit byte
// offsets; a lane whose element does not exist uses offset 2^31, which the hardware range
// check turns into a returned 0 without touching memory.  The host guarantees that every
// existing element of a tile lies below 2^31 bytes from the tile's base.
constexpr uint32_t OOB = 0x80000000u;
constexpr int RSRC_FLAGS = 0x00020000;          // raw 32-bit data format

__device__ inline __amdgpu_buffer_rsrc_t tile_rsrc(const float* p) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p), 0, (int)OOB, RSRC_FLAGS);
}

// ------------------------------------------------------------------------------------------
// Tile loader: global -> registers -> LDS for a ROWS x BK tile, NT threads.
template <int KIND, int VEC, int ROWS, int BK, int NT, int NSETS = 1>
struct TileLoader {
    static constexpr bool kc = (KIND == LOAD_KC);
    static constexpr int FAST = kc ? (BK / VEC) : (ROWS / VEC);   // threads along the contiguous axis
    static constexpr int SLOW_PER_PASS = NT / FAST;               // rows (KC) or k (RC) per pass
    static constexpr int SLOW = kc ? ROWS : BK;
    static constexpr int NLOAD = (SLOW + SLOW_PER_PASS - 1) / SLOW_PER_PASS;
    static constexpr int LDK = BK + KC_PAD;
    static constexpr int LDR = ROWS + RC_PAD;
    static constexpr int LDS_FLOATS = kc ? ROWS * LDK : BK * LDR;
    static_assert(NT % FAST == 0, "threads must tile the contiguous axis");
    static_assert(SLOW % SLOW_PER_PASS == 0 || SLOW < SLOW_PER_PASS, "tile/loader mismatch");

    float reg[NSETS][NLOAD * VEC];   // staging registers: tiles of coming K steps on their way to LDS
    int fast, slow0;
    bool active;                 // false when SLOW < SLOW_PER_PASS leaves the thread idle
    const float* base;           // first element of the tile (RC: at k = 0)
    __amdgpu_buffer_rsrc_t rsrc; // KC / IM2COL: fixed for the whole K walk
    int ld, K;
    // KC: byte offset of each pass's row (OOB when the row does not exist).
    // RC: byte offset of the thread's column at k = slow0.  IM2COL: element offset of the
    // column's window origin relative to the tile's first image (may be negative).
    uint32_t voff[kc ? NLOAD : 1];
    bool col_ok;
    int ih0, iw0;                // IM2COL: input coordinate of the window's first tap

    __device__ inline void init(const float* p, int64_t ld_, int row0, int rows_total, int K_,
                                bool images, const ContractionParams& cp) {
        ld = (int)ld_; K = K_;
        const int t = threadIdx.x;
        fast = t % FAST;
        slow0 = t / FAST;
        if (FAST % 64 == 0) slow0 = __builtin_amdgcn_readfirstlane(slow0);   // uniform per wavefront
        active = slow0 < SLOW;
        ih0 = 0; iw0 = 0; col_ok = true;
        if (kc) {
            base = p + (int64_t)row0 * ld_;
#pragma unroll
            for (int p_ = 0; p_ < NLOAD; ++p_) {
                const int slow = slow0 + p_ * SLOW_PER_PASS;
                const bool ok = active && row0 + slow < rows_total;
                voff[p_] = ok ? (uint32_t)(slow * ld + fast * VEC) * 4u : OOB;
            }
        } else {
            const int j = row0 + fast * VEC;
            col_ok = active && j < rows_total;
            const uint32_t jj = col_ok ? (uint32_t)j : (uint32_t)row0;
            if (KIND == LOAD_RC || KIND == LOAD_RCS) {
                if (images) {
                    uint32_t n0_, p0_, n, px;
                    cp.colP.divmod((uint32_t)row0, n0_, p0_);
                    cp.colP.divmod(jj, n, px);
                    if (KIND == LOAD_RCS) {               // output pixel -> input pixel of the strided 1x1 window
                        uint32_t oh, ow;
                        cp.ic.OW.divmod(px, oh, ow);
                        px = oh * (uint32_t)(cp.ic.sH * cp.ic.W) + ow * (uint32_t)cp.ic.sW;
                    }
                    base = p + (int64_t)n0_ * cp.b_img;
                    voff[0] = (uint32_t)((int)(n - n0_) * (int)cp.b_img + (int)px + slow0 * ld) * 4u;
                } else {
                    base = p + row0;
                    voff[0] = (uint32_t)((int)(jj - (uint32_t)row0) + slow0 * ld) * 4u;
                }
            } else {
                uint32_t n0_, p0_, n, px, oh, ow;
                cp.colP.divmod((uint32_t)row0, n0_, p0_);
                cp.colP.divmod(jj, n, px);
                cp.ic.OW.divmod(px, oh, ow);
                ih0 = (int)oh * cp.ic.sH - cp.ic.pT;
                iw0 = (int)ow * cp.ic.sW - cp.ic.pL;
                base = p + (int64_t)n0_ * cp.ic.image_stride;
                voff[0] = (uint32_t)((int)(n - n0_) * cp.ic.image_stride + ih0 * cp.ic.W + iw0);
            }
        }
        rsrc = tile_rsrc(base);
    }

    template <int S>
    __device__ inline void load(__amdgpu_buffer_rsrc_t r, uint32_t off, int soff, int p) {
        if (VEC == 4) {
            const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, soff, 0));
            reg[S][p * 4 + 0] = v.x; reg[S][p * 4 + 1] = v.y; reg[S][p * 4 + 2] = v.z; reg[S][p * 4 + 3] = v.w;
        } else {
            reg[S][p] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, soff, 0));
        }
    }

    // Issue the global loads of the tile whose first k is k0 into register set S (k0 >= K loads nothing).
    template <int S>
    __device__ inline void fetch(int k0, const ContractionParams& cp) {
        if constexpr (kc) {
            const bool k_ok = k0 + fast * VEC < K;
#pragma unroll
            for (int p = 0; p < NLOAD; ++p) load<S>(rsrc, k_ok ? voff[p] : OOB, k0 * 4, p);
        } else if constexpr (KIND == LOAD_RC || KIND == LOAD_RCS) {
            // the resource is re-based at row k0 so that offsets stay small whatever K is
            const __amdgpu_buffer_rsrc_t r = tile_rsrc(base + (int64_t)k0 * ld);
#pragma unroll
            for (int p = 0; p < NLOAD; ++p) {
                const bool good = col_ok && (k0 + slow0 + p * SLOW_PER_PASS < K);
                load<S>(r, good ? voff[0] : OOB, p * SLOW_PER_PASS * ld * 4, p);
            }
        } else {
            // k -> (c, kh, kw) is the same for every column, so the BK decompositions of this
            // step are computed once, lane q of each wavefront taking k0 + q; each load then
            // fetches the one it needs from that lane (its k row is uniform per wavefront).
            static_assert(FAST % 64 == 0 && BK <= 64, "IM2COL tiles: columns in multiples of 64");
            const uint32_t kq = (uint32_t)(k0 + (int)(threadIdx.x & (BK - 1)));
            uint32_t c, rem, kh, kw;
            cp.ic.kHW.divmod(kq, c, rem);
            cp.ic.kW.divmod(rem, kh, kw);
            const int dh_l = (int)kh * cp.ic.dH, dw_l = (int)kw * cp.ic.dW;
            const int koff_l = (int)kq < K ? ((int)c * cp.ic.H + dh_l) * cp.ic.W + dw_l : -1;
            const int dhw_l = (dh_l << 16) | dw_l;
#pragma unroll
            for (int p = 0; p < NLOAD; ++p) {
                const int q = slow0 + p * SLOW_PER_PASS;
                const int koff = __builtin_amdgcn_readlane(koff_l, q);
                const int dhw = __builtin_amdgcn_readlane(dhw_l, q);
                const int ih = ih0 + (dhw >> 16), iw = iw0 + (dhw & 0xffff);
                const bool good = col_ok && koff >= 0 && (unsigned)ih < (unsigned)cp.ic.H &&
                                  (unsigned)iw < (unsigned)cp.ic.W;
                load<S>(rsrc, good ? (voff[0] + (uint32_t)koff) * 4u : OOB, 0, p);
            }
        }
    }

    // Write the tile held in register set S into an LDS buffer.
    template <int S>
    __device__ inline void commit(float* lds) const {
        if (!active) return;
#pragma unroll
        for (int p = 0; p < NLOAD; ++p) {
            const int slow = slow0 + p * SLOW_PER_PASS;
            float* dst = kc ? lds + slow * LDK + fast * VEC : lds + slow * LDR + fast * VEC;
            if (VEC == 4) {
                floatx4 v = {reg[S][p * 4 + 0], reg[S][p * 4 + 1], reg[S][p * 4 + 2], reg[S][p * 4 + 3]};
                *reinterpret_cast<floatx4*>(dst) = v;
            } else {
                *dst = reg[S][p];
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

// Values that are the same in every lane but were computed by vector instructions (the integer
// divisions of the tile and z-slice decompositions are) and end up in a buffer resource or a
// scalar offset: taken into scalar registers here, once.  Left to itself the compiler usually
// does the same (it does in every instance of contraction_kernel), but in some instances of the
// LDS-patch and 16-bit kernels it kept them in vector registers and wrapped every buffer access
// that used them in a loop over the distinct values; those kernels call this.
__device__ inline int scalar(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline int64_t scalar(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of logical
// tile numbers so that tiles sharing A rows / B columns meet in the same L2.
__device__ inline int xcd_contiguous(int bid, int nblocks) {
    const int xcd = bid % NUM_XCD, local = bid / NUM_XCD;
    const int per = nblocks / NUM_XCD, rem = nblocks % NUM_XCD;
    return xcd < rem ? xcd * (per + 1) + local : rem * (per + 1) + (xcd - rem) * per + local;
}

// Epilogue for one 32x32 accumulator block: alpha*acc + beta*bias (+ residual), Relu, store.
// Accumulator register r holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.  Y, the
// residual and a full-matrix bias are addressed through buffer resources based at the
// tile's first element: `voff` is the lane's byte offset for register 0 (OOB when its column
// does not exist) and the rows of the other registers are reached through the scalar offset.
// GUARD adds the test for rows beyond M (only tiles on the bottom edge need it): such a row
// turns the offset into OOB, which makes the hardware return 0 for loads and drop the store.
struct EpilogueSrc {
    __amdgpu_buffer_rsrc_t ry, rr, rfull, rrow;   // Y, residual, full-matrix bias, per-row bias
    bool has_res;
    int mode;
    bool relu;
};

// C0, C1: the groups of four accumulator registers (eight rows apart) to store, all four by default.
template <bool GUARD, int C0 = 0, int C1 = 4>
__device__ inline void store_block(const floatx16& acc, int row0, float col_bias, uint32_t voff,
                                   const EpilogueSrc& e, const ContractionParams& cp) {
    const int row_stride_bytes = (int)cp.y_rs * 4;
#pragma unroll
    for (int c = C0; c < C1; ++c) {
        float add[4];
        uint32_t off[4];
        // four consecutive rows: one 16-byte load fetches their per-row bias
        floatx4 rb = {0.f, 0.f, 0.f, 0.f};
        if (e.mode == BIAS_ROW) {
            if (!GUARD) {
                rb = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(e.rrow, (row0 + 8 * c) * 4, 0, 0));
            } else {     // rows may run past M: dword loads, each range-checked on its own
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    rb[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(e.rrow, (row0 + 8 * c + q) * 4, 0, 0));
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            off[q] = (!GUARD || row0 + 8 * c + q < cp.M) ? voff : OOB;
            add[q] = col_bias + cp.beta * rb[q];
        }
        if (e.mode == BIAS_FULL) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                add[q] += cp.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                        e.rfull, (int)off[q], (8 * c + q) * row_stride_bytes, 0));
        }
        if (e.has_res) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                add[q] += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                        e.rr, (int)off[q], (8 * c + q) * row_stride_bytes, 0));
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // Relu as v > 0 ? v : 0 (a NaN becomes 0); without Relu the value is stored as it is
            const float lin = fmaf(cp.alpha, acc[4 * c + q], add[q]);
            const float v = e.relu ? fmaxf(lin, 0.f) : lin;
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), e.ry, (int)off[q],
                                                  (8 * c + q) * row_stride_bytes, 0);
        }
    }
}

// What a workgroup of a contraction launch computes: the tile at (m0, n0) of z-slice `zslice`,
// K steps of share `split` out of `ksplit`; with ksplit > 1 its partial tile goes to slot
// `slot` of the workspace.
struct TileWork {
    int m0, n0, zslice, split, ksplit;
    int64_t slot;
};

// Logical tile number -> tile origin: tiles are swept 8 tile-rows at a time, column by column,
// so that consecutive numbers share B columns and stay within a few A row panels.
__device__ inline void tile_origin(const ContractionParams& cp, int logical, int BM, int BN, int& m0, int& n0) {
    constexpr int GROUP = 8;
    const int per_group = GROUP * cp.tiles_n;
    const int grp = logical / per_group;
    const int first_m = grp * GROUP;
    const int rows_here = min(cp.tiles_m - first_m, GROUP);
    const int in_grp = logical - grp * per_group;
    m0 = (first_m + in_grp % rows_here) * BM;
    n0 = (in_grp / rows_here) * BN;
}

// blockIdx.x below tail_begin: a whole tile (or, with ksplit > 1, share blockIdx.y % ksplit of
// it; blockIdx.y also carries the overflow of the z-slice count).  From tail_begin on: share
// t % tail_split of tail tile t / tail_split.  False when the block has nothing to do.
__device__ inline bool tile_work(const ContractionParams& cp, int BM, int BN, TileWork& w) {
    const int ntiles = cp.tiles_m * cp.tiles_n;
    int logical;
    if ((int)blockIdx.x < cp.tail_begin) {
        w.ksplit = cp.ksplit;
        w.split = blockIdx.y % cp.ksplit;
        w.zslice = (blockIdx.y / cp.ksplit) * gridDim.z + blockIdx.z;
        logical = xcd_contiguous(blockIdx.x, cp.tail_begin);
        w.slot = ((int64_t)w.zslice * ntiles + blockIdx.x) * cp.ksplit + w.split;
    } else {
        const int t = (int)blockIdx.x - cp.tail_begin;
        w.ksplit = cp.tail_split;
        w.split = t % cp.tail_split;
        w.zslice = 0;
        logical = cp.tail_begin + t / cp.tail_split;
        w.slot = t;
    }
    if (w.zslice >= cp.nz) return false;
    tile_origin(cp, logical, BM, BN, w.m0, w.n0);
    return true;
}

// Offsets of the z-slice's A and B operands (batch broadcasting / convolution groups).
__device__ inline void slice_offsets(const ContractionParams& cp, int zslice, int64_t& a_off, int64_t& b_off) {
    a_off = 0; b_off = 0;
    int z = zslice;
    for (int d = cp.nbd - 1; d >= 0; --d) {
        const int idx = z % cp.bdim[d];
        z /= cp.bdim[d];
        a_off += idx * cp.a_bs[d];
        b_off += idx * cp.b_bs[d];
    }
}

// Epilogue of a workgroup tile whose wavefront (wm, wn) holds TM x TN accumulator blocks.
template <int TM, int TN, int WTM, int WTN, int C0 = 0, int C1 = 4>
__device__ inline void store_tile(const floatx16 (&acc)[TM][TN], int m0, int n0, int zslice, int wm, int wn,
                                  int li, int h, const ContractionParams& cp) {
    const int64_t zi = zslice;
    int64_t tile_off = (int64_t)m0 * cp.y_rs + n0;          // first element of the tile in Y
    uint32_t img0 = 0;
    if (cp.col_images) {
        uint32_t px0;
        cp.colP.divmod((uint32_t)n0, img0, px0);
        tile_off = (int64_t)m0 * cp.y_rs + (int64_t)img0 * cp.y_img + px0;
    }
    tile_off += zi * cp.y_zs;
    EpilogueSrc e;
    e.ry = tile_rsrc(cp.Y + tile_off);
    e.has_res = cp.residual != nullptr;
    e.rr = tile_rsrc(e.has_res ? cp.residual + tile_off : cp.Y + tile_off);
    e.mode = cp.bias ? cp.bias_mode : BIAS_NONE;
    e.rfull = tile_rsrc(e.mode == BIAS_FULL ? cp.bias + tile_off : cp.Y + tile_off);
    // per-row bias: a resource over exactly the M values of this z-slice, so that rows beyond
    // M (their stores are dropped anyway) read as 0 instead of running past the array
    const float* brow = e.mode == BIAS_ROW ? cp.bias + zi * cp.bias_zs : cp.Y;
    e.rrow = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(brow), 0, cp.M * 4, RSRC_FLAGS);
    e.relu = cp.relu != 0;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int cl = wn * WTN + j * 32 + li;            // column within the tile
        const int col = n0 + cl;
        const bool col_ok = col < cp.N;
        const int cj = col_ok ? col : n0;
        int crel = cl;                                    // element offset from the tile's first column
        if (cp.col_images) {
            uint32_t n, px, px0;
            cp.colP.divmod((uint32_t)cj, n, px);
            px0 = (uint32_t)n0 - img0 * cp.colP.d;
            crel = (int)(n - img0) * (int)cp.y_img + (int)px - (int)px0;
        }
        float col_bias = 0.f;
        if (e.mode == BIAS_COL) col_bias = cp.beta * cp.bias[(int64_t)cj * cp.bias_cs];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rl = wm * WTM + i * 32 + 4 * h;     // row within the tile of register 0
            const uint32_t voff = col_ok ? (uint32_t)(rl * (int)cp.y_rs + crel) * 4u : OOB;
            // the 32 rows of this block all exist unless the block reaches past M (uniform test)
            if (m0 + wm * WTM + i * 32 + 32 <= cp.M) store_block<false, C0, C1>(acc[i][j], m0 + rl, col_bias, voff, e, cp);
            else store_block<true, C0, C1>(acc[i][j], m0 + rl, col_bias, voff, e, cp);
        }
    }
}

// The K steps [kt0, kt1) of `nk` that split `split` of `ksplit` owns.
__device__ inline void split_range(int nk, int ksplit, int split, int& kt0, int& kt1) {
    const int per = (nk + ksplit - 1) / ksplit;
    kt0 = split * per;
    kt1 = min(nk, kt0 + per);
    if (kt0 > kt1) kt0 = kt1;
}

// End of a workgroup's K walk.  Without split-K: the epilogue.  With split-K: park the partial
// accumulators in the workspace (register-major, thread-minor, so every access is
// coalesced); splitk_finish_kernel, launched right behind on the same stream, adds a tile's
// partials in split order and runs the epilogue.  Two launches rather than a fence and an
// arrival counter inside one: the XCDs' L2 caches are only coherent with each other at
// kernel boundaries, and a device-scope fence per workgroup writes back and invalidates them.
template <int TM, int TN, int WTM, int WTN, int NT>
__device__ inline void finish_tile(floatx16 (&acc)[TM][TN], const TileWork& w, int wm, int wn, int li, int h,
                                   const ContractionParams& cp) {
    if (w.ksplit > 1) {
        constexpr int TILE = NT * TM * TN * 16;
        float* mine = cp.ws_partial + w.slot * TILE + threadIdx.x;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) mine[((i * TN + j) * 16 + r) * NT] = acc[i][j][r];
        return;
    }
    store_tile<TM, TN, WTM, WTN>(acc, w.m0, w.n0, w.zslice, wm, wn, li, h, cp);
}

// Second half of a split-K product: same thread-to-accumulator mapping as the kernel that
// produced the partials.  tail = false: all tiles of a launch with ksplit > 1; tail = true: only
// the tail tiles of a launch with a tail split.  SL = 1: one workgroup per tile.  SL = 4: four
// workgroups per tile, each adding and storing one group of four accumulator registers per
// 32 x 32 block (launches with few tiles: a workgroup then waits for a quarter of the partial
// sums, all of its loads in flight at once, and four times as many CUs pull them in).
//
// The partial tiles come from other XCDs, i.e. from memory: their latency, not their volume, is
// what this kernel waits for.  AHEAD shares are fetched at a time, every load issued before the
// first add (a share past the last one is an out-of-range offset that returns 0), and added in
// split order.
template <int TM, int TN, int WTM, int WTN, int NT, int C0, int C1>
__device__ inline void finish_registers(const ContractionParams& cp, const __amdgpu_buffer_rsrc_t rp, int ksplit, int m0,
                                        int n0, int zslice, int wm, int wn, int li, int h) {
    constexpr int TILE = NT * TM * TN * 16;
    constexpr int NREG = 4 * (C1 - C0);                               // registers per block this workgroup owns
    constexpr int AHEAD = 64 / (TM * TN * NREG) >= 16 ? 16 : (64 / (TM * TN * NREG) >= 4 ? 64 / (TM * TN * NREG) : 4);
    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int s0 = 0; s0 < ksplit; s0 += AHEAD) {
        float v[AHEAD][TM][TN][NREG];
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) {
            const uint32_t share = s0 + u < ksplit ? (uint32_t)threadIdx.x * 4u : OOB;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < NREG; ++r)
                        v[u][i][j][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                            rp, (int)share, ((s0 + u) * TILE + ((i * TN + j) * 16 + 4 * C0 + r) * NT) * 4, 0));
        }
#pragma unroll
        for (int u = 0; u < AHEAD; ++u)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < NREG; ++r) acc[i][j][4 * C0 + r] += v[u][i][j][r];
    }
    store_tile<TM, TN, WTM, WTN, C0, C1>(acc, m0, n0, zslice, wm, wn, li, h, cp);
}

template <int BM, int BN, int WM, int WN, int SL>
__global__ __launch_bounds__(64 * WM * WN) void splitk_finish_kernel(const ContractionParams cp, const bool tail) {
    constexpr int NT = 64 * WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int TILE = NT * TM * TN * 16;
    static_assert(SL == 1 || SL == 4, "whole blocks or single register groups");
    const int zslice = blockIdx.y * gridDim.z + blockIdx.z;
    if (zslice >= cp.nz) return;
    const int ntiles = cp.tiles_m * cp.tiles_n;
    const int ksplit = tail ? cp.tail_split : cp.ksplit;
    const int tile_index = (int)blockIdx.x / SL, part = (int)blockIdx.x % SL;
    const int logical = tail ? cp.tail_begin + tile_index : xcd_contiguous(tile_index, ntiles);
    const int64_t first_slot = tail ? (int64_t)tile_index * ksplit : ((int64_t)zslice * ntiles + tile_index) * ksplit;
    int m0, n0;
    tile_origin(cp, logical, BM, BN, m0, n0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, h = lane >> 5;
    const __amdgpu_buffer_rsrc_t rp = tile_rsrc(cp.ws_partial + first_slot * TILE);
    if constexpr (SL == 1) {
        finish_registers<TM, TN, WTM, WTN, NT, 0, 4>(cp, rp, ksplit, m0, n0, zslice, wm, wn, li, h);
    } else {
        switch (part) {                                  // uniform for the workgroup
            case 0: finish_registers<TM, TN, WTM, WTN, NT, 0, 1>(cp, rp, ksplit, m0, n0, zslice, wm, wn, li, h); break;
            case 1: finish_registers<TM, TN, WTM, WTN, NT, 1, 2>(cp, rp, ksplit, m0, n0, zslice, wm, wn, li, h); break;
            case 2: finish_registers<TM, TN, WTM, WTN, NT, 2, 3>(cp, rp, ksplit, m0, n0, zslice, wm, wn, li, h); break;
            default: finish_registers<TM, TN, WTM, WTN, NT, 3, 4>(cp, rp, ksplit, m0, n0, zslice, wm, wn, li, h); break;
        }
    }
}

// Tail split for a launch of `tiles` whole tiles that walk `nk` K steps each: how many tiles
// to leave to the tail and in how many shares to cut each of them.  A CU keeps several
// workgroups resident, so the launch ends when the CUs that received one tile more than the
// rest are done; cutting the surplus tiles into shares that cover all CUs removes most of that
// last round.  Worth it only when the last round is a sizeable part of the launch and the
// surplus is small enough that its shares get short.
struct TailSplit {
    int tiles, split;
};
inline TailSplit pick_tail(int64_t tiles, int nk, int64_t tile_elems, const float* ws, int64_t ws_floats) {
    TailSplit none = {0, 1};
    const int cus = 256;
    if (!ws || tiles <= cus || tiles > 8 * cus || nk < 8) return none;
    const int r = (int)(tiles % cus);
    if (r == 0 || r > cus / 2) return none;
    int s = cus / r;
    if (s > 16) s = 16;
    if (s > nk / 4) s = nk / 4;
    if (s < 2 || (int64_t)r * s * tile_elems > ws_floats) return none;
    TailSplit t = {r, s};
    return t;
}

constexpr int64_t kFinishSliceTiles = 128;     // up to this many tiles the finishing kernel runs four workgroups per tile

// Host side: enqueue `kernel` for the tiles of `p` and, when K ranges are split, the finishing
// kernel behind it.  `nk` = K steps a whole tile walks.
// KS = K slices inside the main kernel's workgroup (it runs 64*WM*WN*KS threads).
// SPLIT = false: a tile shape that is only ever chosen for outputs that fill whole rounds of the
// CUs (the caller passes ksplit = 1): no tail either, and no finishing kernel is instantiated.
template <int BM, int BN, int WM, int WN, int KS = 1, bool SPLIT = true, typename Kernel>
inline hipError_t launch_with_split(Kernel kernel, ContractionParams& p, int nz, int nk, int64_t ws_floats,
                                    hipStream_t stream) {
    const unsigned gz = nz < 32768 ? (unsigned)nz : 32768u;
    const unsigned gy = ((unsigned)nz + gz - 1) / gz;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    if (tiles > 0x7fffffffLL || gy > 2047u) return hipErrorInvalidValue;
    TailSplit tail = {0, 1};
    if (SPLIT && p.ksplit == 1 && nz == 1) tail = pick_tail(tiles, nk, (int64_t)BM * BN, p.ws_partial, ws_floats);
    p.tail_begin = (int)tiles - tail.tiles;
    p.tail_split = tail.split;
    const unsigned gx = (unsigned)(p.tail_begin + tail.tiles * tail.split);
    hipLaunchKernelGGL(kernel, dim3(gx, gy * (unsigned)p.ksplit, gz), dim3(64 * WM * WN * KS), 0, stream, p);
    hipError_t e = hipGetLastError();
    if constexpr (!SPLIT) return p.ksplit == 1 ? e : hipErrorInvalidValue;
    // few tiles to finish: four workgroups per tile, a group of accumulator registers each
    else if (e == hipSuccess && p.ksplit > 1) {
        if (tiles * nz <= kFinishSliceTiles)
            hipLaunchKernelGGL((splitk_finish_kernel<BM, BN, WM, WN, 4>), dim3((unsigned)tiles * 4u, gy, gz), dim3(64 * WM * WN),
                               0, stream, p, false);
        else
            hipLaunchKernelGGL((splitk_finish_kernel<BM, BN, WM, WN, 1>), dim3((unsigned)tiles, gy, gz), dim3(64 * WM * WN), 0,
                               stream, p, false);
        e = hipGetLastError();
    } else if (e == hipSuccess && tail.tiles > 0) {
        if (tail.tiles <= kFinishSliceTiles)
            hipLaunchKernelGGL((splitk_finish_kernel<BM, BN, WM, WN, 4>), dim3((unsigned)tail.tiles * 4u, 1, 1),
                               dim3(64 * WM * WN), 0, stream, p, true);
        else
            hipLaunchKernelGGL((splitk_finish_kernel<BM, BN, WM, WN, 1>), dim3((unsigned)tail.tiles, 1, 1), dim3(64 * WM * WN),
                               0, stream, p, true);
        e = hipGetLastError();
    }
    return e;
}

// KS > 1 adds K slices inside the workgroup: KS groups of WM x WN wavefronts share the staged
// tiles, slice ks walking the half-step groups [ks*G/KS, (ks+1)*G/KS) of every K step, and the
// slices' accumulators are added through LDS before the epilogue.  It doubles the wavefronts
// per SIMD for outputs with too few tiles to give every CU more than one workgroup, at the
// same LDS and global traffic per flop.
template <int BM, int BN, int BK, int WM, int WN, int KS, int AKIND, int BKIND, int AVEC, int BVEC_>
__global__ __launch_bounds__(64 * WM * WN * KS) void contraction_kernel(const ContractionParams cp) {
    constexpr int NW = WM * WN;                     // wavefronts of one K slice
    constexpr int NT = 64 * NW * KS;
    constexpr int WTM = BM / WM, WTN = BN / WN;     // wavefront sub-tile
    constexpr int TM = WTM / 32, TN = WTN / 32;     // 32x32 accumulators per wavefront
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "sub-tile of 32x32 blocks");
    static_assert(BK % 8 == 0, "K step is a multiple of the 8-wide half-step");
    constexpr int BVEC = (BKIND == LOAD_IM2COL || BKIND == LOAD_RCS) ? 1 : BVEC_;
    // Steps the global loads run ahead of the MFMAs.  Two hides the memory latency behind a whole
    // step of MFMAs; one where a step is long anyway (BK = 32 without K slices: measured 1-2 %
    // faster; with K slices a step is half or a quarter as long and two is 2-7 % faster, 20 % on a
    // 200-tile layer with K = 2048) or where the second staging set would not fit in the 128
    // registers a 1024-thread workgroup has.
    constexpr int PF = ((BK >= 32 && KS == 1) || (BM * BN >= 256 * 256 && BKIND == LOAD_IM2COL)) ? 1 : 2;
    using ALoader = TileLoader<AKIND, AVEC, BM, BK, NT, PF>;
    using BLoader = TileLoader<BKIND, BVEC, BN, BK, NT, PF>;

    // One LDS array: two buffers of the A tile, two of the B tile; the slices' partial
    // accumulators reuse it once the K walk is over.
    constexpr int A_FLOATS = ALoader::LDS_FLOATS, B_FLOATS = BLoader::LDS_FLOATS;
    constexpr int RED_FLOATS = (KS - 1) * NW * TM * TN * 16 * 64;
    constexpr int LDS_TOTAL = 2 * (A_FLOATS + B_FLOATS) > RED_FLOATS ? 2 * (A_FLOATS + B_FLOATS) : RED_FLOATS;
    static_assert(A_FLOATS % 4 == 0 && B_FLOATS % 4 == 0, "tiles keep 16-byte alignment");
    __shared__ __attribute__((aligned(16))) float lds[LDS_TOTAL];
    auto lds_a = [&](int buf) { return lds + buf * A_FLOATS; };
    auto lds_b = [&](int buf) { return lds + 2 * A_FLOATS + buf * B_FLOATS; };

    TileWork w;
    if (!tile_work(cp, BM, BN, w)) return;          // uniform for the whole workgroup
    const int m0 = w.m0, n0 = w.n0;
    int64_t a_off, b_off;
    slice_offsets(cp, w.zslice, a_off, b_off);

    ALoader la;
    BLoader lb;
    la.init(cp.A + a_off, cp.a_ld, m0, cp.M, cp.K, false, cp);
    lb.init(cp.B + b_off, cp.b_ld, n0, cp.N, cp.K, cp.col_images != 0, cp);

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ks = wave_all / NW, wave = wave_all % NW;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, h = lane >> 5;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int kt0, kt1;
    split_range((cp.K + BK - 1) / BK, w.ksplit, w.split, kt0, kt1);

    constexpr int G = BK / 8 / KS;                  // half-step groups per K step and slice
    const int g0 = ks * G;                          // this slice's first group
    constexpr int NREAD = (TM * (AKIND == LOAD_KC ? 1 : 4)) + (TN * (BKIND == LOAD_KC ? 1 : 4));   // LDS reads per group
    constexpr int NMFMA = 4 * TM * TN;              // MFMAs per group
    static_assert((BK / 8) % KS == 0 && G % 2 == 0, "fragment sets alternate per group");
    float fa[2][TM][4], fb[2][TN][4];               // fragments of two groups: one in use, one arriving
    auto frags = [&](int f, int buf, int g) {
#pragma unroll
        for (int i = 0; i < TM; ++i) ALoader::frag(lds_a(buf), wm * WTM + i * 32 + li, g, h, fa[f][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) BLoader::frag(lds_b(buf), wn * WTN + j * 32 + li, g, h, fb[f][j]);
    };
    auto mfmas = [&](int f, int s_lo, int s_hi) {
#pragma unroll
        for (int s = s_lo; s < s_hi; ++s)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[f][i][s], fb[f][j][s], acc[i][j], 0, 0, 0);
    };
    using Par0 = std::integral_constant<int, 0>;
    using Par1 = std::integral_constant<int, 1>;

    // One K step.  On entry LDS buffer s holds step kt and the fragments of the slice's first
    // group are in fragment set 0; the loads of steps kt+1 .. kt+PF-1 are in flight.
    //   issue the loads of step kt+PF
    //   groups 0 .. G-2: MFMAs of group g, the LDS reads of group g+1 in between them
    //   last group: first half of its MFMAs with the LDS stores of step kt+1 in between;
    //   barrier; second half with the LDS reads of step kt+1's first group in between.
    auto step = [&](int kt, auto S) {
        constexpr int s = decltype(S)::value;
        constexpr int set_in = PF == 2 ? s : 0;         // register set the new loads go to
        constexpr int set_out = PF == 2 ? (s ^ 1) : 0;  // register set that holds step kt+1
        la.template fetch<set_in>((kt + PF) * BK, cp);
        lb.template fetch<set_in>((kt + PF) * BK, cp);
#pragma unroll
        for (int g = 0; g + 1 < G; ++g) {
            frags((g + 1) & 1, s, g0 + g + 1);
            mfmas(g & 1, 0, 4);
#pragma unroll
            for (int q = 0; q < NMFMA; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, (NREAD + NMFMA - 1) / NMFMA, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        la.template commit<set_out>(lds_a(s ^ 1));
        lb.template commit<set_out>(lds_b(s ^ 1));
        mfmas((G - 1) & 1, 0, 2);
        __syncthreads();
        frags(0, s ^ 1, g0);
        mfmas((G - 1) & 1, 2, 4);
#pragma unroll
        for (int q = 0; q < NMFMA / 2; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, (NREAD + NMFMA / 2 - 1) / (NMFMA / 2), 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    la.template fetch<0>(kt0 * BK, cp);
    lb.template fetch<0>(kt0 * BK, cp);
    if (PF == 2) {
        la.template fetch<PF - 1>((kt0 + 1) * BK, cp);
        lb.template fetch<PF - 1>((kt0 + 1) * BK, cp);
    }
    la.template commit<0>(lds_a(0));
    lb.template commit<0>(lds_b(0));
    __syncthreads();
    frags(0, 0, g0);
    for (int kt = kt0; kt < kt1; kt += 2) {
        step(kt, Par0{});
        if (kt + 1 < kt1) step(kt + 1, Par1{});
    }

    if constexpr (KS > 1) {
        // Add the slices' accumulators in slice order: slices 1.. park theirs in LDS (register-major,
        // lane-minor: conflict-free), slice 0 adds them and goes on to the epilogue alone.
        constexpr int PER_WAVE = TM * TN * 16 * 64;
        __syncthreads();                            // every wavefront is done with the staged tiles
        if (ks > 0) {
            float* mine = lds + ((ks - 1) * NW + wave) * PER_WAVE + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mine[((i * TN + j) * 16 + r) * 64] = acc[i][j][r];
        }
        __syncthreads();
        if (ks > 0) return;
#pragma unroll
        for (int q = 1; q < KS; ++q) {
            const float* theirs = lds + ((q - 1) * NW + wave) * PER_WAVE + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += theirs[((i * TN + j) * 16 + r) * 64];
        }
    }
    finish_tile<TM, TN, WTM, WTN, 64 * NW>(acc, w, wm, wn, li, h, cp);
}

}  // namespace onnxhip
