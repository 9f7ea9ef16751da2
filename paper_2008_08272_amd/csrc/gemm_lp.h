// Contractions on 16-bit inputs (IEEE half or bfloat16) with fp32 accumulation, on the gfx950
// matrix cores: the tuned kernel behind onnx_gemm_lp, onnx_matmul_lp and the 1x1 case of
// onnx_conv_lp.
//
// The paper's operator definitions admit 16-bit floating-point tensors (Section 3.1: the
// LeakyRelu definition lists F16 next to F32 and F64).  Here Y = alpha * A * B + beta * C per
// z-slice for A [M, K], K-contiguous, and B either [N, K] (K-contiguous: Gemm with transB) or
// [K, N] (row-contiguous: Gemm without transB, MatMul, the input of a 1x1 stride-1 convolution),
// both stored as 16-bit values; products are exact in fp32 and the sum is kept in fp32
// accumulators (v_mfma_f32_32x32x16_{f16,bf16}: one MFMA consumes 16 k, each lane supplying 8
// consecutive k of its row or column).  The bias C and the epilogue arithmetic are fp32; Y is
// stored as fp32 or rounded to the input type (nearest even).
//
// Same decomposition as contraction.h: a workgroup of WM x WN wavefronts owns a BM x BN tile,
// walks K in steps of BK through two LDS buffers, global loads one or two steps ahead in
// staging registers, the 16-byte LDS reads of the next 16-k group issued in between the MFMAs
// of the current one.  LDS rows are [BK + 8] 16-bit values: the 16-byte pad makes the 16-byte reads of
// 8 neighbouring rows hit disjoint banks.
#pragma once
#include "contraction.h"

namespace onnxhip {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

enum { LP_F16 = 1, LP_BF16 = 2 };

template <int DT>
__device__ inline floatx16 mfma16(const floatx4& a, const floatx4& b, const floatx16& c) {
    if (DT == LP_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// fp32 -> 16-bit storage, round to nearest even
template <int DT>
__device__ inline uint16_t to_lp(float v) {
    if (DT == LP_F16) return __builtin_bit_cast(uint16_t, (_Float16)v);
    return __builtin_bit_cast(uint16_t, (__bf16)v);          // the hardware conversion (v_cvt_pk_bf16_f32): nearest even, NaN stays NaN
}

// K-contiguous tile loader for 16-bit elements: ROWS x BK values, 16-byte chunks of 8.
template <int ROWS, int BK, int NT, int NSETS>
struct LpLoader {
    static constexpr int CPR = BK / 8;                     // chunks per row
    static constexpr int ROWS_PER_PASS = NT / CPR;
    static constexpr int NLOAD = (ROWS + ROWS_PER_PASS - 1) / ROWS_PER_PASS;
    static constexpr int LDB = (BK + 8) * 2;               // bytes per LDS row
    static constexpr int LDS_BYTES = ROWS * LDB;
    static_assert(NT % CPR == 0 && ROWS % ROWS_PER_PASS == 0, "tile/loader mismatch");

    floatx4 reg[NSETS][NLOAD];             // staging registers: tiles of coming K steps on their way to LDS
    uint32_t voff[NLOAD];
    int chunk, row0;
    int K;
    __amdgpu_buffer_rsrc_t rsrc;

    __device__ inline void init(const uint16_t* p, int64_t ld, int first_row, int rows_total, int K_) {
        K = K_;
        chunk = threadIdx.x % CPR;
        row0 = threadIdx.x / CPR;
        const uint16_t* base = p + (int64_t)first_row * ld;
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, (int)OOB, RSRC_FLAGS);
#pragma unroll
        for (int q = 0; q < NLOAD; ++q) {
            const int row = row0 + q * ROWS_PER_PASS;
            voff[q] = first_row + row < rows_total ? (uint32_t)(row * (int)ld + chunk * 8) * 2u : OOB;
        }
    }
    // loads of the tile whose first k is k0 into register set S (k0 >= K loads nothing)
    template <int S>
    __device__ inline void fetch(int k0) {
        const bool k_ok = k0 + chunk * 8 < K;
#pragma unroll
        for (int q = 0; q < NLOAD; ++q)
            reg[S][q] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(k_ok ? voff[q] : OOB), k0 * 2, 0));
    }
    template <int S>
    __device__ inline void commit(char* lds) const {
#pragma unroll
        for (int q = 0; q < NLOAD; ++q)
            *reinterpret_cast<floatx4*>(lds + (row0 + q * ROWS_PER_PASS) * LDB + chunk * 16) = reg[S][q];
    }
    // the 8 consecutive k this lane feeds for tile-row `row`, 16-k group g, lane half h
    __device__ static inline floatx4 frag(const char* lds, int row, int g, int h) {
        return *reinterpret_cast<const floatx4*>(lds + row * LDB + g * 32 + h * 16);
    }
};

// Row-contiguous tile loader for 16-bit elements: the operand is stored [k][row] (rows next to each
// other in memory, `ld` elements between consecutive k), but the MFMA wants 8 consecutive k of one
// row from every lane.  A thread therefore fetches the same VEC rows of two consecutive k (two
// loads of VEC * 2 bytes), interleaves them in registers into (k, k+1) pairs and stores those: LDS
// holds [k pair][row] as 4-byte pairs, and a lane's 8 k of a 16-k group are four 4-byte reads, the
// lanes of a wavefront on consecutive banks.  The k order inside a group is the same as the
// K-contiguous loader's, so the two kinds can be mixed in one MFMA.
template <int ROWS, int BK, int NT, int NSETS, int VEC>
struct LpRowLoader {
    static constexpr int CPR = ROWS / VEC;                 // chunks of VEC rows per k
    static constexpr int KPP = NT / CPR;                   // k pairs per pass
    static constexpr int NTASK = (BK / 2) / KPP;           // (chunk, k pair) tasks per thread and K step
    // pairs of one k pair row; (ROWS + 8) * 4 = 32 mod 64 dwords, so the two lane halves of a
    // fragment read (4 k pairs apart) use disjoint banks
    static constexpr int LDP = (ROWS + 8) * 4;             // bytes per k pair
    static constexpr int LDS_BYTES = (BK / 2) * LDP;
    static_assert(VEC == 8 || VEC == 4, "chunks of 16 or 8 bytes");
    static_assert(NT % CPR == 0 && (BK / 2) % KPP == 0 && NTASK >= 1, "tile/loader mismatch");
    typedef uint32_t chunk_t __attribute__((ext_vector_type(VEC / 2)));

    chunk_t reg[NSETS][NTASK][2];          // [k, k+1] of each task
    const uint16_t* base;                  // column 0 of the tile (its first image), k = 0
    uint32_t vbase;                        // byte offset of (this thread's first k pair, its chunk), or OOB
    int k_first, dst0;                     // first k of that pair; where its (k, k+1) pairs go in an LDS buffer
    int K, ld;

    __device__ inline void init(const uint16_t* p, int64_t ld_, int first_col, int cols_total, int K_,
                                const ContractionParams& cp) {
        K = K_; ld = (int)ld_;
        const int chunk = threadIdx.x % CPR, kp0 = threadIdx.x / CPR;
        k_first = 2 * kp0;
        dst0 = kp0 * LDP + chunk * VEC * 4;
        const int j = first_col + chunk * VEC;
        const bool ok = j < cols_total;                    // chunks never straddle the end: cols_total % VEC == 0
        int col_off = chunk * VEC;
        base = p + first_col;
        if (cp.col_images) {                               // column j is pixel j % P of image j / P
            uint32_t n0, p0, n, px;
            cp.colP.divmod((uint32_t)first_col, n0, p0);
            cp.colP.divmod((uint32_t)(ok ? j : first_col), n, px);
            n0 = (uint32_t)scalar((int)n0);
            base = p + (int64_t)n0 * cp.b_img;
            col_off = (int)(n - n0) * (int)cp.b_img + (int)px;
        }
        vbase = ok ? (uint32_t)(col_off + 2 * kp0 * ld) * 2u : OOB;
    }
    template <int S>
    __device__ inline void fetch(int k0) {
        // the resource is re-based at row k0 so that offsets stay small whatever K is
        const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base + (int64_t)k0 * ld), 0, (int)OOB, RSRC_FLAGS);
#pragma unroll
        for (int q = 0; q < NTASK; ++q) {
            const int k = k0 + k_first + 2 * q * KPP;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int off = (int)(k + u < K ? vbase + (uint32_t)(u * ld * 2) : OOB);
                const int soff = 2 * q * KPP * ld * 2;
                if constexpr (VEC == 8) reg[S][q][u] = __builtin_bit_cast(chunk_t, __builtin_amdgcn_raw_buffer_load_b128(r, off, soff, 0));
                else reg[S][q][u] = __builtin_bit_cast(chunk_t, __builtin_amdgcn_raw_buffer_load_b64(r, off, soff, 0));
            }
        }
    }
    template <int S>
    __device__ inline void commit(char* lds) const {
#pragma unroll
        for (int q = 0; q < NTASK; ++q) {
            uint32_t out[VEC];
#pragma unroll
            for (int j = 0; j < VEC / 2; ++j) {
                const uint32_t lo = reg[S][q][0][j], hi = reg[S][q][1][j];      // rows 2j, 2j+1 of k and of k+1
                out[2 * j] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);        // row 2j:   (k, k+1)
                out[2 * j + 1] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);    // row 2j+1: (k, k+1)
            }
            char* dst = lds + dst0 + q * KPP * LDP;
#pragma unroll
            for (int j = 0; j < VEC / 4; ++j) {
                const floatx4 v = {__builtin_bit_cast(float, out[4 * j]), __builtin_bit_cast(float, out[4 * j + 1]),
                                   __builtin_bit_cast(float, out[4 * j + 2]), __builtin_bit_cast(float, out[4 * j + 3])};
                *reinterpret_cast<floatx4*>(dst + 16 * j) = v;
            }
        }
    }
    // the 8 consecutive k this lane feeds for tile-row `row`, 16-k group g, lane half h
    __device__ static inline floatx4 frag(const char* lds, int row, int g, int h) {
        floatx4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const float*>(lds + (g * 8 + h * 4 + q) * LDP + row * 4);
        return v;
    }
};

// The value a 16-bit storage word denotes.
template <int DT>
__device__ inline float from_lp(uint32_t bits16) {
    return DT == LP_F16 ? (float)__builtin_bit_cast(_Float16, (uint16_t)bits16) : __builtin_bit_cast(float, bits16 << 16);
}

// What the lane next door (lane ^ 1) holds.
__device__ inline uint32_t neighbour(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1 /* quad_perm: 1, 0, 3, 2 */, 0xf, 0xf, false);
}

// Stores a tile as 16-bit values: alpha*acc + beta*bias (none / per column / per row / full
// fp32 matrix) (+ a 16-bit residual laid out like Y), Relu, rounding.  Columns are plain columns
// of Y, or, for a convolution, (image, pixel) pairs as in store_tile.  Stores outside Y are dropped
// by the range check of the buffer resource.
//
// A lane holds one column of sixteen rows.  PAIRS = false: 2-byte stores (and residual loads), one
// per element.  PAIRS = true (every row of Y starts on a 4-byte boundary and has an even number
// of elements): two lanes next to each other, which hold columns c and c + 1 of the same rows,
// trade values so that the even lane stores both columns of one row and the odd lane both columns
// of the next row as one 4-byte word each: half as many stores, twice as wide, and the residual is
// fetched the same way.
template <int DT, int TM, int TN, int WTM, int WTN, bool HAS_RES, bool PAIRS>
__device__ __forceinline__ void store_tile_lp_as(const floatx16 (&acc)[TM][TN], const TileWork& w, int wm, int wn, int li, int h,
                                                 const ContractionParams& cp) {
    const int64_t zi = w.zslice;
    int64_t tile_off = (int64_t)w.m0 * cp.y_rs + w.n0;
    uint32_t img0 = 0, px0 = 0;
    if (cp.col_images) {
        cp.colP.divmod((uint32_t)w.n0, img0, px0);
        tile_off = (int64_t)w.m0 * cp.y_rs + (int64_t)img0 * cp.y_img + px0;
    }
    tile_off = scalar(tile_off + zi * cp.y_zs);
    img0 = (uint32_t)scalar((int)img0);
    px0 = (uint32_t)scalar((int)px0);
    uint16_t* Y = reinterpret_cast<uint16_t*>(cp.Y);
    const uint16_t* R = reinterpret_cast<const uint16_t*>(cp.residual);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(Y + tile_off, 0, (int)OOB, RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(HAS_RES ? R + tile_off : Y + tile_off), 0, (int)OOB, RSRC_FLAGS);
    const int mode = cp.bias ? cp.bias_mode : BIAS_NONE;
    const float* bias = cp.bias ? cp.bias + zi * cp.bias_zs : nullptr;
    // per-row bias through a resource over exactly the M values of this z-slice: rows beyond M read as 0
    const __amdgpu_buffer_rsrc_t rrow = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(mode == BIAS_ROW ? bias : reinterpret_cast<const float*>(Y)), 0,
                                                                          mode == BIAS_ROW ? cp.M * 4 : 0, RSRC_FLAGS);
    const bool relu = cp.relu != 0;
    const bool odd = (li & 1) != 0;
    // what depends on the column only
    int crel[TN], colv[TN];
    bool col_ok[TN];
    float col_bias[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int cl = wn * WTN + j * 32 + li;
        colv[j] = w.n0 + cl;
        col_ok[j] = colv[j] < cp.N;
        const int cj = col_ok[j] ? colv[j] : w.n0;
        crel[j] = cl;
        if (cp.col_images) {
            uint32_t n, px;
            cp.colP.divmod((uint32_t)cj, n, px);
            crel[j] = (int)(n - img0) * (int)cp.y_img + (int)px - (int)px0;
        }
        col_bias[j] = mode == BIAS_COL ? cp.beta * bias[(int64_t)cj * cp.bias_cs] : 0.f;
    }
    auto finish = [&](float a, float add) {
        const float lin = fmaf(cp.alpha, a, add);
        return relu ? fmaxf(lin, 0.f) : lin;                    // no clamp without Relu: a NaN stays a NaN
    };
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        // the bias of the 16 rows this lane's registers of block row i hold: register r is row
        // rl0 + 8*(r/4) + r%4; four consecutive rows are one 16-byte load where the block lies inside M
        const int rl0 = wm * WTM + i * 32 + 4 * h;
        float row_bias[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) row_bias[r] = 0.f;
        if (mode == BIAS_ROW) {
            if (w.m0 + wm * WTM + i * 32 + 32 <= cp.M) {         // uniform for the wavefront
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rrow, (w.m0 + rl0 + 8 * c) * 4, 0, 0));
#pragma unroll
                    for (int q = 0; q < 4; ++q) row_bias[4 * c + q] = cp.beta * v[q];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    row_bias[r] = cp.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rrow, (w.m0 + rl0 + 8 * (r / 4) + r % 4) * 4, 0, 0));
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            auto bias_of = [&](bool ok, int r, int row) {
                float add = col_bias[j] + row_bias[r];
                if (mode == BIAS_FULL) add = cp.beta * bias[ok ? (int64_t)row * cp.N + colv[j] : 0];
                return add;
            };
            if constexpr (!PAIRS) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rl = rl0 + 8 * (r / 4) + (r % 4);
                    const int row = w.m0 + rl;
                    const bool ok = col_ok[j] && row < cp.M;
                    const int off = ok ? (rl * (int)cp.y_rs + crel[j]) * 2 : (int)OOB;
                    float add = bias_of(ok, r, row);
                    if constexpr (HAS_RES) add += from_lp<DT>((uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rr, off, 0, 0));
                    __builtin_amdgcn_raw_buffer_store_b16((short)to_lp<DT>(finish(acc[i][j][r], add)), ry, off, 0, 0);
                }
            } else {
                // registers 2q and 2q + 1 hold rows rl and rl + 1 of this lane's column; the even lane
                // of a pair writes (and reads the residual of) row rl, the odd lane row rl + 1, columns
                // c and c + 1 each (N is even, so both columns exist or neither does)
                const int crel_pair = crel[j] - (odd ? 1 : 0);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int r0 = 2 * q;
                    const int rl = rl0 + 8 * (r0 / 4) + (r0 % 4);
                    const int row = w.m0 + rl;
                    const bool ok0 = col_ok[j] && row < cp.M, ok1 = col_ok[j] && row + 1 < cp.M;
                    const int my_rl = rl + (odd ? 1 : 0);
                    const int off = (odd ? ok1 : ok0) ? (my_rl * (int)cp.y_rs + crel_pair) * 2 : (int)OOB;
                    float add0 = bias_of(ok0, r0, row), add1 = bias_of(ok1, r0 + 1, row + 1);
                    if constexpr (HAS_RES) {
                        const uint32_t mine = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rr, off, 0, 0);
                        const uint32_t theirs = neighbour(mine);
                        // even lane: its word is (row rl: c, c+1), the odd lane's (row rl+1: c, c+1)
                        add0 += from_lp<DT>(odd ? theirs >> 16 : mine & 0xffffu);
                        add1 += from_lp<DT>(odd ? mine >> 16 : theirs & 0xffffu);
                    }
                    const uint32_t c0 = to_lp<DT>(finish(acc[i][j][r0], add0)), c1 = to_lp<DT>(finish(acc[i][j][r0 + 1], add1));
                    const uint32_t s0 = neighbour(c0), s1 = neighbour(c1);
                    const uint32_t lo = odd ? s1 : c0, hi = odd ? c1 : s0;
                    __builtin_amdgcn_raw_buffer_store_b32((int)(lo | (hi << 16)), ry, off, 0, 0);
                }
            }
            // one accumulator block at a time: with up to 8 blocks live, loads hoisted across blocks spill
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// The same epilogue with whole rows: a wavefront passes each 32-row strip of its WTM x WTN sub-tile
// through a piece of LDS of its own (`strip`, 32 x (WTN + 4) floats; no barrier, the wavefront
// reads back what it wrote), after which a lane owns CW = 8 (or 4) consecutive columns of one row:
// one 16-byte (8-byte) load of the residual, one such store, WTN / CW lanes next to each other
// covering a row of the sub-tile (128 contiguous bytes for a sub-tile 64 columns wide) instead of
// 4-byte words scattered over four rows.  Same arithmetic as store_tile_lp_as, in the same order except with a per-column bias.  Needs every group of 8
// columns that starts at a multiple of 8 to be contiguous in Y and 16-byte aligned (see
// store_tile_lp), and a bias that is per row or per column with unit stride.
template <int DT, int TM, int TN, int WTM, int WTN, bool HAS_RES, int CW>
__device__ __forceinline__ void store_tile_lp_rows(const floatx16 (&acc)[TM][TN], const TileWork& w, int wm, int wn, int lane,
                                                   const ContractionParams& cp, float* strip) {
    constexpr int PITCH = WTN + 4;            // floats: the 16-byte reads of two neighbouring rows hit disjoint banks
    constexpr int CPR = WTN / CW;             // chunks of CW columns per row
    typedef uint32_t chunk_t __attribute__((ext_vector_type(CW / 2)));
    static_assert(CW == 8 || CW == 4, "16-byte or 8-byte chunks");
    constexpr int RPP = 64 / CPR;             // rows per pass of the wavefront
    static_assert(WTN % 32 == 0 && 32 % RPP == 0, "strip shape");
    const int li = lane & 31, h = lane >> 5;
    const int64_t zi = w.zslice;
    int64_t tile_off = (int64_t)w.m0 * cp.y_rs + w.n0;
    uint32_t img0 = 0, px0 = 0;
    if (cp.col_images) {
        cp.colP.divmod((uint32_t)w.n0, img0, px0);
        tile_off = (int64_t)w.m0 * cp.y_rs + (int64_t)img0 * cp.y_img + px0;
    }
    tile_off = scalar(tile_off + zi * cp.y_zs);
    img0 = (uint32_t)scalar((int)img0);
    px0 = (uint32_t)scalar((int)px0);
    uint16_t* Y = reinterpret_cast<uint16_t*>(cp.Y);
    const uint16_t* R = reinterpret_cast<const uint16_t*>(cp.residual);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(Y + tile_off, 0, (int)OOB, RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(HAS_RES ? R + tile_off : Y + tile_off), 0, (int)OOB, RSRC_FLAGS);
    const int mode = cp.bias ? cp.bias_mode : BIAS_NONE;
    const float* bias = cp.bias ? cp.bias + zi * cp.bias_zs : nullptr;
    const __amdgpu_buffer_rsrc_t rrow = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(mode == BIAS_ROW ? bias : reinterpret_cast<const float*>(Y)), 0,
                                                                          mode == BIAS_ROW ? cp.M * 4 : 0, RSRC_FLAGS);
    const bool relu = cp.relu != 0;
    // this lane's chunk of 8 columns, the same in every pass
    const int cc = lane % CPR, rsub = lane / CPR;
    const int cl = wn * WTN + cc * CW;
    const int col = w.n0 + cl;
    const bool col_ok = col < cp.N;           // N is a multiple of CW: all columns of the chunk exist or none
    int crel = cl;
    if (cp.col_images) {
        uint32_t n, px;
        cp.colP.divmod((uint32_t)(col_ok ? col : w.n0), n, px);
        crel = (int)(n - img0) * (int)cp.y_img + (int)px - (int)px0;
    }
    // A per-column bias is added on the way into the strip, where a lane holds one column per block (one value
    // per block instead of eight per lane afterwards): alpha * acc + bias is rounded there and the residual added
    // to it, where the other bias kinds add bias and residual first.
    const bool colmode = mode == BIAS_COL;
    float col_bias[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int c = w.n0 + wn * WTN + j * 32 + li;
        col_bias[j] = (colmode && c < cp.N) ? cp.beta * bias[c] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        constexpr int NPASS = 32 / RPP;
        // what the passes of this strip need from memory, all requested before the strip goes through LDS
        int off[NPASS];
        float row_bias[NPASS];
        chunk_t res[NPASS];
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            const int row_in_tile = wm * WTM + i * 32 + pass * RPP + rsub;
            const int row = w.m0 + row_in_tile;
            off[pass] = (col_ok && row < cp.M) ? (row_in_tile * (int)cp.y_rs + crel) * 2 : (int)OOB;
            row_bias[pass] = 0.f;
            if (mode == BIAS_ROW) row_bias[pass] = cp.beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rrow, row * 4, 0, 0));
            if constexpr (HAS_RES) {
                if constexpr (CW == 8) res[pass] = __builtin_bit_cast(chunk_t, __builtin_amdgcn_raw_buffer_load_b128(rr, off[pass], 0, 0));
                else res[pass] = __builtin_bit_cast(chunk_t, __builtin_amdgcn_raw_buffer_load_b64(rr, off[pass], 0, 0));
            }
        }
        // register r of block (i, j) is row 4h + 8*(r/4) + r%4, column j*32 + li of the strip
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                strip[(4 * h + 8 * (r / 4) + (r % 4)) * PITCH + j * 32 + li] = colmode ? fmaf(cp.alpha, acc[i][j][r], col_bias[j]) : acc[i][j][r];
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            const int rl = pass * RPP + rsub;
            float a[CW];
#pragma unroll
            for (int q = 0; q < CW / 4; ++q) {
                const floatx4 v = *reinterpret_cast<const floatx4*>(strip + rl * PITCH + cc * CW + 4 * q);
                a[4 * q] = v.x; a[4 * q + 1] = v.y; a[4 * q + 2] = v.z; a[4 * q + 3] = v.w;
            }
            chunk_t out;
#pragma unroll
            for (int k = 0; k < CW / 2; ++k) {
                float add0 = row_bias[pass], add1 = row_bias[pass];
                if constexpr (HAS_RES) {
                    add0 += from_lp<DT>(res[pass][k] & 0xffffu);
                    add1 += from_lp<DT>(res[pass][k] >> 16);
                }
                const float l0 = colmode ? a[2 * k] + add0 : fmaf(cp.alpha, a[2 * k], add0);
                const float l1 = colmode ? a[2 * k + 1] + add1 : fmaf(cp.alpha, a[2 * k + 1], add1);
                const uint32_t c0 = to_lp<DT>(relu ? fmaxf(l0, 0.f) : l0), c1 = to_lp<DT>(relu ? fmaxf(l1, 0.f) : l1);
                out[k] = c0 | (c1 << 16);
            }
            if constexpr (CW == 8) __builtin_amdgcn_raw_buffer_store_b128(out, ry, off[pass], 0, 0);
            else __builtin_amdgcn_raw_buffer_store_b64(out, ry, off[pass], 0, 0);
        }
        // one strip at a time: loads hoisted across strips would keep their registers live through the whole epilogue
        __builtin_amdgcn_sched_barrier(0);
    }
}

// LDS bytes a wavefront's strip takes in store_tile_lp_rows.
template <int WTN>
constexpr int lp_strip_bytes() { return 32 * (WTN + 4) * 4; }

// `strip`: this wavefront's lp_strip_bytes<WTN>() of LDS that nothing else uses any more (the caller
// has passed a barrier behind the last read of its operand buffers), or nullptr.
template <int DT, int TM, int TN, int WTM, int WTN>
__device__ __forceinline__ void store_tile_lp(const floatx16 (&acc)[TM][TN], const TileWork& w, int wm, int wn, int li, int h,
                                              const ContractionParams& cp, float* strip = nullptr) {
    // whole rows: every aligned group of 8 (or 4) columns contiguous in Y (and the residual) and on a 16-byte (8-byte) boundary
    const int64_t strides = cp.N | cp.y_rs | cp.y_zs | (cp.col_images ? (int64_t)cp.colP.d | cp.y_img : 0);
    const uintptr_t bases = reinterpret_cast<uintptr_t>(cp.Y) | reinterpret_cast<uintptr_t>(cp.residual);
    const int bmode = cp.bias ? cp.bias_mode : BIAS_NONE;
    const bool rows_ok = strip != nullptr && bmode != BIAS_FULL && (bmode != BIAS_COL || cp.bias_cs == 1);
    if (rows_ok && (strides & 7) == 0 && (bases & 15u) == 0) {
        if (cp.residual) store_tile_lp_rows<DT, TM, TN, WTM, WTN, true, 8>(acc, w, wm, wn, li + 32 * h, cp, strip);
        else store_tile_lp_rows<DT, TM, TN, WTM, WTN, false, 8>(acc, w, wm, wn, li + 32 * h, cp, strip);
        return;
    }
    if (rows_ok && (strides & 3) == 0 && (bases & 7u) == 0) {
        if (cp.residual) store_tile_lp_rows<DT, TM, TN, WTM, WTN, true, 4>(acc, w, wm, wn, li + 32 * h, cp, strip);
        else store_tile_lp_rows<DT, TM, TN, WTM, WTN, false, 4>(acc, w, wm, wn, li + 32 * h, cp, strip);
        return;
    }
    // Copies of the epilogue rather than tests per element; all must be inlined: a call would pass the
    // accumulators through memory.  Pairs need every (row, even column) of Y and of the residual on a
    // 4-byte boundary and both columns of a pair in the same row or image.
    const bool even_strides = ((cp.N | cp.y_rs | cp.y_zs | (cp.col_images ? (int64_t)cp.colP.d | cp.y_img : 0)) & 1) == 0;
    const bool pairs = even_strides && (reinterpret_cast<uintptr_t>(cp.Y) & 3u) == 0 && (reinterpret_cast<uintptr_t>(cp.residual) & 3u) == 0;
    if (cp.residual) {
        if (pairs) store_tile_lp_as<DT, TM, TN, WTM, WTN, true, true>(acc, w, wm, wn, li, h, cp);
        else store_tile_lp_as<DT, TM, TN, WTM, WTN, true, false>(acc, w, wm, wn, li, h, cp);
    } else {
        if (pairs) store_tile_lp_as<DT, TM, TN, WTM, WTN, false, true>(acc, w, wm, wn, li, h, cp);
        else store_tile_lp_as<DT, TM, TN, WTM, WTN, false, false>(acc, w, wm, wn, li, h, cp);
    }
}

// A workgroup's share of a tile whose K range is split: parked in the workspace, register-major and
// thread-minor (every access coalesced), for lp_finish_kernel.
template <int TM, int TN, int NT>
__device__ __forceinline__ void park_partial_tile(const floatx16 (&acc)[TM][TN], const TileWork& w, const ContractionParams& cp) {
    constexpr int TILE = NT * TM * TN * 16;
    float* mine = cp.ws_partial + w.slot * TILE + threadIdx.x;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[((i * TN + j) * 16 + r) * NT] = acc[i][j][r];
}

// Second half of a product whose K range was split over several workgroups per tile (park_partial_tile
// above).  One wavefront per workgroup, WM * WN workgroups per tile (these launches have few tiles: as one
// workgroup per tile they took half as long again), each with the thread-to-accumulator mapping of the
// wavefront that parked its part of the shares; the shares of a tile are added in split order (four
// requested at a time, a share past the last one being an out-of-range offset that returns 0), then the
// same epilogues.  Grid: (tiles * WM * WN, z-slices).
template <int BM, int BN, int WM, int WN, int DT, bool LP_OUT>
__global__ __launch_bounds__(64) void lp_finish_kernel(const ContractionParams cp) {
    constexpr int NT = 64 * WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int TILE = NT * TM * TN * 16;
    constexpr int AHEAD = 4;
    TileWork w;
    w.zslice = blockIdx.y * gridDim.z + blockIdx.z;
    if (w.zslice >= cp.nz) return;
    const int ntiles = cp.tiles_m * cp.tiles_n;
    const int tile = blockIdx.x / (WM * WN), wave = blockIdx.x % (WM * WN);
    w.ksplit = 1; w.split = 0; w.slot = 0;
    tile_origin(cp, xcd_contiguous(tile, ntiles), BM, BN, w.m0, w.n0);
    w.m0 = scalar(w.m0); w.n0 = scalar(w.n0); w.zslice = scalar(w.zslice);
    const int lane = threadIdx.x;
    const int tid = wave * 64 + lane;                // this thread's index in the workgroup that parked the shares
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, h = lane >> 5;
    const int64_t first_slot = ((int64_t)w.zslice * ntiles + tile) * cp.ksplit;
    const __amdgpu_buffer_rsrc_t rp = tile_rsrc(cp.ws_partial + first_slot * TILE);
    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            for (int s0 = 0; s0 < cp.ksplit; s0 += AHEAD) {
                float v[AHEAD][16];
#pragma unroll
                for (int u = 0; u < AHEAD; ++u) {
                    const uint32_t share = s0 + u < cp.ksplit ? (uint32_t)tid * 4u : OOB;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        v[u][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                      rp, (int)share, ((s0 + u) * TILE + ((i * TN + j) * 16 + r) * NT) * 4, 0));
                }
#pragma unroll
                for (int u = 0; u < AHEAD; ++u)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += v[u][r];
            }
        }
    if constexpr (LP_OUT) store_tile_lp<DT, TM, TN, WTM, WTN>(acc, w, wm, wn, li, h, cp);
    else store_tile<TM, TN, WTM, WTN>(acc, w.m0, w.n0, w.zslice, wm, wn, li, h, cp);
}

// BKIND: LOAD_KC (B stored [N][K], 16-byte chunks of 8 k) or LOAD_RC (B stored [K][N], chunks of
// BVEC columns).
template <int BM, int BN, int BK, int WM, int WN, int DT, bool LP_OUT, int PF, int BKIND, int BVEC>
__global__ __launch_bounds__(64 * WM * WN) void gemm_lp_kernel(const ContractionParams cp) {
    constexpr int NT = 64 * WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int G = BK / 16;                       // 16-k groups per K step
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0 && BK % 32 == 0, "tile shape");
    static_assert(BKIND == LOAD_KC || BKIND == LOAD_RC, "B is K-contiguous or row-contiguous");
    using ALoader = LpLoader<BM, BK, NT, PF>;
    using BLoader = std::conditional_t<BKIND == LOAD_KC, LpLoader<BN, BK, NT, PF>, LpRowLoader<BN, BK, NT, PF, BVEC>>;

    __shared__ __attribute__((aligned(16))) char lds_a[2][ALoader::LDS_BYTES];
    __shared__ __attribute__((aligned(16))) char lds_b[2][BLoader::LDS_BYTES];

    TileWork w;
    if (!tile_work(cp, BM, BN, w)) return;
    w.m0 = scalar(w.m0); w.n0 = scalar(w.n0); w.zslice = scalar(w.zslice);
    const int m0 = w.m0, n0 = w.n0;
    int64_t a_off, b_off;
    slice_offsets(cp, w.zslice, a_off, b_off);
    a_off = scalar(a_off);
    b_off = scalar(b_off);

    ALoader la;
    BLoader lb;
    la.init(reinterpret_cast<const uint16_t*>(cp.A) + a_off, cp.a_ld, m0, cp.M, cp.K);
    if constexpr (BKIND == LOAD_KC) lb.init(reinterpret_cast<const uint16_t*>(cp.B) + b_off, cp.b_ld, n0, cp.N, cp.K);
    else lb.init(reinterpret_cast<const uint16_t*>(cp.B) + b_off, cp.b_ld, n0, cp.N, cp.K, cp);

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

    int kt0, kt1;
    split_range((cp.K + BK - 1) / BK, w.ksplit, w.split, kt0, kt1);
    kt0 = scalar(kt0); kt1 = scalar(kt1);

    floatx4 fa[2][TM], fb[2][TN];                    // fragments of two groups: one in use, one arriving
    auto frags = [&](int f, int buf, int g) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[f][i] = ALoader::frag(lds_a[buf], wm * WTM + i * 32 + li, g, h);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[f][j] = BLoader::frag(lds_b[buf], wn * WTN + j * 32 + li, g, h);
    };
    auto mfmas = [&](int f, int i_lo, int i_hi) {
#pragma unroll
        for (int i = i_lo; i < i_hi; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = mfma16<DT>(fa[f][i], fb[f][j], acc[i][j]);
    };
    constexpr int NREAD = TM + TN * (BKIND == LOAD_KC ? 1 : 4), NMFMA = TM * TN;
    constexpr int HALF = TM > 1 ? TM / 2 : 1;        // rows of accumulator blocks issued before the barrier

    // One K step (see contraction.h): loads PF steps ahead issued first; groups 0 .. G-2 with the
    // next group's LDS reads in between their MFMAs; the last group split around the barrier,
    // the LDS stores of the next tile before it, the first reads of the next step after it.
    using Par0 = std::integral_constant<int, 0>;
    using Par1 = std::integral_constant<int, 1>;
    auto step = [&](int kt, auto S) {
        constexpr int s = decltype(S)::value;
        constexpr int set_in = PF == 2 ? s : 0, set_out = PF == 2 ? (s ^ 1) : 0;
        la.template fetch<set_in>((kt + PF) * BK);
        lb.template fetch<set_in>((kt + PF) * BK);
#pragma unroll
        for (int g = 0; g + 1 < G; ++g) {
            frags((g + 1) & 1, s, g + 1);
            mfmas(g & 1, 0, TM);
#pragma unroll
            for (int q = 0; q < NMFMA; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, (NREAD + NMFMA - 1) / NMFMA, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        la.template commit<set_out>(lds_a[s ^ 1]);
        lb.template commit<set_out>(lds_b[s ^ 1]);
        mfmas((G - 1) & 1, 0, HALF);
        __syncthreads();
        frags(0, s ^ 1, 0);
        if (HALF < TM) mfmas((G - 1) & 1, HALF, TM);
        __builtin_amdgcn_sched_barrier(0);
    };

    la.template fetch<0>(kt0 * BK);
    lb.template fetch<0>(kt0 * BK);
    if (PF == 2) {
        la.template fetch<PF - 1>((kt0 + 1) * BK);
        lb.template fetch<PF - 1>((kt0 + 1) * BK);
    }
    la.template commit<0>(lds_a[0]);
    lb.template commit<0>(lds_b[0]);
    __syncthreads();
    frags(0, 0, 0);
    for (int kt = kt0; kt < kt1; kt += 2) {
        step(kt, Par0{});
        if (kt + 1 < kt1) step(kt + 1, Par1{});
    }

    // K split over several workgroups (only the 64 x 64 tile is ever launched that way; in the larger instances the
    // parking code alone cost the registers of their second workgroup per CU): lp_finish_kernel does the rest
    if constexpr (BM == 64 && BN == 64) {
        if (w.ksplit > 1) {
            park_partial_tile<TM, TN, NT>(acc, w, cp);
            return;
        }
    }
    if constexpr (LP_OUT) {
        static_assert(WM * WN * lp_strip_bytes<WTN>() <= 2 * ALoader::LDS_BYTES, "the strips of the epilogue fit in A's buffers");
        __syncthreads();                             // every wavefront is done reading the operand buffers
        store_tile_lp<DT, TM, TN, WTM, WTN>(acc, w, wm, wn, li, h, cp,
                                            reinterpret_cast<float*>(&lds_a[0][0] + wave * lp_strip_bytes<WTN>()));
    } else {
        finish_tile<TM, TN, WTM, WTN, NT>(acc, w, wm, wn, li, h, cp);
    }
}

}  // namespace onnxhip
