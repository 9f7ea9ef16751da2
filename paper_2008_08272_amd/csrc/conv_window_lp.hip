// 3x3 convolution on 16-bit tensors (IEEE half or bfloat16, fp32 accumulation) with an
// LDS-resident input patch, on the gfx950 matrix cores: the tuned kernel behind the 3x3 case of
// onnx_conv_lp.
//
// Same ONNX Conv semantics and the same tiling and patch geometry as conv_window.h (BM output
// channels x BN consecutive positions of the flattened (image, oh, ow) index; the rectangle of
// input rows and columns those positions touch is staged in LDS once per K step and every
// filter tap reads it at lane base + a uniform offset).  What differs is the MFMA:
// v_mfma_f32_32x32x16 consumes 16 k, each lane supplying 8 consecutive k of its row or column.
// Here the 16 k of one MFMA are 16 input channels at one filter tap, a K step is 16 channels x
// 9 taps, and both operands are laid out so that a lane's 8 channels are one 16-byte LDS read:
//   patch:   [8-channel half][patch row][patch column][8 channels]; the input is NCHW, so a thread
//            loads the 8 channels of one patch position with eight 2-byte loads (coalesced along
//            the row across lanes), packs them and stores 16 bytes.  When the input rows have even
//            length (and the tensor starts on a 4-byte boundary) the patch starts at an even input
//            column instead and a thread loads two neighbouring positions with eight 4-byte loads;
//   filters: rows of [tap][16 channels] per K step.  ONNX stores them [channel][tap], which no
//            16-byte load can turn into channel-contiguous fragments, so a small kernel ahead of
//            the convolution rewrites the filter bank once into [M][C/16][tap][16 channels] (in the
//            caller's workspace); the main kernel then loads whole 16-byte fragments, coalesced.
#include "gemm_lp.h"
#include "internal.h"

namespace onnxhip {

namespace {

constexpr int LPW_CB = 16;                    // input channels per K step
constexpr int LPW_TAPS = 9;
constexpr int LPW_KA = LPW_CB * LPW_TAPS;     // filter values per row per step: 288 bytes
constexpr int LPW_CPR = LPW_KA / 8;           // 16-byte chunks per row per step: chunk q = tap * 2 + channel half
constexpr int LPW_LDA = LPW_KA * 2 + 16;      // bytes per LDS row: 16-byte reads of 16 neighbouring rows hit disjoint banks

// W [rows][Cg][9] -> P [rows][Cg/16][9][16], one 16-byte chunk of P per thread.  (A thread per 288-byte
// row block with 16-byte loads and the pairing done in registers was slower: 5-10 us against 2.5-7, too few threads.)
__global__ __launch_bounds__(256) void lp_filter_taps_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ P,
                                                            int64_t chunks, int Cg) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= chunks) return;
    const int per_row = Cg / 16 * LPW_CPR;
    const int64_t row = e / per_row;
    const int r = (int)(e - row * per_row);
    const int g16 = r / LPW_CPR, q = r % LPW_CPR;
    const int tap = q >> 1, half = q & 1;
    const uint16_t* src = W + (row * Cg + g16 * 16 + half * 8) * LPW_TAPS + tap;
    uint32_t v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = (uint32_t)src[2 * c * LPW_TAPS] | ((uint32_t)src[(2 * c + 1) * LPW_TAPS] << 16);
    uint4 o;
    o.x = v[0]; o.y = v[1]; o.z = v[2]; o.w = v[3];
    reinterpret_cast<uint4*>(P)[e] = o;
}

// NPU = passes of NT threads over the units of one step, a unit being (channel half, patch
// position) or, with PAIR, (channel half, two neighbouring positions of a patch row); surplus
// units are out-of-range buffer loads, which fetch nothing and return zero.  The host sets the
// geometry to match: patch pitch PC (even with PAIR), plane = patch rows * PC, and the divisors
// planed / PCd = units per channel half / per patch row.  With PAIR patch column 0 is input column
// -pL rounded down to an even one, so an odd pL shifts every read one column to the right.
//
// Schedule of one K step, as in conv_window.h: global loads of step ks+2 first; the three filter
// rows of taps one after the other, the next row's LDS reads in between the current row's MFMAs;
// the LDS stores of step ks+1 and the barrier inside the last row.
template <int BM, int BN, int WM, int WN, int DT, bool LP_OUT, bool PAIR, int NPU>
__global__ __launch_bounds__(64 * WM * WN) void conv_window_lp_kernel(const ContractionParams cp) {
    constexpr int UW = PAIR ? 2 : 1;            // patch positions per unit
    constexpr int NT = 64 * WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int NA = BM * LPW_CPR;            // 16-byte loads per filter tile
    constexpr int PA = (NA + NT - 1) / NT;
    constexpr int NG = 3, GT = 3;               // tap groups (filter rows) per step, taps per group
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "sub-tile of 32x32 blocks");

    __shared__ __attribute__((aligned(16))) char lds_a[2][BM * LPW_LDA + 16];   // + a slot that absorbs the stores of surplus threads
    __shared__ __attribute__((aligned(16))) char lds_b[2][NPU * NT * UW * 16];

    TileWork w;
    if (!tile_work(cp, BM, BN, w)) return;
    w.m0 = scalar(w.m0); w.n0 = scalar(w.n0); w.zslice = scalar(w.zslice);
    const int m0 = w.m0, n0 = w.n0;
    int64_t a_off, b_off;
    slice_offsets(cp, w.zslice, a_off, b_off);
    a_off = scalar(a_off); b_off = scalar(b_off);
    const Im2colGeom& g = cp.ic;
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, h = lane >> 5;

    // ---- geometry of this tile's patch (see conv_window.h)
    uint32_t q_first, ow_first, img_first, oh0;
    g.OW.divmod((uint32_t)n0, q_first, ow_first);
    g.OHd.divmod(q_first, img_first, oh0);
    img_first = (uint32_t)scalar((int)img_first);
    oh0 = (uint32_t)scalar((int)oh0);
    const int PS1 = (g.OH - 1 - (int)oh0) * g.sH + g.E;
    const int n_images = cp.N / (int)cp.colP.d;
    const int pshift = PAIR ? (g.pL & 1) : 0;

    // ---- filter tile loader: thread -> (row, 16-byte chunk), fixed for the whole K walk
    const uint16_t* a_base = reinterpret_cast<const uint16_t*>(cp.A) + a_off + (int64_t)m0 * cp.K;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a_base), 0, (int)OOB, RSRC_FLAGS);
    uint32_t voff_a[PA];
    int dst_a[PA];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int e = t + p * NT;
        const int row = e / LPW_CPR, q = e % LPW_CPR;
        const bool ok = e < NA && m0 + row < cp.M;
        voff_a[p] = ok ? (uint32_t)(row * cp.K + q * 8) * 2u : OOB;
        dst_a[p] = e < NA ? row * LPW_LDA + q * 16 : BM * LPW_LDA;
    }
    // ---- patch loader: thread -> (channel half, patch row, patch col), fixed for the whole K walk
    const uint16_t* b_base = reinterpret_cast<const uint16_t*>(cp.B) + b_off + (int64_t)img_first * g.image_stride;
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(b_base), 0, (int)OOB, RSRC_FLAGS);
    const int HW = g.H * g.W;
    uint32_t voff_b[NPU];
#pragma unroll
    for (int p = 0; p < NPU; ++p) {
        const uint32_t e = (uint32_t)(t + p * NT);
        uint32_t hh, rem, pr, pu;
        g.planed.divmod(e, hh, rem);
        g.PCd.divmod(rem, pr, pu);
        uint32_t a = 0, local = pr;
        if ((int)pr >= PS1) {
            g.IPRd.divmod(pr - (uint32_t)PS1, a, local);
            a += 1;
        }
        const int ih = (a == 0 ? (int)oh0 * g.sH : 0) - g.pT + (int)local;
        const int iw = (int)pu * UW - g.pL - pshift;     // PAIR: even, and so is W: both columns exist or neither
        const bool ok = hh < 2u && (int)(img_first + a) < n_images && (unsigned)ih < (unsigned)g.H &&
                        (unsigned)iw < (unsigned)g.W;
        voff_b[p] = ok ? (uint32_t)((int)a * g.image_stride + (int)hh * 8 * HW + ih * g.W + iw) * 2u : OOB;
    }
    // ---- where this lane reads its operands for the MFMAs (byte offsets)
    int rd_a[TM], rd_b[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) rd_a[i] = (wm * WTM + i * 32 + li) * LPW_LDA + h * 16;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int col = n0 + wn * WTN + j * 32 + li;
        if (col >= cp.N) col = n0;
        uint32_t q, ow, img, oh;
        g.OW.divmod((uint32_t)col, q, ow);
        g.OHd.divmod(q, img, oh);
        const int a = (int)(img - img_first);
        const int prow = a == 0 ? ((int)oh - (int)oh0) * g.sH : PS1 + (a - 1) * g.IPR + (int)oh * g.sH;
        rd_b[j] = (prow * g.PC + (int)ow * g.sW + pshift + h * g.plane) * 16;
    }
    int tap_b[LPW_TAPS];                             // uniform patch offset of each tap, in bytes
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) tap_b[kh * 3 + kw] = (kh * g.dH * g.PC + kw * g.dW) * 16;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int ks0, ks1;                                   // the K steps this workgroup walks (all of them unless K is split)
    split_range(g.Cg / LPW_CB, w.ksplit, w.split, ks0, ks1);
    ks0 = scalar(ks0); ks1 = scalar(ks1);
    const int chan_bytes = scalar(HW * 2);

    floatx4 reg_a[2][PA];
    std::conditional_t<PAIR, uint32_t, uint16_t> reg_b[2][NPU][8];
    using Set0 = std::integral_constant<int, 0>;
    using Set1 = std::integral_constant<int, 1>;

    // Loads of step ks into register set S; a step past the end of the walk loads nothing.
    auto fetch = [&](int ks, auto S) {
        constexpr int s = decltype(S)::value;
        const uint32_t past = ks < ks1 ? 0u : OOB;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            reg_a[s][p] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(ra, (int)(voff_a[p] | past), ks * LPW_KA * 2, 0));
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int soff = (ks * LPW_CB + c) * chan_bytes;
#pragma unroll
            for (int p = 0; p < NPU; ++p) {
                if constexpr (PAIR) reg_b[s][p][c] = __builtin_amdgcn_raw_buffer_load_b32(rb, (int)(voff_b[p] | past), soff, 0);
                else reg_b[s][p][c] = __builtin_amdgcn_raw_buffer_load_b16(rb, (int)(voff_b[p] | past), soff, 0);
            }
        }
    };
    auto commit = [&](int buf, auto S) {
        constexpr int s = decltype(S)::value;
#pragma unroll
        for (int p = 0; p < PA; ++p) *reinterpret_cast<floatx4*>(lds_a[buf] + dst_a[p]) = reg_a[s][p];
#pragma unroll
        for (int p = 0; p < NPU; ++p) {
            uint4 v;
            if constexpr (PAIR) {                    // low halves: the even column; high halves: its right neighbour
                uint4 v1;
                v.x = __builtin_amdgcn_perm(reg_b[s][p][1], reg_b[s][p][0], 0x05040100u);
                v.y = __builtin_amdgcn_perm(reg_b[s][p][3], reg_b[s][p][2], 0x05040100u);
                v.z = __builtin_amdgcn_perm(reg_b[s][p][5], reg_b[s][p][4], 0x05040100u);
                v.w = __builtin_amdgcn_perm(reg_b[s][p][7], reg_b[s][p][6], 0x05040100u);
                v1.x = __builtin_amdgcn_perm(reg_b[s][p][1], reg_b[s][p][0], 0x07060302u);
                v1.y = __builtin_amdgcn_perm(reg_b[s][p][3], reg_b[s][p][2], 0x07060302u);
                v1.z = __builtin_amdgcn_perm(reg_b[s][p][5], reg_b[s][p][4], 0x07060302u);
                v1.w = __builtin_amdgcn_perm(reg_b[s][p][7], reg_b[s][p][6], 0x07060302u);
                *reinterpret_cast<uint4*>(lds_b[buf] + (t + p * NT) * 32) = v;
                *reinterpret_cast<uint4*>(lds_b[buf] + (t + p * NT) * 32 + 16) = v1;
            } else {
                v.x = (uint32_t)reg_b[s][p][0] | ((uint32_t)reg_b[s][p][1] << 16);
                v.y = (uint32_t)reg_b[s][p][2] | ((uint32_t)reg_b[s][p][3] << 16);
                v.z = (uint32_t)reg_b[s][p][4] | ((uint32_t)reg_b[s][p][5] << 16);
                v.w = (uint32_t)reg_b[s][p][6] | ((uint32_t)reg_b[s][p][7] << 16);
                *reinterpret_cast<uint4*>(lds_b[buf] + (t + p * NT) * 16) = v;
            }
        }
    };
    floatx4 fa[2][GT][TM], fb[2][GT][TN];
    auto frags = [&](int f, const char* sa, const char* sb, int grp) {
#pragma unroll
        for (int u = 0; u < GT; ++u) {
            const int tap = grp * GT + u;
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[f][u][i] = *reinterpret_cast<const floatx4*>(sa + rd_a[i] + tap * 32);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[f][u][j] = *reinterpret_cast<const floatx4*>(sb + rd_b[j] + tap_b[tap]);
        }
    };
    auto mfmas = [&](int f, int u_lo, int u_hi) {
#pragma unroll
        for (int u = u_lo; u < u_hi; ++u)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = mfma16<DT>(fa[f][u][i], fb[f][u][j], acc[i][j]);
    };
    constexpr int NREAD = GT * (TM + TN), NMFMA = GT * TM * TN;
    // On entry LDS buffer s holds step ks and the fragments of its first tap group are in
    // fragment set s (the sets alternate with the groups, three groups per step).
    auto step = [&](int ks, auto S, auto SN) {
        constexpr int s = decltype(S)::value;
        fetch(ks + 2, S);
#pragma unroll
        for (int grp = 0; grp + 1 < NG; ++grp) {
            frags((grp + 1 + s) & 1, lds_a[s], lds_b[s], grp + 1);
            mfmas((grp + s) & 1, 0, GT);
#pragma unroll
            for (int q = 0; q < NMFMA; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, (NREAD + NMFMA - 1) / NMFMA, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        commit(s ^ 1, SN);                           // past the end this stores zeros nobody reads
        mfmas((NG - 1 + s) & 1, 0, 1);
        __syncthreads();
        frags((NG + s) & 1, lds_a[s ^ 1], lds_b[s ^ 1], 0);      // next step's first group
        mfmas((NG - 1 + s) & 1, 1, GT);
        constexpr int NREST = (GT - 1) * TM * TN;
#pragma unroll
        for (int q = 0; q < NREST; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, (NREAD + NREST - 1) / NREST, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    fetch(ks0, Set0{});
    fetch(ks0 + 1, Set1{});
    commit(0, Set0{});
    __syncthreads();
    frags(0, lds_a[0], lds_b[0], 0);
    for (int ks = ks0; ks < ks1; ks += 2) {
        step(ks, Set0{}, Set1{});
        if (ks + 1 < ks1) step(ks + 1, Set1{}, Set0{});
    }
    // With K split over several workgroups the partial tile is parked in the workspace (register-major,
    // thread-minor, as finish_tile does) and lp_finish_kernel adds the shares and runs the epilogue.
    if constexpr (BM == BN) {                        // (the 64 x 128 tile is never launched with a split)
        if (w.ksplit > 1) {
            park_partial_tile<TM, TN, NT>(acc, w, cp);
            return;
        }
    }
    if constexpr (LP_OUT) {
        static_assert(WM * WN * lp_strip_bytes<WTN>() <= 2 * (BM * LPW_LDA + 16), "the strips of the epilogue fit in the filter buffers");
        __syncthreads();                             // every wavefront is done reading the operand buffers
        store_tile_lp<DT, TM, TN, WTM, WTN>(acc, w, wm, wn, li, h, cp,
                                            reinterpret_cast<float*>(&lds_a[0][0] + wave * lp_strip_bytes<WTN>()));
    }
    else finish_tile<TM, TN, WTM, WTN, NT>(acc, w, wm, wn, li, h, cp);
}

struct WindowLpConfig {
    int bm, bn, nt, max_units;
    int resident;      // workgroups all CUs hold at once (LDS-limited)
    double weight;     // time of one workgroup relative to the 64 x 64 tile's
};
// Keep in step with the template instances in launch_config below.  Measured on ResNet-50's 3x3 layers at batch 32
// (bf16): a 128 x 128 workgroup of eight wavefronts takes 1.1-1.45 times as long as a 64 x 64 one of four, a
// 64 x 128 one of four (for layers with 64 filters or fewer: twice the positions per filter tile) 1.5 times.
const WindowLpConfig kConfigs[] = {
    {64, 64, 256, 8, 512, 1.0},
    {128, 128, 512, 4, 256, 1.4},
    {64, 128, 256, 8, 512, 1.5},
};
const int kNumConfigs = sizeof(kConfigs) / sizeof(kConfigs[0]);

// Patch rows a tile of `bn` consecutive output positions can need, in the worst case.
int patch_rows(int bn, int OH, int OW, int sH, int E) {
    const int nr = bn == 1 ? 1 : (bn - 2) / OW + 2;             // output rows touched
    int nimg = nr == 1 ? 1 : (nr - 2) / OH + 2;                 // images touched
    if (nimg > nr) nimg = nr;
    const int per_image = E > sH ? E : sH;
    return (nr - nimg) * sH + nimg * per_image;
}

// The workspace a launch may park split-K shares in (what is left of the caller's behind the rewritten
// filter bank, if that lives there too).
struct SplitSpace {
    float* partial;
    int64_t floats;
};

template <int BM, int BN, int WM, int WN, int DT, bool LP_OUT, bool PAIR, int NPU>
hipError_t launch_instance(ContractionParams& p, int nz, const SplitSpace& space, hipStream_t stream) {
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    p.nz = nz;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const Workspace ws = {space.partial, space.floats};
    // few tiles (small batches, the 7 x 7 layers): split the channel steps over several workgroups per tile.  The
    // 64 x 128 tile is only ever chosen for more tiles than a split pays for: it has no finishing kernel.
    constexpr bool kMaySplit = BM == BN;
    p.ksplit = kMaySplit ? pick_split(tiles * nz, p.ic.Cg / LPW_CB, (int64_t)BM * BN, 4.0, ws) : 1;
    p.ws_partial = space.partial;
    p.tail_begin = (int)tiles;
    p.tail_split = 1;
    const unsigned gz = nz < 32768 ? (unsigned)nz : 32768u;
    const unsigned gy = ((unsigned)nz + gz - 1) / gz;
    if (tiles * (WM * WN) > 0x7fffffffLL || gy * (unsigned)p.ksplit > 65535u) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv_window_lp_kernel<BM, BN, WM, WN, DT, LP_OUT, PAIR, NPU>), dim3((unsigned)tiles, gy * (unsigned)p.ksplit, gz),
                       dim3(64 * WM * WN), 0, stream, p);
    hipError_t e = hipGetLastError();
    if constexpr (kMaySplit) {
        if (e == hipSuccess && p.ksplit > 1) {
            hipLaunchKernelGGL((lp_finish_kernel<BM, BN, WM, WN, DT, LP_OUT>), dim3((unsigned)tiles * (WM * WN), gy, gz), dim3(64), 0,
                               stream, p);
            e = hipGetLastError();
        }
    }
    record_launch(LaunchRecord{"conv_window_lp", BM, BN, LPW_KA, WM, WN, 1, LOAD_KC, LOAD_IM2COL, 8, PAIR ? 2 : 1, NPU, p.ksplit, 0, 1});
    return e;
}

// npu = passes over the single-position units; a pair unit covers two of them.
template <int BM, int BN, int WM, int WN, int DT, bool LP_OUT>
hipError_t launch_units(ContractionParams& p, bool pair, int npu, int nz, const SplitSpace& space, hipStream_t stream) {
    if (pair) {
        if (npu <= 2) return launch_instance<BM, BN, WM, WN, DT, LP_OUT, true, 1>(p, nz, space, stream);
        if (npu <= 4) return launch_instance<BM, BN, WM, WN, DT, LP_OUT, true, 2>(p, nz, space, stream);
        if constexpr (WM * WN <= 4) {
            if (npu <= 8) return launch_instance<BM, BN, WM, WN, DT, LP_OUT, true, 4>(p, nz, space, stream);
        }
        return hipErrorInvalidValue;
    }
    if (npu <= 2) return launch_instance<BM, BN, WM, WN, DT, LP_OUT, false, 2>(p, nz, space, stream);
    if (npu <= 4) return launch_instance<BM, BN, WM, WN, DT, LP_OUT, false, 4>(p, nz, space, stream);
    if constexpr (WM * WN <= 4) {
        if (npu <= 8) return launch_instance<BM, BN, WM, WN, DT, LP_OUT, false, 8>(p, nz, space, stream);
    }
    return hipErrorInvalidValue;
}

template <int DT, bool LP_OUT>
hipError_t launch_config(ContractionParams& p, int cfg, bool pair, int npu, int nz, const SplitSpace& space, hipStream_t stream) {
    switch (cfg) {
        case 0: return launch_units<64, 64, 2, 2, DT, LP_OUT>(p, pair, npu, nz, space, stream);
        case 1: return launch_units<128, 128, 2, 4, DT, LP_OUT>(p, pair, npu, nz, space, stream);
        case 2: return launch_units<64, 128, 2, 2, DT, LP_OUT>(p, pair, npu, nz, space, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_lp_filter_taps(const void* W, void* packed, int64_t rows, int Cg, hipStream_t stream) {
    const int64_t chunks = rows * Cg * LPW_TAPS / 8;
    if (Cg % LPW_CB != 0 || (chunks + 255) / 256 > 0x7fffffffLL) return hipErrorInvalidValue;
    if (chunks == 0) return hipSuccess;
    hipLaunchKernelGGL(lp_filter_taps_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const uint16_t*>(W), static_cast<uint16_t*>(packed), chunks, Cg);
    return hipGetLastError();
}

bool launch_conv_window_lp(ContractionParams& p, int kH, int kW, int OH, int OW, int Cg, int nz, int in_type, int out_type,
                           bool filters_in_tap_order, const Workspace& ws, hipStream_t stream, hipError_t* status) {
    if (!(kH == 3 && kW == 3) || Cg % LPW_CB != 0) return false;
    // the rewritten filter bank lives in the workspace, unless the caller hands it over rewritten
    const int64_t filter_values = (int64_t)p.M * nz * Cg * LPW_TAPS;
    if (!filters_in_tap_order && (!ws.partial || filter_values * 2 > ws.partial_floats * 4)) return false;
    if ((reinterpret_cast<uintptr_t>(p.A) & 15u) != 0 && filters_in_tap_order) return false;
    // 32-bit byte offsets from a tile's first image: the input of the images one tile touches, and their output
    const int64_t P = (int64_t)OH * OW, tile_images = (256 + P - 1) / P + 1, span = (1LL << 31) - 64;
    if (tile_images * p.ic.image_stride * 2 >= span || (256 * P + tile_images * p.y_img) * 4 >= span || (int64_t)256 * p.K * 2 >= span)
        return false;
    Im2colGeom& g = p.ic;
    const int E = (kH - 1) * g.dH + 1;
    // pairs of columns: the patch starts at an even input column and has an even pitch
    const bool pair = g.W % 2 == 0 && (reinterpret_cast<uintptr_t>(p.B) & 3u) == 0;
    const int shift = pair ? (g.pL & 1) : 0;
    int PC = (OW - 1) * g.sW + (kW - 1) * g.dW + 1 + shift;
    if (pair) PC = (PC + 1) & ~1;
    int best = -1, best_plane = 0;
    double best_cost = 0.0;
    for (int c = 0; c < kNumConfigs; ++c) {
        const WindowLpConfig& k = kConfigs[c];
        if (OW > k.bn) continue;
        const int64_t plane = (int64_t)patch_rows(k.bn, OH, OW, g.sH, E) * PC;
        if (2 * plane > (int64_t)k.max_units * k.nt) continue;
        const double tiles = (double)((p.M + k.bm - 1) / k.bm) * (double)((p.N + k.bn - 1) / k.bn) * nz;
        double rounds = tiles / k.resident;
        if (rounds < 1.0) rounds = 1.0;
        // every pass over the patch units beyond the first adds loads and LDS stores to each K step
        const int64_t passes = (2 * plane + k.nt - 1) / k.nt;
        const double cost = rounds * k.weight * (1.0 + 0.25 * (double)(passes - 1));
        if (best < 0 || cost < best_cost) { best = c; best_cost = cost; best_plane = (int)plane; }
    }
    if (best < 0) return false;
    // Long channel walks over few tiles (ResNet-50's 3x3 layers on 7 x 7 planes at batch 32: 32 steps, 200 tiles of 64 x 64):
    // both square tiles run in one round and split their walk, and the 128 x 128 one, split four ways over a quarter of
    // the tiles, ends sooner (27.6 against 32.9 us with their finishing kernels).
    if (best == 0 && ws.partial && Cg / LPW_CB >= 32 && OW <= kConfigs[1].bn) {
        const WindowLpConfig& k = kConfigs[1];
        const int64_t plane = (int64_t)patch_rows(k.bn, OH, OW, g.sH, E) * PC;
        const int64_t tiles = (int64_t)((p.M + k.bm - 1) / k.bm) * ((p.N + k.bn - 1) / k.bn) * nz;
        if (2 * plane <= (int64_t)k.max_units * k.nt && tiles >= 32 && tiles * 4 <= k.resident) { best = 1; best_plane = (int)plane; }
    }
    g.OH = OH; g.Cg = Cg; g.E = E; g.IPR = (OH - 1) * g.sH + E; g.PC = PC; g.plane = best_plane;
    g.OHd = FastDiv::make((uint32_t)OH);
    g.PCd = FastDiv::make((uint32_t)(pair ? PC / 2 : PC));
    g.planed = FastDiv::make((uint32_t)(pair ? best_plane / 2 : best_plane));
    g.IPRd = FastDiv::make((uint32_t)g.IPR);

    SplitSpace space = {ws.partial, ws.partial ? ws.partial_floats : 0};
    if (!filters_in_tap_order) {
        const hipError_t e = launch_lp_filter_taps(p.A, ws.partial, (int64_t)p.M * nz, Cg, stream);
        if (e != hipSuccess) { *status = e; return true; }
        p.A = ws.partial;
        const int64_t used = (filter_values * 2 + 255) / 256 * 64;          // floats, a multiple of 256 bytes
        space.partial += used;
        space.floats -= used;
    }

    const int npu = (2 * best_plane + kConfigs[best].nt - 1) / kConfigs[best].nt;
    const bool lp_out = out_type != 0;
    if (in_type == LP_BF16) *status = lp_out ? launch_config<LP_BF16, true>(p, best, pair, npu, nz, space, stream) : launch_config<LP_BF16, false>(p, best, pair, npu, nz, space, stream);
    else *status = lp_out ? launch_config<LP_F16, true>(p, best, pair, npu, nz, space, stream) : launch_config<LP_F16, false>(p, best, pair, npu, nz, space, stream);
    return true;
}

}  // namespace onnxhip
