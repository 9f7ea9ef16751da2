// Convolution with an LDS-resident input patch, on the matrix cores.
//
// The generic implicit-GEMM path gathers every (k, pixel) element of the patch matrix from
// global memory: a KH x KW filter re-reads each input value KH*KW times and pays an address
// computation per element.  Here a workgroup loads, per step of 4 input channels, the
// rectangle of input rows and columns its BN output pixels touch (the "patch", zero padding
// included) into LDS once, and every filter tap reads it from there at lane base + a uniform
// offset.  Same ONNX Conv semantics (Section 4.1 of the paper lists convolution among the
// supported operators; Section 4.2's ResNet50 spends nearly all its arithmetic in them).
//
// Tiling is the same as in contraction.h (BM output channels x BN consecutive positions of
// the flattened (image, oh, ow) index), so the epilogue is shared.  The output rows a tile
// touches may belong to several images; patch rows are laid out image after image:
//   image a = 0 (the tile's first):  rows for oh = oh0 .. OH-1      start at patch row 0
//   image a >= 1:                    rows for oh = 0 .. OH-1        start at PS1 + (a-1)*IPR
// with PS1 = (OH-1-oh0)*sH + E, IPR = (OH-1)*sH + E, E = (KH-1)*dH + 1.  Output row oh of image a
// reads patch rows start(a) + (oh - first oh of a)*sH + kh*dH, columns ow*sW + kw*dW.
//
// K is walked 4 channels at a time.  One MFMA (32x32x2) consumes two k: lanes 0-31 supply
// channel 2c', lanes 32-63 channel 2c'+1, both at the same tap; A (filters, in LDS as
// [row][channel][taps padded to a multiple of 4], so that a lane fetches its channel's taps
// with 16-byte reads) and B (patch, [channel][patch row][patch col]) use the same dealing.
#pragma once
#include <type_traits>

#include "contraction.h"

namespace onnxhip {

constexpr int WIN_CB = 4;      // input channels per K step

// NPB = passes of NT threads that cover one step's patch (4 channels x plane values); the
// launcher picks the smallest instance that fits, so the main loop has no data-dependent
// branch: every load and LDS store below is unconditional (surplus ones are out-of-range
// buffer loads, which fetch nothing and return zero).
//
// Schedule of one K step (LDS buffer s holds step ks, register set s^1 holds step ks+1, whose
// loads were issued a whole step ago):
//   issue global loads of step ks+2 into register set s
//   pair 0's MFMAs (fragments read during the previous step), pair 1's LDS reads in between
//   store register set s^1 into LDS buffer s^1 in between the first half of pair 1's MFMAs
//   barrier; the second half, with the LDS reads of step ks+1's pair 0 in between
template <int BM, int BN, int WM, int WN, int KH, int KW, int NPB>
__global__ __launch_bounds__(64 * WM * WN) void conv_window_kernel(const ContractionParams cp) {
    constexpr int NT = 64 * WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int KHW = KH * KW;
    constexpr int KA = WIN_CB * KHW;            // filter values per row per step (contiguous in W)
    constexpr int CH = (KHW + 3) / 4 * 4;       // floats per (row, channel) in LDS: the taps, padded to 16 bytes
    constexpr int LDA = WIN_CB * CH + 4;        // row stride: 16-byte fragment reads of 8 neighbouring rows hit disjoint banks
    constexpr int NA4 = BM * KA / 4;            // 16-byte loads per A tile
    constexpr int PA = (NA4 + NT - 1) / NT;
    constexpr int NMFMA = KHW * TM * TN;        // MFMAs per channel pair
    constexpr int NFRAG = CH / 4 * TM + KHW * TN;   // LDS reads per channel pair
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "sub-tile of 32x32 blocks");

    __shared__ __attribute__((aligned(16))) float lds_a[2][BM * LDA + 4];   // + a slot that absorbs the stores of surplus threads
    __shared__ float lds_b[2][NPB * NT];

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

    // ---- geometry of this tile's patch
    uint32_t q_first, ow_first, img_first, oh0;
    g.OW.divmod((uint32_t)n0, q_first, ow_first);
    g.OHd.divmod(q_first, img_first, oh0);
    img_first = (uint32_t)scalar((int)img_first);
    oh0 = (uint32_t)scalar((int)oh0);
    const int PS1 = (g.OH - 1 - (int)oh0) * g.sH + g.E;
    const int n_images = cp.N / (int)cp.colP.d;      // images in the batch

    // ---- filter tile loader: thread -> (row, 16-byte chunk), fixed for the whole K walk
    const float* a_base = cp.A + a_off + (int64_t)m0 * cp.K;
    const __amdgpu_buffer_rsrc_t ra = tile_rsrc(a_base);
    uint32_t voff_a[PA];
    int dst_a[PA][4];                               // LDS position of each of a chunk's 4 values
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int e = t + p * NT;
        const int row = e / KHW, q = e % KHW;        // KA/4 == KHW chunks per row
        const bool ok = e < NA4 && m0 + row < cp.M;
        voff_a[p] = ok ? (uint32_t)(row * cp.K + q * 4) * 4u : OOB;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = q * 4 + j;                     // position in the row's KA = 4 channels x KHW taps
            dst_a[p][j] = e < NA4 ? row * LDA + (k / KHW) * CH + k % KHW : BM * LDA;
        }
    }
    // ---- patch loader: thread -> (channel, patch row, patch col), fixed for the whole K walk
    const float* b_base = cp.B + b_off + (int64_t)img_first * g.image_stride;
    const __amdgpu_buffer_rsrc_t rb = tile_rsrc(b_base);
    const int HW = g.H * g.W;
    uint32_t voff_b[NPB];
#pragma unroll
    for (int p = 0; p < NPB; ++p) {
        const uint32_t e = (uint32_t)(t + p * NT);
        uint32_t c, rem, pr, pc;
        g.planed.divmod(e, c, rem);
        g.PCd.divmod(rem, pr, pc);
        uint32_t a = 0, local = pr;
        if ((int)pr >= PS1) {
            g.IPRd.divmod(pr - (uint32_t)PS1, a, local);
            a += 1;
        }
        const int ih = (a == 0 ? (int)oh0 * g.sH : 0) - g.pT + (int)local;
        const int iw = (int)pc - g.pL;
        const bool ok = c < (uint32_t)WIN_CB && (int)(img_first + a) < n_images && (unsigned)ih < (unsigned)g.H &&
                        (unsigned)iw < (unsigned)g.W;
        voff_b[p] = ok ? (uint32_t)((int)a * g.image_stride + (int)c * HW + ih * g.W + iw) * 4u : OOB;
    }
    // ---- where this lane reads its operands for the MFMAs
    int rd_a[TM], rd_b[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) rd_a[i] = (wm * WTM + i * 32 + li) * LDA + h * CH;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int col = n0 + wn * WTN + j * 32 + li;
        if (col >= cp.N) col = n0;
        uint32_t q, ow, img, oh;
        g.OW.divmod((uint32_t)col, q, ow);
        g.OHd.divmod(q, img, oh);
        const int a = (int)(img - img_first);
        const int prow = a == 0 ? ((int)oh - (int)oh0) * g.sH : PS1 + (a - 1) * g.IPR + (int)oh * g.sH;
        rd_b[j] = prow * g.PC + (int)ow * g.sW + h * g.plane;
    }
    int tap_b[KHW];                                  // uniform patch offset of each tap
#pragma unroll
    for (int kh = 0; kh < KH; ++kh)
#pragma unroll
        for (int kw = 0; kw < KW; ++kw) tap_b[kh * KW + kw] = kh * g.dH * g.PC + kw * g.dW;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int ks0, ks1;
    split_range(g.Cg / WIN_CB, w.ksplit, w.split, ks0, ks1);
    ks0 = scalar(ks0); ks1 = scalar(ks1);

    floatx4 reg_a[2][PA];
    float reg_b[2][NPB];
    using Set0 = std::integral_constant<int, 0>;
    using Set1 = std::integral_constant<int, 1>;

    // Loads of step ks into register set S; a step past the end of the walk loads nothing.
    auto fetch = [&](int ks, auto S) {
        constexpr int s = decltype(S)::value;
        const uint32_t past = ks < ks1 ? 0u : OOB;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            reg_a[s][p] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(ra, (int)(voff_a[p] | past), ks * KA * 4, 0));
#pragma unroll
        for (int p = 0; p < NPB; ++p)
            reg_b[s][p] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, (int)(voff_b[p] | past), ks * WIN_CB * HW * 4, 0));
    };
    auto commit = [&](int buf, auto S) {
        constexpr int s = decltype(S)::value;
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            float* d = lds_a[buf];
            d[dst_a[p][0]] = reg_a[s][p].x; d[dst_a[p][1]] = reg_a[s][p].y;
            d[dst_a[p][2]] = reg_a[s][p].z; d[dst_a[p][3]] = reg_a[s][p].w;
        }
#pragma unroll
        for (int p = 0; p < NPB; ++p) lds_b[buf][t + p * NT] = reg_b[s][p];
    };
    float fa[2][CH][TM], fb[2][KHW][TN];
    auto frags = [&](int f, const float* sa, const float* sb, int cc) {
#pragma unroll
        for (int tap = 0; tap < KHW; ++tap) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (tap % 4 == 0) {                      // the lane's channel: CH / 4 reads of 16 bytes
                    const floatx4 v = *reinterpret_cast<const floatx4*>(sa + rd_a[i] + 2 * cc * CH + tap);
                    fa[f][tap][i] = v.x; fa[f][tap + 1][i] = v.y; fa[f][tap + 2][i] = v.z; fa[f][tap + 3][i] = v.w;
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[f][tap][j] = sb[rd_b[j] + 2 * cc * g.plane + tap_b[tap]];
        }
    };
    auto mfmas = [&](int f, int tap_lo, int tap_hi) {
#pragma unroll
        for (int tap = tap_lo; tap < tap_hi; ++tap)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[f][tap][i], fb[f][tap][j], acc[i][j], 0, 0, 0);
    };
    // On entry LDS buffer s holds step ks and pair 0's fragments (set 0) are already in registers.
    auto step = [&](int ks, auto S, auto SN) {
        constexpr int s = decltype(S)::value;
        constexpr int HALF = KHW / 2;
        fetch(ks + 2, S);
        static_assert(WIN_CB == 4, "two channel pairs per step");
        frags(1, lds_a[s], lds_b[s], 1);
        mfmas(0, 0, KHW);
#pragma unroll
        for (int q = 0; q < NMFMA; ++q) {            // one MFMA, then its share of pair 1's LDS reads
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, (NFRAG + NMFMA - 1) / NMFMA, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        commit(s ^ 1, SN);                           // past the end this stores zeros nobody reads
        mfmas(1, 0, HALF);
        __syncthreads();
        frags(0, lds_a[s ^ 1], lds_b[s ^ 1], 0);     // next step's pair 0, behind the rest of pair 1
        mfmas(1, HALF, KHW);
        constexpr int NREST = (KHW - HALF) * TM * TN;
#pragma unroll
        for (int q = 0; q < NREST; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, (NFRAG + NREST - 1) / NREST, 0);
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
    finish_tile<TM, TN, WTM, WTN, NT>(acc, w, wm, wn, li, h, cp);
}

}  // namespace onnxhip
