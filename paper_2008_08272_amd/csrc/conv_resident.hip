// Convolution with the filters resident in registers, on the matrix cores: for layers with few
// input channels and a large window, first of all ResNet50's 7x7 stride-2 stem (Section 4.2 of
// the paper: 3 -> 64 channels on 224 x 224 images).  Same ONNX Conv semantics as the other paths.
//
// Such a layer has a short reduction (K = Cg*kH*kW = 147 for the stem) and a huge number of
// output positions, so the generic implicit-GEMM path spends its time gathering patch elements
// (every input value is fetched kH*kW/(sH*sW) = 12 times, each with its own address) and
// re-staging the same small filter matrix for every tile.  Here
//   * a workgroup of 8 wavefronts is persistent: it loads its 64 filters once, straight into
//     registers in the layout the MFMA wants (lane = filter row, one register per k pair; a
//     wavefront holds 32 of the 64 rows), and then walks over output tiles;
//   * a tile is 8 x 16 output positions of one image (a wavefront owns 32 filters x 2 rows x 16
//     columns: one 32x32 accumulator); the rectangle of input the tile touches, zero padding
//     included, is staged in LDS once per tile (two buffers: the loads of the next tile are
//     issued before the MFMAs of the current one) and every tap reads it at lane base +
//     compile-time offset: no address arithmetic in the inner loop, one 4-byte LDS read per two
//     MFMAs, no filter traffic at all.
// One MFMA (32x32x2) consumes two k.  Lanes 0-31 supply the first, lanes 32-63 the second; the
// two k of a pair are neighbours along kw, or (odd kW) along kh in the last column, or (odd kH
// too) along c at the last tap, so that the second differs from the first by one constant LDS
// offset per kind of pair, which a per-lane base register absorbs.
#include <type_traits>

#include "internal.h"

namespace onnxhip {

struct ResidentParams {
    const float* X;
    const float* W;
    const float* bias;       // NULL or [M]
    const float* residual;   // NULL or laid out like Y
    float* Y;
    int N, C, H, Wd, M, OH, OW, pT, pL;
    int tiles_x, tiles_y;    // tiles per image along ow and oh
    int total_tiles;         // N * tiles_y * tiles_x
    int relu;
};

namespace {

template <int KH, int KW, int CG, int SH, int SW>
struct ResidentShape {
    static constexpr int K = CG * KH * KW;
    static constexpr int RH = 2, RW = 16;              // a wavefront's 32 positions
    static constexpr int NWAVE = 4;                    // wavefronts along the positions (times 2 along the filters)
    static constexpr int NT = 64 * NWAVE * 2;
    static constexpr int TH = NWAVE * RH, TW = RW;     // workgroup tile in output positions
    static constexpr int PR = (TH - 1) * SH + KH;      // patch rows
    static constexpr int PCOLS = (TW - 1) * SW + KW;   // patch columns
    // Row pitch: the second position row of a wavefront sits SH*PITCH floats after the first;
    // making that 32 mod 64 puts its lanes on the banks the first row leaves free (the lanes of
    // a row are SW apart; with SW = 2 the two k of a pair take the even and the odd banks).
    static constexpr int pitch() {
        for (int p = PCOLS; p < PCOLS + 64; ++p)
            if ((SH * p) % 64 == 32) return p;
        return PCOLS | 1;
    }
    static constexpr int PITCH = pitch();
    static constexpr int PLANE = PR * PITCH;
    static constexpr int PATCH = CG * PLANE;           // floats per LDS buffer
    static constexpr int ELEMS = CG * PR * PCOLS;      // values actually loaded per tile
    static constexpr int NL = (ELEMS + NT - 1) / NT;
    // k pairs: first k of the pair and which neighbour the second one is
    enum { ALONG_KW = 0, ALONG_KH = 1, ALONG_C = 2, ALONE = 3 };
    static constexpr int pairs_per_row = KW / 2;
    static constexpr int NP = CG * KH * pairs_per_row + (KW % 2 ? CG * (KH / 2) + (KH % 2 ? (CG + 1) / 2 : 0) : 0);
    struct Table {
        int k0[NP];
        int kind[NP];
    };
    static constexpr Table table() {
        Table t = {};
        int n = 0;
        for (int c = 0; c < CG; ++c)
            for (int kh = 0; kh < KH; ++kh)
                for (int kw = 0; kw + 1 < KW; kw += 2) { t.k0[n] = (c * KH + kh) * KW + kw; t.kind[n++] = ALONG_KW; }
        if (KW % 2) {
            for (int c = 0; c < CG; ++c)
                for (int kh = 0; kh + 1 < KH; kh += 2) { t.k0[n] = (c * KH + kh) * KW + KW - 1; t.kind[n++] = ALONG_KH; }
            if (KH % 2) {
                for (int c = 0; c + 1 < CG; c += 2) { t.k0[n] = (c * KH + KH - 1) * KW + KW - 1; t.kind[n++] = ALONG_C; }
                if (CG % 2) { t.k0[n] = ((CG - 1) * KH + KH - 1) * KW + KW - 1; t.kind[n++] = ALONE; }
            }
        }
        return t;
    }
    // distance in k between the two members of a pair of each kind, and the same in LDS floats
    static constexpr int kdelta(int kind) { return kind == ALONG_KW ? 1 : kind == ALONG_KH ? KW : kind == ALONG_C ? KH * KW : 0; }
    static constexpr int ldelta(int kind) { return kind == ALONG_KW ? 1 : kind == ALONG_KH ? PITCH : kind == ALONG_C ? PLANE : 0; }
    // LDS offset of tap k relative to a position's window origin
    static constexpr int loff(int k) { return (k / (KH * KW)) * PLANE + ((k / KW) % KH) * PITCH + k % KW; }
};

template <int KH, int KW, int CG, int SH, int SW>
__global__ __launch_bounds__(512, 2) void conv_resident_kernel(const ResidentParams cp) {
    using S = ResidentShape<KH, KW, CG, SH, SW>;
    constexpr int NP = S::NP, NL = S::NL, NT = S::NT;
    constexpr auto T = S::table();

    __shared__ float lds[2][S::PATCH + 4];              // + a slot that stays zero (see bb below)

    const int t = threadIdx.x;
    const int lane = t & 63, wave_all = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave_all / S::NWAVE, wave = wave_all % S::NWAVE;      // filter half, position strip
    const int li = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * 64 + 32 * wm;

    // ---- filters: a[p] = W[m0 + li][k0(p) + h * kdelta(p)], zero where that does not exist
    float a[NP];
    {
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(cp.W), 0, cp.M * S::K * 4, RSRC_FLAGS);
        const int row = m0 + li;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const bool ok = row < cp.M && !(T.kind[p] == S::ALONE && h == 1);
            const int k = T.k0[p] + h * S::kdelta(T.kind[p]);
            a[p] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rw, ok ? (row * S::K + k) * 4 : (int)OOB, 0, 0));
        }
    }
    // ---- where this lane's position reads the patch: one base per kind of pair
    const int pos_r = wave * S::RH + li / S::RW, pos_c = li % S::RW;      // position within the tile
    const int base = pos_r * SH * S::PITCH + pos_c * SW;
    // The k left without a partner is multiplied, in lanes 32-63, by a zero filter value; those
    // lanes read the slot that holds 0 rather than patch data, so that an infinity or NaN in
    // the input is not turned into 0 * inf for positions it does not belong to.
    constexpr int alone_off = T.kind[NP - 1] == S::ALONE ? S::loff(T.k0[NP - 1]) : 0;
    const int bb[4] = {base + h * S::ldelta(S::ALONG_KW), base + h * S::ldelta(S::ALONG_KH), base + h * S::ldelta(S::ALONG_C),
                       h ? S::PATCH - alone_off : base};
    if (t < 2) lds[t][S::PATCH] = 0.f;

    const int HW = cp.H * cp.Wd, P = cp.OH * cp.OW;
    const int per_image = cp.tiles_x * cp.tiles_y;
    float stage[NL];

    // Global loads of tile `tile`'s patch into the staging registers.
    auto fetch = [&](int tile) {
        const int n = tile / per_image, rem = tile - n * per_image;
        const int ty = rem / cp.tiles_x, tx = rem - ty * cp.tiles_x;
        const int ih0 = ty * S::TH * SH - cp.pT, iw0 = tx * S::TW * SW - cp.pL;
        const __amdgpu_buffer_rsrc_t rx = tile_rsrc(cp.X + (int64_t)n * cp.C * HW);
#pragma unroll
        for (int q = 0; q < NL; ++q) {
            const int e = t + q * NT;
            const int c = e / (S::PR * S::PCOLS), r2 = e % (S::PR * S::PCOLS);
            const int pr = r2 / S::PCOLS, pc = r2 % S::PCOLS;
            const int ih = ih0 + pr, iw = iw0 + pc;
            const bool ok = e < S::ELEMS && (unsigned)ih < (unsigned)cp.H && (unsigned)iw < (unsigned)cp.Wd;
            stage[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rx, ok ? (c * HW + ih * cp.Wd + iw) * 4 : (int)OOB, 0, 0));
        }
    };
    auto commit = [&](float* buf) {
#pragma unroll
        for (int q = 0; q < NL; ++q) {
            const int e = t + q * NT;
            const int c = e / (S::PR * S::PCOLS), r2 = e % (S::PR * S::PCOLS);
            const int pr = r2 / S::PCOLS, pc = r2 % S::PCOLS;
            if (e < S::ELEMS) buf[c * S::PLANE + pr * S::PITCH + pc] = stage[q];
        }
    };

    // the bias of the 16 filter rows this lane's accumulator registers hold: the same for every tile
    float bias_r[16];
    {
        const __amdgpu_buffer_rsrc_t rbias = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(cp.bias ? cp.bias : cp.W), 0, cp.bias ? cp.M * 4 : 0, RSRC_FLAGS);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            bias_r[r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rbias, (m0 + 8 * (r / 4) + 4 * h + r % 4) * 4, 0, 0));
    }
    const bool has_res = cp.residual != nullptr;
    const bool relu = cp.relu != 0;

    // Epilogue of one tile: bias, residual, Relu, store.
    auto epilogue = [&](int tile, const floatx16& acc) {
        const int n = tile / per_image, rem = tile - n * per_image;
        const int ty = rem / cp.tiles_x, tx = rem - ty * cp.tiles_x;
        const int oh = ty * S::TH + pos_r, ow = tx * S::TW + pos_c;
        const bool pos_ok = oh < cp.OH && ow < cp.OW;
        const int64_t img = (int64_t)n * cp.M * P;
        const __amdgpu_buffer_rsrc_t ry = tile_rsrc(cp.Y + img);
        const __amdgpu_buffer_rsrc_t rr = tile_rsrc(has_res ? cp.residual + img : cp.Y + img);
        const int pix = oh * cp.OW + ow;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + 8 * (r / 4) + 4 * h + r % 4;   // accumulator register r holds this row
            const int off = (pos_ok && m < cp.M) ? (m * P + pix) * 4 : (int)OOB;
            float v = acc[r] + bias_r[r];
            if (has_res) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, off, 0, 0));
            if (relu) v = fmaxf(v, 0.f);
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), ry, off, 0, 0);
        }
    };

    int tile = blockIdx.x;
    if (tile >= cp.total_tiles) return;                 // uniform per workgroup
    fetch(tile);
    commit(lds[0]);
    __syncthreads();
    int buf = 0;
    while (true) {
        const int next = tile + (int)gridDim.x;
        const bool more = next < cp.total_tiles;
        if (more) fetch(next);

        // ---- the MFMAs of this tile: B fragments read a few pairs ahead
        floatx16 acc, acc_odd;          // even and odd pairs accumulate apart: two independent MFMA chains
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[r] = 0.f; acc_odd[r] = 0.f; }
        constexpr int AHEAD = 4, RING = 8;
        float fb[RING];
        const float* src = lds[buf];
#pragma unroll
        for (int p = 0; p < AHEAD && p < NP; ++p) fb[p % RING] = src[bb[T.kind[p]] + S::loff(T.k0[p])];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (p + AHEAD < NP) fb[(p + AHEAD) % RING] = src[bb[T.kind[p + AHEAD]] + S::loff(T.k0[p + AHEAD])];
            if (p % 2 == 0) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[p], fb[p % RING], acc, 0, 0, 0);
            else acc_odd = __builtin_amdgcn_mfma_f32_32x32x2f32(a[p], fb[p % RING], acc_odd, 0, 0, 0);
            // keep the read AHEAD pairs in front of its MFMA: left alone, the scheduler sinks every
            // read to just before its use and each MFMA then waits out a whole LDS round trip
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += acc_odd[r];

        if (more) commit(lds[buf ^ 1]);
        __syncthreads();
        epilogue(tile, acc);
        if (!more) break;
        tile = next;
        buf ^= 1;
    }
}

template <int KH, int KW, int CG, int SH, int SW>
hipError_t launch_resident(ResidentParams& p, hipStream_t stream) {
    using S = ResidentShape<KH, KW, CG, SH, SW>;
    p.tiles_x = (p.OW + S::TW - 1) / S::TW;
    p.tiles_y = (p.OH + S::TH - 1) / S::TH;
    const int64_t total = (int64_t)p.N * p.tiles_x * p.tiles_y;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    const int mblocks = (p.M + 63) / 64;
    // one workgroup (8 wavefronts, two per SIMD) per CU stays resident; spread them over the filter blocks
    int per_block = (256 + mblocks - 1) / mblocks;
    if (per_block > p.total_tiles) per_block = p.total_tiles;
    hipLaunchKernelGGL((conv_resident_kernel<KH, KW, CG, SH, SW>), dim3((unsigned)per_block, (unsigned)mblocks, 1), dim3(S::NT), 0,
                       stream, p);
    record_launch(LaunchRecord{"conv_resident", 64, S::TH * S::TW, S::K, 2, 4, 1, LOAD_KC, LOAD_IM2COL, 1, 1, S::NL, 1, 0, 1});
    return hipGetLastError();
}

}  // namespace

bool launch_conv_resident(const float* X, const float* W, const float* B, const float* residual, float* Y,
                          const WindowGeom& g, int M, int Cg, int relu, hipStream_t stream, hipError_t* status) {
    const bool stem = g.kH == 7 && g.kW == 7 && Cg == 3 && g.C == 3 && g.sH == 2 && g.sW == 2 && g.dH == 1 && g.dW == 1;
    if (!stem) return false;
    // Every workgroup first loads its 64 filters into registers; that only pays once a workgroup has a few tiles
    // to run them over.  With fewer than two tiles per CU (batch 1 to 4 at 224x224: 12 us against 17.5 us at
    // batch 1, level at batch 4) the gathering contraction kernel is the faster one.
    using Stem = ResidentShape<7, 7, 3, 2, 2>;
    const int64_t stem_tiles = (int64_t)g.N * ((g.OW + Stem::TW - 1) / Stem::TW) * ((g.OH + Stem::TH - 1) / Stem::TH);
    if (stem_tiles * ((M + 63) / 64) < 2 * 256) return false;
    // 32-bit byte offsets inside one image of X and of Y, and inside W
    if ((int64_t)g.C * g.H * g.W * 4 >= (1LL << 31) || (int64_t)(M + 64) * g.OH * g.OW * 4 >= (1LL << 31) ||
        (int64_t)(M + 64) * Cg * g.kH * g.kW * 4 >= (1LL << 31))
        return false;
    ResidentParams p;
    p.X = X; p.W = W; p.bias = B; p.residual = residual; p.Y = Y;
    p.N = g.N; p.C = g.C; p.H = g.H; p.Wd = g.W; p.M = M; p.OH = g.OH; p.OW = g.OW; p.pT = g.pT; p.pL = g.pL;
    p.relu = relu;
    *status = launch_resident<7, 7, 3, 2, 2>(p, stream);
    return true;
}

}  // namespace onnxhip
