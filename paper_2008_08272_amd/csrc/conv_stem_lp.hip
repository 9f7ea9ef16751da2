// The stem of ResNet50 (Section 4.2) on 16-bit tensors: a 7x7 convolution at stride 2 with pads of 3
// on 3 input channels into 64 feature maps.  Three channels give the 16-channel K step of the LDS-patch
// kernel for 3x3 windows (conv_window_lp.hip) nothing to hold on to, and the general kernel gathers
// every input element on its own.  Here K is laid out as (channel, window row, 8 window columns):
// the 7 taps of a window row plus one zero tap are the 8 consecutive k that one lane hands to
// v_mfma_f32_32x32x16_{f16,bf16}, and for an output position they are 8 consecutive input values
// of one row, which a lane reads from an LDS copy of the input patch in one go.  21 window rows
// (3 channels x 7) make 10.5 MFMA K steps; the filter bank, padded the same way, sits in LDS for
// the life of a persistent workgroup.
//
// A workgroup computes R whole output rows of one image for all 64 filters: R * OW output positions,
// 32 consecutive ones per wavefront, so that for one filter a wavefront stores 32 neighbouring
// elements (rows of an output plane are contiguous, so positions that wrap into the next row still
// are).  The patch holds input rows 2 * oh0 - 3 .. 2 * (oh0 + R - 1) + 3 with three zero columns in
// front: the window of output column ow then starts at patch column 2 * ow, an even one, and the
// lane's 16 bytes are four 4-byte aligned LDS words.
#include "gemm_lp.h"
#include "internal.h"

namespace onnxhip {

namespace {

constexpr int STEM_M = 64;                      // filters
constexpr int STEM_C = 3, STEM_K = 7;           // input channels, window
constexpr int STEM_ROWS = STEM_C * STEM_K;      // 21 window rows of 8 k each
constexpr int STEM_STEPS = (STEM_ROWS + 1) / 2; // 11 MFMA K steps of 16
constexpr int STEM_A_PITCH = STEM_STEPS * 16 + 8;   // 184 values per filter: 16-byte fragment reads of 16 neighbouring filters hit disjoint banks
constexpr int STEM_NT = 512;                    // 8 wavefronts: up to 256 output positions per tile
constexpr int STEM_PATCH_MAX = 12800;           // 16-bit values of LDS for the patch (all channels)
constexpr int STEM_STRIP_PITCH = 40;             // 16-bit values per filter row of a wavefront's epilogue strip (32 + 8: rows stay 16-byte aligned)
constexpr int STEM_MAX_CHUNKS = 5;              // rows of up to 320 patch columns: 157 output columns
constexpr int STEM_SLOTS = 16;                  // patch values a thread loads per tile, at most

struct StemParams {
    const uint16_t* X;
    const uint16_t* W;
    const float* bias;
    void* Y;
    int N, H, Wd, OH, OW;
    int R;                  // output rows per tile
    int PR, PW;             // patch rows (2R + 5) and columns (2 OW + 6) per channel
    int bands;              // tiles per image
    int rows_per_wave, chunks;          // patch rows per wavefront, 64-column pieces per row
    int relu;
    int wide_rows;          // 16-bit Y: tiles, planes and the base address allow 16-byte stores of 8 positions
    FastDiv bandsd, PWd, PRd, OWd;
};

// CHUNKS: 64-column pieces of a patch row, ceil(PW / 64).
template <int DT, bool LP_OUT, int CHUNKS>
__global__ __launch_bounds__(STEM_NT) __attribute__((amdgpu_waves_per_eu(4, 4))) void conv_stem_lp_kernel(const StemParams sp) {
    __shared__ __attribute__((aligned(16))) uint16_t lds_a[STEM_M * STEM_A_PITCH];
    __shared__ __attribute__((aligned(16))) uint16_t patch[STEM_PATCH_MAX];
    __shared__ float lds_bias[STEM_M];
    __shared__ __attribute__((aligned(16))) uint16_t strips[LP_OUT ? (STEM_NT / 64) * 32 * STEM_STRIP_PITCH : 8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, h = lane >> 5;

    // the filter bank as [filter][window row q = c * 7 + kh][8]: taps 0..6 and a zero; rows 21.. are zero.  All loads
    // of a thread's rows are requested before the first LDS store (one 16-byte store per row).
    {
        constexpr int ROWS = STEM_M * 2 * STEM_STEPS, PER = (ROWS + STEM_NT - 1) / STEM_NT;
        uint32_t v[PER][8];
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            const int e = tid + it * STEM_NT;
            const int m = e / (2 * STEM_STEPS), q = e % (2 * STEM_STEPS);
            const bool real = e < ROWS && q < STEM_ROWS;
#pragma unroll
            for (int t = 0; t < 8; ++t) v[it][t] = (real && t < STEM_K) ? sp.W[(m * STEM_ROWS + q) * STEM_K + t] : 0u;
        }
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            const int e = tid + it * STEM_NT;
            if (e < ROWS) {
                const uintx4 w = {v[it][0] | (v[it][1] << 16), v[it][2] | (v[it][3] << 16), v[it][4] | (v[it][5] << 16), v[it][6] | (v[it][7] << 16)};
                *reinterpret_cast<uintx4*>(lds_a + (e / (2 * STEM_STEPS)) * STEM_A_PITCH + (e % (2 * STEM_STEPS)) * 8) = w;
            }
        }
        if (tid < STEM_M) lds_bias[tid] = sp.bias ? sp.bias[tid] : 0.f;
    }

    // this lane's output position within a tile and where its windows start in the patch (the same for every tile)
    const int px = wave * 32 + li;
    const bool px_in_tile = px < sp.R * sp.OW;
    uint32_t prow = 0, pcol = 0;
    sp.OWd.divmod((uint32_t)(px_in_tile ? px : 0), prow, pcol);
    const int window0 = (int)prow * 2 * sp.PW + 2 * (int)pcol;         // patch element of (window row 0, tap 0) in channel 0
    // Patch rows (channel, patch row) are dealt to the wavefronts in runs of `rows_per_wave` (at most ROWS); a lane takes
    // the columns lane, lane + 64, ... of each.  What a row needs beyond the lane's column is uniform and advances from
    // row to row without a division.  The values of the next tile are requested before this tile's MFMAs and parked in
    // registers, two 16-bit values per register.
    constexpr int ROWS = STEM_SLOTS / CHUNKS;
    const int rows_total = STEM_C * sp.PR;
    const int first_row = scalar(wave * sp.rows_per_wave);
    uint32_t first_c, first_pr;
    sp.PRd.divmod((uint32_t)first_row, first_c, first_pr);
    typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
    u16x2 parked[(ROWS * CHUNKS + 1) / 2];
    auto fetch = [&](int tile) {
        uint32_t n, band;
        sp.bandsd.divmod((uint32_t)tile, n, band);
        const int ih_first = 2 * (int)band * sp.R - 3;
        // loads through a buffer resource on the image: a value outside it (or of a row this wavefront does not own) is
        // an out-of-range offset, which reads 0 without a branch, so that all of a tile's loads are in flight together
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(sp.X) + (int64_t)scalar((int)n) * STEM_C * sp.H * sp.Wd, 0, (int)OOB, RSRC_FLAGS);
        int c = (int)first_c, pr = (int)first_pr;
#pragma unroll
        for (int ri = 0; ri < ROWS; ++ri) {
            const int ih = ih_first + pr;
            const bool row_ok = ri < sp.rows_per_wave && first_row + ri < rows_total && ih >= 0 && ih < sp.H;      // uniform
            const int row_first = (c * sp.H + ih) * sp.Wd;                  // element of (c, ih, 0) in the image
#pragma unroll
            for (int k = 0; k < CHUNKS; ++k) {
                const int iw = lane + 64 * k - 3;
                const uint32_t off = (row_ok && iw >= 0 && iw < sp.Wd) ? (uint32_t)(row_first + iw) * 2u : OOB;
                const int i = ri * CHUNKS + k;
                parked[i / 2][i & 1] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, (int)off, 0, 0);
            }
            if (++pr == sp.PR) { pr = 0; ++c; }
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int ri = 0; ri < ROWS; ++ri) {
            const int row = first_row + ri;
            const bool row_ok = ri < sp.rows_per_wave && row < rows_total;
#pragma unroll
            for (int k = 0; k < CHUNKS; ++k) {
                const int j = lane + 64 * k, i = ri * CHUNKS + k;
                if (row_ok && j < sp.PW) patch[row * sp.PW + j] = parked[i / 2][i & 1];
            }
        }
    };

    const int64_t plane = (int64_t)sp.OH * sp.OW;
    const int tiles = sp.N * sp.bands;
    if ((int)blockIdx.x < tiles) fetch(blockIdx.x);
    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        uint32_t n, band;
        sp.bandsd.divmod((uint32_t)tile, n, band);
        const int oh0 = (int)band * sp.R;
        __syncthreads();                          // the filters are in place; nobody still reads the previous patch
        commit();
        __syncthreads();
        if (tile + (int)gridDim.x < tiles) fetch(tile + gridDim.x);

        if (wave * 32 < sp.R * sp.OW) {           // wavefronts past the tile's positions have nothing to do
            floatx16 acc[2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
#pragma unroll
            for (int s = 0; s < STEM_STEPS; ++s) {
                // B: 8 consecutive patch values from an even column (4-byte aligned words); the eighth is not a tap
                // the window row of this lane's half of the step: q = 2 s + h, in channel q / 7
                const int q0 = 2 * s, q1 = q0 + 1;
                const int off0 = ((q0 / STEM_K) * sp.PR + (q0 % STEM_K)) * sp.PW;
                const int off1 = q1 < STEM_ROWS ? ((q1 / STEM_K) * sp.PR + (q1 % STEM_K)) * sp.PW : -1;
                const int row_off = h ? off1 : off0;
                uintx4 fb = {0u, 0u, 0u, 0u};
                if (row_off >= 0) {
                    const uint32_t* w4 = reinterpret_cast<const uint32_t*>(patch + row_off + window0);
                    fb[0] = w4[0]; fb[1] = w4[1]; fb[2] = w4[2]; fb[3] = w4[3] & 0xffffu;
                }
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const floatx4 fa = *reinterpret_cast<const floatx4*>(lds_a + (32 * b + li) * STEM_A_PITCH + s * 16 + h * 8);
                    acc[b] = mfma16<DT>(fa, __builtin_bit_cast(floatx4, fb), acc[b]);
                }
            }
            // positions of a tile are consecutive elements of an output plane
            const int64_t lin0 = (int64_t)oh0 * sp.OW + wave * 32;           // this wavefront's first position in the image
            if (LP_OUT && sp.wide_rows) {
                // 16-bit results in rows: a block of 32 filters x 32 positions goes through this wavefront's own strip of
                // LDS (no barrier: the wavefront reads back what it wrote), after which a lane holds 8 neighbouring
                // positions of one filter: one 16-byte store instead of eight 2-byte ones.  Tiles and planes are
                // multiples of 8 positions long here, so a group of 8 exists as a whole or not at all.
                uint16_t* strip = strips + wave * (32 * STEM_STRIP_PITCH);
                const int chunk = lane & 3, srow = lane >> 2;
                const bool chunk_ok = wave * 32 + chunk * 8 < sp.R * sp.OW && lin0 + chunk * 8 < plane;
#pragma unroll
                for (int b = 0; b < 2; ++b) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int fm = 8 * (r / 4) + 4 * h + (r % 4);
                        float v = acc[b][r] + lds_bias[32 * b + fm];
                        if (sp.relu) v = fmaxf(v, 0.f);
                        strip[fm * STEM_STRIP_PITCH + li] = to_lp<DT>(v);
                    }
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int pass = 0; pass < 2; ++pass) {
                        const int fm = srow + 16 * pass;
                        const uintx4 w = *reinterpret_cast<const uintx4*>(strip + fm * STEM_STRIP_PITCH + chunk * 8);
                        if (chunk_ok)
                            *reinterpret_cast<uintx4*>(static_cast<uint16_t*>(sp.Y) + ((int64_t)n * STEM_M + 32 * b + fm) * plane + lin0 + chunk * 8) = w;
                    }
                    asm volatile("" ::: "memory");
                }
            } else if (px_in_tile && lin0 + li < plane) {
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        // register r of block b is filter 32 b + 8 (r / 4) + 4 h + r % 4
                        const int m = 32 * b + 8 * (r / 4) + 4 * h + (r % 4);
                        float v = acc[b][r] + lds_bias[m];
                        if (sp.relu) v = fmaxf(v, 0.f);
                        const int64_t o = ((int64_t)n * STEM_M + m) * plane + lin0 + li;
                        if constexpr (LP_OUT) static_cast<uint16_t*>(sp.Y)[o] = to_lp<DT>(v);
                        else static_cast<float*>(sp.Y)[o] = v;
                    }
            }
        }
    }
}

}  // namespace

bool launch_conv_stem_lp(const void* X, const void* W, const float* B, void* Y, const WindowGeom& g, int M, int Cg, int group,
                         bool has_residual, int relu, int in_type, int out_type, hipStream_t stream, hipError_t* status) {
    if (group != 1 || has_residual || M != STEM_M || Cg != STEM_C || g.C != STEM_C || g.kH != STEM_K || g.kW != STEM_K || g.sH != 2 ||
        g.sW != 2 || g.dH != 1 || g.dW != 1 || g.pT != 3 || g.pL != 3 || g.pB != 3 || g.pR != 3)
        return false;
    if (g.OW < 1 || g.OW > 256 || g.OH < 1 || (int64_t)g.N * g.OH > 0x7fffffffLL) return false;
    if ((int64_t)STEM_C * g.H * g.W * 2 >= 0x7fffffffLL) return false;          // 32-bit byte offsets inside an image
    StemParams sp;
    sp.X = static_cast<const uint16_t*>(X);
    sp.W = static_cast<const uint16_t*>(W);
    sp.bias = B;
    sp.Y = Y;
    sp.N = g.N; sp.H = g.H; sp.Wd = g.W; sp.OH = g.OH; sp.OW = g.OW;
    sp.R = 256 / g.OW < g.OH ? 256 / g.OW : g.OH;
    sp.PW = 2 * g.OW + 6;                          // windows end at patch column 2 (OW - 1) + 7
    sp.chunks = (sp.PW + 63) / 64;
    if (sp.chunks > STEM_MAX_CHUNKS) return false;
    // fewer rows per tile until the patch fits the LDS array and a thread's share of it its registers
    auto shape = [&](int R) {
        sp.R = R;
        sp.PR = 2 * R + 5;
        sp.rows_per_wave = (STEM_C * sp.PR + STEM_NT / 64 - 1) / (STEM_NT / 64);
        return (int64_t)STEM_C * sp.PR * sp.PW <= STEM_PATCH_MAX && sp.rows_per_wave <= STEM_SLOTS / sp.chunks;
    };
    int R = sp.R;
    while (R > 1 && !shape(R)) --R;
    if (!shape(R)) return false;
    sp.bands = (g.OH + sp.R - 1) / sp.R;
    sp.relu = relu;
    sp.wide_rows = ((int64_t)g.OH * g.OW) % 8 == 0 && (sp.R * g.OW) % 8 == 0 && aligned16(Y);
    sp.bandsd = FastDiv::make((uint32_t)sp.bands);
    sp.PWd = FastDiv::make((uint32_t)sp.PW);
    sp.PRd = FastDiv::make((uint32_t)sp.PR);
    sp.OWd = FastDiv::make((uint32_t)g.OW);
    const int64_t tiles = (int64_t)g.N * sp.bands;
    if (tiles > 0x7fffffffLL) return false;
    // persistent workgroups: the 23 KB filter bank is loaded once per workgroup; two workgroups of 8 wavefronts are
    // resident per CU
    const unsigned grid = (unsigned)(tiles < 2 * 256 ? tiles : 2 * 256);
    const bool lp_out = out_type != 0;
    const dim3 grid_dim(grid), block(STEM_NT);
#define ONNXHIP_STEM_CASE(CH)                                                                                                   \
    case CH:                                                                                                                    \
        if (in_type == LP_F16) {                                                                                                \
            if (lp_out) hipLaunchKernelGGL((conv_stem_lp_kernel<LP_F16, true, CH>), grid_dim, block, 0, stream, sp);            \
            else hipLaunchKernelGGL((conv_stem_lp_kernel<LP_F16, false, CH>), grid_dim, block, 0, stream, sp);                  \
        } else {                                                                                                                \
            if (lp_out) hipLaunchKernelGGL((conv_stem_lp_kernel<LP_BF16, true, CH>), grid_dim, block, 0, stream, sp);           \
            else hipLaunchKernelGGL((conv_stem_lp_kernel<LP_BF16, false, CH>), grid_dim, block, 0, stream, sp);                 \
        }                                                                                                                       \
        break;
    switch (sp.chunks) {
        ONNXHIP_STEM_CASE(1)
        ONNXHIP_STEM_CASE(2)
        ONNXHIP_STEM_CASE(3)
        ONNXHIP_STEM_CASE(4)
        ONNXHIP_STEM_CASE(5)
        default: return false;
    }
#undef ONNXHIP_STEM_CASE
    *status = hipGetLastError();
    record_launch(LaunchRecord{"conv_stem_lp", STEM_M, 256, 16, 1, 8, 1, LOAD_KC, LOAD_IM2COL, 1, sp.chunks, in_type + (lp_out ? 2 : 0), 1, 0, 1});
    return true;
}

}  // namespace onnxhip
