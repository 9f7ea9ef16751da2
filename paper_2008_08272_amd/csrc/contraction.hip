// Instances of the matrix-core contraction kernel and their launcher.
#include "internal.h"

namespace onnxhip {

template <int BM, int BN, int BK, int WM, int WN, int KS, int AK, int BKIND, int AVEC, int BVEC>
static hipError_t launch_one(ContractionParams& p, int nz, const Workspace& ws, hipStream_t stream) {
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    p.nz = nz;
    // The 16-wavefront tiles are chosen only where their tile count fills whole rounds of the 256 CUs
    // (pick_tile), which is exactly where neither a K split nor a tail split pays: they never split.
    constexpr bool kMaySplit = BM * BN < 128 * 128;
    p.ksplit = kMaySplit ? pick_split((int64_t)p.tiles_m * p.tiles_n * nz, (p.K + BK - 1) / BK, (int64_t)BM * BN, 6.0, ws) : 1;
    p.ws_partial = ws.partial;
    const hipError_t e = launch_with_split<BM, BN, WM, WN, KS, kMaySplit>(
        contraction_kernel<BM, BN, BK, WM, WN, KS, AK, BKIND, AVEC, BVEC>, p, nz, (p.K + BK - 1) / BK, ws.partial_floats, stream);
    const int ntiles = p.tiles_m * p.tiles_n;
    record_launch(LaunchRecord{"contraction", BM, BN, BK, WM, WN, KS, AK, BKIND, AVEC, BVEC, 0, p.ksplit,
                               ntiles - p.tail_begin, p.tail_split});
    return e;
}

template <int AK, int BKIND, int AVEC, int BVEC>
static hipError_t launch_tile(ContractionParams& p, int tile, int nz, const Workspace& ws, hipStream_t stream) {
    switch (tile) {
        case TILE_64:
            // short K: the 16-wide step leaves room for 8 workgroups per CU, which hides the
            // per-tile prologue and epilogue better; long K: fewer, longer steps (measured
            // crossover between K = 256 and K = 512)
            if (p.K < 512) return launch_one<64, 64, 16, 2, 2, 1, AK, BKIND, AVEC, BVEC>(p, nz, ws, stream);
            return launch_one<64, 64, 32, 2, 2, 1, AK, BKIND, AVEC, BVEC>(p, nz, ws, stream);
        case TILE_64_SLICED: return launch_one<64, 64, 32, 2, 2, 2, AK, BKIND, AVEC, BVEC>(p, nz, ws, stream);
        case TILE_128: return launch_one<128, 128, 16, 4, 4, 1, AK, BKIND, AVEC, BVEC>(p, nz, ws, stream);
        case TILE_256: return launch_one<256, 256, 16, 4, 4, 1, AK, BKIND, AVEC, BVEC>(p, nz, ws, stream);
        case TILE_32_SLICED:
            // the gather loader works on 64 columns at a time: no 32-wide form
            if constexpr (BKIND == LOAD_IM2COL) return launch_one<64, 64, 32, 2, 2, 2, AK, BKIND, AVEC, BVEC>(p, nz, ws, stream);
            else return launch_one<32, 32, 64, 1, 1, 4, AK, BKIND, AVEC, BVEC>(p, nz, ws, stream);
        default: return hipErrorInvalidValue;
    }
}

// Estimated time of each tile shape, in units of (output elements per CU) / efficiency:
// the workgroups a CU has to run, times the tile area, over the fraction of the MFMA rate
// that shape sustains when the chip is full.  The 16-wavefront shapes (128 and 256) run one
// workgroup per CU at a time, so their tile count is rounded up to whole rounds of 256: they
// win exactly where that rounding is cheap (2048^2 outputs = 256 tiles of 128: measured 130
// against 123 TFLOP/s for the 64 tile; 4096^2 = 256 tiles of 256: 147 against 144 and 130).
int pick_tile(int64_t M, int64_t N, int64_t K, int64_t nz, bool narrow_ok) {
    static const int bm[TILE_COUNT] = {64, 64, 128, 256, 32};
    static const double eff[TILE_COUNT] = {0.92, 0.92, 0.93, 0.94, 0.5};
    static const int resident[TILE_COUNT] = {8, 4, 1, 1, 8};    // workgroups that share a CU
    const double cus = 256.0;
    int best = TILE_64;
    double best_cost = 0.0;
    for (int t = 0; t < TILE_COUNT; ++t) {
        if (t == TILE_64_SLICED || t == TILE_32_SLICED) continue;
        // 16 wavefronts on a 128 x 128 tile pay off on a long K walk only (96 products of
        // 512 x 512 x 64 ran at 60 instead of 75 TFLOP/s with it)
        if (t == TILE_128 && K < 512) continue;
        const double tiles = (double)((M + bm[t] - 1) / bm[t]) * (double)((N + bm[t] - 1) / bm[t]) * (double)nz;
        double rounds = tiles / cus;
        if (resident[t] == 1) rounds = (double)(int64_t)((tiles + cus - 1) / cus);
        if (rounds < 1.0) rounds = 1.0;
        const double cost = rounds * bm[t] * bm[t] / eff[t];
        if (t == 0 || cost < best_cost) { best = t; best_cost = cost; }
    }
    // Few 64 x 64 tiles and a long K walk: a CU would hold one or two 4-wavefront workgroups,
    // one wavefront per SIMD with every wait exposed; the sliced form runs 8 wavefronts on the
    // same tile.
    if (best == TILE_64) {
        const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64) * nz;
        if (tiles <= 2 * 256 && K >= 256) best = TILE_64_SLICED;
        // Fewer tiles than half the CUs (batch-1 layers): a quarter of the tile with four K slices
        // gives four times the workgroups, each with a quarter of the K walk, and usually makes
        // the split-K finishing launch unnecessary (ResNet-50 at batch 1: 8-12 us per layer
        // instead of 10-14).
        if (narrow_ok && tiles <= 128 && K >= 128) best = TILE_32_SLICED;
    }
    return best;
}

int pick_split(int64_t tiles, int nk, int64_t tile_elems, double overhead, const Workspace& w) {
    if (!w.partial || tiles >= 512 || nk < 4) return 1;
    int best = 1;
    double best_cost = 0.0;
    for (int s = 1; s <= 32 && s * 2 <= nk; ++s) {
        if (s > 1 && tiles * s * tile_elems > w.partial_floats) break;
        const double per_cu = (double)((tiles * s + 255) / 256);
        const double steps = (double)((nk + s - 1) / s) + overhead + (s > 1 ? 0.25 * s + 6.0 : 0.0);
        // A CU that holds a single 4-wavefront workgroup keeps its matrix pipes busy less than a
        // third of the time (every wait of that one wavefront per SIMD is exposed); with several
        // resident workgroups they fill each other's waits.  Fractions measured on ResNet-50
        // (batch 1, 8 and 32 all run fastest with these).
        static const double eff[5] = {1.0, 0.3, 0.5, 0.6, 0.7};
        const int occ = per_cu < 4.0 ? (int)per_cu : 4;
        const double cost = per_cu * steps / (tile_elems <= 64 * 64 ? eff[occ] : eff[4]);
        if (s == 1 || cost < best_cost * 0.97) { best = s; best_cost = cost; }
    }
    return best;
}

hipError_t launch_contraction(ContractionParams& p, int akind, int bkind, int avec, int bvec, int tile, int nz,
                              const Workspace& ws, hipStream_t stream) {
    if ((avec != 1 && avec != 4) || (bvec != 1 && bvec != 4)) return hipErrorInvalidValue;
    // the gather kinds fetch B one value at a time whatever the caller's alignment
    if (bkind == LOAD_IM2COL || bkind == LOAD_RCS) bvec = 1;
    // instances exist for 16-byte loads of both operands, of A only, and of neither
    if (avec == 1) bvec = 1;
#define ONNXHIP_CASE(AK, BKK)                                                                          \
    if (akind == AK && bkind == BKK) {                                                                 \
        if (avec == 4 && bvec == 4) return launch_tile<AK, BKK, 4, 4>(p, tile, nz, ws, stream);        \
        if (avec == 4) return launch_tile<AK, BKK, 4, 1>(p, tile, nz, ws, stream);                     \
        return launch_tile<AK, BKK, 1, 1>(p, tile, nz, ws, stream);                                    \
    }
#define ONNXHIP_CASE_GATHER(AK, BKK)                                                                   \
    if (akind == AK && bkind == BKK) {                                                                 \
        if (avec == 4) return launch_tile<AK, BKK, 4, 1>(p, tile, nz, ws, stream);                     \
        return launch_tile<AK, BKK, 1, 1>(p, tile, nz, ws, stream);                                    \
    }
    ONNXHIP_CASE(LOAD_KC, LOAD_KC)
    ONNXHIP_CASE(LOAD_KC, LOAD_RC)
    ONNXHIP_CASE(LOAD_RC, LOAD_KC)
    ONNXHIP_CASE(LOAD_RC, LOAD_RC)
    ONNXHIP_CASE_GATHER(LOAD_KC, LOAD_IM2COL)
    ONNXHIP_CASE_GATHER(LOAD_KC, LOAD_RCS)
#undef ONNXHIP_CASE
#undef ONNXHIP_CASE_GATHER
    return hipErrorInvalidValue;
}

}  // namespace onnxhip
