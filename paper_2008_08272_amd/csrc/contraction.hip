// Instances of the matrix-core contraction kernel and their launcher.
#include "internal.h"

namespace onnxhip {

template <int BM, int BN, int BK, int WM, int WN, int AK, int BKIND, int VEC>
static hipError_t launch_one(ContractionParams& p, int nz, hipStream_t stream) {
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    p.nz = nz;
    p.ksplit = pick_split((int64_t)p.tiles_m * p.tiles_n * nz, (p.K + BK - 1) / BK, (int64_t)BM * BN, 6.0);
    p.ws_partial = workspace().partial;
    return launch_with_split<BM, BN, WM, WN>(contraction_kernel<BM, BN, BK, WM, WN, AK, BKIND, VEC>, p, nz,
                                             (p.K + BK - 1) / BK, workspace().partial_floats, stream);
}

template <int AK, int BKIND, int VEC>
static hipError_t launch_tile(ContractionParams& p, int tile, int nz, hipStream_t stream) {
    switch (tile) {
        case TILE_64:
            // short K: the 16-wide step leaves room for 8 workgroups per CU, which hides the
            // per-tile prologue and epilogue better; long K: fewer, longer steps (measured
            // crossover between K = 256 and K = 512)
            if (p.K < 512) return launch_one<64, 64, 16, 2, 2, AK, BKIND, VEC>(p, nz, stream);
            return launch_one<64, 64, 32, 2, 2, AK, BKIND, VEC>(p, nz, stream);
        case TILE_128: return launch_one<128, 128, 16, 4, 2, AK, BKIND, VEC>(p, nz, stream);
        case TILE_256: return launch_one<256, 256, 16, 4, 4, AK, BKIND, VEC>(p, nz, stream);
        default: return hipErrorInvalidValue;
    }
}

// Estimated time of each tile shape, in units of (output elements per CU) / efficiency:
// the workgroups a CU has to run, times the tile area, over the fraction of the MFMA rate
// that shape sustains when the chip is full (measured on 2048^3 and 4096^3: the 64 tile
// reaches 0.92, the 128 tile slightly less at mid sizes, the 256 tile 0.94).
int pick_tile(int64_t M, int64_t N, int64_t nz) {
    static const int bm[TILE_COUNT] = {64, 128, 256};
    static const double eff[TILE_COUNT] = {0.92, 0.90, 0.94};
    static const int resident[TILE_COUNT] = {8, 2, 1};    // workgroups that share a CU
    const double cus = 256.0;
    int best = TILE_64;
    double best_cost = 0.0;
    for (int t = 0; t < TILE_COUNT; ++t) {
        const double tiles = (double)((M + bm[t] - 1) / bm[t]) * (double)((N + bm[t] - 1) / bm[t]) * (double)nz;
        double rounds = tiles / cus;
        if (resident[t] == 1) rounds = (double)(int64_t)((tiles + cus - 1) / cus);
        if (rounds < 1.0) rounds = 1.0;
        const double cost = rounds * bm[t] * bm[t] / eff[t];
        if (t == 0 || cost < best_cost) { best = t; best_cost = cost; }
    }
    return best;
}

int pick_split(int64_t tiles, int nk, int64_t tile_elems, double overhead) {
    const Workspace& w = workspace();
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

hipError_t launch_contraction(ContractionParams& p, int akind, int bkind, int vec, int tile, int nz,
                              hipStream_t stream) {
    if (vec != 1 && vec != 4) return hipErrorInvalidValue;
#define ONNXHIP_CASE(AK, BKK)                                                    \
    if (akind == AK && bkind == BKK)                                             \
        return vec == 4 ? launch_tile<AK, BKK, 4>(p, tile, nz, stream)           \
                        : launch_tile<AK, BKK, 1>(p, tile, nz, stream);
    ONNXHIP_CASE(LOAD_KC, LOAD_KC)
    ONNXHIP_CASE(LOAD_KC, LOAD_RC)
    ONNXHIP_CASE(LOAD_RC, LOAD_KC)
    ONNXHIP_CASE(LOAD_RC, LOAD_RC)
    ONNXHIP_CASE(LOAD_KC, LOAD_IM2COL)
    ONNXHIP_CASE(LOAD_KC, LOAD_RCS)
#undef ONNXHIP_CASE
    return hipErrorInvalidValue;
}

}  // namespace onnxhip
