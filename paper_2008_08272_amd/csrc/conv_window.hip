// Instances of the LDS-patch convolution kernel and their launcher.
#include "conv_window.h"
#include "internal.h"

namespace onnxhip {

namespace {

struct WindowConfig {
    int bm, bn, nt, maxpb;
    double eff;        // fraction of the MFMA rate the shape sustains on a full chip (measured)
};
// Keep in step with the template instances in launch_config below.
const WindowConfig kConfigs[] = {
    {64, 64, 256, 9, 0.75},
    {128, 128, 512, 8, 0.80},
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

template <int BM, int BN, int WM, int WN, int KH, int KW, int NPB>
hipError_t launch_instance(ContractionParams& p, int nz, const Workspace& ws, hipStream_t stream) {
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    p.nz = nz;
    p.ksplit = pick_split((int64_t)p.tiles_m * p.tiles_n * nz, p.ic.Cg / WIN_CB, (int64_t)BM * BN, 4.0, ws);
    p.ws_partial = ws.partial;
    const hipError_t e = launch_with_split<BM, BN, WM, WN>(conv_window_kernel<BM, BN, WM, WN, KH, KW, NPB>, p, nz,
                                                           p.ic.Cg / WIN_CB, ws.partial_floats, stream);
    record_launch(LaunchRecord{"conv_window", BM, BN, WIN_CB * KH * KW, WM, WN, 1, LOAD_KC, LOAD_IM2COL, 4, 1, NPB, p.ksplit,
                               p.tiles_m * p.tiles_n - p.tail_begin, p.tail_split});
    return e;
}

// npb = passes the patch needs; the instance with the next larger pass count runs it.
template <int BM, int BN, int WM, int WN, int KH, int KW>
hipError_t launch_passes(ContractionParams& p, int npb, int nz, const Workspace& ws, hipStream_t stream) {
    if (npb <= 2) return launch_instance<BM, BN, WM, WN, KH, KW, 2>(p, nz, ws, stream);
    if (npb <= 3) return launch_instance<BM, BN, WM, WN, KH, KW, 3>(p, nz, ws, stream);
    if (npb <= 4) return launch_instance<BM, BN, WM, WN, KH, KW, 4>(p, nz, ws, stream);
    if (npb <= 5) return launch_instance<BM, BN, WM, WN, KH, KW, 5>(p, nz, ws, stream);
    if (npb <= 6) return launch_instance<BM, BN, WM, WN, KH, KW, 6>(p, nz, ws, stream);
    if (npb <= 8) return launch_instance<BM, BN, WM, WN, KH, KW, 8>(p, nz, ws, stream);
    // nine passes: the stride-2 3x3 convolution of a 56 x 56 plane (ResNet50's first down-sampling block)
    // needs 2052 patch floats per channel block on the 64 x 64 tile, four more than eight passes hold
    if constexpr (BM == 64) {
        if (npb <= 9) return launch_instance<BM, BN, WM, WN, KH, KW, 9>(p, nz, ws, stream);
    }
    return hipErrorInvalidValue;
}

template <int KH, int KW>
hipError_t launch_config(ContractionParams& p, int cfg, int npb, int nz, const Workspace& ws, hipStream_t stream) {
    switch (cfg) {
        case 0: return launch_passes<64, 64, 2, 2, KH, KW>(p, npb, nz, ws, stream);
        case 1: return launch_passes<128, 128, 4, 2, KH, KW>(p, npb, nz, ws, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool launch_conv_window(ContractionParams& p, int kH, int kW, int OH, int OW, int Cg, int nz,
                        const Workspace& ws, hipStream_t stream, hipError_t* status) {
    if (!(kH == 3 && kW == 3)) return false;
    if (Cg % WIN_CB != 0) return false;
    Im2colGeom& g = p.ic;
    const int E = (kH - 1) * g.dH + 1;
    const int PC = (OW - 1) * g.sW + (kW - 1) * g.dW + 1;
    int best = -1, best_plane = 0;
    double best_cost = 0.0;
    for (int c = 0; c < kNumConfigs; ++c) {
        const WindowConfig& k = kConfigs[c];
        if (OW > k.bn) continue;
        const int64_t plane = (int64_t)patch_rows(k.bn, OH, OW, g.sH, E) * PC;
        if (WIN_CB * plane > (int64_t)k.maxpb * k.nt) continue;
        const double tiles = (double)((p.M + k.bm - 1) / k.bm) * (double)((p.N + k.bn - 1) / k.bn) * nz;
        double rounds = tiles / 256.0;
        if (rounds < 1.0) rounds = 1.0;
        // the nine-pass instance keeps three instead of four wavefronts per SIMD: on a full chip it ran
        // the 56 -> 28 stride-2 layer at 73 TFLOP/s where the 128 x 128 tile reaches 82; with few tiles
        // (batch 1: 18 against 29 us) it is the better one
        const double eff = WIN_CB * plane > (int64_t)8 * k.nt ? 0.55 : k.eff;
        const double cost = rounds * k.bm * k.bn / eff;
        if (best < 0 || cost < best_cost) { best = c; best_cost = cost; best_plane = (int)plane; }
    }
    if (best < 0) return false;
    g.OH = OH; g.Cg = Cg; g.E = E; g.IPR = (OH - 1) * g.sH + E; g.PC = PC; g.plane = best_plane;
    g.OHd = FastDiv::make((uint32_t)OH);
    g.PCd = FastDiv::make((uint32_t)PC);
    g.planed = FastDiv::make((uint32_t)best_plane);
    g.IPRd = FastDiv::make((uint32_t)g.IPR);
    const int npb = (WIN_CB * best_plane + kConfigs[best].nt - 1) / kConfigs[best].nt;
    *status = launch_config<3, 3>(p, best, npb, nz, ws, stream);
    return true;
}

}  // namespace onnxhip
