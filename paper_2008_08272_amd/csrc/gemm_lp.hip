// Gemm on 16-bit inputs: kernel instances, tile choice and the C-ABI entry point.
#include <stdio.h>
#include <string.h>

#include "../../include/onnxhip.h"
#include "gemm_lp.h"
#include "internal.h"

using namespace onnxhip;

namespace {

#define fail(st, ...) static_cast<onnx_status>(fail_with((st), __VA_ARGS__))

template <int BM, int BN, int BK, int WM, int WN, int DT, bool LP_OUT, int PF, int BKIND, int BVEC>
hipError_t launch_instance(ContractionParams& p, int nz, const Workspace& ws, hipStream_t stream) {
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    p.nz = nz;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    // The 64 x 64 tile is the one chosen for outputs with few tiles: with a workspace its K range may be split over
    // several workgroups per tile (lp_finish_kernel adds the shares); the larger tiles walk their whole K range.
    // Only outputs that leave half the CUs idle: with more tiles than that the shares and the finishing kernel (whose
    // 16-bit epilogue has no LDS strip) cost more than they save (ResNet-50 in bf16 at batch 32: 1.78 against 1.51 ms).
    constexpr bool kMaySplit = BM == 64;
    p.ksplit = kMaySplit && tiles * nz <= 128 ? pick_split(tiles * nz, (p.K + BK - 1) / BK, (int64_t)BM * BN, 4.0, ws) : 1;
    p.ws_partial = ws.partial;
    const unsigned gz = nz < 32768 ? (unsigned)nz : 32768u;
    const unsigned gy = ((unsigned)nz + gz - 1) / gz;
    if (tiles * (WM * WN) > 0x7fffffffLL || gy * (unsigned)p.ksplit > 65535u) return hipErrorInvalidValue;
    p.tail_begin = (int)tiles;
    p.tail_split = 1;
    hipLaunchKernelGGL((gemm_lp_kernel<BM, BN, BK, WM, WN, DT, LP_OUT, PF, BKIND, BVEC>), dim3((unsigned)tiles, gy * (unsigned)p.ksplit, gz),
                       dim3(64 * WM * WN), 0, stream, p);
    hipError_t e = hipGetLastError();
    if constexpr (kMaySplit) {
        if (e == hipSuccess && p.ksplit > 1) {
            hipLaunchKernelGGL((lp_finish_kernel<BM, BN, WM, WN, DT, LP_OUT>), dim3((unsigned)tiles * (WM * WN), gy, gz), dim3(64), 0, stream, p);
            e = hipGetLastError();
        }
    }
    record_launch(LaunchRecord{"gemm_lp", BM, BN, BK, WM, WN, 1, LOAD_KC, BKIND, 8, BVEC, DT + (LP_OUT ? 2 : 0), p.ksplit, 0, 1});
    return e;
}

// Tile by the same estimate as the fp32 kernel: workgroups per CU x tile area / efficiency.
template <int DT, bool LP_OUT, int BKIND, int BVEC>
hipError_t launch_tile(ContractionParams& p, int nz, const Workspace& ws, hipStream_t stream) {
    const double cus = 256.0;
    const double t256 = (double)((p.M + 255) / 256) * (double)((p.N + 255) / 256) * nz;
    const double t128 = (double)((p.M + 127) / 128) * (double)((p.N + 127) / 128) * nz;
    const double c256 = (double)(int64_t)((t256 + cus - 1) / cus) * 65536.0 / 1.0;
    // (1x1 convolutions with K <= 256 are bound by their stores, and the 128 x 128 tile's are the less efficient ones:
    // ResNet-50's 64 -> 256 at 56 x 56 and 128 / 256 -> 512 at 28 x 28 take 33.6 / 20.0 us on 256 x 256 tiles against
    // 37.1 / 22.9-23.8)
    const double eff128 = (p.col_images && p.K <= 256) ? 0.75 : 0.85;
    const double c128 = (t128 / cus < 1.0 ? 1.0 : t128 / cus) * 16384.0 / eff128;
    // at most 64 rows: a larger tile would be half empty (ResNet-50's 1x1 layers with 64 filters at batch 32: 18.6 -> 12.4
    // and 25.6 -> 18.4 us)
    if (p.M <= 64) return launch_instance<64, 64, 64, 2, 2, DT, LP_OUT, 2, BKIND, BVEC>(p, nz, ws, stream);
    // (loads two steps ahead for a K-contiguous B; the row-contiguous loader's pairing needs the registers of
    // the second staging set: with it the kernel spills inside its main loop)
    if (c256 <= c128) return launch_instance<256, 256, 64, 2, 4, DT, LP_OUT, BKIND == LOAD_KC ? 2 : 1, BKIND, BVEC>(p, nz, ws, stream);
    // fewer 128 x 128 tiles than half the CUs (than all CUs when K is short): 64 x 64 tiles spread the product
    // over the chip (measured 1024^3: 213 vs 121 TFLOP/s; from 2048^3 on the larger tile wins; 2048 x 1568 x 512:
    // 21.8 vs 33.6 us)
    if (t128 < cus / 2 || (t128 < cus && p.K <= 512)) return launch_instance<64, 64, 64, 2, 2, DT, LP_OUT, 2, BKIND, BVEC>(p, nz, ws, stream);
    return launch_instance<128, 128, 64, 2, 2, DT, LP_OUT, 1, BKIND, BVEC>(p, nz, ws, stream);
}

template <int BKIND, int BVEC>
hipError_t launch_types(ContractionParams& p, int nz, int in_type, int out_type, const Workspace& ws, hipStream_t s) {
    if (in_type == LP_F16) return out_type == 0 ? launch_tile<LP_F16, false, BKIND, BVEC>(p, nz, ws, s) : launch_tile<LP_F16, true, BKIND, BVEC>(p, nz, ws, s);
    return out_type == 0 ? launch_tile<LP_BF16, false, BKIND, BVEC>(p, nz, ws, s) : launch_tile<LP_BF16, true, BKIND, BVEC>(p, nz, ws, s);
}

bool multiple_of(const int64_t* v, int n, int64_t m) {
    for (int i = 0; i < n; ++i)
        if (v[i] % m) return false;
    return true;
}

}  // namespace

namespace onnxhip {

int lp_tuned_fits(const ContractionParams& p, int akind, int bkind, int nz) {
    const int64_t span = (1LL << 31) - 64, rows = 256, bk = 64;
    if (akind != LOAD_KC || (bkind != LOAD_KC && bkind != LOAD_RC) || nz < 1 || nz > 32768LL * 65535LL) return 0;
    // A: 16-byte chunks of 8 k, also at the start of every z-slice; 32-bit offsets inside a 256-row tile
    if (p.K % 8 || p.a_ld % 8 || !aligned16(p.A) || !multiple_of(p.a_bs, p.nbd, 8) || (rows * p.a_ld + p.K) * 2 >= span) return 0;
    // Y (and a residual laid out like it): 32-bit offsets inside a tile, which for a convolution
    // spans the images its columns belong to
    const int64_t P = p.col_images ? (int64_t)p.colP.d : 0;
    const int64_t tile_images = p.col_images ? (rows + P - 1) / P + 1 : 0;
    if ((rows * p.y_rs + (p.col_images ? tile_images * p.y_img : rows)) * 4 >= span) return 0;
    if (bkind == LOAD_KC)
        return (p.b_ld % 8 == 0 && aligned16(p.B) && multiple_of(p.b_bs, p.nbd, 8) && (rows * p.b_ld + p.K) * 2 < span) ? 8 : 0;
    // B row-contiguous: chunks of 8 or 4 columns that never straddle the end of a k row or of an image
    if ((bk * p.b_ld + (p.col_images ? tile_images * p.b_img : rows)) * 2 >= span) return 0;
    for (int vec = 8; vec >= 4; vec /= 2) {
        const bool ok = p.N % vec == 0 && p.b_ld % vec == 0 && (reinterpret_cast<uintptr_t>(p.B) % (2 * vec)) == 0 &&
                        multiple_of(p.b_bs, p.nbd, vec) && (!p.col_images || (P % vec == 0 && p.b_img % vec == 0));
        if (ok) return vec;
    }
    return 0;
}

hipError_t launch_lp_tuned(ContractionParams& p, int bkind, int bvec, int nz, int in_type, int out_type, const Workspace& ws,
                           hipStream_t stream) {
    if (bkind == LOAD_KC) return launch_types<LOAD_KC, 8>(p, nz, in_type, out_type, ws, stream);
    if (bvec == 8) return launch_types<LOAD_RC, 8>(p, nz, in_type, out_type, ws, stream);
    if (bvec == 4) return launch_types<LOAD_RC, 4>(p, nz, in_type, out_type, ws, stream);
    return hipErrorInvalidValue;
}

}  // namespace onnxhip

extern "C" {

onnx_status onnx_gemm_lp(const void* A, const int64_t a_dims[2], const void* B, const int64_t b_dims[2], const float* C,
                         const int64_t* c_dims, int c_rank, float alpha, float beta, int transA, int transB, onnx_act act,
                         void* Y, const int64_t y_dims[2], onnx_dtype in_type, onnx_dtype out_type, void* stream) {
    if (!a_dims || !b_dims || !y_dims) return fail(ONNX_ERR_NULL, "gemm_lp: NULL dims array");
    if (in_type != ONNX_F16 && in_type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "gemm_lp: in_type must be ONNX_F16 or ONNX_BF16");
    if (out_type != ONNX_F32 && out_type != in_type) return fail(ONNX_ERR_ATTR, "gemm_lp: out_type must be ONNX_F32 or in_type");
    for (int i = 0; i < 2; ++i)
        if (a_dims[i] < 0 || b_dims[i] < 0) return fail(ONNX_ERR_SHAPE, "gemm_lp: negative dimension");
    const int64_t M = transA ? a_dims[1] : a_dims[0], K = transA ? a_dims[0] : a_dims[1];
    const int64_t Kb = transB ? b_dims[1] : b_dims[0], N = transB ? b_dims[0] : b_dims[1];
    if (Kb != K) return fail(ONNX_ERR_SHAPE, "gemm_lp: inner dimensions differ (%lld vs %lld)", (long long)K, (long long)Kb);
    if (y_dims[0] != M || y_dims[1] != N)
        return fail(ONNX_ERR_SHAPE, "gemm_lp: y_dims is {%lld,%lld} but the result is {%lld,%lld}", (long long)y_dims[0],
                    (long long)y_dims[1], (long long)M, (long long)N);
    if (act != ONNX_ACT_NONE && act != ONNX_ACT_RELU) return fail(ONNX_ERR_ATTR, "gemm_lp: unknown activation");
    int64_t crs = 0, ccs = 0, nc = 0;
    if (C) {
        int64_t r = 1, c = 1;
        if (c_rank < 0 || c_rank > 2) return fail(ONNX_ERR_RANK, "gemm_lp: C must have rank 0, 1 or 2");
        if (c_rank > 0 && !c_dims) return fail(ONNX_ERR_NULL, "gemm_lp: c_dims is NULL");
        if (c_rank == 1) c = c_dims[0];
        if (c_rank == 2) { r = c_dims[0]; c = c_dims[1]; }
        if (!((r == 1 || r == M) && (c == 1 || c == N)))
            return fail(ONNX_ERR_SHAPE, "gemm_lp: C {%lld,%lld} does not broadcast to {%lld,%lld}", (long long)r, (long long)c,
                        (long long)M, (long long)N);
        crs = (r == 1) ? 0 : c;
        ccs = (c == 1) ? 0 : 1;
        nc = r * c;
    }
    if (M * N == 0) return ONNX_OK;
    if (!Y || (K > 0 && (!A || !B))) return fail(ONNX_ERR_NULL, "gemm_lp: A, B and Y must not be NULL");
    const int64_t ysz = out_type == ONNX_F32 ? 4 : 2;
    if (overlaps(Y, M * N * ysz, A, M * K * 2) || overlaps(Y, M * N * ysz, B, K * N * 2) || overlaps(Y, M * N * ysz, C, nc * 4))
        return fail(ONNX_ERR_ALIAS, "gemm_lp: Y overlaps an input");
    if (M > 0x7fffffffLL || N > 0x7fffffffLL || K > 0x7fffffffLL) return fail(ONNX_ERR_UNSUPPORTED, "gemm_lp: extent above 2^31-1");
    ContractionParams p;
    memset(&p, 0, sizeof(p));
    for (int i = 0; i < MAX_BATCH_DIMS; ++i) p.bdim[i] = 1;
    p.colP = FastDiv::make(1);
    p.ic.kHW = p.ic.kW = p.ic.OW = FastDiv::make(1);
    p.A = static_cast<const float*>(A);
    p.B = static_cast<const float*>(B);
    p.Y = static_cast<float*>(Y);
    p.bias = C;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.a_ld = a_dims[1]; p.b_ld = b_dims[1]; p.y_rs = N;
    p.nz = 1;
    p.alpha = alpha; p.beta = beta; p.relu = act == ONNX_ACT_RELU;
    p.bias_mode = (crs != 0 && ccs != 0) ? BIAS_FULL : (crs != 0 ? BIAS_ROW : BIAS_COL);
    p.bias_cs = (int)ccs;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the tuned kernel: A K-contiguous, 16-byte loads, 32-bit tile offsets; everything else: the general kernel
    const int akind = transA ? LOAD_RC : LOAD_KC, bkind = transB ? LOAD_KC : LOAD_RC;
    const int bvec = lp_tuned_fits(p, akind, bkind, 1);
    const hipError_t e = bvec ? launch_lp_tuned(p, bkind, bvec, 1, (int)in_type, (int)out_type, workspace(), s)
                              : launch_lp_generic(p, akind, bkind, 1, (int)in_type, (int)out_type, s);
    if (e != hipSuccess) return fail(ONNX_ERR_DEVICE, "gemm_lp: %s", hipGetErrorString(e));
    return ONNX_OK;
}

}  // extern "C"
