// C-ABI layer: argument validation, shape inference and kernel selection.
// Everything here runs on the host; the arithmetic of every operator runs in the kernels.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "../../include/onnxhip.h"
#include "internal.h"

using namespace onnxhip;

namespace {

thread_local char g_err[320] = "";
thread_local LaunchRecord g_launch = {};
thread_local char g_launch_text[200] = "";

#define fail(st, ...) static_cast<onnx_status>(fail_with((st), __VA_ARGS__))

const int64_t kIntMax = 0x7fffffffLL;

int64_t floordiv(int64_t a, int64_t b) {
    int64_t q = a / b;
    if ((a % b != 0) && ((a < 0) != (b < 0))) --q;
    return q;
}

// One axis of a sliding window. Returns false when the window exceeds the padded input.
bool window_extent(int64_t in, int64_t k, int64_t pb, int64_t pe, int64_t s, int64_t d, int ceil_mode,
                   int64_t* out) {
    const int64_t eff = (k - 1) * d + 1;
    const int64_t span = in + pb + pe - eff;
    if (span < 0) return false;
    int64_t o;
    if (ceil_mode) {
        o = floordiv(span + s - 1, s) + 1;
        if ((o - 1) * s >= in + pb) --o;     // last window would start past the input: drop it
    } else {
        o = floordiv(span, s) + 1;
    }
    *out = o;
    return true;
}

// The kernels address each operand tile with 32-bit byte offsets below 2^31 from the tile's
// first element (tiles have at most 256 rows and walk K in steps of at most 32).
const int64_t kTileRows = 256, kTileK = 32, kSpan = (1LL << 31) - 64;
bool kc_fits(int64_t ld, int64_t K) { return (kTileRows * ld + K) * 4 < kSpan; }
bool rc_fits(int64_t ld, int64_t lead) { return (kTileK * ld + lead) * 4 < kSpan; }

void no_batch(ContractionParams& p) {
    p.nbd = 0;
    for (int i = 0; i < MAX_BATCH_DIMS; ++i) { p.bdim[i] = 1; p.a_bs[i] = 0; p.b_bs[i] = 0; }
    p.y_zs = 0;
    p.bias_zs = 0;
    p.col_images = 0;
    p.colP = FastDiv::make(1);
    p.y_img = 0;
    p.b_img = 0;
    memset(&p.ic, 0, sizeof(p.ic));
    p.ic.kHW = p.ic.kW = p.ic.OW = FastDiv::make(1);
}

// What onnx_set_workspace last stored.  Setting it and reading it are serialised, so a call
// always sees a matching pointer and size; which of two racing settings a call sees is up to
// the caller to order.
std::mutex g_ws_mutex;
Workspace g_ws = {nullptr, 0};

onnx_status device_status(hipError_t e, const char* what) {
    if (e == hipSuccess) return ONNX_OK;
    return fail(ONNX_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

namespace onnxhip {
Workspace workspace() {
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    return g_ws;
}
int report_error(int status, const char* message) {
    snprintf(g_err, sizeof(g_err), "%s", message);
    return status;
}
void record_launch(const LaunchRecord& r) { g_launch = r; }
int fail_with(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}
}  // namespace onnxhip

// ---- the entry point that may not allocate: its split-K scratch is this fixed array -----------
namespace {

constexpr int64_t kFixedScratchFloats = (int64_t)ONNX_CONV_FIXED_SCRATCH_BYTES / 4;
static __device__ __align__(256) float scratch[kFixedScratchFloats];

// Every GPU holds its own copy of `scratch` at its own address; in host code the array's name is
// only a handle for hipGetSymbolAddress.  The address is looked up once per device, with that
// device current, and kept here.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

onnx_status fixed_scratch(Workspace* out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ONNX_ERR_DEVICE, "conv (fixed scratch): hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(ONNX_ERR_UNSUPPORTED, "conv (fixed scratch): device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(ONNX_ERR_DEVICE, "conv (fixed scratch): hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<float*>(ptr);
    }
    out->partial = g_scratch_ptr[dev];
    out->partial_floats = kFixedScratchFloats;
    return ONNX_OK;
}

}  // namespace

namespace {

// ONNX Conv with the split-K scratch `caller_ws` (possibly none), or, when that is NULL, with
// the library's fixed array, whose address is looked up once the arguments have passed
// validation.  max_outputs > 0 caps the number of output elements (the fixed-scratch entry
// point's limit).
onnx_status conv_with_workspace(const float* X, const int64_t x_dims[4], const float* W, const int64_t w_dims[4],
                                const float* B, const int64_t pads[4], const int64_t strides[2],
                                const int64_t dilations[2], int64_t group, const float* residual, onnx_act act,
                                float* Y, const int64_t y_dims[4], const Workspace* caller_ws, int64_t max_outputs,
                                void* stream, onnx_dtype in_type = ONNX_F32, onnx_dtype out_type = ONNX_F32,
                                bool filters_in_tap_order = false) {
    if (!x_dims || !w_dims || !y_dims) return fail(ONNX_ERR_NULL, "conv: NULL dims array");
    int64_t yd[4];
    const onnx_status st = onnx_conv_infer(x_dims, w_dims, pads, strides, dilations, group, yd);
    if (st != ONNX_OK) return st;
    for (int i = 0; i < 4; ++i)
        if (yd[i] != y_dims[i])
            return fail(ONNX_ERR_SHAPE, "conv: y_dims[%d]=%lld but the inferred extent is %lld", i,
                        (long long)y_dims[i], (long long)yd[i]);
    if (act != ONNX_ACT_NONE && act != ONNX_ACT_RELU) return fail(ONNX_ERR_ATTR, "conv: unknown activation");
    const int64_t N = x_dims[0], C = x_dims[1], H = x_dims[2], Wd = x_dims[3];
    const int64_t M = w_dims[0], Cg = w_dims[1], kH = w_dims[2], kW = w_dims[3];
    const int64_t OH = yd[2], OW = yd[3], P = OH * OW;
    const int64_t ny = N * M * P;
    if (ny == 0) return ONNX_OK;
    if (max_outputs > 0 && ny > max_outputs)
        return fail(ONNX_ERR_UNSUPPORTED, "conv: %lld output elements exceed the %lld this entry point's fixed scratch is "
                    "sized for; use onnx_conv with onnx_set_workspace", (long long)ny, (long long)max_outputs);
    if (!X || !W || !Y) return fail(ONNX_ERR_NULL, "conv: X, W and Y must not be NULL");
    const int64_t nx = N * C * H * Wd, nw = M * Cg * kH * kW;
    const int64_t esz = in_type == ONNX_F32 ? 4 : 2, ysz = out_type == ONNX_F32 ? 4 : 2;     // bytes per element
    if (overlaps(Y, ny * ysz, X, nx * esz) || overlaps(Y, ny * ysz, W, nw * esz) || overlaps(Y, ny * ysz, B, M * 4) ||
        overlaps(Y, ny * ysz, residual, ny * ysz))
        return fail(ONNX_ERR_ALIAS, "conv: Y overlaps an input");
    const int64_t K = Cg * kH * kW, Mg = M / group, NP = N * P;
    if (C * H * Wd > kIntMax || M * P > kIntMax || K > kIntMax || pads[0] > kIntMax || pads[1] > kIntMax ||
        strides[0] > kIntMax || strides[1] > kIntMax || kH * dilations[0] > kIntMax ||
        kW * dilations[1] > kIntMax || N > kIntMax || group > 32768LL * 65535LL)
        return fail(ONNX_ERR_UNSUPPORTED, "conv: a single image / filter bank exceeds 2^31 elements");
    hipStream_t s = static_cast<hipStream_t>(stream);
    Workspace ws = {nullptr, 0};
    if (caller_ws) {
        ws = *caller_ws;
    } else {
        const onnx_status sst = fixed_scratch(&ws);
        if (sst != ONNX_OK) return sst;
    }

    WindowGeom g;
    g.N = (int)N; g.C = (int)C; g.H = (int)H; g.W = (int)Wd; g.OH = (int)OH; g.OW = (int)OW;
    g.kH = (int)kH; g.kW = (int)kW; g.sH = (int)strides[0]; g.sW = (int)strides[1];
    g.pT = (int)pads[0]; g.pL = (int)pads[1]; g.pB = (int)pads[2]; g.pR = (int)pads[3];
    g.dH = (int)dilations[0]; g.dW = (int)dilations[1];

    if (in_type != ONNX_F32) {
        // 16-bit tensors: the pointwise case reads the input as a row-contiguous [C][H*W] matrix per
        // image (through the tuned kernel when its alignment conditions hold), everything else
        // gathers it element by element in the general kernel
        if (NP > kIntMax || group > 32768LL * 65535LL)
            return fail(ONNX_ERR_UNSUPPORTED, "conv (16-bit): more than 2^31-1 output positions");
        ContractionParams p;
        no_batch(p);
        p.A = W; p.B = X; p.Y = Y; p.bias = B; p.residual = residual;
        p.M = (int)(M / group); p.N = (int)NP; p.K = (int)(Cg * kH * kW);
        p.a_ld = p.K;
        p.nbd = 1; p.bdim[0] = (int)group; p.a_bs[0] = (M / group) * p.K; p.b_bs[0] = Cg * H * Wd;
        p.y_zs = (M / group) * P; p.bias_zs = M / group; p.y_rs = P;
        p.col_images = 1; p.colP = FastDiv::make((uint32_t)P); p.y_img = M * P; p.b_img = C * H * Wd;
        p.alpha = 1.f; p.beta = 1.f; p.bias_mode = BIAS_ROW; p.bias_cs = 0; p.relu = act == ONNX_ACT_RELU;
        const bool unpadded_1x1 = kH == 1 && kW == 1 && pads[0] == 0 && pads[1] == 0 && pads[2] == 0 && pads[3] == 0;
        bool pw = unpadded_1x1 && strides[0] == 1 && strides[1] == 1;
        p.ic.C = (int)C; p.ic.H = (int)H; p.ic.W = (int)Wd;
        p.ic.sH = g.sH; p.ic.sW = g.sW; p.ic.pT = g.pT; p.ic.pL = g.pL; p.ic.dH = g.dH; p.ic.dW = g.dW;
        p.ic.kHW = FastDiv::make((uint32_t)(kH * kW));
        p.ic.kW = FastDiv::make((uint32_t)kW);
        p.ic.OW = FastDiv::make((uint32_t)OW);
        p.ic.image_stride = (int)(C * H * Wd);
        // Layout passes through the workspace (lp_layout.hip) for 1x1 convolutions the tuned kernel cannot read
        // as they are: first the positions a strided one reads, then, if the planes still have no aligned
        // chunks of columns, one K-contiguous row per position.
        char* ws_free = reinterpret_cast<char*>(ws.partial);
        int64_t ws_bytes = ws.partial ? ws.partial_floats * 4 : 0;
        const int64_t copy_bytes = ((N * C * P * 2 + 255) / 256) * 256;
        if (unpadded_1x1 && !pw && K % 8 == 0 && copy_bytes <= ws_bytes && N * C * P <= kIntMax) {
            const hipError_t e = launch_lp_subsample(X, ws_free, N * C, (int)H, (int)Wd, (int)OH, (int)OW, g.sH, g.sW, s);
            if (e != hipSuccess) return device_status(e, "conv (16-bit, subsample)");
            p.B = reinterpret_cast<const float*>(ws_free);
            ws_free += copy_bytes; ws_bytes -= copy_bytes;
            p.b_bs[0] = Cg * P; p.b_img = C * P;
            p.ic.H = (int)OH; p.ic.W = (int)OW; p.ic.sH = 1; p.ic.sW = 1; p.ic.image_stride = (int)(C * P);
            pw = true;
        }
        p.b_ld = pw ? P : 0;
        int bvec = pw ? lp_tuned_fits(p, LOAD_KC, LOAD_RC, (int)group) : 0;
        if (pw && !bvec && K % 8 == 0 && copy_bytes <= ws_bytes && N <= 65535) {
            const hipError_t e = launch_lp_planes_to_rows(p.B, ws_free, (int)N, (int)C, (int)P, s);
            if (e != hipSuccess) return device_status(e, "conv (16-bit, planes to rows)");
            ContractionParams q = p;                 // B as an [N*P][C] K-contiguous matrix; Y keeps its (image, position) columns
            q.B = reinterpret_cast<const float*>(ws_free);
            q.b_ld = C; q.b_bs[0] = Cg; q.b_img = 0;
            if (lp_tuned_fits(q, LOAD_KC, LOAD_KC, (int)group))
                return device_status(launch_lp_tuned(q, LOAD_KC, 8, (int)group, (int)in_type, (int)out_type,
                                                     Workspace{reinterpret_cast<float*>(ws_free + copy_bytes), (ws_bytes - copy_bytes) / 4}, s),
                                     "conv (16-bit)");
        }
        if (bvec)
            return device_status(launch_lp_tuned(p, LOAD_RC, bvec, (int)group, (int)in_type, (int)out_type,
                                                 Workspace{ws_bytes > 0 ? reinterpret_cast<float*>(ws_free) : nullptr, ws_bytes / 4}, s),
                                 "conv (16-bit)");
        if (!pw && !filters_in_tap_order) {
            hipError_t e = hipSuccess;
            if (launch_conv_stem_lp(X, W, B, Y, g, (int)M, (int)Cg, (int)group, residual != nullptr, act == ONNX_ACT_RELU, (int)in_type,
                                    (int)out_type, s, &e))
                return device_status(e, "conv (16-bit, stem)");
        }
        if (!pw) {
            hipError_t e = hipSuccess;
            if (launch_conv_window_lp(p, (int)kH, (int)kW, (int)OH, (int)OW, (int)Cg, (int)group, (int)in_type, (int)out_type,
                                      filters_in_tap_order, ws, s, &e))
                return device_status(e, "conv (16-bit, lds patch)");
        }
        if (filters_in_tap_order)
            return fail(ONNX_ERR_UNSUPPORTED, "conv_lp_taps: only 3x3 convolutions with a multiple of 16 channels per group whose "
                        "patch fits the LDS-patch kernel take filters in tap order; use onnx_conv_lp");
        return device_status(launch_lp_generic(p, LOAD_KC, pw ? LOAD_RC : LOAD_IM2COL, (int)group, (int)in_type,
                                               (int)out_type, s), "conv (16-bit)");
    }

    if (group == 1) {
        hipError_t e = hipSuccess;
        if (launch_conv_resident(X, W, B, residual, Y, g, (int)M, (int)Cg, act == ONNX_ACT_RELU, s, &e))
            return device_status(e, "conv (resident filters)");
    }

    // images one tile of columns can touch, and the span of input they cover
    const int64_t tile_images = (kTileRows + P - 1) / P + 1;
    const bool use_mfma = Mg >= 16 && K >= 8 && NP <= kIntMax && kc_fits(K, K) &&
                          tile_images * C * H * Wd * 4 < kSpan &&
                          (kTileRows * P + tile_images * M * P) * 4 < kSpan;
    if (!use_mfma)
        return device_status(launch_conv_direct(X, W, B, residual, Y, g, (int)M, (int)Cg, (int)group,
                                                act == ONNX_ACT_RELU, s), "conv (direct)");

    ContractionParams p;
    no_batch(p);
    p.A = W; p.B = X; p.Y = Y; p.bias = B; p.residual = residual;
    p.M = (int)Mg; p.N = (int)NP; p.K = (int)K;
    p.a_ld = K;
    p.nbd = 1; p.bdim[0] = (int)group; p.a_bs[0] = Mg * K; p.b_bs[0] = Cg * H * Wd;
    p.y_zs = Mg * P; p.bias_zs = Mg; p.y_rs = P;
    p.col_images = 1; p.colP = FastDiv::make((uint32_t)P); p.y_img = M * P; p.b_img = C * H * Wd;
    p.alpha = 1.f; p.beta = 1.f; p.bias_mode = BIAS_ROW; p.bias_cs = 0; p.relu = act == ONNX_ACT_RELU;
    const bool unpadded_1x1 = kH == 1 && kW == 1 && pads[0] == 0 && pads[1] == 0 && pads[2] == 0 && pads[3] == 0;
    const bool pointwise = unpadded_1x1 && strides[0] == 1 && strides[1] == 1;
    int bkind, bvec = 1;
    // 16-byte loads per operand: the filters when every row starts aligned, the input of a
    // pointwise convolution when every plane does
    const bool a_vec = (K % 4 == 0) && aligned16(W);
    if (pointwise) {
        bkind = LOAD_RC;
        p.b_ld = H * Wd;
        bvec = (P % 4 == 0 && aligned16(X)) ? 4 : 1;
    } else if (unpadded_1x1) {
        // strided 1x1 (ResNet's projection shortcuts): rows of B are still whole planes apart
        bkind = LOAD_RCS;
        p.b_ld = H * Wd;
        p.ic.W = (int)Wd; p.ic.sH = g.sH; p.ic.sW = g.sW;
        p.ic.OW = FastDiv::make((uint32_t)OW);
    } else {
        bkind = LOAD_IM2COL;
        p.b_ld = 0;
        p.ic.C = (int)C; p.ic.H = (int)H; p.ic.W = (int)Wd;
        p.ic.sH = g.sH; p.ic.sW = g.sW; p.ic.pT = g.pT; p.ic.pL = g.pL; p.ic.dH = g.dH; p.ic.dW = g.dW;
        p.ic.kHW = FastDiv::make((uint32_t)(kH * kW));
        p.ic.kW = FastDiv::make((uint32_t)kW);
        p.ic.OW = FastDiv::make((uint32_t)OW);
        p.ic.image_stride = (int)(C * H * Wd);
    }
    if (bkind == LOAD_IM2COL && a_vec) {
        hipError_t e = hipSuccess;
        if (launch_conv_window(p, (int)kH, (int)kW, (int)OH, (int)OW, (int)Cg, (int)group, ws, s, &e))
            return device_status(e, "conv (lds patch)");
    }
    const int tile = pick_tile(Mg, NP, K, group, bkind != LOAD_IM2COL);
    return device_status(launch_contraction(p, LOAD_KC, bkind, a_vec ? 4 : 1, bvec, tile, (int)group, ws, s),
                         "conv (mfma)");
}

}  // namespace

namespace {

// ONNX MatMul on fp32 tensors (in_type ONNX_F32) or on 16-bit tensors with the result stored as
// out_type (fp32 or the input type).
onnx_status matmul_any(const float* A, const int64_t* a_dims, int a_rank, const float* B,
                       const int64_t* b_dims, int b_rank, float* Y, const int64_t* y_dims, int y_rank,
                       onnx_dtype in_type, onnx_dtype out_type, void* stream) {
    int64_t yd[ONNX_MAX_RANK];
    int yr = 0;
    const onnx_status st = onnx_matmul_infer(a_dims, a_rank, b_dims, b_rank, yd, &yr);
    if (st != ONNX_OK) return st;
    if (yr != y_rank) return fail(ONNX_ERR_RANK, "matmul: y_rank is %d but the result has rank %d", y_rank, yr);
    if (yr > 0 && !y_dims) return fail(ONNX_ERR_NULL, "matmul: y_dims is NULL");
    for (int i = 0; i < yr; ++i)
        if (yd[i] != y_dims[i])
            return fail(ONNX_ERR_SHAPE, "matmul: y_dims[%d]=%lld but the inferred extent is %lld", i,
                        (long long)y_dims[i], (long long)yd[i]);
    const int64_t M = a_rank >= 2 ? a_dims[a_rank - 2] : 1, K = a_dims[a_rank - 1];
    const int64_t N = b_rank >= 2 ? b_dims[b_rank - 1] : 1;
    const int nba = a_rank >= 2 ? a_rank - 2 : 0, nbb = b_rank >= 2 ? b_rank - 2 : 0;
    const int nb = nba > nbb ? nba : nbb;
    int64_t nz = 1, na = M * K, nbel = K * N;
    ContractionParams p;
    no_batch(p);
    {
        int64_t stra = M * K, strb = K * N;
        for (int t = nb - 1; t >= 0; --t) {
            const int ia = t - (nb - nba), ib = t - (nb - nbb);
            const int64_t da = ia >= 0 ? a_dims[ia] : 1, db = ib >= 0 ? b_dims[ib] : 1;
            const int64_t dy = (da == 1) ? db : da;
            if (dy > kIntMax) return fail(ONNX_ERR_UNSUPPORTED, "matmul: batch extent above 2^31-1");
            p.bdim[t] = (int)dy;
            p.a_bs[t] = (da == 1) ? 0 : stra;
            p.b_bs[t] = (db == 1) ? 0 : strb;
            stra *= da; strb *= db;
            nz *= dy;
        }
        na = stra; nbel = strb;
        p.nbd = nb;
    }
    if (nz * M * N == 0) return ONNX_OK;
    if (!Y || (K > 0 && (!A || !B))) return fail(ONNX_ERR_NULL, "matmul: A, B and Y must not be NULL");
    const int64_t ny = nz * M * N;
    const int64_t esz = in_type == ONNX_F32 ? 4 : 2, ysz = out_type == ONNX_F32 ? 4 : 2;     // bytes per element
    if (overlaps(Y, ny * ysz, A, na * esz) || overlaps(Y, ny * ysz, B, nbel * esz))
        return fail(ONNX_ERR_ALIAS, "matmul: Y overlaps an input");
    if (M > kIntMax || N > kIntMax || K > kIntMax) return fail(ONNX_ERR_UNSUPPORTED, "matmul: extent above 2^31-1");
    if (!kc_fits(K, K) || !rc_fits(N, kTileRows) || !kc_fits(N, N))
        return fail(ONNX_ERR_UNSUPPORTED, "matmul: a row of A, B or Y is too long for 32-bit tile offsets");

    p.A = A; p.B = B; p.Y = Y; p.bias = nullptr; p.residual = nullptr;
    int64_t Meff = M;
    // When B is shared by every batch entry and A's batch is dense, the whole product is one
    // matrix product with batch*M rows.
    bool b_shared = true, a_dense = true;
    {
        int64_t expect = M * K;
        for (int t = nb - 1; t >= 0; --t) {
            if (p.b_bs[t] != 0 && p.bdim[t] != 1) b_shared = false;
            if (p.bdim[t] != 1 && p.a_bs[t] != expect) a_dense = false;
            expect *= p.bdim[t];
        }
    }
    if (nz > 1 && b_shared && a_dense && nz * M <= kIntMax) {
        Meff = nz * M;
        nz = 1;
        p.nbd = 0;
    }
    if (nz > 32768LL * 65535LL) return fail(ONNX_ERR_UNSUPPORTED, "matmul: too many batch entries");
    p.M = (int)Meff; p.N = (int)N; p.K = (int)K;
    p.a_ld = K; p.b_ld = N; p.y_rs = N; p.y_zs = M * N;
    p.alpha = 1.f; p.beta = 0.f; p.bias_mode = BIAS_NONE; p.bias_cs = 0; p.relu = 0;
    if (in_type != ONNX_F32) {
        const int bvec = lp_tuned_fits(p, LOAD_KC, LOAD_RC, (int)nz);
        if (bvec)
            return device_status(launch_lp_tuned(p, LOAD_RC, bvec, (int)nz, (int)in_type, (int)out_type, workspace(),
                                                 static_cast<hipStream_t>(stream)), "matmul (16-bit)");
        return device_status(launch_lp_generic(p, LOAD_KC, LOAD_RC, (int)nz, (int)in_type, (int)out_type,
                                               static_cast<hipStream_t>(stream)), "matmul (16-bit)");
    }
    const bool a4 = aligned16(A) && K % 4 == 0, b4 = aligned16(B) && N % 4 == 0;
    const int tile = pick_tile(Meff, N, K, nz);
    return device_status(launch_contraction(p, LOAD_KC, LOAD_RC, a4 ? 4 : 1, b4 ? 4 : 1, tile, (int)nz, workspace(),
                                            static_cast<hipStream_t>(stream)), "matmul");
}

}  // namespace

extern "C" {

const char* onnx_last_error(void) { return g_err; }

const char* onnx_last_launch(void) {
    static const char* const kinds[] = {"KC", "RC", "IM2COL", "RCS"};
    const LaunchRecord& r = g_launch;
    if (!r.family) return "";
    snprintf(g_launch_text, sizeof(g_launch_text), "%s %dx%dx%d waves %dx%dx%d A=%s/%d B=%s/%d npb=%d ksplit=%d tail=%dx%d",
             r.family, r.bm, r.bn, r.bk, r.wm, r.wn, r.ks, kinds[r.akind & 3], r.avec, kinds[r.bkind & 3], r.bvec, r.npb,
             r.ksplit, r.tail_tiles, r.tail_split);
    return g_launch_text;
}

onnx_status onnx_set_workspace(void* device_ptr, size_t bytes) {
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    g_ws = Workspace{nullptr, 0};
    if (!device_ptr || bytes == 0) return ONNX_OK;
    if ((reinterpret_cast<uintptr_t>(device_ptr) & 255u) != 0)
        return fail(ONNX_ERR_ATTR, "workspace: the pointer must be 256-byte aligned");
    if (bytes < (1u << 20)) return fail(ONNX_ERR_ATTR, "workspace: at least 1 MiB is needed");
    g_ws.partial = static_cast<float*>(device_ptr);
    g_ws.partial_floats = (int64_t)(bytes / sizeof(float));
    return ONNX_OK;
}

onnx_status onnx_conv_infer(const int64_t x[4], const int64_t w[4], const int64_t pads[4],
                            const int64_t strides[2], const int64_t dil[2], int64_t group, int64_t y[4]) {
    if (!x || !w || !pads || !strides || !dil || !y) return fail(ONNX_ERR_NULL, "conv: NULL dims/attribute array");
    for (int i = 0; i < 4; ++i)
        if (x[i] < 0 || w[i] < 0) return fail(ONNX_ERR_SHAPE, "conv: negative dimension");
    if (strides[0] < 1 || strides[1] < 1 || dil[0] < 1 || dil[1] < 1)
        return fail(ONNX_ERR_ATTR, "conv: strides and dilations must be >= 1");
    for (int i = 0; i < 4; ++i)
        if (pads[i] < 0) return fail(ONNX_ERR_ATTR, "conv: pads must be >= 0");
    if (group < 1) return fail(ONNX_ERR_ATTR, "conv: group must be >= 1");
    if (w[2] < 1 || w[3] < 1) return fail(ONNX_ERR_SHAPE, "conv: kernel extent must be >= 1");
    if (x[1] % group || w[0] % group || w[1] * group != x[1])
        return fail(ONNX_ERR_SHAPE, "conv: group %lld must divide C=%lld and M=%lld, and W dim 1 (%lld) must be C/group",
                    (long long)group, (long long)x[1], (long long)w[0], (long long)w[1]);
    int64_t oh, ow;
    if (!window_extent(x[2], w[2], pads[0], pads[2], strides[0], dil[0], 0, &oh) ||
        !window_extent(x[3], w[3], pads[1], pads[3], strides[1], dil[1], 0, &ow))
        return fail(ONNX_ERR_SHAPE, "conv: dilated kernel larger than the padded input");
    y[0] = x[0]; y[1] = w[0]; y[2] = oh; y[3] = ow;
    return ONNX_OK;
}

onnx_status onnx_pool_infer(const int64_t x[4], const int64_t kernel[2], const int64_t pads[4],
                            const int64_t strides[2], const int64_t dil[2], int ceil_mode, int64_t y[4]) {
    if (!x || !kernel || !pads || !strides || !y) return fail(ONNX_ERR_NULL, "pool: NULL dims/attribute array");
    const int64_t d0 = dil ? dil[0] : 1, d1 = dil ? dil[1] : 1;
    for (int i = 0; i < 4; ++i)
        if (x[i] < 0) return fail(ONNX_ERR_SHAPE, "pool: negative dimension");
    if (kernel[0] < 1 || kernel[1] < 1 || strides[0] < 1 || strides[1] < 1 || d0 < 1 || d1 < 1)
        return fail(ONNX_ERR_ATTR, "pool: kernel, strides and dilations must be >= 1");
    for (int i = 0; i < 4; ++i)
        if (pads[i] < 0) return fail(ONNX_ERR_ATTR, "pool: pads must be >= 0");
    const int64_t e0 = (kernel[0] - 1) * d0 + 1, e1 = (kernel[1] - 1) * d1 + 1;
    if (pads[0] >= e0 || pads[2] >= e0 || pads[1] >= e1 || pads[3] >= e1)
        return fail(ONNX_ERR_ATTR, "pool: each pad must be smaller than the (dilated) window");
    int64_t oh, ow;
    if (!window_extent(x[2], kernel[0], pads[0], pads[2], strides[0], d0, ceil_mode, &oh) ||
        !window_extent(x[3], kernel[1], pads[1], pads[3], strides[1], d1, ceil_mode, &ow))
        return fail(ONNX_ERR_SHAPE, "pool: window larger than the padded input");
    y[0] = x[0]; y[1] = x[1]; y[2] = oh; y[3] = ow;
    return ONNX_OK;
}

onnx_status onnx_matmul_infer(const int64_t* a, int ra, const int64_t* b, int rb, int64_t* y, int* ry) {
    if (!a || !b || !y || !ry) return fail(ONNX_ERR_NULL, "matmul: NULL dims array");
    if (ra < 1 || rb < 1 || ra > ONNX_MAX_RANK || rb > ONNX_MAX_RANK)
        return fail(ONNX_ERR_RANK, "matmul: ranks must be in 1..%d", ONNX_MAX_RANK);
    for (int i = 0; i < ra; ++i) if (a[i] < 0) return fail(ONNX_ERR_SHAPE, "matmul: negative dimension");
    for (int i = 0; i < rb; ++i) if (b[i] < 0) return fail(ONNX_ERR_SHAPE, "matmul: negative dimension");
    const int64_t K = a[ra - 1];
    const int64_t Kb = rb == 1 ? b[0] : b[rb - 2];
    if (K != Kb) return fail(ONNX_ERR_SHAPE, "matmul: inner dimensions differ (%lld vs %lld)", (long long)K, (long long)Kb);
    const int nba = ra >= 2 ? ra - 2 : 0, nbb = rb >= 2 ? rb - 2 : 0;
    const int nb = nba > nbb ? nba : nbb;
    int r = 0;
    for (int t = 0; t < nb; ++t) {
        const int ia = t - (nb - nba), ib = t - (nb - nbb);
        const int64_t da = ia >= 0 ? a[ia] : 1, db = ib >= 0 ? b[ib] : 1;
        if (da != db && da != 1 && db != 1)
            return fail(ONNX_ERR_SHAPE, "matmul: batch dimensions %lld and %lld do not broadcast", (long long)da, (long long)db);
        y[r++] = (da == 1) ? db : da;
    }
    if (ra >= 2) y[r++] = a[ra - 2];
    if (rb >= 2) y[r++] = b[rb - 1];
    *ry = r;
    return ONNX_OK;
}

onnx_status onnx_conv(const float* X, const int64_t x_dims[4], const float* W, const int64_t w_dims[4],
                      const float* B, const int64_t pads[4], const int64_t strides[2],
                      const int64_t dilations[2], int64_t group, const float* residual, onnx_act act,
                      float* Y, const int64_t y_dims[4], void* stream) {
    const Workspace ws = workspace();
    return conv_with_workspace(X, x_dims, W, w_dims, B, pads, strides, dilations, group, residual, act, Y, y_dims,
                               &ws, 0, stream);
}

onnx_status onnx_conv_fixed_scratch(const float* X, const int64_t x_dims[4], const float* W, const int64_t w_dims[4],
                                    const float* B, const int64_t pads[4], const int64_t strides[2],
                                    const int64_t dilations[2], int64_t group, const float* residual, onnx_act act,
                                    float* Y, const int64_t y_dims[4], void* stream) {
    return conv_with_workspace(X, x_dims, W, w_dims, B, pads, strides, dilations, group, residual, act, Y, y_dims,
                               nullptr, ONNX_CONV_FIXED_SCRATCH_MAX_OUTPUTS, stream);
}

onnx_status onnx_gemm(const float* A, const int64_t a_dims[2], const float* B, const int64_t b_dims[2],
                      const float* C, const int64_t* c_dims, int c_rank, float alpha, float beta,
                      int transA, int transB, onnx_act act, float* Y, const int64_t y_dims[2],
                      void* stream) {
    if (!a_dims || !b_dims || !y_dims) return fail(ONNX_ERR_NULL, "gemm: NULL dims array");
    for (int i = 0; i < 2; ++i)
        if (a_dims[i] < 0 || b_dims[i] < 0) return fail(ONNX_ERR_SHAPE, "gemm: negative dimension");
    const int64_t M = transA ? a_dims[1] : a_dims[0], K = transA ? a_dims[0] : a_dims[1];
    const int64_t Kb = transB ? b_dims[1] : b_dims[0], N = transB ? b_dims[0] : b_dims[1];
    if (K != Kb) return fail(ONNX_ERR_SHAPE, "gemm: inner dimensions differ (%lld vs %lld)", (long long)K, (long long)Kb);
    if (y_dims[0] != M || y_dims[1] != N)
        return fail(ONNX_ERR_SHAPE, "gemm: y_dims is {%lld,%lld} but the result is {%lld,%lld}",
                    (long long)y_dims[0], (long long)y_dims[1], (long long)M, (long long)N);
    if (act != ONNX_ACT_NONE && act != ONNX_ACT_RELU) return fail(ONNX_ERR_ATTR, "gemm: unknown activation");
    int64_t crs = 0, ccs = 0, nc = 0;
    if (C) {
        int64_t r = 1, c = 1;
        if (c_rank < 0 || c_rank > 2) return fail(ONNX_ERR_RANK, "gemm: C must have rank 0, 1 or 2");
        if (c_rank > 0 && !c_dims) return fail(ONNX_ERR_NULL, "gemm: c_dims is NULL");
        if (c_rank == 1) c = c_dims[0];
        if (c_rank == 2) { r = c_dims[0]; c = c_dims[1]; }
        if (!((r == 1 || r == M) && (c == 1 || c == N)))
            return fail(ONNX_ERR_SHAPE, "gemm: C {%lld,%lld} does not broadcast to {%lld,%lld}", (long long)r,
                        (long long)c, (long long)M, (long long)N);
        crs = (r == 1) ? 0 : c;
        ccs = (c == 1) ? 0 : 1;
        nc = r * c;
    }
    if (M * N == 0) return ONNX_OK;
    // with K == 0 the sum is empty and A, B are never read (they may be NULL)
    if (!Y || (K > 0 && (!A || !B))) return fail(ONNX_ERR_NULL, "gemm: A, B and Y must not be NULL");
    if (overlaps(Y, M * N * 4, A, M * K * 4) || overlaps(Y, M * N * 4, B, K * N * 4) ||
        overlaps(Y, M * N * 4, C, nc * 4))
        return fail(ONNX_ERR_ALIAS, "gemm: Y overlaps an input");
    if (M > kIntMax || N > kIntMax || K > kIntMax) return fail(ONNX_ERR_UNSUPPORTED, "gemm: extent above 2^31-1");
    if (!(transA ? rc_fits(M, kTileRows) : kc_fits(K, K)) || !(transB ? kc_fits(K, K) : rc_fits(N, kTileRows)) ||
        !kc_fits(N, N))
        return fail(ONNX_ERR_UNSUPPORTED, "gemm: a row of A, B or Y is too long for 32-bit tile offsets");

    ContractionParams p;
    no_batch(p);
    p.A = A; p.B = B; p.Y = Y; p.bias = C; p.residual = nullptr;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.a_ld = a_dims[1];
    p.b_ld = b_dims[1];
    p.y_rs = N;
    p.alpha = alpha; p.beta = beta; p.relu = act == ONNX_ACT_RELU;
    // C broadcast: {M,N} is laid out like Y; {M,1} is one value per row; everything else one per column
    p.bias_mode = (crs != 0 && ccs != 0) ? BIAS_FULL : (crs != 0 ? BIAS_ROW : BIAS_COL);
    p.bias_cs = (int)ccs;
    const int akind = transA ? LOAD_RC : LOAD_KC;
    const int bkind = transB ? LOAD_KC : LOAD_RC;
    // 16-byte loads of an operand need an aligned base and every row start a multiple of 4
    const bool a4 = aligned16(A) && a_dims[1] % 4 == 0;
    const bool b4 = aligned16(B) && b_dims[1] % 4 == 0;
    const int tile = pick_tile(M, N, K, 1);
    return device_status(launch_contraction(p, akind, bkind, a4 ? 4 : 1, b4 ? 4 : 1, tile, 1, workspace(),
                                            static_cast<hipStream_t>(stream)), "gemm");
}

onnx_status onnx_matmul(const float* A, const int64_t* a_dims, int a_rank, const float* B,
                        const int64_t* b_dims, int b_rank, float* Y, const int64_t* y_dims, int y_rank,
                        void* stream) {
    return matmul_any(A, a_dims, a_rank, B, b_dims, b_rank, Y, y_dims, y_rank, ONNX_F32, ONNX_F32, stream);
}

onnx_status onnx_matmul_lp(const void* A, const int64_t* a_dims, int a_rank, const void* B, const int64_t* b_dims,
                           int b_rank, void* Y, const int64_t* y_dims, int y_rank, onnx_dtype in_type,
                           onnx_dtype out_type, void* stream) {
    if (in_type != ONNX_F16 && in_type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "matmul_lp: in_type must be ONNX_F16 or ONNX_BF16");
    if (out_type != ONNX_F32 && out_type != in_type) return fail(ONNX_ERR_ATTR, "matmul_lp: out_type must be ONNX_F32 or in_type");
    return matmul_any(static_cast<const float*>(A), a_dims, a_rank, static_cast<const float*>(B), b_dims, b_rank,
                      static_cast<float*>(Y), y_dims, y_rank, in_type, out_type, stream);
}

onnx_status onnx_conv_lp_filter_taps(const void* W, const int64_t w_dims[4], void* packed, void* stream) {
    if (!w_dims) return fail(ONNX_ERR_NULL, "conv_lp_filter_taps: NULL dims array");
    for (int i = 0; i < 4; ++i)
        if (w_dims[i] < 0) return fail(ONNX_ERR_SHAPE, "conv_lp_filter_taps: negative dimension");
    if (w_dims[2] != 3 || w_dims[3] != 3 || w_dims[1] % 16 != 0 || w_dims[1] > kIntMax)
        return fail(ONNX_ERR_UNSUPPORTED, "conv_lp_filter_taps: W must be [M, C/group, 3, 3] with C/group a multiple of 16");
    const int64_t n = w_dims[0] * w_dims[1] * 9;
    if (n == 0) return ONNX_OK;
    if (!W || !packed) return fail(ONNX_ERR_NULL, "conv_lp_filter_taps: W and packed must not be NULL");
    if ((reinterpret_cast<uintptr_t>(packed) & 15u) != 0) return fail(ONNX_ERR_ATTR, "conv_lp_filter_taps: packed must be 16-byte aligned");
    if (overlaps(packed, n * 2, W, n * 2)) return fail(ONNX_ERR_ALIAS, "conv_lp_filter_taps: packed overlaps W");
    return device_status(launch_lp_filter_taps(W, packed, w_dims[0], (int)w_dims[1], static_cast<hipStream_t>(stream)),
                         "conv_lp_filter_taps");
}

onnx_status onnx_conv_lp_taps(const void* X, const int64_t x_dims[4], const void* packed, const int64_t w_dims[4], const float* B,
                              const int64_t pads[4], const int64_t strides[2], const int64_t dilations[2], int64_t group,
                              const void* residual, onnx_act act, void* Y, const int64_t y_dims[4], onnx_dtype in_type,
                              onnx_dtype out_type, void* stream) {
    if (in_type != ONNX_F16 && in_type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "conv_lp_taps: in_type must be ONNX_F16 or ONNX_BF16");
    if (out_type != ONNX_F32 && out_type != in_type) return fail(ONNX_ERR_ATTR, "conv_lp_taps: out_type must be ONNX_F32 or in_type");
    if (packed && (reinterpret_cast<uintptr_t>(packed) & 15u) != 0)
        return fail(ONNX_ERR_ATTR, "conv_lp_taps: the rewritten filter bank must be 16-byte aligned");
    const Workspace ws = workspace();      // only for split-K shares, when the output has few tiles
    return conv_with_workspace(static_cast<const float*>(X), x_dims, static_cast<const float*>(packed), w_dims, B, pads, strides,
                               dilations, group, static_cast<const float*>(residual), act, static_cast<float*>(Y), y_dims,
                               &ws, 0, stream, in_type, out_type, true);
}

onnx_status onnx_conv_lp(const void* X, const int64_t x_dims[4], const void* W, const int64_t w_dims[4], const float* B,
                         const int64_t pads[4], const int64_t strides[2], const int64_t dilations[2], int64_t group,
                         const void* residual, onnx_act act, void* Y, const int64_t y_dims[4], onnx_dtype in_type,
                         onnx_dtype out_type, void* stream) {
    if (in_type != ONNX_F16 && in_type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "conv_lp: in_type must be ONNX_F16 or ONNX_BF16");
    if (out_type != ONNX_F32 && out_type != in_type) return fail(ONNX_ERR_ATTR, "conv_lp: out_type must be ONNX_F32 or in_type");
    const Workspace ws = workspace();      // the tuned 3x3 kernel keeps its rewritten filter bank there
    return conv_with_workspace(static_cast<const float*>(X), x_dims, static_cast<const float*>(W), w_dims, B, pads, strides,
                               dilations, group, static_cast<const float*>(residual), act, static_cast<float*>(Y), y_dims,
                               &ws, 0, stream, in_type, out_type);
}

}  // extern "C"

namespace {

// ONNX MaxPool on fp32 tensors (type ONNX_F32, optional Indices) or on 16-bit tensors (no Indices).
onnx_status maxpool_any(const void* X, const int64_t x_dims[4], const int64_t kernel[2],
                        const int64_t pads[4], const int64_t strides[2], const int64_t dilations[2],
                        int ceil_mode, void* Y, int64_t* Indices, const int64_t y_dims[4], onnx_dtype type, void* stream) {
    if (!x_dims || !y_dims) return fail(ONNX_ERR_NULL, "maxpool: NULL dims array");
    const int64_t esz = type == ONNX_F32 ? 4 : 2;
    int64_t yd[4];
    const onnx_status st = onnx_pool_infer(x_dims, kernel, pads, strides, dilations, ceil_mode, yd);
    if (st != ONNX_OK) return st;
    for (int i = 0; i < 4; ++i)
        if (yd[i] != y_dims[i])
            return fail(ONNX_ERR_SHAPE, "maxpool: y_dims[%d]=%lld but the inferred extent is %lld", i,
                        (long long)y_dims[i], (long long)yd[i]);
    const int64_t ny = yd[0] * yd[1] * yd[2] * yd[3], nx = x_dims[0] * x_dims[1] * x_dims[2] * x_dims[3];
    if (ny == 0) return ONNX_OK;
    if (!X || !Y) return fail(ONNX_ERR_NULL, "maxpool: X and Y must not be NULL");
    if (overlaps(Y, ny * esz, X, nx * esz) || overlaps(Indices, ny * 8, X, nx * esz) || overlaps(Indices, ny * 8, Y, ny * esz))
        return fail(ONNX_ERR_ALIAS, "maxpool: outputs overlap X or each other");
    const int64_t d0 = dilations ? dilations[0] : 1, d1 = dilations ? dilations[1] : 1;
    if (x_dims[2] * x_dims[3] > kIntMax || x_dims[0] > kIntMax || x_dims[1] > kIntMax ||
        x_dims[1] * yd[2] * yd[3] >= (1LL << 30) || kernel[0] * d0 > kIntMax || kernel[1] * d1 > kIntMax ||
        strides[0] > kIntMax || strides[1] > kIntMax)
        return fail(ONNX_ERR_UNSUPPORTED, "maxpool: one image exceeds the 32-bit index range");
    WindowGeom g;
    g.N = (int)x_dims[0]; g.C = (int)x_dims[1]; g.H = (int)x_dims[2]; g.W = (int)x_dims[3];
    g.OH = (int)yd[2]; g.OW = (int)yd[3]; g.kH = (int)kernel[0]; g.kW = (int)kernel[1];
    g.sH = (int)strides[0]; g.sW = (int)strides[1]; g.pT = (int)pads[0]; g.pL = (int)pads[1];
    g.pB = (int)pads[2]; g.pR = (int)pads[3]; g.dH = (int)d0; g.dW = (int)d1;
    if (type != ONNX_F32) {
        if (ny > kIntMax) return fail(ONNX_ERR_UNSUPPORTED, "maxpool (16-bit): more than 2^31-1 output elements");
        return device_status(launch_maxpool_lp(X, Y, g, (int)type, static_cast<hipStream_t>(stream)), "maxpool (16-bit)");
    }
    return device_status(launch_maxpool(static_cast<const float*>(X), static_cast<float*>(Y), Indices, g,
                                        static_cast<hipStream_t>(stream)), "maxpool");
}

// ONNX AveragePool / GlobalAveragePool on fp32 or 16-bit tensors.
onnx_status avgpool_any(const void* X, const int64_t x_dims[4], const int64_t* kernel, const int64_t* pads,
                        const int64_t* strides, int ceil_mode, int count_include_pad, void* Y,
                        const int64_t y_dims[4], onnx_dtype type, void* stream) {
    if (!x_dims || !y_dims) return fail(ONNX_ERR_NULL, "avgpool: NULL dims array");
    const int64_t esz = type == ONNX_F32 ? 4 : 2;
    for (int i = 0; i < 4; ++i)
        if (x_dims[i] < 0) return fail(ONNX_ERR_SHAPE, "avgpool: negative dimension");
    const int64_t nx = x_dims[0] * x_dims[1] * x_dims[2] * x_dims[3];
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!kernel) {
        if (x_dims[2] * x_dims[3] == 0 && x_dims[0] * x_dims[1] != 0)
            return fail(ONNX_ERR_SHAPE, "avgpool: global pool over an empty plane");
        if (y_dims[0] != x_dims[0] || y_dims[1] != x_dims[1] || y_dims[2] != 1 || y_dims[3] != 1)
            return fail(ONNX_ERR_SHAPE, "avgpool: a global pool yields {N,C,1,1}");
        const int64_t planes = x_dims[0] * x_dims[1];
        if (planes == 0) return ONNX_OK;
        if (!X || !Y) return fail(ONNX_ERR_NULL, "avgpool: X and Y must not be NULL");
        if (overlaps(Y, planes * esz, X, nx * esz)) return fail(ONNX_ERR_ALIAS, "avgpool: Y overlaps X");
        if (x_dims[2] * x_dims[3] > kIntMax) return fail(ONNX_ERR_UNSUPPORTED, "avgpool: plane above 2^31-1 elements");
        if (type != ONNX_F32)
            return device_status(launch_global_avgpool_lp(X, Y, planes, (int)(x_dims[2] * x_dims[3]), (int)type, s),
                                 "avgpool (global, 16-bit)");
        return device_status(launch_global_avgpool(static_cast<const float*>(X), static_cast<float*>(Y), planes,
                                                   (int)(x_dims[2] * x_dims[3]), s), "avgpool (global)");
    }
    const int64_t zero4[4] = {0, 0, 0, 0}, one2[2] = {1, 1};
    if (!pads) pads = zero4;
    if (!strides) strides = one2;
    int64_t yd[4];
    const onnx_status st = onnx_pool_infer(x_dims, kernel, pads, strides, nullptr, ceil_mode, yd);
    if (st != ONNX_OK) return st;
    for (int i = 0; i < 4; ++i)
        if (yd[i] != y_dims[i])
            return fail(ONNX_ERR_SHAPE, "avgpool: y_dims[%d]=%lld but the inferred extent is %lld", i,
                        (long long)y_dims[i], (long long)yd[i]);
    const int64_t ny = yd[0] * yd[1] * yd[2] * yd[3];
    if (ny == 0) return ONNX_OK;
    if (!X || !Y) return fail(ONNX_ERR_NULL, "avgpool: X and Y must not be NULL");
    if (overlaps(Y, ny * esz, X, nx * esz)) return fail(ONNX_ERR_ALIAS, "avgpool: Y overlaps X");
    if (x_dims[2] * x_dims[3] > kIntMax || x_dims[0] > kIntMax || x_dims[1] > kIntMax ||
        x_dims[1] * yd[2] * yd[3] >= (1LL << 30) || kernel[0] > kIntMax || kernel[1] > kIntMax ||
        strides[0] > kIntMax || strides[1] > kIntMax)
        return fail(ONNX_ERR_UNSUPPORTED, "avgpool: one image exceeds the 32-bit index range");
    WindowGeom g;
    g.N = (int)x_dims[0]; g.C = (int)x_dims[1]; g.H = (int)x_dims[2]; g.W = (int)x_dims[3];
    g.OH = (int)yd[2]; g.OW = (int)yd[3]; g.kH = (int)kernel[0]; g.kW = (int)kernel[1];
    g.sH = (int)strides[0]; g.sW = (int)strides[1]; g.pT = (int)pads[0]; g.pL = (int)pads[1];
    g.pB = (int)pads[2]; g.pR = (int)pads[3]; g.dH = 1; g.dW = 1;
    if (type != ONNX_F32) {
        if (ny > kIntMax) return fail(ONNX_ERR_UNSUPPORTED, "avgpool (16-bit): more than 2^31-1 output elements");
        return device_status(launch_avgpool_lp(X, Y, g, count_include_pad, (int)type, s), "avgpool (16-bit)");
    }
    return device_status(launch_avgpool(static_cast<const float*>(X), static_cast<float*>(Y), g, count_include_pad, s), "avgpool");
}

}  // namespace

extern "C" {

onnx_status onnx_maxpool(const float* X, const int64_t x_dims[4], const int64_t kernel[2],
                         const int64_t pads[4], const int64_t strides[2], const int64_t dilations[2],
                         int ceil_mode, float* Y, int64_t* Indices, const int64_t y_dims[4], void* stream) {
    return maxpool_any(X, x_dims, kernel, pads, strides, dilations, ceil_mode, Y, Indices, y_dims, ONNX_F32, stream);
}

onnx_status onnx_avgpool(const float* X, const int64_t x_dims[4], const int64_t* kernel, const int64_t* pads,
                         const int64_t* strides, int ceil_mode, int count_include_pad, float* Y,
                         const int64_t y_dims[4], void* stream) {
    return avgpool_any(X, x_dims, kernel, pads, strides, ceil_mode, count_include_pad, Y, y_dims, ONNX_F32, stream);
}

onnx_status onnx_maxpool_lp(const void* X, const int64_t x_dims[4], const int64_t kernel[2],
                            const int64_t pads[4], const int64_t strides[2], const int64_t dilations[2],
                            int ceil_mode, void* Y, const int64_t y_dims[4], onnx_dtype type, void* stream) {
    if (type != ONNX_F16 && type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "maxpool_lp: type must be ONNX_F16 or ONNX_BF16");
    return maxpool_any(X, x_dims, kernel, pads, strides, dilations, ceil_mode, Y, nullptr, y_dims, type, stream);
}

onnx_status onnx_leakyrelu_lp(const void* X, int64_t count, float alpha, void* Y, onnx_dtype type, void* stream) {
    if (type != ONNX_F16 && type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "leakyrelu_lp: type must be ONNX_F16 or ONNX_BF16");
    if (count < 0) return fail(ONNX_ERR_SHAPE, "leakyrelu_lp: negative element count");
    if (count == 0) return ONNX_OK;
    if (!X || !Y) return fail(ONNX_ERR_NULL, "leakyrelu_lp: X and Y must not be NULL");
    if (overlaps(Y, count * 2, X, count * 2)) return fail(ONNX_ERR_ALIAS, "leakyrelu_lp: Y overlaps X");
    return device_status(launch_leakyrelu_lp(X, Y, count, alpha, (int)type, static_cast<hipStream_t>(stream)), "leakyrelu_lp");
}

onnx_status onnx_avgpool_lp(const void* X, const int64_t x_dims[4], const int64_t* kernel, const int64_t* pads,
                            const int64_t* strides, int ceil_mode, int count_include_pad, void* Y,
                            const int64_t y_dims[4], onnx_dtype type, void* stream) {
    if (type != ONNX_F16 && type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "avgpool_lp: type must be ONNX_F16 or ONNX_BF16");
    return avgpool_any(X, x_dims, kernel, pads, strides, ceil_mode, count_include_pad, Y, y_dims, type, stream);
}

}  // extern "C"
