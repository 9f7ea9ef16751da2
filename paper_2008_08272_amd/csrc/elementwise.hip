// Element-wise, reduction and softmax operators: ONNX Add (the paper's running example,
// Section 3), Relu / LeakyRelu (the operator definition shown in Section 3.1), Abs and ReduceSum
// (the two operators ReduceL1 decomposes into, Section 3.4) and Softmax.  All of them move
// every element once and do next to no arithmetic: they are bound by HBM bandwidth, so the
// kernels are about coalesced 16-byte accesses and enough independent loads in flight.
// This file holds the kernels and their C-ABI entry points.
#include <stdio.h>

#include "../../include/onnxhip.h"
#include "gemm_lp.h"
#include "internal.h"

using namespace onnxhip;

namespace {

constexpr int EW_MAX_DIMS = ONNX_MAX_RANK;
const int64_t kMaxElems = 0x7fffffffLL;

#define fail(st, ...) static_cast<onnx_status>(fail_with((st), __VA_ARGS__))

onnx_status device_status(hipError_t e, const char* what) {
    if (e == hipSuccess) return ONNX_OK;
    return fail(ONNX_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

unsigned blocks_for(int64_t work_items, int per_block = 256, unsigned cap = 256u * 32u) {
    const int64_t b = (work_items + per_block - 1) / per_block;
    return (unsigned)(b < 1 ? 1 : (b > cap ? cap : b));
}

// Storage types of the reductions and of Softmax: DT = 0 is fp32, LP_F16 / LP_BF16 the 16-bit types; arithmetic is
// fp32 for all of them, a 16-bit result rounded once on the way out.
template <int DT>
struct Elem {
    typedef uint16_t type;
    static __device__ inline float load(const uint16_t* p) { return from_lp<DT>(*p); }
    static __device__ inline void store(uint16_t* p, float v) { *p = to_lp<DT>(v); }
};
template <>
struct Elem<0> {
    typedef float type;
    static __device__ inline float load(const float* p) { return *p; }
    static __device__ inline void store(float* p, float v) { *p = v; }
};

template <int DT>
__global__ __launch_bounds__(256) void fill_kernel(typename Elem<DT>::type* __restrict__ Y, int64_t n, float v) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) Elem<DT>::store(Y + i, v);
}

// ---------------------------------------------------------------------------- unary

enum UnaryOp { UN_RELU = 0, UN_LEAKY = 1, UN_ABS = 2 };

template <int OP>
__device__ inline float unary(float x, float alpha) {
    if (OP == UN_RELU) return x > 0.f ? x : 0.f;
    if (OP == UN_LEAKY) return x >= 0.f ? x : alpha * x;
    return fabsf(x);
}

// Grid-stride over 16-byte groups; `tail` elements after the last full group go one by one.
template <int OP, bool VEC4>
__global__ __launch_bounds__(256) void unary_kernel(const float* __restrict__ X, float* __restrict__ Y,
                                                    int64_t n, float alpha) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (VEC4) {
        const int64_t n4 = n >> 2;
        const floatx4* x4 = reinterpret_cast<const floatx4*>(X);
        floatx4* y4 = reinterpret_cast<floatx4*>(Y);
        for (int64_t j = i; j < n4; j += stride) {
            floatx4 v = x4[j];
            v.x = unary<OP>(v.x, alpha); v.y = unary<OP>(v.y, alpha);
            v.z = unary<OP>(v.z, alpha); v.w = unary<OP>(v.w, alpha);
            y4[j] = v;
        }
        for (int64_t j = (n4 << 2) + i; j < n; j += stride) Y[j] = unary<OP>(X[j], alpha);
    } else {
        for (; i < n; i += stride) Y[i] = unary<OP>(X[i], alpha);
    }
}

template <int OP>
onnx_status run_unary(const char* name, const float* X, int64_t count, float alpha, float* Y, void* stream) {
    if (count < 0) return fail(ONNX_ERR_SHAPE, "%s: negative element count", name);
    if (count == 0) return ONNX_OK;
    if (!X || !Y) return fail(ONNX_ERR_NULL, "%s: X and Y must not be NULL", name);
    if (overlaps(Y, count * 4, X, count * 4)) return fail(ONNX_ERR_ALIAS, "%s: Y overlaps X", name);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (aligned16(X) && aligned16(Y))
        hipLaunchKernelGGL((unary_kernel<OP, true>), dim3(blocks_for((count + 3) / 4)), dim3(256), 0, s, X, Y, count, alpha);
    else
        hipLaunchKernelGGL((unary_kernel<OP, false>), dim3(blocks_for(count)), dim3(256), 0, s, X, Y, count, alpha);
    return device_status(hipGetLastError(), name);
}

// Abs on 16-bit elements of either type: the sign bit cleared, 8 elements per 16-byte access (VEC = 8) or one.
template <int VEC>
__global__ __launch_bounds__(256) void abs_lp_kernel(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int64_t count) {
    for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC; i < count; i += (int64_t)gridDim.x * 256 * VEC) {
        if constexpr (VEC == 8) {
            uintx4 v = *reinterpret_cast<const uintx4*>(X + i);
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] &= 0x7fff7fffu;
            *reinterpret_cast<uintx4*>(Y + i) = v;
        } else {
            Y[i] = X[i] & 0x7fffu;
        }
    }
}

// ---------------------------------------------------------------------------- broadcasting Add

// Output index space after merging: up to EW_MAX_DIMS extents, row-major, with the element
// stride of each operand per extent (0 where the operand is broadcast along it).
struct BroadcastMap {
    int nd;
    FastDiv dim[EW_MAX_DIMS];       // dim[nd-1] is the innermost extent, in groups of VEC elements
    int64_t sa[EW_MAX_DIMS], sb[EW_MAX_DIMS];
};

// One thread per group of VEC consecutive innermost outputs.  An operand whose innermost
// stride is 1 is read with one (16-byte when VEC = 4) load, one whose stride is 0 with a
// single scalar load that all VEC outputs share.
template <int VEC>
__global__ __launch_bounds__(256) void add_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                  float* __restrict__ Y, uint32_t groups, BroadcastMap m) {
    for (uint32_t gidx = blockIdx.x * 256u + threadIdx.x; gidx < groups; gidx += gridDim.x * 256u) {
        uint32_t rest = gidx, i;
        int64_t oa = 0, ob = 0;
        for (int d = m.nd - 1; d >= 0; --d) {
            m.dim[d].divmod(rest, rest, i);
            const int64_t step = (d == m.nd - 1) ? (int64_t)i * VEC : (int64_t)i;
            oa += step * m.sa[d];
            ob += step * m.sb[d];
        }
        const bool ca = m.sa[m.nd - 1] != 0, cb = m.sb[m.nd - 1] != 0;
        float a[VEC], b[VEC];
        if (VEC == 4) {
            if (ca) { const floatx4 v = *reinterpret_cast<const floatx4*>(A + oa); a[0] = v.x; a[1] = v.y; a[2] = v.z; a[3] = v.w; }
            else { const float v = A[oa]; a[0] = a[1] = a[2] = a[3] = v; }
            if (cb) { const floatx4 v = *reinterpret_cast<const floatx4*>(B + ob); b[0] = v.x; b[1] = v.y; b[2] = v.z; b[3] = v.w; }
            else { const float v = B[ob]; b[0] = b[1] = b[2] = b[3] = v; }
            floatx4 y = {a[0] + b[0], a[1] + b[1], a[2] + b[2], a[3] + b[3]};
            *reinterpret_cast<floatx4*>(Y + (int64_t)gidx * 4) = y;
        } else {
            Y[gidx] = A[oa] + B[ob];
        }
    }
}

// The same on 16-bit tensors (DT: LP_F16 / LP_BF16): groups of 8 innermost outputs through 16-byte
// accesses (VEC = 8) or single elements; the sum is taken in fp32 and rounded to the type.
template <int DT, int VEC>
__global__ __launch_bounds__(256) void add_lp_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                                     uint16_t* __restrict__ Y, uint32_t groups, BroadcastMap m) {
    for (uint32_t gidx = blockIdx.x * 256u + threadIdx.x; gidx < groups; gidx += gridDim.x * 256u) {
        uint32_t rest = gidx, i;
        int64_t oa = 0, ob = 0;
        for (int d = m.nd - 1; d >= 0; --d) {
            m.dim[d].divmod(rest, rest, i);
            const int64_t step = (d == m.nd - 1) ? (int64_t)i * VEC : (int64_t)i;
            oa += step * m.sa[d];
            ob += step * m.sb[d];
        }
        if constexpr (VEC == 8) {
            const bool ca = m.sa[m.nd - 1] != 0, cb = m.sb[m.nd - 1] != 0;
            uintx4 a, b, y;
            if (ca) a = *reinterpret_cast<const uintx4*>(A + oa);
            else { const uint32_t v = A[oa]; a[0] = a[1] = a[2] = a[3] = v | (v << 16); }
            if (cb) b = *reinterpret_cast<const uintx4*>(B + ob);
            else { const uint32_t v = B[ob]; b[0] = b[1] = b[2] = b[3] = v | (v << 16); }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t lo = to_lp<DT>(from_lp<DT>(a[k] & 0xffffu) + from_lp<DT>(b[k] & 0xffffu));
                const uint32_t hi = to_lp<DT>(from_lp<DT>(a[k] >> 16) + from_lp<DT>(b[k] >> 16));
                y[k] = lo | (hi << 16);
            }
            *reinterpret_cast<uintx4*>(Y + (int64_t)gidx * 8) = y;
        } else {
            Y[gidx] = to_lp<DT>(from_lp<DT>(A[oa]) + from_lp<DT>(B[ob]));
        }
    }
}

// numpy-style broadcast of two shapes; false when they are not compatible
bool broadcast_shape(const int64_t* a, int ra, const int64_t* b, int rb, int64_t* y, int* ry) {
    const int r = ra > rb ? ra : rb;
    for (int d = 0; d < r; ++d) {
        const int64_t ea = d < r - ra ? 1 : a[d - (r - ra)], eb = d < r - rb ? 1 : b[d - (r - rb)];
        if (ea != eb && ea != 1 && eb != 1) return false;
        y[d] = ea == 1 ? eb : ea;
    }
    *ry = r;
    return true;
}

// ---------------------------------------------------------------------------- ReduceSum

struct ReduceMap {
    int nk, nr;                               // kept / reduced extents after merging
    FastDiv kdim[EW_MAX_DIMS], rdim[EW_MAX_DIMS];
    int64_t ks[EW_MAX_DIMS], rs[EW_MAX_DIMS]; // element strides in X
    uint32_t outputs, reduced;                // products of the kept / reduced extents
};

__device__ inline int64_t offset_of(uint32_t idx, int n, const FastDiv* dims, const int64_t* strides) {
    int64_t off = 0;
    uint32_t rest = idx, i;
    for (int d = n - 1; d >= 0; --d) {
        dims[d].divmod(rest, rest, i);
        off += (int64_t)i * strides[d];
    }
    return off;
}

// The innermost extent of X is reduced: one wavefront per (output, chunk); its lanes walk the
// chunk of the reduced index space together (coalesced along the innermost extent), each
// keeps a private fp32 sum, and a butterfly adds the 64 of them.  `chunks` > 1 is the first
// stage of a two-stage reduction: it writes chunk sums, chunk-minor, for a second launch.
// DTI / DTO: storage types of X and Y (the chunk sums of a two-stage reduction are fp32 whatever the tensors are).
template <int DTI, int DTO>
__global__ __launch_bounds__(256) void reduce_inner_kernel(const typename Elem<DTI>::type* __restrict__ X,
                                                           typename Elem<DTO>::type* __restrict__ Y, ReduceMap m, uint32_t chunks,
                                                           uint32_t per_chunk) {
    typedef typename Elem<DTI>::type in_t;
    const uint32_t wave = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (wave >= m.outputs * chunks) return;
    const uint32_t out = wave / chunks, chunk = wave - out * chunks;
    const int lane = threadIdx.x & 63;
    const in_t* base = X + offset_of(out, m.nk, m.kdim, m.ks);
    const uint32_t r0 = chunk * per_chunk;
    const uint32_t r1 = min(m.reduced, r0 + per_chunk);
    float acc = 0.f;
    if (m.nr == 1 && m.rs[0] == 1) {
        // contiguous run: scalar head up to a 16-byte boundary, 16-byte loads (EPV elements each) with four
        // independent partial sums per lane (four loads in flight), scalar tail
        constexpr uint32_t EPV = 16 / sizeof(in_t);
        const in_t* p = base + r0;
        const uint32_t n = r1 > r0 ? r1 - r0 : 0u;
        uint32_t head = (uint32_t)((16u - (uint32_t)(reinterpret_cast<uintptr_t>(p) & 15u)) & 15u) / (uint32_t)sizeof(in_t);
        if (head > n) head = n;
        if ((uint32_t)lane < head) acc += Elem<DTI>::load(p + lane);
        const uint32_t nv = (n - head) / EPV;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        uint32_t j = lane;
        if constexpr (DTI == 0) {
            const floatx4* p4 = reinterpret_cast<const floatx4*>(p + head);
            for (; j + 192 < nv; j += 256) {
                const floatx4 v0 = p4[j], v1 = p4[j + 64], v2 = p4[j + 128], v3 = p4[j + 192];
                a0 += (v0.x + v0.y) + (v0.z + v0.w);
                a1 += (v1.x + v1.y) + (v1.z + v1.w);
                a2 += (v2.x + v2.y) + (v2.z + v2.w);
                a3 += (v3.x + v3.y) + (v3.z + v3.w);
            }
            for (; j < nv; j += 64) {
                const floatx4 v = p4[j];
                a0 += (v.x + v.y) + (v.z + v.w);
            }
        } else {
            const uintx4* p8 = reinterpret_cast<const uintx4*>(p + head);
            auto sum8 = [](const uintx4& v) {
                float t[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) t[k] = from_lp<DTI>(v[k] & 0xffffu) + from_lp<DTI>(v[k] >> 16);
                return (t[0] + t[1]) + (t[2] + t[3]);
            };
            for (; j + 192 < nv; j += 256) {
                const uintx4 v0 = p8[j], v1 = p8[j + 64], v2 = p8[j + 128], v3 = p8[j + 192];
                a0 += sum8(v0); a1 += sum8(v1); a2 += sum8(v2); a3 += sum8(v3);
            }
            for (; j < nv; j += 64) a0 += sum8(p8[j]);
        }
        acc += (a0 + a1) + (a2 + a3);
        for (uint32_t t = head + nv * EPV + lane; t < n; t += 64) acc += Elem<DTI>::load(p + t);
    } else if (m.nr == 1) {
        for (uint32_t r = r0 + lane; r < r1; r += 64) acc += Elem<DTI>::load(base + (int64_t)r * m.rs[0]);
    } else {
        for (uint32_t r = r0 + lane; r < r1; r += 64) acc += Elem<DTI>::load(base + offset_of(r, m.nr, m.rdim, m.rs));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) Elem<DTO>::store(Y + wave, acc);
}

// The innermost extent of X is kept: one thread per output, neighbouring threads on
// neighbouring innermost positions, each walks the reduced index space on its own (every step
// is a coalesced row read across the threads).
template <int DT>
__global__ __launch_bounds__(256) void reduce_outer_kernel(const typename Elem<DT>::type* __restrict__ X,
                                                           typename Elem<DT>::type* __restrict__ Y, ReduceMap m) {
    const uint32_t out = blockIdx.x * 256u + threadIdx.x;
    if (out >= m.outputs) return;
    const typename Elem<DT>::type* base = X + offset_of(out, m.nk, m.kdim, m.ks);
    float acc = 0.f;
    if (m.nr == 1) {
        for (uint32_t r = 0; r < m.reduced; ++r) acc += Elem<DT>::load(base + (int64_t)r * m.rs[0]);
    } else {
        for (uint32_t r = 0; r < m.reduced; ++r) acc += Elem<DT>::load(base + offset_of(r, m.nr, m.rdim, m.rs));
    }
    Elem<DT>::store(Y + out, acc);
}

// Normalises `axes` (negative values count from the end; none = all) into a per-dimension flag.
onnx_status reduce_flags(const char* name, int rank, const int64_t* axes, int naxes, bool* reduced) {
    if (rank < 0 || rank > ONNX_MAX_RANK) return fail(ONNX_ERR_RANK, "%s: rank %d outside 0..%d", name, rank, ONNX_MAX_RANK);
    if (naxes < 0 || (naxes > 0 && !axes)) return fail(ONNX_ERR_NULL, "%s: axes missing", name);
    for (int d = 0; d < rank; ++d) reduced[d] = (naxes == 0);
    for (int i = 0; i < naxes; ++i) {
        int64_t a = axes[i];
        if (a < -rank || a >= rank) return fail(ONNX_ERR_ATTR, "%s: axis %lld out of range for rank %d", name, (long long)a, rank);
        if (a < 0) a += rank;
        if (reduced[a]) return fail(ONNX_ERR_ATTR, "%s: axis %lld listed twice", name, (long long)a);
        reduced[a] = true;
    }
    return ONNX_OK;
}

// ---------------------------------------------------------------------------- Softmax

// Softmax over an axis of extent L; `inner` = product of the extents after it.
// inner == 1: one wavefront per row, the row is read once into registers when it is short
// enough (L <= 64 * ROW_REGS), else three passes over it.
constexpr int ROW_REGS = 16;

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int DT>
__global__ __launch_bounds__(256) void softmax_rows_kernel(const typename Elem<DT>::type* __restrict__ X,
                                                           typename Elem<DT>::type* __restrict__ Y, uint32_t rows, uint32_t L) {
    const uint32_t row = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int lane = threadIdx.x & 63;
    const typename Elem<DT>::type* x = X + (int64_t)row * L;
    typename Elem<DT>::type* y = Y + (int64_t)row * L;
    if (L <= 64u * ROW_REGS) {
        float v[ROW_REGS];
        float mx = -__builtin_inff();
#pragma unroll
        for (int i = 0; i < ROW_REGS; ++i) {
            const uint32_t j = lane + 64u * i;
            v[i] = j < L ? Elem<DT>::load(x + j) : -__builtin_inff();
            mx = fmaxf(mx, v[i]);
        }
        mx = wave_max(mx);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < ROW_REGS; ++i) {
            v[i] = expf(v[i] - mx);               // exp(-inf) = 0 for the lanes past the row
            sum += v[i];
        }
        const float inv = 1.0f / wave_sum(sum);
#pragma unroll
        for (int i = 0; i < ROW_REGS; ++i) {
            const uint32_t j = lane + 64u * i;
            if (j < L) Elem<DT>::store(y + j, v[i] * inv);
        }
    } else {
        float mx = -__builtin_inff();
        for (uint32_t j = lane; j < L; j += 64) mx = fmaxf(mx, Elem<DT>::load(x + j));
        mx = wave_max(mx);
        float sum = 0.f;
        for (uint32_t j = lane; j < L; j += 64) sum += expf(Elem<DT>::load(x + j) - mx);
        const float inv = 1.0f / wave_sum(sum);
        for (uint32_t j = lane; j < L; j += 64) Elem<DT>::store(y + j, expf(Elem<DT>::load(x + j) - mx) * inv);
    }
}

// inner > 1: one thread per (outer, inner) column, neighbouring threads on neighbouring inner
// positions; three passes over the column (each step a coalesced read across the threads).
template <int DT>
__global__ __launch_bounds__(256) void softmax_cols_kernel(const typename Elem<DT>::type* __restrict__ X,
                                                           typename Elem<DT>::type* __restrict__ Y, uint32_t cols, uint32_t L, FastDiv innerd) {
    const uint32_t c = blockIdx.x * 256u + threadIdx.x;
    if (c >= cols) return;
    uint32_t outer, in;
    innerd.divmod(c, outer, in);
    const int64_t inner = innerd.d;
    const typename Elem<DT>::type* x = X + (int64_t)outer * L * inner + in;
    typename Elem<DT>::type* y = Y + (int64_t)outer * L * inner + in;
    float mx = -__builtin_inff();
    for (uint32_t j = 0; j < L; ++j) mx = fmaxf(mx, Elem<DT>::load(x + (int64_t)j * inner));
    float sum = 0.f;
    for (uint32_t j = 0; j < L; ++j) sum += expf(Elem<DT>::load(x + (int64_t)j * inner) - mx);
    const float inv = 1.0f / sum;
    for (uint32_t j = 0; j < L; ++j) Elem<DT>::store(y + (int64_t)j * inner, expf(Elem<DT>::load(x + (int64_t)j * inner) - mx) * inv);
}

// ReduceSum on tensors of storage type DT (0: fp32): checks, the merged index spaces, the launches.
template <int DT>
onnx_status reducesum_impl(const typename Elem<DT>::type* X, const int64_t* x_dims, int rank, const int64_t* axes, int naxes,
                           int keepdims, typename Elem<DT>::type* Y, const int64_t* y_dims, int y_rank, void* stream) {
    constexpr int64_t esz = sizeof(typename Elem<DT>::type);
    int64_t yd[ONNX_MAX_RANK];
    int r = 0;
    onnx_status st = onnx_reduce_infer(x_dims, rank, axes, naxes, keepdims, yd, &r);
    if (st != ONNX_OK) return st;
    if (y_rank != r || (r && !y_dims)) return fail(ONNX_ERR_SHAPE, "reducesum: y_rank %d but the inferred rank is %d", y_rank, r);
    for (int d = 0; d < r; ++d)
        if (y_dims[d] != yd[d])
            return fail(ONNX_ERR_SHAPE, "reducesum: y_dims[%d]=%lld but the inferred extent is %lld", d, (long long)y_dims[d], (long long)yd[d]);
    bool red[ONNX_MAX_RANK];
    reduce_flags("reducesum", rank, axes, naxes, red);
    int64_t nx = 1, ny = 1, nred = 1;
    for (int d = 0; d < rank; ++d) {
        if (x_dims[d] != 0 && nx > kMaxElems / x_dims[d]) return fail(ONNX_ERR_UNSUPPORTED, "reducesum: more than 2^31-1 input elements");
        nx *= x_dims[d];
        if (red[d]) nred *= x_dims[d]; else ny *= x_dims[d];
    }
    if (ny == 0) return ONNX_OK;
    if (!Y || (nx != 0 && !X)) return fail(ONNX_ERR_NULL, "reducesum: X and Y must not be NULL");
    if (overlaps(Y, ny * esz, X, nx * esz)) return fail(ONNX_ERR_ALIAS, "reducesum: Y overlaps X");
    // merged kept / reduced extents with their strides in X (unit extents dropped)
    ReduceMap m;
    m.nk = m.nr = 0;
    int64_t kd[ONNX_MAX_RANK], rd[ONNX_MAX_RANK];
    {
        int64_t stride[ONNX_MAX_RANK], sacc = 1;
        for (int d = rank - 1; d >= 0; --d) { stride[d] = sacc; sacc *= x_dims[d]; }
        int last = -1;                                   // 0 = kept, 1 = reduced: kind of the previous extent
        for (int d = 0; d < rank; ++d) {
            if (x_dims[d] == 1) continue;
            const int kind = red[d] ? 1 : 0;
            if (kind == last) {                          // adjacent extents of one kind: one longer extent
                if (kind) { rd[m.nr - 1] *= x_dims[d]; m.rs[m.nr - 1] = stride[d]; }
                else { kd[m.nk - 1] *= x_dims[d]; m.ks[m.nk - 1] = stride[d]; }
            } else if (kind) { rd[m.nr] = x_dims[d]; m.rs[m.nr] = stride[d]; ++m.nr; }
            else { kd[m.nk] = x_dims[d]; m.ks[m.nk] = stride[d]; ++m.nk; }
            last = kind;
        }
        if (m.nr == 0) { rd[0] = nred; m.rs[0] = 0; m.nr = 1; }     // nothing (or only unit extents) to add up
        for (int i = 0; i < m.nk; ++i) m.kdim[i] = FastDiv::make((uint32_t)kd[i]);
        for (int i = 0; i < m.nr; ++i) m.rdim[i] = FastDiv::make((uint32_t)rd[i]);
        m.outputs = (uint32_t)ny;
        m.reduced = (uint32_t)nred;
        // which kind is innermost in memory
        int inner_kind = 0;
        for (int d = rank - 1; d >= 0; --d) if (x_dims[d] != 1) { inner_kind = red[d] ? 1 : 0; break; }
        hipStream_t s = static_cast<hipStream_t>(stream);
        if (nred == 0) {                                 // empty sum: every output is 0
            hipLaunchKernelGGL(fill_kernel<DT>, dim3(blocks_for(ny)), dim3(256), 0, s, Y, ny, 0.f);
            return device_status(hipGetLastError(), "reducesum");
        }
        if (inner_kind == 1 || ny < 64) {
            // few outputs and a long sum: cut the reduced range into chunks when a workspace can hold the chunk sums
            const Workspace& w = workspace();
            uint32_t chunks = 1;
            if (w.partial && ny < 2048 && nred >= 32768) {
                int64_t c = nred / 8192;
                const int64_t cap = 4096 / ny > 1 ? 4096 / ny : 1;
                if (c > cap) c = cap;
                if (c >= 2 && ny * c <= w.partial_floats) chunks = (uint32_t)c;
            }
            if (chunks > 1) {
                const uint32_t per = (uint32_t)((nred + chunks - 1) / chunks);
                hipLaunchKernelGGL((reduce_inner_kernel<DT, 0>), dim3((unsigned)((ny * chunks + 3) / 4)), dim3(256), 0, s, X, w.partial, m, chunks, per);
                ReduceMap m2;
                m2.nk = 1; m2.nr = 1;
                m2.kdim[0] = FastDiv::make((uint32_t)ny); m2.ks[0] = chunks;
                m2.rdim[0] = FastDiv::make(chunks); m2.rs[0] = 1;
                m2.outputs = (uint32_t)ny; m2.reduced = chunks;
                hipLaunchKernelGGL((reduce_inner_kernel<0, DT>), dim3((unsigned)((ny + 3) / 4)), dim3(256), 0, s, static_cast<const float*>(w.partial), Y, m2, 1u, chunks);
            } else {
                hipLaunchKernelGGL((reduce_inner_kernel<DT, DT>), dim3((unsigned)((ny + 3) / 4)), dim3(256), 0, s, X, Y, m, 1u, (uint32_t)nred);
            }
        } else {
            hipLaunchKernelGGL(reduce_outer_kernel<DT>, dim3((unsigned)((ny + 255) / 256)), dim3(256), 0, s, X, Y, m);
        }
    }
    return device_status(hipGetLastError(), "reducesum");
}

// Softmax on tensors of storage type DT (0: fp32).
template <int DT>
onnx_status softmax_impl(const typename Elem<DT>::type* X, const int64_t* x_dims, int rank, int axis, typename Elem<DT>::type* Y, void* stream) {
    constexpr int64_t esz = sizeof(typename Elem<DT>::type);
    if (rank < 1 || rank > ONNX_MAX_RANK) return fail(ONNX_ERR_RANK, "softmax: rank %d outside 1..%d", rank, ONNX_MAX_RANK);
    if (!x_dims) return fail(ONNX_ERR_NULL, "softmax: NULL dims");
    if (axis < -rank || axis >= rank) return fail(ONNX_ERR_ATTR, "softmax: axis %d out of range for rank %d", axis, rank);
    if (axis < 0) axis += rank;
    int64_t outer = 1, inner = 1, n = 1;
    for (int d = 0; d < rank; ++d) {
        if (x_dims[d] < 0) return fail(ONNX_ERR_SHAPE, "softmax: negative extent");
        if (x_dims[d] != 0 && n > kMaxElems / x_dims[d]) return fail(ONNX_ERR_UNSUPPORTED, "softmax: more than 2^31-1 elements");
        n *= x_dims[d];
        if (d < axis) outer *= x_dims[d];
        if (d > axis) inner *= x_dims[d];
    }
    const int64_t L = x_dims[axis];
    if (n == 0) return ONNX_OK;
    if (!X || !Y) return fail(ONNX_ERR_NULL, "softmax: X and Y must not be NULL");
    if (overlaps(Y, n * esz, X, n * esz)) return fail(ONNX_ERR_ALIAS, "softmax: Y overlaps X");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (inner == 1)
        hipLaunchKernelGGL(softmax_rows_kernel<DT>, dim3((unsigned)((outer + 3) / 4)), dim3(256), 0, s, X, Y, (uint32_t)outer, (uint32_t)L);
    else
        hipLaunchKernelGGL(softmax_cols_kernel<DT>, dim3((unsigned)((outer * inner + 255) / 256)), dim3(256), 0, s, X, Y,
                           (uint32_t)(outer * inner), (uint32_t)L, FastDiv::make((uint32_t)inner));
    return device_status(hipGetLastError(), "softmax");
}

}  // namespace

extern "C" {

onnx_status onnx_relu(const float* X, int64_t count, float* Y, void* stream) {
    return run_unary<UN_RELU>("relu", X, count, 0.f, Y, stream);
}

onnx_status onnx_leakyrelu(const float* X, int64_t count, float alpha, float* Y, void* stream) {
    return run_unary<UN_LEAKY>("leakyrelu", X, count, alpha, Y, stream);
}

onnx_status onnx_abs(const float* X, int64_t count, float* Y, void* stream) {
    return run_unary<UN_ABS>("abs", X, count, 0.f, Y, stream);
}

onnx_status onnx_abs_lp(const void* X, int64_t count, void* Y, onnx_dtype type, void* stream) {
    if (type != ONNX_F16 && type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "abs_lp: type must be ONNX_F16 or ONNX_BF16");
    if (count < 0) return fail(ONNX_ERR_SHAPE, "abs_lp: negative element count");
    if (count == 0) return ONNX_OK;
    if (!X || !Y) return fail(ONNX_ERR_NULL, "abs_lp: X and Y must not be NULL");
    if (overlaps(Y, count * 2, X, count * 2)) return fail(ONNX_ERR_ALIAS, "abs_lp: Y overlaps X");
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* y = static_cast<uint16_t*>(Y);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (count % 8 == 0 && aligned16(X) && aligned16(Y))
        hipLaunchKernelGGL((abs_lp_kernel<8>), dim3(blocks_for(count / 8)), dim3(256), 0, s, x, y, count);
    else
        hipLaunchKernelGGL((abs_lp_kernel<1>), dim3(blocks_for(count)), dim3(256), 0, s, x, y, count);
    return device_status(hipGetLastError(), "abs_lp");
}

onnx_status onnx_broadcast_infer(const int64_t* a_dims, int a_rank, const int64_t* b_dims, int b_rank,
                                 int64_t* y_dims, int* y_rank) {
    if (a_rank < 0 || a_rank > ONNX_MAX_RANK || b_rank < 0 || b_rank > ONNX_MAX_RANK)
        return fail(ONNX_ERR_RANK, "broadcast: ranks %d and %d outside 0..%d", a_rank, b_rank, ONNX_MAX_RANK);
    if ((a_rank && !a_dims) || (b_rank && !b_dims) || !y_dims || !y_rank) return fail(ONNX_ERR_NULL, "broadcast: NULL dims");
    for (int d = 0; d < a_rank; ++d) if (a_dims[d] < 0) return fail(ONNX_ERR_SHAPE, "broadcast: negative extent");
    for (int d = 0; d < b_rank; ++d) if (b_dims[d] < 0) return fail(ONNX_ERR_SHAPE, "broadcast: negative extent");
    if (!broadcast_shape(a_dims, a_rank, b_dims, b_rank, y_dims, y_rank))
        return fail(ONNX_ERR_SHAPE, "broadcast: the shapes are not broadcast-compatible");
    return ONNX_OK;
}

// Add on fp32 (type 0) or 16-bit (LP_F16 / LP_BF16) tensors: checks, the merged index space, the launch.
static onnx_status add_any(const void* A, const int64_t* a_dims, int a_rank, const void* B, const int64_t* b_dims, int b_rank,
                           void* Y, const int64_t* y_dims, int y_rank, int type, void* stream) {
    const int64_t esz = type == 0 ? 4 : 2, vecw = 16 / esz;
    int64_t yd[ONNX_MAX_RANK];
    int r = 0;
    const onnx_status st = onnx_broadcast_infer(a_dims, a_rank, b_dims, b_rank, yd, &r);
    if (st != ONNX_OK) return st;
    if (y_rank != r || (r && !y_dims)) return fail(ONNX_ERR_SHAPE, "add: y_rank %d but the broadcast rank is %d", y_rank, r);
    int64_t ny = 1, na = 1, nb = 1;
    for (int d = 0; d < r; ++d) {
        if (y_dims[d] != yd[d])
            return fail(ONNX_ERR_SHAPE, "add: y_dims[%d]=%lld but the broadcast extent is %lld", d, (long long)y_dims[d], (long long)yd[d]);
        if (yd[d] != 0 && ny > kMaxElems / yd[d]) return fail(ONNX_ERR_UNSUPPORTED, "add: more than 2^31-1 output elements");
        ny *= yd[d];
    }
    for (int d = 0; d < a_rank; ++d) na *= a_dims[d];
    for (int d = 0; d < b_rank; ++d) nb *= b_dims[d];
    if (ny == 0) return ONNX_OK;
    if (!A || !B || !Y) return fail(ONNX_ERR_NULL, "add: A, B and Y must not be NULL");
    if (overlaps(Y, ny * esz, A, na * esz) || overlaps(Y, ny * esz, B, nb * esz)) return fail(ONNX_ERR_ALIAS, "add: Y overlaps an input");
    // per-dimension strides (0 = broadcast), unit extents dropped, neighbours merged when both
    // operands walk them like one longer extent
    int64_t dim[ONNX_MAX_RANK], sa[ONNX_MAX_RANK], sb[ONNX_MAX_RANK];
    int nd = 0;
    {
        int64_t stra = 1, strb = 1;
        int64_t tdim[ONNX_MAX_RANK], tsa[ONNX_MAX_RANK], tsb[ONNX_MAX_RANK];
        for (int d = r - 1; d >= 0; --d) {
            const int64_t ea = d < r - a_rank ? 1 : a_dims[d - (r - a_rank)], eb = d < r - b_rank ? 1 : b_dims[d - (r - b_rank)];
            tdim[d] = yd[d];
            tsa[d] = ea == 1 ? 0 : stra;
            tsb[d] = eb == 1 ? 0 : strb;
            stra *= ea;
            strb *= eb;
        }
        for (int d = 0; d < r; ++d) {
            if (tdim[d] == 1) continue;
            if (nd > 0 && sa[nd - 1] == tsa[d] * tdim[d] && sb[nd - 1] == tsb[d] * tdim[d]) {
                dim[nd - 1] *= tdim[d]; sa[nd - 1] = tsa[d]; sb[nd - 1] = tsb[d];
            } else {
                dim[nd] = tdim[d]; sa[nd] = tsa[d]; sb[nd] = tsb[d]; ++nd;
            }
        }
        if (nd == 0) { dim[0] = 1; sa[0] = 0; sb[0] = 0; nd = 1; }
    }
    // wide accesses: an operand walked with stride 1 needs 16-byte aligned groups (its other strides then are multiples
    // of the group too, the innermost extent being one); a broadcast one is read element by element
    const bool vec = dim[nd - 1] % vecw == 0 && (sa[nd - 1] == 0 || aligned16(A)) && (sb[nd - 1] == 0 || aligned16(B)) && aligned16(Y);
    BroadcastMap m;
    m.nd = nd;
    for (int d = 0; d < nd; ++d) {
        m.dim[d] = FastDiv::make((uint32_t)((d == nd - 1 && vec) ? dim[d] / vecw : dim[d]));
        m.sa[d] = sa[d]; m.sb[d] = sb[d];
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t groups = (uint32_t)(vec ? ny / vecw : ny);
    const dim3 grid(blocks_for(groups)), block(256);
    if (type == 0) {
        const float* a = static_cast<const float*>(A);
        const float* b = static_cast<const float*>(B);
        float* y = static_cast<float*>(Y);
        if (vec) hipLaunchKernelGGL((add_kernel<4>), grid, block, 0, s, a, b, y, groups, m);
        else hipLaunchKernelGGL((add_kernel<1>), grid, block, 0, s, a, b, y, groups, m);
    } else {
        const uint16_t* a = static_cast<const uint16_t*>(A);
        const uint16_t* b = static_cast<const uint16_t*>(B);
        uint16_t* y = static_cast<uint16_t*>(Y);
        if (type == LP_BF16) {
            if (vec) hipLaunchKernelGGL((add_lp_kernel<LP_BF16, 8>), grid, block, 0, s, a, b, y, groups, m);
            else hipLaunchKernelGGL((add_lp_kernel<LP_BF16, 1>), grid, block, 0, s, a, b, y, groups, m);
        } else {
            if (vec) hipLaunchKernelGGL((add_lp_kernel<LP_F16, 8>), grid, block, 0, s, a, b, y, groups, m);
            else hipLaunchKernelGGL((add_lp_kernel<LP_F16, 1>), grid, block, 0, s, a, b, y, groups, m);
        }
    }
    return device_status(hipGetLastError(), "add");
}

onnx_status onnx_add(const float* A, const int64_t* a_dims, int a_rank, const float* B, const int64_t* b_dims,
                     int b_rank, float* Y, const int64_t* y_dims, int y_rank, void* stream) {
    return add_any(A, a_dims, a_rank, B, b_dims, b_rank, Y, y_dims, y_rank, 0, stream);
}

onnx_status onnx_add_lp(const void* A, const int64_t* a_dims, int a_rank, const void* B, const int64_t* b_dims, int b_rank,
                        void* Y, const int64_t* y_dims, int y_rank, onnx_dtype type, void* stream) {
    if (type != ONNX_F16 && type != ONNX_BF16) return fail(ONNX_ERR_ATTR, "add_lp: type must be ONNX_F16 or ONNX_BF16");
    return add_any(A, a_dims, a_rank, B, b_dims, b_rank, Y, y_dims, y_rank, type == ONNX_F16 ? LP_F16 : LP_BF16, stream);
}

onnx_status onnx_reduce_infer(const int64_t* x_dims, int rank, const int64_t* axes, int naxes, int keepdims,
                              int64_t* y_dims, int* y_rank) {
    bool red[ONNX_MAX_RANK];
    const onnx_status st = reduce_flags("reduce", rank, axes, naxes, red);
    if (st != ONNX_OK) return st;
    if ((rank && !x_dims) || !y_dims || !y_rank) return fail(ONNX_ERR_NULL, "reduce: NULL dims");
    int r = 0;
    for (int d = 0; d < rank; ++d) {
        if (x_dims[d] < 0) return fail(ONNX_ERR_SHAPE, "reduce: negative extent");
        if (!red[d]) y_dims[r++] = x_dims[d];
        else if (keepdims) y_dims[r++] = 1;
    }
    *y_rank = r;
    return ONNX_OK;
}

onnx_status onnx_reducesum(const float* X, const int64_t* x_dims, int rank, const int64_t* axes, int naxes,
                           int keepdims, float* Y, const int64_t* y_dims, int y_rank, void* stream) {
    return reducesum_impl<0>(X, x_dims, rank, axes, naxes, keepdims, Y, y_dims, y_rank, stream);
}

onnx_status onnx_reducesum_lp(const void* X, const int64_t* x_dims, int rank, const int64_t* axes, int naxes, int keepdims,
                              void* Y, const int64_t* y_dims, int y_rank, onnx_dtype type, void* stream) {
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* y = static_cast<uint16_t*>(Y);
    if (type == ONNX_F16) return reducesum_impl<LP_F16>(x, x_dims, rank, axes, naxes, keepdims, y, y_dims, y_rank, stream);
    if (type == ONNX_BF16) return reducesum_impl<LP_BF16>(x, x_dims, rank, axes, naxes, keepdims, y, y_dims, y_rank, stream);
    return fail(ONNX_ERR_ATTR, "reducesum_lp: type must be ONNX_F16 or ONNX_BF16");
}

onnx_status onnx_softmax(const float* X, const int64_t* x_dims, int rank, int axis, float* Y, void* stream) {
    return softmax_impl<0>(X, x_dims, rank, axis, Y, stream);
}

onnx_status onnx_softmax_lp(const void* X, const int64_t* x_dims, int rank, int axis, void* Y, onnx_dtype type, void* stream) {
    const uint16_t* x = static_cast<const uint16_t*>(X);
    uint16_t* y = static_cast<uint16_t*>(Y);
    if (type == ONNX_F16) return softmax_impl<LP_F16>(x, x_dims, rank, axis, y, stream);
    if (type == ONNX_BF16) return softmax_impl<LP_BF16>(x, x_dims, rank, axis, y, stream);
    return fail(ONNX_ERR_ATTR, "softmax_lp: type must be ONNX_F16 or ONNX_BF16");
}

}  // extern "C"
