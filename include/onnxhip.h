/*
 * onnxhip -- the dense-contraction operators of an ONNX inference graph on one gfx950 GPU.
 *
 * The paper's compiler turns an ONNX model into one C-callable entry whose inputs and
 * outputs mirror the graph's (Section 3, "_dyn_entry_point_main_graph"); tensors are dense
 * row-major buffers with run-time dimensions (Section 2.2, tensor / memref types), each
 * operator writes a freshly allocated result (Section 3.1, lowering to krnl), attributes
 * carry the ONNX defaults (Section 3.2, Listing 6) and output shapes follow from shape
 * inference (Section 3.4).  This library offers the operators that dominate its two
 * experiments (Section 4.2: MNIST and ResNet50 -- convolution, pooling, MatMul/Gemm) as
 * direct calls with the same conventions.
 *
 * Conventions for every compute entry point
 *   - float* / int64_t* tensor arguments are DEVICE pointers (hipMalloc'ed memory of the
 *     current device); every dims / attribute array is a HOST pointer read before return.
 *   - Tensors are fp32, dense, row-major, last dimension contiguous; 4-D tensors are NCHW.
 *   - The caller owns every buffer.  The library never allocates or frees device memory.
 *   - The output must not overlap any input (ONNX_ERR_ALIAS when the byte ranges intersect).
 *   - y_dims must equal the inferred output shape (ONNX_ERR_SHAPE otherwise).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null stream)
 *     and the call returns without waiting.  Launch failures are reported as
 *     ONNX_ERR_DEVICE.
 *   - All validation happens before anything is enqueued: on any error nothing is written.
 *   - A zero-sized output returns ONNX_OK without launching.
 *   - pads are in ONNX order {top, left, bottom, right}.
 */
#ifndef ONNXHIP_H
#define ONNXHIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ONNX_OK = 0,
    ONNX_ERR_NULL = 1,        /* a required pointer is NULL                                */
    ONNX_ERR_RANK = 2,        /* a rank outside what the operator accepts                  */
    ONNX_ERR_SHAPE = 3,       /* dimensions inconsistent with each other or with y_dims    */
    ONNX_ERR_ATTR = 4,        /* stride/dilation/kernel < 1, pad < 0, pad >= window (pools)*/
    ONNX_ERR_UNSUPPORTED = 5, /* a valid request this library does not implement           */
    ONNX_ERR_ALIAS = 6,       /* output overlaps an input                                  */
    ONNX_ERR_DEVICE = 7       /* the HIP runtime reported an error                         */
} onnx_status;

typedef enum { ONNX_ACT_NONE = 0, ONNX_ACT_RELU = 1 } onnx_act;

#define ONNX_MAX_RANK 8

/* Message for the most recent non-OK status on the calling thread (static storage). */
const char* onnx_last_error(void);

/*
 * Which kernel instance the calling thread's most recent Conv / Gemm / MatMul launch on the
 * matrix cores used, as text: family, tile (rows x columns x K step), wavefront grid
 * (rows x columns x K slices), operand loader kinds and load widths, split factors.  Empty
 * before the first such launch.  For tests and tuning; static thread-local storage.
 */
const char* onnx_last_launch(void);

/*
 * Optional scratch memory (Section 3.1 notes that memory management is decided once operators
 * have been lowered to loops over buffers; here the caller decides it).  The library never
 * allocates: when a workspace is set, products whose output has too few tiles to occupy the
 * GPU split their K range over several workgroups, which park partial tiles in it, and a
 * second kernel on the same stream adds them and runs the epilogue (the same is done for the
 * few tiles by which a tile count exceeds a multiple of the 256 CUs, and onnx_reducesum uses it
 * for the chunk sums of a long sum into few outputs); without a workspace those products run
 * unsplit.  `device_ptr` is device memory (256-byte aligned, at least 1 MiB; 64
 * MiB serves every workload here) that the caller keeps alive and does not touch while calls
 * are in flight; it needs no initialisation.  All calls share it, so operators that may use it
 * must not run concurrently on different streams.  NULL or 0 bytes removes the workspace.
 * The setting is process-wide: a call uses the workspace that was set when it was made (setting
 * and reading are serialised against each other, so host threads never see a torn pointer/size
 * pair), but two host threads that set different workspaces must order their calls themselves.
 * Results do not depend on it beyond fp32 summation order and are reproducible run to run.
 */
onnx_status onnx_set_workspace(void* device_ptr, size_t bytes);

/* ---- shape inference (host only; Section 3.4, the shape-inference pass) ------------- */

/* Conv: y = {N, M, OH, OW}, OH = floor((H + pT + pB - ((kH-1)*dH + 1)) / sH) + 1. */
onnx_status onnx_conv_infer(const int64_t x_dims[4], const int64_t w_dims[4],
                            const int64_t pads[4], const int64_t strides[2],
                            const int64_t dilations[2], int64_t group, int64_t y_dims[4]);

/* MaxPool / AveragePool: as Conv per axis; ceil_mode rounds up and drops a last window that
 * would start beyond the input plus its leading padding. dilations may be NULL (= {1,1}). */
onnx_status onnx_pool_infer(const int64_t x_dims[4], const int64_t kernel[2],
                            const int64_t pads[4], const int64_t strides[2],
                            const int64_t dilations[2], int ceil_mode, int64_t y_dims[4]);

/* MatMul: numpy.matmul shape rules; y_dims must hold max(a_rank, b_rank) entries. */
onnx_status onnx_matmul_infer(const int64_t* a_dims, int a_rank, const int64_t* b_dims,
                              int b_rank, int64_t* y_dims, int* y_rank);

/* ---- operators ---------------------------------------------------------------------- */

/*
 * ONNX Conv, 2-D (Section 4.1 "convolution"; the bulk of ResNet50's time, Section 4.2).
 *   Y[n,m,oh,ow] = B[m] + sum_{c<C/group, kh, kw}
 *                    X~[n, g*C/group + c, oh*sH - pT + kh*dH, ow*sW - pL + kw*dW] * W[m,c,kh,kw]
 * g = m / (M/group), X~ = 0 outside the image, no kernel flip.  Fused epilogue, applied
 * in this order: + residual[n,m,oh,ow] (NULL = none; same shape as Y), then Relu if
 * act == ONNX_ACT_RELU.
 *   X [N,C,H,W]  W [M,C/group,kH,kW]  B [M] or NULL  residual [N,M,OH,OW] or NULL  Y [N,M,OH,OW]
 * group must divide C and M, w_dims[1]*group == C (ONNX_ERR_SHAPE); strides, dilations >= 1,
 * pads >= 0 (ONNX_ERR_ATTR).  auto_pad is resolved by the caller into explicit pads.
 */
onnx_status onnx_conv(const float* X, const int64_t x_dims[4], const float* W,
                      const int64_t w_dims[4], const float* B, const int64_t pads[4],
                      const int64_t strides[2], const int64_t dilations[2], int64_t group,
                      const float* residual, onnx_act act, float* Y, const int64_t y_dims[4],
                      void* stream);

/*
 * onnx_conv for callers that cannot allocate or hand over device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and
 * errors as onnx_conv.  The split-K scratch that onnx_conv takes from onnx_set_workspace is here a
 * fixed array of ONNX_CONV_FIXED_SCRATCH_BYTES inside the library's device image (every GPU the
 * library runs on holds its copy until the process ends); the workspace set by
 * onnx_set_workspace is neither used nor changed.  The call allocates and frees nothing.
 * Outputs of more than ONNX_CONV_FIXED_SCRATCH_MAX_OUTPUTS elements are refused with
 * ONNX_ERR_UNSUPPORTED (larger convolutions fill the GPU without split-K: use onnx_conv).
 * The array needs no initialisation (every partial tile is written before it is read), and all
 * calls on one GPU share it: calls that overlap in time on one GPU, on whatever streams, race.
 */
#define ONNX_CONV_FIXED_SCRATCH_BYTES (16u << 20)
#define ONNX_CONV_FIXED_SCRATCH_MAX_OUTPUTS (1 << 21)
onnx_status onnx_conv_fixed_scratch(const float* X, const int64_t x_dims[4], const float* W,
                                    const int64_t w_dims[4], const float* B, const int64_t pads[4],
                                    const int64_t strides[2], const int64_t dilations[2],
                                    int64_t group, const float* residual, onnx_act act, float* Y,
                                    const int64_t y_dims[4], void* stream);

/*
 * ONNX Gemm (Section 3.4: the target of the MatMul+Add rewrite; Section 4.1).
 *   Y = alpha * op(A) * op(B) + beta * C~,  op(.) = transpose when the flag is non-zero,
 * op(A) is M x K, op(B) is K x N, C~ is C broadcast to M x N from rank 0 (c_rank = 0, one
 * element), {N}, {1,N}, {M,1}, {M,N} or {1,1}; C == NULL omits the term.  Relu optional.
 * a_dims / b_dims are the stored shapes of A and B.
 */
onnx_status onnx_gemm(const float* A, const int64_t a_dims[2], const float* B,
                      const int64_t b_dims[2], const float* C, const int64_t* c_dims, int c_rank,
                      float alpha, float beta, int transA, int transB, onnx_act act, float* Y,
                      const int64_t y_dims[2], void* stream);

/*
 * ONNX MatMul (Section 3.4; MNIST's "matrix multiplication", Section 4.2), numpy.matmul
 * semantics: a rank-1 A acts as [1,K] and a rank-1 B as [K,1] with the unit dimension
 * dropped from Y; leading dimensions broadcast right-aligned.  Ranks 1..ONNX_MAX_RANK.
 */
onnx_status onnx_matmul(const float* A, const int64_t* a_dims, int a_rank, const float* B,
                        const int64_t* b_dims, int b_rank, float* Y, const int64_t* y_dims,
                        int y_rank, void* stream);

/*
 * ONNX MaxPool, 2-D (Section 4.1 "pooling"; Section 4.2 MNIST "max pooling").
 * Maximum over the taps inside the image.  Indices (NULL = not wanted) receives, as int64,
 * the flat row-major position in the whole X tensor of the winning tap; among equal
 * maxima the first in (kh, kw) scan order wins (storage_order 0).  Pads must be smaller
 * than the dilated window so that no window is empty (ONNX_ERR_ATTR).
 */
onnx_status onnx_maxpool(const float* X, const int64_t x_dims[4], const int64_t kernel[2],
                         const int64_t pads[4], const int64_t strides[2],
                         const int64_t dilations[2], int ceil_mode, float* Y, int64_t* Indices,
                         const int64_t y_dims[4], void* stream);

/*
 * ONNX AveragePool / GlobalAveragePool, 2-D (Section 4.1 "pooling"; ResNet50's last pool).
 * Sum of the in-image taps divided by their count (count_include_pad = 0) or by the number
 * of taps inside the padded image (count_include_pad = 1).  kernel == NULL means global:
 * window H x W, pads and strides ignored, Y is [N,C,1,1].
 */
onnx_status onnx_avgpool(const float* X, const int64_t x_dims[4], const int64_t* kernel,
                         const int64_t* pads, const int64_t* strides, int ceil_mode,
                         int count_include_pad, float* Y, const int64_t y_dims[4], void* stream);

/*
 * Element-wise, reduction and softmax operators: the operators the paper walks through next
 * to the contractions.  Same conventions as above (device tensors, host dims, caller-owned
 * memory, no overlap of output and inputs, validation before any launch, zero-sized outputs
 * return ONNX_OK without launching).  Tensors of up to 2^31-1 elements (ONNX_ERR_UNSUPPORTED
 * beyond), ranks 0..ONNX_MAX_RANK.
 */

/* Shape of a numpy-style (ONNX "multidirectional") broadcast of two shapes: aligned at the
 * last axis, each pair of extents equal or one of them 1.  Pure host function. */
onnx_status onnx_broadcast_infer(const int64_t* a_dims, int a_rank, const int64_t* b_dims, int b_rank,
                                 int64_t* y_dims, int* y_rank);

/*
 * ONNX Add (the running example of Section 3: two 3x4x5 tensors added element by element):
 * Y = A + B with multidirectional broadcasting; y_dims/y_rank must be the broadcast shape.
 */
onnx_status onnx_add(const float* A, const int64_t* a_dims, int a_rank, const float* B,
                     const int64_t* b_dims, int b_rank, float* Y, const int64_t* y_dims, int y_rank,
                     void* stream);

/* ONNX Relu, y = max(0, x), over `count` elements. */
onnx_status onnx_relu(const float* X, int64_t count, float* Y, void* stream);

/* ONNX LeakyRelu (its operator definition is the example of Section 3.1): y = x for x >= 0,
 * alpha * x otherwise; the ONNX default of alpha is 0.01. */
onnx_status onnx_leakyrelu(const float* X, int64_t count, float alpha, float* Y, void* stream);

/* ONNX Abs, y = |x| (with ReduceSum it makes up ReduceL1: the decomposition of Section 3.4). */
onnx_status onnx_abs(const float* X, int64_t count, float* Y, void* stream);

/* Output shape of a reduction over `axes` (negative values count from the last axis; naxes = 0
 * reduces every axis; an axis out of range or listed twice is ONNX_ERR_ATTR): reduced axes keep
 * extent 1 when keepdims != 0 and disappear otherwise.  Pure host function. */
onnx_status onnx_reduce_infer(const int64_t* x_dims, int rank, const int64_t* axes, int naxes,
                              int keepdims, int64_t* y_dims, int* y_rank);

/*
 * ONNX ReduceSum (Section 3.4): Y = sum of X over the listed axes, shape as onnx_reduce_infer.
 * Sums are formed in fp32 (64 partial sums per output where the innermost axis is reduced, one
 * running sum otherwise).  With a workspace set (onnx_set_workspace), a long sum into few
 * outputs is cut into chunks that run in parallel and are added by a second launch.
 */
onnx_status onnx_reducesum(const float* X, const int64_t* x_dims, int rank, const int64_t* axes,
                           int naxes, int keepdims, float* Y, const int64_t* y_dims, int y_rank,
                           void* stream);

/*
 * ONNX Softmax along one axis (negative values count from the last axis):
 * y_i = exp(x_i - m) / sum_j exp(x_j - m) with m the maximum along the axis.  (The paper leaves
 * operator semantics to the ONNX standard, Section 3.1; older operator sets flatten the tensor
 * to 2-D at `axis` instead: for the classifier's [N, classes] logits with axis 1 or -1 both
 * readings coincide.)  Rank 1..ONNX_MAX_RANK.
 */
onnx_status onnx_softmax(const float* X, const int64_t* x_dims, int rank, int axis, float* Y,
                         void* stream);

/* Element types of the 16-bit entry point below (storage: IEEE binary16, or bfloat16 = the upper
 * half of a binary32). */
typedef enum { ONNX_F32 = 0, ONNX_F16 = 1, ONNX_BF16 = 2 } onnx_dtype;

/*
 * ONNX Gemm on 16-bit floating-point inputs (the operator definitions admit F16 tensors,
 * Section 3.1): Y = alpha * op(A) * op(B) + beta * C with A and B stored as in_type, every
 * transA / transB combination, any K.  Products are exact and summed in fp32; C (NULL, or fp32
 * broadcastable to [M,N] as for onnx_gemm) and the epilogue are fp32; Y is stored as out_type:
 * ONNX_F32, or in_type with round-to-nearest-even.  The tuned kernel takes transA = 0 with K a
 * multiple of 8 and A 16-byte aligned, and B either K-contiguous (transB = 1, 16-byte aligned)
 * or row-contiguous (transB = 0, N a multiple of 4, 8-byte aligned); every other case runs
 * through a general, slower kernel that transposes operands element by element on their way
 * into LDS.
 */
onnx_status onnx_gemm_lp(const void* A, const int64_t a_dims[2], const void* B, const int64_t b_dims[2],
                         const float* C, const int64_t* c_dims, int c_rank, float alpha, float beta,
                         int transA, int transB, onnx_act act, void* Y, const int64_t y_dims[2],
                         onnx_dtype in_type, onnx_dtype out_type, void* stream);

/*
 * ONNX MatMul on 16-bit inputs: numpy.matmul semantics as onnx_matmul, A and B stored as in_type,
 * fp32 accumulation, Y stored as out_type (ONNX_F32 or in_type, rounded to nearest even).  The
 * tuned kernel takes K a multiple of 8 and N a multiple of 4 with aligned operands, as for
 * onnx_gemm_lp with transB = 0; other shapes run through the general kernel.
 */
onnx_status onnx_matmul_lp(const void* A, const int64_t* a_dims, int a_rank, const void* B,
                           const int64_t* b_dims, int b_rank, void* Y, const int64_t* y_dims, int y_rank,
                           onnx_dtype in_type, onnx_dtype out_type, void* stream);

/*
 * ONNX Conv on 16-bit inputs: the semantics, attributes and errors of onnx_conv; X and W stored
 * as in_type, the bias B in fp32 ([M] or NULL), fp32 accumulation, Y and the optional residual
 * stored as out_type (ONNX_F32 or in_type, rounded to nearest even).  A 1x1 convolution with
 * stride 1 and no padding whose C/group is a multiple of 8 and whose H*W is a multiple of 4 runs
 * through the tuned kernel of onnx_gemm_lp (the input of an image is a row-contiguous
 * [C][H*W] matrix).  A 3x3 convolution (any stride, dilation and padding) whose C/group is a
 * multiple of 16 runs through a kernel that stages the input patch of a tile in LDS, provided
 * the workspace of onnx_set_workspace can hold a rewritten copy of the filter bank
 * (M * C/group * 9 16-bit values; a small kernel ahead of the convolution writes it on every
 * call, so calls that share the workspace on different streams race, as for split-K).  With a
 * workspace, strided 1x1 convolutions and pointwise ones whose H*W is not a multiple of 4 are
 * first copied into a layout the tuned kernel reads.  The first layer of ResNet50 (Section 4.2:
 * 7x7, stride 2, pads 3, 3 -> 64 channels, no residual, at most 157 output columns) has a
 * kernel of its own that needs no workspace.  Every other shape runs through one general kernel
 * that gathers the input element by element and uses no workspace.
 */
onnx_status onnx_conv_lp(const void* X, const int64_t x_dims[4], const void* W, const int64_t w_dims[4],
                         const float* B, const int64_t pads[4], const int64_t strides[2],
                         const int64_t dilations[2], int64_t group, const void* residual, onnx_act act,
                         void* Y, const int64_t y_dims[4], onnx_dtype in_type, onnx_dtype out_type,
                         void* stream);

/*
 * The 3x3 case of onnx_conv_lp for filters that do not change between calls (inference): the
 * LDS-patch kernel reads the filter bank in tap order, [M][C/group / 16][9 taps][16 channels],
 * and onnx_conv_lp rewrites W into that order in the workspace on every call.
 * onnx_conv_lp_filter_taps does the rewriting once, into `packed` (device memory of the size of
 * W, 16-byte aligned, caller-owned); onnx_conv_lp_taps is onnx_conv_lp with `packed` in place of
 * W (w_dims still the ONNX shape [M, C/group, 3, 3]); it needs no workspace and uses one only
 * to split K when the output has few tiles.  Both need 3x3
 * windows and C/group a multiple of 16; onnx_conv_lp_taps returns ONNX_ERR_UNSUPPORTED, before
 * any launch, for shapes whose input patch does not fit the kernel (the caller then uses
 * onnx_conv_lp with W).
 */
onnx_status onnx_conv_lp_filter_taps(const void* W, const int64_t w_dims[4], void* packed, void* stream);
onnx_status onnx_conv_lp_taps(const void* X, const int64_t x_dims[4], const void* packed, const int64_t w_dims[4],
                              const float* B, const int64_t pads[4], const int64_t strides[2],
                              const int64_t dilations[2], int64_t group, const void* residual,
                              onnx_act act, void* Y, const int64_t y_dims[4], onnx_dtype in_type,
                              onnx_dtype out_type, void* stream);

/*
 * ONNX MaxPool and AveragePool / GlobalAveragePool on 16-bit tensors (type ONNX_F16 or
 * ONNX_BF16 for X and Y alike): what lies between the 16-bit convolutions of a network whose
 * activations stay in the 16-bit type.  Semantics, attributes, limits and errors of
 * onnx_maxpool (without Indices) and onnx_avgpool.  The maximum is stored with the bits of the
 * winning input; an average is summed in fp32 in scan order, divided, and rounded to the type
 * once (nearest even).  At most 2^31-1 output elements.
 */
onnx_status onnx_maxpool_lp(const void* X, const int64_t x_dims[4], const int64_t kernel[2],
                            const int64_t pads[4], const int64_t strides[2],
                            const int64_t dilations[2], int ceil_mode, void* Y,
                            const int64_t y_dims[4], onnx_dtype type, void* stream);
onnx_status onnx_avgpool_lp(const void* X, const int64_t x_dims[4], const int64_t* kernel,
                            const int64_t* pads, const int64_t* strides, int ceil_mode,
                            int count_include_pad, void* Y, const int64_t y_dims[4],
                            onnx_dtype type, void* stream);

/*
 * ONNX LeakyRelu on a 16-bit tensor (Section 3.1: the operator's definition lists F16 among its
 * element types): Y[i] = X[i] for X[i] >= 0, alpha * X[i] otherwise, the product taken in fp32 and
 * rounded to the type (nearest even); alpha = 0 is Relu.  `count` elements of `type` (ONNX_F16 or
 * ONNX_BF16); Y must not overlap X.
 */
onnx_status onnx_leakyrelu_lp(const void* X, int64_t count, float alpha, void* Y, onnx_dtype type, void* stream);

/*
 * ONNX Add and Abs on 16-bit tensors (Section 3: Add is the running example; Section 3.4: Abs is
 * one of the two operators ReduceL1 decomposes into; `type` ONNX_F16 or ONNX_BF16 for every
 * operand).  Add: shapes, broadcasting, y_dims and errors as for onnx_add; every sum is taken in
 * fp32 and rounded to the type (nearest even), which for two 16-bit addends is the correctly
 * rounded sum.  Abs clears the sign bit (of a NaN too).  Y must not overlap an input.
 */
onnx_status onnx_add_lp(const void* A, const int64_t* a_dims, int a_rank, const void* B, const int64_t* b_dims,
                        int b_rank, void* Y, const int64_t* y_dims, int y_rank, onnx_dtype type, void* stream);
onnx_status onnx_abs_lp(const void* X, int64_t count, void* Y, onnx_dtype type, void* stream);

/*
 * ONNX ReduceSum and Softmax on 16-bit tensors (`type` ONNX_F16 or ONNX_BF16 for X and Y): shapes,
 * axes, keepdims, y_dims, the optional workspace and errors as for onnx_reducesum / onnx_softmax
 * (Section 3.4: ReduceSum is the other half of the ReduceL1 decomposition).  Sums, the maximum,
 * the exponentials and the division are fp32; only the result is rounded to the type (nearest
 * even).  Y must not overlap X.
 */
onnx_status onnx_reducesum_lp(const void* X, const int64_t* x_dims, int rank, const int64_t* axes, int naxes,
                              int keepdims, void* Y, const int64_t* y_dims, int y_rank, onnx_dtype type,
                              void* stream);
onnx_status onnx_softmax_lp(const void* X, const int64_t* x_dims, int rank, int axis, void* Y, onnx_dtype type,
                            void* stream);

/*
 * ONNX LSTM (named among the supported operators, Section 4.1), layout 0, default activations
 * (sigmoid, tanh, tanh), no peepholes, every sequence of full length.  X [seq, batch, input];
 * W [dirs, 4H, input] and R [dirs, 4H, H] with the gate blocks in the order i, o, f, c;
 * B NULL or [dirs, 8H] (input biases, then recurrent biases); initial_h / initial_c NULL (zeros)
 * or [dirs, batch, H]; dirs = 2 for ONNX_LSTM_BIDIRECTIONAL, else 1.  Per step
 *   i,o,f = sigmoid(x W' + h R' + Wb + Rb),  g = tanh(...),  c = f*c + i*g,  h = o*tanh(c).
 * Outputs (each may be NULL, not all): Y [seq, dirs, batch, H], Y_h and Y_c [dirs, batch, H].
 * The input projection of the whole sequence runs through the same kernel as onnx_gemm; every
 * time step is then one launch that multiplies h by R' on the matrix cores and applies the gates
 * (both directions of a bidirectional LSTM in the same launch).  `scratch` is caller-owned device memory of at least
 * onnx_lstm_scratch_bytes(...) bytes, 256-byte aligned, contents irrelevant; it must not overlap
 * any input or output (ONNX_ERR_ALIAS).
 */
enum { ONNX_LSTM_FORWARD = 0, ONNX_LSTM_REVERSE = 1, ONNX_LSTM_BIDIRECTIONAL = 2 };
size_t onnx_lstm_scratch_bytes(const int64_t x_dims[3], int64_t hidden_size, int direction);
onnx_status onnx_lstm(const float* X, const int64_t x_dims[3], const float* W, const float* R,
                      const float* B, const float* initial_h, const float* initial_c,
                      int64_t hidden_size, int direction, float* Y, float* Y_h, float* Y_c,
                      void* scratch, size_t scratch_bytes, void* stream);

/*
 * A whole small model as one launch (Section 3: the compiler emits one entry function per
 * model; Section 4.2: the MNIST network, two convolutions with Relu, two max pools and a matrix
 * product with bias).  `ops` (host memory) is a linear chain of 1..ONNX_CHAIN_MAX_OPS operators;
 * the first consumes X [N,C,H,W], each other one the result of its predecessor; a Gemm consumes
 * its input flattened to [1, C*H*W] per image (the Reshape / Flatten in front of it is implied).
 * One workgroup runs the whole chain for one image with all weights and every activation in LDS:
 * nothing but X, the weights and the requested results touches device memory.
 *   ONNX_CHAIN_CONV     onnx_conv with group 1: W [outputs, C, kernel[0], kernel[1]], B NULL or
 *                       [outputs]; pads, strides, dilations, act as there
 *   ONNX_CHAIN_MAXPOOL  onnx_maxpool without Indices: kernel, pads, strides, dilations, ceil_mode
 *   ONNX_CHAIN_AVGPOOL  onnx_avgpool: kernel, pads, strides, ceil_mode, count_include_pad;
 *                       kernel {0,0} means global
 *   ONNX_CHAIN_GEMM     Y = alpha * x * op(W) + beta * B, x the flattened input [1,K], W [K,outputs]
 *                       (transB = 0) or [outputs,K], B NULL or [outputs]; act as for onnx_gemm
 * Each operator's Y is NULL (the result stays on chip) or device memory for the result of every
 * image, [N, ...] in the shape the matching *_infer call gives; the last operator's Y is
 * required.  Limits (ONNX_ERR_UNSUPPORTED beyond them): every activation, counted with the
 * zero padding of the Conv that consumes it, has at most ONNX_CHAIN_MAX_ACTIVATION floats per
 * image; all weights and biases together at most ONNX_CHAIN_MAX_WEIGHTS floats (a Conv's filter
 * rows count as C*kH*kW rounded up to a multiple of 16, plus 4); a Conv's C*kH*kW at most
 * ONNX_CHAIN_MAX_CONV_K.
 * Attribute and shape errors are those of the single operators.  Everything is validated before
 * the launch; nothing is allocated; a Y buffer that overlaps X, a weight, a bias or another Y is refused
 * (ONNX_ERR_ALIAS).
 */
#define ONNX_CHAIN_MAX_OPS 8
#define ONNX_CHAIN_MAX_ACTIVATION 10240
#define ONNX_CHAIN_MAX_WEIGHTS 14336
#define ONNX_CHAIN_MAX_CONV_K 2048
typedef enum { ONNX_CHAIN_CONV = 0, ONNX_CHAIN_MAXPOOL = 1, ONNX_CHAIN_AVGPOOL = 2, ONNX_CHAIN_GEMM = 3 } onnx_chain_kind;
typedef struct {
    int32_t kind;               /* onnx_chain_kind */
    int32_t act;                /* onnx_act, Conv and Gemm */
    int64_t outputs;            /* Conv: output channels; Gemm: columns of the result */
    int64_t kernel[2];
    int64_t pads[4];
    int64_t strides[2];
    int64_t dilations[2];
    int32_t ceil_mode;
    int32_t count_include_pad;
    int32_t transB;
    float alpha, beta;
    const float* W;             /* device */
    const float* B;             /* device or NULL */
    float* Y;                   /* device or NULL */
} onnx_chain_op;
onnx_status onnx_chain(const onnx_chain_op* ops, int n_ops, const float* X, const int64_t x_dims[4],
                       void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ONNXHIP_H */
