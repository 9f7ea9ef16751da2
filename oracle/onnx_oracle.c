/*
 * CPU oracle for the ONNX contraction and pooling operators the paper's compiler
 * lowers (Section 4.1 lists convolution, pooling and Gemm among the supported
 * operators; Section 3.1 says the onnx dialect carries the ONNX standard's
 * semantics; Section 3.4's MulAddToGemmPattern ties MatMul+Add to Gemm).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain loop nests that follow the operator
 * definitions term by term: fp32 inputs, every product and sum taken in double
 * (a product of two fp32 values is exact in double), results returned as double
 * without an intermediate fp32 rounding.  No blocking, no fusion, no
 * reordering; the only parallelism is an OpenMP loop over the outermost output
 * index.  It shares no code with the GPU library.
 *
 * All tensors are dense, row-major, last dimension contiguous; 4-D tensors are
 * NCHW.  Every function returns 0 on success and a positive code on an
 * argument it rejects (nothing is written then).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

enum { OR_OK = 0, OR_NULL = 1, OR_SHAPE = 3, OR_ATTR = 4 };

/* floor division for a possibly negative numerator, positive denominator */
static int64_t floordiv(int64_t a, int64_t b) {
    int64_t q = a / b;
    if ((a % b != 0) && ((a < 0) != (b < 0))) --q;
    return q;
}

/*
 * Output extent of a sliding window along one axis (Conv, MaxPool, AveragePool):
 *   floor((in + pad_begin + pad_end - ((k-1)*d + 1)) / stride) + 1,
 * with ceil instead of floor when ceil_mode is set; in ceil mode a last window
 * that would begin at or beyond the end of the input plus its leading padding
 * is dropped.  Returns -1 when the padded input is smaller than the window and
 * -2 for a non-positive kernel, stride or dilation or a negative pad.
 */
int64_t oracle_window_out(int64_t in, int64_t k, int64_t pad_begin, int64_t pad_end,
                          int64_t stride, int64_t dilation, int ceil_mode) {
    if (k < 1 || stride < 1 || dilation < 1 || pad_begin < 0 || pad_end < 0 || in < 0) return -2;
    int64_t eff = (k - 1) * dilation + 1;
    int64_t span = in + pad_begin + pad_end - eff;
    if (span < 0) return -1;
    int64_t out;
    if (ceil_mode) {
        out = floordiv(span + stride - 1, stride) + 1;
        if ((out - 1) * stride >= in + pad_begin) --out;
    } else {
        out = floordiv(span, stride) + 1;
    }
    return out;
}

/*
 * ONNX Conv, 2-D, NCHW.  X[N,C,H,W], W[M,C/group,kH,kW], optional B[M].
 *   Y[n,m,oh,ow] = B[m] + sum_{c,kh,kw} X~[n, g*Cg+c, oh*sH-pT+kh*dH, ow*sW-pL+kw*dW] * W[m,c,kh,kw]
 * with g = m / (M/group), X~ zero outside the image, no kernel flip.
 * Epilogue (the fused form the library offers): + residual[n,m,oh,ow] if given,
 * then max(.,0) if relu.  Y (double) holds N*M*OH*OW values.  If S is not NULL
 * it receives sum|x||w| + |b| + |residual| per output, the scale against which
 * an a-priori fp32 rounding bound is stated.
 */
int oracle_conv(const float* X, const int64_t xd[4], const float* Wt, const int64_t wd[4],
                const float* B, const int64_t pads[4], const int64_t strides[2],
                const int64_t dil[2], int64_t group, const float* residual, int relu,
                double* Y, double* S) {
    if (!X || !Wt || !Y) return OR_NULL;
    const int64_t N = xd[0], C = xd[1], H = xd[2], W = xd[3];
    const int64_t M = wd[0], Cg = wd[1], kH = wd[2], kW = wd[3];
    if (group < 1 || strides[0] < 1 || strides[1] < 1 || dil[0] < 1 || dil[1] < 1) return OR_ATTR;
    if (pads[0] < 0 || pads[1] < 0 || pads[2] < 0 || pads[3] < 0) return OR_ATTR;
    if (C % group || M % group || Cg * group != C) return OR_SHAPE;
    const int64_t pT = pads[0], pL = pads[1], pB = pads[2], pR = pads[3];
    const int64_t sH = strides[0], sW = strides[1], dH = dil[0], dW = dil[1];
    const int64_t OH = oracle_window_out(H, kH, pT, pB, sH, dH, 0);
    const int64_t OW = oracle_window_out(W, kW, pL, pR, sW, dW, 0);
    if (OH < 0 || OW < 0) return OR_SHAPE;
    const int64_t Mg = M / group;
    const int64_t NM = N * M;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t nm = 0; nm < NM; ++nm) {
        const int64_t n = nm / M, m = nm % M;
        const int64_t g = m / Mg;
        for (int64_t oh = 0; oh < OH; ++oh) {
            for (int64_t ow = 0; ow < OW; ++ow) {
                double acc = 0.0, mag = 0.0;
                for (int64_t c = 0; c < Cg; ++c) {
                    const float* xc = X + ((n * C + g * Cg + c) * H) * W;
                    const float* wc = Wt + ((m * Cg + c) * kH) * kW;
                    for (int64_t kh = 0; kh < kH; ++kh) {
                        const int64_t ih = oh * sH - pT + kh * dH;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t kw = 0; kw < kW; ++kw) {
                            const int64_t iw = ow * sW - pL + kw * dW;
                            if (iw < 0 || iw >= W) continue;
                            const double t = (double)xc[ih * W + iw] * (double)wc[kh * kW + kw];
                            acc += t;
                            mag += fabs(t);
                        }
                    }
                }
                const int64_t o = (nm * OH + oh) * OW + ow;
                if (B) { acc += (double)B[m]; mag += fabs((double)B[m]); }
                if (residual) { acc += (double)residual[o]; mag += fabs((double)residual[o]); }
                if (relu && !(acc > 0.0)) acc = 0.0;
                Y[o] = acc;
                if (S) S[o] = mag;
            }
        }
    }
    return OR_OK;
}

/* C operand of Gemm, unidirectionally broadcast to M x N: scalar (rank 0, or
 * every dim 1), (N), (1,N), (M,1) or (M,N). Returns element strides. */
static int gemm_c_strides(const int64_t* cd, int crank, int64_t M, int64_t N,
                          int64_t* si, int64_t* sj) {
    int64_t r = 1, c = 1;
    if (crank == 0) { r = 1; c = 1; }
    else if (crank == 1) { r = 1; c = cd[0]; }
    else if (crank == 2) { r = cd[0]; c = cd[1]; }
    else return OR_SHAPE;
    if (!((r == 1 || r == M) && (c == 1 || c == N))) return OR_SHAPE;
    *si = (r == 1) ? 0 : c;
    *sj = (c == 1) ? 0 : 1;
    return OR_OK;
}

/*
 * ONNX Gemm.  A' = transA ? A^T : A  (M x K),  B' = transB ? B^T : B  (K x N),
 *   Y[i,j] = alpha * sum_k A'[i,k] * B'[k,j] + beta * C~[i,j],
 * C~ the broadcast of C (term absent when C is NULL); then max(.,0) if relu.
 * ad/bd are the stored shapes of A and B.  S (optional) = |alpha| sum|a||b| + |beta c|.
 */
int oracle_gemm(const float* A, const int64_t ad[2], const float* B, const int64_t bd[2],
                const float* C, const int64_t* cd, int crank, float alpha, float beta,
                int transA, int transB, int relu, double* Y, double* S) {
    if (!A || !B || !Y) return OR_NULL;
    const int64_t M = transA ? ad[1] : ad[0], K = transA ? ad[0] : ad[1];
    const int64_t Kb = transB ? bd[1] : bd[0], N = transB ? bd[0] : bd[1];
    if (K != Kb) return OR_SHAPE;
    int64_t ci = 0, cj = 0;
    if (C) { int e = gemm_c_strides(cd, crank, M, N, &ci, &cj); if (e) return e; }
    const int64_t lda = ad[1], ldb = bd[1];
    const double al = (double)alpha, be = (double)beta;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0, mag = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double a = transA ? (double)A[k * lda + i] : (double)A[i * lda + k];
                const double b = transB ? (double)B[j * ldb + k] : (double)B[k * ldb + j];
                acc += a * b;
                mag += fabs(a * b);
            }
            double v = al * acc, s = fabs(al) * mag;
            if (C) { const double c = be * (double)C[i * ci + j * cj]; v += c; s += fabs(c); }
            if (relu && !(v > 0.0)) v = 0.0;
            Y[i * N + j] = v;
            if (S) S[i * N + j] = s;
        }
    }
    return OR_OK;
}

/*
 * ONNX MatMul (numpy.matmul rules).  A rank-1 A is treated as [1,K] and a rank-1
 * B as [K,1]; the inserted unit dimension is dropped from the result.  Leading
 * (batch) dimensions broadcast right-aligned: each pair is equal or one is 1.
 *   Y[..., i, j] = sum_k A[..., i, k] * B[..., k, j]
 * yd/yr receive the result shape (yd must hold max(ar,br) entries); pass
 * Y == NULL to obtain the shape only.
 */
#define OR_MAXRANK 8
int oracle_matmul(const float* A, const int64_t* ad, int ar, const float* B, const int64_t* bd,
                  int br, double* Y, double* S, int64_t* yd, int* yr) {
    if (ar < 1 || br < 1 || ar > OR_MAXRANK || br > OR_MAXRANK) return OR_SHAPE;
    int64_t a2[OR_MAXRANK + 1], b2[OR_MAXRANK + 1];
    int ra = ar, rb = br;
    if (ar == 1) { a2[0] = 1; a2[1] = ad[0]; ra = 2; } else for (int i = 0; i < ar; ++i) a2[i] = ad[i];
    if (br == 1) { b2[0] = bd[0]; b2[1] = 1; rb = 2; } else for (int i = 0; i < br; ++i) b2[i] = bd[i];
    const int64_t M = a2[ra - 2], K = a2[ra - 1], Kb = b2[rb - 2], N = b2[rb - 1];
    if (K != Kb) return OR_SHAPE;
    const int nba = ra - 2, nbb = rb - 2, nb = nba > nbb ? nba : nbb;
    int64_t bdim[OR_MAXRANK], sa[OR_MAXRANK], sb[OR_MAXRANK];
    /* element strides of each batch dim in A and B (0 where broadcast) */
    int64_t stra = M * K, strb = K * N;
    for (int t = nb - 1; t >= 0; --t) {
        const int ia = t - (nb - nba), ib = t - (nb - nbb);
        const int64_t da = ia >= 0 ? a2[ia] : 1, db = ib >= 0 ? b2[ib] : 1;
        if (da != db && da != 1 && db != 1) return OR_SHAPE;
        bdim[t] = da > db ? da : db;
        if (da == 0 || db == 0) bdim[t] = 0;
        sa[t] = (da == 1) ? 0 : stra;
        sb[t] = (db == 1) ? 0 : strb;
        stra *= da; strb *= db;
    }
    int r = 0;
    for (int t = 0; t < nb; ++t) yd[r++] = bdim[t];
    if (ar != 1) yd[r++] = M;
    if (br != 1) yd[r++] = N;
    *yr = r;
    if (!Y) return OR_OK;
    if (!A || !B) return OR_NULL;
    int64_t nbatch = 1;
    for (int t = 0; t < nb; ++t) nbatch *= bdim[t];
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int64_t z = 0; z < nbatch; ++z) {
        for (int64_t i = 0; i < M; ++i) {
            int64_t rem = z, oa = 0, ob = 0;
            for (int t = nb - 1; t >= 0; --t) {
                const int64_t idx = rem % bdim[t];
                rem /= bdim[t];
                oa += idx * sa[t];
                ob += idx * sb[t];
            }
            const float* Az = A + oa;
            const float* Bz = B + ob;
            for (int64_t j = 0; j < N; ++j) {
                double acc = 0.0, mag = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    const double t = (double)Az[i * K + k] * (double)Bz[k * N + j];
                    acc += t;
                    mag += fabs(t);
                }
                Y[(z * M + i) * N + j] = acc;
                if (S) S[(z * M + i) * N + j] = mag;
            }
        }
    }
    return OR_OK;
}

/*
 * ONNX MaxPool, 2-D, NCHW, storage_order 0.  The maximum runs over the taps that
 * fall inside the image (padding never wins).  Taps are scanned kh outer, kw
 * inner and a later tap replaces the current one only when strictly greater, so
 * ties keep the first.  Indices (optional) is the flat row-major position of
 * the winning tap in the whole N*C*H*W input.
 */
int oracle_maxpool(const float* X, const int64_t xd[4], const int64_t kernel[2],
                   const int64_t pads[4], const int64_t strides[2], const int64_t dil[2],
                   int ceil_mode, float* Y, int64_t* Ind) {
    if (!X || !Y) return OR_NULL;
    const int64_t N = xd[0], C = xd[1], H = xd[2], W = xd[3];
    const int64_t kH = kernel[0], kW = kernel[1];
    if (kH < 1 || kW < 1 || strides[0] < 1 || strides[1] < 1 || dil[0] < 1 || dil[1] < 1) return OR_ATTR;
    for (int i = 0; i < 4; ++i) if (pads[i] < 0) return OR_ATTR;
    /* a window must always contain an in-range tap */
    if (pads[0] >= (kH - 1) * dil[0] + 1 || pads[2] >= (kH - 1) * dil[0] + 1) return OR_ATTR;
    if (pads[1] >= (kW - 1) * dil[1] + 1 || pads[3] >= (kW - 1) * dil[1] + 1) return OR_ATTR;
    const int64_t OH = oracle_window_out(H, kH, pads[0], pads[2], strides[0], dil[0], ceil_mode);
    const int64_t OW = oracle_window_out(W, kW, pads[1], pads[3], strides[1], dil[1], ceil_mode);
    if (OH < 0 || OW < 0) return OR_SHAPE;
    const int64_t NC = N * C;
#pragma omp parallel for schedule(static)
    for (int64_t nc = 0; nc < NC; ++nc) {
        const float* xc = X + nc * H * W;
        for (int64_t oh = 0; oh < OH; ++oh) {
            for (int64_t ow = 0; ow < OW; ++ow) {
                int found = 0;
                float best = 0.0f;
                int64_t bi = -1;
                for (int64_t kh = 0; kh < kH; ++kh) {
                    const int64_t ih = oh * strides[0] - pads[0] + kh * dil[0];
                    if (ih < 0 || ih >= H) continue;
                    for (int64_t kw = 0; kw < kW; ++kw) {
                        const int64_t iw = ow * strides[1] - pads[1] + kw * dil[1];
                        if (iw < 0 || iw >= W) continue;
                        const float v = xc[ih * W + iw];
                        if (!found || v > best) { best = v; bi = nc * H * W + ih * W + iw; found = 1; }
                    }
                }
                const int64_t o = (nc * OH + oh) * OW + ow;
                Y[o] = best;
                if (Ind) Ind[o] = bi;
            }
        }
    }
    return OR_OK;
}

/*
 * ONNX AveragePool, 2-D, NCHW.  Sum over the in-range taps divided by the number
 * of in-range taps (count_include_pad = 0), or by the number of taps that lie
 * inside the padded image [-pT, H+pB) x [-pL, W+pR) (count_include_pad = 1;
 * that is kH*kW for every window unless ceil_mode lets the last one overhang).
 * kernel == NULL selects GlobalAveragePool: window = H x W, no pads, stride 1.
 */
int oracle_avgpool(const float* X, const int64_t xd[4], const int64_t* kernel,
                   const int64_t* pads, const int64_t* strides, int ceil_mode,
                   int count_include_pad, double* Y) {
    if (!X || !Y) return OR_NULL;
    const int64_t N = xd[0], C = xd[1], H = xd[2], W = xd[3];
    int64_t kH, kW, p[4] = {0, 0, 0, 0}, s[2] = {1, 1};
    if (kernel) {
        kH = kernel[0]; kW = kernel[1];
        if (pads) for (int i = 0; i < 4; ++i) p[i] = pads[i];
        if (strides) { s[0] = strides[0]; s[1] = strides[1]; }
    } else { kH = H; kW = W; }
    if (kH < 1 || kW < 1 || s[0] < 1 || s[1] < 1) return OR_ATTR;
    for (int i = 0; i < 4; ++i) if (p[i] < 0) return OR_ATTR;
    if (p[0] >= kH || p[2] >= kH || p[1] >= kW || p[3] >= kW) return OR_ATTR;
    const int64_t OH = oracle_window_out(H, kH, p[0], p[2], s[0], 1, ceil_mode);
    const int64_t OW = oracle_window_out(W, kW, p[1], p[3], s[1], 1, ceil_mode);
    if (OH < 0 || OW < 0) return OR_SHAPE;
    const int64_t NC = N * C;
#pragma omp parallel for schedule(static)
    for (int64_t nc = 0; nc < NC; ++nc) {
        const float* xc = X + nc * H * W;
        for (int64_t oh = 0; oh < OH; ++oh) {
            for (int64_t ow = 0; ow < OW; ++ow) {
                double acc = 0.0;
                int64_t cnt = 0, cnt_padded = 0;
                for (int64_t kh = 0; kh < kH; ++kh) {
                    const int64_t ih = oh * s[0] - p[0] + kh;
                    if (ih >= H + p[2]) continue;
                    for (int64_t kw = 0; kw < kW; ++kw) {
                        const int64_t iw = ow * s[1] - p[1] + kw;
                        if (iw >= W + p[3]) continue;
                        ++cnt_padded;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                        acc += (double)xc[ih * W + iw];
                        ++cnt;
                    }
                }
                const double div = count_include_pad ? (double)cnt_padded : (double)cnt;
                Y[(nc * OH + oh) * OW + ow] = acc / div;
            }
        }
    }
    return OR_OK;
}
