/*
 * fp64 CPU oracle for the five operator programs of the Ansor evaluation
 * (arXiv 2006.06762): GMM, C2D, DEP (single-operator benchmark, Sec. 7.1 and
 * Appendix C) and the ConvLayer / TBS subgraphs (Sec. 7.2).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the HIP kernels can be
 * compared element by element with the plain mathematical definition of each
 * operator.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it; the product path never does.  It shares no code, header, table
 * or helper with the HIP path.
 *
 * Every function is the definition written out as nested loops: no blocking,
 * no im2col, no BLAS, no reordering.  Inputs are the fp32 values the GPU gets,
 * widened to double; all arithmetic and the result are double.  The only
 * concession to run time is an OpenMP "parallel for" over the outermost
 * independent loop (the iterations never share an accumulator, so the result
 * does not depend on the thread count).
 *
 * All tensors are packed (no strides) except the GEMM, which takes row-major
 * leading dimensions as the matmul definition's natural generalisation.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the parallel loops will use (1 without OpenMP). */
int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * GMM, Sec. 4.1 (the matmul used to explain rule 3): C(i,j) = sum_k A[i,k] * B[k,j].
 * Row-major, element (i,k) of A at A[i*lda+k]; "batch" independent products
 * whose operands are strideA/strideB/strideC elements apart (the benchmark's
 * batch size for GMM, Sec. 7.1).
 */
void orc_gemm(int64_t M, int64_t N, int64_t K,
              const float *A, int64_t lda, const float *B, int64_t ldb,
              double *C, int64_t ldc,
              int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC)
{
    for (int64_t b = 0; b < batch; ++b) {
        const float *Ab = A + b * strideA;
        const float *Bb = B + b * strideB;
        double *Cb = C + b * strideC;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < M; ++i) {
            for (int64_t j = 0; j < N; ++j) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    acc += (double)Ab[i * lda + k] * (double)Bb[k * ldb + j];
                Cb[i * ldc + j] = acc;
            }
        }
    }
}

/*
 * C2D, Sec. 7.1 / Appendix C (fields: height, width, input channels, output
 * channels, kernel size, stride, padding).  Cross-correlation (no kernel
 * flip), zero padding of pad_h/pad_w on both sides, output extent
 * floor((H + 2*pad - R)/stride) + 1.  x is NCHW [N,C,H,W], w is OIHW
 * [K,C,R,S], y is NCHW [N,K,OH,OW] with OH, OW as computed by the caller by
 * the same formula.
 */
void orc_conv2d(int N, int C, int H, int W, int K, int R, int S,
                int stride_h, int stride_w, int pad_h, int pad_w,
                const float *x, const float *w, double *y)
{
    const int OH = (H + 2 * pad_h - R) / stride_h + 1;
    const int OW = (W + 2 * pad_w - S) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int oh = 0; oh < OH; ++oh) {
                for (int ow = 0; ow < OW; ++ow) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c) {
                        for (int r = 0; r < R; ++r) {
                            const int ih = oh * stride_h - pad_h + r;
                            if (ih < 0 || ih >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int iw = ow * stride_w - pad_w + s;
                                if (iw < 0 || iw >= W) continue;
                                const double xv = x[(((size_t)n * C + c) * H + ih) * W + iw];
                                const double wv = w[(((size_t)k * C + c) * R + r) * S + s];
                                acc += xv * wv;
                            }
                        }
                    }
                    y[(((size_t)n * K + k) * OH + oh) * OW + ow] = acc;
                }
            }
        }
    }
}

/*
 * ConvLayer, Sec. 7.2: 2-D convolution, then batch normalisation, then ReLU.
 * Inference-time batch norm with per-output-channel running statistics,
 *     y = gamma * (v - mean) / sqrt(var + eps) + beta,
 * applied in this unfolded form (no pre-computed scale/shift), then
 * max(y, 0).  The four vectors have length K.
 */
void orc_conv_bn_relu(int N, int C, int H, int W, int K, int R, int S,
                      int stride_h, int stride_w, int pad_h, int pad_w,
                      const float *x, const float *w,
                      const float *gamma, const float *beta,
                      const float *mean, const float *var, float eps,
                      double *y)
{
    const int OH = (H + 2 * pad_h - R) / stride_h + 1;
    const int OW = (W + 2 * pad_w - S) / stride_w + 1;
    orc_conv2d(N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, x, w, y);
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            const double g = gamma[k], b = beta[k], mu = mean[k];
            const double denom = sqrt((double)var[k] + (double)eps);
            double *plane = y + ((size_t)n * K + k) * OH * OW;
            for (int p = 0; p < OH * OW; ++p) {
                const double v = g * (plane[p] - mu) / denom + b;
                plane[p] = v > 0.0 ? v : 0.0;
            }
        }
    }
}

/*
 * GRP and DIL, Sec. 7.1 / Appendix C (fields as C2D plus "groups", resp.
 * "dilation"): the convolution above with the two generalisations the paper's
 * operator list names.
 *   dilation d: tap (r, s) reads input row oh*stride - pad + r*d_h and column
 *     ow*stride - pad + s*d_w; output extent
 *     floor((H + 2*pad - d*(R-1) - 1)/stride) + 1.
 *   groups g: input and output channels are cut into g equal runs; output
 *     channel k of run k / (K/g) only sees the C/g input channels of the same
 *     run.  w is [K, C/g, R, S].
 * g = 1, d = 1 is orc_conv2d.  Returns 0, or -1 when C or K is not a multiple
 * of the group count.
 */
int orc_conv2d_general(int N, int C, int H, int W, int K, int R, int S,
                       int stride_h, int stride_w, int pad_h, int pad_w,
                       int dil_h, int dil_w, int groups,
                       const float *x, const float *w, double *y)
{
    if (groups < 1 || C % groups != 0 || K % groups != 0) return -1;
    const int Cg = C / groups, Kg = K / groups;
    const int OH = (H + 2 * pad_h - dil_h * (R - 1) - 1) / stride_h + 1;
    const int OW = (W + 2 * pad_w - dil_w * (S - 1) - 1) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            const int g = k / Kg;
            for (int oh = 0; oh < OH; ++oh) {
                for (int ow = 0; ow < OW; ++ow) {
                    double acc = 0.0;
                    for (int cg = 0; cg < Cg; ++cg) {
                        const int c = g * Cg + cg;
                        for (int r = 0; r < R; ++r) {
                            const int ih = oh * stride_h - pad_h + r * dil_h;
                            if (ih < 0 || ih >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int iw = ow * stride_w - pad_w + s * dil_w;
                                if (iw < 0 || iw >= W) continue;
                                const double xv = x[(((size_t)n * C + c) * H + ih) * W + iw];
                                const double wv = w[(((size_t)k * Cg + cg) * R + r) * S + s];
                                acc += xv * wv;
                            }
                        }
                    }
                    y[(((size_t)n * K + k) * OH + oh) * OW + ow] = acc;
                }
            }
        }
    }
    return 0;
}

/*
 * DEP, Sec. 7.1 / Appendix C (fields: height, width, channels, kernel size,
 * stride, padding): depthwise convolution with channel multiplier 1.  Channel
 * c of the output only sees channel c of the input.  w is [C,1,R,S].
 */
void orc_dwconv(int N, int C, int H, int W, int R, int S,
                int stride_h, int stride_w, int pad_h, int pad_w,
                const float *x, const float *w, double *y)
{
    const int OH = (H + 2 * pad_h - R) / stride_h + 1;
    const int OW = (W + 2 * pad_w - S) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c) {
            const float *xp = x + ((size_t)n * C + c) * H * W;
            const float *wp = w + (size_t)c * R * S;
            for (int oh = 0; oh < OH; ++oh) {
                for (int ow = 0; ow < OW; ++ow) {
                    double acc = 0.0;
                    for (int r = 0; r < R; ++r) {
                        const int ih = oh * stride_h - pad_h + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int iw = ow * stride_w - pad_w + s;
                            if (iw < 0 || iw >= W) continue;
                            acc += (double)xp[(size_t)ih * W + iw] * (double)wp[r * S + s];
                        }
                    }
                    y[(((size_t)n * C + c) * OH + oh) * OW + ow] = acc;
                }
            }
        }
    }
}

/*
 * NRM, Sec. 7.1 / Appendix C (fields: N, M): "matrix 2-norm", named in Sec. 4.1
 * as the example of an operator with almost no parallelism in its space
 * dimensions and ample parallelism in its reduction dimensions, i.e. a plain
 * reduction over all entries of a matrix to one number.  Reading: the entrywise
 * 2-norm  out[b] = sqrt(sum_{i,j} x[b,i,j]^2)  of each N x M matrix of the batch
 * (row stride ld, matrix stride `stride`, in elements).
 */
void orc_nrm(int64_t batch, int64_t N, int64_t M, int64_t ld, int64_t stride,
             const float *x, double *out)
{
    for (int64_t b = 0; b < batch; ++b) {
        const float *xb = x + b * stride;
        double acc = 0.0;
        for (int64_t i = 0; i < N; ++i)
            for (int64_t j = 0; j < M; ++j) {
                const double v = xb[i * ld + j];
                acc += v * v;
            }
        out[b] = sqrt(acc);
    }
}

/*
 * TBS without its softmax ("TBG"), Sec. 7.2: two matrix transposes and one
 * batch matrix multiplication of multi-head attention.  q and k are
 * [B,S,H,D].  Step 1 and 2: materialise the transposed copies qt, kt =
 * [B,H,S,D].  Step 3: for every (b,h), out = qt . kt^T, an S x S matrix.
 * out is [B,H,S,S].  No 1/sqrt(D) scaling.  Returns 0, or -1 if the two
 * temporaries cannot be allocated.
 */
int orc_tbg(int B, int S, int H, int D, const float *q, const float *k, double *out)
{
    const size_t n = (size_t)B * S * H * D;
    double *qt = (double *)malloc(n * sizeof(double));
    double *kt = (double *)malloc(n * sizeof(double));
    if (!qt || !kt) { free(qt); free(kt); return -1; }

    for (int b = 0; b < B; ++b)
        for (int s = 0; s < S; ++s)
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d) {
                    const size_t src = (((size_t)b * S + s) * H + h) * D + d;
                    const size_t dst = (((size_t)b * H + h) * S + s) * D + d;
                    qt[dst] = q[src];
                    kt[dst] = k[src];
                }

#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const double *qm = qt + ((size_t)b * H + h) * S * D;
            const double *km = kt + ((size_t)b * H + h) * S * D;
            double *om = out + ((size_t)b * H + h) * S * S;
            for (int i = 0; i < S; ++i) {
                for (int j = 0; j < S; ++j) {
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d)
                        acc += qm[(size_t)i * D + d] * km[(size_t)j * D + d];
                    om[(size_t)i * S + j] = acc;
                }
            }
        }
    }
    free(qt);
    free(kt);
    return 0;
}

/*
 * Full TBS, Sec. 7.2: the batch matmul above followed by a softmax over the
 * last axis (each row of every S x S score matrix), computed as
 * exp(v - rowmax) / sum exp(v - rowmax).
 */
int orc_tbs(int B, int S, int H, int D, const float *q, const float *k, double *out)
{
    if (orc_tbg(B, S, H, D, q, k, out) != 0) return -1;
    const size_t rows = (size_t)B * H * S;
#pragma omp parallel for schedule(static)
    for (size_t r = 0; r < rows; ++r) {
        double *v = out + r * S;
        double mx = v[0];
        for (int j = 1; j < S; ++j) if (v[j] > mx) mx = v[j];
        double sum = 0.0;
        for (int j = 0; j < S; ++j) { v[j] = exp(v[j] - mx); sum += v[j]; }
        for (int j = 0; j < S; ++j) v[j] /= sum;
    }
    return 0;
}
