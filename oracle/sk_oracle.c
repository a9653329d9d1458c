/*
 * CPU oracle for the coalesced-superkernel path -- TEST INFRASTRUCTURE ONLY.
 *
 * The paper's superkernel (Sections 1 and 5.3) packs many mutually independent
 * tensor operators from separate inference streams into one launch.  Packing
 * changes the schedule, not the mathematics: each operator's result is still
 * the plain product C = A.B of the GEMM that backs it (Section 5.3, Figure 6
 * caption: a convolution is executed through the SGEMM behind it, coalesced
 * via a batched GEMM).  The oracle is therefore that plain definition, one
 * operator at a time, accumulated in fp64, written as the textbook loops with
 * no blocking, fusion or reordering.
 *
 * Inputs are float arrays holding values that are already rounded to the
 * problem's storage type (bf16 / fp16 / fp32 values are all exact in a float);
 * every product and sum is done in double.
 *
 * Nothing in the product path may link, import or call this file.  It shares
 * no code, header, table or constant with the HIP implementation.
 *
 * Parity pins (tests/test_oracle_*.py): hand-computed 2x2 / 3x3 GEMM and
 * convolution examples, closed forms (rank-one, identity, unit vector),
 * numpy's fp64 matmul on random inputs, 1x1 convolution == GEMM, direct
 * convolution == explicit patch matrix times GEMM, centre-tap delta filter;
 * the NCHW form against the NHWC form on permuted arrays, against a library
 * 2-D correlation per channel pair, and against hand examples.
 */
#include <math.h>
#include <stddef.h>

/* C[m,n] = sum_k A[m,k] * B[n,k]   (B is stored K-contiguous, i.e. as the
 * transpose of the mathematical K x N operand).  k ascends.
 * If S is non-NULL it receives S[m,n] = sum_k |A[m,k]| * |B[n,k]|, the
 * magnitude sum used for summation-order-independent error bounds.
 * lda, ldb, ldc: row strides in elements (S uses ldc too). */
void sk_oracle_gemm(int M, int N, int K,
                    const float *A, long lda,
                    const float *B, long ldb,
                    double *C, long ldc, double *S)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double sum = 0.0, mag = 0.0;
            for (int k = 0; k < K; ++k) {
                double a = (double)A[(size_t)m * lda + k];
                double b = (double)B[(size_t)n * ldb + k];
                sum += a * b;
                mag += fabs(a) * fabs(b);
            }
            C[(size_t)m * ldc + n] = sum;
            if (S) S[(size_t)m * ldc + n] = mag;
        }
    }
}

/* Direct NHWC convolution (cross-correlation: the filter is NOT flipped),
 * the same stride in both directions, dilation 1, one group, zero padding:
 *   Y[b,ho,wo,co] = sum_{r,s,c} X[b, ho*stride-pad_h+r, wo*stride-pad_w+s, c] * W[co,r,s,c]
 * where taps that fall outside the image contribute nothing.
 *   Ho = (H + 2*pad_h - R) / stride + 1,  Wo = (W + 2*pad_w - S) / stride + 1
 * (integer division: the filter positions that fit the padded image).
 * X is [Nb,H,W,Cin], W is [Cout,R,S,Cin], Y (and Sabs, if non-NULL) are
 * [Nb,Ho,Wo,Cout], all dense. */
void sk_oracle_conv2d_nhwc(int Nb, int H, int W, int Cin, int Cout,
                           int R, int S, int pad_h, int pad_w, int stride,
                           const float *X, const float *Wt,
                           double *Y, double *Sabs)
{
    const int Ho = (H + 2 * pad_h - R) / stride + 1;
    const int Wo = (W + 2 * pad_w - S) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < Nb; ++b) {
        for (int ho = 0; ho < Ho; ++ho) {
            for (int wo = 0; wo < Wo; ++wo) {
                for (int co = 0; co < Cout; ++co) {
                    double sum = 0.0, mag = 0.0;
                    for (int r = 0; r < R; ++r) {
                        const int h = ho * stride - pad_h + r;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int w = wo * stride - pad_w + s;
                            if (w < 0 || w >= W) continue;
                            const float *x = X + (((size_t)b * H + h) * W + w) * Cin;
                            const float *f = Wt + (((size_t)co * R + r) * S + s) * Cin;
                            for (int c = 0; c < Cin; ++c) {
                                double a = (double)x[c];
                                double g = (double)f[c];
                                sum += a * g;
                                mag += fabs(a) * fabs(g);
                            }
                        }
                    }
                    const size_t o = (((size_t)b * Ho + ho) * Wo + wo) * Cout + co;
                    Y[o] = sum;
                    if (Sabs) Sabs[o] = mag;
                }
            }
        }
    }
}

/* The same convolution on channel-major arrays (the other common storage
 * order of inference frameworks): X is [Nb,Cin,H,W], W is [Cout,Cin,R,S],
 * Y (and Sabs, if non-NULL) are [Nb,Cout,Ho,Wo], all dense:
 *   Y[b,co,ho,wo] = sum_{c,r,s} X[b, c, ho*stride-pad_h+r, wo*stride-pad_w+s] * W[co,c,r,s]
 * Same output size, same treatment of taps outside the image. */
void sk_oracle_conv2d_nchw(int Nb, int H, int W, int Cin, int Cout,
                           int R, int S, int pad_h, int pad_w, int stride,
                           const float *X, const float *Wt,
                           double *Y, double *Sabs)
{
    const int Ho = (H + 2 * pad_h - R) / stride + 1;
    const int Wo = (W + 2 * pad_w - S) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < Nb; ++b) {
        for (int co = 0; co < Cout; ++co) {
            for (int ho = 0; ho < Ho; ++ho) {
                for (int wo = 0; wo < Wo; ++wo) {
                    double sum = 0.0, mag = 0.0;
                    for (int c = 0; c < Cin; ++c) {
                        for (int r = 0; r < R; ++r) {
                            const int h = ho * stride - pad_h + r;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int w = wo * stride - pad_w + s;
                                if (w < 0 || w >= W) continue;
                                double a = (double)X[(((size_t)b * Cin + c) * H + h) * W + w];
                                double g = (double)Wt[(((size_t)co * Cin + c) * R + r) * S + s];
                                sum += a * g;
                                mag += fabs(a) * fabs(g);
                            }
                        }
                    }
                    const size_t o = (((size_t)b * Cout + co) * Ho + ho) * Wo + wo;
                    Y[o] = sum;
                    if (Sabs) Sabs[o] = mag;
                }
            }
        }
    }
}
