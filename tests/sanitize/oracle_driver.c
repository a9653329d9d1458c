/* The C oracle under AddressSanitizer / UndefinedBehaviorSanitizer: small GEMMs and convolutions
 * (all paddings, strides, magnitudes on and off) into exactly sized heap buffers, so that any
 * access past an operand or an output is reported. */
#include <stdio.h>
#include <stdlib.h>

void sk_oracle_gemm(int M, int N, int K, const float *A, long lda, const float *B, long ldb, double *C, long ldc,
                    double *Sabs);
void sk_oracle_conv2d_nhwc(int Nb, int H, int W, int Cin, int Cout, int R, int S, int pad_h, int pad_w, int stride,
                           const float *X, const float *Wt, double *Y, double *Sabs);
void sk_oracle_conv2d_nchw(int Nb, int H, int W, int Cin, int Cout, int R, int S, int pad_h, int pad_w, int stride,
                           const float *X, const float *Wt, double *Y, double *Sabs);

static float *filled(size_t n, unsigned seed) {
    float *p = (float *)malloc((n ? n : 1) * sizeof(float));
    for (size_t i = 0; i < n; ++i) {
        seed = seed * 1664525u + 1013904223u;
        p[i] = (float)((int)(seed >> 20) % 17 - 8) / 4.0f;
    }
    return p;
}

int main(void) {
    for (int M = 1; M <= 5; M += 2)
        for (int N = 1; N <= 7; N += 3)
            for (int K = 1; K <= 9; K += 4) {
                float *A = filled((size_t)M * K, 1u + M), *B = filled((size_t)N * K, 2u + N);
                double *C = (double *)malloc((size_t)M * N * sizeof(double));
                double *S = (double *)malloc((size_t)M * N * sizeof(double));
                sk_oracle_gemm(M, N, K, A, K, B, K, C, N, S);
                sk_oracle_gemm(M, N, K, A, K, B, K, C, N, NULL);
                free(A); free(B); free(C); free(S);
            }
    for (int H = 1; H <= 7; H += 3)
        for (int W = 1; W <= 6; W += 5)
            for (int R = 1; R <= 3; R += 2)
                for (int pad = 0; pad <= 2; ++pad)
                    for (int st = 1; st <= 3; ++st) {
                        const int S = R, Cin = 3, Cout = 2, Nb = 2;
                        if (H + 2 * pad < R || W + 2 * pad < S) continue;
                        const int Ho = (H + 2 * pad - R) / st + 1, Wo = (W + 2 * pad - S) / st + 1;
                        float *X = filled((size_t)Nb * H * W * Cin, 3u + H), *F = filled((size_t)Cout * R * S * Cin, 4u + R);
                        double *Y = (double *)malloc((size_t)Nb * Ho * Wo * Cout * sizeof(double));
                        double *Sm = (double *)malloc((size_t)Nb * Ho * Wo * Cout * sizeof(double));
                        sk_oracle_conv2d_nhwc(Nb, H, W, Cin, Cout, R, S, pad, pad, st, X, F, Y, Sm);
                        sk_oracle_conv2d_nhwc(Nb, H, W, Cin, Cout, R, S, pad, pad, st, X, F, Y, NULL);
                        sk_oracle_conv2d_nchw(Nb, H, W, Cin, Cout, R, S, pad, pad, st, X, F, Y, Sm);
                        sk_oracle_conv2d_nchw(Nb, H, W, Cin, Cout, R, S, pad, pad, st, X, F, Y, NULL);
                        free(X); free(F); free(Y); free(Sm);
                    }
    puts("oracle_driver: ok");
    return 0;
}
