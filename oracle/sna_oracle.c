/*
 * CPU oracle primitives for SubNetAct's WeightSlice layers -- TEST INFRASTRUCTURE.
 *
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * use this file; the GPU library shares nothing with it.
 *
 * Each routine is the textbook sum for its layer, evaluated directly on the
 * max-size SuperNet weight tensor: WeightSlice (section "SubNetAct", WeightSlice
 * paragraph) hands a layer the number of active output / input channels, and
 * the layer reads the leading [0:K, 0:C] block (and, for an elastic kernel, the
 * centre k x k window) of the shared weights through the tensor's own strides.
 * Nothing is copied, blocked or reordered beyond the loop nest written here.
 *
 * Activations are double precision, NHWC, densely packed at their ACTIVE channel
 * count.  Weights are float (they hold fp32 or bf16-representable values).
 * Every product and every sum is carried out in double.
 */
#include <stddef.h>

/* y[n,p,q,k] = sum_{r<R, s<S, c<C} x[n, p*stride+r-pad, q*stride+s-pad, c]
 *                                  * w[k*wk + (r0+r)*wr + (s0+s)*ws + c]
 * with x taken as zero outside [0,H) x [0,W).
 * (wk, wr, ws) are the element strides of the stored max-size tensor
 * [K_max][R_max][S_max][C_max]; (r0, s0) is the window's offset inside the
 * stored kernel.  Ho, Wo are given by the caller. */
void ora_conv2d(const double *x, int N, int H, int W, int C,
                const float *w, long wk, long wr, long ws,
                int K, int R, int S, int r0, int s0,
                int stride, int pad,
                double *y, int Ho, int Wo)
{
#pragma omp parallel for collapse(3) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < Ho; ++p)
            for (int k = 0; k < K; ++k)
                for (int q = 0; q < Wo; ++q) {
                    double acc = 0.0;
                    for (int r = 0; r < R; ++r) {
                        int ih = p * stride + r - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            int iw = q * stride + s - pad;
                            if (iw < 0 || iw >= W) continue;
                            const double *xp = x + (((size_t)n * H + ih) * W + iw) * C;
                            const float *wp = w + (size_t)k * wk + (size_t)(r0 + r) * wr
                                                + (size_t)(s0 + s) * ws;
                            double a = 0.0;
#pragma omp simd reduction(+ : a)
                            for (int c = 0; c < C; ++c)
                                a += xp[c] * (double)wp[c];
                            acc += a;
                        }
                    }
                    y[(((size_t)n * Ho + p) * Wo + q) * K + k] = acc;
                }
}

/* Depthwise: y[n,p,q,c] = sum_{r<R, s<S} x[n, p*stride+r-pad, q*stride+s-pad, c]
 *                                        * w[(r0+r)*wr + (s0+s)*ws + c],  c < C.
 * Stored tensor [R_max][S_max][C_max]. */
void ora_depthwise(const double *x, int N, int H, int W, int C,
                   const float *w, long wr, long ws,
                   int R, int S, int r0, int s0,
                   int stride, int pad,
                   double *y, int Ho, int Wo)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < Ho; ++p)
            for (int q = 0; q < Wo; ++q) {
                double *yp = y + (((size_t)n * Ho + p) * Wo + q) * C;
                for (int c = 0; c < C; ++c) yp[c] = 0.0;
                for (int r = 0; r < R; ++r) {
                    int ih = p * stride + r - pad;
                    if (ih < 0 || ih >= H) continue;
                    for (int s = 0; s < S; ++s) {
                        int iw = q * stride + s - pad;
                        if (iw < 0 || iw >= W) continue;
                        const double *xp = x + (((size_t)n * H + ih) * W + iw) * C;
                        const float *wp = w + (size_t)(r0 + r) * wr + (size_t)(s0 + s) * ws;
                        for (int c = 0; c < C; ++c)
                            yp[c] += xp[c] * (double)wp[c];
                    }
                }
            }
}

/* y[m,k] = sum_{c<C} x[m*xs + c] * w[k*wk + c],  k < K  (no bias).
 * xs is the row stride of x (>= C); wk the row stride of the stored
 * [K_max][C_max] matrix. */
void ora_linear(const double *x, int M, long xs, int C,
                const float *w, long wk, int K,
                double *y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k) {
            const double *xp = x + (size_t)m * xs;
            const float *wp = w + (size_t)k * wk;
            double a = 0.0;
#pragma omp simd reduction(+ : a)
            for (int c = 0; c < C; ++c)
                a += xp[c] * (double)wp[c];
            y[(size_t)m * K + k] = a;
        }
}
