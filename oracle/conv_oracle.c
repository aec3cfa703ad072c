/*
 * CPU oracle for the multi-tenant convolution path.  TEST INFRASTRUCTURE ONLY: the product library
 * never links, loads or calls anything in this directory; only tests, the smoke check and the
 * benchmark's cpu_baseline leg do.  It shares no code with the HIP path.
 *
 * What it computes.  The space-time scheduler changes where and when each tenant's layer runs, not
 * its result (Section 4: kernels of disjoint graphs are merged; Section 4.1: every tenant has its
 * own weights and inputs).  So the oracle is the plain definition of the layer, one tenant at a
 * time.  Section 4.1 expresses the layer as the im2col matrix product with M = output pixels,
 * N = filters, K = C*R*S (its worked example: 3x3, 128->128 channels, 16x16 outputs gives
 * M=256, N=128, K=1152), i.e. a dense cross-channel cross-correlation:
 *
 *   y[n,k,p,q] = sum_{c,r,s} x[n,c,p*stride-pad+r, q*stride-pad+s] * w[k,c,r,s],
 *   x = 0 outside the image,  P = floor((H+2*pad-R)/stride)+1,  Q likewise.
 *
 * All arithmetic is IEEE binary64, accumulated in the fixed order c, r, s.
 * Layouts: x NCHW, w KCRS, y NKPQ, contiguous doubles.
 *
 * The element-wise pieces a ResNet-50-shaped stack needs between conv steps (ReLU, residual add,
 * 3x3/2 max-pool, rounding of activations to bfloat16) are here too; they follow their textbook
 * definitions.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_out_dim(int in, int filt, int stride, int pad) {
    int span = in + 2 * pad - filt;
    if (span < 0 || stride <= 0) return 0;
    return span / stride + 1;
}

/* One output element, straight from the definition. */
static double conv_point(const double* x, const double* w, int C, int H, int W, int R, int S,
                         int stride, int pad, int n, int k, int p, int q) {
    double acc = 0.0;
    for (int c = 0; c < C; ++c)
        for (int r = 0; r < R; ++r) {
            int h = p * stride - pad + r;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < S; ++s) {
                int v = q * stride - pad + s;
                if (v < 0 || v >= W) continue;
                acc += x[(((size_t)n * C + c) * H + h) * W + v] *
                       w[(((size_t)k * C + c) * R + r) * S + s];
            }
        }
    return acc;
}

void oracle_conv2d_f64(const double* x, const double* w, double* y,
                       int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    const int P = oracle_out_dim(H, R, stride, pad), Q = oracle_out_dim(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q)
                    y[(((size_t)n * K + k) * P + p) * Q + q] =
                        conv_point(x, w, C, H, W, R, S, stride, pad, n, k, p, q);
}

/* Selected output elements only: idx holds npts rows of (n,k,p,q). */
void oracle_conv2d_f64_points(const double* x, const double* w, const int32_t* idx, double* out,
                              int64_t npts, int N, int C, int H, int W, int K, int R, int S,
                              int stride, int pad) {
    (void)N; (void)K;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npts; ++i)
        out[i] = conv_point(x, w, C, H, W, R, S, stride, pad,
                            idx[4 * i], idx[4 * i + 1], idx[4 * i + 2], idx[4 * i + 3]);
}

/* Max-pool with window `win`, padding treated as -infinity (never selected). NCHW. */
void oracle_maxpool2d_f64(const double* x, double* y, int N, int C, int H, int W,
                          int win, int stride, int pad) {
    const int P = oracle_out_dim(H, win, stride, pad), Q = oracle_out_dim(W, win, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double m = -INFINITY;
                    for (int r = 0; r < win; ++r) {
                        int h = p * stride - pad + r;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < win; ++s) {
                            int v = q * stride - pad + s;
                            if (v < 0 || v >= W) continue;
                            double t = x[(((size_t)n * C + c) * H + h) * W + v];
                            if (t > m) m = t;
                        }
                    }
                    y[(((size_t)n * C + c) * P + p) * Q + q] = m;
                }
}

/* Round to the nearest bfloat16 (8 exponent bits, 8 significant bits), ties to even; NaN and
 * infinities pass through; results beyond the largest finite bfloat16 become infinity. */
double oracle_round_bf16_scalar(double v) {
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e = ilogb(v);
    if (e < -126) e = -126;                 /* subnormal range: fixed spacing 2^-133 */
    double r = scalbn(rint(scalbn(v, 7 - e)), e - 7);   /* rint: ties to even by default */
    const double max_bf16 = 0x1.FEp127;
    if (fabs(r) > max_bf16) return copysign(INFINITY, v);
    return r;
}

void oracle_round_bf16(const double* in, double* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_round_bf16_scalar(in[i]);
}

int oracle_num_threads(void) {
    int t = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        t = omp_get_num_threads();
    }
#endif
    return t;
}
