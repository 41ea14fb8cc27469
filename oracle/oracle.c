/*
 * CPU oracle for the CNN forward pass that runs on a gpu-let
 * (arXiv 2109.01611: Sec. 3.1 / Fig. 3 measure its latency L(b, p);
 * Sec. 5 says the backend runs the model's forward pass through PyTorch;
 * Table 4 lists the models).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may call it.  It shares no code
 * with the HIP library.
 *
 * The paper defines none of the operators itself; it runs PyTorch's.  Each
 * function below is therefore the textbook definition under PyTorch's
 * conventions, written out in fp64 with the loops in the obvious order:
 * activations are (N, C, H, W), convolution weights (K, C, R, S), FC weights
 * (Out, In).  No blocking, no reordering, no rounding between layers.
 * OpenMP only spreads independent (image, output-channel) planes over cores.
 */
#include <math.h>
#include <stddef.h>

/* Output extent of a window op: floor((in + 2*pad - k) / stride) + 1. */
int oracle_out_dim(int in, int k, int stride, int pad)
{
    int span = in + 2 * pad - k;
    if (span < 0 || stride <= 0)
        return 0;
    return span / stride + 1;
}

/*
 * Convolution as cross-correlation (the kernel is not flipped):
 *   y[n,k,p,q] = b[k] + sum_{c,r,s} xz[n,c,p*stride-pad+r,q*stride-pad+s] * w[k,c,r,s]
 * where xz is x extended by zeros outside 0<=h<H, 0<=w<W.  Then, if
 * `residual` is not NULL, residual[n,k,p,q] is added; then, if `relu`,
 * negative values become +0.  `b` may be NULL (no bias).
 */
void oracle_conv2d(const double *x, const double *w, const double *b, const double *residual,
                   double *y, int N, int C, int H, int W, int K, int R, int S, int stride,
                   int pad, int relu)
{
    const int P = oracle_out_dim(H, R, stride, pad);
    const int Q = oracle_out_dim(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double acc = b ? b[k] : 0.0;
                    for (int c = 0; c < C; ++c) {
                        for (int r = 0; r < R; ++r) {
                            const int h = p * stride - pad + r;
                            if (h < 0 || h >= H)
                                continue;
                            for (int s = 0; s < S; ++s) {
                                const int v = q * stride - pad + s;
                                if (v < 0 || v >= W)
                                    continue;
                                acc += x[(((size_t)n * C + c) * H + h) * W + v] *
                                       w[(((size_t)k * C + c) * R + r) * S + s];
                            }
                        }
                    }
                    const size_t o = (((size_t)n * K + k) * P + p) * Q + q;
                    if (residual)
                        acc += residual[o];
                    if (relu && !(acc > 0.0))
                        acc = 0.0;
                    y[o] = acc;
                }
            }
        }
    }
}

/*
 * Depthwise convolution (one filter per channel, as in the depthwise-separable
 * blocks of MobileNet; the SSD-MobileNet of the paper's Table 4):
 *   y[n,c,p,q] = b[c] + sum_{r,s} xz[n,c,p*stride-pad+r,q*stride-pad+s] * w[c,r,s]
 * with the same zero extension, bias and ReLU rules as oracle_conv2d.
 */
void oracle_depthwise_conv2d(const double *x, const double *w, const double *b, double *y, int N, int C,
                             int H, int W, int R, int S, int stride, int pad, int relu)
{
    const int P = oracle_out_dim(H, R, stride, pad);
    const int Q = oracle_out_dim(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c) {
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double acc = b ? b[c] : 0.0;
                    for (int r = 0; r < R; ++r) {
                        const int h = p * stride - pad + r;
                        if (h < 0 || h >= H)
                            continue;
                        for (int s = 0; s < S; ++s) {
                            const int v = q * stride - pad + s;
                            if (v < 0 || v >= W)
                                continue;
                            acc += x[(((size_t)n * C + c) * H + h) * W + v] * w[((size_t)c * R + r) * S + s];
                        }
                    }
                    if (relu && !(acc > 0.0))
                        acc = 0.0;
                    y[(((size_t)n * C + c) * P + p) * Q + q] = acc;
                }
            }
        }
    }
}

/*
 * Max pooling over a k x k window: only taps inside the image take part
 * (padding acts as minus infinity).  A window with no tap inside the image
 * cannot occur when pad < k.
 */
void oracle_maxpool(const double *x, double *y, int N, int C, int H, int W, int k, int stride,
                    int pad)
{
    const int P = oracle_out_dim(H, k, stride, pad);
    const int Q = oracle_out_dim(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c) {
            const double *xp = x + ((size_t)n * C + c) * H * W;
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double m = -INFINITY;
                    for (int r = 0; r < k; ++r) {
                        const int h = p * stride - pad + r;
                        if (h < 0 || h >= H)
                            continue;
                        for (int s = 0; s < k; ++s) {
                            const int v = q * stride - pad + s;
                            if (v < 0 || v >= W)
                                continue;
                            if (xp[(size_t)h * W + v] > m)
                                m = xp[(size_t)h * W + v];
                        }
                    }
                    y[(((size_t)n * C + c) * P + p) * Q + q] = m;
                }
            }
        }
    }
}

/*
 * Average pooling over a k x k window, PyTorch's default convention:
 * padding taps count as zeros and the divisor is always k*k.
 */
void oracle_avgpool(const double *x, double *y, int N, int C, int H, int W, int k, int stride,
                    int pad)
{
    const int P = oracle_out_dim(H, k, stride, pad);
    const int Q = oracle_out_dim(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c) {
            const double *xp = x + ((size_t)n * C + c) * H * W;
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double sum = 0.0;
                    for (int r = 0; r < k; ++r) {
                        const int h = p * stride - pad + r;
                        if (h < 0 || h >= H)
                            continue;
                        for (int s = 0; s < k; ++s) {
                            const int v = q * stride - pad + s;
                            if (v < 0 || v >= W)
                                continue;
                            sum += xp[(size_t)h * W + v];
                        }
                    }
                    y[(((size_t)n * C + c) * P + p) * Q + q] = sum / (double)(k * k);
                }
            }
        }
    }
}

/* Global average pooling: y[n,c] = mean over the H*W plane. */
void oracle_global_avgpool(const double *x, double *y, int N, int C, int H, int W)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c) {
            const double *xp = x + ((size_t)n * C + c) * H * W;
            double sum = 0.0;
            for (int i = 0; i < H * W; ++i)
                sum += xp[i];
            y[(size_t)n * C + c] = sum / (double)(H * W);
        }
    }
}

/*
 * Fully connected layer: y[n,o] = b[o] + sum_i x[n,i] * w[o,i], optional ReLU.
 * `b` may be NULL.
 */
void oracle_fc(const double *x, const double *w, const double *b, double *y, int N, int In,
               int Out, int relu)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int o = 0; o < Out; ++o) {
            double acc = b ? b[o] : 0.0;
            for (int i = 0; i < In; ++i)
                acc += x[(size_t)n * In + i] * w[(size_t)o * In + i];
            if (relu && !(acc > 0.0))
                acc = 0.0;
            y[(size_t)n * Out + o] = acc;
        }
    }
}

/* Number of host threads the loops above spread over. */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
