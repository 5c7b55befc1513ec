/*
 * CPU oracle for the operators of a multi-tenant CNN forward pass.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain definition of every
 * operator the GPU library executes. It shares no code with the GPU path and
 * must never be linked into, or called from, the product library.
 *
 * The paper (Sec. III-A) states the workload: each tenant is a serial list of
 * operators (conv, bn, relu, pooling, ...) whose results do not depend on the
 * schedule; only the time at which an operator runs changes.  Hence the
 * oracle is simply the textbook definition of each operator, evaluated with
 * direct loops:
 *
 *   conv      Y[n,p,q,k] = act(b[k] + sum_{r,s,c} X[n, p*sh-ph+r, q*sw-pw+s, c] * W[k,r,s,c] (+ Res[n,p,q,k]))
 *   depthwise Y[n,p,q,c] = act(b[c] + sum_{r,s}   X[n, p*sh-ph+r, q*sw-pw+s, c] * W[c,r,s])
 *   max pool  window maximum, padding never selected
 *   avg pool  window mean over the in-bounds taps only
 *   global avg pool  mean over H*W
 *   fc        y[n,k] = act(b[k] + sum_j x[n,j] * W[k,j])   (x flattened in H,W,C order)
 *
 * Tensors are NHWC float arrays whose values are already representable in the
 * storage type (fp32 / fp16 / bf16).  Every sum is accumulated in double;
 * bias, residual and activation are applied in double; the result is rounded
 * ONCE to the storage type (round to nearest, ties to even) and stored.
 *
 * No im2col, no GEMM, no blocking, no intrinsics.  Output channels (or output
 * rows for the channel-wise operators) are split across OpenMP threads; that
 * is the only parallelism.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2 };
enum { ORC_ACT_NONE = 0, ORC_ACT_RELU = 1, ORC_ACT_RELU6 = 2 };

/* Round a double to the nearest value representable in the storage type,
 * ties to even (the default floating-point rounding mode is assumed, which
 * nearbyint() and the double->float cast both honour).
 * fp16: 11 significant bits, min normal exponent -14, max finite 65504.
 * bf16:  8 significant bits, min normal exponent -126, max finite (2-2^-7)*2^127. */
double orc_round_store(double v, int dtype)
{
    if (dtype == ORC_F32) return (double)(float)v;
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int sig_bits = (dtype == ORC_F16) ? 11 : 8;
    int min_exp = (dtype == ORC_F16) ? -14 : -126;
    double max_finite = (dtype == ORC_F16) ? 65504.0 : ldexp(2.0 - ldexp(1.0, -7), 127);
    int e;
    (void)frexp(v, &e);       /* |v| = m * 2^e with m in [0.5, 1) => floor(log2|v|) = e - 1 */
    e -= 1;
    if (e < min_exp) e = min_exp;          /* subnormal range: fixed quantum */
    double quantum = ldexp(1.0, e - (sig_bits - 1));
    double r = nearbyint(v / quantum) * quantum;
    /* Overflow rule of IEEE round-to-nearest: values that round beyond the
     * largest finite number become infinity. */
    if (fabs(r) > max_finite) return (v > 0) ? INFINITY : -INFINITY;
    return r;
}

static double apply_act(double v, int act)
{
    if (act == ORC_ACT_RELU) return v > 0.0 ? v : 0.0;
    if (act == ORC_ACT_RELU6) return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
    return v;
}

static int out_dim(int in, int pad, int k, int stride)
{
    return (in + 2 * pad - k) / stride + 1;
}

/* Convolution with fused bias, optional residual and activation.
 * x: [N,H,W,C] dense.  w: [K,R,S,C].  bias: [K] or NULL.
 * res: NULL or [N,P,Q,res_ctot] read at channel k.
 * y: [N,P,Q,y_ctot], written at channels y_coff .. y_coff+K-1. */
void orc_conv(const float *x, int N, int H, int W, int C,
              const float *w, int K, int R, int S,
              int stride_h, int stride_w, int pad_h, int pad_w,
              const float *bias, const float *res, int res_ctot,
              int act, int dtype,
              float *y, int y_coff, int y_ctot)
{
    int P = out_dim(H, pad_h, R, stride_h);
    int Q = out_dim(W, pad_w, S, stride_w);
    #pragma omp parallel for schedule(dynamic, 1)
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
            double acc = 0.0;
            for (int r = 0; r < R; ++r) {
                int ih = p * stride_h - pad_h + r;
                if (ih < 0 || ih >= H) continue;
                for (int s = 0; s < S; ++s) {
                    int iw = q * stride_w - pad_w + s;
                    if (iw < 0 || iw >= W) continue;
                    const float *xp = x + (((size_t)n * H + ih) * W + iw) * C;
                    const float *wp = w + (((size_t)k * R + r) * S + s) * C;
                    for (int c = 0; c < C; ++c)
                        acc += (double)xp[c] * (double)wp[c];
                }
            }
            if (bias) acc += (double)bias[k];
            size_t pix = ((size_t)n * P + p) * Q + q;
            if (res) acc += (double)res[pix * res_ctot + k];
            acc = apply_act(acc, act);
            y[pix * y_ctot + y_coff + k] = (float)orc_round_store(acc, dtype);
        }
    }
}

/* Depthwise convolution: one R x S filter per channel.  w: [C,R,S]. */
void orc_dwconv(const float *x, int N, int H, int W, int C,
                const float *w, int R, int S,
                int stride_h, int stride_w, int pad_h, int pad_w,
                const float *bias, int act, int dtype,
                float *y, int y_coff, int y_ctot)
{
    int P = out_dim(H, pad_h, R, stride_h);
    int Q = out_dim(W, pad_w, S, stride_w);
    #pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
            double acc = 0.0;
            for (int r = 0; r < R; ++r) {
                int ih = p * stride_h - pad_h + r;
                if (ih < 0 || ih >= H) continue;
                for (int s = 0; s < S; ++s) {
                    int iw = q * stride_w - pad_w + s;
                    if (iw < 0 || iw >= W) continue;
                    acc += (double)x[(((size_t)n * H + ih) * W + iw) * C + c]
                         * (double)w[((size_t)c * R + r) * S + s];
                }
            }
            if (bias) acc += (double)bias[c];
            acc = apply_act(acc, act);
            size_t pix = ((size_t)n * P + p) * Q + q;
            y[pix * y_ctot + y_coff + c] = (float)orc_round_store(acc, dtype);
        }
    }
}

/* Max pooling.  Padded positions are never selected (treated as -infinity).
 * A window with no in-bounds tap cannot occur for pad < window size. */
void orc_maxpool(const float *x, int N, int H, int W, int C,
                 int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                 int dtype, float *y, int y_coff, int y_ctot)
{
    int P = out_dim(H, pad_h, R, stride_h);
    int Q = out_dim(W, pad_w, S, stride_w);
    #pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
            double m = -INFINITY;
            for (int r = 0; r < R; ++r) {
                int ih = p * stride_h - pad_h + r;
                if (ih < 0 || ih >= H) continue;
                for (int s = 0; s < S; ++s) {
                    int iw = q * stride_w - pad_w + s;
                    if (iw < 0 || iw >= W) continue;
                    double v = (double)x[(((size_t)n * H + ih) * W + iw) * C + c];
                    if (v > m) m = v;
                }
            }
            size_t pix = ((size_t)n * P + p) * Q + q;
            y[pix * y_ctot + y_coff + c] = (float)orc_round_store(m, dtype);
        }
    }
}

/* Average pooling; the divisor is the number of in-bounds taps. */
void orc_avgpool(const float *x, int N, int H, int W, int C,
                 int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                 int dtype, float *y, int y_coff, int y_ctot)
{
    int P = out_dim(H, pad_h, R, stride_h);
    int Q = out_dim(W, pad_w, S, stride_w);
    #pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
            double acc = 0.0;
            int cnt = 0;
            for (int r = 0; r < R; ++r) {
                int ih = p * stride_h - pad_h + r;
                if (ih < 0 || ih >= H) continue;
                for (int s = 0; s < S; ++s) {
                    int iw = q * stride_w - pad_w + s;
                    if (iw < 0 || iw >= W) continue;
                    acc += (double)x[(((size_t)n * H + ih) * W + iw) * C + c];
                    ++cnt;
                }
            }
            size_t pix = ((size_t)n * P + p) * Q + q;
            y[pix * y_ctot + y_coff + c] = (float)orc_round_store(acc / (double)cnt, dtype);
        }
    }
}

/* Global average pooling: [N,H,W,C] -> [N,1,1,C]. */
void orc_global_avgpool(const float *x, int N, int H, int W, int C,
                        int dtype, float *y, int y_coff, int y_ctot)
{
    #pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int i = 0; i < H * W; ++i)
                acc += (double)x[((size_t)n * H * W + i) * C + c];
            y[(size_t)n * y_ctot + y_coff + c] =
                (float)orc_round_store(acc / (double)(H * W), dtype);
        }
    }
}

/* Fully connected layer.  x: [N,J] (an NHWC tensor flattened in H,W,C order),
 * w: [K,J], bias: [K] or NULL, y: [N,K]. */
void orc_fc(const float *x, int N, int J, const float *w, int K,
            const float *bias, int act, int dtype, float *y)
{
    #pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int j = 0; j < J; ++j)
                acc += (double)x[(size_t)n * J + j] * (double)w[(size_t)k * J + j];
            if (bias) acc += (double)bias[k];
            acc = apply_act(acc, act);
            y[(size_t)n * K + k] = (float)orc_round_store(acc, dtype);
        }
    }
}

/* Round an array in place to the storage type (used for inputs and weights). */
void orc_round_array(float *a, size_t n, int dtype)
{
    for (size_t i = 0; i < n; ++i) a[i] = (float)orc_round_store((double)a[i], dtype);
}

/* Round a double array to the storage type, into a float array (results computed in numpy in double). */
void orc_round_array_f64(const double *in, float *out, size_t n, int dtype)
{
    for (size_t i = 0; i < n; ++i) out[i] = (float)orc_round_store(in[i], dtype);
}

/* One output element of a convolution, for spot checks of large tensors. */
double orc_conv_point(const float *x, int H, int W, int C,
                      const float *w, int R, int S,
                      int stride_h, int stride_w, int pad_h, int pad_w,
                      int n, int p, int q, int k)
{
    double acc = 0.0;
    for (int r = 0; r < R; ++r) {
        int ih = p * stride_h - pad_h + r;
        if (ih < 0 || ih >= H) continue;
        for (int s = 0; s < S; ++s) {
            int iw = q * stride_w - pad_w + s;
            if (iw < 0 || iw >= W) continue;
            const float *xp = x + (((size_t)n * H + ih) * W + iw) * C;
            const float *wp = w + (((size_t)k * R + r) * S + s) * C;
            for (int c = 0; c < C; ++c) acc += (double)xp[c] * (double)wp[c];
        }
    }
    return acc;
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
