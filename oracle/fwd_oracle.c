/*
 * CPU oracle for the forward passes of the co-located inference models.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library's outputs are compared with; nothing in the product path may link or
 * call it.  It shares no code with the GPU kernels.
 *
 * The paper co-locates stock DNN inference models (Sec. IV-A, "Inference
 * Models") and defines no network arithmetic of its own, so every routine here
 * is the textbook definition of the operator, written as its defining sum:
 * activations are fp64, parameters are fp32 values (each exactly representable
 * in the model's storage type), every accumulation is fp64, and nothing is
 * rounded between layers.  Logical layouts: images [N][C][H][W], sequences
 * [N][S][Hd], parameters as in the operator's usual definition.
 *
 * Parity pins (tests/test_oracle_forward.py): identity-kernel convolution,
 * all-ones closed form with borders, 1x1 convolution == linear == fp64 matmul,
 * nested-loop brute force on tiny tensors, an independent fp64 library
 * convolution / pooling / normalisation / attention, softmax row sums and shift
 * invariance, LayerNorm moments, attention with equal keys == mean of V,
 * GELU against erf.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_GELU = 3 };

static double act_apply(int act, double v)
{
    switch (act) {
    case ACT_RELU:  return v > 0.0 ? v : 0.0;
    case ACT_RELU6: return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
    case ACT_GELU:  return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));   /* exact (erf) form */
    default:        return v;
    }
}

/* y = act(x + bias[channel] + res); channel = (i / inner) % channels. bias/res may be NULL. */
void orc_eltwise(const double *x, const float *bias, const double *res, double *y,
                 int64_t n, int64_t channels, int64_t inner, int act)
{
#pragma omp parallel for
    for (int64_t i = 0; i < n; ++i) {
        double v = x[i];
        if (bias) v += (double)bias[(i / inner) % channels];
        if (res) v += res[i];
        y[i] = act_apply(act, v);
    }
}

/* Cross-correlation with zero padding and channel groups.
 * y[n,co,oh,ow] = b[co] + sum_{ci,kh,kw} x[n, g*cig+ci, oh*s-p+kh, ow*s-p+kw] * w[co,ci,kh,kw] */
void orc_conv2d(const double *x, int N, int C, int H, int W,
                const float *w, const float *b, int Cout, int KH, int KW,
                int stride, int pad, int groups, double *y)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
    const int cig = C / groups, cog = Cout / groups;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Cout; ++co) {
            const int g = co / cog;
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = b ? (double)b[co] : 0.0;
                    for (int ci = 0; ci < cig; ++ci)
                        for (int kh = 0; kh < KH; ++kh) {
                            const int ih = oh * stride - pad + kh;
                            if (ih < 0 || ih >= H) continue;
                            for (int kw = 0; kw < KW; ++kw) {
                                const int iw = ow * stride - pad + kw;
                                if (iw < 0 || iw >= W) continue;
                                acc += x[(((size_t)n * C + g * cig + ci) * H + ih) * W + iw] *
                                       (double)w[(((size_t)co * cig + ci) * KH + kh) * KW + kw];
                            }
                        }
                    y[(((size_t)n * Cout + co) * Ho + oh) * Wo + ow] = acc;
                }
        }
}

/* y[m,n] = b[n] + sum_k x[m,k] * w[n,k] */
void orc_linear(const double *x, int64_t M, int64_t K, const float *w, const float *b, int64_t Nn, double *y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < Nn; ++n) {
            double acc = b ? (double)b[n] : 0.0;
            const double *xr = x + m * K;
            const float *wr = w + n * K;
            for (int64_t k = 0; k < K; ++k) acc += xr[k] * (double)wr[k];
            y[m * Nn + n] = acc;
        }
}

/* max over the window; positions outside the image count as -infinity */
void orc_maxpool(const double *x, int N, int C, int H, int W, int KH, int KW, int stride, int pad, double *y)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1;
    const int Wo = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for
    for (int nc = 0; nc < N * C; ++nc)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow) {
                double m = -INFINITY;
                for (int kh = 0; kh < KH; ++kh)
                    for (int kw = 0; kw < KW; ++kw) {
                        const int ih = oh * stride - pad + kh, iw = ow * stride - pad + kw;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                        const double v = x[((size_t)nc * H + ih) * W + iw];
                        if (v > m) m = v;
                    }
                y[((size_t)nc * Ho + oh) * Wo + ow] = m;
            }
}

/* mean over H*W */
void orc_gap(const double *x, int N, int C, int HW, double *y)
{
#pragma omp parallel for
    for (int nc = 0; nc < N * C; ++nc) {
        double s = 0.0;
        for (int i = 0; i < HW; ++i) s += x[(size_t)nc * HW + i];
        y[nc] = s / (double)HW;
    }
}

/* y = (x - mean) / sqrt(var + eps) * gamma + beta, biased variance, per row */
void orc_layernorm(const double *x, int64_t rows, int64_t width, const float *gamma, const float *beta,
                   double eps, double *y)
{
#pragma omp parallel for
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * width;
        double mean = 0.0, var = 0.0;
        for (int64_t i = 0; i < width; ++i) mean += xr[i];
        mean /= (double)width;
        for (int64_t i = 0; i < width; ++i) var += (xr[i] - mean) * (xr[i] - mean);
        var /= (double)width;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int64_t i = 0; i < width; ++i)
            y[r * width + i] = (xr[i] - mean) * rstd * (gamma ? (double)gamma[i] : 1.0) + (beta ? (double)beta[i] : 0.0);
    }
}

/* y_i = exp(x_i - max) / sum_j exp(x_j - max), per row */
void orc_softmax(const double *x, int64_t rows, int64_t width, double *y)
{
#pragma omp parallel for
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * width;
        double m = xr[0], s = 0.0;
        for (int64_t i = 1; i < width; ++i) if (xr[i] > m) m = xr[i];
        for (int64_t i = 0; i < width; ++i) s += exp(xr[i] - m);
        for (int64_t i = 0; i < width; ++i) y[r * width + i] = exp(xr[i] - m) / s;
    }
}

/* qkv: [B][S][3*Hd] with q at column 0, k at Hd, v at 2*Hd, each split head-major into `heads`
 * slices of d = Hd/heads.  out[b,s,h*d+j] = sum_t softmax_t(q_s . k_t / sqrt(d)) * v_t[j] */
void orc_attention(const double *qkv, int B, int S, int Hd, int heads, double *out, double *scratch /* B*heads*S */)
{
    const int d = Hd / heads;
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h) {
            double *p = scratch + ((size_t)b * heads + h) * S;
            for (int s = 0; s < S; ++s) {
                const double *q = qkv + ((size_t)b * S + s) * 3 * Hd + h * d;
                double m = -INFINITY, sum = 0.0;
                for (int t = 0; t < S; ++t) {
                    const double *k = qkv + ((size_t)b * S + t) * 3 * Hd + Hd + h * d;
                    double dot = 0.0;
                    for (int j = 0; j < d; ++j) dot += q[j] * k[j];
                    p[t] = dot * scale;
                    if (p[t] > m) m = p[t];
                }
                for (int t = 0; t < S; ++t) { p[t] = exp(p[t] - m); sum += p[t]; }
                for (int j = 0; j < d; ++j) {
                    double acc = 0.0;
                    for (int t = 0; t < S; ++t)
                        acc += (p[t] / sum) * qkv[((size_t)b * S + t) * 3 * Hd + 2 * Hd + h * d + j];
                    out[((size_t)b * S + s) * Hd + h * d + j] = acc;
                }
            }
        }
}

/* y[b,s,:] = tok[ids[b,s],:] + pos[s,:] + typ[0,:] */
void orc_embed(const int32_t *ids, int B, int S, int Hd, const float *tok, const float *pos, const float *typ, double *y)
{
#pragma omp parallel for
    for (int bs = 0; bs < B * S; ++bs) {
        const int s = bs % S;
        for (int j = 0; j < Hd; ++j)
            y[(size_t)bs * Hd + j] = (double)tok[(size_t)ids[bs] * Hd + j] + (double)pos[(size_t)s * Hd + j] + (double)typ[j];
    }
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
