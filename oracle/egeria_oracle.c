/*
 * CPU oracle for the plasticity-evaluation path of Egeria (arXiv 2201.06227).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the path computes, written from the paper and from the readings listed in
 * the design notes.  It shares no code with the GPU library and must never be
 * called from a product path.  Only tests, the smoke check and the benchmark's
 * CPU-baseline leg use it.
 *
 * Conventions
 *   - integer work (quantised codes, int32 accumulators) is exact;
 *   - fp32 steps that decide an integer downstream (the scale, the rounding of
 *     x*inv, the dequantising epilogue) are done in fp32 in one fixed operation
 *     order, so that a second implementation can match them bit for bit;
 *   - everything else that is floating point (layer norm, softmax attention,
 *     GELU, the plasticity score) is evaluated in fp64 and rounded to fp32
 *     only where a tensor is stored as fp32.
 *   - `#pragma omp parallel for` appears on outermost loops only; there is no
 *     blocking, fusion or reordering.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -ffp-contract=off -fPIC -shared -o libegeria_oracle.so egeria_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <float.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- Section 4.1 (reference model = int8 post-training quantisation) -----
 * The paper delegates the arithmetic to its framework; the reading used here:
 * symmetric, per tensor, zero point 0, codes in [-127, 127], round half to even.
 */

/* max_i |x_i|.  Returns NaN/Inf if any element is not finite. */
float orc_absmax_f32(const float *x, int64_t n)
{
    float m = 0.0f;
    int bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (!(a <= FLT_MAX)) bad = 1;
        if (a > m) m = a;
    }
    return bad ? INFINITY : m;
}

/* scale and its reciprocal from the absolute maximum (dynamic) or from a
 * caller-provided scale (static).  A tensor whose absmax is zero, or so small
 * that the reciprocal overflows fp32, is quantised as the all-zero tensor with
 * scale 1. */
static void orc_scales(float absmax, const float *fixed_scale, float *scale, float *inv)
{
    if (fixed_scale) {
        *scale = *fixed_scale;
        *inv = (float)(1.0 / (double)*fixed_scale);
    } else {
        *scale = (float)((double)absmax / 127.0);
        *inv = (float)(127.0 / (double)absmax);
    }
    if (!(*inv <= FLT_MAX) || !(*scale > 0.0f)) { *scale = 1.0f; *inv = 0.0f; }
}

/* q_i = clamp(rint(x_i * inv), -127, 127).  Returns 0, or 1 when the input
 * holds a NaN or an infinity (outputs then unspecified). */
int orc_quantize_f32(const float *x, int64_t n, const float *fixed_scale, int8_t *q, float *scale_out)
{
    float absmax = orc_absmax_f32(x, n);
    if (!(absmax <= FLT_MAX)) return 1;
    float scale, inv;
    orc_scales(absmax, fixed_scale, &scale, &inv);
    *scale_out = scale;
    for (int64_t i = 0; i < n; ++i) {
        float r = rintf(x[i] * inv);          /* one fp32 multiply, round half to even */
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        q[i] = (int8_t)r;
    }
    return 0;
}

void orc_dequantize(const int8_t *q, float scale, int64_t n, float *x)
{
    for (int64_t i = 0; i < n; ++i) x[i] = (float)q[i] * scale;
}

/* ---- the reference forward's integer contractions ------------------------ */

/* acc[m,n] = sum_k x[m,k] * w[n,k]; weights in [out, in] order. */
void orc_gemm_i8(const int8_t *x, const int8_t *w, int64_t M, int64_t N, int64_t K, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int32_t)x[m * K + k] * (int32_t)w[n * K + k];
            acc[m * N + n] = s;
        }
}

/* Stride-1 2-D cross-correlation with zero padding `pad` on every side.
 * x [B,C,H,W], w [OC,C,KH,KW], acc [B,OC,H,W] (same spatial size, which holds
 * for KH = KW = 2*pad+1).  The pad value is the integer 0, which is exact
 * because the zero point is 0. */
void orc_conv2d_i8(const int8_t *x, const int8_t *w, int64_t B, int64_t C, int64_t H, int64_t W,
                   int64_t OC, int64_t KH, int64_t KW, int64_t pad, int32_t *acc)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oc = 0; oc < OC; ++oc)
            for (int64_t oh = 0; oh < H; ++oh)
                for (int64_t ow = 0; ow < W; ++ow) {
                    int32_t s = 0;
                    for (int64_t c = 0; c < C; ++c)
                        for (int64_t kh = 0; kh < KH; ++kh) {
                            int64_t ih = oh + kh - pad;
                            if (ih < 0 || ih >= H) continue;
                            for (int64_t kw = 0; kw < KW; ++kw) {
                                int64_t iw = ow + kw - pad;
                                if (iw < 0 || iw >= W) continue;
                                s += (int32_t)x[((b * C + c) * H + ih) * W + iw] *
                                     (int32_t)w[((oc * C + c) * KH + kh) * KW + kw];
                            }
                        }
                    acc[((b * OC + oc) * H + oh) * W + ow] = s;
                }
}

/* Dequantising epilogue in fp32, fixed operation order:
 *   s = sx * sw;  y = fma((float)acc, s, bias[c]);
 *   act 1: y = max(y, 0)                       (ReLU)
 *   act 2: y = 0.5*y*(1 + erf(y/sqrt 2))       (GELU, erf form, evaluated in fp64)
 *   residual != NULL: y = y + residual, applied before a ReLU and only then.
 * Elements are indexed [outer][channels][inner]; bias is per channel (may be
 * NULL).  A linear layer has inner = 1, an NCHW convolution inner = H*W. */
void orc_dequant_bias_act(const int32_t *acc, int64_t outer, int64_t channels, int64_t inner,
                          float sx, float sw, const float *bias, int act, const float *residual,
                          float *y)
{
    const float s = sx * sw;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t c = 0; c < channels; ++c) {
            const float bc = bias ? bias[c] : 0.0f;
            for (int64_t i = 0; i < inner; ++i) {
                int64_t idx = (o * channels + c) * inner + i;
                float v = fmaf((float)acc[idx], s, bc);
                if (residual) v = v + residual[idx];
                if (act == 1) v = v > 0.0f ? v : 0.0f;
                else if (act == 2) {
                    double d = (double)v;
                    v = (float)(0.5 * d * (1.0 + erf(d * 0.70710678118654752440)));
                }
                y[idx] = v;
            }
        }
}

/* The same epilogue for weights quantised per output channel (one scale per
 * row of the weight matrix / per output channel of the kernel): the scale of
 * channel c is s_c = sx * sw[c], again one fp32 multiply. */
void orc_dequant_bias_act_pc(const int32_t *acc, int64_t outer, int64_t channels, int64_t inner,
                             float sx, const float *sw, const float *bias, int act,
                             const float *residual, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t c = 0; c < channels; ++c) {
            const float s = sx * sw[c];
            const float bc = bias ? bias[c] : 0.0f;
            for (int64_t i = 0; i < inner; ++i) {
                int64_t idx = (o * channels + c) * inner + i;
                float v = fmaf((float)acc[idx], s, bc);
                if (residual) v = v + residual[idx];
                if (act == 1) v = v > 0.0f ? v : 0.0f;
                else if (act == 2) {
                    double d = (double)v;
                    v = (float)(0.5 * d * (1.0 + erf(d * 0.70710678118654752440)));
                }
                y[idx] = v;
            }
        }
}

/* ---- fp32 glue of a Transformer encoder layer (not quantised under dynamic
 * quantisation, Section 5) ------------------------------------------------- */

/* y[m,:] = gamma * (v - mean(v)) / sqrt(var(v) + eps) + beta with
 * v = x[m,:] + res[m,:] (res may be NULL); biased variance; fp64 inside. */
void orc_layernorm(const float *x, const float *res, int64_t M, int64_t H, const float *gamma,
                   const float *beta, double eps, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double mean = 0.0, var = 0.0;
        for (int64_t h = 0; h < H; ++h)
            mean += (double)x[m * H + h] + (res ? (double)res[m * H + h] : 0.0);
        mean /= (double)H;
        for (int64_t h = 0; h < H; ++h) {
            double v = (double)x[m * H + h] + (res ? (double)res[m * H + h] : 0.0) - mean;
            var += v * v;
        }
        var /= (double)H;
        double rstd = 1.0 / sqrt(var + eps);
        for (int64_t h = 0; h < H; ++h) {
            double v = (double)x[m * H + h] + (res ? (double)res[m * H + h] : 0.0);
            double g = gamma ? (double)gamma[h] : 1.0, bt = beta ? (double)beta[h] : 0.0;
            y[m * H + h] = (float)((v - mean) * rstd * g + bt);
        }
    }
}

/* Multi-head scaled dot-product self-attention, no mask, no dropout.
 * qkv [B,S,3*Hd]: per token the concatenation (q | k | v), head h owning
 * columns [h*dh, (h+1)*dh) of each third.  ctx [B,S,Hd].  fp64 inside. */
void orc_attention(const float *qkv, int64_t B, int64_t S, int64_t Hd, int64_t heads, float *ctx)
{
    const int64_t dh = Hd / heads;
    const double inv_sqrt = 1.0 / sqrt((double)dh);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < heads; ++h) {
            double *p = (double *)malloc(sizeof(double) * (size_t)S);
            for (int64_t i = 0; i < S; ++i) {
                const float *qi = qkv + (b * S + i) * 3 * Hd + h * dh;
                double mx = -INFINITY;
                for (int64_t j = 0; j < S; ++j) {
                    const float *kj = qkv + (b * S + j) * 3 * Hd + Hd + h * dh;
                    double s = 0.0;
                    for (int64_t d = 0; d < dh; ++d) s += (double)qi[d] * (double)kj[d];
                    p[j] = s * inv_sqrt;
                    if (p[j] > mx) mx = p[j];
                }
                double den = 0.0;
                for (int64_t j = 0; j < S; ++j) { p[j] = exp(p[j] - mx); den += p[j]; }
                for (int64_t d = 0; d < dh; ++d) {
                    double o = 0.0;
                    for (int64_t j = 0; j < S; ++j)
                        o += p[j] * (double)qkv[(b * S + j) * 3 * Hd + 2 * Hd + h * dh + d];
                    ctx[(b * S + i) * Hd + h * dh + d] = (float)(o / den);
                }
            }
            free(p);
        }
}

/* ---- Section 4.2, Eq. 1: training plasticity = SP loss ---------------------
 * The paper names the similarity-preserving loss and describes it (activations
 * reshaped to [b, D], b x b pair-wise similarity matrices, compared) without
 * printing the formula; this is the cited loss's definition:
 *   Gt = Q Q^T;  G[i,:] = Gt[i,:] / max(||Gt[i,:]||_2, 1e-12);
 *   P = (1/b^2) * sum_ij (G_T[i,j] - G_R[i,j])^2.
 * gram_t / gram_r (b*b doubles each, may be NULL) receive the un-normalised
 * Gram matrices. */
double orc_sp_loss_f32(const float *a_t, const float *a_r, int64_t b, int64_t D,
                       double *gram_t, double *gram_r)
{
    double *gt = (double *)malloc(sizeof(double) * (size_t)(b * b));
    double *gr = (double *)malloc(sizeof(double) * (size_t)(b * b));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < b; ++i)
        for (int64_t j = 0; j < b; ++j) {
            double st = 0.0, sr = 0.0;
            for (int64_t d = 0; d < D; ++d) {
                st += (double)a_t[i * D + d] * (double)a_t[j * D + d];
                sr += (double)a_r[i * D + d] * (double)a_r[j * D + d];
            }
            gt[i * b + j] = st;
            gr[i * b + j] = sr;
        }
    if (gram_t) for (int64_t i = 0; i < b * b; ++i) gram_t[i] = gt[i];
    if (gram_r) for (int64_t i = 0; i < b * b; ++i) gram_r[i] = gr[i];
    double p = 0.0;
    for (int64_t i = 0; i < b; ++i) {
        double nt = 0.0, nr = 0.0;
        for (int64_t j = 0; j < b; ++j) {
            nt += gt[i * b + j] * gt[i * b + j];
            nr += gr[i * b + j] * gr[i * b + j];
        }
        nt = sqrt(nt); nr = sqrt(nr);
        if (nt < 1e-12) nt = 1e-12;
        if (nr < 1e-12) nr = 1e-12;
        for (int64_t j = 0; j < b; ++j) {
            double d = gt[i * b + j] / nt - gr[i * b + j] / nr;
            p += d * d;
        }
    }
    free(gt); free(gr);
    return p / ((double)b * (double)b);
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
