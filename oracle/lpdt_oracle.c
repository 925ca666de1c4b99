/*
 * CPU oracle for the 8-bit decentralized-training hot path (arXiv 2111.09389).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, by-definition
 * statement of what the GPU library must compute.  It shares no code, header,
 * table or constant with the HIP path; only tests/, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  Never tuned for speed: loops are
 * written in the order the definitions are written; OpenMP is used only across
 * independent outputs.
 *
 * Floating point is fp64 except where a rounding decision produces an integer
 * (quantizer codes, top-k membership, arg-extrema): those decisions are taken
 * in fp32 with single IEEE operations, the precision the method's inputs have.
 *
 * Layouts: activations / gradients NHWC, filters KRSC, parameters [n][d].
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors of the SC'11
 * publication; quantizer grid invariants and a hand example; float64
 * library convolution + autograd; adjoint identities; Range-EvoNorm closed
 * forms, hand example, finite differences and float64 autograd; ring
 * eigen-modes and average preservation for the mix; brute-force sort for
 * top-k.  Whole-step accuracy against the paper's tables: parity unpinned
 * (needs the datasets).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EOVERFLOW -1
#define ORC_EINVAL -2

typedef struct {
    int N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w;
} orc_conv_desc;

static int out_dim(int in, int pad, int filt, int stride) { return (in + 2 * pad - filt) / stride + 1; }

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): 10 rounds; each round
 * multiplies counter words 0 and 2 by two fixed odd constants, and mixes the
 * high halves with the other counter words and the key; the key is advanced
 * by two Weyl constants between rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in [0,1) with 24-bit granularity for logical element i of a tensor:
 * key = seed, counter = (offset + i/4, 0, 0), word i%4, top 24 bits. */
static float sr_uniform(uint64_t seed, uint64_t offset, uint64_t i)
{
    uint64_t blk = offset + (i >> 2);
    uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    return (float)(w[i & 3] >> 8) * 0x1.0p-24f;
}

void orc_sr_uniform(uint64_t seed, uint64_t offset, uint64_t first, uint64_t count, float *u)
{
    for (uint64_t i = 0; i < count; ++i) u[i] = sr_uniform(seed, offset, first + i);
}

/* ------------------------------------------------------------------------- */
/* Symmetric per-tensor 8-bit quantizer (Section 3 "Low Precision Training";
 * grid fixed by the benchmark statement: scale = absmax/127, codes in
 * [-127,127], round-to-nearest-even or stochastic rounding).
 * rounding: 0 = nearest (ties to even), 1 = stochastic. */
int orc_quantize(const float *x, size_t len, int rounding, uint64_t seed, uint64_t offset,
                 int8_t *q, float *scale)
{
    float a = 0.0f;
    for (size_t i = 0; i < len; ++i) {
        float m = fabsf(x[i]);
        if (!(m <= 3.4028234663852886e38f)) return ORC_EINVAL; /* NaN / Inf: caller error */
        if (m > a) a = m;
    }
    volatile float inv = (a > 0.0f) ? 127.0f / a : 0.0f; /* one fp32 divide */
    /* An abs-max so small that 127/a is not a finite float (below about 3.7e-37) cannot carry a grid with
     * |x - q*scale| <= scale/2: such a tensor counts as zero, like a == 0 (codes 0, scale 0). */
    if (!(inv <= 3.4028234663852886e38f)) { inv = 0.0f; a = 0.0f; }
    *scale = a / 127.0f;
    for (size_t i = 0; i < len; ++i) {
        volatile float t = x[i] * inv; /* one fp32 multiply, never fused */
        float r;
        if (rounding == 0) {
            r = rintf(t); /* default rounding mode: ties to even */
        } else {
            float f = floorf(t);
            volatile float frac = t - f; /* exact */
            float u = sr_uniform(seed, offset, (uint64_t)i);
            r = f + ((u < frac) ? 1.0f : 0.0f);
        }
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        q[i] = (int8_t)(int)r;
    }
    return ORC_OK;
}

/* y = sA * sB * acc : the real value an int32 accumulator of two quantized
 * tensors stands for. */
void orc_dequantize(const int32_t *acc, size_t len, float sA, float sB, double *y)
{
    double s = (double)sA * (double)sB;
    for (size_t i = 0; i < len; ++i) y[i] = s * (double)acc[i];
}

/* ------------------------------------------------------------------------- */
/* The three convolution sums (Table "hardware_training", row Conv: forward,
 * gradient w.r.t. input, gradient w.r.t. filter), cross-correlation with
 * zero padding, exact integer arithmetic.  The result must fit int32. */
int orc_qconv_fwd(const orc_conv_desc *d, const int8_t *x, const int8_t *w, int32_t *acc)
{
    const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
    int bad = 0;
#pragma omp parallel for collapse(2) reduction(| : bad)
    for (int n = 0; n < d->N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < d->K; ++k) {
                    int64_t s = 0;
                    for (int r = 0; r < d->R; ++r)
                        for (int t = 0; t < d->S; ++t) {
                            int h = p * d->stride_h + r - d->pad_h, ww = q * d->stride_w + t - d->pad_w;
                            if (h < 0 || h >= d->H || ww < 0 || ww >= d->W) continue;
                            for (int c = 0; c < d->C; ++c)
                                s += (int64_t)x[(((size_t)n * d->H + h) * d->W + ww) * d->C + c] *
                                     (int64_t)w[(((size_t)k * d->R + r) * d->S + t) * d->C + c];
                        }
                    if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                    acc[(((size_t)n * P + p) * Q + q) * d->K + k] = (int32_t)s;
                }
    return bad ? ORC_EOVERFLOW : ORC_OK;
}

int orc_qconv_bwd_data(const orc_conv_desc *d, const int8_t *g, const int8_t *w, int32_t *dx)
{
    const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
    int bad = 0;
#pragma omp parallel for collapse(2) reduction(| : bad)
    for (int n = 0; n < d->N; ++n)
        for (int h = 0; h < d->H; ++h)
            for (int ww = 0; ww < d->W; ++ww)
                for (int c = 0; c < d->C; ++c) {
                    int64_t s = 0;
                    /* every (p,q,r,t) with p*stride + r - pad == h and q*stride + t - pad == ww */
                    for (int p = 0; p < P; ++p)
                        for (int q = 0; q < Q; ++q) {
                            int r = h - p * d->stride_h + d->pad_h, t = ww - q * d->stride_w + d->pad_w;
                            if (r < 0 || r >= d->R || t < 0 || t >= d->S) continue;
                            for (int k = 0; k < d->K; ++k)
                                s += (int64_t)g[(((size_t)n * P + p) * Q + q) * d->K + k] *
                                     (int64_t)w[(((size_t)k * d->R + r) * d->S + t) * d->C + c];
                        }
                    if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                    dx[(((size_t)n * d->H + h) * d->W + ww) * d->C + c] = (int32_t)s;
                }
    return bad ? ORC_EOVERFLOW : ORC_OK;
}

int orc_qconv_bwd_weight(const orc_conv_desc *d, const int8_t *g, const int8_t *x, int32_t *dw)
{
    const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
    int bad = 0;
#pragma omp parallel for collapse(2) reduction(| : bad)
    for (int k = 0; k < d->K; ++k)
        for (int r = 0; r < d->R; ++r)
            for (int t = 0; t < d->S; ++t)
                for (int c = 0; c < d->C; ++c) {
                    int64_t s = 0;
                    for (int n = 0; n < d->N; ++n)
                        for (int p = 0; p < P; ++p)
                            for (int q = 0; q < Q; ++q) {
                                int h = p * d->stride_h + r - d->pad_h, ww = q * d->stride_w + t - d->pad_w;
                                if (h < 0 || h >= d->H || ww < 0 || ww >= d->W) continue;
                                s += (int64_t)g[(((size_t)n * P + p) * Q + q) * d->K + k] *
                                     (int64_t)x[(((size_t)n * d->H + h) * d->W + ww) * d->C + c];
                            }
                    if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                    dw[(((size_t)k * d->R + r) * d->S + t) * d->C + c] = (int32_t)s;
                }
    return bad ? ORC_EOVERFLOW : ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* The weight-gradient product as the paper states it (Section 3, gradient bifurcation): the
 * layer gradient enters in 16-bit floating point rather than as 8-bit codes; the saved 8-bit
 * input codes are used as they are.  bfloat16 here: the upper 16 bits of the fp32 pattern
 * after round-to-nearest-even.
 *   dw[k,r,s,c] = sx * sum_{n,p,q} bf16(g)[n,p,q,k] * xq[n, p*st+r-pad, q*st+s-pad, c]
 * in double; dwabs gets the same sum over |g*x| (the size against which a lower-precision
 * accumulation is judged). */
uint16_t orc_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u); /* nearest, ties to even; inputs are finite */
    return (uint16_t)(u >> 16);
}

void orc_to_bf16(const float *x, size_t len, uint16_t *y)
{
    for (size_t i = 0; i < len; ++i) y[i] = orc_bf16_bits(x[i]);
}

static double bf16_value(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

int orc_qconv_bwd_weight_bf16(const orc_conv_desc *d, const uint16_t *g16, const int8_t *x, float sx, double *dw,
                              double *dwabs)
{
    const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
#pragma omp parallel for collapse(2)
    for (int k = 0; k < d->K; ++k)
        for (int r = 0; r < d->R; ++r)
            for (int t = 0; t < d->S; ++t)
                for (int c = 0; c < d->C; ++c) {
                    double s = 0.0, a = 0.0;
                    for (int n = 0; n < d->N; ++n)
                        for (int p = 0; p < P; ++p)
                            for (int q = 0; q < Q; ++q) {
                                int h = p * d->stride_h + r - d->pad_h, ww = q * d->stride_w + t - d->pad_w;
                                if (h < 0 || h >= d->H || ww < 0 || ww >= d->W) continue;
                                double term = bf16_value(g16[(((size_t)n * P + p) * Q + q) * d->K + k]) *
                                              (double)x[(((size_t)n * d->H + h) * d->W + ww) * d->C + c];
                                s += term;
                                a += fabs(term);
                            }
                    size_t o = (((size_t)k * d->R + r) * d->S + t) * d->C + c;
                    dw[o] = (double)sx * s;
                    dwabs[o] = (double)sx * a;
                }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Range-EvoNorm (Eq. "ren"): per sample and channel group, divide
 * x * hard_sigmoid(v x) by C(m) * (max - min) of the group's raw inputs,
 * m = channels per group, C(m) = 1/sqrt(2 ln m); then the affine gamma, beta.
 * eps is added to the denominator (the equation has none; eps = 0 reproduces
 * it literally).  Also returns, per (sample, group), the range and the first
 * position (lowest index in (h, w, channel-in-group) order) of max and min. */
static double hard_sigmoid(double z) { return fmax(0.0, fmin(1.0, (z + 3.0) / 6.0)); }

int orc_range_evonorm_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v,
                          const float *gamma, const float *beta, double eps, double *y,
                          double *range_out, int32_t *argmax_out, int32_t *argmin_out)
{
    if (groups <= 0 || C % groups != 0 || C / groups < 2) return ORC_EINVAL;
    const int m = C / groups;
    const double Cm = 1.0 / sqrt(2.0 * log((double)m));
#pragma omp parallel for collapse(2)
    for (int n = 0; n < N; ++n)
        for (int G = 0; G < groups; ++G) {
            float mx = 0, mn = 0;
            int32_t imx = -1, imn = -1;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        float e = x[(((size_t)n * H + h) * W + w) * C + G * m + cc];
                        int32_t idx = (h * W + w) * m + cc;
                        if (imx < 0 || e > mx) { mx = e; imx = idx; }
                        if (imn < 0 || e < mn) { mn = e; imn = idx; }
                    }
            double R = (double)mx - (double)mn;
            double D = Cm * R + eps;
            range_out[(size_t)n * groups + G] = R;
            argmax_out[(size_t)n * groups + G] = imx;
            argmin_out[(size_t)n * groups + G] = imn;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        int c = G * m + cc;
                        size_t at = (((size_t)n * H + h) * W + w) * C + c;
                        double xe = x[at];
                        double u = xe * hard_sigmoid((double)v[c] * xe);
                        y[at] = (double)gamma[c] * u / D + (double)beta[c];
                    }
        }
    return ORC_OK;
}

/* Chain rule of the forward above.  Hard-sigmoid slope is 1/6 strictly inside
 * (-3, 3) and 0 elsewhere; the whole gradient of the range goes to the saved
 * first arg-max (+) and first arg-min (-). */
int orc_range_evonorm_bwd(const double *dy, const float *x, int N, int H, int W, int C, int groups,
                          const float *v, const float *gamma, double eps, double *dx, double *dv,
                          double *dgamma, double *dbeta)
{
    if (groups <= 0 || C % groups != 0 || C / groups < 2) return ORC_EINVAL;
    const int m = C / groups;
    const double Cm = 1.0 / sqrt(2.0 * log((double)m));
    for (int c = 0; c < C; ++c) dv[c] = dgamma[c] = dbeta[c] = 0.0;
    for (int n = 0; n < N; ++n)
        for (int G = 0; G < groups; ++G) {
            float mx = 0, mn = 0;
            size_t amx = 0, amn = 0;
            int first = 1;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        size_t at = (((size_t)n * H + h) * W + w) * C + G * m + cc;
                        float e = x[at];
                        if (first || e > mx) { mx = e; amx = at; }
                        if (first || e < mn) { mn = e; amn = at; }
                        first = 0;
                    }
            double D = Cm * ((double)mx - (double)mn) + eps;
            double dD = 0.0;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        int c = G * m + cc;
                        size_t at = (((size_t)n * H + h) * W + w) * C + c;
                        double xe = x[at], z = (double)v[c] * xe;
                        double s = hard_sigmoid(z);
                        double sp = (z > -3.0 && z < 3.0) ? 1.0 / 6.0 : 0.0;
                        double u = xe * s;
                        double du = dy[at] * (double)gamma[c] / D;
                        dbeta[c] += dy[at];
                        dgamma[c] += dy[at] * u / D;
                        dv[c] += du * xe * xe * sp;
                        dx[at] = du * (s + xe * (double)v[c] * sp);
                        dD -= dy[at] * (double)gamma[c] * u / (D * D);
                    }
            double dR = Cm * dD;
            dx[amx] += dR;
            dx[amn] -= dR;
        }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* The two full-precision layers the paper compares Range-EvoNorm with.
 *
 * EvoNorm-S0 (Eq. "en"): per sample n and channel group G (m = C/groups channels),
 *   var = variance of x over the group's (h, w, channel) slab (population form, 1/count),
 *   y   = gamma_c * x * sigmoid(v_c x) / sqrt(var + eps) + beta_c.
 * The paper writes no eps and does not say which variance; eps is an argument (0 allowed)
 * and the population form is the reading taken. */
int orc_evonorm_s0_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v, const float *gamma,
                       const float *beta, double eps, double *y, double *mean_out, double *var_out)
{
    if (groups <= 0 || C % groups != 0) return ORC_EINVAL;
    const int m = C / groups;
    const double cnt = (double)H * W * m;
#pragma omp parallel for collapse(2)
    for (int n = 0; n < N; ++n)
        for (int G = 0; G < groups; ++G) {
            double sum = 0.0;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) sum += x[(((size_t)n * H + h) * W + w) * C + G * m + cc];
            const double mu = sum / cnt;
            double ss = 0.0;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        double e = x[(((size_t)n * H + h) * W + w) * C + G * m + cc] - mu;
                        ss += e * e;
                    }
            const double var = ss / cnt, D = sqrt(var + eps);
            mean_out[(size_t)n * groups + G] = mu;
            var_out[(size_t)n * groups + G] = var;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        int c = G * m + cc;
                        size_t at = (((size_t)n * H + h) * W + w) * C + c;
                        double xe = x[at];
                        double u = xe / (1.0 + exp(-(double)v[c] * xe));
                        y[at] = (double)gamma[c] * u / D + (double)beta[c];
                    }
        }
    return ORC_OK;
}

/* Chain rule of the forward above: u = x s, s = sigmoid(v x), s' = s (1 - s);
 * dD = -sum dy gamma u / D^2 over the slab, and D depends on every x_j of the slab through the variance:
 * dD/dx_j = (x_j - mean) / (count * D). */
int orc_evonorm_s0_bwd(const double *dy, const float *x, int N, int H, int W, int C, int groups, const float *v,
                       const float *gamma, double eps, double *dx, double *dv, double *dgamma, double *dbeta)
{
    if (groups <= 0 || C % groups != 0) return ORC_EINVAL;
    const int m = C / groups;
    const double cnt = (double)H * W * m;
    for (int c = 0; c < C; ++c) dv[c] = dgamma[c] = dbeta[c] = 0.0;
    for (int n = 0; n < N; ++n)
        for (int G = 0; G < groups; ++G) {
            double sum = 0.0, ss = 0.0;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) sum += x[(((size_t)n * H + h) * W + w) * C + G * m + cc];
            const double mu = sum / cnt;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        double e = x[(((size_t)n * H + h) * W + w) * C + G * m + cc] - mu;
                        ss += e * e;
                    }
            const double D = sqrt(ss / cnt + eps);
            double dD = 0.0;
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        int c = G * m + cc;
                        size_t at = (((size_t)n * H + h) * W + w) * C + c;
                        double xe = x[at], s = 1.0 / (1.0 + exp(-(double)v[c] * xe)), sp = s * (1.0 - s);
                        double u = xe * s, du = dy[at] * (double)gamma[c] / D;
                        dbeta[c] += dy[at];
                        dgamma[c] += dy[at] * u / D;
                        dv[c] += du * xe * xe * sp;
                        dx[at] = du * (s + xe * (double)v[c] * sp);
                        dD -= dy[at] * (double)gamma[c] * u / (D * D);
                    }
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int cc = 0; cc < m; ++cc) {
                        size_t at = (((size_t)n * H + h) * W + w) * C + G * m + cc;
                        dx[at] += dD * ((double)x[at] - mu) / (cnt * D);
                    }
        }
    return ORC_OK;
}

/* Range batch-norm (Eq. "rbn"): per channel c, over all samples and pixels,
 *   mu = mean of x,  R = max - min of (x - mu) = max - min of x,  D = C(b) * R + eps,  C(b) = 1/sqrt(2 ln b),
 *   y = gamma_c * (x - mu) / D + beta_c,   b = batch size (needs b >= 2).
 * argmax / argmin: first position (n, h, w order) of the extreme value, as flat index (n*H + h)*W + w. */
int orc_range_bn_fwd(const float *x, int N, int H, int W, int C, const float *gamma, const float *beta, double eps,
                     double *y, double *mean_out, double *range_out, int64_t *argmax_out, int64_t *argmin_out)
{
    if (N < 2) return ORC_EINVAL;
    const double Cb = 1.0 / sqrt(2.0 * log((double)N));
    const size_t pix = (size_t)N * H * W;
#pragma omp parallel for
    for (int c = 0; c < C; ++c) {
        double sum = 0.0;
        float mx = 0, mn = 0;
        int64_t imx = -1, imn = -1;
        for (size_t p = 0; p < pix; ++p) {
            float e = x[p * C + c];
            sum += e;
            if (imx < 0 || e > mx) { mx = e; imx = (int64_t)p; }
            if (imn < 0 || e < mn) { mn = e; imn = (int64_t)p; }
        }
        const double mu = sum / (double)pix, R = (double)mx - (double)mn, D = Cb * R + eps;
        mean_out[c] = mu; range_out[c] = R; argmax_out[c] = imx; argmin_out[c] = imn;
        for (size_t p = 0; p < pix; ++p) y[p * C + c] = (double)gamma[c] * ((double)x[p * C + c] - mu) / D + (double)beta[c];
    }
    return ORC_OK;
}

/* Chain rule: d(x_j - mu)/dx_i = [i == j] - 1/count, and the whole gradient of the range goes to the first arg-max (+)
 * and the first arg-min (-). */
int orc_range_bn_bwd(const double *dy, const float *x, int N, int H, int W, int C, const float *gamma, double eps,
                     double *dx, double *dgamma, double *dbeta)
{
    if (N < 2) return ORC_EINVAL;
    const double Cb = 1.0 / sqrt(2.0 * log((double)N));
    const size_t pix = (size_t)N * H * W;
#pragma omp parallel for
    for (int c = 0; c < C; ++c) {
        double sum = 0.0;
        float mx = 0, mn = 0;
        size_t imx = 0, imn = 0;
        int first = 1;
        for (size_t p = 0; p < pix; ++p) {
            float e = x[p * C + c];
            sum += e;
            if (first || e > mx) { mx = e; imx = p; }
            if (first || e < mn) { mn = e; imn = p; }
            first = 0;
        }
        const double mu = sum / (double)pix, D = Cb * ((double)mx - (double)mn) + eps;
        double sdy = 0.0, sdyx = 0.0;
        for (size_t p = 0; p < pix; ++p) {
            sdy += dy[p * C + c];
            sdyx += dy[p * C + c] * ((double)x[p * C + c] - mu);
        }
        dbeta[c] = sdy;
        dgamma[c] = sdyx / D;
        const double g = (double)gamma[c];
        for (size_t p = 0; p < pix; ++p) dx[p * C + c] = g / D * (dy[p * C + c] - sdy / (double)pix);
        const double dR = Cb * (-g * sdyx / (D * D));
        dx[imx * C + c] += dR;
        dx[imn * C + c] -= dR;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Gossip step (Algorithm 1 step 7; Algorithms 2 and 3 of the supplement).
 *   xhat == NULL : x_i+ = x_i + eta * (sum_j W_ij x_j - x_i)
 *   xhat != NULL : CHOCO.  v = x_i - xhat_i (fp32);  q = v on the top-k |v| of
 *                  each segment, k = max(1, ceil(keep_ratio*len)), ties to the
 *                  lower index;  xhat_i += q (fp32) for every agent first;
 *                  x_i+ = x_i + eta * sum_j W_ij (xhat_j - xhat_i).
 * W is row-major, W[i*n+j] = weight node i gives node j's model. */
typedef struct { uint32_t mag; uint32_t idx; } orc_key;
static int key_cmp(const void *a, const void *b)
{
    const orc_key *p = (const orc_key *)a, *q = (const orc_key *)b;
    if (p->mag != q->mag) return (p->mag > q->mag) ? -1 : 1; /* larger magnitude first */
    return (p->idx < q->idx) ? -1 : (p->idx > q->idx);        /* then lower index */
}

int orc_gossip_mix(const float *x, float *xhat, int n, size_t d, const float *Wm, float eta,
                   double keep_ratio, const int64_t *seg_offsets, int nseg, double *x_out)
{
    if (xhat) {
        for (int i = 0; i < n; ++i)
            for (int sgm = 0; sgm < nseg; ++sgm) {
                size_t lo = (size_t)seg_offsets[sgm], hi = (size_t)seg_offsets[sgm + 1], len = hi - lo;
                if (len == 0) continue;
                int64_t k = (int64_t)ceil(keep_ratio * (double)len);
                if (k < 1) k = 1;
                if ((size_t)k > len) k = (int64_t)len;
                orc_key *keys = (orc_key *)malloc(len * sizeof(orc_key));
                float *vv = (float *)malloc(len * sizeof(float));
                if (!keys || !vv) { free(keys); free(vv); return ORC_EINVAL; }
                for (size_t e = 0; e < len; ++e) {
                    volatile float dv = x[(size_t)i * d + lo + e] - xhat[(size_t)i * d + lo + e];
                    vv[e] = dv;
                    float ab = fabsf(dv);
                    uint32_t bits;
                    memcpy(&bits, &ab, 4);
                    keys[e].mag = bits;
                    keys[e].idx = (uint32_t)e;
                }
                qsort(keys, len, sizeof(orc_key), key_cmp);
                for (int64_t t = 0; t < k; ++t) {
                    size_t e = keys[t].idx;
                    volatile float s = xhat[(size_t)i * d + lo + e] + vv[e];
                    xhat[(size_t)i * d + lo + e] = s;
                }
                free(keys);
                free(vv);
            }
    }
#pragma omp parallel for
    for (int i = 0; i < n; ++i)
        for (size_t e = 0; e < d; ++e) {
            double s = 0.0;
            if (xhat) {
                for (int j = 0; j < n; ++j)
                    s += (double)Wm[(size_t)i * n + j] * ((double)xhat[(size_t)j * d + e] - (double)xhat[(size_t)i * d + e]);
            } else {
                for (int j = 0; j < n; ++j) s += (double)Wm[(size_t)i * n + j] * (double)x[(size_t)j * d + e];
                s -= (double)x[(size_t)i * d + e];
            }
            x_out[(size_t)i * d + e] = (double)x[(size_t)i * d + e] + (double)eta * s;
        }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* The other gossip variants of the supplement (Algorithms "Deep-Squeeze", "Sparse-Push",
 * "Quant-SGP"), one step each, after the local update.
 *   mode 0: no compression    x_i+ = x_i + eta * sum_j (W_ij - I_ij) x_j
 *   mode 1: CHOCO             state = xhat:  q = TopK(x_i - xhat_i); xhat_i += q;
 *                             x_i+ = x_i + eta * sum_j (W_ij - I_ij)(xhat_j - xhat_i)
 *   mode 2: Deep-Squeeze      state = delta (error memory):  v = x_i + delta_i (fp32);
 *                             C[v] = v on the top-k |v| of each segment, 0 elsewhere;
 *                             delta_i = v - C[v];  x_i+ = x_i + eta * sum_j (W_ij - I_ij) C[v_j]
 *   u != NULL (push-sum, Algorithms "Sparse-Push" = mode 2 + u, "Quant-SGP" = mode 1 + u):
 *                             u_i+ = u_i + eta * sum_j (W_ij - I_ij) u_j;   z_i = x_i+ / u_i+
 *                             With u, mode 1 mixes xhat by the same operator as u and as modes 0 and 2,
 *                             x_i+ = x_i + eta * sum_j (W_ij - I_ij) xhat_j.  For a W whose rows sum to 1 this is
 *                             the printed (xhat_j - xhat_i) form; for a merely column-stochastic W the printed form
 *                             would not conserve sum_i x_i, which the de-biasing by u relies on.
 * Top-k as in orc_gossip_mix: k = max(1, ceil(keep_ratio*len)), larger |v| first (fp32 bit
 * pattern), lower index on ties.  W only has to be column stochastic when u is given. */
int orc_gossip_mix_ex(const float *x, float *state, int n, size_t d, const float *Wm, float eta, double keep_ratio,
                      const int64_t *seg_offsets, int nseg, int mode, const float *u, double *x_out, double *u_out,
                      double *z_out)
{
    if (mode < 0 || mode > 2 || (mode != 0 && !state)) return ORC_EINVAL;
    float *cv = NULL; /* mode 2: the compressed vectors C[v_i] */
    if (mode == 2) {
        cv = (float *)calloc((size_t)n * d, sizeof(float));
        if (!cv) return ORC_EINVAL;
    }
    if (mode != 0)
        for (int i = 0; i < n; ++i)
            for (int sgm = 0; sgm < nseg; ++sgm) {
                size_t lo = (size_t)seg_offsets[sgm], hi = (size_t)seg_offsets[sgm + 1], len = hi - lo;
                if (len == 0) continue;
                int64_t k = (int64_t)ceil(keep_ratio * (double)len);
                if (k < 1) k = 1;
                if ((size_t)k > len) k = (int64_t)len;
                orc_key *keys = (orc_key *)malloc(len * sizeof(orc_key));
                float *vv = (float *)malloc(len * sizeof(float));
                if (!keys || !vv) { free(keys); free(vv); free(cv); return ORC_EINVAL; }
                for (size_t e = 0; e < len; ++e) {
                    size_t at = (size_t)i * d + lo + e;
                    volatile float v = (mode == 1) ? x[at] - state[at] : x[at] + state[at];
                    vv[e] = v;
                    float ab = fabsf(v);
                    uint32_t bits;
                    memcpy(&bits, &ab, 4);
                    keys[e].mag = bits;
                    keys[e].idx = (uint32_t)e;
                }
                qsort(keys, len, sizeof(orc_key), key_cmp);
                if (mode == 1) {
                    for (int64_t t = 0; t < k; ++t) {
                        size_t at = (size_t)i * d + lo + keys[t].idx;
                        volatile float s2 = state[at] + vv[keys[t].idx];
                        state[at] = s2;
                    }
                } else {
                    for (size_t e = 0; e < len; ++e) state[(size_t)i * d + lo + e] = vv[e]; /* delta = v ... */
                    for (int64_t t = 0; t < k; ++t) {
                        size_t at = (size_t)i * d + lo + keys[t].idx;
                        cv[at] = vv[keys[t].idx];
                        volatile float r = vv[keys[t].idx] - cv[at];                            /* ... minus C[v] */
                        state[at] = r;
                    }
                }
                free(keys);
                free(vv);
            }
    const float *m = (mode == 0) ? x : (mode == 1) ? state : cv; /* what the neighbours exchange */
    for (int i = 0; i < n; ++i)
        for (size_t e = 0; e < d; ++e) {
            double s = 0.0;
            for (int j = 0; j < n; ++j) {
                double wij = (double)Wm[(size_t)i * n + j] - (i == j ? 1.0 : 0.0);
                double term = (double)m[(size_t)j * d + e];
                if (mode == 1 && !u) term -= (double)m[(size_t)i * d + e];
                s += wij * term;
            }
            x_out[(size_t)i * d + e] = (double)x[(size_t)i * d + e] + (double)eta * s;
        }
    if (u) {
        for (int i = 0; i < n; ++i) {
            double s = 0.0;
            for (int j = 0; j < n; ++j) s += ((double)Wm[(size_t)i * n + j] - (i == j ? 1.0 : 0.0)) * (double)u[j];
            u_out[i] = (double)u[i] + (double)eta * s;
        }
        for (int i = 0; i < n; ++i)
            for (size_t e = 0; e < d; ++e) z_out[(size_t)i * d + e] = x_out[(size_t)i * d + e] / u_out[i];
    }
    free(cv);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Glue layers of the benchmark networks (Table "hardware_training": skip
 * connections, average pool; plus max-pool and the softmax cross-entropy
 * loss, standard definitions), all NHWC, fp64. */
void orc_add(const double *a, const double *b, size_t len, double *y)
{
    for (size_t i = 0; i < len; ++i) y[i] = a[i] + b[i];
}

/* window kxk, stride st, pad pd (padding never wins); idx = winning flat
 * (h*W+w) position, first in window scan order on ties. */
void orc_maxpool_fwd(const float *x, int N, int H, int W, int C, int k, int st, int pd, float *y, int32_t *idx)
{
    int P = out_dim(H, pd, k, st), Q = out_dim(W, pd, k, st);
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int c = 0; c < C; ++c) {
                    float best = 0;
                    int32_t bi = -1;
                    for (int r = 0; r < k; ++r)
                        for (int t = 0; t < k; ++t) {
                            int h = p * st + r - pd, w = q * st + t - pd;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            float e = x[(((size_t)n * H + h) * W + w) * C + c];
                            if (bi < 0 || e > best) { best = e; bi = h * W + w; }
                        }
                    size_t o = (((size_t)n * P + p) * Q + q) * C + c;
                    y[o] = best;
                    idx[o] = bi;
                }
}

void orc_maxpool_bwd(const double *dy, const int32_t *idx, int N, int H, int W, int C, int P, int Q, double *dx)
{
    memset(dx, 0, sizeof(double) * (size_t)N * H * W * C);
    for (int n = 0; n < N; ++n)
        for (int pq = 0; pq < P * Q; ++pq)
            for (int c = 0; c < C; ++c) {
                size_t o = ((size_t)n * P * Q + pq) * C + c;
                dx[((size_t)n * H * W + idx[o]) * C + c] += dy[o];
            }
}

void orc_avgpool_fwd(const float *x, int N, int HW, int C, double *y)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double s = 0;
            for (int i = 0; i < HW; ++i) s += x[((size_t)n * HW + i) * C + c];
            y[(size_t)n * C + c] = s / HW;
        }
}

void orc_avgpool_bwd(const double *dy, int N, int HW, int C, double *dx)
{
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i)
            for (int c = 0; c < C; ++c) dx[((size_t)n * HW + i) * C + c] = dy[(size_t)n * C + c] / HW;
}

/* mean over the batch of -log softmax(logits)[label]; dlogits = (softmax - onehot)/N */
double orc_softmax_xent(const float *logits, const int32_t *labels, int N, int classes, double *dlogits)
{
    double loss = 0;
    for (int n = 0; n < N; ++n) {
        double mx = logits[(size_t)n * classes];
        for (int j = 1; j < classes; ++j) mx = fmax(mx, (double)logits[(size_t)n * classes + j]);
        double z = 0;
        for (int j = 0; j < classes; ++j) z += exp((double)logits[(size_t)n * classes + j] - mx);
        loss += log(z) + mx - (double)logits[(size_t)n * classes + labels[n]];
        for (int j = 0; j < classes; ++j)
            dlogits[(size_t)n * classes + j] =
                (exp((double)logits[(size_t)n * classes + j] - mx) / z - (j == labels[n] ? 1.0 : 0.0)) / N;
    }
    return loss / N;
}

/* local SGD step of Algorithm 1 step 3: x~ = x - lr * g */
void orc_sgd(const float *x, const float *g, size_t len, float lr, double *y)
{
    for (size_t i = 0; i < len; ++i) y[i] = (double)x[i] - (double)lr * (double)g[i];
}
