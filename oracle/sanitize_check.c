/* Runs the oracle's functions on small ragged inputs as one plain executable, meant to be built together with
 * lpdt_oracle.c under -fsanitize=address,undefined (tests/test_oracle_sanitizers.py does that): any out-of-bounds
 * access, signed overflow or misaligned access in the checker itself ends the run with a report.  Test infrastructure,
 * like the rest of this folder; exits 0 when every call returned.  Values are not checked here (the pins do that). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w; } orc_conv_desc;
int orc_quantize(const float *, size_t, int, uint64_t, uint64_t, int8_t *, float *);
void orc_dequantize(const int32_t *, size_t, float, float, double *);
int orc_qconv_fwd(const orc_conv_desc *, const int8_t *, const int8_t *, int32_t *);
int orc_qconv_bwd_data(const orc_conv_desc *, const int8_t *, const int8_t *, int32_t *);
int orc_qconv_bwd_weight(const orc_conv_desc *, const int8_t *, const int8_t *, int32_t *);
void orc_to_bf16(const float *, size_t, uint16_t *);
int orc_range_evonorm_fwd(const float *, int, int, int, int, int, const float *, const float *, const float *, double, double *,
                          double *, int32_t *, int32_t *);
int orc_range_evonorm_bwd(const double *, const float *, int, int, int, int, int, const float *, const float *, double, double *,
                          double *, double *, double *);
int orc_gossip_mix(const float *, float *, int, size_t, const float *, float, double, const int64_t *, int, double *);
int orc_gossip_mix_ex(const float *, float *, int, size_t, const float *, float, double, const int64_t *, int, int, const float *,
                      double *, double *, double *);

static uint32_t state = 12345u;
static uint32_t rnd(void) { state = state * 1664525u + 1013904223u; return state >> 8; }
static float frnd(void) { return (float)(rnd() % 20001) / 10000.0f - 1.0f; }

static int conv_case(int N, int C, int H, int W, int K, int R, int S, int st, int pd)
{
    orc_conv_desc d = {N, C, H, W, K, R, S, st, st, pd, pd};
    const int P = (H + 2 * pd - R) / st + 1, Q = (W + 2 * pd - S) / st + 1;
    const size_t nx = (size_t)N * H * W * C, nw = (size_t)K * R * S * C, ny = (size_t)N * P * Q * K;
    int8_t *x = malloc(nx), *w = malloc(nw), *g = malloc(ny);
    int32_t *y = malloc(ny * 4), *dx = malloc(nx * 4), *dw = malloc(nw * 4);
    for (size_t i = 0; i < nx; ++i) x[i] = (int8_t)(rnd() % 255 - 127);
    for (size_t i = 0; i < nw; ++i) w[i] = (int8_t)(rnd() % 255 - 127);
    for (size_t i = 0; i < ny; ++i) g[i] = (int8_t)(rnd() % 255 - 127);
    int rc = orc_qconv_fwd(&d, x, w, y) | orc_qconv_bwd_data(&d, g, w, dx) | orc_qconv_bwd_weight(&d, g, x, dw);
    free(x); free(w); free(g); free(y); free(dx); free(dw);
    return rc;
}

int main(void)
{
    int rc = 0;
    /* quantizer: ragged lengths, both roundings, a zero tensor, an abs-max too small for a grid */
    for (size_t len = 1; len <= 4099; len = len * 3 + 1) {
        float *x = malloc(len * 4), s;
        int8_t *q = malloc(len);
        for (size_t i = 0; i < len; ++i) x[i] = frnd();
        rc |= orc_quantize(x, len, 0, 7, 0, q, &s) | orc_quantize(x, len, 1, 7, ((uint64_t)1 << 32) - 3, q, &s);
        memset(x, 0, len * 4);
        rc |= orc_quantize(x, len, 1, 7, 0, q, &s);
        x[0] = 1e-44f;
        rc |= orc_quantize(x, len, 0, 7, 0, q, &s);
        uint16_t *h = malloc(len * 2);
        orc_to_bf16(x, len, h);
        free(h); free(x); free(q);
    }
    int32_t acc[5] = {0, 1, -1, 2147483647, -2147483647 - 1};
    double yd[5];
    orc_dequantize(acc, 5, 0.5f, 0.25f, yd);
    /* convolutions: odd sizes, strides, paddings, 1x1, 7x7 */
    rc |= conv_case(2, 3, 9, 11, 5, 3, 3, 1, 1) | conv_case(1, 4, 7, 7, 6, 3, 3, 2, 1) | conv_case(3, 8, 5, 5, 2, 1, 1, 2, 0) |
          conv_case(1, 3, 13, 13, 4, 7, 7, 2, 3) | conv_case(5, 16, 1, 1, 10, 1, 1, 1, 0) | conv_case(1, 2, 4, 6, 3, 3, 3, 1, 0);
    /* Range-EvoNorm forward and backward */
    {
        const int N = 2, H = 5, W = 3, C = 8, groups = 2;
        const size_t n = (size_t)N * H * W * C;
        float *x = malloc(n * 4), v[8], gm[8], bt[8];
        double *y = malloc(n * 8), *dy = malloc(n * 8), *dx = malloc(n * 8), range[4], dv[8], dg[8], db[8];
        int32_t amax[4], amin[4];
        for (size_t i = 0; i < n; ++i) { x[i] = frnd() * 3.0f; dy[i] = frnd(); }
        for (int c = 0; c < C; ++c) { v[c] = 1.0f + 0.1f * frnd(); gm[c] = 1.0f; bt[c] = 0.1f * frnd(); }
        rc |= orc_range_evonorm_fwd(x, N, H, W, C, groups, v, gm, bt, 1e-5, y, range, amax, amin);
        rc |= orc_range_evonorm_bwd(dy, x, N, H, W, C, groups, v, gm, 1e-5, dx, dv, dg, db);
        free(x); free(y); free(dy); free(dx);
    }
    /* gossip: plain, CHOCO with layer-wise top-k and ties, Deep-Squeeze */
    {
        const int n = 4;
        const size_t d = 301;
        float *x = malloc(n * d * 4), *h = malloc(n * d * 4), Wm[16] = {0};
        double *out = malloc(n * d * 8);
        const int64_t seg[4] = {0, 7, 150, 301};
        for (int i = 0; i < n; ++i) { Wm[i * n + i] = Wm[i * n + (i + 1) % n] = Wm[i * n + (i + n - 1) % n] = 1.0f / 3.0f; }
        for (size_t i = 0; i < n * d; ++i) { x[i] = frnd(); h[i] = (i % 3) ? frnd() : x[i]; }
        rc |= orc_gossip_mix(x, NULL, n, d, Wm, 1.0f, 1.0, NULL, 0, out);
        rc |= orc_gossip_mix(x, h, n, d, Wm, 0.3f, 0.05, seg, 3, out);
        rc |= orc_gossip_mix_ex(x, h, n, d, Wm, 0.3f, 0.05, seg, 3, 2, NULL, out, NULL, NULL);
        free(x); free(h); free(out);
    }
    if (rc) { printf("an oracle call returned %d\n", rc); return 1; }
    printf("sanitize_check: every oracle call returned\n");
    return 0;
}
