// The two full-precision layers the paper compares Range-EvoNorm with, as fp32 reference layers (NHWC):
//   EvoNorm-S0 (Eq. "en"):        y = gamma_c * x * sigmoid(v_c x) / sqrt(var_{n,G} + eps) + beta_c
//   range batch-norm (Eq. "rbn"): y = gamma_c * (x - mean_c) / (C(b) * range_c + eps) + beta_c
// All passes are HBM-bound streams over the tensor with the block / thread layout of the Range-EvoNorm kernels
// (a block owns consecutive pixels of one sample, a thread one quad of channels).  Statistics leave a block as
// per-block partials and are folded in a fixed order (double precision where sums of many terms meet), so results
// are identical from run to run.  Unlike the range, a variance or a mean depends on every element, so both backward
// directions need their reductions finished before the first dx can be written: reduce pass, small fold, apply pass.
#include "common.h"
#include "norm_geom.h"
#include <cmath>

namespace lpdt {

constexpr int kRefElems = 16384;   // elements per block of the streaming passes (as for Range-EvoNorm's apply pass)

__device__ __forceinline__ float sigmoid_f(float z) { return __fdiv_rn(1.0f, 1.0f + expf(-z)); }

__device__ __forceinline__ float4 load_or_zero(const float4 *p, bool ok) { return ok ? *p : make_float4(0.f, 0.f, 0.f, 0.f); }

// Sums, per channel and in a fixed order, the values the block's threads hold for it: sred[q][thread * 4 + e] is thread
// (pixel lane k, quad qd)'s value of quantity q for channel 4 * qd + e.  Returns the sum for (q, c) to thread i = q * C + c.
__device__ __forceinline__ float column_sum(const float *sred, int T4, int q, int c, const RenGeom &g) {
    float s = 0.0f;
    for (int k = 0; k < g.ppi; ++k) s += sred[q * T4 + (k * g.cq) * 4 + c];
    return s;
}

// ---------------------------------------------------------------- EvoNorm-S0
// parts[((n * chunks + chunk) * groups + G) * 2 + {0, 1}] = the block's sum / sum of squares over group G
__global__ __launch_bounds__(kRThreads) void evo_stats_kernel(const float *__restrict__ x, RenGeom g, float *__restrict__ parts) {
    extern __shared__ float sred[];  // [2][threads * 4], then [2][C] column sums
    const int n = blockIdx.y;
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    const bool active = (int)threadIdx.x < g.threads;
    float s1[4] = {0, 0, 0, 0}, s2[4] = {0, 0, 0, 0};
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * g.HW * g.C);
    for (int pb = p0 + pl; pb < p1 && active; pb += kRU * g.ppi) {
        float4 a[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) a[k] = load_or_zero(xv + (size_t)(pb + k * g.ppi) * g.cq + qd, pb + k * g.ppi < p1);
#pragma unroll
        for (int k = 0; k < kRU; ++k) {  // pixels past the end contribute zeros
            const float e[4] = {a[k].x, a[k].y, a[k].z, a[k].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) { s1[j] += e[j]; s2[j] += e[j] * e[j]; }
        }
    }
    const int T4 = g.threads * 4;
    if (active) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { sred[threadIdx.x * 4 + j] = s1[j]; sred[T4 + threadIdx.x * 4 + j] = s2[j]; }
    }
    __syncthreads();
    float *col = sred + 2 * T4;
    for (int i = threadIdx.x; i < 2 * g.C; i += blockDim.x) col[i] = column_sum(sred, T4, i / g.C, i % g.C, g);
    __syncthreads();
    float *dst = parts + ((size_t)n * g.chunks + blockIdx.x) * g.groups * 2;
    for (int i = threadIdx.x; i < 2 * g.groups; i += blockDim.x) {
        const int G = i / 2, q = i % 2;
        float s = 0.0f;
        for (int cc = 0; cc < g.m; ++cc) s += col[q * g.C + G * g.m + cc];
        dst[i] = s;
    }
}

// Folds the sample's block partials (every block of the sample does it, in double), then the elementwise work.
__global__ __launch_bounds__(kRThreads) void evo_apply_kernel(const float *__restrict__ x, RenGeom g, const float *__restrict__ v,
                                                              const float *__restrict__ gamma, const float *__restrict__ beta,
                                                              float eps, const float *__restrict__ parts, int stat_chunks,
                                                              float *__restrict__ y, float *__restrict__ mean_out,
                                                              float *__restrict__ var_out) {
    extern __shared__ float sinv[];  // [groups]: 1 / sqrt(var + eps)
    const int n = blockIdx.y;
    const double cnt = (double)g.HW * g.m;
    for (int G = threadIdx.x; G < g.groups; G += blockDim.x) {
        double s1 = 0.0, s2 = 0.0;
        const float *src = parts + (size_t)n * stat_chunks * g.groups * 2 + G * 2;
        for (int ch = 0; ch < stat_chunks; ++ch) { s1 += src[(size_t)ch * g.groups * 2]; s2 += src[(size_t)ch * g.groups * 2 + 1]; }
        const double mu = s1 / cnt;
        double var = s2 / cnt - mu * mu;
        if (var < 0.0) var = 0.0;
        sinv[G] = (float)(1.0 / sqrt(var + (double)eps));
        if (blockIdx.x == 0) { mean_out[(size_t)n * g.groups + G] = (float)mu; var_out[(size_t)n * g.groups + G] = (float)var; }
    }
    __syncthreads();
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    if ((int)threadIdx.x >= g.threads) return;
    float vv[4], gi[4], bb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = qd * 4 + j;
        vv[j] = v[c]; gi[j] = gamma[c] * sinv[c / g.m]; bb[j] = beta[c];
    }
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * g.HW * g.C);
    float4 *yv = reinterpret_cast<float4 *>(y + (size_t)n * g.HW * g.C);
    for (int pb = p0 + pl; pb < p1; pb += kRU * g.ppi) {
        float4 a[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) a[k] = load_or_zero(xv + (size_t)(pb + k * g.ppi) * g.cq + qd, pb + k * g.ppi < p1);
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float e[4] = {a[k].x, a[k].y, a[k].z, a[k].w};
            float o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = gi[j] * (e[j] * sigmoid_f(vv[j] * e[j])) + bb[j];
            yv[(size_t)p * g.cq + qd] = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
}

// Backward, pass 1: per block and channel  sum dy,  (sum dy u) / D,  sum dy gamma / D x^2 s',  sum dy gamma u
// parts[(row * 4 + q) * C + c], row = n * chunks + chunk
__global__ __launch_bounds__(kRThreads) void evo_bwd_reduce_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                                   RenGeom g, const float *__restrict__ v,
                                                                   const float *__restrict__ gamma, float eps,
                                                                   const float *__restrict__ var, float *__restrict__ parts) {
    extern __shared__ float sred[];  // [4][threads * 4]
    const int n = blockIdx.y;
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    const bool active = (int)threadIdx.x < g.threads;
    float vv[4], gg[4], inv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = min(qd * 4 + j, g.C - 1);
        vv[j] = v[c]; gg[j] = gamma[c];
        inv[j] = __fdiv_rn(1.0f, sqrtf(var[(size_t)n * g.groups + c / g.m] + eps));
    }
    float sb[4] = {0, 0, 0, 0}, sg[4] = {0, 0, 0, 0}, sv[4] = {0, 0, 0, 0}, st[4] = {0, 0, 0, 0};
    const size_t base = (size_t)n * g.HW * g.C;
    const float4 *xv = reinterpret_cast<const float4 *>(x + base), *dv4 = reinterpret_cast<const float4 *>(dy + base);
    for (int pb = p0 + pl; pb < p1 && active; pb += kRU * g.ppi) {
        float4 a[kRU], d[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const bool ok = pb + k * g.ppi < p1;
            a[k] = load_or_zero(xv + (size_t)(pb + k * g.ppi) * g.cq + qd, ok);
            d[k] = load_or_zero(dv4 + (size_t)(pb + k * g.ppi) * g.cq + qd, ok);
        }
#pragma unroll
        for (int k = 0; k < kRU; ++k) {  // pixels past the end have dy = 0 and add nothing
            const float e[4] = {a[k].x, a[k].y, a[k].z, a[k].w}, de[4] = {d[k].x, d[k].y, d[k].z, d[k].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float s = sigmoid_f(vv[j] * e[j]), sp = s * (1.0f - s), u = e[j] * s;
                sb[j] += de[j];
                sg[j] += de[j] * u;
                sv[j] += de[j] * gg[j] * inv[j] * e[j] * e[j] * sp;
                st[j] += de[j] * gg[j] * u;
            }
        }
    }
    const int T4 = g.threads * 4;
    if (active) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sred[0 * T4 + threadIdx.x * 4 + j] = sb[j];
            sred[1 * T4 + threadIdx.x * 4 + j] = sg[j] * inv[j];
            sred[2 * T4 + threadIdx.x * 4 + j] = sv[j];
            sred[3 * T4 + threadIdx.x * 4 + j] = st[j];
        }
    }
    __syncthreads();
    const size_t row = (size_t)n * g.chunks + blockIdx.x;
    for (int i = threadIdx.x; i < 4 * g.C; i += blockDim.x) parts[row * 4 * g.C + i] = column_sum(sred, T4, i / g.C, i % g.C, g);
}

// Column sums of `nq` quantities of parts[(row * stride_q + q) * C + c] over all rows, fixed order: 8 channels x 32 row
// lanes per block, four rows in flight per lane.  Thread (row lane sl < nq, channel) of the block ends with the sum.
__device__ __forceinline__ float fold_rows(const float *__restrict__ parts, int rows, int C, int stride_q, int nq, float (*s)[32][8]) {
    const int cl = threadIdx.x % 8, sl = threadIdx.x / 8;
    const int c = blockIdx.x * 8 + cl;
    for (int q = 0; q < nq; ++q) {
        double acc = 0.0;
        if (c < C)
            for (int r = sl; r < rows; r += 128) {
                float t[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) t[k] = r + 32 * k < rows ? parts[((size_t)(r + 32 * k) * stride_q + q) * C + c] : 0.0f;
                acc += ((double)t[0] + (double)t[1]) + ((double)t[2] + (double)t[3]);
            }
        s[q][sl][cl] = (float)acc;
    }
    __syncthreads();
    float t = 0.0f;
    if (sl < nq && c < C) {
        double a = 0.0;
        for (int k = 0; k < 32; ++k) a += s[sl][k][cl];
        t = (float)a;
    }
    return t;
}

// Backward, small launch: blocks [0, ceil(C/8)) finish dbeta, dgamma, dv; the others T[n][G] = sum over the slab of
// dy gamma u, one wave per (sample, group).
__global__ __launch_bounds__(256) void evo_bwd_fold_kernel(const float *__restrict__ parts, int rows, int N, int C, int groups, int m,
                                                           int chunks, float *__restrict__ dbeta, float *__restrict__ dgamma,
                                                           float *__restrict__ dv, float *__restrict__ T) {
    __shared__ float s[3][32][8];
    const int param_blocks = (C + 7) / 8;
    if ((int)blockIdx.x < param_blocks) {
        const float t = fold_rows(parts, rows, C, 4, 3, s);
        const int cl = threadIdx.x % 8, sl = threadIdx.x / 8, c = blockIdx.x * 8 + cl;
        if (sl < 3 && c < C) (sl == 0 ? dbeta : sl == 1 ? dgamma : dv)[c] = t;
        return;
    }
    const int i = (blockIdx.x - param_blocks) * (256 / kWave) + threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (i >= N * groups) return;
    const int n = i / groups, G = i % groups;
    double t = 0.0;
    for (int k = lane; k < chunks * m; k += kWave) {
        const int ch = k / m, cc = k - ch * m;
        t += parts[(((size_t)n * chunks + ch) * 4 + 3) * C + G * m + cc];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, 64);
    if (lane == 0) T[i] = (float)t;
}

// Backward, pass 2: dx = dy gamma / D (s + x v s') + dD (x - mean) / (count D),  dD = -T / D^2
__global__ __launch_bounds__(kRThreads) void evo_bwd_apply_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                                  RenGeom g, const float *__restrict__ v,
                                                                  const float *__restrict__ gamma, float eps,
                                                                  const float *__restrict__ mean, const float *__restrict__ var,
                                                                  const float *__restrict__ T, float *__restrict__ dx) {
    const int n = blockIdx.y;
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    if ((int)threadIdx.x >= g.threads) return;
    const float cnt = (float)g.HW * (float)g.m;
    float vv[4], gi[4], mu[4], coef[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = qd * 4 + j, G = c / g.m;
        const float D = sqrtf(var[(size_t)n * g.groups + G] + eps);
        vv[j] = v[c]; gi[j] = __fdiv_rn(gamma[c], D); mu[j] = mean[(size_t)n * g.groups + G];
        coef[j] = -T[(size_t)n * g.groups + G] / (D * D) / (cnt * D);
    }
    const size_t base = (size_t)n * g.HW * g.C;
    const float4 *xv = reinterpret_cast<const float4 *>(x + base), *dv4 = reinterpret_cast<const float4 *>(dy + base);
    float4 *ov = reinterpret_cast<float4 *>(dx + base);
    for (int pb = p0 + pl; pb < p1; pb += kRU * g.ppi) {
        float4 a[kRU], d[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const bool ok = pb + k * g.ppi < p1;
            a[k] = load_or_zero(xv + (size_t)(pb + k * g.ppi) * g.cq + qd, ok);
            d[k] = load_or_zero(dv4 + (size_t)(pb + k * g.ppi) * g.cq + qd, ok);
        }
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float e[4] = {a[k].x, a[k].y, a[k].z, a[k].w}, de[4] = {d[k].x, d[k].y, d[k].z, d[k].w};
            float o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float s = sigmoid_f(vv[j] * e[j]), sp = s * (1.0f - s);
                o[j] = de[j] * gi[j] * (s + e[j] * vv[j] * sp) + coef[j] * (e[j] - mu[j]);
            }
            ov[(size_t)p * g.cq + qd] = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
}

// ---------------------------------------------------------------- range batch-norm
// Per block and channel: the sum and the first arg-max / arg-min as packed keys (ordered value | ~flat pixel index).
// psum[row * C + c], pkey[(row * C + c) * 2 + {0, 1}]
__global__ __launch_bounds__(kRThreads) void rbn_stats_kernel(const float *__restrict__ x, RenGeom g, float *__restrict__ psum,
                                                              unsigned long long *__restrict__ pkey) {
    extern __shared__ unsigned long long skeys[];  // [C][2], then float [threads * 4]
    float *sred = reinterpret_cast<float *>(skeys + 2 * g.C);
    const int n = blockIdx.y;
    for (int i = threadIdx.x; i < 2 * g.C; i += blockDim.x) skeys[i] = 0ull;
    __syncthreads();
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    const bool active = (int)threadIdx.x < g.threads;
    float s1[4] = {0, 0, 0, 0}, mx[4] = {0, 0, 0, 0}, mn[4] = {0, 0, 0, 0};
    int imx[4] = {-1, -1, -1, -1}, imn[4] = {-1, -1, -1, -1};
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * g.HW * g.C);
    for (int pb = p0 + pl; pb < p1 && active; pb += kRU * g.ppi) {
        float4 a[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) a[k] = load_or_zero(xv + (size_t)(pb + k * g.ppi) * g.cq + qd, pb + k * g.ppi < p1);
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float e[4] = {a[k].x, a[k].y, a[k].z, a[k].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s1[j] += e[j];
                if (imx[j] < 0 || e[j] > mx[j]) { mx[j] = e[j]; imx[j] = p; }
                if (imn[j] < 0 || e[j] < mn[j]) { mn[j] = e[j]; imn[j] = p; }
            }
        }
    }
    if (active) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sred[threadIdx.x * 4 + j] = s1[j];
            if (imx[j] >= 0) {
                const int c = qd * 4 + j;
                const uint32_t fa = ~(uint32_t)(n * g.HW + imx[j]), fb = ~(uint32_t)(n * g.HW + imn[j]);
                atomicMax(&skeys[c * 2 + 0], ((unsigned long long)ordered_bits(mx[j]) << 32) | fa);
                atomicMax(&skeys[c * 2 + 1], ((unsigned long long)(~ordered_bits(mn[j])) << 32) | fb);
            }
        }
    }
    __syncthreads();
    const size_t row = (size_t)n * g.chunks + blockIdx.x;
    for (int c = threadIdx.x; c < g.C; c += blockDim.x) {
        psum[row * g.C + c] = column_sum(sred, 0, 0, c, g);
        pkey[(row * g.C + c) * 2 + 0] = skeys[c * 2 + 0];
        pkey[(row * g.C + c) * 2 + 1] = skeys[c * 2 + 1];
    }
}

// Per channel: mean (sum of the block sums in double), range and the two first positions; 8 channels x 32 row lanes.
__global__ __launch_bounds__(256) void rbn_fold_kernel(const float *__restrict__ psum, const unsigned long long *__restrict__ pkey,
                                                       int rows, int C, double count, float *__restrict__ mean_out,
                                                       float *__restrict__ range_out, long long *__restrict__ argmax_out,
                                                       long long *__restrict__ argmin_out) {
    __shared__ double ss[32][8];
    __shared__ unsigned long long sk[2][32][8];
    const int cl = threadIdx.x % 8, sl = threadIdx.x / 8, c = blockIdx.x * 8 + cl;
    double acc = 0.0;
    unsigned long long ka = 0ull, kb = 0ull;
    if (c < C)
        for (int r = sl; r < rows; r += 32) {
            acc += psum[(size_t)r * C + c];
            ka = max(ka, pkey[((size_t)r * C + c) * 2 + 0]);
            kb = max(kb, pkey[((size_t)r * C + c) * 2 + 1]);
        }
    ss[sl][cl] = acc; sk[0][sl][cl] = ka; sk[1][sl][cl] = kb;
    __syncthreads();
    if (sl == 0 && c < C) {
        double a = 0.0;
        for (int k = 0; k < 32; ++k) { a += ss[k][cl]; ka = max(ka, sk[0][k][cl]); kb = max(kb, sk[1][k][cl]); }
        const float mx = from_ordered_bits((uint32_t)(ka >> 32)), mn = from_ordered_bits(~(uint32_t)(kb >> 32));
        mean_out[c] = (float)(a / count);
        range_out[c] = __fsub_rn(mx, mn);
        argmax_out[c] = (long long)(~(uint32_t)ka);
        argmin_out[c] = (long long)(~(uint32_t)kb);
    }
}

__global__ __launch_bounds__(kRThreads) void rbn_apply_kernel(const float *__restrict__ x, RenGeom g, const float *__restrict__ gamma,
                                                              const float *__restrict__ beta, float cb, float eps,
                                                              const float *__restrict__ mean, const float *__restrict__ range,
                                                              float *__restrict__ y) {
    const int n = blockIdx.y;
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    if ((int)threadIdx.x >= g.threads) return;
    float gi[4], mu[4], bb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = qd * 4 + j;
        gi[j] = __fdiv_rn(gamma[c], __fmaf_rn(cb, range[c], eps)); mu[j] = mean[c]; bb[j] = beta[c];
    }
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * g.HW * g.C);
    float4 *yv = reinterpret_cast<float4 *>(y + (size_t)n * g.HW * g.C);
    for (int pb = p0 + pl; pb < p1; pb += kRU * g.ppi) {
        float4 a[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) a[k] = load_or_zero(xv + (size_t)(pb + k * g.ppi) * g.cq + qd, pb + k * g.ppi < p1);
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float e[4] = {a[k].x, a[k].y, a[k].z, a[k].w};
            yv[(size_t)p * g.cq + qd] = make_float4(gi[0] * (e[0] - mu[0]) + bb[0], gi[1] * (e[1] - mu[1]) + bb[1],
                                                     gi[2] * (e[2] - mu[2]) + bb[2], gi[3] * (e[3] - mu[3]) + bb[3]);
        }
    }
}

// Backward, pass 1: per block and channel  sum dy,  sum dy (x - mean):  parts[(row * 2 + q) * C + c]
__global__ __launch_bounds__(kRThreads) void rbn_bwd_reduce_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                                   RenGeom g, const float *__restrict__ mean,
                                                                   float *__restrict__ parts) {
    extern __shared__ float sred[];  // [2][threads * 4]
    const int n = blockIdx.y;
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    const bool active = (int)threadIdx.x < g.threads;
    float mu[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) mu[j] = mean[min(qd * 4 + j, g.C - 1)];
    float sa[4] = {0, 0, 0, 0}, sb[4] = {0, 0, 0, 0};
    const size_t base = (size_t)n * g.HW * g.C;
    const float4 *xv = reinterpret_cast<const float4 *>(x + base), *dv4 = reinterpret_cast<const float4 *>(dy + base);
    for (int pb = p0 + pl; pb < p1 && active; pb += kRU * g.ppi) {
        float4 a[kRU], d[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const bool ok = pb + k * g.ppi < p1;
            a[k] = load_or_zero(xv + (size_t)(pb + k * g.ppi) * g.cq + qd, ok);
            d[k] = load_or_zero(dv4 + (size_t)(pb + k * g.ppi) * g.cq + qd, ok);
        }
#pragma unroll
        for (int k = 0; k < kRU; ++k) {  // pixels past the end have dy = 0
            const float e[4] = {a[k].x, a[k].y, a[k].z, a[k].w}, de[4] = {d[k].x, d[k].y, d[k].z, d[k].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) { sa[j] += de[j]; sb[j] += de[j] * (e[j] - mu[j]); }
        }
    }
    const int T4 = g.threads * 4;
    if (active) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { sred[threadIdx.x * 4 + j] = sa[j]; sred[T4 + threadIdx.x * 4 + j] = sb[j]; }
    }
    __syncthreads();
    const size_t row = (size_t)n * g.chunks + blockIdx.x;
    for (int i = threadIdx.x; i < 2 * g.C; i += blockDim.x) parts[row * 2 * g.C + i] = column_sum(sred, T4, i / g.C, i % g.C, g);
}

// Per channel: dbeta, dgamma and the three numbers pass 2 needs: gamma / D, mean of dy, the range's gradient
__global__ __launch_bounds__(256) void rbn_bwd_fold_kernel(const float *__restrict__ parts, int rows, int C, float count, float cb,
                                                           float eps, const float *__restrict__ gamma,
                                                           const float *__restrict__ range, float *__restrict__ dgamma,
                                                           float *__restrict__ dbeta, float *__restrict__ coef) {
    __shared__ float s[3][32][8];
    __shared__ float both[2][8];
    const float t = fold_rows(parts, rows, C, 2, 2, s);
    const int cl = threadIdx.x % 8, sl = threadIdx.x / 8, c = blockIdx.x * 8 + cl;
    if (sl < 2) both[sl][cl] = t;
    __syncthreads();
    if (sl == 0 && c < C) {
        const float sdy = both[0][cl], sdyx = both[1][cl];
        const float D = __fmaf_rn(cb, range[c], eps), gd = __fdiv_rn(gamma[c], D);
        dbeta[c] = sdy;
        dgamma[c] = __fdiv_rn(sdyx, D);
        coef[c * 3 + 0] = gd;
        coef[c * 3 + 1] = __fdiv_rn(sdy, count);
        coef[c * 3 + 2] = cb * (-gd * __fdiv_rn(sdyx, D));
    }
}

// Backward, pass 2: dx = gamma / D (dy - mean dy), plus the range's gradient at the saved first arg-max (+) / arg-min (-)
__global__ __launch_bounds__(kRThreads) void rbn_bwd_apply_kernel(const float *__restrict__ dy, RenGeom g,
                                                                  const float *__restrict__ coef,
                                                                  const long long *__restrict__ argmax,
                                                                  const long long *__restrict__ argmin, float *__restrict__ dx) {
    const int n = blockIdx.y;
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    if ((int)threadIdx.x >= g.threads) return;
    float gd[4], md[4], dR[4];
    long long pa[4], pb_[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = qd * 4 + j;
        gd[j] = coef[c * 3]; md[j] = coef[c * 3 + 1]; dR[j] = coef[c * 3 + 2];
        pa[j] = argmax[c] - (long long)n * g.HW; pb_[j] = argmin[c] - (long long)n * g.HW;  // as pixels of this sample
    }
    const size_t base = (size_t)n * g.HW * g.C;
    const float4 *dv4 = reinterpret_cast<const float4 *>(dy + base);
    float4 *ov = reinterpret_cast<float4 *>(dx + base);
    for (int pb = p0 + pl; pb < p1; pb += kRU * g.ppi) {
        float4 d[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) d[k] = load_or_zero(dv4 + (size_t)(pb + k * g.ppi) * g.cq + qd, pb + k * g.ppi < p1);
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float de[4] = {d[k].x, d[k].y, d[k].z, d[k].w};
            float o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[j] = gd[j] * (de[j] - md[j]);
                if (p == pa[j]) o[j] += dR[j];
                if (p == pb_[j]) o[j] -= dR[j];
            }
            ov[(size_t)p * g.cq + qd] = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
}

static int check_shape(const char *what, int N, int H, int W, int C, int groups) {
    LPDT_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0, LPDT_EINVAL, "%s: sizes must be positive", what);
    LPDT_REQUIRE(groups > 0 && C % groups == 0, LPDT_EUNSUPPORTED, "%s: groups (%d) must divide C (%d)", what, groups, C);
    LPDT_REQUIRE(C % 4 == 0 && C / 4 <= kRThreads, LPDT_EUNSUPPORTED, "%s: C must be a multiple of 4, at most %d (got %d)", what,
                 4 * kRThreads, C);
    LPDT_REQUIRE((long long)N * H * W < 0x7fffffffLL && (long long)N * H * W * C < (1LL << 40), LPDT_EUNSUPPORTED,
                 "%s: tensor too large", what);
    return LPDT_OK;
}
static RenGeom geom(int N, int H, int W, int C, int groups) {
    return ren_geom(N, H, W, C, groups, kBwdMinPix, block_cap(N, H, W, C, kRefElems));
}

}  // namespace lpdt

using namespace lpdt;

// ---- EvoNorm-S0 entry points
extern "C" size_t lpdt_evonorm_s0_fwd_workspace_bytes(int N, int H, int W, int C, int groups) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || groups <= 0 || C % groups || C % 4 || C / 4 > kRThreads) return 0;
    return round_up((size_t)N * geom(N, H, W, C, groups).chunks * groups * 2 * sizeof(float), 256);
}
extern "C" size_t lpdt_evonorm_s0_bwd_workspace_bytes(int N, int H, int W, int C, int groups) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || groups <= 0 || C % groups || C % 4 || C / 4 > kRThreads) return 0;
    return round_up((size_t)N * geom(N, H, W, C, groups).chunks * 4 * C * sizeof(float), 256) + round_up((size_t)N * groups * sizeof(float), 256);
}

extern "C" int lpdt_evonorm_s0_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v, const float *gamma,
                                   const float *beta, float eps, float *y, float *mean_out, float *var_out, void *ws,
                                   size_t ws_bytes, void *stream) {
    int rc = check_shape("evonorm_s0_fwd", N, H, W, C, groups);
    if (rc) return rc;
    LPDT_REQUIRE(x && v && gamma && beta && y && mean_out && var_out, LPDT_EINVAL, "evonorm_s0_fwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "evonorm_s0_fwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(y, 16), LPDT_EINVAL, "evonorm_s0_fwd: x and y must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_evonorm_s0_fwd_workspace_bytes(N, H, W, C, groups));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const RenGeom g = geom(N, H, W, C, groups);
    float *parts = static_cast<float *>(ws);
    const size_t lds = ((size_t)8 * g.threads + 2 * C) * sizeof(float);
    hipLaunchKernelGGL(evo_stats_kernel, dim3(g.chunks, N), dim3(g.block), lds, st, x, g, parts);
    hipLaunchKernelGGL(evo_apply_kernel, dim3(g.chunks, N), dim3(g.block), groups * sizeof(float), st, x, g, v, gamma, beta, eps,
                       parts, g.chunks, y, mean_out, var_out);
    return launch_status("lpdt_evonorm_s0_fwd");
}

extern "C" int lpdt_evonorm_s0_bwd(const float *dy, const float *x, int N, int H, int W, int C, int groups, const float *v,
                                   const float *gamma, float eps, const float *mean, const float *var, float *dx, float *dv,
                                   float *dgamma, float *dbeta, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_shape("evonorm_s0_bwd", N, H, W, C, groups);
    if (rc) return rc;
    LPDT_REQUIRE(dy && x && v && gamma && mean && var && dx && dv && dgamma && dbeta, LPDT_EINVAL, "evonorm_s0_bwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "evonorm_s0_bwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(dy, 16) && aligned(dx, 16), LPDT_EINVAL, "evonorm_s0_bwd: x, dy and dx must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_evonorm_s0_bwd_workspace_bytes(N, H, W, C, groups));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const RenGeom g = geom(N, H, W, C, groups);
    const int rows = N * g.chunks;
    float *parts = static_cast<float *>(ws);
    float *T = reinterpret_cast<float *>(static_cast<char *>(ws) + round_up((size_t)rows * 4 * C * sizeof(float), 256));
    hipLaunchKernelGGL(evo_bwd_reduce_kernel, dim3(g.chunks, N), dim3(g.block), (size_t)16 * g.threads * sizeof(float), st, dy, x, g,
                       v, gamma, eps, var, parts);
    hipLaunchKernelGGL(evo_bwd_fold_kernel, dim3((C + 7) / 8 + (N * groups + 3) / 4), dim3(256), 0, st, parts, rows, N, C, groups,
                       C / groups, g.chunks, dbeta, dgamma, dv, T);
    hipLaunchKernelGGL(evo_bwd_apply_kernel, dim3(g.chunks, N), dim3(g.block), 0, st, dy, x, g, v, gamma, eps, mean, var, T, dx);
    return launch_status("lpdt_evonorm_s0_bwd");
}

// ---- range batch-norm entry points
static float range_bn_cb(int N) { return (float)(1.0 / std::sqrt(2.0 * std::log((double)N))); }

extern "C" size_t lpdt_range_bn_fwd_workspace_bytes(int N, int H, int W, int C) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 4 || C / 4 > kRThreads) return 0;
    const size_t rows = (size_t)N * geom(N, H, W, C, 1).chunks;
    return round_up(rows * C * sizeof(float), 256) + round_up(rows * C * 2 * sizeof(unsigned long long), 256);
}
extern "C" size_t lpdt_range_bn_bwd_workspace_bytes(int N, int H, int W, int C) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 4 || C / 4 > kRThreads) return 0;
    const size_t rows = (size_t)N * geom(N, H, W, C, 1).chunks;
    return round_up(rows * 2 * C * sizeof(float), 256) + round_up((size_t)C * 3 * sizeof(float), 256);
}

extern "C" int lpdt_range_bn_fwd(const float *x, int N, int H, int W, int C, const float *gamma, const float *beta, float eps,
                                 float *y, float *mean_out, float *range_out, int64_t *argmax_out, int64_t *argmin_out, void *ws,
                                 size_t ws_bytes, void *stream) {
    int rc = check_shape("range_bn_fwd", N, H, W, C, 1);
    if (rc) return rc;
    LPDT_REQUIRE(N >= 2, LPDT_EUNSUPPORTED, "range_bn_fwd: needs a batch of at least 2 (C(1) = 1/sqrt(2 ln 1) is infinite)");
    LPDT_REQUIRE(x && gamma && beta && y && mean_out && range_out && argmax_out && argmin_out, LPDT_EINVAL, "range_bn_fwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "range_bn_fwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(y, 16), LPDT_EINVAL, "range_bn_fwd: x and y must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_range_bn_fwd_workspace_bytes(N, H, W, C));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const RenGeom g = geom(N, H, W, C, 1);
    const int rows = N * g.chunks;
    float *psum = static_cast<float *>(ws);
    unsigned long long *pkey = reinterpret_cast<unsigned long long *>(static_cast<char *>(ws) + round_up((size_t)rows * C * sizeof(float), 256));
    const size_t lds = (size_t)2 * C * sizeof(unsigned long long) + (size_t)4 * g.threads * sizeof(float);
    hipLaunchKernelGGL(rbn_stats_kernel, dim3(g.chunks, N), dim3(g.block), lds, st, x, g, psum, pkey);
    hipLaunchKernelGGL(rbn_fold_kernel, dim3((C + 7) / 8), dim3(256), 0, st, psum, pkey, rows, C, (double)N * H * W, mean_out,
                       range_out, reinterpret_cast<long long *>(argmax_out), reinterpret_cast<long long *>(argmin_out));
    hipLaunchKernelGGL(rbn_apply_kernel, dim3(g.chunks, N), dim3(g.block), 0, st, x, g, gamma, beta, range_bn_cb(N), eps, mean_out,
                       range_out, y);
    return launch_status("lpdt_range_bn_fwd");
}

extern "C" int lpdt_range_bn_bwd(const float *dy, const float *x, int N, int H, int W, int C, const float *gamma, float eps,
                                 const float *mean, const float *range, const int64_t *argmax, const int64_t *argmin, float *dx,
                                 float *dgamma, float *dbeta, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_shape("range_bn_bwd", N, H, W, C, 1);
    if (rc) return rc;
    LPDT_REQUIRE(N >= 2, LPDT_EUNSUPPORTED, "range_bn_bwd: needs a batch of at least 2");
    LPDT_REQUIRE(dy && x && gamma && mean && range && argmax && argmin && dx && dgamma && dbeta, LPDT_EINVAL, "range_bn_bwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "range_bn_bwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(dy, 16) && aligned(dx, 16), LPDT_EINVAL, "range_bn_bwd: x, dy and dx must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_range_bn_bwd_workspace_bytes(N, H, W, C));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const RenGeom g = geom(N, H, W, C, 1);
    const int rows = N * g.chunks;
    float *parts = static_cast<float *>(ws);
    float *coef = reinterpret_cast<float *>(static_cast<char *>(ws) + round_up((size_t)rows * 2 * C * sizeof(float), 256));
    hipLaunchKernelGGL(rbn_bwd_reduce_kernel, dim3(g.chunks, N), dim3(g.block), (size_t)8 * g.threads * sizeof(float), st, dy, x, g,
                       mean, parts);
    hipLaunchKernelGGL(rbn_bwd_fold_kernel, dim3((C + 7) / 8), dim3(256), 0, st, parts, rows, C, (float)((double)N * H * W),
                       range_bn_cb(N), eps, gamma, range, dgamma, dbeta, coef);
    hipLaunchKernelGGL(rbn_bwd_apply_kernel, dim3(g.chunks, N), dim3(g.block), 0, st, dy, g, coef, reinterpret_cast<const long long *>(argmax),
                       reinterpret_cast<const long long *>(argmin), dx);
    return launch_status("lpdt_range_bn_bwd");
}
