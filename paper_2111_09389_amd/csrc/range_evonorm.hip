// Range-EvoNorm forward and backward (Eq. "ren"), fp32, NHWC.
//
// Both directions are HBM-bound.  A block owns a run of consecutive pixels of
// one sample, so its loads are one contiguous stream; the block's thread count
// is a multiple of C/4, which pins every thread to one quad of channels and lets
// it keep its running extrema / channel sums in registers.
//   forward : stats pass (per-block, per-group first arg-max / arg-min as packed 64-bit
//             keys, no global atomics) -> apply pass (each block first folds the block
//             keys of its sample, then does the elementwise work).  Two launches.
//             With int8 output (for layers that feed only convolutions): the stats pass
//             also takes per-channel extremes of u = x*hardsigmoid(v x), a one-block-per-
//             sample fold turns them into the exact max|y|, and the apply pass writes the
//             quantizer's codes instead of y.  Three launches, y never reaches memory.
//   backward: one pass writes the elementwise part of dx and per-block channel
//             partials; a second launch does the fixed-order reductions for dv, dgamma,
//             dbeta and, in its last block, adds the range gradient at the saved
//             arg-max / arg-min and reduces max|dx|.  Two launches.
#include "common.h"
#include "norm_geom.h"
#include <cmath>
#ifdef LPDT_TUNE
#include <cstdlib>
#endif

namespace lpdt {

__device__ __forceinline__ float hard_sigmoid(float z) { return fminf(1.0f, fmaxf(0.0f, (z + 3.0f) * (1.0f / 6.0f))); }
// The forward value with every rounding pinned (no contraction left to the compiler): the plain and the int8-output
// forward must produce the same bits, and the latter derives max|y| from extreme values of u, which relies on y being
// a monotone function of u for fixed gamma, inv > 0, beta -- true of this sequence of correctly rounded operations.
__device__ __forceinline__ float ren_y(float u, float gamma, float inv, float beta) { return __fmaf_rn(__fmul_rn(gamma, u), inv, beta); }

__global__ void ren_clear_kernel(unsigned long long *stats, int count, float *absmax) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) stats[i] = 0ull;
    if (i == 0 && absmax) *absmax = 0.0f;
}

// Key = ordered value (inverted for the minimum) in the high word, ~slab_index in the low word: the
// largest key is the extreme value at its lowest slab index.  pstats[((n*chunks + chunk)*groups + g)*2 + {0,1}]
// = this block's max key / min key (0 = the block saw no element of the group).
// kWithU: also the extreme values of u = x * hardsigmoid(v x) per block and channel, pu[((n*chunks + chunk)*C + c)*2 + {0,1}]
// = max / min (the int8-output forward derives max|y| from them).
template <bool kWithU>
__global__ __launch_bounds__(kRThreads) void ren_stats_kernel(const float *__restrict__ x, RenGeom g,
                                                              unsigned long long *__restrict__ pstats,
                                                              float *__restrict__ absmax_out, const float *__restrict__ vpar,
                                                              float *__restrict__ pu) {
    extern __shared__ unsigned long long skeys[];  // [groups][2]; with kWithU then unsigned su[C][2]
    unsigned int *su = reinterpret_cast<unsigned int *>(skeys + 2 * g.groups);
    const int n = blockIdx.y;
    if (absmax_out && blockIdx.x == 0 && n == 0 && threadIdx.x == 0) *absmax_out = 0.0f;  // a later pass max-es into it
    for (int i = threadIdx.x; i < 2 * g.groups; i += blockDim.x) skeys[i] = 0ull;
    if (kWithU)
        for (int i = threadIdx.x; i < 2 * g.C; i += blockDim.x) su[i] = 0u;
    __syncthreads();
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block;
    const int p1 = min(p0 + g.pix_per_block, g.HW);
    float mx[4], mn[4];
    int imx[4], imn[4];
    float umx[4], umn[4], vv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        imx[e] = -1; imn[e] = -1; mx[e] = 0.f; mn[e] = 0.f;
        umx[e] = -INFINITY; umn[e] = INFINITY; vv[e] = kWithU ? vpar[qd * 4 + e] : 0.f;
    }
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * g.HW * g.C);
    for (int pb = p0 + pl; pb < p1 && (int)threadIdx.x < g.threads; pb += kRU * g.ppi) {
        float4 a[kRU];
#pragma unroll
        for (int u = 0; u < kRU; ++u) {
            const int p = pb + u * g.ppi;
            a[u] = p < p1 ? xv[(size_t)p * g.cq + qd] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < kRU; ++u) {
            const int p = pb + u * g.ppi;
            if (p >= p1) break;
            const float v[4] = {a[u].x, a[u].y, a[u].z, a[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (imx[e] < 0 || v[e] > mx[e]) { mx[e] = v[e]; imx[e] = p; }
                if (imn[e] < 0 || v[e] < mn[e]) { mn[e] = v[e]; imn[e] = p; }
                if (kWithU) {
                    const float u = ren_u(v[e], vv[e]);
                    umx[e] = fmaxf(umx[e], u); umn[e] = fminf(umn[e], u);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (imx[e] < 0) continue;
        const int c = qd * 4 + e, grp = c / g.m, cc = c % g.m;
        const uint32_t lo_mx = ~(uint32_t)(imx[e] * g.m + cc), lo_mn = ~(uint32_t)(imn[e] * g.m + cc);
        atomicMax(&skeys[grp * 2 + 0], ((unsigned long long)ordered_bits(mx[e]) << 32) | lo_mx);
        atomicMax(&skeys[grp * 2 + 1], ((unsigned long long)(~ordered_bits(mn[e])) << 32) | lo_mn);
        if (kWithU) {
            atomicMax(&su[c * 2 + 0], ordered_bits(umx[e]));
            atomicMax(&su[c * 2 + 1], ~ordered_bits(umn[e]));
        }
    }
    __syncthreads();
    unsigned long long *dst = pstats + ((size_t)n * g.chunks + blockIdx.x) * g.groups * 2;
    for (int i = threadIdx.x; i < 2 * g.groups; i += blockDim.x) dst[i] = skeys[i];
    if (kWithU) {  // every block holds at least one pixel, so every channel has been seen
        float *du = pu + ((size_t)n * g.chunks + blockIdx.x) * g.C * 2;
        for (int i = threadIdx.x; i < 2 * g.C; i += blockDim.x) du[i] = from_ordered_bits(i % 2 ? ~su[i] : su[i]);
    }
}

// Any channel count: one element per thread step, keys straight into LDS atomics.
__global__ __launch_bounds__(kRThreads) void ren_stats_generic_kernel(const float *__restrict__ x, int HW, int C,
                                                                      int groups, int m, int elems_per_block,
                                                                      unsigned long long *__restrict__ stats) {
    extern __shared__ unsigned long long skeys[];
    const int n = blockIdx.y;
    for (int i = threadIdx.x; i < 2 * groups; i += blockDim.x) skeys[i] = 0ull;
    __syncthreads();
    const long long total = (long long)HW * C;
    const long long e0 = (long long)blockIdx.x * elems_per_block;
    const long long e1 = min(e0 + (long long)elems_per_block, total);
    const float *xs = x + (size_t)n * total;
    for (long long i = e0 + threadIdx.x; i < e1; i += blockDim.x) {
        const float v = xs[i];
        const int p = (int)(i / C), c = (int)(i % C), grp = c / m, cc = c % m;
        const uint32_t lo = ~(uint32_t)(p * m + cc);
        atomicMax(&skeys[grp * 2 + 0], ((unsigned long long)ordered_bits(v) << 32) | lo);
        atomicMax(&skeys[grp * 2 + 1], ((unsigned long long)(~ordered_bits(v)) << 32) | lo);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * groups; i += blockDim.x)
        if (skeys[i]) atomicMax(&stats[(size_t)n * groups * 2 + i], skeys[i]);
}

__global__ void ren_finalize_kernel(const unsigned long long *__restrict__ stats, int count, float *__restrict__ range_out,
                                    int32_t *__restrict__ argmax_out, int32_t *__restrict__ argmin_out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const unsigned long long kmx = stats[2 * i], kmn = stats[2 * i + 1];
    const float mx = from_ordered_bits((uint32_t)(kmx >> 32));
    const float mn = from_ordered_bits(~(uint32_t)(kmn >> 32));
    range_out[i] = __fsub_rn(mx, mn);
    argmax_out[i] = (int32_t)(~(uint32_t)kmx);
    argmin_out[i] = (int32_t)(~(uint32_t)kmn);
}

__device__ __forceinline__ float inv_denominator(float range, float cm, float eps) {
    return __fdiv_rn(1.0f, __fmaf_rn(cm, range, eps));
}

__device__ __forceinline__ void block_absmax_commit(float m, float *absmax_out, float *lds) {
    m = wave_max(m);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (lane == 0) lds[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = lds[0];
        for (int w = 1; w < (int)(blockDim.x + kWave - 1) / kWave; ++w) r = fmaxf(r, lds[w]);
        atomicMax(reinterpret_cast<unsigned int *>(absmax_out), __float_as_uint(r));  // r >= 0: bit order = value order
    }
}

// max over the block, written (not max-ed) to *dst: partial results, one per block
__device__ __forceinline__ void block_absmax_store(float m, float *dst, float *lds) {
    m = wave_max(m);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (lane == 0) lds[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = lds[0];
        for (int w = 1; w < (int)(blockDim.x + kWave - 1) / kWave; ++w) r = fmaxf(r, lds[w]);
        *dst = r;
    }
}

__global__ __launch_bounds__(kRThreads) void ren_apply_kernel(const float *__restrict__ x, RenGeom g,
                                                              const float *__restrict__ v,
                                                              const float *__restrict__ gamma,
                                                              const float *__restrict__ beta, float cm, float eps,
                                                              const unsigned long long *__restrict__ pstats, int stat_chunks,
                                                              float *__restrict__ y, float *__restrict__ range_out,
                                                              int32_t *__restrict__ argmax_out, int32_t *__restrict__ argmin_out,
                                                              float *__restrict__ absmax_out) {
    extern __shared__ unsigned long long skeys[];  // [groups][2], then float range[groups]
    __shared__ float lds[kRThreads / kWave];
    float *srange = reinterpret_cast<float *>(skeys + 2 * g.groups);
    const int n = blockIdx.y;
    // fold the per-block keys of this sample (every block of the sample does it: a few KB out of L2)
    {
        const int nk = 2 * g.groups;
        for (int i = threadIdx.x; i < nk; i += blockDim.x) skeys[i] = 0ull;
        __syncthreads();
        const unsigned long long *src = pstats + (size_t)n * stat_chunks * nk;  // [chunks][nk]: one contiguous run
        for (int i = threadIdx.x; i < stat_chunks * nk; i += blockDim.x) {
            const unsigned long long k = src[i];
            if (k) atomicMax(&skeys[i % nk], k);
        }
        __syncthreads();
    }
    for (int grp = threadIdx.x; grp < g.groups; grp += blockDim.x) {
        const unsigned long long kmx = skeys[2 * grp], kmn = skeys[2 * grp + 1];
        const float r = __fsub_rn(from_ordered_bits((uint32_t)(kmx >> 32)), from_ordered_bits(~(uint32_t)(kmn >> 32)));
        srange[grp] = r;
        if (blockIdx.x == 0) {
            range_out[(size_t)n * g.groups + grp] = r;
            argmax_out[(size_t)n * g.groups + grp] = (int32_t)(~(uint32_t)kmx);
            argmin_out[(size_t)n * g.groups + grp] = (int32_t)(~(uint32_t)kmn);
        }
    }
    __syncthreads();
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block;
    const int p1 = min(p0 + g.pix_per_block, g.HW);
    const bool active = (int)threadIdx.x < g.threads;
    float vv[4], gg[4], bb[4], inv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int c = qd * 4 + e;
        vv[e] = v[c]; gg[e] = gamma[c]; bb[e] = beta[c];
        inv[e] = inv_denominator(srange[c / g.m], cm, eps);
    }
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * g.HW * g.C);
    float4 *yv = reinterpret_cast<float4 *>(y + (size_t)n * g.HW * g.C);
    float am = 0.0f;
    for (int pb = p0 + pl; pb < p1 && active; pb += kRU * g.ppi) {
        float4 a[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            a[k] = p < p1 ? xv[(size_t)p * g.cq + qd] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float xe[4] = {a[k].x, a[k].y, a[k].z, a[k].w};
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = ren_y(ren_u(xe[e], vv[e]), gg[e], inv[e], bb[e]);
                am = fmaxf(am, fabsf(o[e]));
            }
            yv[(size_t)p * g.cq + qd] = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
    if (absmax_out) block_absmax_commit(am, absmax_out, lds);
}

__global__ __launch_bounds__(kRThreads) void ren_apply_generic_kernel(const float *__restrict__ x, int HW, int C, int groups,
                                                                      int m, int elems_per_block,
                                                                      const float *__restrict__ v,
                                                                      const float *__restrict__ gamma,
                                                                      const float *__restrict__ beta, float cm, float eps,
                                                                      const float *__restrict__ range,
                                                                      float *__restrict__ y, float *__restrict__ absmax_out) {
    __shared__ float lds[kRThreads / kWave];
    const int n = blockIdx.y;
    const long long total = (long long)HW * C;
    const long long e0 = (long long)blockIdx.x * elems_per_block;
    const long long e1 = min(e0 + (long long)elems_per_block, total);
    float am = 0.0f;
    for (long long i = e0 + threadIdx.x; i < e1; i += blockDim.x) {
        const int c = (int)(i % C);
        const float xe = x[(size_t)n * total + i];
        const float inv = inv_denominator(range[(size_t)n * groups + c / m], cm, eps);
        const float o = ren_y(ren_u(xe, v[c]), gamma[c], inv, beta[c]);
        y[(size_t)n * total + i] = o;
        am = fmaxf(am, fabsf(o));
    }
    if (absmax_out) block_absmax_commit(am, absmax_out, lds);
}

// ---- forward with int8 output -------------------------------------------------
// Second launch of the int8-output forward, one block per sample: folds the sample's block keys (range and positions
// for the backward pass) and the per-channel extremes of u, and from those the sample's max|y|: for fixed gamma,
// inv > 0 and beta, y is a monotone function of u, so the extreme y of a channel sit at its extreme u.
__global__ __launch_bounds__(256) void ren_q_fold_kernel(RenGeom g, const unsigned long long *__restrict__ pstats,
                                                         const float *__restrict__ pu, const float *__restrict__ gamma,
                                                         const float *__restrict__ beta, float cm, float eps,
                                                         float *__restrict__ range_out, int32_t *__restrict__ argmax_out,
                                                         int32_t *__restrict__ argmin_out, float *__restrict__ absmax) {
    extern __shared__ unsigned long long skeys[];  // [groups][2], then float inv[groups], then unsigned su[C][2]
    __shared__ float lds[256 / kWave];
    float *sinv = reinterpret_cast<float *>(skeys + 2 * g.groups);
    unsigned int *su = reinterpret_cast<unsigned int *>(sinv + g.groups);
    const int n = blockIdx.x, nk = 2 * g.groups;
    for (int i = threadIdx.x; i < nk; i += blockDim.x) skeys[i] = 0ull;
    for (int i = threadIdx.x; i < 2 * g.C; i += blockDim.x) su[i] = 0u;
    __syncthreads();
    // per-channel extremes of u over the sample's blocks: the threads of a channel split the blocks between them
    {
        const int parts = g.C < 256 ? 256 / g.C : 1;
        const float2 *p2 = reinterpret_cast<const float2 *>(pu + (size_t)n * g.chunks * g.C * 2);
        for (int i = threadIdx.x; i < g.C * parts; i += blockDim.x) {
            const int c = i % g.C, part = i / g.C;
            float hi = -INFINITY, lo = INFINITY;
            for (int ch0 = part; ch0 < g.chunks; ch0 += 4 * parts) {   // 4 loads in flight
                float2 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    v[k] = ch0 + k * parts < g.chunks ? p2[(size_t)(ch0 + k * parts) * g.C + c] : make_float2(-INFINITY, INFINITY);
#pragma unroll
                for (int k = 0; k < 4; ++k) { hi = fmaxf(hi, v[k].x); lo = fminf(lo, v[k].y); }
            }
            if (part < g.chunks) {
                atomicMax(&su[c * 2 + 0], ordered_bits(hi));
                atomicMax(&su[c * 2 + 1], ~ordered_bits(lo));
            }
        }
    }
    const unsigned long long *src = pstats + (size_t)n * g.chunks * nk;
    for (int i0 = threadIdx.x; i0 < g.chunks * nk; i0 += 4 * blockDim.x) {   // 4 loads in flight
        unsigned long long k[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) k[j] = i0 + j * (int)blockDim.x < g.chunks * nk ? src[i0 + j * blockDim.x] : 0ull;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (k[j]) atomicMax(&skeys[(i0 + j * blockDim.x) % nk], k[j]);
    }
    __syncthreads();
    for (int grp = threadIdx.x; grp < g.groups; grp += blockDim.x) {
        const unsigned long long kmx = skeys[2 * grp], kmn = skeys[2 * grp + 1];
        const float r = __fsub_rn(from_ordered_bits((uint32_t)(kmx >> 32)), from_ordered_bits(~(uint32_t)(kmn >> 32)));
        sinv[grp] = inv_denominator(r, cm, eps);
        range_out[(size_t)n * g.groups + grp] = r;
        argmax_out[(size_t)n * g.groups + grp] = (int32_t)(~(uint32_t)kmx);
        argmin_out[(size_t)n * g.groups + grp] = (int32_t)(~(uint32_t)kmn);
    }
    __syncthreads();
    float am = 0.0f;
    for (int c = threadIdx.x; c < g.C; c += blockDim.x) {
        const float hi = from_ordered_bits(su[c * 2 + 0]), lo = from_ordered_bits(~su[c * 2 + 1]);
        const float inv = sinv[c / g.m], gg = gamma[c], bb = beta[c];
        am = fmaxf(am, fmaxf(fabsf(ren_y(hi, gg, inv, bb)), fabsf(ren_y(lo, gg, inv, bb))));
    }
    block_absmax_commit(am, absmax, lds);
}

// First and second launch in one for small samples (the late layers: a sample of 25-100 K elements): one block of
// kSampleThreads threads walks its whole sample, so the sample's fold needs no second launch.  The three launches of
// such a layer are bound by launch latency, not by bytes.  The sample's max|y| goes to sample_abs[n] (a plain store: no
// array to clear first); the pass that emits the codes takes the maximum over the samples.  Same arithmetic and the same
// order-free reductions (maxima of keys) as ren_stats_kernel<true> + ren_q_fold_kernel: same bits.
constexpr int kSampleThreads = 1024;
constexpr int kSampleRU = 8;      // pixels a thread has in flight
__global__ __launch_bounds__(kSampleThreads) void ren_sample_kernel(const float *__restrict__ x, int HW, int C, int groups, int m,
                                                                     const float *__restrict__ vpar, const float *__restrict__ gamma,
                                                                     const float *__restrict__ beta, float cm, float eps,
                                                                     float *__restrict__ range_out, int32_t *__restrict__ argmax_out,
                                                                     int32_t *__restrict__ argmin_out, float *__restrict__ sample_abs) {
    extern __shared__ unsigned long long skeys[];  // [groups][2], then float inv[groups], then unsigned su[C][2]
    __shared__ float lds[kSampleThreads / kWave];
    float *sinv = reinterpret_cast<float *>(skeys + 2 * groups);
    unsigned int *su = reinterpret_cast<unsigned int *>(sinv + groups);
    const int n = blockIdx.x, cq = C / 4;
    for (int i = threadIdx.x; i < 2 * groups; i += blockDim.x) skeys[i] = 0ull;
    for (int i = threadIdx.x; i < 2 * C; i += blockDim.x) su[i] = 0u;
    __syncthreads();
    const int ppi = kSampleThreads / cq;            // pixels per round of the block; threads past ppi * cq only join the barriers
    const int qd = threadIdx.x % cq, pl = threadIdx.x / cq;
    if (pl < ppi) {
        float mx[4], mn[4], umx[4], umn[4], vv[4];
        int imx[4], imn[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            imx[e] = -1; imn[e] = -1; mx[e] = 0.f; mn[e] = 0.f;
            umx[e] = -INFINITY; umn[e] = INFINITY; vv[e] = vpar[qd * 4 + e];
        }
        const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * HW * C);
        for (int pb = pl; pb < HW; pb += kSampleRU * ppi) {
            float4 a[kSampleRU];
#pragma unroll
            for (int u = 0; u < kSampleRU; ++u) {
                const int p = pb + u * ppi;
                a[u] = p < HW ? xv[(size_t)p * cq + qd] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < kSampleRU; ++u) {
                const int p = pb + u * ppi;
                if (p >= HW) break;
                const float v[4] = {a[u].x, a[u].y, a[u].z, a[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (imx[e] < 0 || v[e] > mx[e]) { mx[e] = v[e]; imx[e] = p; }
                    if (imn[e] < 0 || v[e] < mn[e]) { mn[e] = v[e]; imn[e] = p; }
                    const float uu = ren_u(v[e], vv[e]);
                    umx[e] = fmaxf(umx[e], uu); umn[e] = fminf(umn[e], uu);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (imx[e] < 0) continue;
            const int c = qd * 4 + e, grp = c / m, cc = c % m;
            const uint32_t lo_mx = ~(uint32_t)(imx[e] * m + cc), lo_mn = ~(uint32_t)(imn[e] * m + cc);
            atomicMax(&skeys[grp * 2 + 0], ((unsigned long long)ordered_bits(mx[e]) << 32) | lo_mx);
            atomicMax(&skeys[grp * 2 + 1], ((unsigned long long)(~ordered_bits(mn[e])) << 32) | lo_mn);
            atomicMax(&su[c * 2 + 0], ordered_bits(umx[e]));
            atomicMax(&su[c * 2 + 1], ~ordered_bits(umn[e]));
        }
    }
    __syncthreads();
    for (int grp = threadIdx.x; grp < groups; grp += blockDim.x) {
        const unsigned long long kmx = skeys[2 * grp], kmn = skeys[2 * grp + 1];
        const float r = __fsub_rn(from_ordered_bits((uint32_t)(kmx >> 32)), from_ordered_bits(~(uint32_t)(kmn >> 32)));
        sinv[grp] = inv_denominator(r, cm, eps);
        range_out[(size_t)n * groups + grp] = r;
        argmax_out[(size_t)n * groups + grp] = (int32_t)(~(uint32_t)kmx);
        argmin_out[(size_t)n * groups + grp] = (int32_t)(~(uint32_t)kmn);
    }
    __syncthreads();
    float am = 0.0f;
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        const float hi = from_ordered_bits(su[c * 2 + 0]), lo = from_ordered_bits(~su[c * 2 + 1]);
        const float inv = sinv[c / m], gg = gamma[c], bb = beta[c];
        am = fmaxf(am, fmaxf(fabsf(ren_y(hi, gg, inv, bb)), fabsf(ren_y(lo, gg, inv, bb))));
    }
    block_absmax_store(am, sample_abs + n, lds);
}

// The int8-output forward behind a convolution that took the statistics in its epilogue: cstats[n][C][4] holds, as
// ordered bit patterns, max x, ~min x, max u, ~min u of every sample and channel.  One block per sample folds the
// channels of a group into the group's extremes (range for the backward pass, extremes for the position search of the
// apply pass, positions preset to INT_MAX) and evaluates y at the channels' extreme u for the exact max|y|.
__global__ __launch_bounds__(256) void ren_cfold_kernel(RenGeom g, const unsigned *__restrict__ cstats, const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, float cm, float eps,
                                                        float *__restrict__ range_out, float *__restrict__ gext,
                                                        int32_t *__restrict__ argmax_out, int32_t *__restrict__ argmin_out,
                                                        float *__restrict__ absmax) {
    extern __shared__ unsigned sgk[];   // [groups][2] ordered max x, ~ordered min x; then float inv[groups]
    __shared__ float lds[256 / kWave];
    float *sinv = reinterpret_cast<float *>(sgk + 2 * g.groups);
    const int n = blockIdx.x;
    for (int i = threadIdx.x; i < 2 * g.groups; i += blockDim.x) sgk[i] = 0u;
    __syncthreads();
    const unsigned *src = cstats + (size_t)n * g.C * 4;
    for (int c = threadIdx.x; c < g.C; c += blockDim.x) {
        atomicMax(&sgk[(c / g.m) * 2 + 0], src[c * 4 + 0]);
        atomicMax(&sgk[(c / g.m) * 2 + 1], src[c * 4 + 1]);
    }
    __syncthreads();
    for (int grp = threadIdx.x; grp < g.groups; grp += blockDim.x) {
        const float hi = from_ordered_bits(sgk[2 * grp]), lo = from_ordered_bits(~sgk[2 * grp + 1]);
        const float r = __fsub_rn(hi, lo);
        sinv[grp] = inv_denominator(r, cm, eps);
        range_out[(size_t)n * g.groups + grp] = r;
        gext[((size_t)n * g.groups + grp) * 2 + 0] = hi;
        gext[((size_t)n * g.groups + grp) * 2 + 1] = lo;
        argmax_out[(size_t)n * g.groups + grp] = 0x7fffffff;
        argmin_out[(size_t)n * g.groups + grp] = 0x7fffffff;
    }
    __syncthreads();
    float am = 0.0f;
    for (int c = threadIdx.x; c < g.C; c += blockDim.x) {
        const float hi = from_ordered_bits(src[c * 4 + 2]), lo = from_ordered_bits(~src[c * 4 + 3]);
        const float inv = sinv[c / g.m], gg = gamma[c], bb = beta[c];
        am = fmaxf(am, fmaxf(fabsf(ren_y(hi, gg, inv, bb)), fabsf(ren_y(lo, gg, inv, bb))));
    }
    block_absmax_commit(am, absmax, lds);
}

__global__ void ren_cstats_clear_kernel(unsigned *cstats, size_t count, float *absmax) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) cstats[i] = 0u;
    if (i == 0) *absmax = 0.0f;
}

// Third launch: y as the plain forward computes it, rounded to the nearest code with the scale max|y| / 127.
__global__ __launch_bounds__(kRThreads) void ren_apply_q_kernel(const float *__restrict__ x, RenGeom g, const float *__restrict__ v,
                                                                const float *__restrict__ gamma, const float *__restrict__ beta,
                                                                float cm, float eps, const float *__restrict__ range,
                                                                const float *__restrict__ absmax, int nabs, int8_t *__restrict__ q,
                                                                float *__restrict__ scale, float *__restrict__ y,
                                                                const float *__restrict__ gext, int32_t *__restrict__ argmax,
                                                                int32_t *__restrict__ argmin) {
    // gext != NULL: the extremes of every (sample, group) are known ([n][group][max, min]) but not where they sit: every
    // element equal to one reports its position, the lowest wins (argmax / argmin start at INT_MAX)
    // absmax: max|y| of the tensor, or (nabs > 1) of every sample: the same addresses for all threads, loads in flight together
    const int n = blockIdx.y;
    float a = absmax[0];
#pragma unroll 8
    for (int i = 1; i < nabs; ++i) a = fmaxf(a, absmax[i]);
    if (blockIdx.x == 0 && n == 0 && threadIdx.x == 0) *scale = quant_scale(a);
    if ((int)threadIdx.x >= g.threads) return;
    const float qinv = quant_inv(a);
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    float vv[4], gg[4], bb[4], inv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int c = qd * 4 + e;
        vv[e] = v[c]; gg[e] = gamma[c]; bb[e] = beta[c];
        inv[e] = inv_denominator(range[(size_t)n * g.groups + c / g.m], cm, eps);
    }
    float hi[4] = {0.f, 0.f, 0.f, 0.f}, lo[4] = {0.f, 0.f, 0.f, 0.f};
    if (gext) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            hi[e] = gext[((size_t)n * g.groups + (qd * 4 + e) / g.m) * 2 + 0];
            lo[e] = gext[((size_t)n * g.groups + (qd * 4 + e) / g.m) * 2 + 1];
        }
    }
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * g.HW * g.C);
    uint32_t *qv = reinterpret_cast<uint32_t *>(q + (size_t)n * g.HW * g.C);
    for (int pb = p0 + pl; pb < p1; pb += kRU * g.ppi) {
        float4 t[kRU];
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            t[k] = p < p1 ? xv[(size_t)p * g.cq + qd] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < kRU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float xe[4] = {t[k].x, t[k].y, t[k].z, t[k].w};
            float o[4];
            uint32_t word = 0u;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = ren_y(ren_u(xe[e], vv[e]), gg[e], inv[e], bb[e]);
                word |= ((uint32_t)round_code(o[e], qinv, false, 0u) & 0xffu) << (8 * e);
                if (gext) {
                    const int c = qd * 4 + e;
                    if (xe[e] == hi[e]) atomicMin(&argmax[(size_t)n * g.groups + c / g.m], p * g.m + c % g.m);
                    if (xe[e] == lo[e]) atomicMin(&argmin[(size_t)n * g.groups + c / g.m], p * g.m + c % g.m);
                }
            }
            qv[(size_t)p * g.cq + qd] = word;
            if (y) reinterpret_cast<float4 *>(y + (size_t)n * g.HW * g.C)[(size_t)p * g.cq + qd] = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
}

// ---- forward followed by a max-pool --------------------------------------------
struct PoolGeom {   // input width, pooled map, window, stride, padding
    int W, P, Q, k, st, pd;
    unsigned mul_w, mul_q, mul_st;   // multipliers for x/W, x/Q, x/st by a high multiply (0: divide), see pool_geom()
};
// x / d for 0 <= x below the bound its multiplier was made for
__device__ __forceinline__ int pool_div(int x, int d, unsigned mul) { return mul ? (int)__umulhi((unsigned)x, mul) : x / d; }
// z = maxpool(y) and the winners' positions, with y evaluated at the window's pixels instead of being stored: the
// arithmetic of the plain forward (ren_y) and the selection rule of the max-pool kernel (first in window scan order on
// ties, padding never wins), so the results are the two calls' bit for bit.  g describes the POOLED map (HW = P*Q).
__global__ __launch_bounds__(kRThreads) void ren_pool_kernel(const float *__restrict__ x, RenGeom g, int H, int W, PoolGeom pg,
                                                             const float *__restrict__ v, const float *__restrict__ gamma,
                                                             const float *__restrict__ beta, float cm, float eps,
                                                             const unsigned long long *__restrict__ pstats, int stat_chunks,
                                                             float *__restrict__ z, int32_t *__restrict__ idx,
                                                             float *__restrict__ range_out, int32_t *__restrict__ argmax_out,
                                                             int32_t *__restrict__ argmin_out, float *__restrict__ absmax_out) {
    extern __shared__ unsigned long long skeys[];  // [groups][2], then float range[groups]
    __shared__ float lds[kRThreads / kWave];
    float *srange = reinterpret_cast<float *>(skeys + 2 * g.groups);
    const int n = blockIdx.y;
    {
        const int nk = 2 * g.groups;
        for (int i = threadIdx.x; i < nk; i += blockDim.x) skeys[i] = 0ull;
        __syncthreads();
        const unsigned long long *src = pstats + (size_t)n * stat_chunks * nk;
        for (int i = threadIdx.x; i < stat_chunks * nk; i += blockDim.x) {
            const unsigned long long k = src[i];
            if (k) atomicMax(&skeys[i % nk], k);
        }
        __syncthreads();
    }
    for (int grp = threadIdx.x; grp < g.groups; grp += blockDim.x) {
        const unsigned long long kmx = skeys[2 * grp], kmn = skeys[2 * grp + 1];
        const float r = __fsub_rn(from_ordered_bits((uint32_t)(kmx >> 32)), from_ordered_bits(~(uint32_t)(kmn >> 32)));
        srange[grp] = r;
        if (blockIdx.x == 0) {
            range_out[(size_t)n * g.groups + grp] = r;
            argmax_out[(size_t)n * g.groups + grp] = (int32_t)(~(uint32_t)kmx);
            argmin_out[(size_t)n * g.groups + grp] = (int32_t)(~(uint32_t)kmn);
        }
    }
    __syncthreads();
    const bool active = (int)threadIdx.x < g.threads;
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block, p1 = min(p0 + g.pix_per_block, g.HW);
    float vv[4], gg[4], bb[4], inv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int c = qd * 4 + e;
        vv[e] = v[c]; gg[e] = gamma[c]; bb[e] = beta[c];
        inv[e] = inv_denominator(srange[c / g.m], cm, eps);
    }
    const float4 *xv = reinterpret_cast<const float4 *>(x + (size_t)n * H * W * g.C);
    float4 *zv = reinterpret_cast<float4 *>(z + (size_t)n * g.HW * g.C);
    int4 *iv = reinterpret_cast<int4 *>(idx + (size_t)n * g.HW * g.C);
    float am = 0.0f;
    for (int pp = p0 + pl; pp < p1 && active; pp += g.ppi) {
        const int p = pool_div(pp, pg.Q, pg.mul_q), q = pp - p * pg.Q;
        float best[4] = {0.f, 0.f, 0.f, 0.f};
        int bi[4] = {-1, -1, -1, -1};
        auto take = [&](const float4 &t, int pos) {   // window scan order: a later pixel wins only if strictly larger
            const float xe[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float y = ren_y(ren_u(xe[e], vv[e]), gg[e], inv[e], bb[e]);
                if (bi[e] < 0 || y > best[e]) { best[e] = y; bi[e] = pos; }
            }
        };
        if (pg.k <= 3) {
            // windows of up to 3 x 3: all loads of the window go out together (a pixel outside the window or the map
            // is fetched from a clamped position and skipped)
            float4 t[9];
            int pos[9];
#pragma unroll
            for (int i = 0; i < 3; ++i)
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const int h = p * pg.st + i - pg.pd, w = q * pg.st + j - pg.pd;
                    const bool ok = i < pg.k && j < pg.k && h >= 0 && h < H && w >= 0 && w < W;
                    const int hc = min(max(h, 0), H - 1), wc = min(max(w, 0), W - 1);
                    pos[i * 3 + j] = ok ? h * W + w : -1;
                    t[i * 3 + j] = xv[(size_t)(hc * W + wc) * g.cq + qd];
                }
#pragma unroll
            for (int s = 0; s < 9; ++s)
                if (pos[s] >= 0) take(t[s], pos[s]);
        } else {
            for (int i = 0; i < pg.k; ++i) {
                const int h = p * pg.st + i - pg.pd;
                if (h < 0 || h >= H) continue;
                for (int j = 0; j < pg.k; ++j) {
                    const int w = q * pg.st + j - pg.pd;
                    if (w < 0 || w >= W) continue;
                    take(xv[(size_t)(h * W + w) * g.cq + qd], h * W + w);
                }
            }
        }
        zv[(size_t)pp * g.cq + qd] = make_float4(best[0], best[1], best[2], best[3]);
        iv[(size_t)pp * g.cq + qd] = make_int4(bi[0], bi[1], bi[2], bi[3]);
        am = fmaxf(fmaxf(am, fmaxf(fabsf(best[0]), fabsf(best[1]))), fmaxf(fabsf(best[2]), fabsf(best[3])));
    }
    if (absmax_out) block_absmax_commit(am, absmax_out, lds);   // zeroed by the stats pass
}

// ---- backward ---------------------------------------------------------------
// Per element: z = v x, s = hs(z), s' = 1/6 on (-3,3), u = x s, du = dy gamma / D,
//   dx = du (s + x v s'),  dbeta += dy,  dgamma += dy u / D,  dv += du x^2 s',
//   T += dy gamma u   (dD = -T / D^2, dRange = C(m) dD).
// parts layout: [row = n*chunks + chunk][4 quantities][C]
// The layer's output gradient at one pixel when the output went through a max-pool only: the sum, over the (at most
// 2 x 2) windows holding the pixel, of the pooled gradients whose winner it was -- the arithmetic of the max-pool
// backward kernel (same order of additions), evaluated where it is consumed.  dz, idx: this sample's pooled maps.
__device__ __forceinline__ float4 pooled_grad(const float4 *__restrict__ dz, const int4 *__restrict__ idx, int p, const PoolGeom &pg,
                                              int cq, int qd) {
    // (a negative numerator means no window that far up or left: the first window is 0 either way)
    const int h = pool_div(p, pg.W, pg.mul_w), w = p - h * pg.W;
    const int p_lo = pool_div(max(0, h + pg.pd - pg.k + pg.st), pg.st, pg.mul_st), p_hi = min(pg.P - 1, pool_div(h + pg.pd, pg.st, pg.mul_st));
    const int q_lo = pool_div(max(0, w + pg.pd - pg.k + pg.st), pg.st, pg.mul_st), q_hi = min(pg.Q - 1, pool_div(w + pg.pd, pg.st, pg.mul_st));
    int4 id[4];
    float4 gq[4];
    size_t at[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int pp = p_lo + j / 2, qq = q_lo + j % 2;
        const bool ok = pp <= p_hi && qq <= q_hi;
        at[j] = (size_t)(pp * pg.Q + qq) * cq + qd;
        id[j] = ok ? idx[at[j]] : make_int4(-1, -1, -1, -1);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // a window's gradient is fetched only where the pixel won one of the 4 channels (~40% of the time)
        const bool hit = id[j].x == p || id[j].y == p || id[j].z == p || id[j].w == p;
        gq[j] = hit ? dz[at[j]] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (id[j].x == p) s.x += gq[j].x;
        if (id[j].y == p) s.y += gq[j].y;
        if (id[j].z == p) s.z += gq[j].z;
        if (id[j].w == p) s.w += gq[j].w;
    }
    return s;
}

// kPooled: dy is not read; it is gathered from the pooled gradient dz and the winners idx (see pooled_grad).
template <bool kPooled>
__global__ __launch_bounds__(kRThreads) void ren_bwd_main_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                                 RenGeom g, const float *__restrict__ v,
                                                                 const float *__restrict__ gamma, float cm, float eps,
                                                                 const float *__restrict__ range,
                                                                 const int32_t *__restrict__ argmax,
                                                                 const int32_t *__restrict__ argmin,
                                                                 float *__restrict__ dx, float *__restrict__ parts,
                                                                 float *__restrict__ pabs, float *__restrict__ absmax_out,
                                                                 const float *__restrict__ dz, const int32_t *__restrict__ idx,
                                                                 PoolGeom pg) {
    extern __shared__ float sred[];  // [4][threads*4]
    __shared__ float lds[kRThreads / kWave];
    const int n = blockIdx.y;
    if (absmax_out && blockIdx.x == 0 && n == 0 && threadIdx.x == 0) *absmax_out = 0.0f;  // the second launch max-es into it
    const int qd = threadIdx.x % g.cq, pl = threadIdx.x / g.cq;
    const int p0 = blockIdx.x * g.pix_per_block;
    const int p1 = min(p0 + g.pix_per_block, g.HW);
    float vv[4], gg[4], inv[4];
    int skip_a[4], skip_b[4];  // pixel of this channel's arg-max / arg-min element (or -1)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int c = qd * 4 + e, grp = c / g.m, cc = c % g.m;
        vv[e] = v[c]; gg[e] = gamma[c];
        inv[e] = inv_denominator(range[(size_t)n * g.groups + grp], cm, eps);
        const int ia = argmax[(size_t)n * g.groups + grp], ib = argmin[(size_t)n * g.groups + grp];
        skip_a[e] = (ia % g.m == cc) ? ia / g.m : -1;
        skip_b[e] = (ib % g.m == cc) ? ib / g.m : -1;
    }
    float sb[4] = {0, 0, 0, 0}, sg[4] = {0, 0, 0, 0}, sv[4] = {0, 0, 0, 0}, st[4] = {0, 0, 0, 0};
    const size_t base = (size_t)n * g.HW * g.C;
    const float4 *xv = reinterpret_cast<const float4 *>(x + base);
    const float4 *dv4 = kPooled ? nullptr : reinterpret_cast<const float4 *>(dy + base);
    const size_t pooled_base = kPooled ? (size_t)n * pg.P * pg.Q * g.C : 0;
    const float4 *dz4 = kPooled ? reinterpret_cast<const float4 *>(dz + pooled_base) : nullptr;
    const int4 *idx4 = kPooled ? reinterpret_cast<const int4 *>(idx + pooled_base) : nullptr;
    float4 *ov = reinterpret_cast<float4 *>(dx + base);
    float am = 0.0f;
    const bool active = (int)threadIdx.x < g.threads;
    // pixels in flight per thread: the pooled variant holds 4 winner quads and up to 4 gradient quads per pixel as well
    constexpr int RU = kPooled ? 2 : kRU;
    for (int pb = p0 + pl; pb < p1 && active; pb += RU * g.ppi) {
        float4 a4[RU], d4[RU];
#pragma unroll
        for (int k = 0; k < RU; ++k) {
            const int p = pb + k * g.ppi;
            // the stem's 205 MB input is read here for the last time and was written long ago: a streaming load (measured: the
            // layers whose input the previous kernels just touched lose with it, this one gains 3 %)
            if (kPooled) a4[k] = p < p1 ? load_stream(xv + (size_t)p * g.cq + qd) : make_float4(0.f, 0.f, 0.f, 0.f);
            else a4[k] = p < p1 ? xv[(size_t)p * g.cq + qd] : make_float4(0.f, 0.f, 0.f, 0.f);
            if (kPooled) d4[k] = p < p1 ? pooled_grad(dz4, idx4, p, pg, g.cq, qd) : make_float4(0.f, 0.f, 0.f, 0.f);
            else d4[k] = p < p1 ? dv4[(size_t)p * g.cq + qd] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < RU; ++k) {
            const int p = pb + k * g.ppi;
            if (p >= p1) break;
            const float xe[4] = {a4[k].x, a4[k].y, a4[k].z, a4[k].w};
            const float de[4] = {d4[k].x, d4[k].y, d4[k].z, d4[k].w};
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float z = vv[e] * xe[e];
                const float s = hard_sigmoid(z);
                const float sp = (z > -3.0f && z < 3.0f) ? (1.0f / 6.0f) : 0.0f;
                const float u = xe[e] * s;
                const float du = de[e] * gg[e] * inv[e];
                o[e] = du * (s + xe[e] * vv[e] * sp);
                sb[e] += de[e];
                sg[e] += de[e] * u;
                sv[e] += du * xe[e] * xe[e] * sp;
                st[e] += de[e] * gg[e] * u;
                if (p != skip_a[e] && p != skip_b[e]) am = fmaxf(am, fabsf(o[e]));
            }
            ov[(size_t)p * g.cq + qd] = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
    // fixed-order block reduction over the threads that share a channel quad
    const int T4 = g.threads * 4;
    if (active) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sred[0 * T4 + threadIdx.x * 4 + e] = sb[e];
            sred[1 * T4 + threadIdx.x * 4 + e] = sg[e] * inv[e];
            sred[2 * T4 + threadIdx.x * 4 + e] = sv[e];
            sred[3 * T4 + threadIdx.x * 4 + e] = st[e];
        }
    }
    __syncthreads();
    const size_t row = (size_t)n * g.chunks + blockIdx.x;
    for (int i = threadIdx.x; i < 4 * g.C; i += blockDim.x) {
        const int qn = i / g.C, c = i % g.C;
        float s = 0.0f;
        for (int k = 0; k < g.ppi; ++k) s += sred[qn * T4 + (k * g.cq) * 4 + c];
        parts[(row * 4 + qn) * g.C + c] = s;
    }
    block_absmax_store(am, pabs + row, lds);
}

__global__ __launch_bounds__(kRThreads) void ren_bwd_generic_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                                    int HW, int C, int groups, int m, int pix_per_block,
                                                                    int chunks, const float *__restrict__ v,
                                                                    const float *__restrict__ gamma, float cm, float eps,
                                                                    const float *__restrict__ range,
                                                                    const int32_t *__restrict__ argmax,
                                                                    const int32_t *__restrict__ argmin,
                                                                    float *__restrict__ dx, float *__restrict__ parts,
                                                                    float *__restrict__ pabs, float *__restrict__ absmax_out) {
    // one thread per channel (strided), serial over the block's pixels: slow, any C
    __shared__ float lds[kRThreads / kWave];
    const int n = blockIdx.y;
    if (absmax_out && blockIdx.x == 0 && n == 0 && threadIdx.x == 0) *absmax_out = 0.0f;
    const int p0 = blockIdx.x * pix_per_block, p1 = min(p0 + pix_per_block, HW);
    const size_t row = (size_t)n * chunks + blockIdx.x;
    float am = 0.0f;
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        const int grp = c / m, cc = c % m;
        const float vv = v[c], gg = gamma[c];
        const float inv = inv_denominator(range[(size_t)n * groups + grp], cm, eps);
        const int ia = argmax[(size_t)n * groups + grp], ib = argmin[(size_t)n * groups + grp];
        const int skip_a = (ia % m == cc) ? ia / m : -1, skip_b = (ib % m == cc) ? ib / m : -1;
        float sb = 0, sg = 0, sv = 0, st = 0;
        for (int p = p0; p < p1; ++p) {
            const size_t at = ((size_t)n * HW + p) * C + c;
            const float xe = x[at], de = dy[at];
            const float z = vv * xe, s = hard_sigmoid(z);
            const float sp = (z > -3.0f && z < 3.0f) ? (1.0f / 6.0f) : 0.0f;
            const float u = xe * s, du = de * gg * inv;
            const float o = du * (s + xe * vv * sp);
            dx[at] = o;
            sb += de; sg += de * u; sv += du * xe * xe * sp; st += de * gg * u;
            if (p != skip_a && p != skip_b) am = fmaxf(am, fabsf(o));
        }
        parts[(row * 4 + 0) * C + c] = sb;
        parts[(row * 4 + 1) * C + c] = sg * inv;
        parts[(row * 4 + 2) * C + c] = sv;
        parts[(row * 4 + 3) * C + c] = st;
    }
    block_absmax_store(am, pabs + row, lds);
}

// Second backward launch, blocks of kFinishThreads threads.  Blocks [0, 3 ceil(C/8)): dbeta, dgamma, dv = column sums of
// parts over all rows in a fixed order (one quantity, 8 channels x 32 row lanes per block: the first 256 threads; the
// others only meet the barrier).  The remaining blocks take 16 (sample, group) pairs each, one per wave: the gradient
// through the range, added at the saved extrema; they also fold max|dx| = max(block partials of the first launch, the
// elements just changed) into absmax_out, which the first launch zeroed (a max is order-free, so this stays
// deterministic).  16 pairs per block, not 4: every block ends with an atomic on that one address, those are served one
// after the other (~10 ns each), and with 512 of them they were half of this kernel's 8 us.
constexpr int kFinishThreads = 1024;
constexpr int kFinishPairs = kFinishThreads / kWave;
__global__ __launch_bounds__(kFinishThreads) void ren_bwd_finish_kernel(const float *__restrict__ parts, const float *__restrict__ pabs,
                                                                        int rows, int N, int HW, int C, int groups, int m, int chunks,
                                                                        float cm, float eps, const float *__restrict__ range,
                                                                        const int32_t *__restrict__ argmax, const int32_t *__restrict__ argmin,
                                                                        float *__restrict__ dx, float *__restrict__ dbeta,
                                                                        float *__restrict__ dgamma, float *__restrict__ dv,
                                                                        float *__restrict__ absmax_out) {
    __shared__ float s[32][8];
    __shared__ float lds[kFinishPairs];
    const int param_blocks = 3 * ((C + 7) / 8);
    if ((int)blockIdx.x < param_blocks) {
        // one of the three quantities, 8 channels x 32 row lanes; a lane's rows are summed eight at a time (8 loads in
        // flight) in a fixed order
        const bool worker = threadIdx.x < 256;
        const int q = blockIdx.x % 3, cl = threadIdx.x % 8, sl = (threadIdx.x / 8) % 32;
        const int c = (blockIdx.x / 3) * 8 + cl;
        float acc = 0.0f;
        if (worker && c < C) {
            for (int r = sl; r < rows; r += 256) {
                float t[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) t[k] = r + 32 * k < rows ? parts[((size_t)(r + 32 * k) * 4 + q) * C + c] : 0.0f;
                acc += ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
            }
        }
        if (worker) s[sl][cl] = acc;
        __syncthreads();
        if (worker && sl == 0 && c < C) {
            float t = 0;
            for (int k = 0; k < 32; ++k) t += s[k][cl];
            (q == 0 ? dbeta : q == 1 ? dgamma : dv)[c] = t;
        }
        return;
    }
    // range blocks: one wave per (sample, group) pair; its lanes share the pair's chunks x channels partial sums
    const int rb = blockIdx.x - param_blocks, nrb = gridDim.x - param_blocks;
    float am = 0.0f;
    const int i = rb * kFinishPairs + threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (i < N * groups) {
        const int n = i / groups, grp = i % groups;
        // the two elements to change are fetched while the partial sums are still being added up
        // (positions outside the slab -- not what the forward pass saved -- are taken as its first element: nothing is
        // read or written out of bounds)
        const int lim = HW * m;
        const int ia = (unsigned)argmax[i] < (unsigned)lim ? argmax[i] : 0, ib = (unsigned)argmin[i] < (unsigned)lim ? argmin[i] : 0;
        const size_t base = (size_t)n * HW * C + (size_t)grp * m;
        const size_t pa = base + (size_t)(ia / m) * C + ia % m, pb = base + (size_t)(ib / m) * C + ib % m;
        const float da = dx[pa], db = dx[pb];
        const float inv = inv_denominator(range[i], cm, eps);
        float t = 0.0f;
        for (int k0 = lane; k0 < chunks * m; k0 += 4 * kWave) {
            float q[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = k0 + j * kWave, ch = k / m, cc = k - ch * m;
                q[j] = k < chunks * m ? parts[(((size_t)n * chunks + ch) * 4 + 3) * C + grp * m + cc] : 0.0f;
            }
            t += (q[0] + q[1]) + (q[2] + q[3]);
        }
        t = wave_sum(t);
        if (lane == 0) {
            const float dR = -cm * t * inv * inv;
            if (pa != pb) {
                const float na = da + dR, nb = db - dR;
                dx[pa] = na;
                dx[pb] = nb;
                am = fmaxf(fabsf(na), fabsf(nb));
            } else {  // a constant slab: both extrema are its first element
                const float na = (da + dR) - dR;
                dx[pa] = na;
                am = fabsf(na);
            }
        }
    }
    if (absmax_out) {
        for (int r = rb * kFinishThreads + threadIdx.x; r < rows; r += nrb * kFinishThreads) am = fmaxf(am, pabs[r]);
        block_absmax_commit(am, absmax_out, lds);
    }
}

static int check_ren(const void *x, int N, int H, int W, int C, int groups) {
    LPDT_REQUIRE(x, LPDT_EINVAL, "range_evonorm: NULL tensor");
    LPDT_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0, LPDT_EINVAL, "range_evonorm: sizes must be positive");
    LPDT_REQUIRE(groups > 0 && C % groups == 0, LPDT_EUNSUPPORTED, "range_evonorm: groups (%d) must divide C (%d)", groups, C);
    LPDT_REQUIRE(C / groups >= 2, LPDT_EUNSUPPORTED,
                 "range_evonorm: needs at least 2 channels per group (C(1) = 1/sqrt(2 ln 1) is infinite)");
    LPDT_REQUIRE(groups <= 2048, LPDT_EUNSUPPORTED, "range_evonorm: at most 2048 groups");
    LPDT_REQUIRE((long long)H * W * (C / groups) < 0x7fffffffLL && (long long)N * H * W * C < (1LL << 40), LPDT_EUNSUPPORTED,
                 "range_evonorm: slab too large");
    return LPDT_OK;
}
static bool ren_fast(int C) { return C % 4 == 0 && C / 4 <= kRThreads; }
// floor(x / d) == umulhi(x, 2^32/d + 1) for every 0 <= x <= xmax when xmax * d < 2^32 (the error term x / 2^32 stays
// below 1/d); 0 asks for a plain division
static unsigned pool_mul(int d, long long xmax) {
    if (d <= 1 || xmax * d >= (1ll << 32)) return 0u;
    return (unsigned)((1ull << 32) / (unsigned)d + 1);
}
static PoolGeom pool_geom(int H, int W, int P, int Q, int k, int st, int pd) {
    PoolGeom pg;
    pg.W = W; pg.P = P; pg.Q = Q; pg.k = k; pg.st = st; pg.pd = pd;
    pg.mul_w = pool_mul(W, (long long)H * W);
    pg.mul_q = pool_mul(Q, (long long)P * Q);
    pg.mul_st = pool_mul(st, (long long)(H > W ? H : W) + pd + st);
    return pg;
}
static float ren_cm(int m) { return (float)(1.0 / std::sqrt(2.0 * std::log((double)m))); }
constexpr int kGenericElems = 8192;
constexpr int kGenericPix = 64;


// ---- the normalisation behind a convolution that took its statistics (see qconv_internal.h) ----
bool ren_chain_supported(int C, int groups) { return groups > 0 && C % groups == 0 && C / groups >= 2 && C % 4 == 0 && C / 4 <= kRThreads; }
size_t ren_chain_ws_bytes(int N, int C, int groups) {
    return round_up((size_t)N * C * 4 * sizeof(unsigned), 256) + round_up((size_t)N * groups * 2 * sizeof(float), 256) + 256;
}
static float ren_cm_of(int m) { return (float)(1.0 / std::sqrt(2.0 * std::log((double)m))); }
unsigned *ren_chain_begin(int N, int C, int groups, void *ws, hipStream_t st) {
    unsigned *cstats = static_cast<unsigned *>(ws);
    float *absmax = reinterpret_cast<float *>(static_cast<char *>(ws) + ren_chain_ws_bytes(N, C, groups) - 256);
    const size_t count = (size_t)N * C * 4;
    hipLaunchKernelGGL(ren_cstats_clear_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, cstats, count, absmax);
    return cstats;
}
void ren_chain_finish(const float *x, int N, int H, int W, int C, int groups, const float *v, const float *gamma, const float *beta,
                      float eps, int8_t *q, float *scale, float *z, float *range_out, int32_t *argmax_out, int32_t *argmin_out,
                      void *ws, hipStream_t st) {
    const unsigned *cstats = static_cast<const unsigned *>(ws);
    float *gext = reinterpret_cast<float *>(static_cast<char *>(ws) + round_up((size_t)N * C * 4 * sizeof(unsigned), 256));
    float *absmax = reinterpret_cast<float *>(static_cast<char *>(ws) + ren_chain_ws_bytes(N, C, groups) - 256);
    const float cm = ren_cm_of(C / groups);
    const RenGeom ga = ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kApplyElems));
    hipLaunchKernelGGL(ren_cfold_kernel, dim3(N), dim3(256), (size_t)2 * groups * sizeof(unsigned) + groups * sizeof(float), st, ga, cstats,
                       gamma, beta, cm, eps, range_out, gext, argmax_out, argmin_out, absmax);
    hipLaunchKernelGGL(ren_apply_q_kernel, dim3(ga.chunks, N), dim3(ga.block), 0, st, x, ga, v, gamma, beta, cm, eps, range_out, absmax, 1, q,
                       scale, z, gext, argmax_out, argmin_out);
}

}  // namespace lpdt

using namespace lpdt;

static size_t ren_rows(int N, int H, int W, int C, int groups) {
    if (ren_fast(C)) return (size_t)N * ren_geom(N, H, W, C, groups, kBwdMinPix, block_cap(N, H, W, C, kBwdElems)).chunks;
    return (size_t)N * (((size_t)H * W + kGenericPix - 1) / kGenericPix);
}

extern "C" size_t lpdt_range_evonorm_fwd_workspace_bytes(int N, int H, int W, int C, int groups) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || groups <= 0 || C % groups) return 0;
    const size_t blocks = ren_fast(C) ? (size_t)N * ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kStatsElems)).chunks : (size_t)N;
    return round_up(blocks * groups * 2 * sizeof(unsigned long long), 256);
}

// Samples small enough for the one-block-per-sample statistics (ren_sample_kernel); the keys' room (at least 256 bytes
// per sample: 2 keys per group and block) also holds its N floats.
static bool ren_sample_path(int N, int H, int W, int C) {
    long long limit = 64 * 1024;
#ifdef LPDT_TUNE
    if (const char *e = getenv("LPDT_REN_SAMPLE_ELEMS")) limit = atoll(e);
#endif
    return (long long)H * W * C <= limit && C / 4 <= kSampleThreads && N <= 256;   // every apply thread reads the N maxima
}

// int8-output forward: block keys, then the per-block channel extremes of u, then the scalar max|y|
static size_t ren_q_key_bytes(const RenGeom &g) { return round_up((size_t)g.N * g.chunks * g.groups * 2 * sizeof(unsigned long long), 256); }
static size_t ren_q_u_bytes(const RenGeom &g) { return round_up((size_t)g.N * g.chunks * g.C * 2 * sizeof(float), 256); }

extern "C" size_t lpdt_range_evonorm_fwd_q_workspace_bytes(int N, int H, int W, int C, int groups) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || groups <= 0 || C % groups || !ren_fast(C)) return 0;
    const RenGeom g = ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kStatsElems));
    return ren_q_key_bytes(g) + ren_q_u_bytes(g) + 256;
}

extern "C" int lpdt_range_evonorm_fwd_q(const float *x, int N, int H, int W, int C, int groups, const float *v,
                                        const float *gamma, const float *beta, float eps, int8_t *q, float *scale, float *y,
                                        float *range_out, int32_t *argmax_out, int32_t *argmin_out, void *ws, size_t ws_bytes,
                                        void *stream) {
    int rc = check_ren(x, N, H, W, C, groups);
    if (rc) return rc;
    LPDT_REQUIRE(v && gamma && beta && q && scale && range_out && argmax_out && argmin_out, LPDT_EINVAL,
                 "range_evonorm_fwd_q: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "range_evonorm_fwd_q: eps must be >= 0");
    LPDT_REQUIRE(ren_fast(C), LPDT_EUNSUPPORTED, "range_evonorm_fwd_q: C must be a multiple of 4, at most %d (got %d)", 4 * kRThreads, C);
    LPDT_REQUIRE(aligned(x, 16) && aligned(q, 4) && aligned(scale, 4) && aligned(y, 16), LPDT_EINVAL,
                 "range_evonorm_fwd_q: x and y must be 16-byte aligned, q and scale 4-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_range_evonorm_fwd_q_workspace_bytes(N, H, W, C, groups));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const float cm = ren_cm(C / groups);
    const RenGeom g = ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kStatsElems));
    const RenGeom ga = ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kApplyElems));
    unsigned long long *keys = static_cast<unsigned long long *>(ws);
    float *pu = reinterpret_cast<float *>(static_cast<char *>(ws) + ren_q_key_bytes(g));
    float *absmax = reinterpret_cast<float *>(static_cast<char *>(ws) + ren_q_key_bytes(g) + ren_q_u_bytes(g));
    const size_t key_lds = (size_t)2 * groups * sizeof(unsigned long long);
    const size_t fold_lds = key_lds + groups * sizeof(float) + (size_t)2 * C * sizeof(unsigned int);
    if (ren_sample_path(N, H, W, C)) {
        float *sample_abs = static_cast<float *>(ws);     // [N]: fits the room of the block keys it replaces
        hipLaunchKernelGGL(ren_sample_kernel, dim3(N), dim3(kSampleThreads), fold_lds, st, x, H * W, C, groups, C / groups, v, gamma, beta,
                           cm, eps, range_out, argmax_out, argmin_out, sample_abs);
        hipLaunchKernelGGL(ren_apply_q_kernel, dim3(ga.chunks, N), dim3(ga.block), 0, st, x, ga, v, gamma, beta, cm, eps, range_out,
                           sample_abs, N, q, scale, y, nullptr, nullptr, nullptr);
        return launch_status("lpdt_range_evonorm_fwd_q");
    }
    hipLaunchKernelGGL(ren_stats_kernel<true>, dim3(g.chunks, N), dim3(g.block), key_lds + (size_t)2 * C * sizeof(unsigned int), st, x, g,
                       keys, absmax, v, pu);
    hipLaunchKernelGGL(ren_q_fold_kernel, dim3(N), dim3(256), fold_lds, st, g, keys, pu, gamma, beta, cm, eps,
                       range_out, argmax_out, argmin_out, absmax);
    hipLaunchKernelGGL(ren_apply_q_kernel, dim3(ga.chunks, N), dim3(ga.block), 0, st, x, ga, v, gamma, beta, cm, eps, range_out,
                       absmax, 1, q, scale, y, nullptr, nullptr, nullptr);
    return launch_status("lpdt_range_evonorm_fwd_q");
}

extern "C" size_t lpdt_range_evonorm_bwd_workspace_bytes(int N, int H, int W, int C, int groups) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || groups <= 0 || C % groups) return 0;
    const size_t rows = ren_rows(N, H, W, C, groups);
    return round_up(rows * 4 * C * sizeof(float), 256) + round_up(rows * sizeof(float), 256);
}

extern "C" int lpdt_range_evonorm_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v,
                                      const float *gamma, const float *beta, float eps, float *y, float *range_out,
                                      int32_t *argmax_out, int32_t *argmin_out, float *absmax_out, void *ws,
                                      size_t ws_bytes, void *stream) {
    int rc = check_ren(x, N, H, W, C, groups);
    if (rc) return rc;
    LPDT_REQUIRE(v && gamma && beta && y && range_out && argmax_out && argmin_out, LPDT_EINVAL,
                 "range_evonorm_fwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "range_evonorm_fwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(y, 16), LPDT_EINVAL, "range_evonorm_fwd: x and y must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_range_evonorm_fwd_workspace_bytes(N, H, W, C, groups));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    unsigned long long *stats = static_cast<unsigned long long *>(ws);
    const int count = N * groups, m = C / groups;
    const float cm = ren_cm(m);
    const size_t smem = (size_t)2 * groups * sizeof(unsigned long long);
    if (ren_fast(C)) {
        const RenGeom g = ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kStatsElems));
        hipLaunchKernelGGL(ren_stats_kernel<false>, dim3(g.chunks, N), dim3(g.block), smem, st, x, g, stats, absmax_out,
                           (const float *)nullptr, (float *)nullptr);
        const RenGeom ga = ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kApplyElems));
        hipLaunchKernelGGL(ren_apply_kernel, dim3(ga.chunks, N), dim3(ga.block), smem + groups * sizeof(float), st, x, ga, v, gamma,
                           beta, cm, eps, stats, g.chunks, y, range_out, argmax_out, argmin_out, absmax_out);
    } else {
        hipLaunchKernelGGL(ren_clear_kernel, dim3((2 * count + 255) / 256), dim3(256), 0, st, stats, 2 * count, absmax_out);
        const long long total = (long long)H * W * C;
        const int blocks = (int)((total + kGenericElems - 1) / kGenericElems);
        hipLaunchKernelGGL(ren_stats_generic_kernel, dim3(blocks, N), dim3(kRThreads), smem, st, x, H * W, C, groups, m,
                           kGenericElems, stats);
        hipLaunchKernelGGL(ren_finalize_kernel, dim3((count + 255) / 256), dim3(256), 0, st, stats, count, range_out,
                           argmax_out, argmin_out);
        hipLaunchKernelGGL(ren_apply_generic_kernel, dim3(blocks, N), dim3(kRThreads), 0, st, x, H * W, C, groups, m,
                           kGenericElems, v, gamma, beta, cm, eps, range_out, y, absmax_out);
    }
    return launch_status("lpdt_range_evonorm_fwd");
}

static int check_ren_pool(const char *what, int N, int H, int W, int C, int groups, int k, int st, int pd) {
    LPDT_REQUIRE(ren_fast(C), LPDT_EUNSUPPORTED, "%s: C must be a multiple of 4, at most %d (got %d)", what, 4 * kRThreads, C);
    LPDT_REQUIRE(k > 0 && st > 0 && pd >= 0 && pd < k, LPDT_EINVAL, "%s: need k > 0, stride > 0, 0 <= pad < k", what);
    LPDT_REQUIRE(H + 2 * pd >= k && W + 2 * pd >= k, LPDT_EINVAL, "%s: window larger than the padded map", what);
    LPDT_REQUIRE((size_t)N * H * W * C < ((size_t)1 << 31), LPDT_EUNSUPPORTED, "%s: tensor too large", what);
    (void)groups;
    return LPDT_OK;
}

extern "C" size_t lpdt_range_evonorm_maxpool_fwd_workspace_bytes(int N, int H, int W, int C, int groups) {
    return ren_fast(C) ? lpdt_range_evonorm_fwd_workspace_bytes(N, H, W, C, groups) : 0;
}
// The backward pass that gathers its gradient from a pooled map does more per pixel than the plain one and holds fewer
// pixels in flight: its grid may grow to twice the other streaming passes' (measured on ResNet-18's 64 x 112 x 112 x 64
// stem: at most 1024 blocks 162 us, 2048 171 us, 4096 149 us, 8192 176 us).
constexpr int kPooledBwdMaxBlocks = 4096;
static RenGeom pooled_bwd_geom(int N, int H, int W, int C, int groups) {
    const long long b = (long long)N * H * W * C / kBwdElems;
    return ren_geom(N, H, W, C, groups, kBwdMinPix, (int)(b < 256 ? 256 : b > kPooledBwdMaxBlocks ? kPooledBwdMaxBlocks : b));
}
extern "C" size_t lpdt_range_evonorm_maxpool_bwd_workspace_bytes(int N, int H, int W, int C, int groups) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || groups <= 0 || C % groups || !ren_fast(C)) return 0;
    const size_t rows = (size_t)N * pooled_bwd_geom(N, H, W, C, groups).chunks;
    return round_up(rows * 4 * C * sizeof(float), 256) + round_up(rows * sizeof(float), 256);
}

extern "C" int lpdt_range_evonorm_maxpool_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v,
                                              const float *gamma, const float *beta, float eps, int k, int st_, int pd, float *z,
                                              int32_t *idx, float *range_out, int32_t *argmax_out, int32_t *argmin_out,
                                              float *absmax_out, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_ren(x, N, H, W, C, groups);
    if (rc) return rc;
    rc = check_ren_pool("range_evonorm_maxpool_fwd", N, H, W, C, groups, k, st_, pd);
    if (rc) return rc;
    LPDT_REQUIRE(v && gamma && beta && z && idx && range_out && argmax_out && argmin_out, LPDT_EINVAL,
                 "range_evonorm_maxpool_fwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "range_evonorm_maxpool_fwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(z, 16) && aligned(idx, 16), LPDT_EINVAL,
                 "range_evonorm_maxpool_fwd: x, z and idx must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_range_evonorm_maxpool_fwd_workspace_bytes(N, H, W, C, groups));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const int P = conv_out(H, pd, k, st_), Q = conv_out(W, pd, k, st_);
    const RenGeom g = ren_geom(N, H, W, C, groups, 0, block_cap(N, H, W, C, kStatsElems));
    const RenGeom gp = ren_geom(N, P, Q, C, groups, 0, block_cap(N, P, Q, C, kApplyElems / 4));
    unsigned long long *stats = static_cast<unsigned long long *>(ws);
    const size_t smem = (size_t)2 * groups * sizeof(unsigned long long);
    hipLaunchKernelGGL(ren_stats_kernel<false>, dim3(g.chunks, N), dim3(g.block), smem, st, x, g, stats, absmax_out,
                       (const float *)nullptr, (float *)nullptr);
    hipLaunchKernelGGL(ren_pool_kernel, dim3(gp.chunks, N), dim3(gp.block), smem + groups * sizeof(float), st, x, gp, H, W,
                       pool_geom(H, W, P, Q, k, st_, pd), v, gamma, beta, ren_cm(C / groups), eps, stats, g.chunks, z, idx, range_out,
                       argmax_out, argmin_out, absmax_out);
    return launch_status("lpdt_range_evonorm_maxpool_fwd");
}

extern "C" int lpdt_range_evonorm_maxpool_bwd(const float *dz, const int32_t *idx, const float *x, int N, int H, int W, int C,
                                              int groups, const float *v, const float *gamma, float eps, int k, int st_, int pd,
                                              const float *range, const int32_t *argmax, const int32_t *argmin, float *dx,
                                              float *dv, float *dgamma, float *dbeta, float *absmax_out, void *ws, size_t ws_bytes,
                                              void *stream) {
    int rc = check_ren(x, N, H, W, C, groups);
    if (rc) return rc;
    rc = check_ren_pool("range_evonorm_maxpool_bwd", N, H, W, C, groups, k, st_, pd);
    if (rc) return rc;
    LPDT_REQUIRE((k + st_ - 1) / st_ <= 2, LPDT_EUNSUPPORTED,
                 "range_evonorm_maxpool_bwd: a pixel may lie in at most 2 x 2 windows (k <= 2 * stride)");
    LPDT_REQUIRE(dz && idx && v && gamma && range && argmax && argmin && dx && dv && dgamma && dbeta, LPDT_EINVAL,
                 "range_evonorm_maxpool_bwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "range_evonorm_maxpool_bwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(dz, 16) && aligned(idx, 16) && aligned(dx, 16), LPDT_EINVAL,
                 "range_evonorm_maxpool_bwd: x, dz, idx and dx must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_range_evonorm_maxpool_bwd_workspace_bytes(N, H, W, C, groups));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const int m = C / groups, P = conv_out(H, pd, k, st_), Q = conv_out(W, pd, k, st_);
    const float cm = ren_cm(m);
    const RenGeom g = pooled_bwd_geom(N, H, W, C, groups);
    const size_t rows = (size_t)N * g.chunks;
    float *parts = static_cast<float *>(ws);
    float *pabs = reinterpret_cast<float *>(static_cast<char *>(ws) + round_up(rows * 4 * C * sizeof(float), 256));
    hipLaunchKernelGGL(ren_bwd_main_kernel<true>, dim3(g.chunks, N), dim3(g.block), (size_t)16 * g.threads * sizeof(float), st,
                       (const float *)nullptr, x, g, v, gamma, cm, eps, range, argmax, argmin, dx, parts, pabs, absmax_out, dz, idx,
                       pool_geom(H, W, P, Q, k, st_, pd));
    hipLaunchKernelGGL(ren_bwd_finish_kernel, dim3(3 * ((C + 7) / 8) + (N * groups + kFinishPairs - 1) / kFinishPairs), dim3(kFinishThreads), 0, st, parts, pabs, (int)rows, N, H * W, C,
                       groups, m, g.chunks, cm, eps, range, argmax, argmin, dx, dbeta, dgamma, dv, absmax_out);
    return launch_status("lpdt_range_evonorm_maxpool_bwd");
}

extern "C" int lpdt_range_evonorm_bwd(const float *dy, const float *x, int N, int H, int W, int C, int groups,
                                      const float *v, const float *gamma, float eps, const float *range,
                                      const int32_t *argmax, const int32_t *argmin, float *dx, float *dv, float *dgamma,
                                      float *dbeta, float *absmax_out, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_ren(x, N, H, W, C, groups);
    if (rc) return rc;
    LPDT_REQUIRE(dy && v && gamma && range && argmax && argmin && dx && dv && dgamma && dbeta, LPDT_EINVAL,
                 "range_evonorm_bwd: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "range_evonorm_bwd: eps must be >= 0");
    LPDT_REQUIRE(aligned(x, 16) && aligned(dy, 16) && aligned(dx, 16), LPDT_EINVAL,
                 "range_evonorm_bwd: x, dy and dx must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_range_evonorm_bwd_workspace_bytes(N, H, W, C, groups));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const int m = C / groups;
    const float cm = ren_cm(m);
    const size_t rows = ren_rows(N, H, W, C, groups);
    float *parts = static_cast<float *>(ws);
    float *pabs = reinterpret_cast<float *>(static_cast<char *>(ws) + round_up(rows * 4 * C * sizeof(float), 256));
    int chunks;
    if (ren_fast(C)) {
        const RenGeom g = ren_geom(N, H, W, C, groups, kBwdMinPix, block_cap(N, H, W, C, kBwdElems));
        chunks = g.chunks;
        const size_t smem = (size_t)16 * g.threads * sizeof(float);
        hipLaunchKernelGGL(ren_bwd_main_kernel<false>, dim3(g.chunks, N), dim3(g.block), smem, st, dy, x, g, v, gamma, cm, eps,
                           range, argmax, argmin, dx, parts, pabs, absmax_out, (const float *)nullptr, (const int32_t *)nullptr,
                           PoolGeom{});
    } else {
        chunks = (H * W + kGenericPix - 1) / kGenericPix;
        hipLaunchKernelGGL(ren_bwd_generic_kernel, dim3(chunks, N), dim3(kRThreads), 0, st, dy, x, H * W, C, groups, m,
                           kGenericPix, chunks, v, gamma, cm, eps, range, argmax, argmin, dx, parts, pabs, absmax_out);
    }
    hipLaunchKernelGGL(ren_bwd_finish_kernel, dim3(3 * ((C + 7) / 8) + (N * groups + kFinishPairs - 1) / kFinishPairs), dim3(kFinishThreads), 0, st, parts, pabs, (int)rows, N, H * W, C,
                       groups, m, chunks, cm, eps, range, argmax, argmin, dx, dbeta, dgamma, dv, absmax_out);
    return launch_status("lpdt_range_evonorm_bwd");
}
