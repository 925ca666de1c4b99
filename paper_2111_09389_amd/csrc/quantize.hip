// 8-bit symmetric per-tensor quantizer with round-to-nearest-even or Philox
// stochastic rounding, and the dequantizing scale of int32 accumulators
// (Section 3, "Low Precision Training").  HBM-bound kernels: 16-byte loads,
// 4-byte packed code stores, no atomics (abs-max goes through per-block
// partials that every block of the rounding pass re-reduces from L2).
#include "qconv_internal.h"
#include <mutex>

namespace lpdt {

constexpr int kQThreads = 256;
constexpr int kMaxParts = 1024;  // abs-max partials = upper bound of the first pass's grid

// ---- Philox4x32-10 (Salmon et al., SC'11) ----------------------------------
// One call yields the four 32-bit words used by four consecutive elements.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1, uint32_t out[4]) {
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint64_t lo = (uint64_t)c0 * 0xD2511F53ull;
        const uint64_t hi = (uint64_t)c2 * 0xCD9E8D57ull;
        const uint32_t t0 = (uint32_t)(hi >> 32) ^ c1 ^ k0;
        const uint32_t t2 = (uint32_t)(lo >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)hi;
        c3 = (uint32_t)lo;
        c0 = t0;
        c2 = t2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ float block_max(float v, float *lds) {
    v = wave_max(v);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    float r = lds[0];
#pragma unroll
    for (int w = 1; w < kQThreads / kWave; ++w) r = fmaxf(r, lds[w]);
    __syncthreads();
    return r;
}

__global__ __launch_bounds__(kQThreads) void absmax_kernel(const float *__restrict__ x, size_t len,
                                                           float *__restrict__ parts) {
    __shared__ float lds[kQThreads / kWave];
    const size_t nvec = len / 4;
    const float4 *xv = reinterpret_cast<const float4 *>(x);
    float m = 0.0f;
    for (size_t i = (size_t)blockIdx.x * kQThreads + threadIdx.x; i < nvec; i += (size_t)gridDim.x * kQThreads) {
        const float4 a = xv[i];
        m = fmaxf(fmaxf(m, fmaxf(fabsf(a.x), fabsf(a.y))), fmaxf(fabsf(a.z), fabsf(a.w)));
    }
    if (blockIdx.x == 0 && threadIdx.x < (len & 3)) m = fmaxf(m, fabsf(x[nvec * 4 + threadIdx.x]));
    m = block_max(m, lds);
    if (threadIdx.x == 0) parts[blockIdx.x] = m;
}

template <bool kStochastic>
__global__ __launch_bounds__(kQThreads) void round_kernel(const float *__restrict__ x, size_t len,
                                                          const float *__restrict__ parts, int nparts,
                                                          uint64_t seed, uint64_t offset, int8_t *__restrict__ q,
                                                          float *__restrict__ scale) {
    __shared__ float lds[kQThreads / kWave];
    float a = 0.0f;
    for (int i = threadIdx.x; i < nparts; i += kQThreads) a = fmaxf(a, parts[i]);
    a = block_max(a, lds);
    const float inv = quant_inv(a);
    if (blockIdx.x == 0 && threadIdx.x == 0) *scale = quant_scale(a);

    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const size_t nvec = len / 4;
    const float4 *xv = reinterpret_cast<const float4 *>(x);
    uint32_t *qv = reinterpret_cast<uint32_t *>(q);
    for (size_t i = (size_t)blockIdx.x * kQThreads + threadIdx.x; i < nvec; i += (size_t)gridDim.x * kQThreads) {
        const float4 v = xv[i];
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (kStochastic) {
            const uint64_t blk = offset + i;
            philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), k0, k1, w);
        }
        const uint32_t b0 = (uint32_t)round_code(v.x, inv, kStochastic, w[0]) & 0xffu;
        const uint32_t b1 = (uint32_t)round_code(v.y, inv, kStochastic, w[1]) & 0xffu;
        const uint32_t b2 = (uint32_t)round_code(v.z, inv, kStochastic, w[2]) & 0xffu;
        const uint32_t b3 = (uint32_t)round_code(v.w, inv, kStochastic, w[3]) & 0xffu;
        qv[i] = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
    }
    const int tail = (int)(len & 3);
    if (blockIdx.x == 0 && threadIdx.x < tail) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (kStochastic) {
            const uint64_t blk = offset + nvec;
            philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), k0, k1, w);
        }
        q[nvec * 4 + threadIdx.x] = (int8_t)round_code(x[nvec * 4 + threadIdx.x], inv, kStochastic, w[threadIdx.x]);
    }
}

// Small tensors (a classifier's input, the loss gradient): one block finds the abs-max and emits the codes, one launch
// instead of two -- at this size a launch costs more than the work.  Same arithmetic as absmax_kernel + round_kernel.
constexpr int kSmallThreads = 1024, kSmallVecs = 16;                  // up to 16 float4 per thread: 64 Ki elements
constexpr size_t kSmallLen = (size_t)kSmallThreads * kSmallVecs * 4;
template <bool kStochastic>
__global__ __launch_bounds__(kSmallThreads) void quantize_small_kernel(const float *__restrict__ x, size_t len, uint64_t seed,
                                                                       uint64_t offset, int8_t *__restrict__ q,
                                                                       float *__restrict__ scale) {
    __shared__ float lds[kSmallThreads / kWave];
    const size_t nvec = len / 4;
    const int tail = (int)(len & 3);
    const float4 *xv = reinterpret_cast<const float4 *>(x);
    float4 v[kSmallVecs];
    float m = 0.0f;
#pragma unroll
    for (int k = 0; k < kSmallVecs; ++k) {
        const size_t i = threadIdx.x + (size_t)kSmallThreads * k;
        v[k] = i < nvec ? xv[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        m = fmaxf(fmaxf(m, fmaxf(fabsf(v[k].x), fabsf(v[k].y))), fmaxf(fabsf(v[k].z), fabsf(v[k].w)));
    }
    const float t = (int)threadIdx.x < tail ? x[nvec * 4 + threadIdx.x] : 0.0f;
    m = wave_max(fmaxf(m, fabsf(t)));
    if (threadIdx.x % kWave == 0) lds[threadIdx.x / kWave] = m;
    __syncthreads();
    float a = lds[0];
#pragma unroll
    for (int w = 1; w < kSmallThreads / kWave; ++w) a = fmaxf(a, lds[w]);
    const float inv = quant_inv(a);
    if (threadIdx.x == 0) *scale = quant_scale(a);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t *qv = reinterpret_cast<uint32_t *>(q);
#pragma unroll
    for (int k = 0; k < kSmallVecs; ++k) {
        const size_t i = threadIdx.x + (size_t)kSmallThreads * k;
        if (i >= nvec) break;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (kStochastic) {
            const uint64_t blk = offset + i;
            philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), k0, k1, w);
        }
        const uint32_t b0 = (uint32_t)round_code(v[k].x, inv, kStochastic, w[0]) & 0xffu;
        const uint32_t b1 = (uint32_t)round_code(v[k].y, inv, kStochastic, w[1]) & 0xffu;
        const uint32_t b2 = (uint32_t)round_code(v[k].z, inv, kStochastic, w[2]) & 0xffu;
        const uint32_t b3 = (uint32_t)round_code(v[k].w, inv, kStochastic, w[3]) & 0xffu;
        qv[i] = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
    }
    if ((int)threadIdx.x < tail) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (kStochastic) {
            const uint64_t blk = offset + nvec;
            philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), k0, k1, w);
        }
        q[nvec * 4 + threadIdx.x] = (int8_t)round_code(t, inv, kStochastic, w[threadIdx.x]);
    }
}

// ---- many slices of one buffer in two launches --------------------------------
// Slice table in device memory: begin[s], end[s] (element indices), written from kernel arguments so that the call
// needs no host-to-device copy and can be captured in a graph.
constexpr int kSegChunk = 128;
constexpr int kSegTile = kQThreads * 64;  // elements per block: few blocks (and few atomics) per slice, 16 quads per thread
struct SegChunk { long long v[2 * kSegChunk]; };

__global__ void seg_upload_kernel(SegChunk c, long long *table, unsigned int *amax, int first, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 2 * count) table[2 * first + i] = c.v[i];
    if (i < count) amax[first + i] = 0u;
}

// grid (tiles of the longest slice, slices); |x| >= 0, so its maximum is also the maximum of the bit patterns
__global__ __launch_bounds__(kQThreads) void seg_absmax_kernel(const float *__restrict__ x, const long long *__restrict__ table,
                                                               unsigned int *__restrict__ amax) {
    __shared__ float lds[kQThreads / kWave];
    const long long begin = table[2 * blockIdx.y], len = table[2 * blockIdx.y + 1] - begin;
    const long long t0 = (long long)blockIdx.x * kSegTile;
    if (t0 >= len) return;
    const long long t1 = min(t0 + (long long)kSegTile, len);
    const float *xs = x + begin;
    float m = 0.0f;
    if (((begin & 3) == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0)) {
        const long long v1 = t1 / 4;
        // four loads are issued before the first is used
        for (long long i0 = t0 / 4 + threadIdx.x; i0 < v1; i0 += 4 * kQThreads) {
            float4 a[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const long long i = i0 + (long long)k * kQThreads;
                a[k] = i < v1 ? reinterpret_cast<const float4 *>(xs)[i] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) m = fmaxf(fmaxf(m, fmaxf(fabsf(a[k].x), fabsf(a[k].y))), fmaxf(fabsf(a[k].z), fabsf(a[k].w)));
        }
        for (long long i = v1 * 4 + threadIdx.x; i < t1; i += kQThreads) m = fmaxf(m, fabsf(xs[i]));
    } else {
        for (long long i = t0 + threadIdx.x; i < t1; i += kQThreads) m = fmaxf(m, fabsf(xs[i]));
    }
    m = block_max(m, lds);
    if (threadIdx.x == 0) atomicMax(&amax[blockIdx.y], __float_as_uint(m));
}

template <bool kStochastic>
__global__ __launch_bounds__(kQThreads) void seg_round_kernel(const float *__restrict__ x, const long long *__restrict__ table,
                                                              const unsigned int *__restrict__ amax, uint64_t seed,
                                                              uint64_t offset, int8_t *__restrict__ q,
                                                              float *__restrict__ scales) {
    const int s = blockIdx.y;
    const long long begin = table[2 * s], len = table[2 * s + 1] - begin;
    const float a = __uint_as_float(amax[s]);
    if (blockIdx.x == 0 && threadIdx.x == 0) scales[s] = quant_scale(a);
    const long long t0 = (long long)blockIdx.x * kSegTile;
    if (t0 >= len) return;
    const long long t1 = min(t0 + (long long)kSegTile, len);
    const float inv = quant_inv(a);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const uint64_t base = offset + ((uint64_t)s << 24);  // slice s has its own counter range
    const float *xs = x + begin;
    int8_t *qs = q + begin;
    const bool vec = ((begin & 3) == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(q) & 3) == 0);
    long long done = t0;
    if (vec) {
        const long long v1 = t1 / 4;
        for (long long i = t0 / 4 + threadIdx.x; i < v1; i += kQThreads) {
            const float4 v = reinterpret_cast<const float4 *>(xs)[i];
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            if (kStochastic) {
                const uint64_t blk = base + (uint64_t)i;
                philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), k0, k1, w);
            }
            const uint32_t b0 = (uint32_t)round_code(v.x, inv, kStochastic, w[0]) & 0xffu;
            const uint32_t b1 = (uint32_t)round_code(v.y, inv, kStochastic, w[1]) & 0xffu;
            const uint32_t b2 = (uint32_t)round_code(v.z, inv, kStochastic, w[2]) & 0xffu;
            const uint32_t b3 = (uint32_t)round_code(v.w, inv, kStochastic, w[3]) & 0xffu;
            reinterpret_cast<uint32_t *>(qs)[i] = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
        }
        done = v1 * 4;
    }
    for (long long i = done + threadIdx.x; i < t1; i += kQThreads) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (kStochastic) {
            const uint64_t blk = base + (uint64_t)(i / 4);
            philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), k0, k1, w);
        }
        qs[i] = (int8_t)round_code(xs[i], inv, kStochastic, w[i & 3]);
    }
}

template <bool kAccumulate>
__global__ __launch_bounds__(kQThreads) void dequant_kernel(const int32_t *__restrict__ acc, size_t len,
                                                            const float *__restrict__ sA,
                                                            const float *__restrict__ sB, float *__restrict__ y) {
    const float s = __fmul_rn(*sA, *sB);
    const size_t nvec = len / 4;
    const int4 *av = reinterpret_cast<const int4 *>(acc);
    float4 *yv = reinterpret_cast<float4 *>(y);
    for (size_t i = (size_t)blockIdx.x * kQThreads + threadIdx.x; i < nvec; i += (size_t)gridDim.x * kQThreads) {
        const int4 a = av[i];
        float4 o = make_float4(s * (float)a.x, s * (float)a.y, s * (float)a.z, s * (float)a.w);
        if (kAccumulate) {
            const float4 p = yv[i];
            o.x += p.x; o.y += p.y; o.z += p.z; o.w += p.w;
        }
        yv[i] = o;
    }
    if (blockIdx.x == 0 && threadIdx.x < (len & 3)) {
        const size_t i = nvec * 4 + threadIdx.x;
        const float o = s * (float)acc[i];
        y[i] = kAccumulate ? y[i] + o : o;
    }
}

static int grid_for(size_t len, int per_thread) {
    size_t blocks = (len + (size_t)kQThreads * per_thread - 1) / ((size_t)kQThreads * per_thread);
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    return (int)blocks;
}

static int check_quant_args(const float *x, size_t len, int rounding, const int8_t *q, const float *scale) {
    LPDT_REQUIRE(x && q && scale, LPDT_EINVAL, "quantize: x, q and scale must be non-NULL");
    LPDT_REQUIRE(len > 0, LPDT_EUNSUPPORTED, "quantize: len must be positive");
    LPDT_REQUIRE(rounding == LPDT_ROUND_NEAREST || rounding == LPDT_ROUND_STOCHASTIC, LPDT_EINVAL,
                 "quantize: rounding must be LPDT_ROUND_NEAREST or LPDT_ROUND_STOCHASTIC (got %d)", rounding);
    LPDT_REQUIRE(aligned(x, 16) && aligned(q, 4) && aligned(scale, 4), LPDT_EINVAL,
                 "quantize: x must be 16-byte aligned, q and scale 4-byte aligned");
    return LPDT_OK;
}

// out = max of n non-negative partials (one block)
__global__ __launch_bounds__(1024) void absmax_fold_kernel(const float *__restrict__ parts, int n, float *__restrict__ out) {
    __shared__ float lds[1024 / kWave];
    float m = 0.0f;
    for (int i = threadIdx.x; i < n; i += 1024) m = fmaxf(m, parts[i]);
    m = wave_max(m);
    if (threadIdx.x % kWave == 0) lds[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = lds[0];
        for (int w = 1; w < 1024 / kWave; ++w) r = fmaxf(r, lds[w]);
        *out = r;
    }
}

void launch_absmax_fold(const float *parts, int n, float *out, hipStream_t st) {
    hipLaunchKernelGGL(absmax_fold_kernel, dim3(1), dim3(1024), 0, st, parts, n, out);
}

int absmax_scratch_floats() { return kMaxParts; }

void launch_absmax(const float *x, size_t len, float *scratch, float *out, hipStream_t st) {
    int g1 = grid_for(len, 16);
    if (g1 > kMaxParts) g1 = kMaxParts;
    hipLaunchKernelGGL(absmax_kernel, dim3(g1), dim3(kQThreads), 0, st, x, len, scratch);
    launch_absmax_fold(scratch, g1, out, st);
}

void launch_dequant(const int32_t *acc, size_t len, const float *sA, const float *sB, float *y, bool accumulate, hipStream_t st) {
    const int g = grid_for(len, 16);
    if (accumulate) hipLaunchKernelGGL(dequant_kernel<true>, dim3(g), dim3(kQThreads), 0, st, acc, len, sA, sB, y);
    else hipLaunchKernelGGL(dequant_kernel<false>, dim3(g), dim3(kQThreads), 0, st, acc, len, sA, sB, y);
}

}  // namespace lpdt

using namespace lpdt;

extern "C" size_t lpdt_quantize_workspace_bytes(size_t len) {
    (void)len;
    return kMaxParts * sizeof(float);
}

extern "C" int lpdt_quantize(const float *x, size_t len, int rounding, uint64_t seed, uint64_t offset, int8_t *q,
                             float *scale, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_quant_args(x, len, rounding, q, scale);
    if (rc) return rc;
    rc = check_ws(ws, ws_bytes, lpdt_quantize_workspace_bytes(len));
    if (rc) return rc;
    if (len <= kSmallLen) {
        if (rounding == LPDT_ROUND_STOCHASTIC)
            hipLaunchKernelGGL(quantize_small_kernel<true>, dim3(1), dim3(kSmallThreads), 0, as_stream(stream), x, len, seed, offset, q, scale);
        else
            hipLaunchKernelGGL(quantize_small_kernel<false>, dim3(1), dim3(kSmallThreads), 0, as_stream(stream), x, len, seed, offset, q, scale);
        return launch_status("lpdt_quantize");
    }
    float *parts = static_cast<float *>(ws);
    int g1 = grid_for(len, 16);
    if (g1 > kMaxParts) g1 = kMaxParts;
    hipLaunchKernelGGL(absmax_kernel, dim3(g1), dim3(kQThreads), 0, as_stream(stream), x, len, parts);
    const int g2 = grid_for(len, 16);
    if (rounding == LPDT_ROUND_STOCHASTIC)
        hipLaunchKernelGGL(round_kernel<true>, dim3(g2), dim3(kQThreads), 0, as_stream(stream), x, len, parts, g1,
                           seed, offset, q, scale);
    else
        hipLaunchKernelGGL(round_kernel<false>, dim3(g2), dim3(kQThreads), 0, as_stream(stream), x, len, parts, g1,
                           seed, offset, q, scale);
    return launch_status("lpdt_quantize");
}

extern "C" int lpdt_quantize_with_absmax(const float *x, size_t len, const float *absmax, int rounding,
                                         uint64_t seed, uint64_t offset, int8_t *q, float *scale, void *stream) {
    int rc = check_quant_args(x, len, rounding, q, scale);
    if (rc) return rc;
    LPDT_REQUIRE(absmax && aligned(absmax, 4), LPDT_EINVAL, "quantize_with_absmax: absmax must be a non-NULL device scalar");
    const int g2 = grid_for(len, 16);
    if (rounding == LPDT_ROUND_STOCHASTIC)
        hipLaunchKernelGGL(round_kernel<true>, dim3(g2), dim3(kQThreads), 0, as_stream(stream), x, len, absmax, 1,
                           seed, offset, q, scale);
    else
        hipLaunchKernelGGL(round_kernel<false>, dim3(g2), dim3(kQThreads), 0, as_stream(stream), x, len, absmax, 1,
                           seed, offset, q, scale);
    return launch_status("lpdt_quantize_with_absmax");
}

extern "C" int lpdt_dequantize(const int32_t *acc, size_t len, const float *sA, const float *sB, float *y,
                               int accumulate, void *stream) {
    LPDT_REQUIRE(acc && sA && sB && y, LPDT_EINVAL, "dequantize: NULL argument");
    LPDT_REQUIRE(len > 0, LPDT_EUNSUPPORTED, "dequantize: len must be positive");
    LPDT_REQUIRE(aligned(acc, 16) && aligned(y, 16), LPDT_EINVAL, "dequantize: acc and y must be 16-byte aligned");
    launch_dequant(acc, len, sA, sB, y, accumulate != 0, as_stream(stream));
    return launch_status("lpdt_dequantize");
}

extern "C" size_t lpdt_quantize_segments_workspace_bytes(int nseg) {
    if (nseg <= 0) return 0;
    return round_up((size_t)nseg * 2 * sizeof(long long), 256) + round_up((size_t)nseg * sizeof(unsigned int), 256);
}

extern "C" int lpdt_quantize_segments(const float *x, const int64_t *seg_begin, const int64_t *seg_end, int nseg, int rounding,
                                      uint64_t seed, uint64_t offset, int8_t *q, float *scales, void *ws, size_t ws_bytes,
                                      void *stream) {
    LPDT_REQUIRE(x && q && scales && seg_begin && seg_end, LPDT_EINVAL, "quantize_segments: NULL argument");
    LPDT_REQUIRE(nseg > 0, LPDT_EUNSUPPORTED, "quantize_segments: nseg must be positive");
    LPDT_REQUIRE(nseg <= 65535, LPDT_EUNSUPPORTED, "quantize_segments: at most 65535 slices");
    LPDT_REQUIRE(rounding == LPDT_ROUND_NEAREST || rounding == LPDT_ROUND_STOCHASTIC, LPDT_EINVAL,
                 "quantize_segments: rounding must be 0 (nearest) or 1 (stochastic)");
    LPDT_REQUIRE(aligned(x, 4) && aligned(scales, 4), LPDT_EINVAL, "quantize_segments: x and scales must be 4-byte aligned");
    long long longest = 0;
    for (int s = 0; s < nseg; ++s) {
        LPDT_REQUIRE(seg_begin[s] >= 0 && seg_end[s] > seg_begin[s], LPDT_EUNSUPPORTED,
                     "quantize_segments: slice %d is empty or negative", s);
        LPDT_REQUIRE(seg_end[s] - seg_begin[s] <= (1ll << 26), LPDT_EUNSUPPORTED,
                     "quantize_segments: slice %d has more than 2^26 elements (its stochastic-rounding counters would overlap the next slice's)", s);
        if (seg_end[s] - seg_begin[s] > longest) longest = seg_end[s] - seg_begin[s];
    }
    int rc = check_ws(ws, ws_bytes, lpdt_quantize_segments_workspace_bytes(nseg));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    long long *table = static_cast<long long *>(ws);
    unsigned int *amax = reinterpret_cast<unsigned int *>(static_cast<char *>(ws) + round_up((size_t)nseg * 2 * sizeof(long long), 256));
    for (int o = 0; o < nseg; o += kSegChunk) {
        SegChunk c;
        const int m = nseg - o < kSegChunk ? nseg - o : kSegChunk;
        for (int i = 0; i < m; ++i) { c.v[2 * i] = seg_begin[o + i]; c.v[2 * i + 1] = seg_end[o + i]; }
        hipLaunchKernelGGL(seg_upload_kernel, dim3(1), dim3(2 * kSegChunk), 0, st, c, table, amax, o, m);
    }
    const dim3 grid((unsigned)((longest + kSegTile - 1) / kSegTile), (unsigned)nseg);
    hipLaunchKernelGGL(seg_absmax_kernel, grid, dim3(kQThreads), 0, st, x, table, amax);
    if (rounding == LPDT_ROUND_STOCHASTIC)
        hipLaunchKernelGGL(seg_round_kernel<true>, grid, dim3(kQThreads), 0, st, x, table, amax, seed, offset, q, scales);
    else
        hipLaunchKernelGGL(seg_round_kernel<false>, grid, dim3(kQThreads), 0, st, x, table, amax, seed, offset, q, scales);
    return launch_status("lpdt_quantize_segments");
}

// ---- the quantizer for callers that cannot hand over a workspace ----------------------------------------------------
// Same two kernels as lpdt_quantize; the abs-max partials live in a file-scope device array instead of the caller's
// workspace.  Every GPU holds its own copy of the array; its address there is looked up once per device (the array's
// name is only a host-side handle and is never passed to a kernel) and kept.
static __device__ __align__(256) float scratch[kMaxParts];

namespace {
constexpr int kMaxDevices = 64;
float *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU; written once, under the mutex
std::mutex g_scratch_mutex;

int static_scratch(float **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(LPDT_EHIP, "quantize_static: hipGetDevice: %s", hipGetErrorString(e));
    LPDT_REQUIRE(dev >= 0 && dev < kMaxDevices, LPDT_EUNSUPPORTED, "quantize_static: device ordinal %d is beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));  // for the device that is current
        if (e != hipSuccess || !ptr) return fail(LPDT_EHIP, "quantize_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<float *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return LPDT_OK;
}
}  // namespace

extern "C" size_t lpdt_quantize_static_max_len(void) { return (size_t)1 << 30; }

extern "C" int lpdt_quantize_static(const float *x, size_t len, int rounding, uint64_t seed, uint64_t offset, int8_t *q,
                                    float *scale, void *stream) {
    int rc = check_quant_args(x, len, rounding, q, scale);
    if (rc) return rc;
    LPDT_REQUIRE(len <= lpdt_quantize_static_max_len(), LPDT_EUNSUPPORTED,
                 "quantize_static: len %zu exceeds the maximum of %zu elements (use lpdt_quantize with a workspace)", len,
                 lpdt_quantize_static_max_len());
    float *parts = nullptr;
    rc = static_scratch(&parts);
    if (rc) return rc;
    // every partial the second kernel reads is written by the first: nothing of the previous call's contents is used
    int g1 = grid_for(len, 16);
    if (g1 > kMaxParts) g1 = kMaxParts;
    hipLaunchKernelGGL(absmax_kernel, dim3(g1), dim3(kQThreads), 0, as_stream(stream), x, len, parts);
    const int g2 = grid_for(len, 16);
    if (rounding == LPDT_ROUND_STOCHASTIC)
        hipLaunchKernelGGL(round_kernel<true>, dim3(g2), dim3(kQThreads), 0, as_stream(stream), x, len, parts, g1,
                           seed, offset, q, scale);
    else
        hipLaunchKernelGGL(round_kernel<false>, dim3(g2), dim3(kQThreads), 0, as_stream(stream), x, len, parts, g1,
                           seed, offset, q, scale);
    return launch_status("lpdt_quantize_static");
}
