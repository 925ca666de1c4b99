// Glue layers of the benchmark networks (Table "hardware_training": skip
// connections, average pool; plus max-pool, softmax cross-entropy and the local
// SGD step of Algorithm 1 step 3).  fp32, NHWC, all bandwidth-trivial.
#include "common.h"

namespace lpdt {

constexpr int kT = 256;

static int grid1d(size_t work) {
    size_t b = (work + kT - 1) / kT;
    if (b < 1) b = 1;
    if (b > 16384) b = 16384;
    return (int)b;
}

__global__ __launch_bounds__(kT) void add_kernel(const float *a, const float *b, size_t len, float *y) {
    const size_t nvec = len / 4;
    for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < nvec; i += (size_t)gridDim.x * kT) {
        const float4 p = reinterpret_cast<const float4 *>(a)[i], q = reinterpret_cast<const float4 *>(b)[i];
        reinterpret_cast<float4 *>(y)[i] = make_float4(p.x + q.x, p.y + q.y, p.z + q.z, p.w + q.w);
    }
    if (blockIdx.x == 0 && threadIdx.x < (len & 3)) {
        const size_t i = nvec * 4 + threadIdx.x;
        y[i] = a[i] + b[i];
    }
}

__global__ __launch_bounds__(kT) void sgd_kernel(float *x, const float *g, size_t len, float lr) {
    const size_t nvec = len / 4;
    for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < nvec; i += (size_t)gridDim.x * kT) {
        float4 p = reinterpret_cast<float4 *>(x)[i];
        const float4 q = reinterpret_cast<const float4 *>(g)[i];
        p.x -= lr * q.x; p.y -= lr * q.y; p.z -= lr * q.z; p.w -= lr * q.w;
        reinterpret_cast<float4 *>(x)[i] = p;
    }
    if (blockIdx.x == 0 && threadIdx.x < (len & 3)) {
        const size_t i = nvec * 4 + threadIdx.x;
        x[i] -= lr * g[i];
    }
}

__global__ __launch_bounds__(kT) void maxpool_fwd_kernel(const float *__restrict__ x, int N, int H, int W, int C, int k, int st,
                                                         int pd, int P, int Q, float *__restrict__ y, int32_t *__restrict__ idx) {
    const size_t total = (size_t)N * P * Q * C;
    for (size_t o = (size_t)blockIdx.x * kT + threadIdx.x; o < total; o += (size_t)gridDim.x * kT) {
        const int c = (int)(o % C);
        size_t r = o / C;
        const int q = (int)(r % Q); r /= Q;
        const int p = (int)(r % P);
        const int n = (int)(r / P);
        float best = 0.0f;
        int bi = -1;
        for (int i = 0; i < k; ++i)
            for (int j = 0; j < k; ++j) {
                const int h = p * st + i - pd, w = q * st + j - pd;
                if (h < 0 || h >= H || w < 0 || w >= W) continue;
                const float e = x[(((size_t)n * H + h) * W + w) * C + c];
                if (bi < 0 || e > best) { best = e; bi = h * W + w; }
            }
        y[o] = best;
        idx[o] = bi;
    }
}

// gather form of the scatter dx[n, idx, c] += dy: each input position sums the outputs whose
// window covers it and whose winner it is (at most ceil(k/st)^2 of them), in a fixed order.
__global__ __launch_bounds__(kT) void maxpool_bwd_kernel(const float *__restrict__ dy, const int32_t *__restrict__ idx, int N,
                                                         int H, int W, int C, int k, int st, int pd, int P, int Q,
                                                         float *__restrict__ dx) {
    const size_t total = (size_t)N * H * W * C;
    for (size_t o = (size_t)blockIdx.x * kT + threadIdx.x; o < total; o += (size_t)gridDim.x * kT) {
        const int c = (int)(o % C);
        size_t r = o / C;
        const int w = (int)(r % W); r /= W;
        const int h = (int)(r % H);
        const int n = (int)(r / H);
        float s = 0.0f;
        // windows covering (h, w): p*st - pd <= h < p*st - pd + k
        const int p_lo = max(0, (h + pd - k + st) / st), p_hi = min(P - 1, (h + pd) / st);
        const int q_lo = max(0, (w + pd - k + st) / st), q_hi = min(Q - 1, (w + pd) / st);
        for (int p = p_lo; p <= p_hi; ++p)
            for (int q = q_lo; q <= q_hi; ++q) {
                const size_t at = (((size_t)n * P + p) * Q + q) * C + c;
                if (idx[at] == h * W + w) s += dy[at];
            }
        dx[o] = s;
    }
}

// 4 channels per thread (16-byte accesses), 32-bit index arithmetic: the form every benchmark shape takes
__global__ __launch_bounds__(kT) void maxpool_fwd_vec_kernel(const float4 *__restrict__ x, int N, int H, int W, int C4, int k, int st,
                                                             int pd, int P, int Q, float4 *__restrict__ y, int4 *__restrict__ idx) {
    const unsigned total = (unsigned)N * P * Q * C4;
    for (unsigned o = blockIdx.x * kT + threadIdx.x; o < total; o += gridDim.x * kT) {
        const unsigned c = o % (unsigned)C4;
        unsigned r = o / (unsigned)C4;
        const int q = (int)(r % (unsigned)Q); r /= (unsigned)Q;
        const int p = (int)(r % (unsigned)P);
        const int n = (int)(r / (unsigned)P);
        float best[4] = {0.f, 0.f, 0.f, 0.f};
        int bi[4] = {-1, -1, -1, -1};
        for (int i = 0; i < k; ++i) {
            const int h = p * st + i - pd;
            if (h < 0 || h >= H) continue;
            for (int j = 0; j < k; ++j) {
                const int w = q * st + j - pd;
                if (w < 0 || w >= W) continue;
                const float4 e4 = x[((unsigned)(n * H + h) * W + w) * (unsigned)C4 + c];
                const float e[4] = {e4.x, e4.y, e4.z, e4.w};
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (bi[u] < 0 || e[u] > best[u]) { best[u] = e[u]; bi[u] = h * W + w; }
            }
        }
        y[o] = make_float4(best[0], best[1], best[2], best[3]);
        idx[o] = make_int4(bi[0], bi[1], bi[2], bi[3]);
    }
}

template <bool kTwoByTwo>
__global__ __launch_bounds__(kT) void maxpool_bwd_vec_kernel(const float4 *__restrict__ dy, const int4 *__restrict__ idx, int N,
                                                             int H, int W, int C4, int k, int st, int pd, int P, int Q,
                                                             float4 *__restrict__ dx) {
    const unsigned total = (unsigned)N * H * W * C4;
    for (unsigned o = blockIdx.x * kT + threadIdx.x; o < total; o += gridDim.x * kT) {
        const unsigned c = o % (unsigned)C4;
        unsigned r = o / (unsigned)C4;
        const int w = (int)(r % (unsigned)W); r /= (unsigned)W;
        const int h = (int)(r % (unsigned)H);
        const int n = (int)(r / (unsigned)H);
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        const int p_lo = max(0, (h + pd - k + st) / st), p_hi = min(P - 1, (h + pd) / st);
        const int q_lo = max(0, (w + pd - k + st) / st), q_hi = min(Q - 1, (w + pd) / st);
        const int me = h * W + w;
        if (kTwoByTwo) {  // at most 2 x 2 windows hold this pixel: all their loads are issued before the first is used
            int4 id[4];
            float4 g[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = p_lo + j / 2, q = q_lo + j % 2;
                const bool ok = p <= p_hi && q <= q_hi;
                const unsigned at = ((unsigned)(n * P + p) * Q + q) * (unsigned)C4 + c;
                id[j] = ok ? idx[at] : make_int4(-1, -1, -1, -1);
                g[j] = ok ? dy[at] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {  // same order as the loops below; a window that is not there adds nothing
                if (id[j].x == me) s.x += g[j].x;
                if (id[j].y == me) s.y += g[j].y;
                if (id[j].z == me) s.z += g[j].z;
                if (id[j].w == me) s.w += g[j].w;
            }
        } else {
            for (int p = p_lo; p <= p_hi; ++p)
                for (int q = q_lo; q <= q_hi; ++q) {
                    const unsigned at = ((unsigned)(n * P + p) * Q + q) * (unsigned)C4 + c;
                    const int4 id = idx[at];
                    const float4 g = dy[at];
                    if (id.x == me) s.x += g.x;
                    if (id.y == me) s.y += g.y;
                    if (id.z == me) s.z += g.z;
                    if (id.w == me) s.w += g.w;
                }
        }
        dx[o] = s;
    }
}

__global__ __launch_bounds__(kT) void avgpool_fwd_kernel(const float *__restrict__ x, int N, int HW, int C, float *__restrict__ y) {
    const int o = blockIdx.x * kT + threadIdx.x;
    if (o >= N * C) return;
    const int n = o / C, c = o % C;
    float s = 0.0f;
#pragma unroll 8
    for (int i = 0; i < HW; ++i) s += x[((size_t)n * HW + i) * C + c];   // same order of additions, loads issued 8 at a time
    y[o] = s / (float)HW;
}

__global__ __launch_bounds__(kT) void avgpool_bwd_kernel(const float *__restrict__ dy, int N, int HW, int C, float *__restrict__ dx) {
    const size_t total = (size_t)N * HW * C;
    const float inv = 1.0f / (float)HW;
    for (size_t o = (size_t)blockIdx.x * kT + threadIdx.x; o < total; o += (size_t)gridDim.x * kT) {
        const int c = (int)(o % C);
        const int n = (int)(o / ((size_t)HW * C));
        dx[o] = dy[(size_t)n * C + c] * inv;
    }
}

// one wave per sample; block 0 also reduces the per-sample losses in a fixed order
__global__ __launch_bounds__(kWave) void xent_kernel(const float *__restrict__ logits, const int32_t *__restrict__ labels, int N,
                                                     int classes, float *__restrict__ sample_loss, float *__restrict__ dlogits) {
    const int n = blockIdx.x, lane = threadIdx.x;
    const float *l = logits + (size_t)n * classes;
    float mx = -3.4e38f;
    for (int j = lane; j < classes; j += kWave) mx = fmaxf(mx, l[j]);
    mx = wave_max(mx);
    float z = 0.0f;
    for (int j = lane; j < classes; j += kWave) z += expf(l[j] - mx);
    z = wave_sum(z);
    // a label outside [0, classes) reads nothing: that sample's loss is NaN and its gradient has no target term
    const int lb = labels[n];
    const bool valid = (unsigned)lb < (unsigned)classes;
    for (int j = lane; j < classes; j += kWave)
        dlogits[(size_t)n * classes + j] = (expf(l[j] - mx) / z - (j == lb ? 1.0f : 0.0f)) / (float)N;
    if (lane == 0) sample_loss[n] = valid ? logf(z) + mx - l[lb] : __builtin_nanf("");
}
__global__ void xent_mean_kernel(const float *__restrict__ sample_loss, int N, float *__restrict__ loss) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        float s = 0.0f;
        for (int n = 0; n < N; ++n) s += sample_loss[n];
        *loss = s / (float)N;
    }
}

}  // namespace lpdt

using namespace lpdt;

extern "C" int lpdt_add(const float *a, const float *b, size_t len, float *y, void *stream) {
    LPDT_REQUIRE(a && b && y, LPDT_EINVAL, "add: NULL argument");
    LPDT_REQUIRE(len > 0, LPDT_EUNSUPPORTED, "add: len must be positive");
    LPDT_REQUIRE(aligned(a, 16) && aligned(b, 16) && aligned(y, 16), LPDT_EINVAL, "add: buffers must be 16-byte aligned");
    hipLaunchKernelGGL(add_kernel, dim3(grid1d(len / 4 + 1)), dim3(kT), 0, as_stream(stream), a, b, len, y);
    return launch_status("lpdt_add");
}

extern "C" int lpdt_sgd(float *x, const float *g, size_t len, float lr, void *stream) {
    LPDT_REQUIRE(x && g, LPDT_EINVAL, "sgd: NULL argument");
    LPDT_REQUIRE(len > 0, LPDT_EUNSUPPORTED, "sgd: len must be positive");
    LPDT_REQUIRE(aligned(x, 16) && aligned(g, 16), LPDT_EINVAL, "sgd: buffers must be 16-byte aligned");
    hipLaunchKernelGGL(sgd_kernel, dim3(grid1d(len / 4 + 1)), dim3(kT), 0, as_stream(stream), x, g, len, lr);
    return launch_status("lpdt_sgd");
}

static bool pool_vec_ok(int N, int H, int W, int C) { return C % 4 == 0 && (size_t)N * H * W * C < ((size_t)1 << 31); }

static int check_pool(int N, int H, int W, int C, int k, int st, int pd) {
    LPDT_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0, LPDT_EINVAL, "maxpool: sizes must be positive");
    LPDT_REQUIRE(k > 0 && st > 0 && pd >= 0 && pd < k, LPDT_EINVAL, "maxpool: need k > 0, stride > 0, 0 <= pad < k");
    LPDT_REQUIRE(H + 2 * pd >= k && W + 2 * pd >= k, LPDT_EINVAL, "maxpool: window larger than padded input");
    return LPDT_OK;
}

extern "C" int lpdt_maxpool_fwd(const float *x, int N, int H, int W, int C, int k, int st, int pd, float *y, int32_t *idx,
                                void *stream) {
    int rc = check_pool(N, H, W, C, k, st, pd);
    if (rc) return rc;
    LPDT_REQUIRE(x && y && idx, LPDT_EINVAL, "maxpool_fwd: NULL argument");
    const int P = conv_out(H, pd, k, st), Q = conv_out(W, pd, k, st);
    if (pool_vec_ok(N, H, W, C) && aligned(x, 16) && aligned(y, 16) && aligned(idx, 16))
        hipLaunchKernelGGL(maxpool_fwd_vec_kernel, dim3(grid1d((size_t)N * P * Q * (C / 4))), dim3(kT), 0, as_stream(stream),
                           reinterpret_cast<const float4 *>(x), N, H, W, C / 4, k, st, pd, P, Q, reinterpret_cast<float4 *>(y),
                           reinterpret_cast<int4 *>(idx));
    else
        hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(grid1d((size_t)N * P * Q * C)), dim3(kT), 0, as_stream(stream), x, N, H, W, C, k,
                           st, pd, P, Q, y, idx);
    return launch_status("lpdt_maxpool_fwd");
}

extern "C" int lpdt_maxpool_bwd(const float *dy, const int32_t *idx, int N, int H, int W, int C, int k, int st, int pd,
                                float *dx, void *stream) {
    int rc = check_pool(N, H, W, C, k, st, pd);
    if (rc) return rc;
    LPDT_REQUIRE(dy && idx && dx, LPDT_EINVAL, "maxpool_bwd: NULL argument");
    const int P = conv_out(H, pd, k, st), Q = conv_out(W, pd, k, st);
    if (pool_vec_ok(N, H, W, C) && aligned(dy, 16) && aligned(idx, 16) && aligned(dx, 16)) {
        const dim3 grid(grid1d((size_t)N * H * W * (C / 4)));
        const float4 *dy4 = reinterpret_cast<const float4 *>(dy);
        const int4 *idx4 = reinterpret_cast<const int4 *>(idx);
        float4 *dx4 = reinterpret_cast<float4 *>(dx);
        if ((k + st - 1) / st <= 2)  // a pixel lies in at most ceil(k / stride) windows per direction
            hipLaunchKernelGGL(maxpool_bwd_vec_kernel<true>, grid, dim3(kT), 0, as_stream(stream), dy4, idx4, N, H, W, C / 4, k, st,
                               pd, P, Q, dx4);
        else
            hipLaunchKernelGGL(maxpool_bwd_vec_kernel<false>, grid, dim3(kT), 0, as_stream(stream), dy4, idx4, N, H, W, C / 4, k, st,
                               pd, P, Q, dx4);
    } else
        hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(grid1d((size_t)N * H * W * C)), dim3(kT), 0, as_stream(stream), dy, idx, N, H, W,
                           C, k, st, pd, P, Q, dx);
    return launch_status("lpdt_maxpool_bwd");
}

extern "C" int lpdt_avgpool_fwd(const float *x, int N, int HW, int C, float *y, void *stream) {
    LPDT_REQUIRE(x && y, LPDT_EINVAL, "avgpool_fwd: NULL argument");
    LPDT_REQUIRE(N > 0 && HW > 0 && C > 0, LPDT_EINVAL, "avgpool_fwd: sizes must be positive");
    hipLaunchKernelGGL(avgpool_fwd_kernel, dim3((N * C + kT - 1) / kT), dim3(kT), 0, as_stream(stream), x, N, HW, C, y);
    return launch_status("lpdt_avgpool_fwd");
}

extern "C" int lpdt_avgpool_bwd(const float *dy, int N, int HW, int C, float *dx, void *stream) {
    LPDT_REQUIRE(dy && dx, LPDT_EINVAL, "avgpool_bwd: NULL argument");
    LPDT_REQUIRE(N > 0 && HW > 0 && C > 0, LPDT_EINVAL, "avgpool_bwd: sizes must be positive");
    hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(grid1d((size_t)N * HW * C)), dim3(kT), 0, as_stream(stream), dy, N, HW, C, dx);
    return launch_status("lpdt_avgpool_bwd");
}

extern "C" int lpdt_softmax_xent(const float *logits, const int32_t *labels, int N, int classes, float *loss, float *dlogits,
                                 void *stream) {
    LPDT_REQUIRE(logits && labels && loss && dlogits, LPDT_EINVAL, "softmax_xent: NULL argument");
    LPDT_REQUIRE(N > 0 && classes > 0, LPDT_EINVAL, "softmax_xent: sizes must be positive");
    LPDT_REQUIRE(classes <= 1024, LPDT_EUNSUPPORTED, "softmax_xent: at most 1024 classes");
    // loss[1..N] hold the per-sample losses; loss[0] their mean, summed in sample order
    hipLaunchKernelGGL(xent_kernel, dim3(N), dim3(kWave), 0, as_stream(stream), logits, labels, N, classes, loss + 1, dlogits);
    hipLaunchKernelGGL(xent_mean_kernel, dim3(1), dim3(64), 0, as_stream(stream), loss + 1, N, loss);
    return launch_status("lpdt_softmax_xent");
}
