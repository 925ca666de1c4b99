// Entry points of the three int8 convolution products with exact int32 accumulation (Table "hardware_training", row
// Conv), and the kernels that take the shapes the matrix-core kernels do not.
//
//  forward / backward-data: out[m][j] = sum_{tap,c} in[pix(m,tap)][c] * wt[j][tap][c], an implicit GEMM (no im2col
//      copy).  The kernels live in qconv_igemm_dma.hip (operands loaded straight into LDS; reductions over a multiple of
//      64 channels), qconv_igemm.hip (register-staged loads, any multiple of 16 channels; splits the reduction over
//      blocks with int32 atomics where there are too few tiles; also the filter transposition backward-data reads) and
//      qconv_narrow.hip (first layer: 3 input channels).  This file chooses between them, stages the int32 sums in the
//      workspace where the chosen kernel cannot apply the dequantizing scale itself, and holds the one-thread-per-output
//      kernels for every other shape.
//  backward-weight: dw[k][tap][c] = sum_m g[m][k] * x[pix(m,tap)][c]; the reduction runs over pixels, the strided
//      axis of both NHWC operands.  qconv_wgrad.hip (rectangle steps, partial tiles, fixed-order reduce) takes the
//      layers of the benchmark networks; wgrad_kernel below is the older per-tap form (one shifted copy of the input
//      tile per tap in LDS, transposing LDS reads, int32 atomic combine) kept for shapes the rectangle plan rejects,
//      and conv_bwd_weight_plain_kernel takes channel counts that are not multiples of 16.
#include "qconv_internal.h"
#include <cstdlib>
#include <type_traits>

namespace lpdt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kCThreads = 256;

// ------------------------------------------------------------------ wgrad
struct WgradParams {
    const int8_t *g;   // [M][K], M = N*P*Q
    const int8_t *x;   // [N][H][W][C]
    int32_t *dw;       // [K][R*S][C], zeroed before the launch
    int M, K, C, H, W, P, Q, R, S, stride, pad;
    int tiles_k;       // ceil(K/64)
    int chunks;        // ceil(M/32)
    int chunks_per_split;
};

constexpr int kWRow = 96;              // LDS bytes per pixel row: 64 channels + 32 pad (8 rows tile the 64 banks)
constexpr int kWTile = 32 * kWRow;     // one [32 px][64 ch] tile

template <int TG>
__global__ __launch_bounds__(kCThreads) void wgrad_kernel(const WgradParams p) {
    constexpr int NT = 1 + TG;             // tile 0 = gradient, tile 1+i = input shifted by tap i
    constexpr int ITEMS = (NT + 1) / 2;    // 16-byte items per thread (128 items per tile, 256 threads)
    constexpr int BUF = NT * kWTile;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF];

    const int t = threadIdx.x, lane = t % 64, wave = t / 64;
    const int g4 = t % 4, px = (t % 128) / 4, tp = t / 128;
    const int k0 = (blockIdx.x % p.tiles_k) * 64, c0 = (blockIdx.x / p.tiles_k) * 64;
    const int tap0 = blockIdx.y * TG, ntaps = p.R * p.S;
    const int ch_begin = blockIdx.z * p.chunks_per_split;
    const int ch_end = min(p.chunks, ch_begin + p.chunks_per_split);

    // this thread's pixel (n, oy, ox), advanced by 32 pixels per step
    const int step_q = 32 / p.Q, step_r = 32 % p.Q;
    int m = ch_begin * 32 + px;
    int n = m / (p.P * p.Q), oy = (m % (p.P * p.Q)) / p.Q, ox = m % p.Q;

    v4i stage[ITEMS];
    auto load_tiles = [&]() {
        const bool mvalid = m < p.M;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int tile = tp + 2 * j;
            v4i v = {0, 0, 0, 0};
            if (tile == 0) {
                if (mvalid && k0 + g4 * 16 < p.K) v = *reinterpret_cast<const v4i *>(p.g + (size_t)m * p.K + k0 + g4 * 16);
            } else if (tile < NT) {
                const int tap = tap0 + tile - 1;
                const int r = tap / p.S, s = tap % p.S;
                const int iy = oy * p.stride + r - p.pad, ix = ox * p.stride + s - p.pad;
                if (mvalid && tap < ntaps && iy >= 0 && iy < p.H && ix >= 0 && ix < p.W && c0 + g4 * 16 < p.C)
                    v = *reinterpret_cast<const v4i *>(p.x + ((size_t)(n * p.H + iy) * p.W + ix) * p.C + c0 + g4 * 16);
            }
            stage[j] = v;
        }
    };
    auto advance = [&]() {
        m += 32;
        ox += step_r;
        oy += step_q;
        if (ox >= p.Q) { ox -= p.Q; ++oy; }
        while (oy >= p.P) { oy -= p.P; ++n; }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int tile = tp + 2 * j;
            if (tile < NT) *reinterpret_cast<v4i *>(lds + buf * BUF + tile * kWTile + px * kWRow + g4 * 16) = stage[j];
        }
    };

    v16i acc[TG];
#pragma unroll
    for (int i = 0; i < TG; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;

    // Transposing LDS read: in each block of 16 lanes, source lane j supplies 8 bytes and result
    // lane i receives byte (i%8) of source lanes i/8, i/8+2, ..., i/8+14.  With source lane j
    // reading pixel j/2 at channel offset 8*(j%2), result lane i holds channel i of 8 pixels.
    const int ti = wave / 2, tj = wave % 2;
    const int blk = lane / 16, j16 = lane % 16;
    const int src_px = 16 * (blk / 2) + j16 / 2;                  // + 8*h for the second half of the operand
    const int src_ch = 16 * (blk % 2) + 8 * (j16 % 2);
    const int a_off = src_px * kWRow + 32 * ti + src_ch;
    const int b_off = src_px * kWRow + 32 * tj + src_ch;
    typedef __attribute__((address_space(3))) v2i lds_v2i;

    if (ch_begin < ch_end) {
        load_tiles();
        store_tiles(0);
        advance();
    }
    __syncthreads();
    for (int ch = ch_begin; ch < ch_end; ++ch) {
        const int buf = (ch - ch_begin) & 1;
        const bool more = ch + 1 < ch_end;
        if (more) load_tiles();
        unsigned char *base = lds + buf * BUF;
        const v2i a_lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off));
        const v2i a_hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off + 8 * kWRow));
        const v4i a = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
#pragma unroll
        for (int i = 0; i < TG; ++i) {
            if (tap0 + i < ntaps) {
                unsigned char *xt = base + (1 + i) * kWTile;
                const v2i b_lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(xt + b_off));
                const v2i b_hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(xt + b_off + 8 * kWRow));
                const v4i b = {b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
            }
        }
        if (more) {
            store_tiles(buf ^ 1);
            advance();
        }
        __syncthreads();
    }

    const int c = c0 + 32 * tj + lane % 32;
#pragma unroll
    for (int i = 0; i < TG; ++i) {
        const int tap = tap0 + i;
        if (tap < ntaps && c < p.C) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + 32 * ti + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                if (k < p.K && acc[i][r] != 0) atomicAdd(p.dw + ((size_t)k * ntaps + tap) * p.C + c, acc[i][r]);
            }
        }
    }
}

// ------------------------------------------------------------------ helpers and plain kernels
__global__ void fill_i32_kernel(int32_t *dst, size_t len) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < len; i += (size_t)gridDim.x * blockDim.x) dst[i] = 0;
}

// one thread per output element; any shape
__global__ __launch_bounds__(kCThreads) void conv_fwd_plain_kernel(const int8_t *__restrict__ x, const int8_t *__restrict__ w,
                                                                   int32_t *__restrict__ acc, lpdt_conv_desc d, int P, int Q) {
    const size_t total = (size_t)d.N * P * Q * d.K;
    for (size_t o = (size_t)blockIdx.x * kCThreads + threadIdx.x; o < total; o += (size_t)gridDim.x * kCThreads) {
        const int k = (int)(o % d.K);
        size_t rest = o / d.K;
        const int q = (int)(rest % Q); rest /= Q;
        const int pp = (int)(rest % P);
        const int n = (int)(rest / P);
        int s = 0;
        for (int r = 0; r < d.R; ++r) {
            const int h = pp * d.stride_h + r - d.pad_h;
            if (h < 0 || h >= d.H) continue;
            for (int t = 0; t < d.S; ++t) {
                const int ww = q * d.stride_w + t - d.pad_w;
                if (ww < 0 || ww >= d.W) continue;
                const int8_t *xp = x + (((size_t)n * d.H + h) * d.W + ww) * d.C;
                const int8_t *wp = w + (((size_t)k * d.R + r) * d.S + t) * d.C;
#pragma unroll 8
                for (int c = 0; c < d.C; ++c) s += (int)xp[c] * (int)wp[c];
            }
        }
        acc[o] = s;
    }
}

__global__ __launch_bounds__(kCThreads) void conv_bwd_data_plain_kernel(const int8_t *__restrict__ g, const int8_t *__restrict__ w,
                                                                        int32_t *__restrict__ dx, lpdt_conv_desc d, int P, int Q) {
    const size_t total = (size_t)d.N * d.H * d.W * d.C;
    for (size_t o = (size_t)blockIdx.x * kCThreads + threadIdx.x; o < total; o += (size_t)gridDim.x * kCThreads) {
        const int c = (int)(o % d.C);
        size_t rest = o / d.C;
        const int ww = (int)(rest % d.W); rest /= d.W;
        const int h = (int)(rest % d.H);
        const int n = (int)(rest / d.H);
        int s = 0;
        for (int r = 0; r < d.R; ++r) {
            const int ty = h + d.pad_h - r;
            if (ty < 0 || ty % d.stride_h) continue;
            const int pp = ty / d.stride_h;
            if (pp >= P) continue;
            for (int t = 0; t < d.S; ++t) {
                const int tx = ww + d.pad_w - t;
                if (tx < 0 || tx % d.stride_w) continue;
                const int q = tx / d.stride_w;
                if (q >= Q) continue;
                const int8_t *gp = g + (((size_t)n * P + pp) * Q + q) * d.K;
#pragma unroll 8
                for (int k = 0; k < d.K; ++k) s += (int)gp[k] * (int)w[(((size_t)k * d.R + r) * d.S + t) * d.C + c];
            }
        }
        dx[o] = s;
    }
}

// one thread per filter element and pixel slice, int32 atomic combine
__global__ __launch_bounds__(kCThreads) void conv_bwd_weight_plain_kernel(const int8_t *__restrict__ g, const int8_t *__restrict__ x,
                                                                          int32_t *__restrict__ dw, lpdt_conv_desc d, int P, int Q,
                                                                          int pix_per_slice) {
    const int total = d.K * d.R * d.S * d.C;
    const int o = blockIdx.x * kCThreads + threadIdx.x;
    if (o >= total) return;
    const int c = o % d.C;
    int rest = o / d.C;
    const int t = rest % d.S; rest /= d.S;
    const int r = rest % d.R;
    const int k = rest / d.R;
    const long long M = (long long)d.N * P * Q;
    const long long m_begin = (long long)blockIdx.y * pix_per_slice, m_end = min(M, m_begin + pix_per_slice);
    int s = 0;
    int n = (int)(m_begin / (P * Q)), pp = (int)((m_begin % (P * Q)) / Q), q = (int)(m_begin % Q);
    for (long long m = m_begin; m < m_end; ++m) {
        const int h = pp * d.stride_h + r - d.pad_h, ww = q * d.stride_w + t - d.pad_w;
        if (h >= 0 && h < d.H && ww >= 0 && ww < d.W)
            s += (int)g[(size_t)m * d.K + k] * (int)x[(((size_t)n * d.H + h) * d.W + ww) * d.C + c];
        if (++q == Q) { q = 0; if (++pp == P) { pp = 0; ++n; } }
    }
    if (s) atomicAdd(dw + o, s);
}


// ---- small linear layers (a network's classifier): 1x1 filters, stride 1, no padding, at most a few million
// multiply-adds.  One thread per result element, any channel counts and alignments, the dequantizing scale (and, for
// forward and backward-data, the addition to what the result holds) applied on the spot: one short launch instead of
// the zero fill, split reduction and dequantizing pass the tiled kernels would need at this size.
// mode 0: int32 sums; 1: fp32 sA*sB*sum; 2: fp32 added to out.  rows = N*H*W.
template <int KIND>  // 0: out[m][k] = sum_c x[m][c] w[k][c]; 1: dx[m][c] = sum_k g[m][k] w[k][c]; 2: dw[k][c] = sum_m g[m][k] x[m][c]
__global__ __launch_bounds__(kCThreads) void linear_small_kernel(const int8_t *__restrict__ a, const int8_t *__restrict__ b,
                                                                 void *__restrict__ out, int rows, int C, int K, int mode,
                                                                 const float *__restrict__ sA, const float *__restrict__ sB) {
    const int total = KIND == 0 ? rows * K : KIND == 1 ? rows * C : K * C;
    const int o = blockIdx.x * kCThreads + threadIdx.x;
    if (o >= total) return;
    int s = 0;
    if (KIND == 0) {
        const int m = o / K, k = o - m * K;
        const int8_t *xp = a + (size_t)m * C, *wp = b + (size_t)k * C;
        // the loops are chains of dependent-free loads: unrolled so that several are in flight (a thread's whole time is
        // load latency), 16 bytes per load where the rows allow it
        int c = 0;
        if (C % 16 == 0 && ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15) == 0) {
            typedef int v4i_t __attribute__((ext_vector_type(4)));
#pragma unroll 4
            for (; c < C; c += 16) {
                const v4i_t xv = *reinterpret_cast<const v4i_t *>(xp + c), wv = *reinterpret_cast<const v4i_t *>(wp + c);
#pragma unroll
                for (int e = 0; e < 4; ++e) s = __builtin_amdgcn_sdot4(xv[e], wv[e], s, false);
            }
        } else if (C % 4 == 0 && ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 3) == 0) {
#pragma unroll 8
            for (; c < C; c += 4)
                s = __builtin_amdgcn_sdot4(*reinterpret_cast<const int *>(xp + c), *reinterpret_cast<const int *>(wp + c), s, false);
        }
        for (; c < C; ++c) s += (int)xp[c] * (int)wp[c];
    } else if (KIND == 1) {
        const int m = o / C, c = o - m * C;
        const int8_t *gp = a + (size_t)m * K;
#pragma unroll 8
        for (int k = 0; k < K; ++k) s += (int)gp[k] * (int)b[(size_t)k * C + c];
    } else {
        const int k = o / C, c = o - k * C;
#pragma unroll 8
        for (int m = 0; m < rows; ++m) s += (int)a[(size_t)m * K + k] * (int)b[(size_t)m * C + c];
    }
    if (mode == 0) static_cast<int32_t *>(out)[o] = s;
    else {
        float *f = static_cast<float *>(out) + o;
        *f = dequant_value(__fmul_rn(*sA, *sB), s, mode == 2 ? *f : 0.0f, mode == 2);
    }
}

static bool small_linear(const lpdt_conv_desc *d) {
    return d->R == 1 && d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 && d->pad_w == 0 &&
           (long long)d->N * d->H * d->W * d->C * d->K <= (4ll << 20);
}
template <int KIND>
static void launch_linear_small(const lpdt_conv_desc *d, const int8_t *a, const int8_t *b, void *out, int mode, const float *sA,
                                const float *sB, hipStream_t st) {
    const int rows = d->N * d->H * d->W;
    const int total = KIND == 0 ? rows * d->K : KIND == 1 ? rows * d->C : d->K * d->C;
    hipLaunchKernelGGL(linear_small_kernel<KIND>, dim3((unsigned)((total + kCThreads - 1) / kCThreads)), dim3(kCThreads), 0, st, a, b, out,
                       rows, d->C, d->K, mode, sA, sB);
}

static int blocks_for(size_t total, int cap = 65536) {
    size_t b = (total + kCThreads - 1) / kCThreads;
    if (b < 1) b = 1;
    if (b > (size_t)cap) b = cap;
    return (int)b;
}

static bool same_stride_pad(const lpdt_conv_desc *d) { return d->stride_h == d->stride_w && d->pad_h == d->pad_w; }

}  // namespace lpdt

using namespace lpdt;

static bool narrow_ok(const lpdt_conv_desc *d) {
    if (!d || d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->stride_h <= 0 ||
        d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0 || d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S)
        return false;
    return narrow_conv_supported(d, conv_out(d->H, d->pad_h, d->R, d->stride_h), conv_out(d->W, d->pad_w, d->S, d->stride_w));
}

extern "C" size_t lpdt_qconv_fwd_workspace_bytes(const lpdt_conv_desc *d) {
    return narrow_ok(d) ? narrow_fwd_workspace(d) : 0;
}
extern "C" size_t lpdt_qconv_bwd_data_workspace_bytes(const lpdt_conv_desc *d) {
    if (!d || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->C <= 0) return 0;
    return round_up((size_t)d->K * d->R * d->S * d->C, 256);
}


// Forward product.  out_mode 0: int32 sums to `out`; 1: fp32 sA*sB*sum.  When the kernel that runs cannot apply the
// scale itself (split reduction, plain kernel) the sums go to the tail of the workspace and a dequantize pass follows.
static size_t fwd_base_ws(const lpdt_conv_desc *d) { return narrow_ok(d) ? narrow_fwd_workspace(d) : 0; }
static bool fwd_vec(const lpdt_conv_desc *d, int P, int Q) { return igemm_fwd_supported(d, P, Q); }
static bool fwd_fusable(const lpdt_conv_desc *d, int P, int Q) {
    if (narrow_conv_supported(d, P, Q)) return true;
    return fwd_vec(d, P, Q) && !igemm_fwd_is_split(d, P, Q);
}

// pabs: room for the abs-max partials of the fused implicit-GEMM epilogue; returns how many were written (0: none, the
// caller takes the abs-max of `out` in a pass of its own)
static int conv_fwd_impl(const lpdt_conv_desc *d, int P, int Q, const int8_t *xq, const int8_t *wq, void *out, int out_mode,
                         const float *sA, const float *sB, void *ws, hipStream_t st, float *pabs = nullptr) {
    int nparts = 0;
    const size_t out_len = (size_t)d->N * P * Q * d->K;
    if (small_linear(d)) {
        launch_linear_small<0>(d, xq, wq, out, out_mode, sA, sB, st);
        return 0;
    }
    // out_mode 2 (fp32, added to what is in `out`) is fused by the implicit-GEMM kernel only; the first-layer kernel stages
    const bool fused = fwd_fusable(d, P, Q) && aligned(xq, 16) && aligned(wq, 16) && !(out_mode == 2 && narrow_conv_supported(d, P, Q));
    const bool stage = out_mode != 0 && !fused;
    int32_t *acc = stage ? reinterpret_cast<int32_t *>(static_cast<char *>(ws) + round_up(fwd_base_ws(d), 256))
                         : static_cast<int32_t *>(out);
    const int mode = stage ? 0 : out_mode;
    if (narrow_conv_supported(d, P, Q)) {
        launch_narrow_fwd(d, P, Q, xq, wq, acc, mode, sA, sB, ws, st);
    } else if (fwd_vec(d, P, Q) && aligned(xq, 16) && aligned(wq, 16)) {
        if (pabs && mode != 0) nparts = igemm_fwd_absmax_parts(d, P, Q);
        launch_igemm_fwd(d, P, Q, xq, wq, acc, mode, sA, sB, st, nparts > 0 ? pabs : nullptr);
    } else {
        hipLaunchKernelGGL(conv_fwd_plain_kernel, dim3(blocks_for(out_len)), dim3(kCThreads), 0, st, xq, wq, acc, *d, P, Q);
    }
    if (stage) launch_dequant(acc, out_len, sA, sB, static_cast<float *>(out), out_mode == 2, st);
    return nparts;
}

extern "C" size_t lpdt_qconv_fwd_f32_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) return 0;
    clear_error();
    return round_up(fwd_base_ws(d), 256) + (fwd_fusable(d, P, Q) ? 0 : round_up((size_t)d->N * P * Q * d->K * 4, 256));
}

extern "C" int lpdt_qconv_fwd(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, int32_t *acc, void *ws,
                              size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(xq && wq && acc, LPDT_EINVAL, "qconv_fwd: NULL tensor");
    LPDT_REQUIRE(aligned(acc, 4), LPDT_EINVAL, "qconv_fwd: acc must be 4-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_qconv_fwd_workspace_bytes(d));
    if (rc) return rc;
    conv_fwd_impl(d, P, Q, xq, wq, acc, 0, nullptr, nullptr, ws, as_stream(stream));
    return launch_status("lpdt_qconv_fwd");
}

extern "C" int lpdt_qconv_fwd_f32(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx, const float *sw,
                                  float *y, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(xq && wq && y && sx && sw, LPDT_EINVAL, "qconv_fwd_f32: NULL argument");
    LPDT_REQUIRE(aligned(y, 16), LPDT_EINVAL, "qconv_fwd_f32: y must be 16-byte aligned");
    // a misaligned operand forces the plain kernel, which stages its sums: ask for that room too
    const bool al = aligned(xq, 16) && aligned(wq, 16);
    const size_t need = al ? lpdt_qconv_fwd_f32_workspace_bytes(d)
                           : round_up(fwd_base_ws(d), 256) + round_up((size_t)d->N * P * Q * d->K * 4, 256);
    rc = check_ws(ws, ws_bytes, need);
    if (rc) return rc;
    conv_fwd_impl(d, P, Q, xq, wq, y, 1, sx, sw, ws, as_stream(stream));
    return launch_status("lpdt_qconv_fwd_f32");
}

extern "C" int lpdt_qconv_fwd_f32_add(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx, const float *sw,
                                      float *y, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(xq && wq && y && sx && sw, LPDT_EINVAL, "qconv_fwd_f32_add: NULL argument");
    LPDT_REQUIRE(aligned(y, 16), LPDT_EINVAL, "qconv_fwd_f32_add: y must be 16-byte aligned");
    // every shape may have to stage its sums here (the first-layer kernel cannot add): ask for that room
    const size_t need = round_up(fwd_base_ws(d), 256) + round_up((size_t)d->N * P * Q * d->K * 4, 256);
    const bool al = aligned(xq, 16) && aligned(wq, 16);
    const bool fused = al && fwd_fusable(d, P, Q) && !narrow_conv_supported(d, P, Q);
    rc = check_ws(ws, ws_bytes, fused ? lpdt_qconv_fwd_f32_workspace_bytes(d) : need);
    if (rc) return rc;
    conv_fwd_impl(d, P, Q, xq, wq, y, 2, sx, sw, ws, as_stream(stream));
    return launch_status("lpdt_qconv_fwd_f32_add");
}

extern "C" size_t lpdt_qconv_fwd_f32_add_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) return 0;
    clear_error();
    if (fwd_fusable(d, P, Q) && !narrow_conv_supported(d, P, Q)) return lpdt_qconv_fwd_f32_workspace_bytes(d);
    return round_up(fwd_base_ws(d), 256) + round_up((size_t)d->N * P * Q * d->K * 4, 256);
}

// Backward-data product; out_mode 2 adds to the gradient already in `out` (fan-out of a skip connection).
static size_t bwd_data_base_ws(const lpdt_conv_desc *d) { return round_up((size_t)d->K * d->R * d->S * d->C, 256); }
static bool bwd_data_vec(const lpdt_conv_desc *d, int P, int Q) { return igemm_bwd_data_supported(d, P, Q); }
static bool bwd_data_fusable(const lpdt_conv_desc *d, int P, int Q) {
    return bwd_data_vec(d, P, Q) && !igemm_bwd_data_is_split(d, P, Q);
}

// packed: the filter's transposed panels made earlier by lpdt_qconv_bwd_data_pack_filter (then wq is not read), else NULL
static int conv_bwd_data_impl(const lpdt_conv_desc *d, int P, int Q, const int8_t *gq, const int8_t *wq, const void *packed,
                              void *out, int out_mode, const float *sA, const float *sB, void *ws, hipStream_t st,
                              float *pabs = nullptr) {
    int nparts = 0;
    const size_t out_len = (size_t)d->N * d->H * d->W * d->C;
    if (small_linear(d) && wq) {
        launch_linear_small<1>(d, gq, wq, out, out_mode, sA, sB, st);
        return 0;
    }
    const bool al = aligned(gq, 16) && (packed || aligned(wq, 16));   // the matrix-core path loads both operands 16 bytes at a time
    const bool stage = out_mode != 0 && !(bwd_data_fusable(d, P, Q) && al);
    int32_t *acc = stage ? reinterpret_cast<int32_t *>(static_cast<char *>(ws) + bwd_data_base_ws(d)) : static_cast<int32_t *>(out);
    const int mode = stage ? 0 : out_mode;
    if (bwd_data_vec(d, P, Q) && al) {
        if (!packed) launch_igemm_pack_bwd_filter(d, P, Q, wq, ws, st);
        if (pabs && mode != 0) nparts = igemm_bwd_data_absmax_parts(d, P, Q);
        launch_igemm_bwd_data(d, P, Q, gq, packed ? packed : ws, acc, mode, sA, sB, st, nparts > 0 ? pabs : nullptr);
    } else {
        hipLaunchKernelGGL(conv_bwd_data_plain_kernel, dim3(blocks_for(out_len)), dim3(kCThreads), 0, st, gq, wq, acc, *d, P, Q);
    }
    if (stage) launch_dequant(acc, out_len, sA, sB, static_cast<float *>(out), out_mode == 2, st);
    return nparts;
}

extern "C" size_t lpdt_qconv_bwd_data_f32_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) return 0;
    clear_error();
    return bwd_data_base_ws(d) + (bwd_data_fusable(d, P, Q) ? 0 : round_up((size_t)d->N * d->H * d->W * d->C * 4, 256));
}

extern "C" int lpdt_qconv_bwd_data(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *wq, int32_t *dx, void *ws,
                                   size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(gq && wq && dx, LPDT_EINVAL, "qconv_bwd_data: NULL tensor");
    LPDT_REQUIRE(aligned(dx, 4), LPDT_EINVAL, "qconv_bwd_data: dx must be 4-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_qconv_bwd_data_workspace_bytes(d));
    if (rc) return rc;
    conv_bwd_data_impl(d, P, Q, gq, wq, nullptr, dx, 0, nullptr, nullptr, ws, as_stream(stream));
    return launch_status("lpdt_qconv_bwd_data");
}

extern "C" int lpdt_qconv_bwd_data_f32(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *wq, const float *sg,
                                       const float *sw, float *dx, int accumulate, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(gq && wq && dx && sg && sw, LPDT_EINVAL, "qconv_bwd_data_f32: NULL argument");
    LPDT_REQUIRE(aligned(dx, 16), LPDT_EINVAL, "qconv_bwd_data_f32: dx must be 16-byte aligned");
    const size_t need = aligned(gq, 16) && aligned(wq, 16) ? lpdt_qconv_bwd_data_f32_workspace_bytes(d)
                                        : bwd_data_base_ws(d) + round_up((size_t)d->N * d->H * d->W * d->C * 4, 256);
    rc = check_ws(ws, ws_bytes, need);
    if (rc) return rc;
    conv_bwd_data_impl(d, P, Q, gq, wq, nullptr, dx, accumulate ? 2 : 1, sg, sw, ws, as_stream(stream));
    return launch_status("lpdt_qconv_bwd_data_f32");
}

extern "C" size_t lpdt_qconv_bwd_data_packed_filter_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) { clear_error(); return 0; }
    return bwd_data_vec(d, P, Q) ? round_up(igemm_bwd_filter_panel_bytes(d), 256) : 0;
}

extern "C" int lpdt_qconv_bwd_data_pack_filter(const lpdt_conv_desc *d, const int8_t *wq, void *packed, size_t packed_bytes,
                                               void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(wq && packed, LPDT_EINVAL, "qconv_bwd_data_pack_filter: NULL argument");
    LPDT_REQUIRE(bwd_data_vec(d, P, Q), LPDT_EUNSUPPORTED, "qconv_bwd_data_pack_filter: this shape has no packed filter");
    LPDT_REQUIRE(aligned(wq, 16) && aligned(packed, 16), LPDT_EINVAL, "qconv_bwd_data_pack_filter: wq and packed must be 16-byte aligned");
    LPDT_REQUIRE(packed_bytes >= lpdt_qconv_bwd_data_packed_filter_bytes(d), LPDT_EWORKSPACE,
                 "qconv_bwd_data_pack_filter: packed needs %zu bytes, got %zu", lpdt_qconv_bwd_data_packed_filter_bytes(d), packed_bytes);
    launch_igemm_pack_bwd_filter(d, P, Q, wq, packed, as_stream(stream));
    return launch_status("lpdt_qconv_bwd_data_pack_filter");
}

extern "C" int lpdt_qconv_bwd_data_pack_filters(const lpdt_conv_desc *descs, int count, const int8_t *const *wq, void *const *packed,
                                                const size_t *packed_bytes, void *stream) {
    LPDT_REQUIRE(count >= 0, LPDT_EINVAL, "qconv_bwd_data_pack_filters: negative count");
    if (count == 0) return LPDT_OK;
    LPDT_REQUIRE(descs && wq && packed && packed_bytes, LPDT_EINVAL, "qconv_bwd_data_pack_filters: NULL argument");
    for (int i = 0; i < count; ++i) {     // every filter is checked before anything is launched
        const lpdt_conv_desc *d = descs + i;
        int P, Q;
        int rc = check_conv(d, &P, &Q);
        if (rc) return rc;
        LPDT_REQUIRE(wq[i] && packed[i], LPDT_EINVAL, "qconv_bwd_data_pack_filters: NULL filter %d", i);
        LPDT_REQUIRE(bwd_data_vec(d, P, Q), LPDT_EUNSUPPORTED, "qconv_bwd_data_pack_filters: filter %d's shape has no packed filter", i);
        LPDT_REQUIRE(aligned(wq[i], 16) && aligned(packed[i], 16), LPDT_EINVAL,
                     "qconv_bwd_data_pack_filters: wq and packed must be 16-byte aligned (filter %d)", i);
        LPDT_REQUIRE(packed_bytes[i] >= lpdt_qconv_bwd_data_packed_filter_bytes(d), LPDT_EWORKSPACE,
                     "qconv_bwd_data_pack_filters: packed[%d] needs %zu bytes, got %zu", i, lpdt_qconv_bwd_data_packed_filter_bytes(d),
                     packed_bytes[i]);
    }
    launch_igemm_pack_bwd_filters(descs, count, wq, packed, as_stream(stream));
    return launch_status("lpdt_qconv_bwd_data_pack_filters");
}

extern "C" int lpdt_qconv_bwd_data_f32_packed(const lpdt_conv_desc *d, const int8_t *gq, const void *packed, const float *sg,
                                              const float *sw, float *dx, int accumulate, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(gq && packed && dx && sg && sw, LPDT_EINVAL, "qconv_bwd_data_f32_packed: NULL argument");
    LPDT_REQUIRE(bwd_data_vec(d, P, Q), LPDT_EUNSUPPORTED, "qconv_bwd_data_f32_packed: this shape has no packed filter");
    LPDT_REQUIRE(aligned(dx, 16) && aligned(gq, 16) && aligned(packed, 16), LPDT_EINVAL,
                 "qconv_bwd_data_f32_packed: gq, packed and dx must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_qconv_bwd_data_f32_workspace_bytes(d));
    if (rc) return rc;
    conv_bwd_data_impl(d, P, Q, gq, nullptr, packed, dx, accumulate ? 2 : 1, sg, sw, ws, as_stream(stream));
    return launch_status("lpdt_qconv_bwd_data_f32_packed");
}

// ---- products that also hand over max |result| (for a quantizer that follows with no normalisation layer between) ----
static size_t absmax_tail_bytes(int parts) {
    const int scratch = absmax_scratch_floats();
    return round_up((size_t)(parts > scratch ? parts : scratch) * sizeof(float), 256);
}
static size_t fwd_f32_any_ws(const lpdt_conv_desc *d, int P, int Q) {   // room lpdt_qconv_fwd_f32 may need, aligned operands or not
    return round_up(fwd_base_ws(d), 256) + round_up((size_t)d->N * P * Q * d->K * 4, 256);
}
static size_t bwd_data_f32_any_ws(const lpdt_conv_desc *d) {
    return bwd_data_base_ws(d) + round_up((size_t)d->N * d->H * d->W * d->C * 4, 256);
}

extern "C" size_t lpdt_qconv_fwd_f32_absmax_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) { clear_error(); return 0; }
    const int parts = fwd_vec(d, P, Q) ? igemm_fwd_absmax_parts(d, P, Q) : 0;
    return fwd_f32_any_ws(d, P, Q) + absmax_tail_bytes(parts);
}

extern "C" int lpdt_qconv_fwd_f32_absmax(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx,
                                         const float *sw, float *y, float *absmax_out, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(xq && wq && y && sx && sw && absmax_out, LPDT_EINVAL, "qconv_fwd_f32_absmax: NULL argument");
    LPDT_REQUIRE(aligned(y, 16) && aligned(absmax_out, 4), LPDT_EINVAL, "qconv_fwd_f32_absmax: y must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_qconv_fwd_f32_absmax_workspace_bytes(d));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    float *tail = reinterpret_cast<float *>(static_cast<char *>(ws) + fwd_f32_any_ws(d, P, Q));
    const int nparts = conv_fwd_impl(d, P, Q, xq, wq, y, 1, sx, sw, ws, st, tail);
    if (nparts > 0) launch_absmax_fold(tail, nparts, absmax_out, st);
    else launch_absmax(y, (size_t)d->N * P * Q * d->K, tail, absmax_out, st);
    return launch_status("lpdt_qconv_fwd_f32_absmax");
}

extern "C" size_t lpdt_qconv_bwd_data_f32_absmax_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) { clear_error(); return 0; }
    const int parts = bwd_data_vec(d, P, Q) ? igemm_bwd_data_absmax_parts(d, P, Q) : 0;
    return bwd_data_f32_any_ws(d) + absmax_tail_bytes(parts);
}

extern "C" int lpdt_qconv_bwd_data_f32_absmax(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *wq, const void *packed,
                                              const float *sg, const float *sw, float *dx, int accumulate, float *absmax_out,
                                              void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(gq && (wq || packed) && dx && sg && sw && absmax_out, LPDT_EINVAL, "qconv_bwd_data_f32_absmax: NULL argument");
    LPDT_REQUIRE(aligned(dx, 16) && aligned(absmax_out, 4), LPDT_EINVAL, "qconv_bwd_data_f32_absmax: dx must be 16-byte aligned");
    if (packed)
        LPDT_REQUIRE(bwd_data_vec(d, P, Q) && aligned(packed, 16) && aligned(gq, 16), LPDT_EINVAL,
                     "qconv_bwd_data_f32_absmax: a packed filter needs a shape that has one and 16-byte aligned gq, packed");
    rc = check_ws(ws, ws_bytes, lpdt_qconv_bwd_data_f32_absmax_workspace_bytes(d));
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    float *tail = reinterpret_cast<float *>(static_cast<char *>(ws) + bwd_data_f32_any_ws(d));
    const int nparts = conv_bwd_data_impl(d, P, Q, gq, packed ? nullptr : wq, packed, dx, accumulate ? 2 : 1, sg, sw, ws, st, tail);
    if (nparts > 0) launch_absmax_fold(tail, nparts, absmax_out, st);
    else launch_absmax(dx, (size_t)d->N * d->H * d->W * d->C, tail, absmax_out, st);
    return launch_status("lpdt_qconv_bwd_data_f32_absmax");
}

// Weight gradient.  Which kernel runs: first-layer path, rectangle-stepped kernel (partial tiles + reduction), the
// flattened-pixel kernel (1x1 spatial maps, large halos) or the plain kernel.  Only the rectangle kernel can apply
// the dequantizing scale itself; the others stage int32 sums in the workspace for the _f32 entry point.
// A pointwise product (1x1 filter, stride 1, no padding: linear layers, transformer-shaped GEMMs) does not care which
// image a pixel belongs to: seen as ONE image of 1 x (N*H*W) pixels it fills the rectangle-stepped kernel's 32-pixel steps
// whatever the real spatial size (a linear layer has H = W = 1).
static lpdt_conv_desc wgrad_view(const lpdt_conv_desc *d, int *P, int *Q) {
    lpdt_conv_desc v = *d;
    const long long pix = (long long)d->N * d->H * d->W;
    if (d->R == 1 && d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 && d->pad_w == 0 && pix <= 0x7fffffffLL) {
        v.N = 1; v.H = 1; v.W = (int)pix;
        *P = 1; *Q = (int)pix;
    }
    return v;
}

static bool wgrad_uses_rect(const lpdt_conv_desc *d, int P, int Q, WgradRectPlan *pl) {
    return !narrow_conv_supported(d, P, Q) && wgrad_rect_plan(d, P, Q, pl);
}

static size_t bwd_weight_base_ws(const lpdt_conv_desc *d0, int P, int Q) {
    const lpdt_conv_desc view = wgrad_view(d0, &P, &Q), *d = &view;
    WgradRectPlan pl;
    WgradRowsPlan rows;
    if (narrow_conv_supported(d, P, Q)) return round_up(narrow_wgrad_workspace(d), 256);
    // (partial tiles: the mode with more blocks needs more room, and the mode may change between query and call)
    if (wgrad_rows_plan(d, P, Q, &rows, 0)) {
        const size_t alone = rows.partial_bytes;
        wgrad_rows_plan(d, P, Q, &rows, 1);
        return alone > rows.partial_bytes ? alone : rows.partial_bytes;
    }
    WgradGemmPlan gemm;
    if (wgrad_gemm_plan(d, P, Q, &gemm)) return gemm.partial_bytes;
    if (wgrad_rect_plan(d, P, Q, &pl, 0)) {
        const size_t alone = pl.partial_bytes;
        wgrad_rect_plan(d, P, Q, &pl, 1);
        return alone > pl.partial_bytes ? alone : pl.partial_bytes;
    }
    if (wgrad_gemm_taps_plan(d, P, Q, &gemm)) return gemm.partial_bytes;
    return 0;
}

static void conv_bwd_weight_impl(const lpdt_conv_desc *d0, int P, int Q, const int8_t *gq, const int8_t *xq, void *out, int out_mode,
                                 const float *sA, const float *sB, void *ws, hipStream_t st) {
    if (small_linear(d0)) {
        launch_linear_small<2>(d0, gq, xq, out, out_mode, sA, sB, st);
        return;
    }
    const lpdt_conv_desc view = wgrad_view(d0, &P, &Q), *d = &view;
    const size_t wlen = (size_t)d->K * d->R * d->S * d->C;
    const long long M = (long long)d->N * P * Q;
    WgradRectPlan pl;
    WgradRowsPlan rows;
    if (aligned(gq, 16) && aligned(xq, 16) && !narrow_conv_supported(d, P, Q) && wgrad_rows_plan(d, P, Q, &rows)) {
        launch_wgrad_rows(d, P, Q, rows, gq, xq, out, out_mode, sA, sB, ws, st);
        return;
    }
    WgradGemmPlan gemm;
    if (aligned(gq, 16) && aligned(xq, 16) && wgrad_gemm_plan(d, P, Q, &gemm)) {
        launch_wgrad_gemm(d, gemm, gq, xq, out, out_mode, sA, sB, ws, st);
        return;
    }
    if (aligned(gq, 16) && aligned(xq, 16) && wgrad_uses_rect(d, P, Q, &pl)) {
        launch_wgrad_rect(d, P, Q, pl, gq, xq, out, out_mode, sA, sB, ws, st);
        return;
    }
    if (aligned(gq, 16) && aligned(xq, 16) && !narrow_conv_supported(d, P, Q) && wgrad_gemm_taps_plan(d, P, Q, &gemm)) {
        launch_wgrad_gemm(d, gemm, gq, xq, out, out_mode, sA, sB, ws, st);
        return;
    }
    if (narrow_conv_supported(d, P, Q) && aligned(gq, 16)) {
        launch_narrow_wgrad(d, P, Q, gq, xq, out, out_mode, sA, sB, ws, st);
        return;
    }
    int32_t *dw = out_mode ? reinterpret_cast<int32_t *>(static_cast<char *>(ws) + bwd_weight_base_ws(d, P, Q)) : static_cast<int32_t *>(out);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks_for(wlen, 1024)), dim3(kCThreads), 0, st, dw, wlen);
    if (d->K % 16 == 0 && d->C % 16 == 0 && same_stride_pad(d) && aligned(gq, 16) && aligned(xq, 16)) {
        WgradParams p = {};
        p.g = gq; p.x = xq; p.dw = dw;
        p.M = (int)M; p.K = d->K; p.C = d->C; p.H = d->H; p.W = d->W; p.P = P; p.Q = Q;
        p.R = d->R; p.S = d->S; p.stride = d->stride_h; p.pad = d->pad_h;
        p.tiles_k = (d->K + 63) / 64;
        const int tiles_c = (d->C + 63) / 64;
        p.chunks = (int)((M + 31) / 32);
        const int ntaps = d->R * d->S;
        const int tg = ntaps == 1 ? 1 : 9;
        const int groups = (ntaps + tg - 1) / tg;
        const long long base_blocks = (long long)p.tiles_k * tiles_c * groups;
        long long splits = (1024 + base_blocks - 1) / base_blocks;  // aim at >= 4 blocks per CU
        if (splits > p.chunks / 8) splits = p.chunks / 8;             // but at least 8 steps per block
        if (splits < 1) splits = 1;
        p.chunks_per_split = (int)((p.chunks + splits - 1) / splits);
        splits = (p.chunks + p.chunks_per_split - 1) / p.chunks_per_split;
        const dim3 grid((unsigned)(p.tiles_k * tiles_c), (unsigned)groups, (unsigned)splits);
        if (tg == 1) hipLaunchKernelGGL(wgrad_kernel<1>, grid, dim3(kCThreads), 0, st, p);
        else hipLaunchKernelGGL(wgrad_kernel<9>, grid, dim3(kCThreads), 0, st, p);
    } else {
        long long slices = (M + 4095) / 4096;
        if (slices > 1024) slices = 1024;
        const int pix = (int)((M + slices - 1) / slices);
        slices = (M + pix - 1) / pix;
        hipLaunchKernelGGL(conv_bwd_weight_plain_kernel, dim3((unsigned)((wlen + kCThreads - 1) / kCThreads), (unsigned)slices),
                           dim3(kCThreads), 0, st, gq, xq, dw, *d, P, Q, pix);
    }
    if (out_mode) launch_dequant(dw, wlen, sA, sB, static_cast<float *>(out), false, st);
}

extern "C" size_t lpdt_qconv_bwd_weight_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) { clear_error(); return 0; }
    return bwd_weight_base_ws(d, P, Q);
}

extern "C" size_t lpdt_qconv_bwd_weight_f32_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) { clear_error(); return 0; }
    // room for staged int32 sums as well, so that a misaligned operand (which rules out the fused kernel) still fits
    return bwd_weight_base_ws(d, P, Q) + round_up((size_t)d->K * d->R * d->S * d->C * 4, 256);
}

extern "C" int lpdt_qconv_bwd_weight(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *xq, int32_t *dw, void *ws,
                                     size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(gq && xq && dw, LPDT_EINVAL, "qconv_bwd_weight: NULL tensor");
    LPDT_REQUIRE(aligned(dw, 4), LPDT_EINVAL, "qconv_bwd_weight: dw must be 4-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_qconv_bwd_weight_workspace_bytes(d));
    if (rc) return rc;
    conv_bwd_weight_impl(d, P, Q, gq, xq, dw, 0, nullptr, nullptr, ws, as_stream(stream));
    return launch_status("lpdt_qconv_bwd_weight");
}

extern "C" int lpdt_qconv_bwd_weight_f32(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *xq, const float *sg,
                                         const float *sx, float *dw, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(gq && xq && dw && sg && sx, LPDT_EINVAL, "qconv_bwd_weight_f32: NULL argument");
    LPDT_REQUIRE(aligned(dw, 16), LPDT_EINVAL, "qconv_bwd_weight_f32: dw must be 16-byte aligned");
    rc = check_ws(ws, ws_bytes, lpdt_qconv_bwd_weight_f32_workspace_bytes(d));
    if (rc) return rc;
    conv_bwd_weight_impl(d, P, Q, gq, xq, dw, 1, sg, sx, ws, as_stream(stream));
    return launch_status("lpdt_qconv_bwd_weight_f32");
}

// ---------------------------------------------------------------- convolution -> Range-EvoNorm -> quantizer
static bool chain_fused(const lpdt_conv_desc *d, int P, int Q, int groups) {
    return !small_linear(d) && ren_chain_supported(d->K, groups) && igemm_fwd_stats_supported(d, P, Q);
}

extern "C" size_t lpdt_qconv_ren_fwd_q_workspace_bytes(const lpdt_conv_desc *d, int groups) {
    int P, Q;
    if (check_conv(d, &P, &Q)) { clear_error(); return 0; }
    if (chain_fused(d, P, Q, groups)) return ren_chain_ws_bytes(d->N, d->K, groups);
    const size_t conv = lpdt_qconv_fwd_f32_add_workspace_bytes(d), ren = lpdt_range_evonorm_fwd_q_workspace_bytes(d->N, P, Q, d->K, groups);
    return conv > ren ? conv : ren;
}

extern "C" int lpdt_qconv_ren_fwd_q(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx, const float *sw,
                                    int accumulate, int groups, const float *v, const float *gamma, const float *beta, float eps,
                                    float *y, float *z, int8_t *q, float *scale, float *range_out, int32_t *argmax_out,
                                    int32_t *argmin_out, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(xq && wq && sx && sw && v && gamma && beta && y && q && scale && range_out && argmax_out && argmin_out, LPDT_EINVAL,
                 "qconv_ren_fwd_q: NULL argument");
    LPDT_REQUIRE(eps >= 0.0f, LPDT_EINVAL, "qconv_ren_fwd_q: eps must be >= 0");
    LPDT_REQUIRE(groups > 0 && d->K % groups == 0 && d->K / groups >= 2, LPDT_EUNSUPPORTED,
                 "qconv_ren_fwd_q: groups must divide K with at least 2 channels per group");
    LPDT_REQUIRE(aligned(y, 16) && aligned(z, 16) && aligned(q, 4) && aligned(scale, 4), LPDT_EINVAL,
                 "qconv_ren_fwd_q: y and z must be 16-byte aligned, q and scale 4-byte aligned");
    hipStream_t st = as_stream(stream);
    if (chain_fused(d, P, Q, groups) && aligned(xq, 16) && aligned(wq, 16)) {
        rc = check_ws(ws, ws_bytes, ren_chain_ws_bytes(d->N, d->K, groups));
        if (rc) return rc;
        unsigned *cstats = ren_chain_begin(d->N, d->K, groups, ws, st);
        launch_igemm_fwd_stats(d, P, Q, xq, wq, y, accumulate ? 2 : 1, sx, sw, cstats, v, st);
        ren_chain_finish(y, d->N, P, Q, d->K, groups, v, gamma, beta, eps, q, scale, z, range_out, argmax_out, argmin_out, ws, st);
        return launch_status("lpdt_qconv_ren_fwd_q");
    }
    // any other shape: the two calls this one stands for
    rc = accumulate ? lpdt_qconv_fwd_f32_add(d, xq, wq, sx, sw, y, ws, ws_bytes, stream) : lpdt_qconv_fwd_f32(d, xq, wq, sx, sw, y, ws, ws_bytes, stream);
    if (rc) return rc;
    return lpdt_range_evonorm_fwd_q(y, d->N, P, Q, d->K, groups, v, gamma, beta, eps, q, scale, z, range_out, argmax_out, argmin_out,
                                    ws, ws_bytes, stream);
}

// ---------------------------------------------------------------- which kernel a call takes
extern "C" int lpdt_qconv_set_wgrad_beside(int beside) {
    set_wgrad_beside(beside);
    return LPDT_OK;
}

extern "C" int lpdt_qconv_kernel_id(const lpdt_conv_desc *d0, int product) {
    int P, Q;
    int rc = check_conv(d0, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(product >= 0 && product <= 3, LPDT_EINVAL,
                 "qconv_kernel_id: product must be 0 (forward), 1 (backward-data), 2 (backward-weight) or 3 (forward inside lpdt_qconv_ren_fwd_q)");
    if (small_linear(d0)) return 3;
    if (product == 3) {   // the statistics ride in the epilogue wherever the shape allows (two channels per group assumed)
        if (chain_fused(d0, P, Q, d0->K / 2)) return 20 + igemm_fwd_kernel_id(d0, P, Q);
        product = 0;
    }
    if (product == 0) {
        if (narrow_conv_supported(d0, P, Q)) return 1;
        return fwd_vec(d0, P, Q) ? igemm_fwd_kernel_id(d0, P, Q) : 0;
    }
    if (product == 1) return bwd_data_vec(d0, P, Q) ? igemm_bwd_data_kernel_id(d0, P, Q) : 0;
    const lpdt_conv_desc view = wgrad_view(d0, &P, &Q), *d = &view;
    WgradRectPlan pl;
    WgradRowsPlan rows;
    if (!narrow_conv_supported(d, P, Q) && wgrad_rows_plan(d, P, Q, &rows)) return 60;  // row-tile kernel
    WgradGemmPlan gemm;
    if (wgrad_gemm_plan(d, P, Q, &gemm)) return 62;                                       // 256 x 256 GEMM tiles
    if (wgrad_uses_rect(d, P, Q, &pl)) {
        // 30 + tile (0: 32 x 64, 1: 64 x 64, 2: 128 x 128) + 4 for 64-pixel steps + 8 for two wave groups per block
        return 30 + (pl.kt == 128 ? 2 : pl.kt == 64 ? 1 : 0) + (pl.ks == 2 ? 4 : 0) + (pl.ng == 2 ? 8 : 0);
    }
    if (!narrow_conv_supported(d, P, Q) && wgrad_gemm_taps_plan(d, P, Q, &gemm)) return 63;   // the same, one tap per block
    if (narrow_conv_supported(d, P, Q)) return 1;
    if (d->K % 16 == 0 && d->C % 16 == 0 && same_stride_pad(d)) return 2;
    return 0;
}
