// Weight gradient from a 16-bit copy of the layer gradient (Section 3, gradient bifurcation: the weight gradient
// keeps a floating-point error signal while the layer gradient is passed on in 8 bits):
//   dw[k][r][s][c] = sx * sum over output pixels of bf16(g)[n,oy,ox,k] * xq[n, oy*st + r - pad, ox*st + s - pad, c]
// g in bfloat16, x as the saved int8 codes (exact in bfloat16: |code| <= 127), fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x16_bf16).  Same rectangle-stepped scheme as the int8 kernel: a step is a rectangle of <= 32
// output pixels of one image; the gradient tile and the input halo patch go to LDS in [pixel][channel] order (the
// patch converted to bfloat16 on the way in) and every tap's operand is read from the patch with the transposing
// LDS load for 16-bit elements (ds_read_b64_tr_b16).  A block accumulates the taps of a 32 x 64 (k x c) tile over
// its share of the steps and writes one partial tile; a second kernel adds the partial tiles in a fixed order and
// applies sx.  fp32 sums depend on the order of accumulation, which is fixed: results are run-to-run identical.
#include "qconv_internal.h"
#include <type_traits>

namespace lpdt {

namespace {

typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kRowG = 96;    // LDS bytes per rectangle slot: 32 k x 2 B + 32 pad
constexpr int kRowX = 160;   // LDS bytes per patch pixel: 64 c x 2 B + 32 pad
constexpr int kItems = 4;    // 16-byte global loads per thread and step
constexpr unsigned kBeyond = 0x80000000u;

struct Params {
    const uint16_t *g;          // bf16 [N][P][Q][K]
    const int8_t *x;            // [N][H][W][C]
    float *partial;             // [splits][K][R*S][C]
    unsigned g_bytes, x_bytes;
    int N, K, C, H, W, P, Q, R, S, stride, pad;
    int ch, cw, ncy, ncx, PHp, PWp;
    int steps, steps_per_split, tiles_k;
    long long out_len;
};

template <int N, typename F>
__device__ __forceinline__ void static_for(F f) {
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>());
    }
}

// 4 int8 codes (one dword) -> 4 bfloat16 patterns (two dwords); exact
__device__ __forceinline__ void codes_to_bf16(unsigned w, unsigned &lo, unsigned &hi) {
    const unsigned b0 = __float_as_uint((float)(int)(signed char)(w)) >> 16;
    const unsigned b1 = __float_as_uint((float)(int)(signed char)(w >> 8)) >> 16;
    const unsigned b2 = __float_as_uint((float)(int)(signed char)(w >> 16)) >> 16;
    const unsigned b3 = __float_as_uint((float)(int)(signed char)(w >> 24)) >> 16;
    lo = b0 | (b1 << 16);
    hi = b2 | (b3 << 16);
}

// TG = taps per block (the filter's taps are dealt to blockIdx.y in groups of TG); the 4 waves = 2 channel halves x 2
// tap parities.  PF = steps of loads in flight in registers.
template <int TG, int PF>
__global__ __launch_bounds__(256, 2) void wgrad_bf16_kernel(const Params p) {
    constexpr int NA = (TG + 1) / 2;  // taps per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int patch_px = p.PHp * p.PWp;
    const int buf_bytes = 32 * kRowG + patch_px * kRowX;

    const int t = threadIdx.x, lane = t % 64, wave = t / 64;
    const int k0 = (blockIdx.x % p.tiles_k) * 32, c0 = (blockIdx.x / p.tiles_k) * 64;
    const int tap0 = blockIdx.y * TG, ntaps = p.R * p.S;
    const int step_begin = blockIdx.z * p.steps_per_split;
    const int step_end = min(p.steps, step_begin + p.steps_per_split);
    const int nsteps = (step_end - step_begin + PF - 1) / PF * PF;

    // load items: id < 128: gradient (slot id/4, 8 bf16 = granule id%4); else patch pixel (id-128)/4, 16 codes
    const __amdgpu_buffer_rsrc_t rs_g = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.g), 0, (int)p.g_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0, (int)p.x_bytes, 0x00020000);
    bool is_g[kItems];
    int ia[kItems], ib[kItems], soff[kItems], dst[kItems];
    unsigned lim_y[kItems], lim_x[kItems];
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int id = t + 256 * j;
        is_g[j] = (wave * 64 + 256 * j) < 128;  // whole waves
        if (is_g[j]) {
            const int slot = id / 4, gran = id % 4;
            ia[j] = slot / p.cw; ib[j] = slot % p.cw;
            const bool ok = ia[j] < p.ch && k0 + gran * 8 < p.K;
            lim_y[j] = ok ? (unsigned)p.P : 0u; lim_x[j] = (unsigned)p.Q;
            soff[j] = ((ia[j] * p.Q + ib[j]) * p.K + k0 + gran * 8) * 2;
            dst[j] = slot * kRowG + gran * 16;
        } else {
            const int pp = (id - 128) / 4, gran = (id - 128) % 4;
            ia[j] = pp / p.PWp; ib[j] = pp % p.PWp;
            const bool ok = pp < patch_px && c0 + gran * 16 < p.C;
            lim_y[j] = ok ? (unsigned)p.H : 0u; lim_x[j] = (unsigned)p.W;
            soff[j] = (ia[j] * p.W + ib[j]) * p.C + c0 + gran * 16;
            dst[j] = ok ? 32 * kRowG + pp * kRowX + gran * 32 : -1;
        }
    }
    const int spi = p.ncy * p.ncx;
    int ld_n = step_begin / spi, ld_cy = (step_begin - ld_n * spi) / p.ncx, ld_cx = step_begin - ld_n * spi - ld_cy * p.ncx;
    int ld_left = step_end - step_begin;

    v4u stage[PF][kItems];
    auto load_items = [&](auto slot_tag) {
        constexpr int SL = decltype(slot_tag)::value;
        const bool live = ld_left > 0;
        const int oy0 = ld_cy * p.ch, ox0 = ld_cx * p.cw;
        const int iy0 = oy0 * p.stride - p.pad, ix0 = ox0 * p.stride - p.pad;
        const int base_g = ((ld_n * p.P + oy0) * p.Q + ox0) * p.K * 2;
        const int base_x = ((ld_n * p.H + iy0) * p.W + ix0) * p.C;
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            const int y = (is_g[j] ? oy0 : iy0) + ia[j], x = (is_g[j] ? ox0 : ix0) + ib[j];
            const bool ok = live && (unsigned)y < lim_y[j] && (unsigned)x < lim_x[j];
            const unsigned off = ok ? (unsigned)((is_g[j] ? base_g : base_x) + soff[j]) : kBeyond;
            stage[SL][j] = __builtin_amdgcn_raw_buffer_load_b128(is_g[j] ? rs_g : rs_x, off, 0, 0);
        }
        --ld_left;
        if (++ld_cx == p.ncx) { ld_cx = 0; if (++ld_cy == p.ncy) { ld_cy = 0; ++ld_n; } }
    };
    auto store_items = [&](auto slot_tag, int buf) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            if (dst[j] < 0) continue;
            unsigned char *at = lds + buf * buf_bytes + dst[j];
            if (is_g[j]) {
                *reinterpret_cast<v4u *>(at) = stage[SL][j];
            } else {
                unsigned w[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) codes_to_bf16(stage[SL][j][e], w[2 * e], w[2 * e + 1]);
                const v4u lo = {w[0], w[1], w[2], w[3]}, hi = {w[4], w[5], w[6], w[7]};
                *reinterpret_cast<v4u *>(at) = lo;
                *reinterpret_cast<v4u *>(at + 16) = hi;
            }
        }
    };

    v16f acc[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;

    // Transposing LDS read for 16-bit elements: in each block of 16 lanes, source lane j supplies 4 elements (8 bytes)
    // and result lane i receives element i%4 of source lanes i/4, i/4+4, i/4+8, i/4+12.  With source lane j reading pixel
    // j/4 at channel offset 4*(j%4), result lane i holds channel i of 4 consecutive pixels.  An MFMA operand (row l%32,
    // reduction elements 8*(l/32)..+7) is two such reads: 16-lane block b covers channels 16*(b%2).., pixels 8*(b/2)..
    const int tj = wave % 2, tw = wave / 2;
    const int blk = lane / 16, j16 = lane % 16;
    const int src_ch = (16 * (blk % 2) + 4 * (j16 % 4)) * 2;  // bytes
    int a_off[2][2], b_off[2][2];                             // [k-group of 16 pixels][half of the lane's 8 pixels]
#pragma unroll
    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int slot = 16 * kg + 8 * (blk / 2) + 4 * h + j16 / 4;
            a_off[kg][h] = slot * kRowG + src_ch;
            const int pr = slot / p.cw, pc = slot - pr * p.cw;
            const int pix = pr < p.ch ? (pr * p.stride) * p.PWp + pc * p.stride : 0;  // empty slots meet zero gradient rows
            b_off[kg][h] = 32 * kRowG + pix * kRowX + 64 * tj + src_ch;
        }
    int tapoff[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int tap = min(tap0 + tw + 2 * i, ntaps - 1);
        tapoff[i] = ((tap / p.S) * p.PWp + tap % p.S) * kRowX;
    }
    typedef __attribute__((address_space(3))) v4s lds_v4s;
    auto operand = [&](const unsigned char *at0, const unsigned char *at1) {
        const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s *)at0);
        const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s *)at1);
        union { short s[8]; v8bf v; } u;
#pragma unroll
        for (int e = 0; e < 4; ++e) { u.s[e] = lo[e]; u.s[4 + e] = hi[e]; }
        return u.v;
    };

    static_assert(PF % 2 == 0, "the LDS buffer of a step is a compile-time constant only for an even PF");
    static_for<PF>([&](auto s) { load_items(s); });
    store_items(std::integral_constant<int, 0>(), 0);
    __syncthreads();
    for (int round = 0; round < nsteps; round += PF) {
        static_for<PF>([&](auto u) {
            constexpr int U = decltype(u)::value;
            constexpr int buf = U & 1;
            load_items(u);
            unsigned char *base = lds + buf * buf_bytes;
#pragma unroll
            for (int kg = 0; kg < 2; ++kg) {
                const v8bf a = operand(base + a_off[kg][0], base + a_off[kg][1]);
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    if (tw + 2 * i < TG && tap0 + tw + 2 * i < ntaps) {
                        const v8bf b = operand(base + b_off[kg][0] + tapoff[i], base + b_off[kg][1] + tapoff[i]);
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
                    }
                }
            }
            store_items(std::integral_constant<int, (U + 1) % PF>(), buf ^ 1);
            __syncthreads();
        });
    }

    float *out = p.partial + (size_t)blockIdx.z * p.out_len;
    const int c = c0 + 32 * tj + lane % 32;
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int tap = tap0 + tw + 2 * i;
        if (tw + 2 * i < TG && tap < ntaps && c < p.C) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                if (k < p.K) out[((size_t)k * ntaps + tap) * p.C + c] = acc[i][r];
            }
        }
    }
}

// dw[i] = sx * sum over splits of partial[z][i], the splits added in a fixed order (8 interleaved chains, then those)
template <int V>
__global__ __launch_bounds__(256) void wgrad_bf16_reduce_kernel(const float *__restrict__ partial, long long out_len, int splits,
                                                                const float *__restrict__ sx, float *__restrict__ dw) {
    typedef float vf __attribute__((ext_vector_type(V)));
    __shared__ float sm[8][32][V];
    const int o = threadIdx.x % 32, zl = threadIdx.x / 32;
    const long long i = ((long long)blockIdx.x * 32 + o) * V;
    float s[V];
#pragma unroll
    for (int e = 0; e < V; ++e) s[e] = 0.0f;
    if (i < out_len)
        for (int z = zl; z < splits; z += 8) {
            if constexpr (V == 4) {
                const vf t = *reinterpret_cast<const vf *>(partial + (size_t)z * out_len + i);
#pragma unroll
                for (int e = 0; e < V; ++e) s[e] += t[e];
            } else {
                s[0] += partial[(size_t)z * out_len + i];
            }
        }
#pragma unroll
    for (int e = 0; e < V; ++e) sm[zl][o][e] = s[e];
    __syncthreads();
    if (zl == 0 && i < out_len) {
        const float sc = *sx;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float tsum = sm[0][o][e];
#pragma unroll
            for (int k = 1; k < 8; ++k) tsum += sm[k][o][e];
            dw[i + e] = sc * tsum;
        }
    }
}

// any shape: one thread per filter element and pixel slice (pixels in order inside a slice); the slices are partial
// tiles for the reduction kernel above
__global__ __launch_bounds__(256) void wgrad_bf16_plain_kernel(const uint16_t *__restrict__ g, const int8_t *__restrict__ x,
                                                               float *__restrict__ partial, lpdt_conv_desc d, int P, int Q,
                                                               int pix_per_slice) {
    const int total = d.K * d.R * d.S * d.C;
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int c = o % d.C;
    const int s = (o / d.C) % d.S;
    const int r = (o / (d.C * d.S)) % d.R;
    const int k = o / (d.C * d.S * d.R);
    const long long M = (long long)d.N * P * Q;
    const long long m0 = (long long)blockIdx.y * pix_per_slice, m1 = min(M, m0 + pix_per_slice);
    float sum = 0.0f;
    for (long long m = m0; m < m1; ++m) {
        const int q = (int)(m % Q), pp = (int)((m / Q) % P), n = (int)(m / ((long long)P * Q));
        const int h = pp * d.stride_h + r - d.pad_h, w = q * d.stride_w + s - d.pad_w;
        if (h < 0 || h >= d.H || w < 0 || w >= d.W) continue;
        const float gv = __uint_as_float((unsigned)g[(size_t)m * d.K + k] << 16);
        sum += gv * (float)x[(((size_t)n * d.H + h) * d.W + w) * d.C + c];
    }
    partial[(size_t)blockIdx.y * total + o] = sum;
}

__global__ __launch_bounds__(256) void to_bf16_kernel(const float *__restrict__ x, size_t len, uint16_t *__restrict__ y) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < len; i += (size_t)gridDim.x * 256) {
        unsigned u = __float_as_uint(x[i]);
        u += 0x7FFFu + ((u >> 16) & 1u);  // nearest, ties to even
        y[i] = (uint16_t)(u >> 16);
    }
}

struct Plan {
    int ch, cw, ncy, ncx, PHp, PWp, steps, steps_per_split, splits, tg, groups, tiles_k, tiles_c;
    long long out_len;
    size_t partial_bytes, lds;
};

bool make_plan(const lpdt_conv_desc *d0, int P, int Q, Plan *pl, lpdt_conv_desc *view) {
    lpdt_conv_desc d = *d0;
    const long long pix = (long long)d.N * d.H * d.W;
    if (d.R == 1 && d.S == 1 && d.stride_h == 1 && d.stride_w == 1 && d.pad_h == 0 && d.pad_w == 0 && pix <= 0x7fffffffLL) {
        d.N = 1; d.H = 1; d.W = (int)pix;  // a pointwise product: one long image (see the int8 kernel)
        P = 1; Q = (int)pix;
    }
    *view = d;
    if (d.K % 8 || d.C % 16 || d.stride_h != d.stride_w || d.pad_h != d.pad_w) return false;
    const size_t lim = ((size_t)1 << 31) - 4096;
    if ((size_t)d.N * P * Q * d.K * 2 >= lim || (size_t)d.N * d.H * d.W * d.C >= lim) return false;
    if (P * Q < 16) return false;
    const int st = d.stride_h, ntaps = d.R * d.S;
    pl->cw = Q >= 32 ? 32 : Q;
    pl->ch = 32 / pl->cw;
    if (pl->ch > P) pl->ch = P;
    if (pl->ch < 1) pl->ch = 1;
    pl->ncx = (Q + pl->cw - 1) / pl->cw;
    pl->ncy = (P + pl->ch - 1) / pl->ch;
    pl->PHp = (pl->ch - 1) * st + d.R;
    pl->PWp = (pl->cw - 1) * st + d.S;
    if (pl->PHp * pl->PWp * 4 + 128 > kItems * 256) return false;
    const long long steps = (long long)d.N * pl->ncy * pl->ncx;
    if (steps > 0x7fffffffLL || steps * 32 * 6 / 10 > (long long)d.N * P * Q) return false;
    pl->steps = (int)steps;
    pl->tg = ntaps == 1 ? 1 : 9;
    pl->groups = (ntaps + pl->tg - 1) / pl->tg;
    pl->tiles_k = (d.K + 31) / 32;
    pl->tiles_c = (d.C + 63) / 64;
    const long long base = (long long)pl->tiles_k * pl->tiles_c * pl->groups;
    long long splits = (512 + base - 1) / base;
    if (splits > steps / 4) splits = steps / 4;
    if (splits < 1) splits = 1;
    pl->steps_per_split = (int)((steps + splits - 1) / splits);
    pl->splits = (int)((steps + pl->steps_per_split - 1) / pl->steps_per_split);
    pl->out_len = (long long)d.K * ntaps * d.C;
    pl->partial_bytes = round_up((size_t)pl->splits * pl->out_len * sizeof(float), 256);
    pl->lds = 2 * ((size_t)32 * kRowG + (size_t)pl->PHp * pl->PWp * kRowX);
    return pl->lds <= 96 * 1024;
}

// any-shape path: pixel slices of >= 256 pixels, at most 1024 of them, at most ~64 MB of partial tiles
struct PlainPlan { int slices, pix; size_t bytes; };
PlainPlan plain_plan(const lpdt_conv_desc *d, int P, int Q) {
    const long long M = (long long)d->N * P * Q, total = (long long)d->K * d->R * d->S * d->C;
    long long slices = (M + 255) / 256;
    if (slices > 1024) slices = 1024;
    const long long cap = (64ll << 20) / (total * 4) > 1 ? (64ll << 20) / (total * 4) : 1;
    if (slices > cap) slices = cap;
    PlainPlan pp;
    pp.pix = (int)((M + slices - 1) / slices);
    pp.slices = (int)((M + pp.pix - 1) / pp.pix);
    pp.bytes = round_up((size_t)pp.slices * total * 4, 256);
    return pp;
}

template <typename K>
void launch_tiled(K kernel, const dim3 &grid, size_t lds, hipStream_t st, const Params &p) {
    if (lds > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kernel, grid, dim3(256), lds, st, p);
}

}  // namespace

}  // namespace lpdt

using namespace lpdt;

extern "C" int lpdt_to_bf16(const float *x, size_t len, uint16_t *y, void *stream) {
    LPDT_REQUIRE(x && y, LPDT_EINVAL, "to_bf16: NULL argument");
    LPDT_REQUIRE(len > 0, LPDT_EUNSUPPORTED, "to_bf16: len must be positive");
    size_t b = (len + 1023) / 1024;
    if (b > 8192) b = 8192;
    hipLaunchKernelGGL(to_bf16_kernel, dim3((unsigned)b), dim3(256), 0, as_stream(stream), x, len, y);
    return launch_status("lpdt_to_bf16");
}

extern "C" size_t lpdt_qconv_bwd_weight_bf16_workspace_bytes(const lpdt_conv_desc *d) {
    int P, Q;
    if (check_conv(d, &P, &Q)) { clear_error(); return 0; }
    Plan pl;
    lpdt_conv_desc view;
    const size_t plain = plain_plan(d, P, Q).bytes;  // also taken when an operand is not 16-byte aligned
    return make_plan(d, P, Q, &pl, &view) && pl.partial_bytes > plain ? pl.partial_bytes : plain;
}

extern "C" int lpdt_qconv_bwd_weight_bf16(const lpdt_conv_desc *d, const uint16_t *g16, const int8_t *xq, const float *sx,
                                          float *dw, void *ws, size_t ws_bytes, void *stream) {
    int P, Q;
    int rc = check_conv(d, &P, &Q);
    if (rc) return rc;
    LPDT_REQUIRE(g16 && xq && sx && dw, LPDT_EINVAL, "qconv_bwd_weight_bf16: NULL argument");
    LPDT_REQUIRE(aligned(dw, 16) && aligned(g16, 2), LPDT_EINVAL, "qconv_bwd_weight_bf16: dw must be 16-byte, g16 2-byte aligned");
    hipStream_t st = as_stream(stream);
    Plan pl;
    lpdt_conv_desc v;
    if (make_plan(d, P, Q, &pl, &v) && aligned(g16, 16) && aligned(xq, 16)) {
        rc = check_ws(ws, ws_bytes, pl.partial_bytes);
        if (rc) return rc;
        Params p = {};
        p.g = g16; p.x = xq; p.partial = static_cast<float *>(ws);
        const int Pv = conv_out(v.H, v.pad_h, v.R, v.stride_h), Qv = conv_out(v.W, v.pad_w, v.S, v.stride_w);
        p.g_bytes = (unsigned)((size_t)v.N * Pv * Qv * v.K * 2); p.x_bytes = (unsigned)((size_t)v.N * v.H * v.W * v.C);
        p.N = v.N; p.K = v.K; p.C = v.C; p.H = v.H; p.W = v.W; p.P = Pv; p.Q = Qv;
        p.R = v.R; p.S = v.S; p.stride = v.stride_h; p.pad = v.pad_h;
        p.ch = pl.ch; p.cw = pl.cw; p.ncy = pl.ncy; p.ncx = pl.ncx; p.PHp = pl.PHp; p.PWp = pl.PWp;
        p.steps = pl.steps; p.steps_per_split = pl.steps_per_split; p.tiles_k = pl.tiles_k; p.out_len = pl.out_len;
        const dim3 grid((unsigned)(pl.tiles_k * pl.tiles_c), (unsigned)pl.groups, (unsigned)pl.splits);
        if (pl.tg == 1) launch_tiled(wgrad_bf16_kernel<1, 2>, grid, pl.lds, st, p);
        else launch_tiled(wgrad_bf16_kernel<9, 2>, grid, pl.lds, st, p);
        const long long rb = (pl.out_len / 4 + 31) / 32;
        hipLaunchKernelGGL(wgrad_bf16_reduce_kernel<4>, dim3((unsigned)rb), dim3(256), 0, st, p.partial, pl.out_len, pl.splits, sx, dw);
    } else {
        const int total = d->K * d->R * d->S * d->C;
        const PlainPlan pp = plain_plan(d, P, Q);
        rc = check_ws(ws, ws_bytes, pp.bytes);
        if (rc) return rc;
        float *partial = static_cast<float *>(ws);
        hipLaunchKernelGGL(wgrad_bf16_plain_kernel, dim3((unsigned)((total + 255) / 256), (unsigned)pp.slices), dim3(256), 0, st, g16, xq,
                           partial, *d, P, Q, pp.pix);
        hipLaunchKernelGGL(wgrad_bf16_reduce_kernel<1>, dim3((unsigned)((total + 31) / 32)), dim3(256), 0, st, partial, (long long)total,
                           pp.slices, sx, dw);
    }
    return launch_status("lpdt_qconv_bwd_weight_bf16");
}
