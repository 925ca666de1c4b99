// Weight gradient of a convolution on int8 codes, rectangle-stepped variant:
//   dw[k][r][s][c] = sum over output pixels (n, oy, ox) of g[n,oy,ox,k] * x[n, oy*st + r - pad, ox*st + s - pad, c]
//
// One K-step of the reduction is a small RECTANGLE of <= 32 or 64 output pixels of one image (ch rows x cw columns), so
// the input pixels all R*S taps need form one halo patch ((ch-1)*st+R) x ((cw-1)*st+S).  The block copies that patch
// and the gradient tile into LDS once per step, in their natural [pixel][channel] order, and every tap's MFMA operand
// is read from it with the transposing LDS load (ds_read_b64_tr_b8): a tap is a constant LDS offset.  Compared with
// staging one shifted copy per tap this moves ~2.4x fewer bytes through the global-load path for a 3x3 filter.
// A block accumulates all taps (up to 9) of a 32 x 64 or 64 x 64 (output x input channel) tile over its share of the steps and
// writes its sums as ONE plain partial tile; a second kernel adds the partial tiles (exact integers: order-free) and applies the
// dequantizing scale when asked.  No atomics, no zero fill, bit-reproducible.
#include "qconv_internal.h"
#include <atomic>
#include <type_traits>
#ifdef LPDT_TUNE
#include <cstdlib>
#endif

namespace lpdt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// LDS bytes per pixel = channels of the wider tile + 32 bytes of padding: with 96 or 160 bytes the 8 pixel rows one
// transposing read touches fall on 8 different groups of banks.
static constexpr int lds_row_bytes(int kt, int ct) { return (kt > ct ? kt : ct) <= 64 ? 96 : 160; }
constexpr int kItems = 4;       // 16-byte items per thread and step (256 threads: up to 1024 items)

struct WgradRectParams {
    const int8_t *g;            // [N][P][Q][K]
    const int8_t *x;            // [N][H][W][C]
    int32_t *partial;           // [splits][K][R*S][C]
    unsigned g_bytes, x_bytes;
    int N, K, C, H, W, P, Q, R, S, stride, pad;
    int ch, cw, ncy, ncx;       // rectangle and rectangles per image
    int PHp, PWp;               // halo patch size in pixels
    int steps, steps_per_split;
    int tiles_k;
    long long out_len;
};

template <int N, typename F>
__device__ __forceinline__ void static_for(F f) {
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>());
    }
}

constexpr unsigned kBeyond = 0x80000000u;  // a buffer offset no tensor reaches: such loads return zeros

// KT x CT = the block's (output x input channel) tile, 32, 64 or 128 each.  The 4 waves cover its 32 x 32 sub-tiles: with
// fewer than 4 of those they share out the taps (wave (ti, tj, tw) accumulates taps tw, tw + WT, ...), with 16 of them
// (128 x 128, single-tap filters only: GEMM-shaped linear layers) each wave owns SK x SC = 2 x 2 sub-tiles.
// PF = steps whose loads are in flight (in registers) ahead of the step being multiplied; the loop runs in rounds of PF
// steps without conditions, steps past the block's share load zeros.
// KS = 32-pixel groups per step: the rectangle has 32*KS slots, one barrier serves KS MFMAs per accumulator.
// NG = groups of 4 waves per block.  With NG = 2 the two groups work on two consecutive pixel splits, each with LDS
// buffers of its own, and add their sums through LDS before one of them writes the partial tile: half the partial
// tiles written and read back for the same number of waves on the chip.
template <int KT, int CT, int TG, int PF, int KS, int NG = 1>
__global__ __launch_bounds__(256 * NG, NG == 1 ? 2 : 1) void wgrad_rect_kernel(const WgradRectParams p) {
    constexpr int SLOTS = 32 * KS;
    constexpr int WK = KT / 32 > 2 ? 2 : KT / 32, WC = CT / 32 > 2 ? 2 : CT / 32, WT = 4 / (WK * WC);
    constexpr int SK = KT / 32 / WK, SC = CT / 32 / WC;   // sub-tiles per wave
    static_assert(SK * SC == 1 || TG == 1, "several sub-tiles per wave only for single-tap filters");
    constexpr int NA = SK * SC > 1 ? SK * SC : (TG + WT - 1) / WT;   // accumulators per wave: sub-tiles or taps
    constexpr int kRow = lds_row_bytes(KT, CT);
    constexpr int GK = KT / 16, GC = CT / 16;    // 16-byte granules per pixel of the two tiles
    static_assert(SLOTS * GK % 64 == 0, "an item index is gradient or patch for a whole wave");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];
    const int patch_px = p.PHp * p.PWp;
    const int buf_bytes = (SLOTS + patch_px) * kRow;

    const int grp = NG == 1 ? 0 : (int)threadIdx.x / 256;       // this thread's group of 4 waves
    unsigned char *lds = lds_all + grp * 2 * buf_bytes;
    const int t = threadIdx.x % 256, lane = t % 64, wave = t / 64;
    const int k0 = (blockIdx.x % p.tiles_k) * KT, c0 = (blockIdx.x / p.tiles_k) * CT;
    const int tap0 = blockIdx.y * TG, ntaps = p.R * p.S;
    const int step_begin = min(p.steps, (int)(blockIdx.z * NG + grp) * p.steps_per_split);
    const int step_end = min(p.steps, step_begin + p.steps_per_split);
    const int nsteps = (p.steps_per_split + PF - 1) / PF * PF;   // the same for every group: the barriers are shared

    // This thread's load items.  id < SLOTS*GK: gradient (rectangle slot id/GK, granule id%GK); else patch pixel
    // (id - SLOTS*GK)/GC.  Per item: position (ia, ib) inside the rectangle / patch, the image limits its position is
    // tested against, and the byte offset relative to the step's corner.  Whether an item is gradient or patch is the
    // same for all lanes of a wave, so the choice of tensor is scalar.
    const __amdgpu_buffer_rsrc_t rs_g = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.g), 0, (int)p.g_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0, (int)p.x_bytes, 0x00020000);
    bool is_g[kItems];
    int ia[kItems], ib[kItems], soff[kItems], dst[kItems];
    unsigned lim_y[kItems], lim_x[kItems];
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int id = t + 256 * j;
        is_g[j] = (wave * 64 + 256 * j) < SLOTS * GK;
        if (is_g[j]) {
            const int slot = id / GK, gran = (id % GK) * 16;
            ia[j] = slot / p.cw; ib[j] = slot % p.cw;
            const bool ok = ia[j] < p.ch && k0 + gran < p.K;
            lim_y[j] = ok ? (unsigned)p.P : 0u; lim_x[j] = (unsigned)p.Q;
            soff[j] = (ia[j] * p.Q + ib[j]) * p.K + k0 + gran;
            dst[j] = slot * kRow + gran;
        } else {
            const int pp = (id - SLOTS * GK) / GC, gran = ((id - SLOTS * GK) % GC) * 16;
            ia[j] = pp / p.PWp; ib[j] = pp % p.PWp;
            const bool ok = pp < patch_px && c0 + gran < p.C;
            lim_y[j] = ok ? (unsigned)p.H : 0u; lim_x[j] = (unsigned)p.W;
            soff[j] = (ia[j] * p.W + ib[j]) * p.C + c0 + gran;
            dst[j] = ok ? (SLOTS + pp) * kRow + gran : -1;
        }
    }

    // position of the next step to load: image n, rectangle (cy, cx)
    const int spi = p.ncy * p.ncx;
    int ld_n = step_begin / spi, ld_cy = (step_begin - ld_n * spi) / p.ncx, ld_cx = step_begin - ld_n * spi - ld_cy * p.ncx;
    int ld_left = step_end - step_begin;  // real steps not yet loaded

    v4u stage[PF][kItems];
    auto load_items = [&](auto slot_tag) {
        constexpr int SL = decltype(slot_tag)::value;
        const bool live = ld_left > 0;
        const int oy0 = ld_cy * p.ch, ox0 = ld_cx * p.cw;
        const int iy0 = oy0 * p.stride - p.pad, ix0 = ox0 * p.stride - p.pad;
        const int base_g = ((ld_n * p.P + oy0) * p.Q + ox0) * p.K;
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
        for (int j = 0; j < kItems; ++j)
            if (dst[j] >= 0) *reinterpret_cast<v4u *>(lds + buf * buf_bytes + dst[j]) = stage[SL][j];
    };

    v16i acc[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;

    // Transposing LDS read: in each block of 16 lanes, source lane j supplies 8 bytes and result lane i receives byte
    // (i%8) of source lanes i/8, i/8+2, ...  With source lane j reading pixel slot j/2 at channel offset 8*(j%2),
    // result lane i holds channel i of 8 pixel slots: the MFMA operand.  Slot -> patch pixel is this lane's business.
    const int ti = wave % WK, tj = (wave / WK) % WC, tw = wave / (WK * WC);
    const int blk = lane / 16, j16 = lane % 16;
    const int src_ch = 16 * (blk % 2) + 8 * (j16 % 2);
    int a_off[KS][2], b_off[KS][2];
#pragma unroll
    for (int g32 = 0; g32 < KS; ++g32)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int slot = 32 * g32 + 16 * (blk / 2) + 8 * h + j16 / 2;
            a_off[g32][h] = slot * kRow + 32 * ti * SK + src_ch;
            const int pr = slot / p.cw, pc = slot - pr * p.cw;
            const int pix = pr < p.ch ? (pr * p.stride) * p.PWp + pc * p.stride : 0;  // empty slots meet zero gradient rows
            b_off[g32][h] = (SLOTS + pix) * kRow + 32 * tj * SC + src_ch;
        }
    int tapoff[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int tap = min(tap0 + tw + WT * i, ntaps - 1);
        tapoff[i] = ((tap / p.S) * p.PWp + tap % p.S) * kRow;
    }
    typedef __attribute__((address_space(3))) v2i lds_v2i;

    static_assert(PF % 2 == 0, "the LDS buffer of a step is a compile-time constant only for an even PF");
    static_for<PF>([&](auto s) { load_items(s); });
    store_items(std::integral_constant<int, 0>(), 0);
    __syncthreads();
    for (int round = 0; round < nsteps; round += PF) {
        static_for<PF>([&](auto u) {
            constexpr int U = decltype(u)::value;
            constexpr int buf = U & 1;
            load_items(u);  // register slot U went to LDS before this step: refill it with the step PF ahead
            unsigned char *base = lds + buf * buf_bytes;
#pragma unroll
            for (int g32 = 0; g32 < KS; ++g32) {
                if constexpr (SK * SC > 1) {
                    v4i a[SK], b[SC];
#pragma unroll
                    for (int sk = 0; sk < SK; ++sk) {
                        const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off[g32][0] + 32 * sk));
                        const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off[g32][1] + 32 * sk));
                        a[sk] = v4i{lo[0], lo[1], hi[0], hi[1]};
                    }
#pragma unroll
                    for (int sc = 0; sc < SC; ++sc) {
                        const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off[g32][0] + 32 * sc));
                        const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off[g32][1] + 32 * sc));
                        b[sc] = v4i{lo[0], lo[1], hi[0], hi[1]};
                    }
#pragma unroll
                    for (int sk = 0; sk < SK; ++sk)
#pragma unroll
                        for (int sc = 0; sc < SC; ++sc)
                            acc[sk * SC + sc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[sk], b[sc], acc[sk * SC + sc], 0, 0, 0);
                } else {
                    const v2i a_lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off[g32][0]));
                    const v2i a_hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off[g32][1]));
                    const v4i a = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
#pragma unroll
                    for (int i = 0; i < NA; ++i) {
                        if (tw + WT * i < TG && tap0 + tw + WT * i < ntaps) {
                            const v2i b_lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off[g32][0] + tapoff[i]));
                            const v2i b_hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off[g32][1] + tapoff[i]));
                            const v4i b = {b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
                            acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
                        }
                    }
                }
            }
            store_items(std::integral_constant<int, (U + 1) % PF>(), buf ^ 1);
            __syncthreads();
        });
    }

    if constexpr (NG == 2) {
        // group 1 hands its sums over through LDS (the staging buffers are free: the loop ended with a barrier)
        int *dump = reinterpret_cast<int *>(lds_all);
        if (grp == 1) {
#pragma unroll
            for (int i = 0; i < NA; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) dump[((wave * NA + i) * 16 + r) * 64 + lane] = acc[i][r];
        }
        __syncthreads();
        if (grp == 1) return;
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] += dump[((wave * NA + i) * 16 + r) * 64 + lane];
    }
    int32_t *out = p.partial + (size_t)blockIdx.z * p.out_len;
    if constexpr (SK * SC > 1) {
#pragma unroll
        for (int sk = 0; sk < SK; ++sk)
#pragma unroll
            for (int sc = 0; sc < SC; ++sc) {
                const int c = c0 + 32 * (tj * SC + sc) + lane % 32;
                if (tap0 < ntaps && c < p.C) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int k = k0 + 32 * (ti * SK + sk) + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                        if (k < p.K) out[((size_t)k * ntaps + tap0) * p.C + c] = acc[sk * SC + sc][r];
                    }
                }
            }
    } else {
        const int c = c0 + 32 * tj + lane % 32;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int tap = tap0 + tw + WT * i;
            if (tw + WT * i < TG && tap < ntaps && c < p.C) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = k0 + 32 * ti + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                    if (k < p.K) out[((size_t)k * ntaps + tap) * p.C + c] = acc[i][r];
                }
            }
        }
    }
}

// out[i] = sum over splits of partial[z][i] (exact integers: any order gives the same bits); as int32, or as fp32
// times the scale product.  A block covers 256/ZL groups of 4 outputs (16-byte loads) with ZL split lanes each, so that
// the loads of one sum run in parallel; ZL follows the number of splits (few splits: every thread walks them all and a
// block covers 4 KiB of every partial tile; hundreds: 32 lanes, each with a handful of loads in flight).
// out_len is a multiple of 4 (K, C multiples of 16).
template <int ZL>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const int32_t *__restrict__ partial, long long out_len, int splits,
                                                           int32_t *__restrict__ out, int out_mode, const float *sA,
                                                           const float *sB) {
    constexpr int QB = 256 / ZL;
    __shared__ v4i sm[ZL][QB];
    const int o = threadIdx.x % QB, zl = threadIdx.x / QB;
    const long long i = ((long long)blockIdx.x * QB + o) * 4;
    v4i s0 = {0, 0, 0, 0}, s1 = s0, s2 = s0, s3 = s0;
    if (i < out_len) {
        int z = zl;
        for (; z + 3 * ZL < splits; z += 4 * ZL) {
            s0 += *reinterpret_cast<const v4i *>(partial + (size_t)z * out_len + i);
            s1 += *reinterpret_cast<const v4i *>(partial + (size_t)(z + ZL) * out_len + i);
            s2 += *reinterpret_cast<const v4i *>(partial + (size_t)(z + 2 * ZL) * out_len + i);
            s3 += *reinterpret_cast<const v4i *>(partial + (size_t)(z + 3 * ZL) * out_len + i);
        }
        for (; z < splits; z += ZL) s0 += *reinterpret_cast<const v4i *>(partial + (size_t)z * out_len + i);
    }
    v4i s = s0 + s1 + s2 + s3;
    if constexpr (ZL > 1) {
        sm[zl][o] = s;
        __syncthreads();
        if (zl != 0) return;
#pragma unroll
        for (int k = 1; k < ZL; ++k) s += sm[k][o];
    }
    if (i < out_len) {
        if (out_mode) {
            const float sc = __fmul_rn(*sA, *sB);
            float *f = reinterpret_cast<float *>(out) + i;
            f[0] = dequant_value(sc, s[0], 0.f, false); f[1] = dequant_value(sc, s[1], 0.f, false);
            f[2] = dequant_value(sc, s[2], 0.f, false); f[3] = dequant_value(sc, s[3], 0.f, false);
        } else {
            out[i] = s[0]; out[i + 1] = s[1]; out[i + 2] = s[2]; out[i + 3] = s[3];
        }
    }
}

static bool rect_plan_with(const lpdt_conv_desc *d, int P, int Q, int ks, WgradRectPlan *pl, int beside);

static std::atomic<int> g_wgrad_beside{0};
int wgrad_beside() { return g_wgrad_beside.load(std::memory_order_relaxed); }
void set_wgrad_beside(int v) { g_wgrad_beside.store(v ? 1 : 0, std::memory_order_relaxed); }

bool wgrad_rect_plan(const lpdt_conv_desc *d, int P, int Q, WgradRectPlan *pl, int beside) {
    if (beside < 0) beside = wgrad_beside();
    // 64-pixel steps (two MFMA k-groups per barrier) for multi-tap filters on maps that can fill them, when the halo
    // patch of such a step still fits the per-step load budget (stride-2 patches are four times larger); else 32.
    if (d->R * d->S > 1 && P * Q >= 64 && rect_plan_with(d, P, Q, 2, pl, beside)) return true;
    return rect_plan_with(d, P, Q, 1, pl, beside);
}

static bool rect_plan_with(const lpdt_conv_desc *d, int P, int Q, int ks, WgradRectPlan *pl, int beside) {
    if (d->K % 16 || d->C % 16 || d->stride_h != d->stride_w || d->pad_h != d->pad_w) return false;
    const size_t lim = ((size_t)1 << 31) - 4096;  // 32-bit buffer offsets
    if ((size_t)d->N * P * Q * d->K >= lim || (size_t)d->N * d->H * d->W * d->C >= lim) return false;
    if (P * Q < 16) return false;  // tiny maps: rectangles cannot be filled from one image
    const int st = d->stride_h;
    const int ntaps = d->R * d->S;
    pl->ks = ks;
    pl->cw = Q >= 32 ? 32 : Q;
    pl->ch = 32 * pl->ks / pl->cw;
    if (pl->ch > P) pl->ch = P;
    if (pl->ch < 1) pl->ch = 1;
    pl->ncx = (Q + pl->cw - 1) / pl->cw;
    pl->ncy = (P + pl->ch - 1) / pl->ch;
    pl->PHp = (pl->ch - 1) * st + d->R;
    pl->PWp = (pl->cw - 1) * st + d->S;
    const long long steps = (long long)d->N * pl->ncy * pl->ncx;
    if (steps > 0x7fffffffLL || steps * 32 * pl->ks * 6 / 10 > (long long)d->N * P * Q) return false;  // < 60% of the slots used
    pl->steps = (int)steps;
    pl->tg = ntaps == 1 ? 1 : 9;
    pl->groups = (ntaps + pl->tg - 1) / pl->tg;
    // Every block writes its tile once per split and the second kernel reads all of that back, so a smaller tile means
    // less traffic; it also means more steps per block.  Measured on the benchmark layers: 32 x 64 for multi-tap filters
    // (the waves share out the 9 taps), 64 x 64 for 1x1 filters.
    pl->kt = ntaps == 1 ? 64 : 32;
    pl->ct = 64;
    // GEMM-shaped single-tap products (both channel counts large): 128 x 128 tiles, 4x the MFMAs per staged byte
    if (ntaps == 1 && d->K >= 256 && d->C >= 256 && (long long)((d->K + 127) / 128) * ((d->C + 127) / 128) >= 32) pl->kt = pl->ct = 128;
    if (pl->PHp * pl->PWp * (pl->ct / 16) + 32 * pl->ks * (pl->kt / 16) > kItems * 256) return false;
    pl->tiles_k = (d->K + pl->kt - 1) / pl->kt;
    pl->tiles_c = (d->C + pl->ct - 1) / pl->ct;
    const long long base = (long long)pl->tiles_k * pl->tiles_c * pl->groups;
    // blocks wanted: 512 is the fastest on an idle chip; 256 when the caller has said that the product runs beside other
    // kernels (lpdt_qconv_set_wgrad_beside; measured in the ResNet-18 step, where it runs on a second stream: 128 +15 us,
    // 512 +20 us, 768 +27 us)
    long long target = beside ? 256 : 512;
#ifdef LPDT_TUNE
    if (const char *e = getenv("LPDT_WGRAD_BLOCKS")) target = atoi(e);
#endif
    long long splits = (target + base - 1) / base;
    if (splits > steps / 4) splits = steps / 4;
    if (splits < 1) splits = 1;
    pl->steps_per_split = (int)((steps + splits - 1) / splits);
    pl->splits = (int)((steps + pl->steps_per_split - 1) / pl->steps_per_split);
    pl->out_len = (long long)d->K * ntaps * d->C;
    pl->lds = 2 * (size_t)(32 * pl->ks + pl->PHp * pl->PWp) * lds_row_bytes(pl->kt, pl->ct);
    if (pl->lds > 64 * 1024) return false;
    // Two wave groups per block (see the kernel) for the multi-tap 32 x 64 tiles when there are splits to pair up
    pl->ng = (pl->tg == 9 && pl->kt == 32 && pl->ct == 64 && pl->splits >= 2) ? 2 : 1;
    if (pl->ng == 2) {
        const size_t dump = (size_t)4 * 5 * 16 * 64 * sizeof(int);   // 4 waves x 5 accumulators of 16 registers
        pl->lds = 2 * pl->lds > dump ? 2 * pl->lds : dump;
        pl->partials = (pl->splits + 1) / 2;
    } else {
        pl->partials = pl->splits;
    }
    pl->partial_bytes = round_up((size_t)pl->partials * pl->out_len * sizeof(int32_t), 256);
    return true;
}

void launch_wgrad_rect(const lpdt_conv_desc *d, int P, int Q, const WgradRectPlan &pl, const int8_t *g, const int8_t *x,
                       void *out, int out_mode, const float *sA, const float *sB, void *partial, hipStream_t st) {
    WgradRectParams p = {};
    p.g = g; p.x = x; p.partial = static_cast<int32_t *>(partial);
    p.g_bytes = (unsigned)((size_t)d->N * P * Q * d->K); p.x_bytes = (unsigned)((size_t)d->N * d->H * d->W * d->C);
    p.N = d->N; p.K = d->K; p.C = d->C; p.H = d->H; p.W = d->W; p.P = P; p.Q = Q;
    p.R = d->R; p.S = d->S; p.stride = d->stride_h; p.pad = d->pad_h;
    p.ch = pl.ch; p.cw = pl.cw; p.ncy = pl.ncy; p.ncx = pl.ncx; p.PHp = pl.PHp; p.PWp = pl.PWp;
    p.steps = pl.steps; p.steps_per_split = pl.steps_per_split; p.tiles_k = pl.tiles_k; p.out_len = pl.out_len;
    const dim3 grid((unsigned)(pl.tiles_k * pl.tiles_c), (unsigned)pl.groups, (unsigned)pl.partials);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, dim3(256), pl.lds, st, p); };
    auto go2 = [&](auto kernel) {   // two wave groups: 512 threads, possibly more than 64 KB of LDS
        if (pl.lds > 48 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds);
        hipLaunchKernelGGL(kernel, grid, dim3(512), pl.lds, st, p);
    };
    if (pl.ng == 2) {
        if (pl.ks == 2) go2(wgrad_rect_kernel<32, 64, 9, 2, 2, 2>);
        else go2(wgrad_rect_kernel<32, 64, 9, 2, 1, 2>);
    } else if (pl.kt == 128) {
        go(wgrad_rect_kernel<128, 128, 1, 4, 1>);
    } else if (pl.kt == 64 && pl.ct == 64) {
        if (pl.tg == 1) go(wgrad_rect_kernel<64, 64, 1, 4, 1>);
        else if (pl.ks == 2) go(wgrad_rect_kernel<64, 64, 9, 2, 2>);
        else go(wgrad_rect_kernel<64, 64, 9, 2, 1>);  // 9 accumulators: no registers for a deeper read-ahead
    } else {
        if (pl.tg == 1) go(wgrad_rect_kernel<32, 64, 1, 4, 1>);
        else if (pl.ks == 2) go(wgrad_rect_kernel<32, 64, 9, 2, 2>);
        else go(wgrad_rect_kernel<32, 64, 9, 2, 1>);
    }
    launch_wgrad_reduce(p.partial, pl.out_len, pl.partials, out, out_mode, sA, sB, st);
}

void launch_wgrad_reduce(const int32_t *partial, long long out_len, int splits, void *out, int out_mode, const float *sA,
                         const float *sB, hipStream_t st) {
    int zl = splits >= 64 ? 32 : splits >= 16 ? 8 : splits >= 8 ? 4 : 1;
#ifdef LPDT_TUNE
    if (const char *e = getenv("LPDT_REDUCE_ZL")) zl = atoi(e);
#endif
    const long long quads = out_len / 4;
    auto go = [&](auto kernel, int z) {
        const long long rb = (quads + 256 / z - 1) / (256 / z);
        hipLaunchKernelGGL(kernel, dim3((unsigned)rb), dim3(256), 0, st, partial, out_len, splits, static_cast<int32_t *>(out), out_mode, sA, sB);
    };
    if (zl >= 32) go(wgrad_reduce_kernel<32>, 32);
    else if (zl >= 8) go(wgrad_reduce_kernel<8>, 8);
    else if (zl >= 4) go(wgrad_reduce_kernel<4>, 4);
    else go(wgrad_reduce_kernel<1>, 1);
}

}  // namespace lpdt
