// Weight gradient of a convolution on int8 codes, rectangle-stepped variant:
//   dw[k][r][s][c] = sum over output pixels (n, oy, ox) of g[n,oy,ox,k] * x[n, oy*st + r - pad, ox*st + s - pad, c]
//
// One K-step of the reduction is a small RECTANGLE of <= 32 output pixels of one image (ch rows x cw columns), so
// the input pixels all R*S taps need form one halo patch ((ch-1)*st+R) x ((cw-1)*st+S).  The block copies that patch
// and the gradient tile into LDS once per step, in their natural [pixel][channel] order, and every tap's MFMA operand
// is read from it with the transposing LDS load (ds_read_b64_tr_b8): a tap is a constant LDS offset.  Compared with
// staging one shifted copy per tap this moves ~2.4x fewer bytes through the global-load path for a 3x3 filter.
// A block accumulates all taps (up to 9) of a 64 x 64 (output x input channel) tile over its share of the steps and
// writes its sums as ONE plain partial tile; a second kernel adds the partial tiles (exact integers: order-free) and applies the
// dequantizing scale when asked.  No atomics, no zero fill, bit-reproducible.
#include "qconv_internal.h"

namespace lpdt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kRow = 96;        // LDS bytes per pixel: 64 channels + 32 pad (8 rows tile the 64 banks)
constexpr int kItems = 4;       // 16-byte items per thread and step (256 threads: up to 1024 items)

struct WgradRectParams {
    const int8_t *g;            // [N][P][Q][K]
    const int8_t *x;            // [N][H][W][C]
    int32_t *partial;           // [splits][K][R*S][C]
    int N, K, C, H, W, P, Q, R, S, stride, pad;
    int ch, cw, ncy, ncx;       // rectangle and rectangles per image
    int PHp, PWp;               // halo patch size in pixels
    int steps, steps_per_split;
    int tiles_k;
    long long out_len;
};

template <int TG>
__global__ __launch_bounds__(256, 2) void wgrad_rect_kernel(const WgradRectParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int patch_px = p.PHp * p.PWp;
    const int buf_bytes = (32 + patch_px) * kRow;

    const int t = threadIdx.x, lane = t % 64, wave = t / 64;
    const int k0 = (blockIdx.x % p.tiles_k) * 64, c0 = (blockIdx.x / p.tiles_k) * 64;
    const int tap0 = blockIdx.y * TG, ntaps = p.R * p.S;
    const int step_begin = blockIdx.z * p.steps_per_split;
    const int step_end = min(p.steps, step_begin + p.steps_per_split);
    const int spi = p.ncy * p.ncx;

    // this thread's load items: id < 128: gradient (slot id/4, granule id%4); else patch pixel (id-128)/4
    int kind[kItems], ia[kItems], ib[kItems], gran[kItems], dst[kItems];
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int id = t + 256 * j;
        gran[j] = (id % 4) * 16;
        if (id < 128) {
            const int slot = id / 4;
            kind[j] = 0; ia[j] = slot / p.cw; ib[j] = slot % p.cw;          // row, column inside the rectangle
            dst[j] = slot * kRow + gran[j];
        } else if ((id - 128) / 4 < patch_px) {
            const int pp = (id - 128) / 4;
            kind[j] = 1; ia[j] = pp / p.PWp; ib[j] = pp % p.PWp;           // row, column inside the patch
            dst[j] = (32 + pp) * kRow + gran[j];
        } else {
            kind[j] = 2; ia[j] = ib[j] = dst[j] = 0;
        }
    }

    v4i stage[kItems];
    auto load_items = [&](int step) {
        const int n = step / spi, rem = step - n * spi;
        const int cy = rem / p.ncx, cx = rem - cy * p.ncx;
        const int oy0 = cy * p.ch, ox0 = cx * p.cw;
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            v4i v = {0, 0, 0, 0};
            if (kind[j] == 0) {
                const int oy = oy0 + ia[j], ox = ox0 + ib[j];
                if (ia[j] < p.ch && oy < p.P && ox < p.Q && k0 + gran[j] < p.K)
                    v = *reinterpret_cast<const v4i *>(p.g + ((size_t)(n * p.P + oy) * p.Q + ox) * p.K + k0 + gran[j]);
            } else if (kind[j] == 1) {
                const int iy = oy0 * p.stride - p.pad + ia[j], ix = ox0 * p.stride - p.pad + ib[j];
                if (iy >= 0 && iy < p.H && ix >= 0 && ix < p.W && c0 + gran[j] < p.C)
                    v = *reinterpret_cast<const v4i *>(p.x + ((size_t)(n * p.H + iy) * p.W + ix) * p.C + c0 + gran[j]);
            }
            stage[j] = v;
        }
    };
    auto store_items = [&](int buf) {
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            if (kind[j] != 2) *reinterpret_cast<v4i *>(lds + buf * buf_bytes + dst[j]) = stage[j];
    };

    v16i acc[TG];
#pragma unroll
    for (int i = 0; i < TG; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;

    // Transposing LDS read: in each block of 16 lanes, source lane j supplies 8 bytes and result lane i receives byte
    // (i%8) of source lanes i/8, i/8+2, ...  With source lane j reading pixel slot j/2 at channel offset 8*(j%2),
    // result lane i holds channel i of 8 pixel slots: the MFMA operand.  Slot -> patch pixel is this lane's business.
    const int ti = wave / 2, tj = wave % 2;
    const int blk = lane / 16, j16 = lane % 16;
    const int src_ch = 16 * (blk % 2) + 8 * (j16 % 2);
    int a_off[2], b_off[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int slot = 16 * (blk / 2) + 8 * h + j16 / 2;
        a_off[h] = slot * kRow + 32 * ti + src_ch;
        const int pr = slot / p.cw, pc = slot - pr * p.cw;
        const int pix = pr < p.ch ? (pr * p.stride) * p.PWp + pc * p.stride : 0;  // empty slots meet zero gradient rows
        b_off[h] = (32 + pix) * kRow + 32 * tj + src_ch;
    }
    int tapoff[TG];
#pragma unroll
    for (int i = 0; i < TG; ++i) {
        const int tap = min(tap0 + i, ntaps - 1);
        tapoff[i] = ((tap / p.S) * p.PWp + tap % p.S) * kRow;
    }
    typedef __attribute__((address_space(3))) v2i lds_v2i;

    if (step_begin < step_end) {
        load_items(step_begin);
        store_items(0);
    }
    __syncthreads();
    for (int st = step_begin; st < step_end; ++st) {
        const int buf = (st - step_begin) & 1;
        const bool more = st + 1 < step_end;
        if (more) load_items(st + 1);
        unsigned char *base = lds + buf * buf_bytes;
        const v2i a_lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off[0]));
        const v2i a_hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off[1]));
        const v4i a = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
#pragma unroll
        for (int i = 0; i < TG; ++i) {
            if (tap0 + i < ntaps) {
                const v2i b_lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off[0] + tapoff[i]));
                const v2i b_hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off[1] + tapoff[i]));
                const v4i b = {b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
            }
        }
        if (more) store_items(buf ^ 1);
        __syncthreads();
    }

    int32_t *out = p.partial + (size_t)blockIdx.z * p.out_len;
    const int c = c0 + 32 * tj + lane % 32;
#pragma unroll
    for (int i = 0; i < TG; ++i) {
        const int tap = tap0 + i;
        if (tap < ntaps && c < p.C) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + 32 * ti + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                if (k < p.K) out[((size_t)k * ntaps + tap) * p.C + c] = acc[i][r];
            }
        }
    }
}

// out[i] = sum over splits of partial[z][i] (exact integers: any order gives the same bits); as int32, or as fp32
// times the scale product.  32 outputs x 8 split lanes per block so that the loads of one sum run in parallel.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const int32_t *__restrict__ partial, long long out_len, int splits,
                                                           int32_t *__restrict__ out, int out_mode, const float *sA,
                                                           const float *sB) {
    __shared__ int sm[8][32];
    const int o = threadIdx.x % 32, zl = threadIdx.x / 32;
    const long long i = (long long)blockIdx.x * 32 + o;
    int s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    if (i < out_len) {
        int z = zl;
        for (; z + 24 < splits; z += 32) {
            s0 += partial[(size_t)z * out_len + i];
            s1 += partial[(size_t)(z + 8) * out_len + i];
            s2 += partial[(size_t)(z + 16) * out_len + i];
            s3 += partial[(size_t)(z + 24) * out_len + i];
        }
        for (; z < splits; z += 8) s0 += partial[(size_t)z * out_len + i];
    }
    sm[zl][o] = s0 + s1 + s2 + s3;
    __syncthreads();
    if (zl == 0 && i < out_len) {
        int s = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) s += sm[k][o];
        if (out_mode) reinterpret_cast<float *>(out)[i] = __fmul_rn(*sA, *sB) * (float)s;
        else out[i] = s;
    }
}

bool wgrad_rect_plan(const lpdt_conv_desc *d, int P, int Q, WgradRectPlan *pl) {
    if (d->K % 16 || d->C % 16 || d->stride_h != d->stride_w || d->pad_h != d->pad_w) return false;
    if (P * Q < 16) return false;  // tiny maps: rectangles cannot be filled from one image
    const int st = d->stride_h;
    pl->cw = Q >= 32 ? 32 : Q;
    pl->ch = 32 / pl->cw;
    if (pl->ch > P) pl->ch = P;
    if (pl->ch < 1) pl->ch = 1;
    pl->ncx = (Q + pl->cw - 1) / pl->cw;
    pl->ncy = (P + pl->ch - 1) / pl->ch;
    pl->PHp = (pl->ch - 1) * st + d->R;
    pl->PWp = (pl->cw - 1) * st + d->S;
    if (pl->PHp * pl->PWp * 4 + 128 > kItems * 256) return false;
    const long long steps = (long long)d->N * pl->ncy * pl->ncx;
    if (steps > 0x7fffffffLL || steps * 32 * 6 / 10 > (long long)d->N * P * Q) return false;  // < 60% of the slots used
    pl->steps = (int)steps;
    const int ntaps = d->R * d->S;
    pl->tg = ntaps == 1 ? 1 : 9;
    pl->groups = (ntaps + pl->tg - 1) / pl->tg;
    pl->tiles_k = (d->K + 63) / 64;
    pl->tiles_c = (d->C + 63) / 64;
    const long long base = (long long)pl->tiles_k * pl->tiles_c * pl->groups;
    long long splits = (512 + base - 1) / base;
    if (splits > steps / 4) splits = steps / 4;
    if (splits < 1) splits = 1;
    pl->steps_per_split = (int)((steps + splits - 1) / splits);
    pl->splits = (int)((steps + pl->steps_per_split - 1) / pl->steps_per_split);
    pl->out_len = (long long)d->K * ntaps * d->C;
    pl->partial_bytes = round_up((size_t)pl->splits * pl->out_len * sizeof(int32_t), 256);
    pl->lds = 2 * (size_t)(32 + pl->PHp * pl->PWp) * kRow;
    return pl->lds <= 64 * 1024;
}

void launch_wgrad_rect(const lpdt_conv_desc *d, int P, int Q, const WgradRectPlan &pl, const int8_t *g, const int8_t *x,
                       void *out, int out_mode, const float *sA, const float *sB, void *partial, hipStream_t st) {
    WgradRectParams p = {};
    p.g = g; p.x = x; p.partial = static_cast<int32_t *>(partial);
    p.N = d->N; p.K = d->K; p.C = d->C; p.H = d->H; p.W = d->W; p.P = P; p.Q = Q;
    p.R = d->R; p.S = d->S; p.stride = d->stride_h; p.pad = d->pad_h;
    p.ch = pl.ch; p.cw = pl.cw; p.ncy = pl.ncy; p.ncx = pl.ncx; p.PHp = pl.PHp; p.PWp = pl.PWp;
    p.steps = pl.steps; p.steps_per_split = pl.steps_per_split; p.tiles_k = pl.tiles_k; p.out_len = pl.out_len;
    const dim3 grid((unsigned)(pl.tiles_k * pl.tiles_c), (unsigned)pl.groups, (unsigned)pl.splits);
    if (pl.tg == 1) hipLaunchKernelGGL(wgrad_rect_kernel<1>, grid, dim3(256), pl.lds, st, p);
    else hipLaunchKernelGGL(wgrad_rect_kernel<9>, grid, dim3(256), pl.lds, st, p);
    const long long rb = (pl.out_len + 31) / 32;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)rb), dim3(256), 0, st, p.partial, pl.out_len, pl.splits,
                       static_cast<int32_t *>(out), out_mode, sA, sB);
}

}  // namespace lpdt
