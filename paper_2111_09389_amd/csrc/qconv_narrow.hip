// First-layer convolutions: very few input channels (the RGB image), so one filter
// ROW (S taps x C channels <= 32 bytes) is one MFMA K-step instead of one tap.
//
// The int8 image is first copied into a zero-padded buffer, so every later access is
// in bounds and needs no mask.  For output pixel (n, oy, ox) and filter row r the
// operand is then the 32 contiguous bytes starting at xp[n][oy*stride + r][ox*stride][0]
// (bytes past S*C meet zero filter entries), read with byte-aligned 16-byte loads.
//   forward : filter rows live in registers for the whole kernel; each wave streams
//             32-pixel row blocks: R loads + R*ceil(K/32) MFMAs + the int32 store, which
//             is what bounds it (4 bytes written per output element).
//   weight gradient: dw[k][r][s*C+c] = sum_m g[m][k] * window(m, r)[s*C+c]; gradient tile
//             and window tile are staged in LDS in [pixel][byte] order and read with the
//             transposing LDS load, exactly as in the general weight-gradient kernel; one
//             filter row is one 32-column MFMA tile.
#include "qconv_internal.h"
#include <type_traits>

namespace lpdt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kNR = 8;  // filter rows supported

__device__ __forceinline__ v4i load16_any(const int8_t *p) {  // no alignment assumed
    v4i v;
    __builtin_memcpy(&v, p, 16);
    return v;
}

// q = m / d for m < 2^24 through one float multiply and a correction step
__device__ __forceinline__ int div24(int m, int d, float inv) {
    int q = (int)((float)m * inv);
    int r = m - q * d;
    if (r < 0) { --q; r += d; }
    if (r >= d) ++q;
    return q;
}

// xp[n][yy][xx][c] = x[n][yy-pad][xx-pad][c] inside the image, 0 in the border and in the slack after the last image.
// A padded row is the image row shifted by pad*C bytes between two runs of zeros, so a thread finds its 4 consecutive
// output bytes with one division (which padded row) and carries from there, and stores them as one word; the buffer is
// a multiple of 4 bytes long (total < 2^31).  Four bytes from inside one image row come from two aligned word loads.
__global__ void pad_image_kernel(const int8_t *__restrict__ x, int N, int H, int W, int C, int pad, int PH, int PW,
                                 int8_t *__restrict__ xp, unsigned total) {
    const unsigned nwords = (total + 3u) / 4u;
    const unsigned row_bytes = (unsigned)(PW * C), src_row = (unsigned)(W * C), shift = (unsigned)(pad * C);
    const size_t src_total = (size_t)N * H * src_row;
    for (unsigned q = blockIdx.x * blockDim.x + threadIdx.x; q < nwords; q += gridDim.x * blockDim.x) {
        const unsigned o = q * 4u;
        unsigned row = o / row_bytes, b = o - row * row_bytes;
        unsigned n = row / (unsigned)PH, yy = row - n * (unsigned)PH;
        {   // the common case, 4 bytes from inside one image row: two aligned word loads and a byte shift
            const unsigned iy = yy - (unsigned)pad, sb = b - shift;   // wrap to huge values outside the image
            const size_t at = ((size_t)n * H + iy) * src_row + sb;
            if (n < (unsigned)N && iy < (unsigned)H && b >= shift && sb + 3u < src_row && at + 8 <= src_total) {
                const uintptr_t addr = reinterpret_cast<uintptr_t>(x) + at;
                const unsigned *w = reinterpret_cast<const unsigned *>(addr & ~(uintptr_t)3);
                reinterpret_cast<unsigned *>(xp)[q] = __builtin_amdgcn_alignbyte(w[1], w[0], (unsigned)(addr & 3u));
                continue;
            }
        }
        unsigned word = 0u;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned iy = yy - (unsigned)pad, sb = b - shift;
            int8_t v = 0;
            if (n < (unsigned)N && iy < (unsigned)H && sb < src_row) v = x[((size_t)n * H + iy) * src_row + sb];
            word |= (unsigned)(uint8_t)v << (8 * k);
            if (++b == row_bytes) { b = 0; if (++yy == (unsigned)PH) { yy = 0; ++n; } }
        }
        reinterpret_cast<unsigned *>(xp)[q] = word;
    }
}

// wr[k][r][j] = w[k][r][j / C][j % C] for j < S*C, else 0   (32 bytes per filter row)
__global__ void pack_filter_rows_kernel(const int8_t *__restrict__ w, int K, int R, int SC, int8_t *__restrict__ wr) {
    const int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= K * R * 32) return;
    const int j = o % 32, kr = o / 32;
    wr[o] = j < SC ? w[(size_t)kr * SC + j] : (int8_t)0;
}

struct NarrowParams {
    const int8_t *xp;   // padded image [N][PH][PW][C] (+ slack)
    const int8_t *wr;   // packed filter rows [K][R][32]            (forward)
    const int8_t *g;    // gradient codes [M][K]                     (weight gradient)
    int32_t *out;       // forward: [M][K] (fp32 when out_mode != 0) ; weight gradient: one [K][R][S*C] partial per block
    int out_mode;       // forward only: 0 int32 sums, 1 fp32 sA*sB*sum
    int vec_out;        // forward only: out is 16-byte aligned (16-byte stores)
    const float *sA, *sB;
    int M, K, C, R, SC, stride, PH, PW, P, Q;
    float inv_pq, inv_q;
    int zero_off;       // weight gradient: offset in xp of 16 zero bytes
    int blocks_total;   // row blocks (forward) / 32-pixel steps (weight gradient)
    int steps_per_block;
};

// NR = filter rows multiplied (4 for R <= 4, 7 for R = 7, else 8).  Nothing in the row sequence depends on R or K at run time, so the
// accumulators stay in place between the MFMAs: rows past R hold zero weights and read row R-1 of the window again,
// channels past K hold zero weights.
template <int NR>
__global__ __launch_bounds__(256) void narrow_fwd_kernel(const NarrowParams p) {
    const int lane = threadIdx.x % 64, half = lane / 32;
    const int gwave = blockIdx.x * 4 + threadIdx.x / 64, nwaves = gridDim.x * 4;
    const int pq = p.P * p.Q;
    v4i b[NR][2];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const int n = lane % 32 + 32 * tn;
            b[r][tn] = v4i{0, 0, 0, 0};
            if (r < p.R && n < p.K) b[r][tn] = *reinterpret_cast<const v4i *>(p.wr + ((size_t)n * p.R + r) * 32 + 16 * half);
        }
    const int row_bytes = p.PW * p.C;
    const float scale = p.out_mode ? __fmul_rn(*p.sA, *p.sB) : 0.0f;
    for (int rb = gwave; rb < p.blocks_total; rb += nwaves) {
        const int m = min(rb * 32 + lane % 32, p.M - 1);
        const int n = div24(m, pq, p.inv_pq), rem = m - n * pq;
        const int oy = div24(rem, p.Q, p.inv_q), ox = rem - oy * p.Q;
        const int8_t *src = p.xp + ((size_t)(n * p.PH + oy * p.stride) * p.PW + ox * p.stride) * p.C + 16 * half;
        v16i acc[2];
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tn][i] = 0;
        v4i a[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) a[r] = load16_any(src + (size_t)min(r, p.R - 1) * row_bytes);
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            // the filter is the row operand: a lane ends with 4 consecutive output channels of ONE pixel (16-byte stores)
            acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[r][0], a[r], acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[r][1], a[r], acc[1], 0, 0, 0);
        }
        const int mm = rb * 32 + lane % 32;
        if (mm < p.M) {
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    const int ch = 32 * tn + 8 * qd + 4 * half;   // K is a multiple of 16: a quad is inside or outside
                    if (ch < p.K) {
                        int32_t *dst = p.out + (size_t)mm * p.K + ch;
                        if (!p.vec_out) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                if (p.out_mode) reinterpret_cast<float *>(dst)[e] = scale * (float)acc[tn][4 * qd + e];
                                else dst[e] = acc[tn][4 * qd + e];
                            }
                        } else if (p.out_mode)
                            *reinterpret_cast<float4 *>(dst) = make_float4(scale * (float)acc[tn][4 * qd], scale * (float)acc[tn][4 * qd + 1],
                                                                           scale * (float)acc[tn][4 * qd + 2], scale * (float)acc[tn][4 * qd + 3]);
                        else
                            *reinterpret_cast<int4 *>(dst) = make_int4(acc[tn][4 * qd], acc[tn][4 * qd + 1], acc[tn][4 * qd + 2], acc[tn][4 * qd + 3]);
                    }
                }
        }
    }
}

constexpr int kGS = 96;  // LDS bytes per pixel of the gradient tile (64 channels + pad)

template <int N, typename F>
__device__ __forceinline__ void narrow_static_for(F f) {
    if constexpr (N > 0) {
        narrow_static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>());
    }
}

// Weight gradient of the first layer.  Every wave works alone on its own run of 32-pixel steps, for the whole filter
// (2 channel tiles x NR filter rows = 2*NR MFMA tiles in its accumulators): it loads the step's gradient rows and window
// rows, passes them through its private LDS area to read them back transposed (pixels become the MFMA's reduction
// axis), and multiplies.  Nothing is shared between waves, so the loop has no barrier, and the next step's loads are in
// flight while this step is multiplied.  At the end the block's four waves add their sums up in LDS and write one copy
// of the filter gradient; a second launch sums the copies.  NR = 4 for R <= 4, 7 for R = 7, else 8: rows past R read row R-1 again
// and their sums are never stored.
template <int NR>
__global__ __launch_bounds__(256, 1) void narrow_wgrad_kernel(const NarrowParams p) {
    constexpr int XS = (NR == 7 ? 8 : NR) * 32 + 32;   // LDS bytes per pixel of the window tile (8 banks from pixel to pixel: the transposing reads meet no conflict; 7 rows keep the pitch of 8)
    constexpr int WAVE_BYTES = 32 * kGS + 32 * XS;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int t = threadIdx.x, lane = t % 64, wave = t / 64, half = lane / 32;
    unsigned char *const base = lds + wave * WAVE_BYTES;
    const int pq = p.P * p.Q, row_bytes = p.PW * p.C;
    const int gw = blockIdx.x * 4 + wave;
    const int step_begin = gw * p.steps_per_block, step_end = min(p.blocks_total, step_begin + p.steps_per_block);

    v16i acc[2][NR];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[kt][r][e] = 0;

    // loads of one step: 2 gradient items (pixel lane/4 + 16j, granule lane%4) and NR window items (pixel lane%32,
    // bytes 16*half.. of filter row min(r, R-1)).  Past the last pixel and past the wave's last step the gradient items read
    // zero bytes, so the loop below runs its steps in groups of D with no condition around the MFMAs.
    const bool g_ok = (lane % 4) * 16 < p.K;
    constexpr int D = 4;   // steps whose loads are in flight (in registers) ahead of the one being multiplied
    v4i gs[D][2], ws[D][NR];
    auto load_step = [&](auto slot_tag, int st) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int m = st * 32 + lane / 4 + 16 * j;
            const bool valid = g_ok && m < p.M && st < step_end;
            gs[SL][j] = load16_any(valid ? p.g + (size_t)m * p.K + (lane % 4) * 16 : p.xp + p.zero_off);
        }
        const int m = min(st * 32 + lane % 32, p.M - 1);
        const int n = div24(m, pq, p.inv_pq), rem = m - n * pq;
        const int oy = div24(rem, p.Q, p.inv_q), ox = rem - oy * p.Q;
        const int8_t *src = p.xp + ((size_t)(n * p.PH + oy * p.stride) * p.PW + ox * p.stride) * p.C + 16 * half;
#pragma unroll
        for (int r = 0; r < NR; ++r) ws[SL][r] = load16_any(src + (size_t)min(r, p.R - 1) * row_bytes);
    };
    auto store_step = [&](auto slot_tag) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int j = 0; j < 2; ++j) *reinterpret_cast<v4i *>(base + (lane / 4 + 16 * j) * kGS + (lane % 4) * 16) = gs[SL][j];
#pragma unroll
        for (int r = 0; r < NR; ++r) *reinterpret_cast<v4i *>(base + 32 * kGS + (lane % 32) * XS + r * 32 + 16 * half) = ws[SL][r];
    };
    // transposing LDS read: source lane j of a 16-lane block reads pixel j/2, byte offset 8*(j%2);
    // result lane i then holds byte column i of 8 pixels (see the general weight-gradient kernel)
    const int blk = lane / 16, j16 = lane % 16;
    const int src_px = 16 * (blk / 2) + j16 / 2, src_ch = 16 * (blk % 2) + 8 * (j16 % 2);
    const int a_off = src_px * kGS + src_ch;
    const int b_off = 32 * kGS + src_px * XS + src_ch;
    typedef __attribute__((address_space(3))) v2i lds_v2i;
    auto multiply = [&]() {
        v4i a[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off + 32 * kt));
            const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + a_off + 32 * kt + 8 * kGS));
            a[kt] = v4i{lo[0], lo[1], hi[0], hi[1]};
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off + r * 32));
            const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(base + b_off + r * 32 + 8 * XS));
            const v4i b = {lo[0], lo[1], hi[0], hi[1]};
            acc[0][r] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[0], b, acc[0][r], 0, 0, 0);
            acc[1][r] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[1], b, acc[1][r], 0, 0, 0);
        }
    };
    // slot (st - step_begin) % D holds step st; the loop body covers D steps so that the slots are compile-time names
    narrow_static_for<D - 1>([&](auto u) { load_step(u, step_begin + decltype(u)::value); });
    for (int st = step_begin; st < step_end; st += D) {
        narrow_static_for<D>([&](auto u) {
            constexpr int U = decltype(u)::value;
            load_step(std::integral_constant<int, (U + D - 1) % D>(), st + U + D - 1);
            store_step(u);
            multiply();
        });
    }
    // the block's sum: every wave adds its tiles into one [K][NR][32] array in LDS (over the staging areas)
    __syncthreads();
    int32_t *sum = reinterpret_cast<int32_t *>(lds);
    for (int i = t; i < 64 * NR * 32; i += 256) sum[i] = 0;
    __syncthreads();
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int k = 32 * kt + 8 * (e / 4) + 4 * half + (e % 4);
                atomicAdd(&sum[(k * NR + r) * 32 + lane % 32], acc[kt][r][e]);
            }
    __syncthreads();
    int32_t *part = p.out + (size_t)blockIdx.x * p.K * p.R * p.SC;
    const int per_k = p.R * p.SC;
    for (int i = t; i < p.K * per_k; i += 256) {
        const int k = i / per_k, rj = i - k * per_k, r = rj / p.SC, j = rj - r * p.SC;
        part[i] = sum[(k * NR + r) * 32 + j];
    }
}

static size_t padded_bytes(int N, int C, int H, int W, int pad_h, int pad_w) {
    return (size_t)N * (H + 2 * pad_h) * (W + 2 * pad_w) * C + 64;
}

bool narrow_conv_supported(const lpdt_conv_desc *d, int P, int Q) {
    if (d->C % 16 == 0) return false;                 // wide inputs take the gather kernels
    if (d->S * d->C > 32 || d->R > kNR) return false;
    if (d->K % 16 || d->K > 64) return false;
    if (d->stride_h != d->stride_w || d->pad_h != d->pad_w) return false;
    if ((long long)d->N * P * Q >= (1 << 24)) return false;  // div24 range
    if (padded_bytes(d->N, d->C, d->H, d->W, d->pad_h, d->pad_w) >= (1ull << 31)) return false;
    return true;
}

size_t narrow_fwd_workspace(const lpdt_conv_desc *d) {
    return round_up(padded_bytes(d->N, d->C, d->H, d->W, d->pad_h, d->pad_w), 256) + round_up((size_t)d->K * d->R * 32, 256);
}
// blocks of the weight-gradient launch (4 waves each) and 32-pixel steps per wave
static void narrow_wgrad_grid(long long M, int *grid, int *steps_per_wave) {
    const int steps = (int)((M + 31) / 32);
    int waves = 1024;                          // one wave per SIMD: the filter's sums fill a wave's accumulators
    if (waves > steps / 4) waves = steps / 4 > 0 ? steps / 4 : 1;
    waves = (waves + 3) / 4 * 4;
    *steps_per_wave = (steps + waves - 1) / waves;
    *grid = ((steps + *steps_per_wave - 1) / *steps_per_wave + 3) / 4;
}
size_t narrow_wgrad_workspace(const lpdt_conv_desc *d) {
    const int P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1, Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    int grid, spb;
    narrow_wgrad_grid((long long)d->N * P * Q, &grid, &spb);
    return round_up(padded_bytes(d->N, d->C, d->H, d->W, d->pad_h, d->pad_w), 256) +
           round_up((size_t)grid * d->K * d->R * d->S * d->C * sizeof(int32_t), 256);
}

static NarrowParams narrow_params(const lpdt_conv_desc *d, int P, int Q, const int8_t *xp) {
    NarrowParams p = {};
    p.xp = xp;
    p.M = d->N * P * Q; p.K = d->K; p.C = d->C; p.R = d->R; p.SC = d->S * d->C; p.stride = d->stride_h;
    p.PH = d->H + 2 * d->pad_h; p.PW = d->W + 2 * d->pad_w; p.P = P; p.Q = Q;
    p.inv_pq = 1.0f / (float)(P * Q);
    p.inv_q = 1.0f / (float)Q;
    return p;
}

static void launch_pad(const lpdt_conv_desc *d, const int8_t *x, int8_t *xp, hipStream_t st) {
    const size_t total = padded_bytes(d->N, d->C, d->H, d->W, d->pad_h, d->pad_w);
    size_t blocks = (total / 4 + 256) / 256;
    if (blocks > 4096) blocks = 4096;   // (measured on the 224 x 224 image at batch 64: 1.6 us less than with 16384)
    hipLaunchKernelGGL(pad_image_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, d->N, d->H, d->W, d->C, d->pad_h,
                       d->H + 2 * d->pad_h, d->W + 2 * d->pad_w, xp, (unsigned)total);
}

void launch_narrow_fwd(const lpdt_conv_desc *d, int P, int Q, const int8_t *x, const int8_t *w, int32_t *acc, int out_mode,
                       const float *sA, const float *sB, void *ws, hipStream_t st) {
    int8_t *xp = static_cast<int8_t *>(ws);
    int8_t *wr = xp + round_up(padded_bytes(d->N, d->C, d->H, d->W, d->pad_h, d->pad_w), 256);
    launch_pad(d, x, xp, st);
    hipLaunchKernelGGL(pack_filter_rows_kernel, dim3((d->K * d->R * 32 + 255) / 256), dim3(256), 0, st, w, d->K, d->R, d->S * d->C, wr);
    NarrowParams p = narrow_params(d, P, Q, xp);
    p.wr = wr; p.out = acc; p.out_mode = out_mode; p.sA = sA; p.sB = sB;
    p.vec_out = aligned(acc, 16) ? 1 : 0;
    p.blocks_total = (p.M + 31) / 32;
    int grid = (p.blocks_total + 3) / 4;
    if (grid > 512) grid = 512;   // two blocks per CU, each wave walking its run of row blocks (measured on the 224 x 224 stem at batch 64:
                                  // 256 blocks 77 us, 512 69 us, 768 71 us, 1024 73 us, 2048 75 us, 4096 82 us)
    // (7 rows, the 7 x 7 stem, have an instantiation of their own: an eighth row would be an eighth of the loads for nothing)
    if (d->R <= 4) hipLaunchKernelGGL(narrow_fwd_kernel<4>, dim3(grid), dim3(256), 0, st, p);
    else if (d->R == 7) hipLaunchKernelGGL(narrow_fwd_kernel<7>, dim3(grid), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(narrow_fwd_kernel<8>, dim3(grid), dim3(256), 0, st, p);
}

void launch_narrow_wgrad(const lpdt_conv_desc *d, int P, int Q, const int8_t *g, const int8_t *x, void *out, int out_mode,
                         const float *sA, const float *sB, void *ws, hipStream_t st) {
    int8_t *xp = static_cast<int8_t *>(ws);
    int32_t *partial = reinterpret_cast<int32_t *>(xp + round_up(padded_bytes(d->N, d->C, d->H, d->W, d->pad_h, d->pad_w), 256));
    launch_pad(d, x, xp, st);
    NarrowParams p = narrow_params(d, P, Q, xp);
    p.g = g; p.out = partial;
    p.blocks_total = (p.M + 31) / 32;
    int grid;
    narrow_wgrad_grid(p.M, &grid, &p.steps_per_block);
    const int NR = d->R <= 4 ? 4 : d->R == 7 ? 7 : 8;
    size_t lds = 4 * (size_t)(32 * kGS + 32 * ((NR == 7 ? 8 : NR) * 32 + 32));
    if (lds < (size_t)64 * NR * 32 * 4) lds = (size_t)64 * NR * 32 * 4;
    p.zero_off = (int)(padded_bytes(d->N, d->C, d->H, d->W, d->pad_h, d->pad_w) - 64);
    auto go = [&](auto kernel) {
        if (lds > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds, st, p);
    };
    if (NR == 4) go(narrow_wgrad_kernel<4>);
    else if (NR == 7) go(narrow_wgrad_kernel<7>);
    else go(narrow_wgrad_kernel<8>);
    launch_wgrad_reduce(partial, (long long)d->K * d->R * d->S * d->C, grid, out, out_mode, sA, sB, st);
}

}  // namespace lpdt
