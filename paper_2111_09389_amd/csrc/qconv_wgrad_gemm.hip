// Weight gradient of a pointwise product on int8 codes (Table "hardware_training", row Linear, third product: linear
// layers at transformer shapes, both channel counts multiples of 256):
//   dw[k][c] = sum over tokens t of g[t][k] * x[t][c]
// a GEMM whose reduction runs over the strided axis of both operands.  A block owns a 256 x 256 tile of dw and a
// contiguous share of the tokens.  A step is 64 tokens: 64 x 256 bytes of each operand go from global memory straight
// into LDS (buffer loads with LDS destination, a ring of 4 stages, one barrier per step) and both MFMA operands are read
// from there with the transposing LDS load.  Tiles of 256 x 256 because the L2 cache delivers only 2-3 times the HBM
// rate: at 128 x 128 the operand bytes per product double and the loop waits for L2.  8 waves: 2 (k) x 4 (c), 128 x 64
// each = 8 accumulators.  A block writes one plain partial tile; the reduction kernel of the other weight-gradient
// kernels adds them (exact integers: order-free) and applies the dequantizing scale when asked.
//
// LDS rows are 256 bytes = the bank period, so the 8 tokens of a transposing read would all hit the same banks: the
// 16-byte granule q of token t sits at position q ^ 2*(t % 8).  The two 16-lane halves that are served together read
// granules q and q + 1 (q even) of 8 consecutive tokens: 16 different positions.
//
// kTaps: the same for stride-1 filters of up to 3 x 3 taps on maps too small for the row-tile kernel (VGG's 4 x 4 and 2 x 2
// maps at 512 channels): a block owns ONE tap of a 256 x 256 channel tile, dw[k][tap][c] = sum over output pixels t of
// g[t][k] * x[t + tap][c]; the loader finds each token's input pixel (a pixel outside the image is fetched from beyond
// the buffer: zeros), everything after the loads is the pointwise kernel.
#include "qconv_internal.h"
#ifdef LPDT_TUNE
#include <cstdlib>
#endif

namespace lpdt {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) v2i lds_v2i;

constexpr unsigned kBeyond = 0x80000000u;  // a buffer offset no tensor reaches: such loads deliver zeros
constexpr int kGemmTile = 256;             // channels of either operand per block
constexpr int kGemmStep = 64;              // tokens per step
constexpr int kGemmStages = 4;
constexpr int kGemmWaves = 8;
constexpr int kGemmLoads = 2 * kGemmStep * kGemmTile / 1024 / kGemmWaves;   // load instructions per wave and step (4)

struct WgradGemmParams {
    const int8_t *g;            // [T][K]
    const int8_t *x;            // [T][C]
    int32_t *partial;           // [splits][K][C]
    unsigned g_bytes, x_bytes;
    int T, K, C;
    int steps, steps_per_split;
    int tiles_k, tiles_kc;
    long long out_len;
    // kTaps only: the maps and the filter (stride 1); T = N * P * Q output pixels, x = [N][H][W][C]
    int ntaps, S, pad_h, pad_w, H, W, P, Q;
    float inv_pq, inv_q;
};

// q = m / d for 0 <= m < 2^24 through one float multiply and a correction step
__device__ __forceinline__ int gemm_div24(int m, int d, float inv) {
    int q = (int)((float)m * inv);
    int r = m - q * d;
    if (r < 0) { --q; r += d; }
    if (r >= d) ++q;
    return q;
}

// Transposing LDS read issued as assembly: the compiler then does not know that it reads LDS and does not put a wait for
// every outstanding direct-to-LDS load in front of it (which took the loads of the following steps out of flight:
// 75.8 -> 62.8 us on the 16384 x 768 x 3072 product).  A result is valid only after a tr_wait that names it; nothing may
// touch (not even copy) the registers before.
__device__ __forceinline__ v2i tr_read(const unsigned char *p) {
    v2i r;
    asm volatile("ds_read_b64_tr_b8 %0, %1" : "=v"(r) : "v"((unsigned)(size_t)(lds_v2i *)p));
    return r;
}
// Waits until at most N of the LDS reads issued after the named results are outstanding (LDS reads complete in issue
// order); the registers pass through the statement so that nothing consuming them is scheduled before it.
template <int N>
__device__ __forceinline__ void tr_wait(v2i &r0, v2i &r1) {
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit count");
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(r0), "+v"(r1) : "n"(N));
}
template <int N>
__device__ __forceinline__ void tr_wait(v2i &r0, v2i &r1, v2i &r2, v2i &r3, v2i &r4, v2i &r5) {
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit count");
    asm volatile("s_waitcnt lgkmcnt(%6)" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3), "+v"(r4), "+v"(r5) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit count");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <bool kTaps>
__global__ __launch_bounds__(64 * kGemmWaves, 1) void wgrad_gemm_kernel(const WgradGemmParams p) {
    constexpr int ST = kGemmStages, NL = kGemmLoads;
    constexpr int kOperand = kGemmStep * kGemmTile;      // bytes of one operand tile
    constexpr int kStage = 2 * kOperand;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int t = threadIdx.x, lane = t % 64, wave = __builtin_amdgcn_readfirstlane(t / 64);

    // the tiles of one token share sit next to each other on one XCD (blocks go round the 8 XCDs): they read the same tokens
    const int nb = gridDim.x;
    const int lid = nb % 8 == 0 ? (int)(blockIdx.x % 8) * (nb / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
    // (with taps: the taps of a channel tile are neighbours too)
    const int per_share = kTaps ? p.tiles_kc * p.ntaps : p.tiles_kc;
    const int z = lid / per_share, rest = lid - z * per_share;
    const int tap = kTaps ? rest / p.tiles_kc : 0, kc = rest - tap * p.tiles_kc;
    const int ty = kTaps ? tap / p.S : 0, tx = tap - ty * p.S;
    const int k0 = (kc % p.tiles_k) * kGemmTile, c0 = (kc / p.tiles_k) * kGemmTile;
    const int step_begin = min(p.steps, z * p.steps_per_split), step_end = min(p.steps, step_begin + p.steps_per_split);

    const __amdgpu_buffer_rsrc_t rs_g = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.g), 0, (int)p.g_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0, (int)p.x_bytes, 0x00020000);

    // ---- loader role.  Instruction i = wave + 8j of a step: i < 16 gradient, else input; each covers 4 tokens x 256 bytes,
    // lane -> (token, position); the lane fetches the granule that belongs at its position.
    int loff[NL], ltok[NL];
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        const int i = wave + kGemmWaves * j, tok = 4 * (i % 16) + (lane >> 4);
        const int gran = (lane & 15) ^ ((tok & 7) << 1);
        ltok[j] = tok;
        loff[j] = i < 16 ? tok * p.K + k0 + gran * 16 : tok * p.C + c0 + gran * 16;
    }
    int ld_step = step_begin;
    auto issue = [&](int buf) {
        const int tok0 = ld_step * kGemmStep;
        const int live = ld_step < step_end ? p.T - tok0 : 0;     // tokens of this step that exist
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int i = wave + kGemmWaves * j;
            const bool ok = ltok[j] < live;
            if (i < 16) {
                const unsigned off = ok ? (unsigned)(tok0 * p.K + loff[j]) : kBeyond;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_g, (lds_void *)(lds + buf * kStage + i * 1024), 16, off, 0, 0, 0);
            } else if (!kTaps) {
                const unsigned off = ok ? (unsigned)(tok0 * p.C + loff[j]) : kBeyond;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(lds + buf * kStage + i * 1024), 16, off, 0, 0, 0);
            } else {
                // output pixel (n, oy, ox) of this lane's token meets input pixel (n, oy + ty - pad, ox + tx - pad)
                const int tk = min(tok0 + ltok[j], p.T - 1);
                const int n = gemm_div24(tk, p.P * p.Q, p.inv_pq), rem = tk - n * p.P * p.Q;
                const int oy = gemm_div24(rem, p.Q, p.inv_q), ox = rem - oy * p.Q;
                const int iy = oy + ty - p.pad_h, ix = ox + tx - p.pad_w;
                const bool in = ok && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
                const unsigned off = in ? (unsigned)(((n * p.H + iy) * p.W + ix) * p.C + (loff[j] - ltok[j] * p.C)) : kBeyond;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(lds + buf * kStage + i * 1024), 16, off, 0, 0, 0);
            }
        }
        ++ld_step;
    };

    // ---- multiplier role.  Transposing LDS read: in each block of 16 lanes, source lane j supplies 8 bytes and result
    // lane i receives byte i%8 of source lanes i/8, i/8+2, ...  With source lane j reading token j/2 at channel offset
    // 8*(j%2), result lane i holds channel i of 8 tokens: the MFMA operand (rows = channels, reduction = tokens).
    // Block b of the wave covers channels 16*(b%2).. and tokens 16*(b/2)..; two reads make the 16 tokens.
    const int wk = wave & 1, wc = wave >> 1;
    const int blk = lane >> 4, j16 = lane & 15;
    int a_off[2][2][4], b_off[2][2][2];   // [32-token group][half][32-channel sub-tile]
#pragma unroll
    for (int kg = 0; kg < 2; ++kg)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int tok = 32 * kg + 16 * (blk >> 1) + 8 * h + (j16 >> 1);
            const int row = tok * kGemmTile + 8 * (j16 & 1), swz = (tok & 7) << 1;
#pragma unroll
            for (int s = 0; s < 4; ++s) a_off[kg][h][s] = row + (((8 * wk + 2 * s + (blk & 1)) ^ swz) << 4);
#pragma unroll
            for (int s = 0; s < 2; ++s) b_off[kg][h][s] = kOperand + row + (((4 * wc + 2 * s + (blk & 1)) ^ swz) << 4);
        }

    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

#pragma unroll
    for (int i = 0; i < ST - 1; ++i) issue(i);
    for (int step = step_begin, it = 0; step < step_end; ++step, ++it) {
        // this step's operands have landed everywhere (the ST - 2 steps issued after it may still be on their way);
        // everybody is done reading the stage of the step before, which the next loads overwrite
        wait_loads_and_barrier<(ST - 2) * NL>();
        issue((it + ST - 1) % ST);
        const unsigned char *const buf = lds + (it % ST) * kStage;
#pragma unroll
        for (int kg = 0; kg < 2; ++kg) {
            // the filter-side operand (both sub-tiles) and the first pixel-side one go out together; each later pixel-side
            // operand is requested before the products of the one before it
            v2i bl[2][2], al[2][2];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                bl[s][0] = tr_read(buf + b_off[kg][0][s]);
                bl[s][1] = tr_read(buf + b_off[kg][1][s]);
            }
            al[0][0] = tr_read(buf + a_off[kg][0][0]);
            al[0][1] = tr_read(buf + a_off[kg][1][0]);
            v4i b[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v2i(&cur)[2] = al[i & 1];
                if (i < 3) {
                    al[(i + 1) & 1][0] = tr_read(buf + a_off[kg][0][i + 1]);
                    al[(i + 1) & 1][1] = tr_read(buf + a_off[kg][1][i + 1]);
                }
                if (i == 0) {
                    tr_wait<2>(bl[0][0], bl[0][1], bl[1][0], bl[1][1], cur[0], cur[1]);
#pragma unroll
                    for (int s = 0; s < 2; ++s) b[s] = v4i{bl[s][0][0], bl[s][0][1], bl[s][1][0], bl[s][1][1]};
                } else if (i < 3) {
                    tr_wait<2>(cur[0], cur[1]);
                } else {
                    tr_wait<0>(cur[0], cur[1]);
                }
                const v4i a = {cur[0][0], cur[0][1], cur[1][0], cur[1][1]};
#pragma unroll
                for (int s = 0; s < 2; ++s) acc[i][s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[s], acc[i][s], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);     // keep the products in front of the next requests and wait
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the zero loads past the last step

    // a lane holds input channel lane%32 of a sub-tile and output channels 8*(r/4) + 4*(lane/32) + r%4
    int32_t *out = p.partial + (size_t)z * p.out_len;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int c = c0 + 64 * wc + 32 * s + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + 128 * wk + 32 * i + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                out[kTaps ? ((size_t)k * p.ntaps + tap) * p.C + c : (size_t)k * p.C + c] = acc[i][s][r];
            }
        }
}

}  // namespace

bool wgrad_gemm_plan(const lpdt_conv_desc *d, int P, int Q, WgradGemmPlan *pl) {
    if (d->R != 1 || d->S != 1 || d->stride_h != 1 || d->stride_w != 1 || d->pad_h != 0 || d->pad_w != 0) return false;
    if (d->K % kGemmTile || d->C % kGemmTile) return false;
    const long long T = (long long)d->N * P * Q;
    const size_t lim = ((size_t)1 << 31) - 4096;  // 32-bit buffer offsets
    if ((size_t)T * d->K >= lim || (size_t)T * d->C >= lim) return false;
    pl->T = (int)T;
    pl->steps = (int)((T + kGemmStep - 1) / kGemmStep);
    pl->tiles_k = d->K / kGemmTile;
    pl->tiles_kc = pl->tiles_k * (d->C / kGemmTile);
    long long splits = 256 / pl->tiles_kc;             // one block per CU
    if (splits > pl->steps / 8) splits = pl->steps / 8;  // a block's ring wants a few steps to pay off
    if (splits < 1) return false;                        // too few tokens: the rectangle-stepped kernel takes it
    pl->steps_per_split = (int)((pl->steps + splits - 1) / splits);
    pl->splits = (pl->steps + pl->steps_per_split - 1) / pl->steps_per_split;
    if ((long long)pl->tiles_kc * pl->splits < 128) return false;   // half the chip idle: smaller tiles do better
    pl->out_len = (long long)d->K * d->C;
    pl->partial_bytes = round_up((size_t)pl->splits * pl->out_len * sizeof(int32_t), 256);
    return true;
}

// Multi-tap form: for what the row-tile and rectangle kernels decline (the caller asks them first).
bool wgrad_gemm_taps_plan(const lpdt_conv_desc *d, int P, int Q, WgradGemmPlan *pl) {
    const int ntaps = d->R * d->S;
    if (ntaps < 2 || d->R > 3 || d->S > 3 || d->stride_h != 1 || d->stride_w != 1) return false;
    if (d->K % kGemmTile || d->C % kGemmTile) return false;
    const long long T = (long long)d->N * P * Q;
    const size_t lim = ((size_t)1 << 31) - 4096;  // 32-bit buffer offsets
    if (T >= (1 << 24) || (size_t)T * d->K >= lim || (size_t)d->N * d->H * d->W * d->C >= lim) return false;
    pl->T = (int)T;
    pl->steps = (int)((T + kGemmStep - 1) / kGemmStep);
    pl->tiles_k = d->K / kGemmTile;
    pl->tiles_kc = pl->tiles_k * (d->C / kGemmTile);
    const long long tiles = (long long)pl->tiles_kc * ntaps;
    // blocks wanted: a few less than CUs, since a share more can push the launch just past one block per CU and into a
    // second round (512 -> 512 on 4 x 4 maps, 36 tiles: 8 shares = 288 blocks 52 us, 5-7 shares 37-39 us, 4 shares 42 us)
    long long target = 192, min_steps = 4;
#ifdef LPDT_TUNE
    if (const char *e = getenv("LPDT_WGRAD_GEMM_BLOCKS")) target = atoi(e);
    if (const char *e = getenv("LPDT_WGRAD_GEMM_MINSTEPS")) min_steps = atoi(e);
#endif
    long long splits = (target + tiles - 1) / tiles;
    if (splits > pl->steps / min_steps) splits = pl->steps / min_steps;  // each share's partial tile is written and read back: no shorter shares
    if (splits < 1) return false;
    pl->steps_per_split = (int)((pl->steps + splits - 1) / splits);
    pl->splits = (pl->steps + pl->steps_per_split - 1) / pl->steps_per_split;
    if (tiles * pl->splits < 64) return false;
    pl->out_len = (long long)d->K * ntaps * d->C;
    pl->partial_bytes = round_up((size_t)pl->splits * pl->out_len * sizeof(int32_t), 256);
    return true;
}

void launch_wgrad_gemm(const lpdt_conv_desc *d, const WgradGemmPlan &pl, const int8_t *g, const int8_t *x, void *out, int out_mode,
                       const float *sA, const float *sB, void *partial, hipStream_t st) {
    WgradGemmParams p = {};
    p.g = g; p.x = x; p.partial = static_cast<int32_t *>(partial);
    p.g_bytes = (unsigned)((size_t)pl.T * d->K); p.x_bytes = (unsigned)((size_t)pl.T * d->C);
    p.T = pl.T; p.K = d->K; p.C = d->C;
    p.steps = pl.steps; p.steps_per_split = pl.steps_per_split; p.tiles_k = pl.tiles_k; p.tiles_kc = pl.tiles_kc;
    p.out_len = pl.out_len;
    const size_t lds = (size_t)kGemmStages * 2 * kGemmStep * kGemmTile;
    const int ntaps = d->R * d->S;
    if (ntaps > 1) {
        const int P = d->H + 2 * d->pad_h - d->R + 1, Q = d->W + 2 * d->pad_w - d->S + 1;   // stride 1
        p.x_bytes = (unsigned)((size_t)d->N * d->H * d->W * d->C);
        p.ntaps = ntaps; p.S = d->S; p.pad_h = d->pad_h; p.pad_w = d->pad_w; p.H = d->H; p.W = d->W; p.P = P; p.Q = Q;
        p.inv_pq = 1.0f / (float)(P * Q); p.inv_q = 1.0f / (float)Q;
        static bool raised_taps = false;
        if (!raised_taps) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_gemm_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            raised_taps = true;
        }
        hipLaunchKernelGGL(wgrad_gemm_kernel<true>, dim3((unsigned)(pl.tiles_kc * ntaps * pl.splits)), dim3(64 * kGemmWaves), lds, st, p);
        launch_wgrad_reduce(p.partial, pl.out_len, pl.splits, out, out_mode, sA, sB, st);
        return;
    }
    static bool raised = false;
    if (!raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_gemm_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        raised = true;
    }
    hipLaunchKernelGGL(wgrad_gemm_kernel<false>, dim3((unsigned)(pl.tiles_kc * pl.splits)), dim3(64 * kGemmWaves), lds, st, p);
    launch_wgrad_reduce(p.partial, pl.out_len, pl.splits, out, out_mode, sA, sB, st);
}

}  // namespace lpdt
