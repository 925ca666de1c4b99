// Weight gradient of a stride-1 convolution on int8 codes (Table "hardware_training", row Conv, third product), row-tile
// variant for filters of up to 3 x 3 taps whose channel counts are multiples of the tile:
//   dw[k][r][s][c] = sum over output pixels (n, oy, ox) of g[n,oy,ox,k] * x[n, oy + r - pad, ox + s - pad, c]
//
// The reduction runs over pixels.  A block owns a KT x 64 (output x input channel) tile of dw for ALL taps and a
// contiguous share of the row tiles of the batch (KT = 32):
//
//   row tile = TR whole output rows of one image (TR * Q <= 128 pixel slots = up to 4 MFMA reduction groups of 32)
//   operands = the tile's gradient pixels [slot][32 bytes] and the (TR + R - 1) x (Q + S - 1) input patch [pixel][80 B],
//              both loaded straight into LDS (buffer loads with LDS destination; what lies outside the image or past
//              the tile arrives as zeros) through a ring of 3 buffers: several tiles are in flight while one is
//              multiplied, one barrier per tile
//   tap      = a constant pixel offset into the patch: every tap's operand is read out of the one patch with the
//              transposing LDS load (the MFMA reduces over pixels, memory is channel-fastest)
//
// 8 waves share the 32 x 64 tile: two 32 x 32 halves times four groups of taps, each wave holding up to 3 accumulators.  At the end a block writes its sums as one plain partial tile; the reduction kernel of the
// rectangle-stepped variant adds the partial tiles (exact integers: order-free, bit-reproducible) and applies the
// dequantizing scale when asked.
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
constexpr int kRowsWaves = 8;
constexpr int kRowsKT = 32;                // output channels of a block's tile
constexpr int kRowsLoads = 3;              // load instructions per wave and tile

struct WgradRowsParams {
    const int8_t *g;            // [N][P][Q][K]
    const int8_t *x;            // [N][H][W][C]
    int32_t *partial;           // [splits][K][R*S][C]
    unsigned g_bytes, x_bytes;
    int K, C, H, W, P, Q, S, pad_h, pad_w, ntaps;
    int TR, PR, PW;             // output rows per tile, patch rows and columns
    int ni;                     // patch load instructions (64 units of 16 bytes, 5 units per pixel)
    int nkg;                    // 32-slot reduction groups per tile
    int tiles_per_image, ntiles, tiles_per_split;
    int tiles_k, tiles_kc;
    float inv_Q, inv_PW;        // reciprocals for the set-up's divisions
    long long out_len;
    // one share only (a block holds the complete sums of its tile): the results go straight to their place, no partial
    // tiles and no second launch.  direct_mode: 0 int32 sums, 1 fp32 sA*sB*sum (the reduction kernel's arithmetic).
    void *direct;
    int direct_mode;
    const float *sA, *sB;
};

// LDS layouts.  Gradient tile: [slot][32 B]; the 8 consecutive slots one transposing read touches are 256 contiguous
// bytes, all banks once.  Patch: a pitch of 80 bytes per pixel (a fifth of the loader's lanes fetch nothing), which
// also spreads 8 consecutive pixels over all banks and, unlike an XOR swizzle, keeps addresses linear in the pixel
// index: a tap is one constant added to a precomputed offset.
constexpr int kPatchPitch = 80;
// Transposing LDS read issued as assembly: the compiler then does not know that it reads LDS and does not put a wait for
// every outstanding direct-to-LDS load in front of it (which took the loads of the following tiles out of flight:
// 30.7 -> 27.7 us on the 64 x 56 x 56 x 64 layer, 43.3 -> 37.8 us on 64 x 7 x 7 x 512).  A result is valid only after a
// tr_wait that names it; nothing may touch (not even copy) the registers before.
__device__ __forceinline__ v2i tr_read(const unsigned char *p) {
    v2i r;
    asm volatile("ds_read_b64_tr_b8 %0, %1" : "=v"(r) : "v"((unsigned)(size_t)(lds_v2i *)p));
    return r;
}
// Waits for all LDS reads issued so far; the named registers pass through the statement so that nothing consuming them
// can be scheduled before it.
__device__ __forceinline__ void tr_wait(v2i &r0, v2i &r1, v2i &r2, v2i &r3) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3));
}
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit count");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// exact a / b for 0 <= a < 2^16, 0 < b < 2^8 with inv = 1.0f / b: (a + 0.5) / b is at least 0.5 / b away from an integer,
// far more than the rounding of two float operations can move it.  A dozen of these in the set-up of a kernel that
// runs for 20 us are worth replacing the integer division sequence.
__device__ __forceinline__ int small_div(int a, float inv) { return (int)(((float)a + 0.5f) * inv); }

// KT: output channels of the block's tile.  ST: LDS stages (ST - 1 tiles in flight ahead of the one being multiplied).
template <int ST>
__global__ __launch_bounds__(64 * kRowsWaves, 2) void wgrad_rows_kernel(const WgradRowsParams p) {
    constexpr int NW = kRowsWaves;                    // waves of the block
    constexpr int NL = kRowsLoads;                    // load instructions per wave and tile
    constexpr int KT = kRowsKT;
    constexpr int WT = kRowsWaves / 2;                // groups of taps (times 2 halves of the input channels)
    constexpr int NA = (9 + WT - 1) / WT;             // accumulators (taps) per wave
    constexpr int GI = 128 * KT / 1024;               // gradient load instructions per tile
    constexpr int KG = 4;                             // reduction groups per tile
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int buf_bytes = (GI + p.ni) * 1024;
    unsigned char *const dump = lds + ST * buf_bytes;  // 1 KiB that takes the loads issued only to keep the count even
    const int t = threadIdx.x, lane = t % 64, wave = __builtin_amdgcn_readfirstlane(t / 64);

    // blocks that share operands (the tiles of one pixel share) sit next to each other on one XCD (blocks go round the 8 XCDs)
    const int nb = gridDim.x;
    const int lid = nb % 8 == 0 ? (int)(blockIdx.x % 8) * (nb / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
    const int z = lid / p.tiles_kc, kc = lid - z * p.tiles_kc;
    const int k0 = (kc % p.tiles_k) * KT, c0 = (kc / p.tiles_k) * 64;
    const int tile_begin = min(p.ntiles, z * p.tiles_per_split), tile_end = min(p.ntiles, tile_begin + p.tiles_per_split);

    const __amdgpu_buffer_rsrc_t rs_g = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.g), 0, (int)p.g_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0, (int)p.x_bytes, 0x00020000);

    // ---- loader role.  Instruction k = wave + NW*j of a tile: k < GI gradient (16 or 32 slots), else 64 units of the patch.
    // Per instruction and lane: the byte offset from the tile's first gradient / input row, and what decides per tile
    // whether the element exists (the slot for the gradient, the patch row for the input).
    int loff[NL], lpos[NL];
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        const int k = wave + NW * j;
        if (k < GI) {
            const int slot = 32 * k + (lane >> 1);
            loff[j] = slot * p.K + k0 + (lane & 1) * 16;
            lpos[j] = slot;
        } else {
            const int q = 64 * (k - GI) + lane;            // 16-byte unit of the patch buffer: pixel q/5, granule q%5
            const int pp = small_div(q, 0.2f), gran = q - 5 * pp;
            const int pr = small_div(pp, p.inv_PW), px = pp - pr * p.PW;
            const int ix = px - p.pad_w;
            const bool ok = gran < 4 && pp < p.PR * p.PW && (unsigned)ix < (unsigned)p.W;
            loff[j] = ((pr - p.pad_h) * p.W + ix) * p.C + c0 + gran * 16;
            lpos[j] = ok ? pr - p.pad_h : -(1 << 20);      // a row offset no tile brings back into the image
        }
    }
    // every wave issues exactly NL loads per tile (the wait below counts them); tiles past the block's share and
    // instructions past the patch load zeros from beyond the tensor.  (ld_n, ld_r0): image and first row of the next tile.
    int ld_tile = tile_begin, ld_n = tile_begin / p.tiles_per_image, ld_r0 = (tile_begin - ld_n * p.tiles_per_image) * p.TR;
    auto issue = [&](int buf) {
        const bool live = ld_tile < tile_end;
        const int live_slots = live ? min(p.TR, p.P - ld_r0) * p.Q : 0;
        const int base_g = (ld_n * p.P + ld_r0) * p.Q * p.K;
        const int base_x = (ld_n * p.H + ld_r0) * p.W * p.C;
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int k = wave + NW * j;
            if (k < GI) {
                const unsigned off = lpos[j] < live_slots ? (unsigned)(base_g + loff[j]) : kBeyond;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_g, (lds_void *)(lds + buf * buf_bytes + k * 1024), 16, off, 0, 0, 0);
            } else {
                const bool ok = live && (unsigned)(ld_r0 + lpos[j]) < (unsigned)p.H;
                const unsigned off = ok ? (unsigned)(base_x + loff[j]) : kBeyond;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void *)(k < GI + p.ni ? lds + buf * buf_bytes + k * 1024 : dump), 16, off, 0, 0, 0);
            }
        }
        ++ld_tile;
        ld_r0 += p.TR;
        if (ld_r0 >= p.P) { ld_r0 = 0; ++ld_n; }
    };

    // ---- multiplier role.  Transposing LDS read: in each block of 16 lanes, source lane j supplies 8 bytes and result
    // lane i receives byte i%8 of source lanes i/8, i/8+2, ...  With source lane j reading pixel slot j/2 at channel
    // offset 8*(j%2), result lane i holds channel i of 8 pixel slots: the MFMA operand (rows = channels, reduction =
    // pixels).  Block b of the wave covers channels 16*(b%2).. and slots 16*(b/2)..; two reads make the 16 slots.
    const int tj = wave & 1, tw = wave >> 1;
    const int blk = lane >> 4, j16 = lane & 15;
    int a_off[KG][2], b_off[KG][2];   // per reduction group and half: byte offsets of the gradient and of the patch under tap (0, 0)
#pragma unroll
    for (int i = 0; i < KG; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int slot = 32 * i + 16 * (blk >> 1) + 8 * h + (j16 >> 1);
            a_off[i][h] = slot * KT + 16 * (blk & 1) + 8 * (j16 & 1);
            const int dy = small_div(slot, p.inv_Q), ox = slot - dy * p.Q;
            const int pp = dy < p.TR ? dy * p.PW + ox : 0;  // slots past the tile meet zero gradient rows
            b_off[i][h] = GI * 1024 + pp * kPatchPitch + 16 * (2 * tj + (blk & 1)) + 8 * (j16 & 1);
        }
    int toff[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int tap = min(tw + WT * i, p.ntaps - 1);
        const int ty = (tap >= p.S) + (tap >= 2 * p.S);     // at most 3 filter rows
        toff[i] = (ty * p.PW + tap - ty * p.S) * kPatchPitch;
    }

    v16i acc[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;

#pragma unroll
    for (int i = 0; i < ST - 1; ++i) issue(i);
    for (int tile = tile_begin, it = 0; tile < tile_end; ++tile, ++it) {
        // this tile's operands have landed everywhere (the ST - 2 tiles issued after it may still be on their way);
        // everybody is done reading the buffer of the tile before, which the next loads overwrite
        wait_loads_and_barrier<(ST - 2) * NL>();
        issue((it + ST - 1) % ST);
        const unsigned char *const gbuf = lds + (it % ST) * buf_bytes;
#pragma unroll
        for (int kgi = 0; kgi < KG; ++kgi) {
            if (kgi < p.nkg) {
                v2i a_lo = tr_read(gbuf + a_off[kgi][0]);
                v2i a_hi = tr_read(gbuf + a_off[kgi][1]);
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    if (tw + WT * i < p.ntaps) {
                        v2i b_lo = tr_read(gbuf + b_off[kgi][0] + toff[i]);
                        v2i b_hi = tr_read(gbuf + b_off[kgi][1] + toff[i]);
                        tr_wait(a_lo, a_hi, b_lo, b_hi);
                        const v4i a = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
                        const v4i b = {b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
                        acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
                    }
                }
            }
        }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the zero loads past the last tile

    // a lane holds input channel lane%32 of its sub-tile and output channels 8*(r/4) + 4*(lane/32) + r%4
    const bool as_float = p.direct && p.direct_mode;
    int32_t *out = p.direct ? static_cast<int32_t *>(p.direct) : p.partial + (size_t)z * p.out_len;
    const float sc = as_float ? __fmul_rn(*p.sA, *p.sB) : 0.0f;
    const int c = c0 + 32 * tj + (lane & 31);
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int tap = tw + WT * i;
        if (tap < p.ntaps) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                const size_t at = ((size_t)k * p.ntaps + tap) * p.C + c;
                if (as_float) reinterpret_cast<float *>(out)[at] = dequant_value(sc, acc[i][r], 0.f, false);
                else out[at] = acc[i][r];
            }
        }
    }
}

}  // namespace

bool wgrad_rows_plan(const lpdt_conv_desc *d, int P, int Q, WgradRowsPlan *pl, int beside) {
    if (beside < 0) beside = wgrad_beside();
    const int ntaps = d->R * d->S;
    if (d->stride_h != 1 || d->stride_w != 1 || d->R > 3 || d->S > 3 || ntaps < 2) return false;
    if (d->K % kRowsKT || d->C % 64 || Q > 128 || P < 1 || Q < 1) return false;
    const size_t lim = ((size_t)1 << 31) - 4096;  // 32-bit buffer offsets
    if ((size_t)d->N * P * Q * d->K >= lim || (size_t)d->N * d->H * d->W * d->C >= lim) return false;
    int tr = 128 / Q < P ? 128 / Q : P;
    const int per_image = (P + tr - 1) / tr;
    tr = (P + per_image - 1) / per_image;            // even out the tiles of an image
    pl->TR = tr;
    pl->nkg = (tr * Q + 31) / 32;
    if (tr * Q * 10 < pl->nkg * 32 * 6) return false;  // < 60 % of the slots used
    pl->PR = tr + d->R - 1;
    pl->PW = Q + d->S - 1;
    pl->ni = (pl->PR * pl->PW * 5 + 63) / 64;
    pl->tiles_per_image = per_image;
    const long long nt = (long long)d->N * per_image;
    if (nt > 0x7fffffff / 2) return false;
    pl->ntiles = (int)nt;
    // 32 x 64 tiles: 64 x 64 halve the operand bytes a block pulls per product but double the partial tiles, which
    // (written here, read back by the reduction kernel) are the larger part of this product's memory traffic; measured
    // slower on every benchmark layer
    pl->kt = kRowsKT;
    const int gi = 128 * pl->kt / 1024;
    if (gi + pl->ni > kRowsLoads * kRowsWaves) return false;   // load instructions per tile the waves share out
    pl->stages = 3;
    pl->lds = (size_t)pl->stages * (gi + pl->ni) * 1024 + 1024;
    if (pl->lds > 80 * 1024) return false;
    pl->tiles_k = d->K / pl->kt;
    pl->tiles_kc = pl->tiles_k * (d->C / 64);
    // One block of 8 waves per CU when the product has the chip to itself.  When the caller has said that it runs beside
    // other kernels (lpdt_qconv_set_wgrad_beside: the training step issues it on a second stream), what counts is how much
    // of the chip it takes from them and the bytes of partial tiles it moves: measured in the ResNet-18 step, 192 blocks
    // give the shortest step (128: +50 us, 256: +45 us, 512: +130 us), although alone they take 40 % longer than 256.
    long long target = beside ? 192 : 256;
#ifdef LPDT_TUNE
    if (const char *e = getenv("LPDT_WGRAD_ROWS_BLOCKS")) target = atoi(e);
#endif
    long long splits = target / pl->tiles_kc;
    if (splits > nt / 2) splits = nt / 2;             // at least two tiles per block: one to hide the other's loads
    if (splits < 1) splits = 1;
    pl->tiles_per_split = (int)((nt + splits - 1) / splits);
    pl->splits = (int)((nt + pl->tiles_per_split - 1) / pl->tiles_per_split);
    pl->out_len = (long long)d->K * ntaps * d->C;
    pl->partial_bytes = round_up((size_t)pl->splits * pl->out_len * sizeof(int32_t), 256);
    return true;
}

void launch_wgrad_rows(const lpdt_conv_desc *d, int P, int Q, const WgradRowsPlan &pl, const int8_t *g, const int8_t *x,
                       void *out, int out_mode, const float *sA, const float *sB, void *partial, hipStream_t st) {
    WgradRowsParams p = {};
    p.g = g; p.x = x; p.partial = static_cast<int32_t *>(partial);
    p.g_bytes = (unsigned)((size_t)d->N * P * Q * d->K); p.x_bytes = (unsigned)((size_t)d->N * d->H * d->W * d->C);
    p.K = d->K; p.C = d->C; p.H = d->H; p.W = d->W; p.P = P; p.Q = Q; p.S = d->S; p.pad_h = d->pad_h; p.pad_w = d->pad_w;
    p.ntaps = d->R * d->S;
    p.TR = pl.TR; p.PR = pl.PR; p.PW = pl.PW; p.ni = pl.ni; p.nkg = pl.nkg;
    p.tiles_per_image = pl.tiles_per_image; p.ntiles = pl.ntiles; p.tiles_per_split = pl.tiles_per_split;
    p.tiles_k = pl.tiles_k; p.tiles_kc = pl.tiles_kc; p.out_len = pl.out_len;
    p.inv_Q = 1.0f / (float)Q; p.inv_PW = 1.0f / (float)pl.PW;
    const unsigned grid = (unsigned)(pl.tiles_kc * pl.splits);
    auto go = [&](auto kernel) {
        static bool raised = false;
        if (!raised) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
            raised = true;
        }
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * kRowsWaves), pl.lds, st, p);
    };
    if (pl.splits == 1) {
        p.direct = out; p.direct_mode = out_mode; p.sA = sA; p.sB = sB;
        go(wgrad_rows_kernel<3>);
        return;
    }
    go(wgrad_rows_kernel<3>);
    launch_wgrad_reduce(p.partial, pl.out_len, pl.splits, out, out_mode, sA, sB, st);
}

}  // namespace lpdt
