// int8 convolution forward and backward-data with exact int32 accumulation (Table
// "hardware_training", row Conv) as an implicit GEMM on the gfx950 matrix cores
// (v_mfma_i32_32x32x32_i8), im2col-free.
//
//   out[pix][j] = sum_{tap, c} in[pix + tap][c] * wt[j][tap][c]        j = output channel
//
// The reduction axis is cut into 16-byte granules (16 channels of one filter tap); a K-step is
// 4 granules.  Both operands are fetched by 16-byte buffer loads in which 4 neighbouring lanes
// read the 64 contiguous bytes of one row (the access shape the texture path serves at full
// rate), staged through LDS in [granule][row][16 B] planes -- the operand order of the MFMA, so
// every LDS read is a contiguous ds_read_b128 -- and double buffered.
//
// What keeps the inner loop short:
//   * every row's image-border test is folded, once, into a bit mask over the filter taps; a
//     masked-off or out-of-range row is read at an offset beyond the buffer's size, for which
//     the hardware returns zeros: no branches, no selects on the data;
//   * the tap-dependent part of the gather address comes from a small LDS table built once per
//     block (one entry per granule of the block's K range);
//   * the weights are the MFMA's row operand, so a lane ends up with 4 consecutive output
//     channels of one pixel: 16-byte stores in the epilogue.
//
// Backward-data is the same kernel on the gradient tensor with the transposed filter.  With a
// stride s > 1 an input pixel only meets the taps of its own residue class ((h + pad) mod s,
// (w + pad) mod s); each class is a dense stride-1 problem over its sub-grid of pixels with its
// own sub-filter, so the s*s classes run as grid.y of one launch and no product with a zero is
// ever issued.
#include "qconv_igemm_plan.h"
#include <type_traits>

namespace lpdt {

namespace {

constexpr int kThreads = 256;
template <int N, typename F>
__device__ __forceinline__ void static_for(F f) {
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>());
    }
}

__device__ __forceinline__ int fast_div(int x, int d, unsigned mul) {
    return mul ? (int)__umulhi((unsigned)x, mul) : x / d;
}

// PF = K-steps whose global loads are in flight (held in registers) ahead of the one being multiplied.
// SPLIT: the reduction is shared between the blocks of grid.z, which add their int32 sums into a zeroed output; the pixels
// are then the MFMA's row operand, so that a lane's atomics of one instruction fall on consecutive addresses.
// KG = granules of a K-step (4 or 8): with 8 a row's fetch is one whole 128-byte cache line.
// ABSMAX (fp32 output, no split): every wave also leaves the largest |value| it stored in p.pabs, for a quantizer that
// follows without a normalisation layer in between.
template <int BM, int BN, int WM, int WN, int PF, bool SPLIT, int KG, bool ABSMAX = false>
__global__ __launch_bounds__(kThreads) void igemm_kernel(const IgemmParams p) {
    constexpr int PAD = 256 / KG;                                  // the KG planes start 64/KG banks apart
    constexpr int PLANE_A = BM * 16 + PAD, PLANE_B = BN * 16 + PAD;
    constexpr int BUF = KG * (PLANE_A + PLANE_B);
    constexpr int RPP = kThreads / KG;                             // rows per pass of the block's loads
    constexpr int RA = BM / RPP, RB = (BN + RPP - 1) / RPP;        // 16-byte items per thread
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    int4 *rows = reinterpret_cast<int4 *>(lds + 2 * BUF);
    int2 *tab = reinterpret_cast<int2 *>(lds + 2 * BUF + BM * sizeof(int4));

    const IgemmClass &c = p.cls[blockIdx.y];
    // Blocks are dealt to the 8 XCDs round-robin; renumber so that each XCD (one L2) works on a contiguous run of tiles.
    const int nb = gridDim.x, per = nb / 8, rem = nb % 8, xcd = blockIdx.x % 8;
    const int tile = xcd * per + min(xcd, rem) + blockIdx.x / 8;
    const int tile_n = tile % p.tiles_n, tile_m = tile / p.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    if (m0 >= c.M) {
        if (ABSMAX && threadIdx.x % 64 == 0) p.pabs[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 4 + threadIdx.x / 64] = 0.0f;
        return;
    }
    const int ks_begin = blockIdx.z * c.kps;
    const int ks_end = min(c.nk, ks_begin + c.kps);
    if (ks_begin >= ks_end && (blockIdx.z > 0)) return;

    const int t = threadIdx.x, lane = t % 64, wave = t / 64;
    const int g4 = t % KG, row0 = t / KG;

    // The K loop runs in rounds of PF steps with no conditions inside; steps past the block's range multiply zeros.
    const int nsteps = (ks_end - ks_begin + PF - 1) / PF * PF;
    // gather table: entry e = granule 4*ks_begin + e -> (byte offset of its tap and channels, tap slot); entries past
    // the range (the padded steps and the PF steps of read-ahead) name the empty slot
    for (int e = t; e < KG * (nsteps + PF); e += kThreads) {
        const int gi = KG * ks_begin + e;
        int2 v = {0, 31};
        if (gi < min(c.gtot, KG * ks_end)) {
            const int slot = fast_div(gi, p.gpt, p.mul_gpt), cg = gi - slot * p.gpt;
            const int ty = fast_div(slot, c.Sc, c.mul_sc), tx = slot - ty * c.Sc;
            v.x = (ty * p.IW + tx) * p.dsign * p.Cin + cg * 16;
            v.y = slot;
        }
        tab[e] = v;
    }

    // Row records, one per pixel of the tile, made by the first BM threads and shared through LDS: byte offset of the
    // pixel under tap (0,0), which taps stay inside the image, and the output pixel (-1: past the end).
    const int hw = c.OHs * c.OWs;
    if (t < BM) {
        const int m = m0 + t;
        int4 rec = {0, 0, -1, 0};
        if (m < c.M) {
            const int n = fast_div(m, hw, c.mul_hw), r = m - n * hw;
            const int qy = fast_div(r, c.OWs, c.mul_w), qx = r - qy * c.OWs;
            const int iy = qy * p.istep + c.iy0, ix = qx * p.istep + c.ix0;
            unsigned xm = 0, mk = 0;
            for (int tx = 0; tx < c.Sc; ++tx) xm |= (unsigned)((unsigned)(ix + tx * p.dsign) < (unsigned)p.IW) << tx;
            for (int ty = 0; ty < c.Rc; ++ty)
                if ((unsigned)(iy + ty * p.dsign) < (unsigned)p.IH) mk |= xm << (ty * c.Sc);
            rec.x = ((n * p.IH + iy) * p.IW + ix) * p.Cin;
            rec.y = (int)mk;
            rec.z = (n * p.OH + qy * p.ostep + c.oy0) * p.OW + (qx * p.ostep + c.ox0);
        }
        rows[t] = rec;
    }
    // this thread's rows of the filter tile
    unsigned boff[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        const int row = row0 + RPP * j;
        boff[j] = (row < BN && n0 + row < p.Cout) ? (unsigned)(c.wt_off + ((n0 + row) * c.gtot + g4) * 16) : kBeyond;
    }
    const __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.in), 0, (int)p.in_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_wt = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.wt), 0, (int)p.wt_bytes, 0x00020000);
    __syncthreads();  // table and row records complete
    int rowoff[RA];
    unsigned mask[RA];
#pragma unroll
    for (int j = 0; j < RA; ++j) {
        const int4 rec = rows[row0 + RPP * j];
        rowoff[j] = rec.x;
        mask[j] = (unsigned)rec.y;
    }

    v4u sa[PF][RA], sb[PF][RB];
    auto load_tiles = [&](auto slot_tag, int step) {  // step counts from the block's first K-step
        constexpr int SL = decltype(slot_tag)::value;
        const int2 e = tab[KG * step + g4];
#pragma unroll
        for (int j = 0; j < RA; ++j) {
            const unsigned off = ((mask[j] >> e.y) & 1u) ? (unsigned)(rowoff[j] + e.x) : kBeyond;
            sa[SL][j] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, off, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < RB; ++j)
            sb[SL][j] = __builtin_amdgcn_raw_buffer_load_b128(rs_wt, boff[j] + (unsigned)(ks_begin + step) * (16u * KG), 0, 0);
    };
    unsigned char *const st_a = lds + g4 * PLANE_A + row0 * 16;
    unsigned char *const st_b = lds + KG * PLANE_A + g4 * PLANE_B + row0 * 16;
    auto store_tiles = [&](auto slot_tag, int buf) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int j = 0; j < RA; ++j) *reinterpret_cast<v4u *>(st_a + buf * BUF + RPP * j * 16) = sa[SL][j];
#pragma unroll
        for (int j = 0; j < RB; ++j)
            if (BN % RPP == 0 || row0 + RPP * j < BN) *reinterpret_cast<v4u *>(st_b + buf * BUF + RPP * j * 16) = sb[SL][j];
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int wm = wave / WN, wn = wave % WN, half = lane / 32;
    const unsigned char *const rd_a = lds + half * PLANE_A + (wm * (BM / WM) + lane % 32) * 16;
    const unsigned char *const rd_b = lds + KG * PLANE_A + half * PLANE_B + (wn * (BN / WN) + lane % 32) * 16;

    // prologue: the first PF K-steps' loads go out together; register slot s holds step s (mod PF afterwards)
    static_for<PF>([&](auto s) { load_tiles(s, decltype(s)::value); });
    store_tiles(std::integral_constant<int, 0>(), 0);
    __syncthreads();
    static_assert(PF % 2 == 0, "the LDS buffer of a step is a compile-time constant only for an even PF");
    for (int base = 0; base < nsteps; base += PF) {
        static_for<PF>([&](auto u) {
            constexpr int U = decltype(u)::value;
            constexpr int buf = U & 1;
            load_tiles(u, base + U + PF);  // slot U went to LDS before this step: refill it
#pragma unroll
            for (int kk = 0; kk < KG / 2; ++kk) {
                v4i a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[i] = *reinterpret_cast<const v4i *>(rd_a + buf * BUF + 2 * kk * PLANE_A + 32 * i * 16);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[j] = *reinterpret_cast<const v4i *>(rd_b + buf * BUF + 2 * kk * PLANE_B + 32 * j * 16);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {  // filter rows are the MFMA's row operand, except in a split reduction
                        if (SPLIT) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
                        else acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[j], a[i], acc[i][j], 0, 0, 0);
                    }
            }
            store_tiles(std::integral_constant<int, (U + 1) % PF>(), buf ^ 1);
            __syncthreads();
        });
    }

    if constexpr (SPLIT) {  // lane: output channel lane%32 of the tile, pixels 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r16 = 0; r16 < 16; ++r16) {
                const int opix = rows[wm * (BM / WM) + 32 * i + 8 * (r16 / 4) + 4 * half + (r16 % 4)].z;
                if (opix < 0) continue;
                const size_t pix = (size_t)opix;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = n0 + wn * (BN / WN) + 32 * j + lane % 32;
                    if (col < p.Cout && acc[i][j][r16] != 0) atomicAdd(static_cast<int32_t *>(p.out) + pix * p.Cout + col, acc[i][j][r16]);
                }
            }
        return;
    }
    // Accumulator layout of the 32x32 MFMA: a lane holds column lane%32 (here: a pixel) and rows 8*(r/4) + 4*(lane/32) + r%4
    // (here: output channels), i.e. four runs of 4 consecutive channels.
    const float scale = p.out_mode ? __fmul_rn(*p.sA, *p.sB) : 0.0f;
    float am = 0.0f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int opix = rows[wm * (BM / WM) + 32 * i + lane % 32].z;
        if (opix < 0) continue;
        const size_t pix = (size_t)opix;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = n0 + wn * (BN / WN) + 32 * j + 8 * q + 4 * half;
                if (col >= p.Cout) continue;
                const v4i s = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                int32_t *dst = static_cast<int32_t *>(p.out) + pix * p.Cout + col;
                if (p.vec_out) {
                    if (p.out_mode) {  // the dequantizing scale applied here: same arithmetic as lpdt_dequantize
                        v4f *fdst = reinterpret_cast<v4f *>(dst);
                        const bool add = p.out_mode == 2;
                        v4f v = {0.f, 0.f, 0.f, 0.f};
                        if (add) v = *fdst;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = dequant_value(scale, s[e], v[e], add);
                        *fdst = v;
                        if (ABSMAX) am = fmaxf(fmaxf(am, fmaxf(fabsf(v[0]), fabsf(v[1]))), fmaxf(fabsf(v[2]), fabsf(v[3])));
                    } else *reinterpret_cast<v4i *>(dst) = s;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (col + e >= p.Cout) break;
                        if (p.out_mode) {
                            float *fdst = reinterpret_cast<float *>(dst + e);
                            const float v = dequant_value(scale, s[e], p.out_mode == 2 ? *fdst : 0.f, p.out_mode == 2);
                            *fdst = v;
                            if (ABSMAX) am = fmaxf(am, fabsf(v));
                        } else dst[e] = s[e];
                    }
                }
            }
        }
    }
    if (ABSMAX) {
        am = wave_max(am);
        if (lane == 0) p.pabs[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 4 + wave] = am;
    }
}

__global__ void fill_zero_kernel(int32_t *dst, size_t len) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < len; i += (size_t)gridDim.x * blockDim.x) dst[i] = 0;
}

// Filter panels for backward-data: class (cy,cx) holds wt[c][a][b][k] = w[k][cy + s*a][cx + s*b][c].
struct PackParams {
    int K, R, S, C, stride, nclasses;
    int off[kMaxClasses + 1];  // element offsets of the panels
    int Rc[kMaxClasses], Sc[kMaxClasses];
};
// A block transposes one 64 (c) x 64 (k) tile of one filter tap through LDS: 16-byte loads along c (contiguous in w),
// 16-byte stores along k (contiguous in the panel).  b = taps of all classes x c-tiles x k-tiles; C, K multiples of 16.
__device__ __forceinline__ void pack_filter_tile(const int8_t *__restrict__ w, int8_t *__restrict__ wt, const PackParams &q, int b,
                                                 unsigned char (*tile)[64 + 16]) {
    const int tc = (q.C + 63) / 64, tk = (q.K + 63) / 64;
    const int kt = b % tk; b /= tk;
    const int ct = b % tc; b /= tc;   // b = tap index over all classes
    int cl = 0;
    while (cl + 1 < q.nclasses && b >= q.Rc[cl] * q.Sc[cl]) { b -= q.Rc[cl] * q.Sc[cl]; ++cl; }
    const int slot = b, nslots = q.Rc[cl] * q.Sc[cl];
    const int tr = cl / q.stride + q.stride * (slot / q.Sc[cl]), ts = cl % q.stride + q.stride * (slot % q.Sc[cl]);
    const int k0 = kt * 64, c0 = ct * 64;
    const int row = threadIdx.x / 4, chunk = (threadIdx.x % 4) * 16;
    if (k0 + row < q.K && c0 + chunk < q.C)
        *reinterpret_cast<int4 *>(&tile[row][chunk]) =
            *reinterpret_cast<const int4 *>(w + ((size_t)((k0 + row) * q.R + tr) * q.S + ts) * q.C + c0 + chunk);
    __syncthreads();
    if (c0 + row < q.C && k0 + chunk < q.K) {   // this thread: channel c0 + row, 16 consecutive k
        unsigned int o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) o[j / 4] |= (unsigned int)tile[chunk + j][row] << (8 * (j % 4));
        *reinterpret_cast<int4 *>(wt + q.off[cl] + ((size_t)(c0 + row) * nslots + slot) * q.K + k0 + chunk) =
            make_int4((int)o[0], (int)o[1], (int)o[2], (int)o[3]);
    }
}
__global__ __launch_bounds__(256) void pack_filter_bwd_kernel(const int8_t *__restrict__ w, int8_t *__restrict__ wt, const PackParams q) {
    __shared__ unsigned char tile[64][64 + 16];  // [k][c], rows padded
    pack_filter_tile(w, wt, q, blockIdx.x, tile);
}
// The same for several filters in one launch (a network's filters are all final at the same moment, and a launch per
// filter is mostly launch latency): the table travels in the kernel arguments; a block finds its filter by its number.
constexpr int kPackBatch = 24;
struct PackBatch {
    int count;
    int first[kPackBatch + 1];   // first block of each filter
    PackParams pk[kPackBatch];
    const int8_t *w[kPackBatch];
    int8_t *wt[kPackBatch];
};
__global__ __launch_bounds__(256) void pack_filter_bwd_batch_kernel(const PackBatch t) {
    __shared__ unsigned char tile[64][64 + 16];
    int f = 0;
    while (f + 1 < t.count && (int)blockIdx.x >= t.first[f + 1]) ++f;
    pack_filter_tile(t.w[f], t.wt[f], t.pk[f], (int)blockIdx.x - t.first[f], tile);
}

unsigned div_multiplier(int d, long long xmax) {
    if (d <= 1 || xmax * d >= (1ll << 32)) return 0;
    return (unsigned)((1ull << 32) / (unsigned)d + 1);
}

struct Tile { int BM, BN, KG; };
// 128 x 64 tiles where they give at least one block per CU (measured faster than 64-row and than 256-row tiles on every
// such layer of the benchmark networks); deeper layers with few pixels take 64 x 64 tiles, which still fill the chip
// without splitting the reduction (so the scale can be applied in the epilogue).
Tile pick_tile(const IgemmParams &p) {
    if (p.Cout < 48) return {128, 32, 4};
    long long blocks = 0;
    int gmin = 1 << 30;
    for (int i = 0; i < p.nclasses; ++i) {
        blocks += (long long)((p.cls[i].M + 127) / 128) * ((p.Cout + 63) / 64);
        if (p.cls[i].gtot < gmin) gmin = p.cls[i].gtot;
    }
    // K-steps of 8 granules fetch whole 128-byte lines of a row and halve the barriers; a short reduction would pay for
    // them with padding (36 granules -> 5 steps of 8) and takes steps of 4
    return {blocks >= 256 ? 128 : 64, 64, gmin >= 64 ? 8 : 4};
}

constexpr int kMinSplitSteps = 24;   // K-steps below which a launch with few tiles keeps its reduction whole

// Fills tile counts and the K split; returns the grid.
dim3 finish_plan(IgemmParams *p, Tile tl, bool allow_split) {
    p->tiles_n = (p->Cout + tl.BN - 1) / tl.BN;
    p->kg = tl.KG;
    for (int i = 0; i < p->nclasses; ++i) p->cls[i].nk = (p->cls[i].gtot + tl.KG - 1) / tl.KG;
    long long blocks = 0;
    int max_tiles_m = 0, max_nk = 0;
    for (int i = 0; i < p->nclasses; ++i) {
        const int tm = (p->cls[i].M + tl.BM - 1) / tl.BM;
        blocks += (long long)tm * p->tiles_n;
        if (tm > max_tiles_m) max_tiles_m = tm;
        if (p->cls[i].nk > max_nk) max_nk = p->cls[i].nk;
    }
    int splits = 1;
    const int min_steps = 16 / tl.KG;                  // a share of the reduction is at least 16 granules deep
    // Too few tiles to fill 256 CUs: split the reduction -- when it is long enough to pay for the two launches a split
    // adds (zero fill before, scale after: ~8 us): a 64 -> 64 layer of ResNet-20 has 9 steps, and splitting them in two
    // made 15 us of launches out of a 7 us kernel.
    if (allow_split && blocks < 256 && max_nk >= 2 * min_steps && max_nk >= kMinSplitSteps) {
        splits = (int)((512 + blocks - 1) / blocks);
        if (splits > max_nk / min_steps) splits = max_nk / min_steps;
        if (splits < 1) splits = 1;
    }
    int zdim = 1;
    for (int i = 0; i < p->nclasses; ++i) {
        IgemmClass &c = p->cls[i];
        c.kps = c.nk > 0 ? (c.nk + splits - 1) / splits : 1;
        const int z = c.nk > 0 ? (c.nk + c.kps - 1) / c.kps : 1;
        if (z > zdim) zdim = z;
    }
    p->atomic_out = zdim > 1;
    return dim3((unsigned)(max_tiles_m * p->tiles_n), (unsigned)p->nclasses, (unsigned)zdim);
}

bool table_fits(const IgemmParams &p) {
    for (int i = 0; i < p.nclasses; ++i)
        if (p.kg * (p.cls[i].kps + 16) > kMaxTableEntries) return false;
    return true;
}

template <int BM, int BN, int WM, int WN, int PF, int KG>
void launch(const IgemmParams &p, dim3 grid, hipStream_t st) {
    int max_kps = 1;
    for (int i = 0; i < p.nclasses; ++i)
        if (p.cls[i].kps > max_kps) max_kps = p.cls[i].kps;
    const size_t lds = 2 * KG * ((BM * 16 + 256 / KG) + (BN * 16 + 256 / KG)) + BM * sizeof(int4) +
                       (size_t)((max_kps + PF - 1) / PF * PF + PF) * KG * sizeof(int2);
    auto go = [&](auto kernel) {
        if (lds > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds, st, p);
    };
    if (p.atomic_out) go(igemm_kernel<BM, BN, WM, WN, PF, true, KG>);
    else if (p.pabs) go(igemm_kernel<BM, BN, WM, WN, PF, false, KG, true>);
    else go(igemm_kernel<BM, BN, WM, WN, PF, false, KG>);
}

// When the result is ADDED to what the output holds (out_mode 2), pixels of a residue class without taps (a 1x1 stride-2
// filter reaches one pixel in four) stay as they are: their blocks are dropped from the launch, after the tile has been
// chosen for the whole problem.  Not when the maximum of the result is wanted, which has to visit every element.
dim3 drop_empty_classes(IgemmParams &p, dim3 grid) {
    if (p.out_mode != 2 || p.pabs) return grid;
    int n = 0;
    for (int i = 0; i < p.nclasses; ++i)
        if (p.cls[i].gtot > 0) p.cls[n++] = p.cls[i];
    p.nclasses = n;
    grid.y = (unsigned)n;
    return grid;
}

void run(IgemmParams &p, size_t out_len, hipStream_t st) {
    int cfg;
    dim3 dgrid;
    if (patch_plan(p)) {
        patch_launch(p, st);
        return;
    }
    if (dma_plan(&p, &cfg, &dgrid)) {
        dgrid = drop_empty_classes(p, dgrid);
        if (dgrid.y > 0) dma_launch(p, cfg, dgrid, st);
        return;
    }
    const Tile tl = pick_tile(p);
    dim3 grid = finish_plan(&p, tl, true);
    if (p.atomic_out) {
        const size_t len = out_len;
        size_t b = (len + 1023) / 1024;
        if (b > 4096) b = 4096;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)b), dim3(256), 0, st, static_cast<int32_t *>(p.out), len);
    } else {
        grid = drop_empty_classes(p, grid);
        if (grid.y == 0) return;
    }
    if (tl.BN == 32) launch<128, 32, 4, 1, 4, 4>(p, grid, st);
    else if (tl.BM == 64 && tl.KG == 8) launch<64, 64, 2, 2, 2, 8>(p, grid, st);
    else if (tl.BM == 64) launch<64, 64, 2, 2, 4, 4>(p, grid, st);
    else if (tl.KG == 8) launch<128, 64, 2, 2, 2, 8>(p, grid, st);
    else launch<128, 64, 2, 2, 4, 4>(p, grid, st);
}

void fwd_params(const lpdt_conv_desc *d, int P, int Q, IgemmParams *p) {
    *p = IgemmParams{};
    p->in_bytes = (unsigned)((size_t)d->N * d->H * d->W * d->C);
    p->wt_bytes = (unsigned)((size_t)d->K * d->R * d->S * d->C);
    p->Cin = d->C; p->Cout = d->K; p->gpt = d->C / 16;
    p->IH = d->H; p->IW = d->W; p->OH = P; p->OW = Q;
    p->istep = d->stride_h; p->ostep = 1; p->dsign = 1;
    p->nclasses = 1;
    IgemmClass &c = p->cls[0];
    c.M = d->N * P * Q; c.OHs = P; c.OWs = Q;
    c.oy0 = 0; c.ox0 = 0; c.iy0 = -d->pad_h; c.ix0 = -d->pad_w;
    c.Rc = d->R; c.Sc = d->S;
    c.gtot = d->R * d->S * p->gpt;
    c.wt_off = 0;
    c.mul_hw = div_multiplier(P * Q, c.M);
    c.mul_w = div_multiplier(Q, (long long)P * Q);
    c.mul_sc = div_multiplier(c.Sc, kMaxTaps + 1);
    p->mul_gpt = div_multiplier(p->gpt, (long long)c.gtot + 64);
}

// Residue classes of backward-data.  Returns false when a class would be empty of pixels only (those are dropped).
void bwd_params(const lpdt_conv_desc *d, int P, int Q, IgemmParams *p, PackParams *pk) {
    *p = IgemmParams{};
    *pk = PackParams{};
    const int s = d->stride_h, pad = d->pad_h;
    p->in_bytes = (unsigned)((size_t)d->N * P * Q * d->K);
    p->wt_bytes = (unsigned)((size_t)d->K * d->R * d->S * d->C);
    p->Cin = d->K; p->Cout = d->C; p->gpt = d->K / 16;
    p->IH = P; p->IW = Q; p->OH = d->H; p->OW = d->W;
    p->istep = 1; p->ostep = s; p->dsign = -1;
    pk->K = d->K; pk->R = d->R; pk->S = d->S; pk->C = d->C; pk->stride = s; pk->nclasses = s * s;
    int n = 0, woff = 0;
    for (int cy = 0; cy < s; ++cy)
        for (int cx = 0; cx < s; ++cx) {
            const int cl = cy * s + cx;
            const int Rc = cy < d->R ? (d->R - 1 - cy) / s + 1 : 0, Sc = cx < d->S ? (d->S - 1 - cx) / s + 1 : 0;
            pk->off[cl] = woff; pk->Rc[cl] = Rc; pk->Sc[cl] = Sc;
            const int h0 = ((cy - pad) % s + s) % s, w0 = ((cx - pad) % s + s) % s;  // first pixel of the class
            const int OHs = h0 < d->H ? (d->H - 1 - h0) / s + 1 : 0, OWs = w0 < d->W ? (d->W - 1 - w0) / s + 1 : 0;
            if (OHs > 0 && OWs > 0) {
                IgemmClass &c = p->cls[n++];
                c.M = d->N * OHs * OWs; c.OHs = OHs; c.OWs = OWs;
                c.oy0 = h0; c.ox0 = w0;
                c.iy0 = (h0 + pad - cy) / s; c.ix0 = (w0 + pad - cx) / s;
                c.Rc = Rc; c.Sc = Sc;
                c.gtot = Rc * Sc * p->gpt;
                c.wt_off = woff;
                c.mul_hw = div_multiplier(OHs * OWs, c.M);
                c.mul_w = div_multiplier(OWs, (long long)OHs * OWs);
                c.mul_sc = div_multiplier(Sc, kMaxTaps + 1);
            }
            woff += Rc * Sc * d->K * d->C;
        }
    pk->off[s * s] = woff;
    p->nclasses = n;
    p->mul_gpt = div_multiplier(p->gpt, (long long)d->R * d->S * p->gpt + 64);
}

bool sizes_ok(const lpdt_conv_desc *d, int P, int Q) {
    const size_t lim = (size_t)1 << 31;
    return (size_t)d->N * d->H * d->W * d->C < lim - 4096 && (size_t)d->N * P * Q * d->K < lim - 4096 &&
           (size_t)d->K * d->R * d->S * d->C < lim - 4096 && d->stride_h == d->stride_w && d->pad_h == d->pad_w;
}

}  // namespace

bool igemm_fwd_supported(const lpdt_conv_desc *d, int P, int Q) {
    if (!(d->C % 16 == 0 && sizes_ok(d, P, Q) && d->R <= 8 && d->S <= 8 && d->R * d->S <= kMaxTaps)) return false;
    IgemmParams p;
    fwd_params(d, P, Q, &p);
    finish_plan(&p, pick_tile(p), true);
    return table_fits(p);
}

bool igemm_bwd_data_supported(const lpdt_conv_desc *d, int P, int Q) {
    if (!(d->K % 16 == 0 && sizes_ok(d, P, Q) && d->stride_h <= 2)) return false;
    IgemmParams p;
    PackParams pk;
    bwd_params(d, P, Q, &p, &pk);
    for (int i = 0; i < p.nclasses; ++i)  // the tap mask of a class has 31 bits
        if (p.cls[i].Rc > 8 || p.cls[i].Sc > 8 || p.cls[i].Rc * p.cls[i].Sc > kMaxTaps) return false;
    finish_plan(&p, pick_tile(p), true);
    return table_fits(p);
}

// Waves of the launch (= abs-max partials an ABSMAX kernel writes); 0 when the reduction is split
static int plan_waves(IgemmParams &p) {
    int cfg;
    dim3 dgrid;
    p.vec_out = p.Cout % 4 == 0;   // the fp32 entry points, the only ones with this output, take 16-byte aligned results
    if (dma_plan(&p, &cfg, &dgrid)) return dma_absmax_parts(cfg, dgrid);
    const dim3 grid = finish_plan(&p, pick_tile(p), true);
    return p.atomic_out ? 0 : (int)(grid.x * grid.y * 4);
}
int igemm_fwd_absmax_parts(const lpdt_conv_desc *d, int P, int Q) {
    IgemmParams p;
    fwd_params(d, P, Q, &p);
    return plan_waves(p);
}
int igemm_bwd_data_absmax_parts(const lpdt_conv_desc *d, int P, int Q) {
    IgemmParams p;
    PackParams pk;
    bwd_params(d, P, Q, &p, &pk);
    return plan_waves(p);
}

// whether a launch with a 16-byte aligned result splits its reduction
static bool plan_is_split(IgemmParams &p) {
    int cfg;
    dim3 dgrid;
    p.vec_out = p.Cout % 4 == 0;
    if (patch_plan(p) || dma_plan(&p, &cfg, &dgrid)) return false;
    finish_plan(&p, pick_tile(p), true);
    return p.atomic_out != 0;
}

// 50: the filter-resident row-tile kernel; 20 + tile of the direct-to-LDS kernel, or 10 + variant of the register-staged one (0: 128 x 32, 1: 64 x 64 with 4-granule
// steps, 2: 64 x 64 with 8, 3: 128 x 64 with 4, 4: 128 x 64 with 8), + 100 when the reduction is split over blocks
static int plan_kernel_id(IgemmParams &p) {
    int cfg;
    dim3 dgrid;
    p.vec_out = p.Cout % 4 == 0;
    if (patch_plan(p)) return 50;
    if (dma_plan(&p, &cfg, &dgrid)) return 20 + cfg;
    const Tile tl = pick_tile(p);
    finish_plan(&p, tl, true);
    const int v = tl.BN == 32 ? 0 : (tl.BM == 64 ? 1 : 3) + (tl.KG == 8 ? 1 : 0);
    return 10 + v + (p.atomic_out ? 100 : 0);
}
int igemm_fwd_kernel_id(const lpdt_conv_desc *d, int P, int Q) {
    IgemmParams p;
    fwd_params(d, P, Q, &p);
    return plan_kernel_id(p);
}
int igemm_bwd_data_kernel_id(const lpdt_conv_desc *d, int P, int Q) {
    IgemmParams p;
    PackParams pk;
    bwd_params(d, P, Q, &p, &pk);
    return plan_kernel_id(p);
}

bool igemm_fwd_is_split(const lpdt_conv_desc *d, int P, int Q) {
    IgemmParams p;
    fwd_params(d, P, Q, &p);
    return plan_is_split(p);
}

bool igemm_bwd_data_is_split(const lpdt_conv_desc *d, int P, int Q) {
    IgemmParams p;
    PackParams pk;
    bwd_params(d, P, Q, &p, &pk);
    return plan_is_split(p);
}

void launch_igemm_fwd(const lpdt_conv_desc *d, int P, int Q, const int8_t *x, const int8_t *w, void *out, int out_mode,
                      const float *sA, const float *sB, hipStream_t st, float *pabs) {
    IgemmParams p;
    fwd_params(d, P, Q, &p);
    p.in = x; p.wt = w; p.out = out; p.out_mode = out_mode; p.sA = sA; p.sB = sB; p.pabs = pabs;
    p.vec_out = d->K % 4 == 0 && aligned(out, 16);
    run(p, (size_t)d->N * P * Q * d->K, st);
}

bool igemm_fwd_stats_supported(const lpdt_conv_desc *d, int P, int Q) {
    if (!igemm_fwd_supported(d, P, Q)) return false;
    IgemmParams p;
    fwd_params(d, P, Q, &p);
    p.vec_out = d->K % 4 == 0;
    p.out_mode = 1;
    p.pix_per_sample = P * Q;
    int cfg;
    dim3 grid;
    return dma_plan(&p, &cfg, &grid) && dma_stats_supported(p, cfg);
}

void launch_igemm_fwd_stats(const lpdt_conv_desc *d, int P, int Q, const int8_t *x, const int8_t *w, float *out, int out_mode,
                            const float *sA, const float *sB, unsigned *cstats, const float *vpar, hipStream_t st) {
    IgemmParams p;
    fwd_params(d, P, Q, &p);
    p.in = x; p.wt = w; p.out = out; p.out_mode = out_mode; p.sA = sA; p.sB = sB;
    p.vec_out = 1;
    p.cstats = cstats; p.vpar = vpar; p.pix_per_sample = P * Q;
    int cfg;
    dim3 grid;
    if (dma_plan(&p, &cfg, &grid)) dma_launch(p, cfg, grid, st);   // igemm_fwd_stats_supported said so
}

size_t igemm_bwd_filter_panel_bytes(const lpdt_conv_desc *d) { return (size_t)d->K * d->R * d->S * d->C; }

static int pack_blocks(const PackParams &pk) {
    int taps = 0;
    for (int cl = 0; cl < pk.nclasses; ++cl) taps += pk.Rc[cl] * pk.Sc[cl];
    return taps * ((pk.C + 63) / 64) * ((pk.K + 63) / 64);
}

void launch_igemm_pack_bwd_filter(const lpdt_conv_desc *d, int P, int Q, const int8_t *w, void *panel, hipStream_t st) {
    IgemmParams p;
    PackParams pk;
    bwd_params(d, P, Q, &p, &pk);
    const int b = pack_blocks(pk);
    if (b > 0) hipLaunchKernelGGL(pack_filter_bwd_kernel, dim3((unsigned)b), dim3(256), 0, st, w, static_cast<int8_t *>(panel), pk);
}

void launch_igemm_pack_bwd_filters(const lpdt_conv_desc *descs, int count, const int8_t *const *w, void *const *panels, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kPackBatch) {
        PackBatch t;
        t.count = 0;
        t.first[0] = 0;
        for (int i = i0; i < count && i < i0 + kPackBatch; ++i) {
            const lpdt_conv_desc *d = descs + i;
            IgemmParams p;
            PackParams pk;
            bwd_params(d, (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1, (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1, &p, &pk);
            const int b = pack_blocks(pk);
            if (b == 0) continue;
            const int k = t.count++;
            t.pk[k] = pk; t.w[k] = w[i]; t.wt[k] = static_cast<int8_t *>(panels[i]);
            t.first[k + 1] = t.first[k] + b;
        }
        if (t.count > 0)
            hipLaunchKernelGGL(pack_filter_bwd_batch_kernel, dim3((unsigned)t.first[t.count]), dim3(256), 0, st, t);
    }
}

void launch_igemm_bwd_data(const lpdt_conv_desc *d, int P, int Q, const int8_t *g, const void *panel, void *out, int out_mode,
                           const float *sA, const float *sB, hipStream_t st, float *pabs) {
    IgemmParams p;
    PackParams pk;
    bwd_params(d, P, Q, &p, &pk);
    p.in = g; p.wt = static_cast<const int8_t *>(panel); p.out = out; p.out_mode = out_mode; p.sA = sA; p.sB = sB; p.pabs = pabs;
    p.vec_out = d->C % 4 == 0 && aligned(out, 16);
    run(p, (size_t)d->N * d->H * d->W * d->C, st);
}

}  // namespace lpdt
