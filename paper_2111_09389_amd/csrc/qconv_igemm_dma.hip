// int8 convolution forward / backward-data (Table "hardware_training", row Conv) as an implicit GEMM whose operand
// tiles go from global memory straight into LDS (buffer loads with the LDS bit: no staging registers, no LDS store
// instructions), for reductions whose channel count is a multiple of 64.
//
//   out[pix][j] = sum_{tap, c} in[pix + tap][c] * wt[j][tap][c]
//
// A K-step is KB = 64 or 128 channels of one filter tap (KB divides the channel count), so the tap (hence the border
// test and the gather offset) is the same for the whole block and lives in scalar registers; the steps visit all taps
// of a channel chunk before the next chunk, which keeps the input lines of a tile in the CU's vector cache.  LDS holds S stages of [BM pixel rows][KB] + [BN filter rows][KB].  A wave's load
// instruction fills 1 KiB: 1024/KB rows, lane -> (row, 16-byte slot); the lane fetches the granule slot ^ swz(row) of
// its row, swz = the bit-reversed row bits just above the bank period, which makes the MFMA operand reads (lane = row,
// 16 bytes) free of bank conflicts whichever way the hardware groups the lanes of a ds_read_b128 (counters: none).
// Masked rows (image border, past the end) fetch at an offset beyond the buffer, for which the hardware delivers zeros.
//
// Pipeline per step: wait until this wave's loads of the step have landed (vmcnt counts exactly: every step issues the
// same number of loads, the steps past the end fetch nothing), barrier, issue the loads of step + S-1 into the stage
// that was multiplied last, multiply the current stage.  One barrier per step; S-1 steps of loads in flight.
//
// What bounds it (counters and timing-only builds on a 16384 x 768 x 3072 product): the matrix cores run at their
// full rate when fed from registers (at the ~1.9 GHz the chip sustains under this load), the LDS reads are free of
// conflicts, and the L2 cache delivers about 0.6 requests of 64 bytes per cycle and channel: 10-15 TB/s for the whole
// chip, only 2-3 times the HBM rate, so the bytes a tile re-reads through L2 decide the speed.  A variant in which the
// two waves of a SIMD alternate between loading and multiplying was slower than this loop and was dropped.
#include "qconv_igemm_plan.h"
#include "norm_geom.h"
#include <type_traits>
#ifdef LPDT_TUNE
#include <cstdlib>
#endif

namespace lpdt {

namespace {

__device__ __forceinline__ int fast_div(int x, int d, unsigned mul) {
    return mul ? (int)__umulhi((unsigned)x, mul) : x / d;
}

typedef __attribute__((address_space(3))) void lds_void;
// added to a filter offset (a valid one below 2^30, or kBeyond) it gives an offset no filter reaches, without wrapping
constexpr unsigned kBeyondStep = 0x40000000u;

template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    // vmcnt(N): at most N of this wave's loads still in flight; lgkmcnt(0): its LDS reads of the previous stage are done
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <int N, typename F>
__device__ __forceinline__ void static_for(F f) {
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>());
    }
}

template <int KB> __device__ __forceinline__ int row_swz(int row) {
    if (KB == 64) return ((row >> 3) & 1) | ((row >> 1) & 2);                         // bits 2..3 reversed
    return ((row >> 3) & 1) | ((row >> 1) & 2) | ((row << 1) & 4);                    // bits 1..3 reversed
}

// TM x TN MFMA tiles (32 x 32) per wave, WGM x WGN waves per block, S LDS stages of KB (64 or 128) bytes of the reduction.
// Passes of the staged epilogue: the tile goes through LDS in 1, 2 or 4 runs of whole wave rows so that a run ([rows][BN + 4]
// words, plus the statistics array when one is taken) fits the operand stages; 0: it does not fit (direct epilogue).
constexpr int staged_passes(int BM, int BN, int WGM, int stage_bytes, int extra) {
    for (int ps = 1; ps <= 4; ps *= 2)
        if (WGM % ps == 0 && (BM / ps) * (BN + 4) * 4 + extra <= stage_bytes) return ps;
    return 0;
}

// ABSMAX: every wave leaves the largest |value| it stored.  STATS: the per-sample, per-channel extremes of the stored
// values x and of u = x * hardsigmoid(v x) go to p.cstats (needs the staged epilogue).
template <int TM, int TN, int WGM, int WGN, int S, int KB, bool ABSMAX, bool STAGED, bool STATS>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_dma_kernel(const IgemmParams p) {
    constexpr int NW = WGM * WGN;
    constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN;
    constexpr int STAGE = (BM + BN) * KB;
    constexpr int RPI = 1024 / KB, LPR = KB / 16, NKK = KB / 32;   // rows per load instruction, lanes per row, MFMA K-chunks per step
    constexpr int LA = BM / RPI / NW, LB = BN / RPI / NW;
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "every wave issues the same number of loads");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    int *const opix_tab = reinterpret_cast<int *>(lds + S * STAGE);   // output pixel of every tile row (-1: none)
    int *const slot_tab = opix_tab + BM;                              // STATS: the row's sample, counted from the tile's first

    const IgemmClass &c = p.cls[blockIdx.y];
    const int nb = gridDim.x, per = nb / 8, rem = nb % 8, xcd = blockIdx.x % 8;
    const int tile = xcd * per + min(xcd, rem) + blockIdx.x / 8;
    const int tile_n = tile % p.tiles_n, tile_m = tile / p.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int t = threadIdx.x, lane = t % 64, wave = __builtin_amdgcn_readfirstlane(t / 64);
    if (m0 >= c.M) {
        if (ABSMAX && lane == 0) p.pabs[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * NW + wave] = 0.0f;
        return;
    }
    // A step is KB channels of one filter tap (the channel count is a multiple of KB).  Steps run over the taps first and
    // the channel chunks second: consecutive steps then read nearly the same input lines (one pixel or one image row
    // further), which the CU's vector cache still holds, instead of fetching every input line once per tap from L2.
    const int ntaps = c.Rc * c.Sc;
    const int nsteps = ntaps * (p.Cin / KB);

    const int lrow = lane / LPR, lslot = lane % LPR;
    // the 16-byte granule of the step this lane fetches for a row: slot ^ swz(row); the swizzle's top bit comes from the
    // instruction's number, the rest from the lane
    const int hw = c.OHs * c.OWs;
    int aoff[LA];
    unsigned amask[LA];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int row = (wave * LA + j) * RPI + lrow, m = m0 + row;
        int off = 0, opix = -1;
        unsigned mk = 0;
        if (m < c.M) {
            const int n = fast_div(m, hw, c.mul_hw), r = m - n * hw;
            const int qy = fast_div(r, c.OWs, c.mul_w), qx = r - qy * c.OWs;
            const int iy = qy * p.istep + c.iy0, ix = qx * p.istep + c.ix0;
            unsigned xm = 0;
            for (int tx = 0; tx < c.Sc; ++tx) xm |= (unsigned)((unsigned)(ix + tx * p.dsign) < (unsigned)p.IW) << tx;
            for (int ty = 0; ty < c.Rc; ++ty)
                if ((unsigned)(iy + ty * p.dsign) < (unsigned)p.IH) mk |= xm << (ty * c.Sc);
            off = ((n * p.IH + iy) * p.IW + ix) * p.Cin + (lslot ^ row_swz<KB>(row)) * 16;
            opix = (n * p.OH + qy * p.ostep + c.oy0) * p.OW + (qx * p.ostep + c.ox0);
        }
        aoff[j] = off;
        amask[j] = mk;
        if (lslot == 0) {
            opix_tab[row] = opix;
            if (STATS) slot_tab[row] = opix >= 0 ? opix / p.pix_per_sample - m0 / p.pix_per_sample : 0;
        }
    }
    unsigned boff[LB];
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int brow = (wave * LB + j) * RPI + lrow, col = n0 + brow;
        boff[j] = col < p.Cout ? (unsigned)(c.wt_off + (col * c.gtot + (lslot ^ row_swz<KB>(brow))) * 16) : kBeyond;
    }
    const __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.in), 0, (int)p.in_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_wt = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.wt), 0, (int)p.wt_bytes, 0x00020000);

    // the step whose loads go out next (all uniform): its tap (slot 31, never set in a row's mask, past the end), the
    // tap's byte offset in the input and the step's byte offset inside a filter row
    int l_step = 0, l_tx = 0, l_ty = 0, l_chunk = 0, l_stage = 0;
    auto issue_loads = [&]() {
        const bool live = l_step < nsteps;
        const unsigned slot = live ? (unsigned)(l_ty * c.Sc + l_tx) : 31u;
        const int tapoff = (l_ty * p.IW + l_tx) * p.dsign * p.Cin + l_chunk;
        const unsigned bstep = live ? (unsigned)((l_ty * c.Sc + l_tx) * p.Cin + l_chunk) : kBeyondStep;
        ++l_step;
        if (++l_tx == c.Sc) {
            l_tx = 0;
            if (++l_ty == c.Rc) { l_ty = 0; l_chunk += KB; }
        }
        unsigned char *const base = lds + l_stage * STAGE;
        {
#pragma unroll
            for (int j = 0; j < LA; ++j) {
                const unsigned off = ((amask[j] >> slot) & 1u) ? (unsigned)(aoff[j] + tapoff) : kBeyond;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_in, (lds_void *)(base + (wave * LA + j) * 1024), 16, off, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < LB; ++j) {
                const unsigned off = boff[j] + bstep;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wt, (lds_void *)(base + BM * KB + (wave * LB + j) * 1024), 16, off, 0, 0, 0);
            }
        }
        l_stage = l_stage + 1 == S ? 0 : l_stage + 1;
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int wm = wave / WGN, wn = wave % WGN, half = lane >> 5, r32 = lane & 31;
    const int g0 = half ^ row_swz<KB>(r32);               // K-chunk kk reads the 16-byte slot g0 ^ 2*kk of its row
    const int rd_a = (wm * TM * 32 + r32) * KB, rd_b = BM * KB + (wn * TN * 32 + r32) * KB;

#pragma unroll
    for (int s = 0; s < S - 1; ++s) issue_loads();
    int stage = 0;
    for (int step = 0; step < nsteps; ++step) {
        wait_loads_and_barrier<(LA + LB) * (S - 2)>();
        issue_loads();
        const unsigned char *const sb = lds + stage * STAGE;
        stage = stage + 1 == S ? 0 : stage + 1;
        static_for<NKK>([&](auto kkc) {
            constexpr int kk = decltype(kkc)::value;
            const int g = (g0 ^ (2 * kk)) * 16;
            v4i a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const v4i *>(sb + rd_a + i * 32 * KB + g);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const v4i *>(sb + rd_b + j * 32 * KB + g);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)  // filter rows are the MFMA's row operand: a lane ends with 4 consecutive channels
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[j], a[i], acc[i][j], 0, 0, 0);
        });
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the empty loads of the last S-1 steps

    // Accumulator layout of the 32x32 MFMA: a lane holds column lane%32 (a pixel) and rows 8*q + 4*(lane/32) + 0..3
    // (output channels), q = 0..3.
    if constexpr (STAGED) {
        // The tile goes through LDS (the operand stages are free now) as [pixel][BN + 4 words], so that the stores to
        // global memory run along the channels: a pixel's BN results are one contiguous run instead of 16-byte pieces
        // BN*4 bytes apart.  The scale (and the addition, out_mode 2) is applied on the way out, with the arithmetic of
        // lpdt_dequantize.  A thread keeps one quad of channels for all its pixels, which is what lets it carry the
        // running extremes of its four channels in registers when the layer's statistics are taken.
        constexpr int RS = BN + 4, NT = 64 * NW, QPR = BN / 4;   // row stride in words, threads, 16-byte pieces per pixel
        constexpr int SB = STATS ? kStatSlots * BN * 16 : 0;
        constexpr int PASSES = staged_passes(BM, BN, WGM, S * STAGE, SB), RP = BM / PASSES;
        static_assert(PASSES > 0, "the staged tile fits the operand stages");
        int *const stg = reinterpret_cast<int *>(lds);
        unsigned *const sst = reinterpret_cast<unsigned *>(lds + RP * RS * 4);   // [slot][channel of the tile][4]
        const float scale = p.out_mode ? __fmul_rn(*p.sA, *p.sB) : 0.0f;
        const int cq = t % QPR, col = n0 + cq * 4;
        float am = 0.0f;
        // running extremes of this thread's channels over its pixels of the current sample: x max, x min, u max, u min
        float ex[4][4], vv[4];
        int cur = -1;
        if constexpr (STATS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) vv[e] = col + e < p.Cout ? p.vpar[col + e] : 0.0f;
        }
        auto flush = [&]() {
            if (cur < 0) return;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                unsigned *d = sst + ((cur * BN + cq * 4 + e) << 2);
                atomicMax(d + 0, ordered_bits(ex[e][0]));
                atomicMax(d + 1, ~ordered_bits(ex[e][1]));
                atomicMax(d + 2, ordered_bits(ex[e][2]));
                atomicMax(d + 3, ~ordered_bits(ex[e][3]));
            }
        };
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // main loop (or the previous run's reads) done everywhere
            if (STATS && ps == 0)
                for (int i = t; i < kStatSlots * BN * 4; i += NT) sst[i] = 0u;
            if (wm / (WGM / PASSES) == ps) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            *reinterpret_cast<v4i *>(stg + ((wm % (WGM / PASSES)) * TM * 32 + 32 * i + r32) * RS + (wn * TN + j) * 32 + 8 * q + 4 * half) =
                                v4i{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            }
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            auto store_rows = [&](auto add_mode) {
              constexpr bool kAdd = decltype(add_mode)::value;
                // rows in groups of 4: a call that adds to the result tensor fetches the group's four old values before it
                // stores anything (row by row, each fetch had to wait for the store before it: the compiler cannot tell
                // that the two never touch the same address, and a wait for a load is also a wait for every older store)
                constexpr int RSTEP = NT / QPR, RU = 4;
                for (int pr0 = t / QPR; pr0 < RP; pr0 += RU * RSTEP) {
                  int opx[RU];
                  v4f old[RU];
#pragma unroll
                  for (int u = 0; u < RU; ++u) {
                      const int pr = pr0 + u * RSTEP;
                      opx[u] = pr < RP ? opix_tab[ps * RP + pr] : -1;
                      old[u] = v4f{0.f, 0.f, 0.f, 0.f};
                      if (kAdd && opx[u] >= 0)
                          old[u] = *reinterpret_cast<const v4f *>(static_cast<const float *>(p.out) + (size_t)opx[u] * p.Cout + col);
                  }
                  // one wait for the four fetches, stated here so that the compiler does not put one in front of every store
                  if (kAdd) __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0)
#pragma unroll
                  for (int u = 0; u < RU; ++u) {
                    const int pr = pr0 + u * RSTEP, opix = opx[u];
                    if (opix < 0) continue;
                    const v4i sv = *reinterpret_cast<const v4i *>(stg + pr * RS + cq * 4);
                    int32_t *dst = static_cast<int32_t *>(p.out) + (size_t)opix * p.Cout + col;
                    if (p.out_mode) {
                        v4f *fdst = reinterpret_cast<v4f *>(dst);
                        const bool add = kAdd;
                        v4f v = old[u];
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = dequant_value(scale, sv[e], v[e], add);
                        *fdst = v;
                        if (ABSMAX) am = fmaxf(fmaxf(am, fmaxf(fabsf(v[0]), fabsf(v[1]))), fmaxf(fabsf(v[2]), fabsf(v[3])));
                        if constexpr (STATS) {
                            const int slot = slot_tab[ps * RP + pr];
                            if (slot != cur) {
                                flush();
                                cur = slot;
#pragma unroll
                                for (int e = 0; e < 4; ++e) { ex[e][0] = -INFINITY; ex[e][1] = INFINITY; ex[e][2] = -INFINITY; ex[e][3] = INFINITY; }
                            }
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float u = ren_u(v[e], vv[e]);
                                ex[e][0] = fmaxf(ex[e][0], v[e]); ex[e][1] = fminf(ex[e][1], v[e]);
                                ex[e][2] = fmaxf(ex[e][2], u); ex[e][3] = fminf(ex[e][3], u);
                            }
                        }
                    } else *reinterpret_cast<v4i *>(dst) = sv;
                  }
                }
            };
            // (two instantiations: with one loop for both, the compiler kept a wait for the fetches in front of every store)
            if (col < p.Cout) {
                if (p.out_mode == 2) store_rows(std::true_type{});
                else store_rows(std::false_type{});
            }
        }
        if (ABSMAX) {
            am = wave_max(am);
            if (lane == 0) p.pabs[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * NW + wave] = am;
        }
        if constexpr (STATS) {
            flush();
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const int n_first = m0 / p.pix_per_sample;
            const int n_last = (min(m0 + BM, c.M) - 1) / p.pix_per_sample;
            for (int i = t; i < (n_last - n_first + 1) * BN * 4; i += NT) {
                const unsigned k = sst[i];
                const int ch = n0 + (i >> 2) % BN;
                if (k && ch < p.Cout) atomicMax(p.cstats + (((size_t)(n_first + (i >> 2) / BN) * p.Cout + ch) << 2) + (i & 3), k);
            }
        }
        return;
    }
    const float scale = p.out_mode ? __fmul_rn(*p.sA, *p.sB) : 0.0f;
    float am = 0.0f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int opix = opix_tab[wm * TM * 32 + 32 * i + r32];
        if (opix < 0) continue;
        const size_t pix = (size_t)opix;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = n0 + (wn * TN + j) * 32 + 8 * q + 4 * half;
                if (col >= p.Cout) continue;
                const v4i s = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                int32_t *dst = static_cast<int32_t *>(p.out) + pix * p.Cout + col;
                if (p.out_mode) {
                    v4f *fdst = reinterpret_cast<v4f *>(dst);
                    const bool add = p.out_mode == 2;
                    v4f v = {0.f, 0.f, 0.f, 0.f};
                    if (add) v = *fdst;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = dequant_value(scale, s[e], v[e], add);
                    *fdst = v;
                    if (ABSMAX) am = fmaxf(fmaxf(am, fmaxf(fabsf(v[0]), fabsf(v[1]))), fmaxf(fabsf(v[2]), fabsf(v[3])));
                } else *reinterpret_cast<v4i *>(dst) = s;
            }
        }
    }
    if (ABSMAX) {
        am = wave_max(am);
        if (lane == 0) p.pabs[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * NW + wave] = am;
    }
}

struct DmaTile { int TM, TN, WGM, WGN, S, KB; };
// 0: 256 x 256, 64-byte steps   1: 128 x 128, 128-byte steps, 8 waves   2: 128 x 128, 64-byte steps, 4 waves (two blocks per CU)
// 3: 64 x 128, 128-byte steps
constexpr DmaTile kTiles[] = {{4, 2, 2, 4, 4, 64}, {2, 1, 2, 4, 4, 128}, {2, 2, 2, 2, 4, 64}, {1, 1, 2, 4, 4, 128}, {2, 2, 4, 2, 3, 64}};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

inline int tile_bm(int cfg) { return 32 * kTiles[cfg].TM * kTiles[cfg].WGM; }
inline int tile_bn(int cfg) { return 32 * kTiles[cfg].TN * kTiles[cfg].WGN; }
inline int tile_waves(int cfg) { return kTiles[cfg].WGM * kTiles[cfg].WGN; }
inline size_t tile_lds(int cfg) { return (size_t)kTiles[cfg].S * (tile_bm(cfg) + tile_bn(cfg)) * kTiles[cfg].KB + (size_t)tile_bm(cfg) * 8; }

long long tiles_of(const IgemmParams &p, int cfg) {
    long long blocks = 0;
    const int tn = (p.Cout + tile_bn(cfg) - 1) / tile_bn(cfg);
    for (int i = 0; i < p.nclasses; ++i) blocks += (long long)((p.cls[i].M + tile_bm(cfg) - 1) / tile_bm(cfg)) * tn;
    return blocks;
}

template <int TM, int TN, int WGM, int WGN, int S, int KB>
void launch_cfg(const IgemmParams &p, dim3 grid, size_t lds, hipStream_t st) {
    auto go = [&](auto kernel) {
        static bool raised = false;  // the limit is a property of the kernel: raised once
        if (!raised && lds > 48 * 1024) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            raised = true;
        }
        hipLaunchKernelGGL(kernel, grid, dim3(64 * WGM * WGN), lds, st, p);
    };
    constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN, STAGES = S * (BM + BN) * KB;
    constexpr bool FITS = staged_passes(BM, BN, WGM, STAGES, 0) > 0;                      // the result tile can go through LDS
    constexpr bool FITS_STATS = staged_passes(BM, BN, WGM, STAGES, kStatSlots * BN * 16) > 0;
    bool staged = FITS;
#ifdef LPDT_TUNE
    if (const char *e = getenv("LPDT_DMA_EPI")) staged = FITS && atoi(e) != 0;
#endif
    if constexpr (FITS_STATS) {
        if (p.cstats) {
            go(igemm_dma_kernel<TM, TN, WGM, WGN, S, KB, false, true, true>);
            return;
        }
    }
    if constexpr (FITS) {
        if (staged) {
            if (p.pabs) go(igemm_dma_kernel<TM, TN, WGM, WGN, S, KB, true, true, false>);
            else go(igemm_dma_kernel<TM, TN, WGM, WGN, S, KB, false, true, false>);
            return;
        }
    }
    if (p.pabs) go(igemm_dma_kernel<TM, TN, WGM, WGN, S, KB, true, false, false>);
    else go(igemm_dma_kernel<TM, TN, WGM, WGN, S, KB, false, false, false>);
}

}  // namespace

// Tile choice, from timings of the benchmark networks' layers and of 16384-token linear layers: the L2 cache delivers
// only about 2.5 times the HBM rate, so the largest tile that still gives most CUs a block wins; 128 x 128 runs as two
// 4-wave blocks per CU where there are enough tiles for that and as one 8-wave block otherwise.  Outputs narrower than
// 96 channels and launches with too few tiles (they split the reduction) stay with the register-staged kernel.
int dma_pick_tile(const IgemmParams &p) {
    if (p.Cin % 64 != 0 || !p.vec_out || p.nclasses < 1 || p.wt_bytes >= kBeyondStep || p.Cout < 96) return -1;
#ifdef LPDT_TUNE
    if (const char *e = getenv("LPDT_DMA_TILE")) {
        const int t = atoi(e);
        return t >= 0 && t < kNumTiles && p.Cin % kTiles[t].KB == 0 ? t : -1;
    }
#endif
    const bool wide = p.Cin % 128 == 0;   // tiles with 128-byte steps
    if (p.Cout >= 192 && tiles_of(p, 0) >= 160) {
        // GEMM-like launches.  With a short reduction the fp32 result is most of the traffic: 256 x 128 tiles on three
        // stages leave room for two blocks per CU, so that one block's stores run under the other's products
        // (16384 x 768 -> 3072: 77 -> 66 us).  With a long one (3072) the two are even and the larger tile re-reads less.
        const long long reduction = (long long)p.cls[0].Rc * p.cls[0].Sc * p.Cin;
        return reduction <= 2048 && p.nclasses == 1 ? 4 : 0;
    }
    const long long t128 = tiles_of(p, 1);
    if (t128 >= 320 || (t128 >= 160 && !wide)) return 2;
    if (t128 >= 160) return 1;
    if (wide && tiles_of(p, 3) >= 128) return 3;
    return -1;
}

bool dma_plan(IgemmParams *p, int *cfg_out, dim3 *grid) {
    const int cfg = dma_pick_tile(*p);
    if (cfg < 0) return false;
    p->tiles_n = (p->Cout + tile_bn(cfg) - 1) / tile_bn(cfg);
    p->kg = 4;
    p->atomic_out = 0;
    int max_tiles_m = 0;
    for (int i = 0; i < p->nclasses; ++i) {
        IgemmClass &c = p->cls[i];
        c.nk = c.gtot / 4;
        c.kps = c.nk;
        const int tm = (c.M + tile_bm(cfg) - 1) / tile_bm(cfg);
        if (tm > max_tiles_m) max_tiles_m = tm;
    }
    *cfg_out = cfg;
    *grid = dim3((unsigned)(max_tiles_m * p->tiles_n), (unsigned)p->nclasses, 1);
    return true;
}

bool dma_stats_supported(const IgemmParams &p, int cfg) {
    if (cfg < 0 || cfg >= kNumTiles || p.nclasses != 1 || p.out_mode == 0 || p.pix_per_sample <= 0) return false;
    const DmaTile &tl = kTiles[cfg];
    const int bm = tile_bm(cfg), bn = tile_bn(cfg);
    if (staged_passes(bm, bn, tl.WGM, tl.S * (bm + bn) * tl.KB, kStatSlots * bn * 16) == 0) return false;
    return (bm - 1) / p.pix_per_sample + 2 <= kStatSlots;   // samples a tile can touch
}

int dma_absmax_parts(int cfg, dim3 grid) { return (int)(grid.x * grid.y) * tile_waves(cfg); }

void dma_launch(const IgemmParams &p, int cfg, dim3 grid, hipStream_t st) {
    const size_t lds = tile_lds(cfg);
    switch (cfg) {
        case 0: launch_cfg<4, 2, 2, 4, 4, 64>(p, grid, lds, st); break;
        case 1: launch_cfg<2, 1, 2, 4, 4, 128>(p, grid, lds, st); break;
        case 2: launch_cfg<2, 2, 2, 2, 4, 64>(p, grid, lds, st); break;
        case 3: launch_cfg<1, 1, 2, 4, 4, 128>(p, grid, lds, st); break;
        default: launch_cfg<2, 2, 4, 2, 3, 64>(p, grid, lds, st); break;
    }
}

}  // namespace lpdt
