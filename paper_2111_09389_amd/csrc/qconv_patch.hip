// int8 convolution forward / backward-data (Table "hardware_training", row Conv) for stride-1 layers with 64 reduction
// channels and at most 64 result channels (the 64 -> 64 stage of the residual networks: the largest feature maps, a
// filter of a few KiB).  Here the implicit GEMM has a reduction of only taps x 64 bytes, so a tile-at-a-time kernel
// spends its time on set-up, on re-fetching every input pixel once per tap and on waiting for its own stores.  This
// kernel keeps the WHOLE filter in LDS for the life of a block and walks over tiles of whole output rows:
//
//   tile  = TR consecutive output rows of one image (TR * OW <= 128 pixels = the rows of the MFMA tile)
//   patch = the (TR + R - 1) x (OW + S - 1) input pixels those rows read, loaded straight into LDS once (zero rows and
//           columns where the image ends), double buffered: the next tile's patch arrives while this one is multiplied
//   tap   = a constant pixel offset into the patch: all taps of the tile are multiplied out of one LDS buffer between
//           two barriers; an input pixel crosses the L2 -> LDS path once per tile instead of once per tap
//
// Patch pixels are 64 bytes; the 16-byte granule g of patch pixel pp sits in slot g ^ swz(pp) (swz = bits 2..3 of pp,
// reversed), which keeps the operand reads (lane = consecutive pixels) off each other's banks; the filter is stored
// per tap as [64 rows][64 B] with the same swizzle on the row.  4 waves: 2 (pixels) x 2 (channels), 64 x 32 each.
// Two blocks share a CU.  The waits of the tile loop are written as s_waitcnt instructions the compiler sees (not as
// inline assembly, which its own wait tracking cannot look into: it then put a wait for everything, the next patch's
// loads included, in front of the first register the loop reuses, and the loads no longer ran under the products).
// The wait for a tile's patch leaves the previous tile's stores outstanding: a wave's vector memory requests complete
// in the order they were issued, the stores are the youngest ones, so "all but the last nst" covers the patch.  The nine
// taps of a 3 x 3 filter are unrolled, which puts a tap's operand reads under the products of the tap before.
// Measured on 64 x 56 x 56 x 64 -> 64: 22.6 -> 18.3 us; with the stores switched off 11.4 us, with the products switched
// off 15 us (a plain fill of the 51 MB result takes 8.7 us).
#include "qconv_igemm_plan.h"

namespace lpdt {

namespace {

typedef __attribute__((address_space(3))) void lds_void;

constexpr int kPatchThreads = 256;
constexpr int kPatchMaxLoads = 6;      // patch load instructions per wave and tile: patches of up to 6 * 4 * 16 pixels
constexpr int kPatchMaxTaps = 16;      // 16 taps x 4 KiB of filter

struct PatchParams {
    IgemmParams g;
    int TR, PR, PW;          // output rows per tile, patch rows and columns
    int rmin, cmin;          // smallest row / column offset of a tap (relative to the output pixel)
    int tiles_per_image, ntiles;
    int ni;                  // load instructions per patch (16 pixels each)
    int patch_bytes;         // one patch buffer, a multiple of 1 KiB
};

__device__ __forceinline__ int pix_swz(int pp) { return ((pp >> 3) & 1) | ((pp >> 1) & 2); }

// kAdd: the call adds to what the result tensor holds (those values are fetched under the products)
template <bool kAdd, int NT>
__global__ __launch_bounds__(kPatchThreads, 2) void patch_conv_kernel(const PatchParams q) {
    const IgemmParams &p = q.g;
    const IgemmClass &c = p.cls[0];
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int ntaps = c.Rc * c.Sc;
    unsigned char *const wlds = lds;                               // [tap][64 rows][64 B]
    unsigned char *const plds = lds + ntaps * 4096;                // two patch buffers
    const int t = threadIdx.x, lane = t % 64, wave = __builtin_amdgcn_readfirstlane(t / 64);
    const __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.in), 0, (int)p.in_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_wt = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.wt), 0, (int)p.wt_bytes, 0x00020000);
    const int lrow = lane >> 2, lslot = lane & 3;

    // ---- the filter, once: instruction k of a tap covers rows 16k..16k+15; the waves share the 4 * ntaps instructions
    for (int k = wave; k < 4 * ntaps; k += 4) {
        const int tap = k >> 2, row = (k & 3) * 16 + lrow;
        const unsigned off = row < p.Cout ? (unsigned)(c.wt_off + row * c.gtot * 16 + tap * 64 + ((lslot ^ pix_swz(row)) << 4)) : kBeyond;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wt, (lds_void *)(wlds + k * 1024), 16, off, 0, 0, 0);
    }

    // ---- loader role: patch pixel pp = 16 * (wave + 4*j) + lane/4 of every tile; its position inside the patch decides
    // the offset from the tile's first input row and whether the column exists; whether the row exists depends on the tile
    int loff[kPatchMaxLoads], lprow[kPatchMaxLoads];
#pragma unroll
    for (int j = 0; j < kPatchMaxLoads; ++j) {
        const int pp = 16 * (wave + 4 * j) + lrow;
        const int pr = pp / q.PW, px = pp - pr * q.PW;
        const int ix = px + q.cmin;
        const bool ok = pp < q.PR * q.PW && (unsigned)ix < (unsigned)p.IW;
        loff[j] = ((pr + q.rmin) * p.IW + ix) * 64 + ((lslot ^ pix_swz(pp)) << 4);
        lprow[j] = ok ? pr + q.rmin : -(1 << 20);       // a row offset no tile brings back into the image
    }
    auto issue_patch = [&](int tile, int buf) {
        const bool live = tile < q.ntiles;
        const int n = tile / q.tiles_per_image, r0 = (tile - n * q.tiles_per_image) * q.TR;
        const int base = (n * p.IH + r0) * p.IW * 64;
#pragma unroll
        for (int j = 0; j < kPatchMaxLoads; ++j) {
            if (wave + 4 * j < q.ni) {
                const bool ok = live && (unsigned)(r0 + lprow[j]) < (unsigned)p.IH;
                const unsigned off = ok ? (unsigned)(base + loff[j]) : kBeyond;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_in, (lds_void *)(plds + buf * q.patch_bytes + (wave + 4 * j) * 1024), 16, off, 0, 0, 0);
            }
        }
    };

    // ---- multiplier role: this wave's pixels wm*64 + 32*i + lane%32 and channels wn*32 + (rows of the 32x32 MFMA)
    const int wm = wave >> 1, wn = wave & 1, half = lane >> 5, r32 = lane & 31;
    int pb[2];   // patch pixel under the tap with the smallest offsets
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int pix = wm * 64 + 32 * i + r32;
        const int dy = pix / c.OWs, ox = pix - dy * c.OWs;
        pb[i] = dy < q.TR ? dy * q.PW + ox : 0;      // rows past the tile multiply some pixel; their sums are not stored
    }
    const int brow = wn * 32 + r32;
    const int boff = brow * 64 + ((half ^ pix_swz(brow)) << 4);

    v16i acc[2];
    const float scale = p.out_mode ? __fmul_rn(*p.sA, *p.sB) : 0.0f;
    int tile = blockIdx.x;
    int nst = 0;     // store instructions this wave issued for the previous tile (a lower bound: those whose first lane stores)
    issue_patch(tile, 0);
    for (int it = 0; tile < q.ntiles; ++it, tile += gridDim.x) {
        // the patch of this tile (and, the first time, the filter) has landed everywhere; everybody is done with the other buffer
        asm volatile("" ::: "memory");
        // this tile's patch was requested before the previous tile's stores: waiting until only those stores (nst of them, the
        // youngest requests) are outstanding is enough -- vector memory requests of a wave complete in issue order
        if (nst >= 8) __builtin_amdgcn_s_waitcnt(0x0078);        // vmcnt(8) lgkmcnt(0)
        else if (nst >= 4) __builtin_amdgcn_s_waitcnt(0x0074);   // vmcnt(4) lgkmcnt(0)
        else __builtin_amdgcn_s_waitcnt(0x0070);                 // vmcnt(0) lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue_patch(tile + gridDim.x, (it + 1) & 1);
        const unsigned char *const pbuf = plds + (it & 1) * q.patch_bytes;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0;
        // a call that adds to what the result tensor holds fetches those values now, under the products
        const int n = tile / q.tiles_per_image, r0 = (tile - n * q.tiles_per_image) * q.TR;
        const int rows = min(q.TR, c.OHs - r0);
        const size_t pix0 = ((size_t)n * p.OH + r0) * p.OW;
        v4f held[2][4];
        if (kAdd) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int pix = wm * 64 + 32 * i + r32;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int col = wn * 32 + 8 * k + 4 * half;
                    held[i][k] = pix < rows * c.OWs && col < p.Cout
                                     ? *reinterpret_cast<const v4f *>(static_cast<const float *>(p.out) + (pix0 + pix) * p.Cout + col)
                                     : v4f{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
        auto tap_products = [&](int tap, int ty, int tx) {
            const int toff = (c.iy0 + ty * p.dsign - q.rmin) * q.PW + (c.ix0 + tx * p.dsign - q.cmin);
            const int w_off = tap * 4096 + boff;
            const v4i b0 = *reinterpret_cast<const v4i *>(wlds + w_off);
            const v4i b1 = *reinterpret_cast<const v4i *>(wlds + (w_off ^ 32));
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int pp = pb[i] + toff;
                const int a_off = pp * 64 + ((half ^ pix_swz(pp)) << 4);
                const v4i a0 = *reinterpret_cast<const v4i *>(pbuf + a_off);
                const v4i a1 = *reinterpret_cast<const v4i *>(pbuf + (a_off ^ 32));
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b0, a0, acc[i], 0, 0, 0);
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b1, a1, acc[i], 0, 0, 0);
            }
        };
        if (NT == 9) {       // 3 x 3: unrolled, so that the operand reads of a tap are issued under the products of the one before
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) tap_products(tap, tap / 3, tap % 3);
        } else {
            int ty = 0, tx = 0;
            for (int tap = 0; tap < ntaps; ++tap) {
                tap_products(tap, ty, tx);
                if (++tx == c.Sc) { tx = 0; ++ty; }
            }
        }
        {
            const int npix = rows * c.OWs;
            const int ni = (wm * 64 < npix) + (wm * 64 + 32 < npix);
            int nk = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) nk += wn * 32 + 8 * k < p.Cout;
            nst = kAdd ? 0 : ni * nk;     // with loads of the values added to in flight, wait for everything
        }
        // one wait for all the values to add to (left to itself the compiler waits before every store, for the loads and
        // with them for the stores before it)
        if (kAdd) __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0)
        // a lane holds pixel lane%32 of sub-tile i and channels wn*32 + 8*k + 4*(lane/32) + 0..3, k = 0..3
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int pix = wm * 64 + 32 * i + r32;
            if (pix >= rows * c.OWs) continue;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int col = wn * 32 + 8 * k + 4 * half;
                if (col >= p.Cout) continue;
                const v4i s = {acc[i][4 * k], acc[i][4 * k + 1], acc[i][4 * k + 2], acc[i][4 * k + 3]};
                int32_t *dst = static_cast<int32_t *>(p.out) + (pix0 + pix) * p.Cout + col;
                if (p.out_mode) {  // the dequantizing scale applied here: same arithmetic as lpdt_dequantize
                    v4f *fdst = reinterpret_cast<v4f *>(dst);
                    const bool add = kAdd;
                    v4f v = {0.f, 0.f, 0.f, 0.f};
                    if (add) v = held[i][k];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = dequant_value(scale, s[e], v[e], add);
                    *fdst = v;
                } else *reinterpret_cast<v4i *>(dst) = s;
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the empty loads of the tile past the last one
}

}  // namespace

// Whether the launch takes this kernel; fills the geometry.
static bool patch_geometry(const IgemmParams &p, PatchParams *q) {
    if (p.nclasses != 1 || p.istep != 1 || p.ostep != 1 || p.Cin != 64 || p.Cout > 64 || !p.vec_out || p.pabs || p.cstats) return false;
    const IgemmClass &c = p.cls[0];
    const int ntaps = c.Rc * c.Sc;
    if (ntaps < 2 || ntaps > kPatchMaxTaps || c.oy0 != 0 || c.ox0 != 0 || c.OHs != p.OH || c.OWs != p.OW || p.OW > 128) return false;
    if (p.wt_bytes >= 0x40000000u) return false;
    q->g = p;
    const int r_a = c.iy0, r_b = c.iy0 + (c.Rc - 1) * p.dsign, c_a = c.ix0, c_b = c.ix0 + (c.Sc - 1) * p.dsign;
    q->rmin = r_a < r_b ? r_a : r_b;
    q->cmin = c_a < c_b ? c_a : c_b;
    q->TR = 128 / p.OW < p.OH ? 128 / p.OW : p.OH;
    q->PR = q->TR + c.Rc - 1;
    q->PW = p.OW + c.Sc - 1;
    q->ni = (q->PR * q->PW + 15) / 16;
    if (q->ni > 4 * kPatchMaxLoads) return false;
    q->patch_bytes = q->ni * 1024;
    q->tiles_per_image = (p.OH + q->TR - 1) / q->TR;
    const long long nt = (long long)(p.cls[0].M / (p.OH * p.OW)) * q->tiles_per_image;
    if (nt > 0x7fffffff / 2 || nt < 256) return false;              // small launches stay with the tile-at-a-time kernels
    if (q->TR * p.OW < 96) return false;                             // tiles that leave a quarter of the MFMA rows empty
    q->ntiles = (int)nt;
    return (size_t)ntaps * 4096 + 2 * (size_t)q->patch_bytes <= 80 * 1024;   // two blocks per CU
}

bool patch_plan(const IgemmParams &p) {
    PatchParams q;
    return patch_geometry(p, &q);
}

void patch_launch(const IgemmParams &p, hipStream_t st) {
    PatchParams q;
    if (!patch_geometry(p, &q)) return;
    const size_t lds = (size_t)p.cls[0].Rc * p.cls[0].Sc * 4096 + 2 * (size_t)q.patch_bytes;
    static bool raised = false;
    if (!raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(patch_conv_kernel<false, 0>), hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(patch_conv_kernel<true, 0>), hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(patch_conv_kernel<false, 9>), hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(patch_conv_kernel<true, 9>), hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        raised = true;
    }
    const int grid = q.ntiles < 512 ? q.ntiles : 512;
    const bool add = p.out_mode == 2, nine = p.cls[0].Rc == 3 && p.cls[0].Sc == 3;
    auto kernel = add ? (nine ? patch_conv_kernel<true, 9> : patch_conv_kernel<true, 0>) : (nine ? patch_conv_kernel<false, 9> : patch_conv_kernel<false, 0>);
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kPatchThreads), lds, st, q);
}

}  // namespace lpdt
