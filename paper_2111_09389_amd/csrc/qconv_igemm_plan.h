// Launch description shared by the implicit-GEMM kernels of forward and backward-data.
#pragma once
#include "qconv_internal.h"

namespace lpdt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kMaxClasses = 4;
constexpr int kMaxTaps = 31;              // bits of the per-row tap mask; bit 31 is the always-clear "no granule" slot
constexpr unsigned kBeyond = 0x80000000u; // a buffer offset no tensor reaches (sizes are checked to stay below it)
constexpr int kMaxTableEntries = 4096;    // granules of one block's K range (32 KB of LDS)

struct IgemmClass {
    int M, OHs, OWs;        // rows of the class = N*OHs*OWs output pixels
    int oy0, ox0;           // output pixel of sub-grid point (0,0); neighbours are `ostep` apart
    int iy0, ix0;           // input pixel read by tap (0,0) at sub-grid point (0,0)
    int Rc, Sc;             // tap grid of the class; tap (ty,tx) reads input pixel (+ty*dsign, +tx*dsign)
    int gtot, nk, kps;      // granules, K-steps, K-steps per blockIdx.z
    int wt_off;             // byte offset of the class's filter panel [Cout][Rc*Sc][Cin]
    unsigned mul_hw, mul_w; // multipliers for x/(OHs*OWs) and x/OWs by umulhi; 0: divide
    unsigned mul_sc;        // the same for x/Sc
};

struct IgemmParams {
    const int8_t *in;       // [N][IH][IW][Cin]
    const int8_t *wt;       // filter panels, see IgemmClass::wt_off
    void *out;              // [N][OH][OW][Cout]: int32 sums, or fp32 when out_mode != 0
    unsigned in_bytes, wt_bytes;
    int out_mode;           // 0: int32 sums; 1: fp32 sA*sB*sum; 2: fp32, added to what is there
    const float *sA, *sB;
    int Cin, Cout, gpt;     // gpt = granules per tap = Cin/16
    unsigned mul_gpt;       // multiplier for x/gpt
    int IH, IW, OH, OW;
    int istep, ostep, dsign;
    int tiles_n, atomic_out, vec_out;
    int kg;                 // granules per K-step
    float *pabs;            // ABSMAX kernels: max |out| per wave, [grid.y][grid.x][4]
    // forward products that also take the statistics of a Range-EvoNorm layer reading the result (fp32 output, one class,
    // direct-to-LDS kernel with a staged epilogue): cstats[n][Cout][4] receives, by atomic max on ordered bit patterns,
    // max x, ~min x, max u, ~min u per sample and channel (u = x * hardsigmoid(v x)); zero-filled before the launch
    unsigned *cstats;
    const float *vpar;      // the layer's v, [Cout]
    int pix_per_sample;     // OH * OW
    int nclasses;
    IgemmClass cls[kMaxClasses];
};


// The kernel that fills LDS straight from global memory (qconv_igemm_dma.hip).  dma_plan returns false for launches it
// does not take (reduction channels not a multiple of 64, unaligned output, too few tiles to fill the chip); otherwise it
// fills tiles_n and the per-class step counts and names the tile in *cfg.  dma_absmax_parts: abs-max partials that launch
// writes (one per wave).
bool dma_plan(IgemmParams *p, int *cfg, dim3 *grid);
// whether the launch dma_plan chose can take the statistics (p->pix_per_sample set)
bool dma_stats_supported(const IgemmParams &p, int cfg);
constexpr int kStatSlots = 8;   // samples one tile may touch in a statistics launch
int dma_absmax_parts(int cfg, dim3 grid);
void dma_launch(const IgemmParams &p, int cfg, dim3 grid, hipStream_t st);

// The kernel that keeps the whole filter in LDS and walks over row tiles (qconv_patch.hip): stride-1 layers with 64
// reduction channels and at most 64 result channels.  patch_plan: whether the launch (out_mode, pabs, cstats set) takes it.
bool patch_plan(const IgemmParams &p);
void patch_launch(const IgemmParams &p, hipStream_t st);

}  // namespace lpdt
