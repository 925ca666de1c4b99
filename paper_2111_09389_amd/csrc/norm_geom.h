// Launch geometry and key encoding shared by the normalisation layers' streaming kernels (NHWC fp32 tensors whose
// channel count is a multiple of 4): a block owns a run of consecutive pixels of one sample and its thread count is a
// multiple of C/4, which pins every thread to one quad of channels.
#pragma once
#include "common.h"

namespace lpdt {

constexpr int kRThreads = 256;
constexpr int kPixIters = 2;     // least pixels per thread in the streaming passes
constexpr int kBwdMinPix = 8;
constexpr int kRU = 4;           // pixels a thread has in flight: the streaming loops load kRU pixels, then work on them
constexpr int kMaxBlocks = 2048;  // the streaming grids are kept near this size: enough to fill the chip, few partial rows

struct RenGeom {
    int N, HW, C, groups, m;
    int cq;       // float4 quads per pixel (C/4)
    int threads;  // working threads per block, multiple of cq
    int block;    // launched block size: threads rounded up to whole waves (the extra threads only join reductions)
    int ppi;      // pixels per block iteration
    int chunks;   // blocks per sample
    int pix_per_block;
};

// Grid size of a streaming pass: about one block per `elems_per_block` elements, between 256 and kMaxBlocks.  Measured
// on the ResNet-18 layer sizes inside the training step (4 K against 8 K and 16 K elements per block in the apply and
// backward passes: 9.6 against 10.0 and 11.2 us, 18.8 against 19.6 and 20.1 us per layer on average; 2 K is no better
// and lengthens the backward pass's second launch, which adds up one row of partial sums per block).
constexpr int kStatsElems = 8192, kApplyElems = 4096, kBwdElems = 4096;
static inline int block_cap(int N, int H, int W, int C, int elems_per_block) {
    const long long b = (long long)N * H * W * C / elems_per_block;
    return (int)(b < 256 ? 256 : b > kMaxBlocks ? kMaxBlocks : b);
}
// min_pix: least pixels per block.  The forward passes leave a few keys per block and take 0; the backward pass leaves
// 4 floats per channel and block, which must stay small beside the 3 floats per channel and pixel it streams.
static inline RenGeom ren_geom(int N, int H, int W, int C, int groups, int min_pix, int max_blocks) {
    RenGeom g;
    g.N = N; g.HW = H * W; g.C = C; g.groups = groups; g.m = C / groups;
    g.cq = C / 4;
    g.threads = (kRThreads / g.cq) * g.cq;
    g.block = (g.threads + kWave - 1) / kWave * kWave;
    g.ppi = g.threads / g.cq;
    int iters = kPixIters;
    while (((long long)N * ((g.HW + g.ppi * iters - 1) / (g.ppi * iters)) > max_blocks || g.ppi * iters < min_pix) && iters < 4096) iters *= 2;
    g.pix_per_block = g.ppi * iters;
    g.chunks = (g.HW + g.pix_per_block - 1) / g.pix_per_block;
    return g;
}

// u = x * hardsigmoid(v x) of Eq. "ren" with every rounding pinned (no contraction left to the compiler): every kernel
// that evaluates it -- the forward passes and the convolution epilogue that takes the layer's statistics on the way
// out -- must produce the same bits.
__device__ __forceinline__ float ren_u(float x, float v) {
    const float z = __fmul_rn(v, x);
    return __fmul_rn(x, fminf(1.0f, fmaxf(0.0f, __fmul_rn(__fadd_rn(z, 3.0f), 1.0f / 6.0f))));
}

// monotone map float -> uint32 (larger float <=> larger key); -0 is folded onto +0
__device__ __forceinline__ uint32_t ordered_bits(float x) {
    const uint32_t b = __float_as_uint(x + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

}  // namespace lpdt
