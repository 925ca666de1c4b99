// Internal interfaces between the convolution translation units.
#pragma once
#include "common.h"

namespace lpdt {

// First-layer path (few input channels): one filter row per MFMA K-step, on a zero-padded copy of the image.
bool narrow_conv_supported(const lpdt_conv_desc *d, int P, int Q);
size_t narrow_fwd_workspace(const lpdt_conv_desc *d);
size_t narrow_wgrad_workspace(const lpdt_conv_desc *d);
void launch_narrow_fwd(const lpdt_conv_desc *d, int P, int Q, const int8_t *x, const int8_t *w, int32_t *acc, int out_mode,
                       const float *sA, const float *sB, void *ws, hipStream_t st);
// out_mode 0: int32 sums; 1: fp32 sA*sB*sum
void launch_narrow_wgrad(const lpdt_conv_desc *d, int P, int Q, const int8_t *g, const int8_t *x, void *out, int out_mode,
                         const float *sA, const float *sB, void *ws, hipStream_t st);

// Implicit-GEMM forward / backward-data on the matrix cores (channel counts of the reduction a multiple of 16).
// `*_supported` is false for shapes that take the plain kernels; `*_is_split` tells that the reduction is split across
// blocks and combined with int32 atomics, which rules out the fused fp32 epilogue (out_mode must be 0 then).
bool igemm_fwd_supported(const lpdt_conv_desc *d, int P, int Q);
bool igemm_bwd_data_supported(const lpdt_conv_desc *d, int P, int Q);
bool igemm_fwd_is_split(const lpdt_conv_desc *d, int P, int Q);
bool igemm_bwd_data_is_split(const lpdt_conv_desc *d, int P, int Q);
// Which kernel and tile a launch with aligned operands takes (see lpdt_qconv_kernel_id).
int igemm_fwd_kernel_id(const lpdt_conv_desc *d, int P, int Q);
int igemm_bwd_data_kernel_id(const lpdt_conv_desc *d, int P, int Q);
// out_mode 0: int32 sums; 1: fp32 sA*sB*sum; 2: fp32 added to `out`.  x, w, g 16-byte aligned.
// pabs (fp32 output, reduction not split): every wave writes the largest |value| it stored, `*_absmax_parts` floats in all
// (0: the reduction is split, no such output).
int igemm_fwd_absmax_parts(const lpdt_conv_desc *d, int P, int Q);
int igemm_bwd_data_absmax_parts(const lpdt_conv_desc *d, int P, int Q);
void launch_igemm_fwd(const lpdt_conv_desc *d, int P, int Q, const int8_t *x, const int8_t *w, void *out, int out_mode,
                      const float *sA, const float *sB, hipStream_t st, float *pabs = nullptr);
// Backward-data reads the filter as transposed panels (one per stride residue class), K*R*S*C bytes in all, 16-byte
// aligned: made by the first call, consumed by the second (g and panel 16-byte aligned).
size_t igemm_bwd_filter_panel_bytes(const lpdt_conv_desc *d);
void launch_igemm_pack_bwd_filter(const lpdt_conv_desc *d, int P, int Q, const int8_t *w, void *panel, hipStream_t st);
void launch_igemm_pack_bwd_filters(const lpdt_conv_desc *descs, int count, const int8_t *const *w, void *const *panels, hipStream_t st);
void launch_igemm_bwd_data(const lpdt_conv_desc *d, int P, int Q, const int8_t *g, const void *panel, void *out, int out_mode,
                           const float *sA, const float *sB, hipStream_t st, float *pabs = nullptr);

// Weight gradient, rectangle-stepped kernel with partial tiles and a fixed-order reduction.
struct WgradRectPlan {
    int ch, cw, ncy, ncx, PHp, PWp, steps, steps_per_split, splits, tg, groups, tiles_k, tiles_c, kt, ct, ks;
    int ng, partials;   // wave groups per block (1 or 2); partial tiles written = ceil(splits / ng)
    long long out_len;
    size_t partial_bytes, lds;
};
// beside: 1 the product runs beside other kernels (fewer blocks), 0 it has the chip to itself, -1 what the caller set
// with lpdt_qconv_set_wgrad_beside
int wgrad_beside();
void set_wgrad_beside(int v);
bool wgrad_rect_plan(const lpdt_conv_desc *d, int P, int Q, WgradRectPlan *plan, int beside = -1);  // false: shape not handled
// out_mode 0: int32 sums; 1: fp32 sA*sB*sum.  `partial` needs plan.partial_bytes.
void launch_wgrad_rect(const lpdt_conv_desc *d, int P, int Q, const WgradRectPlan &plan, const int8_t *g, const int8_t *x,
                       void *out, int out_mode, const float *sA, const float *sB, void *partial, hipStream_t st);

// Row-tile variant for stride-1 filters of up to 3 x 3 taps (qconv_wgrad_rows.hip): same contract, same reduction kernel
struct WgradRowsPlan {
    int kt, stages, TR, PR, PW, ni, nkg, tiles_per_image, ntiles, tiles_per_split, splits, tiles_k, tiles_kc;
    long long out_len;
    size_t partial_bytes, lds;
};
bool wgrad_rows_plan(const lpdt_conv_desc *d, int P, int Q, WgradRowsPlan *plan, int beside = -1);
void launch_wgrad_rows(const lpdt_conv_desc *d, int P, int Q, const WgradRowsPlan &plan, const int8_t *g, const int8_t *x,
                       void *out, int out_mode, const float *sA, const float *sB, void *partial, hipStream_t st);

// GEMM-shaped variant for pointwise products with both channel counts multiples of 256 (qconv_wgrad_gemm.hip)
struct WgradGemmPlan {
    int T, steps, steps_per_split, splits, tiles_k, tiles_kc;
    long long out_len;
    size_t partial_bytes;
};
bool wgrad_gemm_plan(const lpdt_conv_desc *d, int P, int Q, WgradGemmPlan *plan);
bool wgrad_gemm_taps_plan(const lpdt_conv_desc *d, int P, int Q, WgradGemmPlan *plan);   // stride-1 filters of up to 3 x 3 taps
void launch_wgrad_gemm(const lpdt_conv_desc *d, const WgradGemmPlan &plan, const int8_t *g, const int8_t *x, void *out, int out_mode,
                       const float *sA, const float *sB, void *partial, hipStream_t st);

// out[i] = sum over `splits` copies partial[z][i] (out_len a multiple of 4), as int32 or as fp32 times sA*sB
void launch_wgrad_reduce(const int32_t *partial, long long out_len, int splits, void *out, int out_mode, const float *sA,
                         const float *sB, hipStream_t st);

// Range-EvoNorm with int8 output behind a convolution whose epilogue took the layer's statistics (range_evonorm.hip):
// ren_chain_begin zero-fills the statistics array at the head of `ws` (ren_chain_ws_bytes, 256-byte aligned) and returns
// it for the convolution launch; ren_chain_finish folds it and writes codes, scale, range and first arg-max / arg-min of
// x [N,H,W,C] -- the bits of lpdt_range_evonorm_fwd_q.
bool ren_chain_supported(int C, int groups);
size_t ren_chain_ws_bytes(int N, int C, int groups);
unsigned *ren_chain_begin(int N, int C, int groups, void *ws, hipStream_t st);
void ren_chain_finish(const float *x, int N, int H, int W, int C, int groups, const float *v, const float *gamma, const float *beta,
                      float eps, int8_t *q, float *scale, float *z, float *range_out, int32_t *argmax_out, int32_t *argmin_out,
                      void *ws, hipStream_t st);
// Forward product (fp32 result, out_mode 1 or 2) that also fills the statistics array; false (nothing launched) when the
// shape does not take the kernel that can.
bool igemm_fwd_stats_supported(const lpdt_conv_desc *d, int P, int Q);
void launch_igemm_fwd_stats(const lpdt_conv_desc *d, int P, int Q, const int8_t *x, const int8_t *w, float *out, int out_mode,
                            const float *sA, const float *sB, unsigned *cstats, const float *vpar, hipStream_t st);

// *out = max |x[i]| (x 16-byte aligned; scratch: absmax_scratch_floats() floats), and the fold of n ready partials alone
int absmax_scratch_floats();
void launch_absmax(const float *x, size_t len, float *scratch, float *out, hipStream_t st);
void launch_absmax_fold(const float *parts, int n, float *out, hipStream_t st);

// y = (sA*sB) * acc (+ y when accumulate): the kernel behind lpdt_dequantize
void launch_dequant(const int32_t *acc, size_t len, const float *sA, const float *sB, float *y, bool accumulate, hipStream_t st);

}  // namespace lpdt
