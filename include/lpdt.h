/*
 * lpdt - the hot path of low-precision decentralized training (arXiv 2111.09389)
 * as a C-ABI library of hand-written HIP kernels for gfx950 (MI355X).
 *
 * One agent's 8-bit training step (Section 3, "Low Precision Training"):
 * quantize -> int8 convolution forward / backward-data / backward-weight with
 * int32 accumulation -> Range-EvoNorm (Eq. "ren"), plus the gossip step of
 * Algorithm 1 (plain and CHOCO-SGD with layer-wise top-k, supplement
 * Algorithm 3) for several agents simulated on one GPU.
 *
 * Conventions shared by every entry point
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *  - The caller owns every buffer; the library borrows them until the work it
 *    enqueued on `stream` has finished.  No entry point allocates, frees or
 *    synchronises; all work is asynchronous on `stream` (a hipStream_t passed
 *    as void*, NULL = the default stream), so calls can be captured in a HIP
 *    graph.
 *  - Scratch memory comes from the caller: `ws` / `ws_bytes`, sized by the
 *    matching *_workspace_bytes() call; `ws` must be 256-byte aligned.
 *    Workspace contents are undefined on entry and on return.
 *  - Arguments are checked on the host before anything is enqueued.  Return
 *    value 0 = success, negative = lpdt_status; lpdt_last_error() gives a
 *    thread-local message for the last failure.
 *  - Issue calls from one host thread at a time (any stream).  The launchers
 *    keep per-kernel settings of the process (the dynamic-LDS limit a launch
 *    needs is set before it), which two threads could change under each
 *    other's launches.
 *  - Layouts: activations and their gradients NHWC, filters KRSC (K output
 *    channels, R x S taps, C input channels), parameter matrices row-major
 *    [n agents][d parameters].  Tensors are dense and contiguous.
 *  - Scales of quantized tensors are fp32 scalars resident in device memory,
 *    so no call needs a host round trip.
 */
#ifndef LPDT_H
#define LPDT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LPDT_OK = 0,
    LPDT_EINVAL = -1,       /* null pointer, non-positive size, misaligned buffer, bad enum */
    LPDT_EUNSUPPORTED = -2, /* a shape or mode outside what the kernels implement */
    LPDT_EWORKSPACE = -3,   /* ws is NULL / misaligned / smaller than *_workspace_bytes() */
    LPDT_EHIP = -4          /* a HIP runtime call (launch) failed */
} lpdt_status;

/* Thread-local text of the last error returned on this thread ("" if none). */
const char *lpdt_last_error(void);
/* Library version, e.g. 100 = 0.1.0. */
int lpdt_version(void);

/* ------------------------------------------------------------------ quantizer
 * Section 3 "Low Precision Training": weights, activations and layer gradients
 * are quantized to 8 bits in every iteration.  Grid: symmetric, per tensor,
 * scale = absmax/127, codes in [-127,127] (-128 is never produced).
 *   a = max|x_i| ; inv = 127/a (one fp32 divide) ; t_i = x_i*inv (fp32 multiply)
 *   LPDT_ROUND_NEAREST    : q_i = round-half-to-even(t_i)
 *   LPDT_ROUND_STOCHASTIC : q_i = floor(t_i) + [u_i < t_i - floor(t_i)],
 *        u_i = (top 24 bits of a Philox4x32-10 word) * 2^-24, key = seed,
 *        counter = (offset + i/4, 0, 0), word i%4 -- a function of the logical
 *        element index i only, never of the launch geometry.
 *   a == 0 gives all-zero codes and scale 0.  Non-finite inputs are a caller error.
 */
enum { LPDT_ROUND_NEAREST = 0, LPDT_ROUND_STOCHASTIC = 1 };

size_t lpdt_quantize_workspace_bytes(size_t len);

/* x[len] fp32 in; q[len] int8 out; scale: one fp32 out (absmax/127).
 * Two passes over x (abs-max, then rounding). */
int lpdt_quantize(const float *x, size_t len, int rounding, uint64_t seed, uint64_t offset,
                  int8_t *q, float *scale, void *ws, size_t ws_bytes, void *stream);

/* Same, but the abs-max is supplied by the producer of x (one fp32 in device
 * memory, e.g. written by lpdt_range_evonorm_fwd / _bwd): one pass over x. */
int lpdt_quantize_with_absmax(const float *x, size_t len, const float *absmax, int rounding,
                              uint64_t seed, uint64_t offset, int8_t *q, float *scale, void *stream);

/* For callers that cannot allocate or hand over a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): lpdt_quantize with the abs-max partials
 * kept in a fixed 4 KiB device array inside the library (one copy per GPU, held until the process
 * ends) instead of a caller workspace.  Same codes and scale as lpdt_quantize, bit for bit.
 * Calls no allocating routine.  len must not exceed lpdt_quantize_static_max_len() (2^30 elements),
 * else LPDT_EUNSUPPORTED.  All calls on one GPU share the array: two calls that overlap in time
 * on the same GPU (different streams or host threads) race; serialise them. */
size_t lpdt_quantize_static_max_len(void);
int lpdt_quantize_static(const float *x, size_t len, int rounding, uint64_t seed, uint64_t offset,
                         int8_t *q, float *scale, void *stream);

/* Many tensors in one call (the weights of all layers of a model, Section 3: every layer's
 * weights are quantized each iteration): slice s = x[seg_begin[s], seg_end[s]) gets its own
 * scale, scales[s], and its codes go to q[seg_begin[s], seg_end[s]) -- exactly what
 * lpdt_quantize(x + seg_begin[s], seg_end[s] - seg_begin[s], rounding, seed,
 * offset + s*2^24, ...) would write, in three launches for any number of slices.
 * seg_begin, seg_end: HOST arrays of nseg element indices (read before the call returns);
 * slices must be non-empty, at most 2^26 elements each, and should not overlap.
 * x, q, scales: device.  LPDT_EUNSUPPORTED for an empty slice or nseg <= 0. */
size_t lpdt_quantize_segments_workspace_bytes(int nseg);
int lpdt_quantize_segments(const float *x, const int64_t *seg_begin, const int64_t *seg_end, int nseg,
                           int rounding, uint64_t seed, uint64_t offset, int8_t *q, float *scales,
                           void *ws, size_t ws_bytes, void *stream);

/* y_i = (sA*sB) * acc_i, the real value of an int32 accumulator of two quantized
 * tensors; sA, sB: device scalars.  If accumulate != 0, y_i += that value. */
int lpdt_dequantize(const int32_t *acc, size_t len, const float *sA, const float *sB, float *y,
                    int accumulate, void *stream);

/* --------------------------------------------------------------- convolutions
 * Table "hardware_training", row Conv: the forward product and the two
 * backward products of a convolution layer, on int8 codes with exact int32
 * accumulation (cross-correlation, zero padding, dilation 1, one group).
 * Output size P = (H + 2*pad_h - R)/stride_h + 1, Q likewise.
 * Linear layers are the case R = S = H = W = 1.
 * The exact sums must fit int32 (always true when the reduction length is
 * <= 133144; see the bound in the design notes); no saturation is applied.
 */
typedef struct {
    int N, C, H, W;       /* input: batch, channels, height, width */
    int K, R, S;          /* filter: output channels, taps */
    int stride_h, stride_w, pad_h, pad_w;
} lpdt_conv_desc;

size_t lpdt_qconv_fwd_workspace_bytes(const lpdt_conv_desc *d);
size_t lpdt_qconv_bwd_data_workspace_bytes(const lpdt_conv_desc *d);
size_t lpdt_qconv_bwd_weight_workspace_bytes(const lpdt_conv_desc *d);

/* acc[n,p,q,k] = sum_{r,s,c} xq[n, p*stride_h+r-pad_h, q*stride_w+s-pad_w, c] * wq[k,r,s,c]
 * xq int8 [N,H,W,C]; wq int8 [K,R,S,C]; acc int32 [N,P,Q,K], overwritten. */
int lpdt_qconv_fwd(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, int32_t *acc,
                   void *ws, size_t ws_bytes, void *stream);

/* dx[n,h,w,c] = sum over (p,q,r,s,k) with p*stride_h+r-pad_h == h, q*stride_w+s-pad_w == w
 *               of gq[n,p,q,k] * wq[k,r,s,c]
 * gq int8 [N,P,Q,K] (8-bit layer gradient); dx int32 [N,H,W,C], overwritten. */
int lpdt_qconv_bwd_data(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *wq, int32_t *dx,
                        void *ws, size_t ws_bytes, void *stream);

/* dw[k,r,s,c] = sum_{n,p,q} gq[n,p,q,k] * xq[n, p*stride_h+r-pad_h, q*stride_w+s-pad_w, c]
 * dw int32 [K,R,S,C], overwritten.  (The weight gradient leaves the library as
 * fp32 after lpdt_dequantize and is never re-quantized: gradient bifurcation.) */
int lpdt_qconv_bwd_weight(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *xq, int32_t *dw,
                          void *ws, size_t ws_bytes, void *stream);

/* Which kernel a product of this shape takes when its operands are 16-byte aligned, for tests and profiles that
 * must know which code they exercise (the result never affects the arithmetic).  product: 0 forward, 1 backward-data,
 * 2 backward-weight, 3 the forward product inside lpdt_qconv_ren_fwd_q (40 + t when it takes the normalisation's
 * statistics in its epilogue, t as for 20 + t below; else the value for product 0).  Returns a negative lpdt_status for a bad descriptor, else
 *   0   the any-shape kernel (one thread per output; the sliced weight-gradient kernel)
 *   1   the first-layer matrix-core kernel (few input channels)
 *   2   backward-weight only: the per-tap matrix-core kernel with atomic adds
 *   3   the one-launch kernel for small linear layers (1x1, stride 1, at most 4 Mi multiply-adds)
 *   10 + v (+ 100 when the reduction is split over blocks)  register-staged implicit GEMM, v = 0: 128 x 32 tile,
 *       1 / 2: 64 x 64 with 64- / 128-byte steps, 3 / 4: 128 x 64 with 64- / 128-byte steps
 *   20 + t  implicit GEMM with operands loaded straight into LDS, t = 0: 256 x 256, 1: 128 x 128 with 8 waves,
 *       2: 128 x 128 with 4 waves, 3: 64 x 128, 4: 256 x 128 on three stages (two blocks per CU)
 *   50  forward / backward-data of stride-1 layers with 64 reduction channels and at most 64 result channels: the
 *       whole filter stays in LDS, tiles of whole output rows, each input patch loaded once for all taps
 *   30 + t + 4*[64-pixel steps] + 8*[two wave groups per block]  rectangle-stepped backward-weight, t = 0: 32 x 64,
 *       1: 64 x 64, 2: 128 x 128 channel tile
 *   60  backward-weight of stride-1 layers with filters of up to 3 x 3 taps (output channels a multiple of 32, input
 *       channels of 64): tiles of whole output rows, gradient and input patch loaded straight into LDS, all taps
 *       read out of the one patch
 *   62  backward-weight of pointwise products with both channel counts multiples of 256 (linear layers at transformer
 *       shapes): 256 x 256 tiles, both operands loaded straight into LDS and read back transposed
 *   63  the same kernel with one filter tap per block, for stride-1 filters of up to 3 x 3 taps that the row-tile and
 *       rectangle kernels decline (maps of a few pixels at channel counts that are multiples of 256) */
int lpdt_qconv_kernel_id(const lpdt_conv_desc *d, int product);

/* How the backward-weight products size their launches.  beside == 0 (the default): for a product that has the chip to
 * itself (one block per compute unit or more).  beside != 0: for a product issued beside other kernels, as a training
 * step does on a second stream -- fewer blocks, which leaves compute units to the other stream and writes fewer partial
 * tiles; alone such a launch is up to 40 % slower, beside the backward chain of a ResNet-18 step it makes the step ~2 %
 * shorter.  Results are identical, bit for bit (integer sums).  Process-wide, takes effect at the next call; the
 * workspace queries cover both settings.  Always returns LPDT_OK. */
int lpdt_qconv_set_wgrad_beside(int beside);

/* The same three products with the dequantizing scale applied in the kernel epilogue: the result
 * is the fp32 tensor (s_a*s_b)*sum, bit-identical to the int32 call followed by lpdt_dequantize,
 * without the int32 tensor making a round trip through HBM.  s_*: fp32 device scalars (the scales
 * lpdt_quantize wrote).  accumulate != 0 (backward-data only) adds to the gradient already in dx,
 * for tensors that fan out to several consumers.  Shapes whose reduction is split over blocks
 * stage their int32 sums in the workspace, which the *_f32_workspace_bytes queries include.
 * The forward and backward-data queries assume 16-byte aligned operands (xq, wq, gq): a call with a
 * misaligned one takes the any-shape kernel, which stages its sums too, and needs 4*N*P*Q*K + 256
 * (forward) or 4*N*H*W*C + 256 (backward-data) bytes on top, else it returns LPDT_EWORKSPACE. */
size_t lpdt_qconv_fwd_f32_workspace_bytes(const lpdt_conv_desc *d);
size_t lpdt_qconv_bwd_data_f32_workspace_bytes(const lpdt_conv_desc *d);
size_t lpdt_qconv_bwd_weight_f32_workspace_bytes(const lpdt_conv_desc *d);

int lpdt_qconv_fwd_f32(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx,
                       const float *sw, float *y, void *ws, size_t ws_bytes, void *stream);
int lpdt_qconv_bwd_data_f32(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *wq, const float *sg,
                            const float *sw, float *dx, int accumulate, void *ws, size_t ws_bytes,
                            void *stream);

int lpdt_qconv_bwd_weight_f32(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *xq, const float *sg,
                              const float *sx, float *dw, void *ws, size_t ws_bytes, void *stream);

/* The same product with the filter prepared ahead of time.  Backward-data reads the filter transposed; the call above
 * transposes it on every call, although the weights change only once per step (the local update of Algorithm 1).  A training step
 * can make the transposed copy when the weights' codes are final (for instance beside the forward pass, on another
 * stream) and hand it over here.  lpdt_qconv_bwd_data_packed_filter_bytes: size of the copy, 0 when the shape has no
 * prepared form (then only lpdt_qconv_bwd_data_f32 applies).  packed: device, 16-byte aligned, owned by the caller,
 * valid until the weights change.  Results are those of lpdt_qconv_bwd_data_f32, bit for bit.
 * lpdt_qconv_bwd_data_pack_filters prepares `count` filters in one launch (per 24 filters): descs, wq, packed and
 * packed_bytes are HOST arrays of `count` entries (wq[i], packed[i]: device pointers as above); every entry is checked
 * before anything is launched, and an entry whose shape has no prepared form is an error (LPDT_EUNSUPPORTED).  Each
 * packed[i] holds exactly what lpdt_qconv_bwd_data_pack_filter would have written. */
size_t lpdt_qconv_bwd_data_packed_filter_bytes(const lpdt_conv_desc *d);
int lpdt_qconv_bwd_data_pack_filter(const lpdt_conv_desc *d, const int8_t *wq, void *packed, size_t packed_bytes,
                                    void *stream);
int lpdt_qconv_bwd_data_pack_filters(const lpdt_conv_desc *descs, int count, const int8_t *const *wq, void *const *packed,
                                     const size_t *packed_bytes, void *stream);
int lpdt_qconv_bwd_data_f32_packed(const lpdt_conv_desc *d, const int8_t *gq, const void *packed, const float *sg,
                                   const float *sw, float *dx, int accumulate, void *ws, size_t ws_bytes,
                                   void *stream);

/* The two products with max |result| as a by-product: absmax_out (device fp32 scalar) = max over all elements of |y|
 * resp. |dx| as stored (after the addition when accumulate != 0), exactly, for an lpdt_quantize_with_absmax that follows
 * with no normalisation layer in between (linear layers, Table "hardware_training" row Linear; the quantizer's first
 * pass over the tensor then falls away).  Where the matrix-core kernel writes the result itself the maximum is taken in
 * its epilogue; elsewhere (first layer, split reductions, misaligned operands) in a pass over the result.  y, dx and
 * the operands as in lpdt_qconv_fwd_f32 / lpdt_qconv_bwd_data_f32; the backward call takes the filter either as wq or
 * prepared (packed != NULL, see lpdt_qconv_bwd_data_pack_filter; wq may then be NULL). */
size_t lpdt_qconv_fwd_f32_absmax_workspace_bytes(const lpdt_conv_desc *d);
size_t lpdt_qconv_bwd_data_f32_absmax_workspace_bytes(const lpdt_conv_desc *d);
int lpdt_qconv_fwd_f32_absmax(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx,
                              const float *sw, float *y, float *absmax_out, void *ws, size_t ws_bytes, void *stream);
int lpdt_qconv_bwd_data_f32_absmax(const lpdt_conv_desc *d, const int8_t *gq, const int8_t *wq, const void *packed,
                                   const float *sg, const float *sw, float *dx, int accumulate, float *absmax_out,
                                   void *ws, size_t ws_bytes, void *stream);

/* The forward product added to what y already holds (Table "hardware_training", row Skip Connections, done in
 * the convolution's epilogue): y += (sx*sw) * sum, the bits of lpdt_qconv_fwd_f32 into a temporary followed by
 * lpdt_add(y, temporary).  y fp32 [N,P,Q,K], 16-byte aligned, read and overwritten.  A misaligned operand
 * needs the staging room of the largest case: ask lpdt_qconv_fwd_f32_add_workspace_bytes and add
 * 4*N*P*Q*K + 256 bytes. */
size_t lpdt_qconv_fwd_f32_add_workspace_bytes(const lpdt_conv_desc *d);
int lpdt_qconv_fwd_f32_add(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx,
                           const float *sw, float *y, void *ws, size_t ws_bytes, void *stream);

/* The chain convolution -> Range-EvoNorm -> quantizer of a layer whose normalised output only feeds convolutions
 * (Section 3: every layer's input is quantized; Eq. "ren"), as one call: y = (sx*sw) * conv(xq, wq) (added to what y holds
 * when accumulate != 0: a skip connection), then the codes q and scale of Range-EvoNorm(y) and the layer's saved range /
 * argmax / argmin -- the bits of lpdt_qconv_fwd_f32 (or lpdt_qconv_fwd_f32_add) followed by lpdt_range_evonorm_fwd_q;
 * z: NULL, or fp32 [N,P,Q,K] that also receives the normalised output (a skip connection reads it).  Where the matrix-core kernel writes y through LDS it takes the per-sample, per-channel extremes
 * of y and of y*hardsigmoid(v y) on the way out, so the normalisation's statistics pass over y falls away and the
 * positions of the extremes are found by the pass that emits the codes; other shapes run the two calls.
 * y fp32 [N,P,Q,K] (kept: the backward pass reads it), q int8 [N,P,Q,K]; v, gamma, beta fp32 [K]; groups as in
 * lpdt_range_evonorm_fwd (K % groups == 0, K/groups >= 2); K a multiple of 4, at most 1024. */
size_t lpdt_qconv_ren_fwd_q_workspace_bytes(const lpdt_conv_desc *d, int groups);
int lpdt_qconv_ren_fwd_q(const lpdt_conv_desc *d, const int8_t *xq, const int8_t *wq, const float *sx, const float *sw,
                         int accumulate, int groups, const float *v, const float *gamma, const float *beta, float eps,
                         float *y, float *z, int8_t *q, float *scale, float *range_out, int32_t *argmax_out,
                         int32_t *argmin_out, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------ Range-EvoNorm
 * Eq. "ren": for every sample n and channel group G (m = C/groups channels),
 *   range = max - min of x over the group's (h, w, channel) slab
 *   D     = C(m)*range + eps,  C(m) = 1/sqrt(2 ln m)
 *   y     = gamma_c * x * hardsigmoid(v_c * x) / D + beta_c,
 *   hardsigmoid(z) = max(0, min(1, (z+3)/6)).
 * fp32 arithmetic.  groups must divide C and m must be >= 2 (C(1) is infinite):
 * otherwise LPDT_EUNSUPPORTED.  eps = 0 is allowed.
 */
size_t lpdt_range_evonorm_fwd_workspace_bytes(int N, int H, int W, int C, int groups);
size_t lpdt_range_evonorm_bwd_workspace_bytes(int N, int H, int W, int C, int groups);

/* x, y fp32 [N,H,W,C]; v, gamma, beta fp32 [C].
 * Saved for the backward pass, each [N*groups]: range_out (max - min), argmax_out /
 * argmin_out = position of the first maximum / minimum inside the slab, counted as
 * (h*W + w)*m + channel_in_group (lowest such index on ties).
 * absmax_out: optional (may be NULL) fp32 scalar, set to max|y| for a following
 * lpdt_quantize_with_absmax. */
int lpdt_range_evonorm_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v,
                           const float *gamma, const float *beta, float eps, float *y,
                           float *range_out, int32_t *argmax_out, int32_t *argmin_out,
                           float *absmax_out, void *ws, size_t ws_bytes, void *stream);

/* Range-EvoNorm forward whose output leaves as int8 codes (for layers whose only consumers are
 * quantized convolutions): y as lpdt_range_evonorm_fwd computes it, then quantized as
 * lpdt_quantize(y, LPDT_ROUND_NEAREST) would -- the same codes and scale, bit for bit -- without
 * the fp32 tensor y making a round trip through HBM.  q int8 [N,H,W,C] (4-byte aligned), scale:
 * fp32 device scalar; y: NULL, or fp32 [N,H,W,C] (16-byte aligned) that also receives the
 * unquantized output (for tensors with a full-precision reader besides the convolutions: then
 * only the quantizer's read of y is saved); range_out / argmax_out / argmin_out as above.  C must be a multiple of 4,
 * at most 1024 (LPDT_EUNSUPPORTED otherwise: use the two calls). */
size_t lpdt_range_evonorm_fwd_q_workspace_bytes(int N, int H, int W, int C, int groups);
int lpdt_range_evonorm_fwd_q(const float *x, int N, int H, int W, int C, int groups, const float *v,
                             const float *gamma, const float *beta, float eps, int8_t *q, float *scale,
                             float *y, float *range_out, int32_t *argmax_out, int32_t *argmin_out, void *ws,
                             size_t ws_bytes, void *stream);

/* Gradient of the forward above.  dy, x, dx fp32 [N,H,W,C]; range/argmax/argmin as
 * saved by the forward.  The hard-sigmoid slope is 1/6 strictly inside (-3,3), else 0;
 * the gradient through the range goes entirely to the saved arg-max (+) and arg-min (-).
 * dv, dgamma, dbeta fp32 [C] are overwritten (not accumulated).  Results do not depend
 * on launch geometry or run (fixed-order reductions).
 * absmax_out: optional fp32 scalar, set to max|dx|.  A saved position outside its slab (not what the
 * forward pass wrote) is taken as the slab's first element: nothing is read or written out of bounds. */
int lpdt_range_evonorm_bwd(const float *dy, const float *x, int N, int H, int W, int C, int groups,
                           const float *v, const float *gamma, float eps, const float *range,
                           const int32_t *argmax, const int32_t *argmin, float *dx, float *dv,
                           float *dgamma, float *dbeta, float *absmax_out, void *ws, size_t ws_bytes,
                           void *stream);

/* Range-EvoNorm directly followed by a max-pool (the stem of the residual networks), for a normalised tensor
 * that nothing but the pool reads.  Forward: z [N,P,Q,C] and idx as lpdt_maxpool_fwd(lpdt_range_evonorm_fwd(x))
 * would give them, bit for bit, and the layer's saved range / argmax / argmin; the normalised tensor itself is
 * never stored.  absmax_out: optional (may be NULL) fp32 scalar, set to max|z| for a following
 * lpdt_quantize_with_absmax.  Backward: from the pooled gradient dz [N,P,Q,C] and idx, everything
 * lpdt_range_evonorm_bwd(lpdt_maxpool_bwd(dz, idx), x, ...) returns, bit for bit; needs k <= 2 * stride
 * (LPDT_EUNSUPPORTED otherwise: use the two calls).  k, st, pd: window, stride, padding of the pool;
 * C a multiple of 4, at most 1024; x, z, idx, dz, dx 16-byte aligned. */
size_t lpdt_range_evonorm_maxpool_fwd_workspace_bytes(int N, int H, int W, int C, int groups);
size_t lpdt_range_evonorm_maxpool_bwd_workspace_bytes(int N, int H, int W, int C, int groups);
int lpdt_range_evonorm_maxpool_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v,
                                   const float *gamma, const float *beta, float eps, int k, int st, int pd,
                                   float *z, int32_t *idx, float *range_out, int32_t *argmax_out,
                                   int32_t *argmin_out, float *absmax_out, void *ws, size_t ws_bytes,
                                   void *stream);
int lpdt_range_evonorm_maxpool_bwd(const float *dz, const int32_t *idx, const float *x, int N, int H, int W,
                                   int C, int groups, const float *v, const float *gamma, float eps, int k,
                                   int st, int pd, const float *range, const int32_t *argmax,
                                   const int32_t *argmin, float *dx, float *dv, float *dgamma, float *dbeta,
                                   float *absmax_out, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------- full-precision comparison layers
 * The two layers Section 3 sets Range-EvoNorm against, as fp32 reference layers with the same
 * tensor conventions (x, y, dy, dx fp32 [N,H,W,C], 16-byte aligned; per-channel vectors fp32 [C];
 * device pointers; eps >= 0).  C must be a multiple of 4 and at most 1024 (LPDT_EUNSUPPORTED
 * otherwise).  Reductions run in a fixed order: results do not change from run to run.
 *
 * EvoNorm-S0 (Eq. "en"): for every sample n and channel group G (m = C/groups channels),
 *   var = population variance (1/count) of x over the group's (h, w, channel) slab,
 *   y   = gamma_c * x * sigmoid(v_c * x) / sqrt(var + eps) + beta_c.
 * (The paper prints no eps and does not say which variance: eps is an argument and may be 0,
 * the population form is the reading taken.)  mean_out, var_out: fp32 [N*groups], saved for
 * the backward pass.  The backward pass returns dx and the parameter gradients dv, dgamma,
 * dbeta (fp32 [C], overwritten). */
size_t lpdt_evonorm_s0_fwd_workspace_bytes(int N, int H, int W, int C, int groups);
size_t lpdt_evonorm_s0_bwd_workspace_bytes(int N, int H, int W, int C, int groups);
int lpdt_evonorm_s0_fwd(const float *x, int N, int H, int W, int C, int groups, const float *v,
                        const float *gamma, const float *beta, float eps, float *y, float *mean_out,
                        float *var_out, void *ws, size_t ws_bytes, void *stream);
int lpdt_evonorm_s0_bwd(const float *dy, const float *x, int N, int H, int W, int C, int groups,
                        const float *v, const float *gamma, float eps, const float *mean,
                        const float *var, float *dx, float *dv, float *dgamma, float *dbeta, void *ws,
                        size_t ws_bytes, void *stream);

/* Range batch-norm (Eq. "rbn"): per channel c, over all samples and pixels of the batch,
 *   mean  = mean of x,  range = max - min of x (= of x - mean),
 *   y     = gamma_c * (x - mean) / (C(b) * range + eps) + beta_c,   C(b) = 1/sqrt(2 ln b),
 * b = N, the batch size; N must be at least 2 (LPDT_EUNSUPPORTED otherwise).
 * Saved for the backward pass, each [C]: mean_out, range_out (fp32) and argmax_out / argmin_out
 * (int64): the first position of the maximum / minimum as flat pixel index (n*H + h)*W + w.
 * The backward pass gives the range's whole gradient to those two positions and returns dx,
 * dgamma, dbeta. */
size_t lpdt_range_bn_fwd_workspace_bytes(int N, int H, int W, int C);
size_t lpdt_range_bn_bwd_workspace_bytes(int N, int H, int W, int C);
int lpdt_range_bn_fwd(const float *x, int N, int H, int W, int C, const float *gamma, const float *beta,
                      float eps, float *y, float *mean_out, float *range_out, int64_t *argmax_out,
                      int64_t *argmin_out, void *ws, size_t ws_bytes, void *stream);
int lpdt_range_bn_bwd(const float *dy, const float *x, int N, int H, int W, int C, const float *gamma,
                      float eps, const float *mean, const float *range, const int64_t *argmax,
                      const int64_t *argmin, float *dx, float *dgamma, float *dbeta, void *ws,
                      size_t ws_bytes, void *stream);

/* ------------------------------------------------- 16-bit weight gradient
 * The weight-gradient product as Section 3 states it (gradient bifurcation): the layer
 * gradient enters in 16-bit floating point, the saved input codes in 8 bits:
 *   dw[k,r,s,c] = sx * sum_{n,p,q} g16[n,p,q,k] * xq[n, p*stride+r-pad, q*stride+s-pad, c]
 * g16: bfloat16 bit patterns [N,P,Q,K] (lpdt_to_bf16 makes them from fp32: round to nearest
 * even); xq int8 [N,H,W,C]; sx: device scalar, the scale of xq; dw fp32 [K,R,S,C], 16-byte
 * aligned, overwritten.  fp32 accumulation on the matrix cores in a fixed order (run-to-run
 * identical; within ~1e-6 of sum |g*x| of the exact sum).  This is an alternative to
 * lpdt_qconv_bwd_weight(_f32), which takes the 8-bit codes of the gradient.
 */
int lpdt_to_bf16(const float *x, size_t len, uint16_t *y, void *stream);
size_t lpdt_qconv_bwd_weight_bf16_workspace_bytes(const lpdt_conv_desc *d);
int lpdt_qconv_bwd_weight_bf16(const lpdt_conv_desc *d, const uint16_t *g16, const int8_t *xq,
                               const float *sx, float *dw, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------- gossip
 * Algorithm 1 step 7 for n agents whose parameter vectors are the rows of x.
 *   xhat == NULL (plain, D-PSGD / Algorithm 2 without compression):
 *       x_i <- x_i + rate * ( sum_j W_ij x_j - x_i )
 *   xhat != NULL (CHOCO-SGD, supplement Algorithm 3), per agent i and segment:
 *       v = x_i - xhat_i ;  q = v on the k entries of largest |v|, 0 elsewhere,
 *       k = max(1, ceil(keep_ratio*len)), ties resolved towards the lower index,
 *       |v| compared by fp32 bit pattern ;  xhat_i <- xhat_i + q  for all i ;  then
 *       x_i <- x_i + rate * sum_j W_ij (xhat_j - xhat_i).
 * W: HOST pointer, row-major [n][n], W[i*n+j] = weight node i gives node j's model;
 * read during the call (not retained).  Limits: n <= 64 and at most 8 non-zeros per
 * row, else LPDT_EUNSUPPORTED.  seg_offsets: HOST pointer, nseg+1 increasing offsets
 * with seg_offsets[0] = 0 and seg_offsets[nseg] = d (the layers of the model, for
 * layer-wise top-k); NULL / nseg = 0 means one segment [0,d).  Each segment must be
 * shorter than 2^31 elements.  x (and xhat) are updated in place.
 */
size_t lpdt_gossip_mix_workspace_bytes(int n, size_t d, int nseg, int choco);

int lpdt_gossip_mix(float *x, float *xhat, int n, size_t d, const float *W, float rate,
                    double keep_ratio, const int64_t *seg_offsets, int nseg, void *ws, size_t ws_bytes,
                    void *stream);

/* How the top-k selection of lpdt_gossip_mix / lpdt_gossip_mix_ex finds its threshold (the selected set is the same
 * either way, exactly): -1 (the default) lets the library choose by problem size; 0 forces the two-pass form (one pass
 * to histogram every key, one to collect); s > 0 forces the one-pass form that guesses the threshold's neighbourhood
 * from a sample of every s-th 4096-element tile and falls back to two passes for a segment whose guess missed.
 * Process-wide, takes effect at the next call; for tests and tuning.  LPDT_EINVAL for stride < -1. */
int lpdt_gossip_set_sample_stride(int stride);

/* The other gossip variants of the supplement, one step each (Algorithms "Deep-Squeeze",
 * "Sparse-Push", "Quant-SGP"); arguments as for lpdt_gossip_mix, plus:
 *   mode   LPDT_MIX_PLAIN (state must be NULL), LPDT_MIX_CHOCO (state = xhat, as above) or
 *          LPDT_MIX_DEEPSQUEEZE: state = delta [n][d], the error memory (zeros at the start):
 *              v = x_i + delta_i ;  C[v] = v on the top-k |v| of each segment (same rule as
 *              above), 0 elsewhere ;  delta_i <- v - C[v] ;
 *              x_i <- x_i + rate * ( sum_j W_ij C[v_j] - C[v_i] ).
 *   u      NULL, or the push-sum bias weights: n fp32 in DEVICE memory (ones at the start),
 *              u_i <- u_i + rate * ( sum_j W_ij u_j - u_i ),
 *          updated in place.  With u, W only has to be column stochastic (directed graphs), and
 *          LPDT_MIX_CHOCO mixes xhat by the same operator as u: x_i <- x_i + rate *
 *          ( sum_j W_ij xhat_j - xhat_i ), which is the form above whenever the rows of W sum
 *          to 1 (the printed difference form does not conserve sum_i x_i otherwise, and the
 *          de-biasing relies on that).  mode DEEPSQUEEZE + u = Sparse-Push, CHOCO + u = Quant-SGP.
 *   z      NULL, or [n][d] fp32 out (needs u): the de-biased models z_i = x_i / u_i after the step,
 *          on which the next gradients are taken.
 * Without u the rows of W must sum to 1 as well. */
enum { LPDT_MIX_PLAIN = 0, LPDT_MIX_CHOCO = 1, LPDT_MIX_DEEPSQUEEZE = 2 };

size_t lpdt_gossip_mix_ex_workspace_bytes(int n, size_t d, int nseg, int mode, int push_sum);

int lpdt_gossip_mix_ex(float *x, float *state, int n, size_t d, const float *W, float rate,
                       double keep_ratio, const int64_t *seg_offsets, int nseg, int mode, float *u,
                       float *z, void *ws, size_t ws_bytes, void *stream);

/* --------------------------------------------------------------------- glue
 * Table "hardware_training", rows Skip Connections and Average Pool, plus the
 * max-pool, loss and local SGD step (Algorithm 1 step 3) of the benchmark
 * networks.  All fp32, NHWC. */

/* y = a + b (y may alias a or b). */
int lpdt_add(const float *a, const float *b, size_t len, float *y, void *stream);

/* k x k window, stride st, padding pd (padding never wins).  idx[n,p,q,c] = h*W+w of the
 * winner (first in window scan order on ties). */
int lpdt_maxpool_fwd(const float *x, int N, int H, int W, int C, int k, int st, int pd, float *y,
                     int32_t *idx, void *stream);
/* dx[N,H,W,C] is overwritten: zero, then dx[n, idx, c] += dy[n,p,q,c]. */
int lpdt_maxpool_bwd(const float *dy, const int32_t *idx, int N, int H, int W, int C, int k, int st,
                     int pd, float *dx, void *stream);

/* global average pool: y[n,c] = mean over h,w ; dx[n,h,w,c] = dy[n,c]/(H*W). */
int lpdt_avgpool_fwd(const float *x, int N, int HW, int C, float *y, void *stream);
int lpdt_avgpool_bwd(const float *dy, int N, int HW, int C, float *dx, void *stream);

/* loss[0] = mean_n -log softmax(logits[n])[labels[n]] ; dlogits = (softmax - onehot)/N.
 * logits, dlogits fp32 [N,classes] (classes <= 1024); labels int32 [N] in [0,classes).
 * loss must have room for 1 + N floats: loss[1..N] receive the per-sample losses.  A label outside [0,classes)
 * is not dereferenced: that sample's loss (and so the mean) is NaN and its gradient row is softmax/N. */
int lpdt_softmax_xent(const float *logits, const int32_t *labels, int N, int classes, float *loss,
                      float *dlogits, void *stream);

/* x <- x - lr*g. */
int lpdt_sgd(float *x, const float *g, size_t len, float lr, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LPDT_H */
