// Shared host/device helpers of the lpdt HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/lpdt.h"

namespace lpdt {

// Records a thread-local message and returns `code`.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();
// Checks hipGetLastError() after a launch.
int launch_status(const char *what);

static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }
static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int conv_out(int in, int pad, int filt, int stride) { return (in + 2 * pad - filt) / stride + 1; }

// Validates a convolution descriptor; on success fills P, Q.
int check_conv(const lpdt_conv_desc *d, int *P, int *Q);
int check_ws(const void *ws, size_t ws_bytes, size_t need);

#define LPDT_REQUIRE(cond, code, ...) \
    do { if (!(cond)) return ::lpdt::fail(code, __VA_ARGS__); } while (0)

constexpr int kWave = 64;

// A 16-byte load of data that is read once (streaming passes): the nontemporal form, which leaves the caches to data
// that is reused.  On this machine a read-only pass over 1.4 GB runs 10 % faster with it.
typedef float lpdt_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float4 *p) {
    const lpdt_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const lpdt_f32x4 *>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}

// ---- device helpers --------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// s*a (+ prev) as two separately rounded operations: what lpdt_dequantize computes, also in fused epilogues
__device__ __forceinline__ float dequant_value(float s, int a, float prev, bool accumulate) {
#pragma clang fp contract(off)
    const float v = s * (float)a;
    return accumulate ? prev + v : v;
}

// 127 / a, the factor that maps a tensor of abs-max a onto the code grid: one fp32 division; 0 for a == 0 and for an
// abs-max so small (below about 3.7e-37) that the quotient is not a finite float -- such a tensor counts as zero.
__device__ __forceinline__ float quant_inv(float a) {
    const float inv = (a > 0.0f) ? __fdiv_rn(127.0f, a) : 0.0f;
    return inv <= 3.4028234663852886e38f ? inv : 0.0f;
}
// the scale that goes with it: a / 127, or 0 where quant_inv is 0
__device__ __forceinline__ float quant_scale(float a) { return quant_inv(a) > 0.0f ? __fdiv_rn(a, 127.0f) : 0.0f; }

// The quantizer's code for x with inv = 127 / max|x|: nearest (ties to even) or stochastic with the uniform number
// u = (word >> 8) * 2^-24; clipped to [-127, 127].  Shared by every kernel that emits codes.
__device__ __forceinline__ int round_code(float x, float inv, bool stochastic, uint32_t word) {
#pragma clang fp contract(off)
    const float t = __fmul_rn(x, inv);  // its own rounding: must not fuse with the subtraction below
    float r;
    if (stochastic) {
        const float f = floorf(t);
        const float frac = __fsub_rn(t, f);
        const float u = __fmul_rn((float)(word >> 8), 0x1.0p-24f);
        r = f + ((u < frac) ? 1.0f : 0.0f);
    } else {
        r = rintf(t);
    }
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

}  // namespace lpdt
