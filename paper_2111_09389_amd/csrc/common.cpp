// Error reporting and argument checks shared by every entry point.
#include "common.h"
#include <cstdarg>
#include <cstdio>

namespace lpdt {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = 0; }

int launch_status(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LPDT_EHIP, "%s: %s", what, hipGetErrorString(e));
    return LPDT_OK;
}

int check_conv(const lpdt_conv_desc *d, int *P, int *Q) {
    LPDT_REQUIRE(d, LPDT_EINVAL, "conv descriptor is NULL");
    LPDT_REQUIRE(d->N > 0 && d->C > 0 && d->H > 0 && d->W > 0 && d->K > 0 && d->R > 0 && d->S > 0, LPDT_EINVAL,
                 "conv descriptor: sizes must be positive (N=%d C=%d H=%d W=%d K=%d R=%d S=%d)", d->N, d->C, d->H,
                 d->W, d->K, d->R, d->S);
    LPDT_REQUIRE(d->stride_h > 0 && d->stride_w > 0 && d->pad_h >= 0 && d->pad_w >= 0, LPDT_EINVAL,
                 "conv descriptor: stride must be positive and padding non-negative");
    LPDT_REQUIRE(d->H + 2 * d->pad_h >= d->R && d->W + 2 * d->pad_w >= d->S, LPDT_EINVAL,
                 "conv descriptor: filter larger than padded input");
    LPDT_REQUIRE(d->pad_h < d->R && d->pad_w < d->S, LPDT_EUNSUPPORTED, "conv descriptor: padding >= filter size");
    *P = conv_out(d->H, d->pad_h, d->R, d->stride_h);
    *Q = conv_out(d->W, d->pad_w, d->S, d->stride_w);
    const long long lim = 0x7fffffffLL;
    LPDT_REQUIRE((long long)d->N * d->H * d->W * d->C <= lim && (long long)d->N * *P * *Q * d->K <= lim &&
                     (long long)d->K * d->R * d->S * d->C <= lim,
                 LPDT_EUNSUPPORTED, "conv descriptor: a tensor has more than 2^31-1 elements");
    return LPDT_OK;
}

int check_ws(const void *ws, size_t ws_bytes, size_t need) {
    if (need == 0) return LPDT_OK;
    LPDT_REQUIRE(ws, LPDT_EWORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    LPDT_REQUIRE(aligned(ws, 256), LPDT_EWORKSPACE, "workspace must be 256-byte aligned");
    LPDT_REQUIRE(ws_bytes >= need, LPDT_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    return LPDT_OK;
}

}  // namespace lpdt

extern "C" const char *lpdt_last_error(void) { return lpdt::g_err; }
extern "C" int lpdt_version(void) { return 100; }
