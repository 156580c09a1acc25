// Error reporting shared by the host-side source files of the C ABI (text kept per thread,
// returned by petals_last_error()).
#pragma once
#include <hip/hip_runtime.h>

int ps_fail(int code, const char *fmt, ...);
int ps_hip_fail(hipError_t e, const char *what);
#define HIP_TRY(expr)                                           \
    do {                                                        \
        hipError_t e_ = (expr);                                 \
        if (e_ != hipSuccess) return ps_hip_fail(e_, #expr);    \
    } while (0)
