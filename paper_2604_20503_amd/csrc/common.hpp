// Shared host-side plumbing of the faser_verify library: status codes, last-error text,
// launch checking.  Device helpers that several kernels use live in device_utils.hpp.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>

#include "../../include/faser_verify.h"

namespace fsr {

char* error_buffer();  // thread-local, 256 bytes

// A number no earlier call of this process has used (48 bits, never 0): tags what a call leaves in a workspace.
unsigned long long next_call_id();

inline int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 256, fmt, ap);
    va_end(ap);
    return code;
}

inline int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FSR_EHIP, "%s: %s", what, hipGetErrorString(e));
    return FSR_OK;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace fsr
