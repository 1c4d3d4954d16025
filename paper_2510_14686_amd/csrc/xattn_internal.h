// Shared by the host translation units of libxattn.so: error reporting.
#ifndef XATTN_INTERNAL_H_
#define XATTN_INTERNAL_H_

#include <hip/hip_runtime.h>

namespace xattn {

// Record a printf-style message for xattn_last_error() and return `status`.
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
// Same for a failed HIP call: XATTN_ENOMEM for out-of-memory, XATTN_EHIP otherwise.
int fail_hip(hipError_t e, const char* what);

}  // namespace xattn
#endif
