// Error reporting for failed HIP runtime calls (units that include the HIP runtime only).
#ifndef XATTN_HIP_ERROR_H_
#define XATTN_HIP_ERROR_H_

#include <hip/hip_runtime.h>

#include "../../include/xattn.h"
#include "xattn_internal.h"

namespace xattn {

// XATTN_ENOMEM for out-of-memory, XATTN_EHIP otherwise; the message names the call.
inline int fail_hip(hipError_t e, const char* what) {
    const int status = (e == hipErrorOutOfMemory) ? XATTN_ENOMEM : XATTN_EHIP;
    return fail(status, "%s failed: %s (%d)", what, hipGetErrorString(e), (int)e);
}

}  // namespace xattn
#endif
