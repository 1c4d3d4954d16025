// The calling thread's last error message (xattn_last_error) and the helper that records it.
#include <cstdarg>
#include <cstdio>

#include "../../include/xattn.h"
#include "xattn_internal.h"

namespace xattn {

static thread_local char g_error[512] = "";

int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return status;
}

}  // namespace xattn

extern "C" const char* xattn_last_error(void) { return xattn::g_error; }
