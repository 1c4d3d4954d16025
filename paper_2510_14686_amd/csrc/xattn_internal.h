// Shared by the host translation units of libxattn.so: error reporting.  No HIP types here, so that
// the host-only units (page pool, beam search) also compile with a plain C++ compiler.
#ifndef XATTN_INTERNAL_H_
#define XATTN_INTERNAL_H_

namespace xattn {

// Record a printf-style message for xattn_last_error() and return `status`.
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace xattn
#endif
