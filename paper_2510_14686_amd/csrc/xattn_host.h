// Internal interface between the host translation units of libxattn.so.
#ifndef XATTN_HOST_H_
#define XATTN_HOST_H_

#include <stddef.h>
#include <stdint.h>

namespace xattn {

// Supplies a workspace of at least `bytes` bytes on device `device` without allocating, or fails with
// a recorded message.
typedef int (*FixedWorkspaceFn)(const char* who, int device, size_t bytes, char** ws_out);

int decode_call(const char* who, FixedWorkspaceFn fixed_workspace, const void* q, const void* const* k_ptrs,
                const void* const* v_ptrs, const int32_t* kv_lens, int batch, int q_len, int n_q_heads,
                int n_kv_heads, int head_dim, float scale, void* out, float* lse, void* stream);

}  // namespace xattn
#endif
