// xattn_decode_noalloc: the decode call for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid it).  The partial results of split
// sequences, which xattn_decode keeps in a workspace from hipMalloc, live here in a device array of
// fixed size that is part of the library's code object; every GPU holds its own copy until the
// process ends.  Same kernels, same partition and therefore the same bits as xattn_decode.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/xattn.h"
#include "xattn_hip_error.h"
#include "xattn_host.h"

namespace {

constexpr size_t kScratchBytes = XATTN_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 16;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mu;
char* g_scratch_ptr[kMaxDevices] = {};     // the array's address on each device, resolved on first use

// In host code `scratch` is only a handle for the runtime; the memory is reached through the address
// hipGetSymbolAddress returns for the current device.
int scratch_workspace(const char* who, int device, size_t bytes, char** ws_out) {
    if (bytes > kScratchBytes)
        return xattn::fail(XATTN_EUNSUPPORTED, "%s: this shape needs %zu bytes for partial results, the fixed scratch array holds %zu; "
                           "use xattn_decode (or fewer pieces)", who, bytes, kScratchBytes);
    if (device < 0 || device >= kMaxDevices) return xattn::fail(XATTN_EUNSUPPORTED, "%s: device index %d not supported", who, device);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));      // `device` is the current device
        if (e != hipSuccess) return xattn::fail_hip(e, "hipGetSymbolAddress(scratch)");
        if (!ptr) return xattn::fail(XATTN_EHIP, "%s: hipGetSymbolAddress returned no address", who);
        g_scratch_ptr[device] = static_cast<char*>(ptr);
    }
    *ws_out = g_scratch_ptr[device];
    return XATTN_OK;
}

}  // namespace

extern "C" int xattn_decode_noalloc(const void* q, const void* const* k_ptrs, const void* const* v_ptrs,
                                    const int32_t* kv_lens, int batch, int q_len, int n_q_heads, int n_kv_heads,
                                    int head_dim, float scale, void* out, float* lse, void* stream) {
    return xattn::decode_call("xattn_decode_noalloc", scratch_workspace, q, k_ptrs, v_ptrs, kv_lens, batch, q_len,
                              n_q_heads, n_kv_heads, head_dim, scale, out, lse, stream);
}
