// The virtual-memory operations the xTensor page pool needs, behind one table, so that the pool's
// bookkeeping and failure handling can be built against a host-only stand-in (CPU tests, sanitizer
// builds) as well as against the HIP virtual-memory API.  Every function returns an xattn_status
// and, on failure, has recorded a message with fail().  Exactly one translation unit of a library
// defines vmm_driver(): vmm_hip.cpp in libxattn.so, host_test/vmm_fake.cpp in the host test library.
#ifndef XATTN_VMM_DRIVER_H_
#define XATTN_VMM_DRIVER_H_

#include <cstddef>
#include <cstdint>

namespace xattn {

struct VmmDriver {
    int (*check_device)(int device, size_t page_bytes);          // device exists, granularity divides the page
    int (*reserve)(size_t bytes, size_t align, void** va_out);   // unbacked virtual range
    int (*free_va)(void* va, size_t bytes);
    int (*create)(int device, size_t bytes, uint64_t* handle_out);   // one physical page
    int (*release)(uint64_t handle);
    int (*map)(void* va, size_t bytes, uint64_t handle, int device); // map and make read-write on device
    int (*unmap)(void* va, size_t bytes);
    void (*bind_thread)(int device);                             // make `device` current for the calling thread
};

const VmmDriver& vmm_driver();

}  // namespace xattn
#endif
