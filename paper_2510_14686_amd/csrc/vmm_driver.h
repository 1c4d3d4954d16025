// The five virtual-memory operations the xTensor page pool needs, behind one table, so that the
// pool's bookkeeping and failure handling can run against a host-only stand-in (tests without a GPU)
// as well as against the HIP virtual-memory API.  Every function returns an xattn_status and, on
// failure, has recorded a message with fail()/fail_hip().
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
};

// The driver in use: HIP, or the host-only stand-in while xtensor_test_fake_driver is on.
const VmmDriver& vmm_driver();

}  // namespace xattn
#endif
