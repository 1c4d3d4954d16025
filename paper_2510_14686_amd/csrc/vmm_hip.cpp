// The page pool's driver table on the HIP virtual-memory API (hipMemAddressReserve / hipMemCreate /
// hipMemMap / hipMemSetAccess): paper section 4.3, "Physical Memory Page Management" and "On-demand
// Memory Mapping" -- physical pages are created apart from the virtual range and mapped into it later.
#include <hip/hip_runtime.h>

#include "../../include/xattn.h"
#include "vmm_driver.h"
#include "xattn_hip_error.h"

namespace xattn {
namespace {

hipMemAllocationProp page_prop(int device) {
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    return prop;
}

int hip_check_device(int device, size_t page_bytes) {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess) return fail_hip(e, "hipGetDeviceCount");
    if (device < 0 || device >= n) return fail(XATTN_EINVAL, "device %d out of range", device);
    const hipMemAllocationProp prop = page_prop(device);
    size_t gran = 0;
    e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum);
    if (e != hipSuccess) return fail_hip(e, "hipMemGetAllocationGranularity");
    if (gran == 0 || page_bytes % gran != 0)
        return fail(XATTN_EUNSUPPORTED, "mapping granularity %zu does not divide the %zu-byte page", gran, page_bytes);
    return XATTN_OK;
}
int hip_reserve(size_t bytes, size_t align, void** va_out) {
    hipError_t e = hipMemAddressReserve(va_out, bytes, align, nullptr, 0);
    return e == hipSuccess ? XATTN_OK : fail_hip(e, "hipMemAddressReserve");
}
int hip_free_va(void* va, size_t bytes) {
    hipError_t e = hipMemAddressFree(va, bytes);
    return e == hipSuccess ? XATTN_OK : fail_hip(e, "hipMemAddressFree");
}
int hip_create(int device, size_t bytes, uint64_t* handle_out) {
    const hipMemAllocationProp prop = page_prop(device);
    hipMemGenericAllocationHandle_t h;
    hipError_t e = hipMemCreate(&h, bytes, &prop, 0);
    if (e != hipSuccess) return fail_hip(e, "hipMemCreate");
    *handle_out = (uint64_t)(uintptr_t)h;
    return XATTN_OK;
}
int hip_release(uint64_t handle) {
    hipError_t e = hipMemRelease((hipMemGenericAllocationHandle_t)(uintptr_t)handle);
    return e == hipSuccess ? XATTN_OK : fail_hip(e, "hipMemRelease");
}
int hip_map(void* va, size_t bytes, uint64_t handle, int device) {
    hipError_t e = hipMemMap(va, bytes, 0, (hipMemGenericAllocationHandle_t)(uintptr_t)handle, 0);
    if (e != hipSuccess) return fail_hip(e, "hipMemMap");
    hipMemAccessDesc access = {};
    access.location.type = hipMemLocationTypeDevice;
    access.location.id = device;
    access.flags = hipMemAccessFlagsProtReadWrite;
    e = hipMemSetAccess(va, bytes, &access, 1);
    if (e != hipSuccess) {
        (void)hipMemUnmap(va, bytes);
        return fail_hip(e, "hipMemSetAccess");
    }
    return XATTN_OK;
}
int hip_unmap(void* va, size_t bytes) {
    hipError_t e = hipMemUnmap(va, bytes);
    return e == hipSuccess ? XATTN_OK : fail_hip(e, "hipMemUnmap");
}
void hip_bind_thread(int device) { (void)hipSetDevice(device); }

const VmmDriver kHipDriver = {hip_check_device, hip_reserve, hip_free_va, hip_create,
                              hip_release,      hip_map,     hip_unmap,   hip_bind_thread};

}  // namespace

const VmmDriver& vmm_driver() { return kHipDriver; }

}  // namespace xattn
