// xTensor ranges (paper section 4.3): a reserved, initially unbacked virtual range per tensor of a
// request, backed on demand by discrete fixed-size physical chunks through the HIP virtual-memory
// API.  Kernels see one contiguous address range; the MMU does the address -> (page, offset) step.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <new>
#include <unordered_set>
#include <vector>

#include "../../include/xattn.h"
#include "xattn_hip_error.h"

namespace xattn {
namespace {

struct Range {
    int device = 0;
    char* base = nullptr;             // reserved virtual range
    size_t reserve_bytes = 0;
    size_t mapped_chunks = 0;         // chunks [0, mapped_chunks) of the range are mapped
    std::vector<hipMemGenericAllocationHandle_t> chunks;   // physical chunks in creation order
    std::vector<int32_t> order;       // order[i]: creation index of the chunk behind virtual chunk i
    char* view = nullptr;             // optional second mapping in creation order
    size_t view_chunks = 0;
};

std::mutex g_mutex;
std::unordered_set<Range*> g_live;

uint64_t next_u64(uint64_t& s) {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

hipMemAllocationProp chunk_prop(int device) {
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    return prop;
}

// Undo everything a range holds.  Returns the first HIP error met, but keeps going.
hipError_t destroy(Range* r) {
    hipError_t first = hipSuccess;
    auto note = [&](hipError_t e) { if (e != hipSuccess && first == hipSuccess) first = e; };
    if (r->view) {
        for (size_t i = 0; i < r->view_chunks; ++i) note(hipMemUnmap(r->view + i * XTENSOR_CHUNK_BYTES, XTENSOR_CHUNK_BYTES));
        note(hipMemAddressFree(r->view, r->chunks.size() * XTENSOR_CHUNK_BYTES));
        r->view = nullptr;
    }
    for (size_t i = 0; i < r->mapped_chunks; ++i) note(hipMemUnmap(r->base + i * XTENSOR_CHUNK_BYTES, XTENSOR_CHUNK_BYTES));
    r->mapped_chunks = 0;
    for (auto h : r->chunks) note(hipMemRelease(h));
    r->chunks.clear();
    if (r->base) note(hipMemAddressFree(r->base, r->reserve_bytes));
    r->base = nullptr;
    return first;
}

}  // namespace
}  // namespace xattn

using namespace xattn;

extern "C" {

int xtensor_map(size_t reserve_bytes, size_t mapped_bytes, uint64_t seed, int device, void** base_out,
                void** handle_out) {
    if (!base_out || !handle_out) return fail(XATTN_EINVAL, "xtensor_map: base_out and handle_out must not be NULL");
    *base_out = nullptr;
    *handle_out = nullptr;
    if (reserve_bytes == 0) return fail(XATTN_EINVAL, "xtensor_map: reserve_bytes is 0");
    const size_t chunk = XTENSOR_CHUNK_BYTES;
    const size_t n_reserve = (reserve_bytes + chunk - 1) / chunk;
    const size_t n_map = (mapped_bytes + chunk - 1) / chunk;
    if (n_map > n_reserve)
        return fail(XATTN_EINVAL, "xtensor_map: mapped_bytes (%zu) exceeds reserve_bytes (%zu)", mapped_bytes, reserve_bytes);
    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDeviceCount");
    if (device < 0 || device >= n_dev) return fail(XATTN_EINVAL, "xtensor_map: device %d out of range", device);

    hipMemAllocationProp prop = chunk_prop(device);
    size_t gran = 0;
    e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum);
    if (e != hipSuccess) return fail_hip(e, "hipMemGetAllocationGranularity");
    if (gran == 0 || chunk % gran != 0)
        return fail(XATTN_EUNSUPPORTED, "xtensor_map: mapping granularity %zu does not divide the 2 MiB chunk", gran);

    Range* r = new (std::nothrow) Range();
    if (!r) return fail(XATTN_ENOMEM, "xtensor_map: host allocation failed");
    r->device = device;
    r->reserve_bytes = n_reserve * chunk;

    int status = XATTN_OK;
    do {
        void* base = nullptr;
        e = hipMemAddressReserve(&base, r->reserve_bytes, chunk, nullptr, 0);
        if (e != hipSuccess) { status = fail_hip(e, "hipMemAddressReserve"); break; }
        r->base = static_cast<char*>(base);
        r->chunks.reserve(n_map);
        for (size_t i = 0; i < n_map; ++i) {
            hipMemGenericAllocationHandle_t h;
            e = hipMemCreate(&h, chunk, &prop, 0);
            if (e != hipSuccess) { status = fail_hip(e, "hipMemCreate"); break; }
            r->chunks.push_back(h);
        }
        if (status != XATTN_OK) break;
        // Fisher-Yates shuffle of the creation indices.
        r->order.resize(n_map);
        for (size_t i = 0; i < n_map; ++i) r->order[i] = (int32_t)i;
        uint64_t s = seed;
        for (size_t i = n_map; i > 1; --i) {
            const size_t j = (size_t)(next_u64(s) % i);
            const int32_t t = r->order[i - 1];
            r->order[i - 1] = r->order[j];
            r->order[j] = t;
        }
        hipMemAccessDesc access = {};
        access.location.type = hipMemLocationTypeDevice;
        access.location.id = device;
        access.flags = hipMemAccessFlagsProtReadWrite;
        for (size_t i = 0; i < n_map; ++i) {
            char* va = r->base + i * chunk;
            e = hipMemMap(va, chunk, 0, r->chunks[r->order[i]], 0);
            if (e != hipSuccess) { status = fail_hip(e, "hipMemMap"); break; }
            r->mapped_chunks = i + 1;
            e = hipMemSetAccess(va, chunk, &access, 1);
            if (e != hipSuccess) { status = fail_hip(e, "hipMemSetAccess"); break; }
        }
    } while (false);

    if (status != XATTN_OK) {
        (void)destroy(r);      // keeps the message of the first failure
        delete r;
        return status;
    }
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        g_live.insert(r);
    }
    *base_out = r->base;
    *handle_out = r;
    return XATTN_OK;
}

int xtensor_unmap(void* handle) {
    Range* r = static_cast<Range*>(handle);
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        if (!r || g_live.erase(r) == 0) return fail(XATTN_EINVAL, "xtensor_unmap: not a live xTensor handle");
    }
    const hipError_t e = destroy(r);
    delete r;
    if (e != hipSuccess) return fail_hip(e, "xtensor_unmap (unmap / release / address free)");
    return XATTN_OK;
}

int xtensor_chunk_order(void* handle, int32_t* order_out, int n) {
    Range* r = static_cast<Range*>(handle);
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!r || g_live.count(r) == 0) return fail(XATTN_EINVAL, "xtensor_chunk_order: not a live xTensor handle");
    const int count = (int)r->order.size();
    if (count > 0 && (!order_out || n < count))
        return fail(XATTN_EINVAL, "xtensor_chunk_order: order_out holds %d entries, %d needed", n, count);
    for (int i = 0; i < count; ++i) order_out[i] = r->order[i];
    return count;
}

int xtensor_physical_view(void* handle, void** view_out) {
    if (!view_out) return fail(XATTN_EINVAL, "xtensor_physical_view: view_out is NULL");
    *view_out = nullptr;
    Range* r = static_cast<Range*>(handle);
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!r || g_live.count(r) == 0) return fail(XATTN_EINVAL, "xtensor_physical_view: not a live xTensor handle");
    if (r->chunks.empty()) return fail(XATTN_EINVAL, "xtensor_physical_view: the range has no mapped chunk");
    if (r->view) { *view_out = r->view; return XATTN_OK; }
    const size_t chunk = XTENSOR_CHUNK_BYTES;
    const size_t bytes = r->chunks.size() * chunk;
    void* base = nullptr;
    hipError_t e = hipMemAddressReserve(&base, bytes, chunk, nullptr, 0);
    if (e != hipSuccess) return fail_hip(e, "hipMemAddressReserve(view)");
    r->view = static_cast<char*>(base);
    r->view_chunks = 0;
    hipMemAccessDesc access = {};
    access.location.type = hipMemLocationTypeDevice;
    access.location.id = r->device;
    access.flags = hipMemAccessFlagsProtReadWrite;
    int status = XATTN_OK;
    for (size_t i = 0; i < r->chunks.size(); ++i) {
        char* va = r->view + i * chunk;
        e = hipMemMap(va, chunk, 0, r->chunks[i], 0);
        if (e != hipSuccess) { status = fail_hip(e, "hipMemMap(view)"); break; }
        r->view_chunks = i + 1;
        e = hipMemSetAccess(va, chunk, &access, 1);
        if (e != hipSuccess) { status = fail_hip(e, "hipMemSetAccess(view)"); break; }
    }
    if (status != XATTN_OK) {
        for (size_t i = 0; i < r->view_chunks; ++i) (void)hipMemUnmap(r->view + i * chunk, chunk);
        (void)hipMemAddressFree(r->view, bytes);
        r->view = nullptr;
        r->view_chunks = 0;
        return status;
    }
    *view_out = r->view;
    return XATTN_OK;
}

}  // extern "C"
