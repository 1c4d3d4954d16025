// Host-only stand-in for the virtual-memory driver (see xtensor_test_hooks.h).  Test library only.
#include <cstdint>
#include <mutex>

#include "../../../include/xattn.h"
#include "../vmm_driver.h"
#include "../xattn_internal.h"
#include "xtensor_test_hooks.h"

namespace xattn {
namespace {

struct FakeState {
    std::mutex mu;
    uint64_t next_va = 0x100000000000ull;
    uint64_t next_handle = 1;
    size_t reservations = 0, handles = 0, mappings = 0;
    int fail_op = -1;        // index into the driver table (1 reserve, 3 create, 5 map, 6 unmap)
    int fail_after = 0;      // that many calls of fail_op succeed first
} g_fake;

bool should_fail(int op) {
    if (g_fake.fail_op != op) return false;
    if (g_fake.fail_after > 0) { --g_fake.fail_after; return false; }
    g_fake.fail_op = -1;     // fail once
    return true;
}
int fake_check_device(int device, size_t) {
    return device == 0 ? XATTN_OK : fail(XATTN_EINVAL, "device %d out of range", device);
}
int fake_reserve(size_t bytes, size_t align, void** va_out) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    if (should_fail(1)) return fail(XATTN_ENOMEM, "fake driver: reserve refused");
    g_fake.next_va = (g_fake.next_va + align - 1) / align * align;
    *va_out = reinterpret_cast<void*>(g_fake.next_va);
    g_fake.next_va += bytes;
    ++g_fake.reservations;
    return XATTN_OK;
}
int fake_free_va(void*, size_t) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    --g_fake.reservations;
    return XATTN_OK;
}
int fake_create(int, size_t, uint64_t* handle_out) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    if (should_fail(3)) return fail(XATTN_ENOMEM, "fake driver: create refused");
    *handle_out = g_fake.next_handle++;
    ++g_fake.handles;
    return XATTN_OK;
}
int fake_release(uint64_t) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    --g_fake.handles;
    return XATTN_OK;
}
int fake_map(void*, size_t, uint64_t, int) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    if (should_fail(5)) return fail(XATTN_EHIP, "fake driver: map refused");
    ++g_fake.mappings;
    return XATTN_OK;
}
int fake_unmap(void*, size_t) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    if (should_fail(6)) return fail(XATTN_EHIP, "fake driver: unmap refused");
    --g_fake.mappings;
    return XATTN_OK;
}
void fake_bind_thread(int) {}

const VmmDriver kFakeDriver = {fake_check_device, fake_reserve, fake_free_va, fake_create,
                               fake_release,      fake_map,     fake_unmap,   fake_bind_thread};

}  // namespace

const VmmDriver& vmm_driver() { return kFakeDriver; }

}  // namespace xattn

using namespace xattn;

extern "C" {

int xtensor_test_fail_next(int fail_op, int fail_after) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    g_fake.fail_op = fail_op;
    g_fake.fail_after = fail_after;
    return XATTN_OK;
}

int xtensor_test_fake_counts(size_t* reservations, size_t* handles, size_t* mappings) {
    std::lock_guard<std::mutex> lock(g_fake.mu);
    if (reservations) *reservations = g_fake.reservations;
    if (handles) *handles = g_fake.handles;
    if (mappings) *mappings = g_fake.mappings;
    return XATTN_OK;
}

}  // extern "C"
