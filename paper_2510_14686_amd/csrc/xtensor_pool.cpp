// xTensor page pool and per-request ranges (paper section 4.3):
//   * "Physical Memory Page Management": a pool of fixed-size physical pages created up front, each
//     with the triple <PageID, Status, OwnerSession>, Status in {Free, Allocated, Mapped, Reusable};
//   * "Virtual Memory Tensor Management": a request reserves MaxSeqLen worth of virtual addresses
//     that are not backed at first;
//   * "On-demand Memory Mapping": as the sequence grows, free pages are mapped at the next address;
//   * "Low Overhead Allocation": a finished request's pages stay mapped and are marked Reusable; a new
//     request whose size matches such a set takes the whole range over (no Map/Unmap); pages for the
//     next tokens are mapped ahead of time by a background thread.
// Host code only, no HIP types: the driver calls go through the table of vmm_driver.h.  The kernels
// never see any of this (they get a base address and a length).
#include <condition_variable>
#include <cstdint>
#include <deque>
#include <list>
#include <mutex>
#include <new>
#include <thread>
#include <unordered_set>
#include <vector>

#include "../../include/xattn.h"
#include "vmm_driver.h"
#include "xattn_internal.h"

namespace xattn {
namespace {

// ------------------------------------------------------------------------------------ pool
constexpr size_t kPage = XTENSOR_CHUNK_BYTES;

struct Pool;

struct PoolRange {
    Pool* pool = nullptr;
    uint64_t session = 0;
    char* base = nullptr;
    size_t reserve_pages = 0;
    std::vector<int64_t> pages;      // page ids behind virtual pages 0, 1, ...
    bool reusable = false;           // closed, pages kept mapped for a later request
    int async_status = XATTN_OK;     // result of the last pre-mapping request
    int async_pending = 0;
};

struct Page {
    uint64_t handle = 0;
    int status = XTENSOR_PAGE_FREE;
    uint64_t owner = 0;
};

struct PremapJob {
    PoolRange* range;
    size_t pages;
};

struct Pool {
    int device = 0;
    std::mutex mu;                      // guards everything below, driver calls included
    std::condition_variable cv_jobs, cv_done;
    std::vector<Page> pages;
    std::vector<int64_t> free_list;     // taken from the back
    std::unordered_set<PoolRange*> live;
    std::list<PoolRange*> reusable;     // oldest first
    std::deque<PremapJob> jobs;
    std::thread worker;
    bool stop = false;
};

std::mutex g_pools_mu;
std::unordered_set<Pool*> g_pools;
std::unordered_set<PoolRange*> g_ranges;     // every live or reusable range of every pool

uint64_t mix(uint64_t& s) {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Unmap a range's pages back to Free and free its addresses.  Pool mutex held.
int drop_range(Pool* p, PoolRange* r) {
    int first = XATTN_OK;
    for (size_t i = r->pages.size(); i-- > 0;) {
        const int st = vmm_driver().unmap(r->base + i * kPage, kPage);
        if (st != XATTN_OK && first == XATTN_OK) first = st;
        Page& pg = p->pages[(size_t)r->pages[i]];
        pg.status = XTENSOR_PAGE_FREE;
        pg.owner = 0;
        p->free_list.push_back(r->pages[i]);
    }
    r->pages.clear();
    const int st = vmm_driver().free_va(r->base, r->reserve_pages * kPage);
    if (st != XATTN_OK && first == XATTN_OK) first = st;
    return first;
}

// Make the first want_pages pages of the range backed.  Pool mutex held.  Returns pages mapped or <0.
int grow_locked(Pool* p, PoolRange* r, size_t want_pages) {
    if (want_pages > r->reserve_pages)
        return fail(XATTN_EINVAL, "xtensor: %zu pages asked, the range reserves %zu", want_pages, r->reserve_pages);
    int mapped = 0;
    while (r->pages.size() < want_pages) {
        if (p->free_list.empty()) {
            // Lazy release: give up the oldest Reusable set.
            if (p->reusable.empty())
                return fail(XATTN_ENOMEM, "xtensor: page pool exhausted (%zu pages, none free or reusable)", p->pages.size());
            PoolRange* victim = p->reusable.front();
            p->reusable.pop_front();
            const int st = drop_range(p, victim);
            {
                std::lock_guard<std::mutex> lock(g_pools_mu);
                g_ranges.erase(victim);
            }
            delete victim;
            if (st != XATTN_OK) return st;
            continue;
        }
        const int64_t id = p->free_list.back();
        p->free_list.pop_back();
        Page& pg = p->pages[(size_t)id];
        pg.status = XTENSOR_PAGE_ALLOCATED;
        pg.owner = r->session;
        const int st = vmm_driver().map(r->base + r->pages.size() * kPage, kPage, pg.handle, p->device);
        if (st != XATTN_OK) {
            pg.status = XTENSOR_PAGE_FREE;
            pg.owner = 0;
            p->free_list.push_back(id);
            return st;
        }
        pg.status = XTENSOR_PAGE_MAPPED;
        r->pages.push_back(id);
        ++mapped;
    }
    return mapped;
}

void worker_main(Pool* p) {
    vmm_driver().bind_thread(p->device);
    std::unique_lock<std::mutex> lock(p->mu);
    for (;;) {
        p->cv_jobs.wait(lock, [&] { return p->stop || !p->jobs.empty(); });
        if (p->jobs.empty()) return;       // stop requested and nothing left
        const PremapJob job = p->jobs.front();
        p->jobs.pop_front();
        const int st = grow_locked(p, job.range, job.pages);
        job.range->async_status = st < 0 ? st : XATTN_OK;
        --job.range->async_pending;
        p->cv_done.notify_all();
    }
}

Pool* live_pool(void* handle) {
    Pool* p = static_cast<Pool*>(handle);
    std::lock_guard<std::mutex> lock(g_pools_mu);
    return (p && g_pools.count(p)) ? p : nullptr;
}
PoolRange* live_range(void* handle) {
    PoolRange* r = static_cast<PoolRange*>(handle);
    std::lock_guard<std::mutex> lock(g_pools_mu);
    return (r && g_ranges.count(r)) ? r : nullptr;
}
size_t pages_for(size_t bytes) { return (bytes + kPage - 1) / kPage; }

}  // namespace

}  // namespace xattn

using namespace xattn;

extern "C" {

int xtensor_pool_create(int device, size_t n_pages, uint64_t seed, void** pool_out) {
    if (!pool_out) return fail(XATTN_EINVAL, "xtensor_pool_create: pool_out is NULL");
    *pool_out = nullptr;
    if (n_pages == 0 || n_pages > ((size_t)1 << 24)) return fail(XATTN_EINVAL, "xtensor_pool_create: n_pages %zu out of range", n_pages);
    int st = vmm_driver().check_device(device, kPage);
    if (st != XATTN_OK) return st;
    Pool* p = new (std::nothrow) Pool();
    if (!p) return fail(XATTN_ENOMEM, "xtensor_pool_create: host allocation failed");
    p->device = device;
    p->pages.reserve(n_pages);
    for (size_t i = 0; i < n_pages; ++i) {
        Page pg;
        st = vmm_driver().create(device, kPage, &pg.handle);
        if (st != XATTN_OK) break;
        p->pages.push_back(pg);
    }
    if (st != XATTN_OK) {
        for (auto& pg : p->pages) (void)vmm_driver().release(pg.handle);
        delete p;
        return st;
    }
    // Free list in a seeded random order, so that pages taken one after the other are not neighbours.
    p->free_list.resize(n_pages);
    for (size_t i = 0; i < n_pages; ++i) p->free_list[i] = (int64_t)i;
    uint64_t s = seed;
    for (size_t i = n_pages; i > 1; --i) {
        const size_t j = (size_t)(mix(s) % i);
        std::swap(p->free_list[i - 1], p->free_list[j]);
    }
    p->worker = std::thread(worker_main, p);
    {
        std::lock_guard<std::mutex> lock(g_pools_mu);
        g_pools.insert(p);
    }
    *pool_out = p;
    return XATTN_OK;
}

int xtensor_pool_destroy(void* pool) {
    Pool* p = live_pool(pool);
    if (!p) return fail(XATTN_EINVAL, "xtensor_pool_destroy: not a live pool");
    {
        std::unique_lock<std::mutex> lock(p->mu);
        if (!p->live.empty())
            return fail(XATTN_EINVAL, "xtensor_pool_destroy: %zu ranges are still open", p->live.size());
        p->stop = true;
        p->cv_jobs.notify_all();
    }
    p->worker.join();
    int first = XATTN_OK;
    {
        std::lock_guard<std::mutex> lock(p->mu);
        for (PoolRange* r : p->reusable) {
            const int st = drop_range(p, r);
            if (st != XATTN_OK && first == XATTN_OK) first = st;
            {
                std::lock_guard<std::mutex> l2(g_pools_mu);
                g_ranges.erase(r);
            }
            delete r;
        }
        p->reusable.clear();
        for (auto& pg : p->pages) {
            const int st = vmm_driver().release(pg.handle);
            if (st != XATTN_OK && first == XATTN_OK) first = st;
        }
    }
    {
        std::lock_guard<std::mutex> lock(g_pools_mu);
        g_pools.erase(p);
    }
    delete p;
    return first;
}

int xtensor_pool_counts(void* pool, size_t* counts_out) {
    Pool* p = live_pool(pool);
    if (!p || !counts_out) return fail(XATTN_EINVAL, "xtensor_pool_counts: not a live pool, or counts_out is NULL");
    std::lock_guard<std::mutex> lock(p->mu);
    for (int i = 0; i < 4; ++i) counts_out[i] = 0;
    for (const auto& pg : p->pages) ++counts_out[pg.status];
    return XATTN_OK;
}

int xtensor_page_info(void* pool, size_t page_id, int* status_out, uint64_t* owner_out) {
    Pool* p = live_pool(pool);
    if (!p) return fail(XATTN_EINVAL, "xtensor_page_info: not a live pool");
    std::lock_guard<std::mutex> lock(p->mu);
    if (page_id >= p->pages.size()) return fail(XATTN_EINVAL, "xtensor_page_info: page %zu of %zu", page_id, p->pages.size());
    if (status_out) *status_out = p->pages[page_id].status;
    if (owner_out) *owner_out = p->pages[page_id].owner;
    return XATTN_OK;
}

int xtensor_open(void* pool, uint64_t session, size_t reserve_bytes, size_t mapped_bytes, void** base_out,
                 void** range_out, int* reused_out) {
    if (!base_out || !range_out) return fail(XATTN_EINVAL, "xtensor_open: base_out and range_out must not be NULL");
    *base_out = nullptr;
    *range_out = nullptr;
    if (reused_out) *reused_out = 0;
    Pool* p = live_pool(pool);
    if (!p) return fail(XATTN_EINVAL, "xtensor_open: not a live pool");
    if (reserve_bytes == 0 || mapped_bytes > reserve_bytes)
        return fail(XATTN_EINVAL, "xtensor_open: reserve_bytes %zu, mapped_bytes %zu", reserve_bytes, mapped_bytes);
    const size_t reserve_pages = pages_for(reserve_bytes), want = pages_for(mapped_bytes);
    std::lock_guard<std::mutex> lock(p->mu);
    // Page reuse: a Reusable set of exactly the wanted size, in a range at least as large, is taken
    // over as it is (newest first: its pages are the likeliest to be warm in the TLBs).
    if (want > 0) {
        for (auto it = p->reusable.rbegin(); it != p->reusable.rend(); ++it) {
            PoolRange* r = *it;
            if (r->pages.size() != want || r->reserve_pages < reserve_pages) continue;
            p->reusable.erase(std::next(it).base());
            r->reusable = false;
            r->session = session;
            for (int64_t id : r->pages) {
                p->pages[(size_t)id].status = XTENSOR_PAGE_MAPPED;
                p->pages[(size_t)id].owner = session;
            }
            p->live.insert(r);
            *base_out = r->base;
            *range_out = r;
            if (reused_out) *reused_out = 1;
            return XATTN_OK;
        }
    }
    PoolRange* r = new (std::nothrow) PoolRange();
    if (!r) return fail(XATTN_ENOMEM, "xtensor_open: host allocation failed");
    r->pool = p;
    r->session = session;
    r->reserve_pages = reserve_pages;
    void* va = nullptr;
    int st = vmm_driver().reserve(reserve_pages * kPage, kPage, &va);
    if (st != XATTN_OK) {
        delete r;
        return st;
    }
    r->base = static_cast<char*>(va);
    st = grow_locked(p, r, want);
    if (st < 0) {
        (void)drop_range(p, r);      // keeps the first failure's message
        delete r;
        return st;
    }
    p->live.insert(r);
    {
        std::lock_guard<std::mutex> l2(g_pools_mu);
        g_ranges.insert(r);
    }
    *base_out = r->base;
    *range_out = r;
    return XATTN_OK;
}

int xtensor_grow(void* range, size_t mapped_bytes) {
    PoolRange* r = live_range(range);
    if (!r || r->reusable) return fail(XATTN_EINVAL, "xtensor_grow: not an open range");
    Pool* p = r->pool;
    std::unique_lock<std::mutex> lock(p->mu);
    p->cv_done.wait(lock, [&] { return r->async_pending == 0; });     // pre-mapping in flight goes first
    return grow_locked(p, r, pages_for(mapped_bytes));
}

int xtensor_premap_async(void* range, size_t mapped_bytes) {
    PoolRange* r = live_range(range);
    if (!r || r->reusable) return fail(XATTN_EINVAL, "xtensor_premap_async: not an open range");
    Pool* p = r->pool;
    const size_t want = pages_for(mapped_bytes);
    if (want > r->reserve_pages)
        return fail(XATTN_EINVAL, "xtensor_premap_async: %zu pages asked, the range reserves %zu", want, r->reserve_pages);
    std::lock_guard<std::mutex> lock(p->mu);
    ++r->async_pending;
    p->jobs.push_back({r, want});
    p->cv_jobs.notify_one();
    return XATTN_OK;
}

int xtensor_premap_wait(void* range) {
    PoolRange* r = live_range(range);
    if (!r) return fail(XATTN_EINVAL, "xtensor_premap_wait: not a range");
    Pool* p = r->pool;
    std::unique_lock<std::mutex> lock(p->mu);
    p->cv_done.wait(lock, [&] { return r->async_pending == 0; });
    const int st = r->async_status;
    r->async_status = XATTN_OK;
    if (st != XATTN_OK) return fail(st, "xtensor_premap_wait: the pre-mapping request failed (status %d)", st);
    return XATTN_OK;
}

int xtensor_close(void* range, int keep_reusable) {
    PoolRange* r = live_range(range);
    if (!r || r->reusable) return fail(XATTN_EINVAL, "xtensor_close: not an open range");
    Pool* p = r->pool;
    std::unique_lock<std::mutex> lock(p->mu);
    p->cv_done.wait(lock, [&] { return r->async_pending == 0; });
    p->live.erase(r);
    if (keep_reusable && !r->pages.empty()) {
        r->reusable = true;
        for (int64_t id : r->pages) p->pages[(size_t)id].status = XTENSOR_PAGE_REUSABLE;
        p->reusable.push_back(r);
        return XATTN_OK;
    }
    const int st = drop_range(p, r);
    {
        std::lock_guard<std::mutex> l2(g_pools_mu);
        g_ranges.erase(r);
    }
    delete r;
    return st;
}

int xtensor_range_pages(void* range, int64_t* page_ids_out, int n) {
    PoolRange* r = live_range(range);
    if (!r) return fail(XATTN_EINVAL, "xtensor_range_pages: not a range");
    std::lock_guard<std::mutex> lock(r->pool->mu);
    const int count = (int)r->pages.size();
    if (count > 0 && (!page_ids_out || n < count))
        return fail(XATTN_EINVAL, "xtensor_range_pages: page_ids_out holds %d entries, %d needed", n, count);
    for (int i = 0; i < count; ++i) page_ids_out[i] = r->pages[(size_t)i];
    return count;
}

}  // extern "C"
