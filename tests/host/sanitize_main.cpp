// Host-code exerciser for sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer, and
// ThreadSanitizer): links the page pool on its host-only stand-in driver, the beam-search selection,
// the partition arithmetic, the CPU oracle and the input generator into one executable and drives
// them through their C entry points, several threads at once where the code has threads and locks.
// It checks results only coarsely (the pytest suites do that); its job is to reach the code paths --
// roll-backs after injected driver failures, lazy release, page reuse, the background pre-mapping
// thread racing with grow / close -- so that the sanitizers see them.  Exit code 0 = nothing found.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "../../include/xattn.h"
#include "../../include/xbeam.h"
#include "../../paper_2510_14686_amd/csrc/host_test/xtensor_test_hooks.h"

extern "C" {
// oracle/oracle_attn.c, workloads/gen.c, csrc/host_test/plan_shim.cpp
int oracle_attn(const uint16_t* q, const uint16_t* const* k_ptrs, const uint16_t* const* v_ptrs, const int32_t* kv_lens,
                int batch, int q_len, int n_q_heads, int n_kv_heads, int head_dim, float scale, double* out, double* lse);
int oracle_merge(const double* out_parts, const double* lse_parts, int n_parts, long rows, int head_dim, double* out, double* lse);
int oracle_write_kvcache(const uint16_t* k_new, const uint16_t* v_new, uint16_t* const* k_ptrs, uint16_t* const* v_ptrs,
                         const int32_t* kv_lens, int batch, int q_len, int row_elems);
int oracle_mla(const uint16_t* q, const uint16_t* const* c_ptrs, const int32_t* kv_lens, int batch, int q_len, int n_heads,
               int d_qk, int d_v, float scale, double* out, double* lse);
void oracle_page_of(uint64_t va, uint64_t va_start, uint64_t page_size, uint64_t* page_idx, uint64_t* offset);
void wl_normal_bf16(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, uint16_t* out);
void wl_uniform_u64(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, uint64_t* out);
int xattn_test_plan(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int32_t* total_out);
int xattn_test_piece_bounds(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int32_t* bounds_out);
int xattn_test_piece_segments(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int p,
                              int32_t* segs_out, int max_segs);
int xattn_test_meta(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int32_t* meta_out);
}

static int g_failures = 0;
#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            std::fprintf(stderr, "CHECK failed at line %d: %s (%s)\n", __LINE__, #cond, xattn_last_error()); \
            ++g_failures;                                                            \
        }                                                                            \
    } while (0)

static const size_t kPage = XTENSOR_CHUNK_BYTES;

static void fake_counts(size_t* r, size_t* h, size_t* m) { CHECK(xtensor_test_fake_counts(r, h, m) == 0); }

// One request's life on a shared pool: open, grow on demand, pre-map ahead, close (kept or not).
static void request_loop(void* pool, int id, int rounds) {
    for (int i = 0; i < rounds; ++i) {
        void *base = nullptr, *rng = nullptr;
        int reused = 0;
        const size_t pages0 = 1 + (size_t)((id + i) % 3);
        int st = xtensor_open(pool, (uint64_t)(100 * id + i), 16 * kPage, pages0 * kPage, &base, &rng, &reused);
        if (st == XATTN_ENOMEM) continue;              // the pool is shared: running dry is a legal outcome
        CHECK(st == XATTN_OK && base && rng);
        if (st != XATTN_OK) continue;
        for (size_t want = pages0 + 1; want <= pages0 + 4; ++want) {
            if ((want + (size_t)id) % 2) {
                CHECK(xtensor_premap_async(rng, want * kPage) == XATTN_OK);
                if (want % 3 == 0) (void)xtensor_premap_wait(rng);       // may report ENOMEM of the request
            } else {
                st = xtensor_grow(rng, want * kPage);
                CHECK(st >= 0 || st == XATTN_ENOMEM);
            }
        }
        int64_t ids[32];
        const int n = xtensor_range_pages(rng, ids, 32);
        CHECK(n >= (int)pages0 && n <= 16);
        CHECK(xtensor_close(rng, (i + id) % 2) == XATTN_OK);
    }
}

static void pool_scenarios() {
    size_t r0, h0, m0;
    fake_counts(&r0, &h0, &m0);
    // bookkeeping, reuse, lazy release
    void* pool = nullptr;
    CHECK(xtensor_pool_create(0, 24, 7, &pool) == XATTN_OK);
    size_t counts[4];
    CHECK(xtensor_pool_counts(pool, counts) == XATTN_OK && counts[XTENSOR_PAGE_FREE] == 24);
    void *base = nullptr, *a = nullptr, *b = nullptr;
    int reused = 0;
    CHECK(xtensor_open(pool, 1, 8 * kPage, 3 * kPage, &base, &a, &reused) == XATTN_OK && !reused);
    CHECK(xtensor_grow(a, 5 * kPage) == 2);
    CHECK(xtensor_grow(a, 9 * kPage) == XATTN_EINVAL);                     // beyond the reserved range
    CHECK(xtensor_close(a, 1) == XATTN_OK);
    CHECK(xtensor_open(pool, 2, 8 * kPage, 5 * kPage, &base, &b, &reused) == XATTN_OK && reused);
    CHECK(xtensor_close(b, 1) == XATTN_OK);
    void* big = nullptr;
    CHECK(xtensor_open(pool, 3, 24 * kPage, 24 * kPage, &base, &big, &reused) == XATTN_OK);   // forces the lazy release
    CHECK(xtensor_pool_destroy(pool) == XATTN_EINVAL);                     // a range is still open
    void* none = nullptr;
    CHECK(xtensor_open(pool, 4, 2 * kPage, kPage, &base, &none, &reused) == XATTN_ENOMEM);
    CHECK(xtensor_close(big, 0) == XATTN_OK);
    CHECK(xtensor_close(big, 0) == XATTN_EINVAL);                          // closed handles are refused
    // injected driver failures: map inside open, map inside grow, reserve, create
    CHECK(xtensor_test_fail_next(5, 1) == 0);
    CHECK(xtensor_open(pool, 5, 8 * kPage, 4 * kPage, &base, &a, &reused) == XATTN_EHIP);
    CHECK(xtensor_open(pool, 5, 8 * kPage, 2 * kPage, &base, &a, &reused) == XATTN_OK);
    CHECK(xtensor_test_fail_next(5, 1) == 0);
    CHECK(xtensor_grow(a, 6 * kPage) == XATTN_EHIP);
    CHECK(xtensor_range_pages(a, nullptr, 0) == XATTN_EINVAL);
    CHECK(xtensor_close(a, 0) == XATTN_OK);
    CHECK(xtensor_test_fail_next(1, 0) == 0);
    CHECK(xtensor_open(pool, 6, 8 * kPage, kPage, &base, &a, &reused) == XATTN_ENOMEM);
    CHECK(xtensor_test_fail_next(6, 0) == 0);
    CHECK(xtensor_open(pool, 7, 8 * kPage, 2 * kPage, &base, &a, &reused) == XATTN_OK);
    CHECK(xtensor_close(a, 0) == XATTN_EHIP);                              // unmap refused once: reported, bookkeeping stays sound
    CHECK(xtensor_pool_destroy(pool) == XATTN_OK);
    CHECK(xtensor_test_fail_next(3, 5) == 0);
    CHECK(xtensor_pool_create(0, 16, 1, &pool) == XATTN_ENOMEM);          // the sixth page cannot be created
    CHECK(xtensor_test_fail_next(-1, 0) == 0);
    size_t r1, h1, m1;
    fake_counts(&r1, &h1, &m1);
    CHECK(r1 == r0 && h1 == h0);                                           // nothing leaked (one mapping was refused its unmap)

    // several requests at once on one pool, with the background pre-mapping thread in the middle
    CHECK(xtensor_pool_create(0, 40, 3, &pool) == XATTN_OK);
    std::vector<std::thread> threads;
    for (int t = 0; t < 6; ++t) threads.emplace_back(request_loop, pool, t, 40);
    for (auto& t : threads) t.join();
    CHECK(xtensor_pool_counts(pool, counts) == XATTN_OK);
    CHECK(counts[XTENSOR_PAGE_FREE] + counts[XTENSOR_PAGE_REUSABLE] == 40 && counts[XTENSOR_PAGE_MAPPED] == 0);
    CHECK(xtensor_pool_destroy(pool) == XATTN_OK);
    size_t r2, h2, m2;
    fake_counts(&r2, &h2, &m2);
    CHECK(r2 == r1 && h2 == h1 && m2 == m1);
}

static void beam_scenarios_once() {
    for (int cfg = 0; cfg < 3; ++cfg) {
        const int R = 3, W = cfg == 0 ? 1 : cfg == 1 ? 8 : 33, K = cfg == 0 ? 5 : cfg == 1 ? 8 : 70;
        std::vector<uint64_t> u((size_t)R * W * K + (size_t)R * W);
        wl_uniform_u64(11 + cfg, 0, 0, u.size(), u.data());
        std::vector<float> beam((size_t)R * W), cand((size_t)R * W * K);
        std::vector<int32_t> tok((size_t)R * W * K);
        for (size_t i = 0; i < beam.size(); ++i) beam[i] = -2.0f - (float)(u[i] % 1000) / 100.0f;
        for (int rw = 0; rw < R * W; ++rw) {
            float v = -0.1f;
            for (int k = 0; k < K; ++k) {
                v -= (float)(u[beam.size() + (size_t)rw * K + k] % 4) / 4.0f;      // descending, with ties
                cand[(size_t)rw * K + k] = v;
                tok[(size_t)rw * K + k] = (int32_t)(u[beam.size() + (size_t)rw * K + k] % 50000);
            }
        }
        std::vector<float> lp_a((size_t)R * W), lp_b((size_t)R * W);
        std::vector<int32_t> par_a((size_t)R * W), par_b((size_t)R * W), tok_a((size_t)R * W), tok_b((size_t)R * W);
        std::vector<int64_t> visited(R);
        CHECK(xbeam_select(beam.data(), cand.data(), tok.data(), R, W, K, XBEAM_CHECK_INPUT, lp_a.data(), par_a.data(),
                           tok_a.data(), visited.data()) == XATTN_OK);
        CHECK(xbeam_select(beam.data(), cand.data(), nullptr, R, W, K, XBEAM_FULL_SORT, lp_b.data(), par_b.data(), tok_b.data(),
                           nullptr) == XATTN_OK);
        for (size_t i = 0; i < lp_a.size(); ++i) CHECK(lp_a[i] == lp_b[i] && par_a[i] == par_b[i]);
        cand[1] = cand[0] + 1.0f;                                          // ascending step: rejected when checked
        CHECK(xbeam_select(beam.data(), cand.data(), tok.data(), R, W, K > 1 ? K : 2, XBEAM_CHECK_INPUT, lp_a.data(),
                           par_a.data(), tok_a.data(), nullptr) == XATTN_EINVAL || K == 1);
        CHECK(xbeam_select(nullptr, cand.data(), tok.data(), R, W, K, 0, lp_a.data(), par_a.data(), tok_a.data(), nullptr) ==
              XATTN_EINVAL);
    }
}

static void beam_scenarios() {
    beam_scenarios_once();
    std::thread t1(beam_scenarios_once), t2(beam_scenarios_once);       // the heap storage is per thread
    t1.join();
    t2.join();
}

static void plan_scenarios() {
    std::vector<uint64_t> u(4096);
    wl_uniform_u64(21, 0, 0, u.size(), u.data());
    const int batches[] = {1, 7, 64, 65, 1000, 4096};
    for (int batch : batches) {
        std::vector<int32_t> lens(batch);
        for (int b = 0; b < batch; ++b) lens[b] = (int32_t)(u[b] % 3 == 0 ? 0 : u[b] % (batch > 64 ? 300 : 9000));
        const int pieces_list[] = {1, 8, 256, 1000};
        for (int pieces : pieces_list) {
            for (int skew : {0, 32, 200}) {
                int32_t total = 0;
                const int used = xattn_test_plan(lens.data(), batch, pieces, 16, 16, skew, &total);
                CHECK(used >= 1 && used <= pieces);
                std::vector<int32_t> bounds(pieces + 2), meta(2 * (size_t)batch), segs(5 * 4200);
                CHECK(xattn_test_piece_bounds(lens.data(), batch, pieces, 16, 16, skew, bounds.data()) == used);
                CHECK(bounds[0] == 0 && bounds[used] == total);
                CHECK(xattn_test_meta(lens.data(), batch, pieces, 16, 16, skew, meta.data()) == 0);
                long tokens = 0, want = 0;
                for (int b = 0; b < batch; ++b) want += lens[b] > 0 ? lens[b] : 0;
                for (int p = 0; p < used; ++p) {
                    const int n = xattn_test_piece_segments(lens.data(), batch, pieces, 16, 16, skew, p, segs.data(), 4200);
                    CHECK(n >= 0 && n <= 4200);
                    for (int i = 0; i < n && i < 4200; ++i) tokens += segs[5 * i + 2] - segs[5 * i + 1];
                }
                CHECK(tokens == want);
            }
        }
    }
}

static void oracle_scenarios() {
    const int B = 3, T = 2, Hq = 4, Hkv = 2, D = 16;
    const int32_t lens[B] = {2, 9, 40};
    std::vector<uint16_t> q((size_t)B * T * Hq * D);
    wl_normal_bf16(5, 0, 0, q.size(), q.data());
    std::vector<std::vector<uint16_t>> ks(B), vs(B);
    const uint16_t *kp[B], *vp[B];
    uint16_t *kw[B], *vw[B];
    for (int b = 0; b < B; ++b) {
        ks[b].resize((size_t)lens[b] * Hkv * D);
        vs[b].resize((size_t)lens[b] * Hkv * D);
        wl_normal_bf16(5, 1 + 2 * b, 0, ks[b].size(), ks[b].data());
        wl_normal_bf16(5, 2 + 2 * b, 0, vs[b].size(), vs[b].data());
        kp[b] = kw[b] = ks[b].data();
        vp[b] = vw[b] = vs[b].data();
    }
    std::vector<double> out((size_t)B * T * Hq * D), lse((size_t)B * T * Hq);
    CHECK(oracle_attn(q.data(), kp, vp, lens, B, T, Hq, Hkv, D, 0.25f, out.data(), lse.data()) == 0);
    for (double x : out) CHECK(std::isfinite(x));
    CHECK(oracle_attn(q.data(), kp, vp, lens, B, 3, Hq, Hkv, D, 0.25f, out.data(), nullptr) == -1);    // kv_len < q_len
    // the aggregation of a row with itself leaves it unchanged and adds ln 2 to its lse
    std::vector<double> parts(2 * out.size()), lparts(2 * lse.size()), mo(out.size()), ml(lse.size());
    for (size_t i = 0; i < out.size(); ++i) parts[i] = parts[out.size() + i] = out[i];
    for (size_t i = 0; i < lse.size(); ++i) lparts[i] = lparts[lse.size() + i] = lse[i];
    CHECK(oracle_merge(parts.data(), lparts.data(), 2, (long)lse.size(), D, mo.data(), ml.data()) == 0);
    for (size_t i = 0; i < lse.size(); ++i) CHECK(std::fabs(ml[i] - lse[i] - std::log(2.0)) < 1e-12);
    std::vector<uint16_t> k_new((size_t)B * T * Hkv * D, 0x3f80), v_new((size_t)B * T * Hkv * D, 0x4000);
    CHECK(oracle_write_kvcache(k_new.data(), v_new.data(), kw, vw, lens, B, T, Hkv * D) == 0);
    CHECK(ks[2][(size_t)(lens[2] - 1) * Hkv * D] == 0x3f80 && vs[0][0] == 0x4000);
    // latent-KV rows: key width 24, value width 16
    std::vector<uint16_t> q2((size_t)B * T * Hq * 24);
    wl_normal_bf16(6, 0, 0, q2.size(), q2.data());
    std::vector<std::vector<uint16_t>> cs(B);
    const uint16_t* cp[B];
    for (int b = 0; b < B; ++b) {
        cs[b].resize((size_t)lens[b] * 24);
        wl_normal_bf16(6, 1 + b, 0, cs[b].size(), cs[b].data());
        cp[b] = cs[b].data();
    }
    std::vector<double> out2((size_t)B * T * Hq * 16), lse2((size_t)B * T * Hq);
    CHECK(oracle_mla(q2.data(), cp, lens, B, T, Hq, 24, 16, 0.2f, out2.data(), lse2.data()) == 0);
    uint64_t page = 0, off = 0;
    oracle_page_of(0x7000 + 5 * 4096 + 17, 0x7000, 4096, &page, &off);
    CHECK(page == 5 && off == 17);
}

int main() {
    pool_scenarios();
    beam_scenarios();
    plan_scenarios();
    oracle_scenarios();
    if (g_failures) {
        std::fprintf(stderr, "%d check(s) failed\n", g_failures);
        return 1;
    }
    std::puts("host sanitizer exerciser: all scenarios ran");
    return 0;
}
