// Host-side beam-search selection (section 4.5.1, "Beam Search Optimization"): partial selection with a
// bounded min-heap and an early exit per sequence that relies on descending candidate log-probabilities.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/xattn.h"
#include "../../include/xbeam.h"
#include "xattn_internal.h"

namespace {

struct Cand {
    float score;
    int32_t w, k;
};

// a is worse than b in the order "score descending, then w, then k ascending"
inline bool worse(const Cand& a, const Cand& b) {
    if (a.score != b.score) return a.score < b.score;
    if (a.w != b.w) return a.w > b.w;
    return a.k > b.k;
}

// Min-heap on `worse`: heap[0] is the worst entry.
inline void sift_down(Cand* heap, int n, int i) {
    const Cand x = heap[i];
    for (;;) {
        int c = 2 * i + 1;
        if (c >= n) break;
        if (c + 1 < n && worse(heap[c + 1], heap[c])) ++c;
        if (!worse(heap[c], x)) break;
        heap[i] = heap[c];
        i = c;
    }
    heap[i] = x;
}
inline void sift_up(Cand* heap, int i) {
    const Cand x = heap[i];
    while (i > 0) {
        const int p = (i - 1) / 2;
        if (!worse(x, heap[p])) break;
        heap[i] = heap[p];
        i = p;
    }
    heap[i] = x;
}

thread_local std::vector<Cand> t_heap;      // reused across calls: no allocation in steady state

}  // namespace

extern "C" int xbeam_select(const float* beam_lp, const float* cand_lp, const int32_t* cand_tok, int n_req,
                            int beam_width, int top_k, int flags, float* out_lp, int32_t* out_parent,
                            int32_t* out_tok, int64_t* visited) {
    using xattn::fail;
    if (n_req < 0 || beam_width < 1 || beam_width > 65536 || top_k < 1 || top_k > 65536)
        return fail(XATTN_EINVAL, "xbeam_select: n_req %d, beam_width %d, top_k %d out of range", n_req, beam_width, top_k);
    if (n_req > 0 && (!beam_lp || !cand_lp || !out_lp || !out_parent || !out_tok))
        return fail(XATTN_EINVAL, "xbeam_select: beam_lp, cand_lp and the three outputs must not be NULL");
    if (flags & ~(XBEAM_FULL_SORT | XBEAM_CHECK_INPUT)) return fail(XATTN_EINVAL, "xbeam_select: unknown flags %d", flags);
    const int W = beam_width, K = top_k;
    const size_t need = (flags & XBEAM_FULL_SORT) ? (size_t)W * K : (size_t)W;
    if (t_heap.size() < need) t_heap.resize(need);
    Cand* heap = t_heap.data();
    for (int r = 0; r < n_req; ++r) {
        const float* blp = beam_lp + (size_t)r * W;
        const float* clp = cand_lp + (size_t)r * W * K;
        const int32_t* ctk = cand_tok ? cand_tok + (size_t)r * W * K : nullptr;
        if (flags & XBEAM_CHECK_INPUT) {
            for (int w = 0; w < W; ++w) {
                if (std::isnan(blp[w])) return fail(XATTN_EINVAL, "xbeam_select: beam_lp[%d][%d] is NaN", r, w);
                for (int k = 0; k < K; ++k) {
                    const float v = clp[(size_t)w * K + k];
                    if (std::isnan(v) || (k > 0 && v > clp[(size_t)w * K + k - 1]))
                        return fail(XATTN_EINVAL, "xbeam_select: cand_lp[%d][%d][%d] is NaN or breaks the descending order", r, w, k);
                }
            }
        }
        int64_t seen = 0;
        int n = 0;
        if (flags & XBEAM_FULL_SORT) {
            for (int w = 0; w < W; ++w)
                for (int k = 0; k < K; ++k) heap[n++] = Cand{blp[w] + clp[(size_t)w * K + k], w, k};
            seen = n;
            std::sort(heap, heap + n, [](const Cand& a, const Cand& b) { return worse(b, a); });
            for (int i = 0; i < W; ++i) {
                out_lp[(size_t)r * W + i] = heap[i].score;
                out_parent[(size_t)r * W + i] = heap[i].w;
                out_tok[(size_t)r * W + i] = ctk ? ctk[(size_t)heap[i].w * K + heap[i].k] : heap[i].k;
            }
        } else {
            for (int w = 0; w < W; ++w) {
                const float base = blp[w];
                const float* row = clp + (size_t)w * K;
                for (int k = 0; k < K; ++k) {
                    const Cand c{base + row[k], w, k};
                    ++seen;
                    if (n < W) {
                        heap[n] = c;
                        sift_up(heap, n++);
                    } else if (worse(heap[0], c)) {
                        heap[0] = c;
                        sift_down(heap, n, 0);
                    } else {
                        break;      // the later candidates of this sequence score no higher and come later in the order
                    }
                }
            }
            // n == W here (W * K >= W candidates, and the heap only refuses when full)
            for (int i = W - 1; i >= 0; --i) {
                const Cand c = heap[0];
                heap[0] = heap[--n];
                if (n > 0) sift_down(heap, n, 0);
                out_lp[(size_t)r * W + i] = c.score;
                out_parent[(size_t)r * W + i] = c.w;
                out_tok[(size_t)r * W + i] = ctk ? ctk[(size_t)c.w * K + c.k] : c.k;
            }
        }
        if (visited) visited[r] = seen;
    }
    return XATTN_OK;
}
