// Host test library only: the partition of xattn_plan.h (the same code the kernels run) behind C entry
// points, with the wave-parallel steps of the device front end (total, locate) replaced by plain loops.
#include <cstdint>

#include "../xattn_plan.h"

using namespace xattn;

namespace {

Plan plan_of(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew) {
    int64_t total = 0;
    for (int b = 0; b < batch; ++b) total += stream_len(kv_lens[b], seg_cost);
    if (total > INT32_MAX) total = -1;          // outside the documented limit: reported, not wrapped
    return plan_for_total((int)total, n_pieces, min_piece, seg_cost, xcd_skew);
}

}  // namespace

extern "C" {

// total_out: stream positions N (-1 when N would exceed 2^31 - 1); returns the number of pieces in use.
int xattn_test_plan(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int32_t* total_out) {
    const Plan pl = plan_of(kv_lens, batch, n_pieces, min_piece, seg_cost, xcd_skew);
    if (total_out) *total_out = pl.total;
    return pl.total < 0 ? -1 : pl.n_pieces;
}

// bounds_out[0 .. n_used]: piece_bound(p) for p = 0 .. n_used.
int xattn_test_piece_bounds(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew,
                            int32_t* bounds_out) {
    const Plan pl = plan_of(kv_lens, batch, n_pieces, min_piece, seg_cost, xcd_skew);
    if (pl.total < 0) return -1;
    for (int p = 0; p <= pl.n_pieces; ++p) bounds_out[p] = piece_bound(pl, p);
    return pl.n_pieces;
}

int xattn_test_piece_of(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int position) {
    const Plan pl = plan_of(kv_lens, batch, n_pieces, min_piece, seg_cost, xcd_skew);
    if (pl.total < 0 || position < 0 || position >= pl.total) return -1;
    return piece_of(pl, position);
}

// The segments of piece p as the kernels walk them: rows of (b, j0, j1, slot, whole) in segs_out
// (up to max_segs rows); returns their number.
int xattn_test_piece_segments(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int p,
                              int32_t* segs_out, int max_segs) {
    const Plan pl = plan_of(kv_lens, batch, n_pieces, min_piece, seg_cost, xcd_skew);
    if (pl.total < 0 || p < 0 || p >= pl.n_pieces) return -1;
    const int s0 = piece_bound(pl, p), s1 = piece_bound(pl, p + 1);
    // locate: the sequence that holds position s0 and the offset within its positions
    Walk w = {0, 0, s1 - s0};
    int before = 0;
    for (w.b = 0; w.b < batch; ++w.b) {
        const int v = stream_len(kv_lens[w.b], seg_cost);
        if (s0 < before + v) break;
        before += v;
    }
    w.j = s0 - before;
    int n = 0;
    PieceSeg ps;
    while (next_segment(w, batch, seg_cost, [&](int b) { return clamp_len(kv_lens[b]); }, ps)) {
        if (n < max_segs) {
            int32_t* row = segs_out + 5 * n;
            row[0] = ps.b; row[1] = ps.j0; row[2] = ps.j1; row[3] = p + ps.b; row[4] = ps.whole ? 1 : 0;
        }
        ++n;
    }
    return n;
}

// meta_out[2 b], meta_out[2 b + 1]: (first partial slot, number of segments) of sequence b.
int xattn_test_meta(const int32_t* kv_lens, int batch, int n_pieces, int min_piece, int seg_cost, int xcd_skew, int32_t* meta_out) {
    const Plan pl = plan_of(kv_lens, batch, n_pieces, min_piece, seg_cost, xcd_skew);
    if (pl.total < 0) return -1;
    int start = 0;
    for (int b = 0; b < batch; ++b) {
        const int len = clamp_len(kv_lens[b]);
        const SeqMeta m = seq_meta(pl, b, start, len);
        meta_out[2 * b] = m.first_slot;
        meta_out[2 * b + 1] = m.n_seg;
        start += stream_len(len, seg_cost);
    }
    return 0;
}

}  // extern "C"
