// The token-stream partition of the decode kernels (paper section 4.4.3, "Layer 3": balance compute
// units by token count, split long sequences, let short ones share a unit) as plain integer code that
// compiles for the device and for the host: the kernels use it through the wave-level front end in
// xattn_device.h, the CPU property tests through host_test/plan_shim.cpp.
//
// All keys of the batch form one stream that is cut into pieces of equal COST.  A sequence of L > 0
// tokens occupies L + seg_cost positions of the stream: its tokens, then seg_cost positions that stand
// for the fixed work every (piece, sequence) segment costs (first loads, Q, the stores of its result),
// so a workgroup whose piece spans a sequence boundary gets correspondingly fewer tokens.  A piece
// bound that falls into those extra positions means "the end of that sequence".  seg_cost = 0 gives
// pieces of equal token count.  Sequences without tokens occupy no positions.
//
// Limits: stream positions are 32-bit.  N = sum_b (L_b + seg_cost) must stay below 2^31, which the
// memory of one GPU guarantees for real caches (2^31 tokens of the smallest supported row, 256 bytes
// of K plus 256 of V, are 1 TiB); n_pieces <= 65536.
#ifndef XATTN_PLAN_H_
#define XATTN_PLAN_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define XATTN_HD __host__ __device__ __forceinline__
#else
#define XATTN_HD inline
#endif

namespace xattn {

constexpr int kPlanRound = 16;        // piece bounds are multiples of the 16-key block (except the last)
constexpr int kMaxPieces = 65536;

struct Plan {
    int total;      // N: positions of the whole stream
    int n_pieces;   // pieces in use: min(launched pieces, N / minimum piece size), at least 1
    int seg_cost;
    int xcd_skew;   // per mille; see piece_bound
};
constexpr int kMaxXcdSkew = 200;
constexpr int kMinSkewPiece = 32 * kPlanRound;      // positions per piece from which the XCD skew applies

XATTN_HD int clamp_len(int v) { return v > 0 ? v : 0; }
// Stream positions of a sequence of `len` tokens (any sign).
XATTN_HD int stream_len(int len, int seg_cost) { return len > 0 ? len + seg_cost : 0; }

XATTN_HD Plan plan_for_total(int total, int n_pieces, int min_piece, int seg_cost, int xcd_skew = 0) {
    int n = total / (min_piece > 0 ? min_piece : 1);
    n = n < 1 ? 1 : n;
    Plan pl;
    pl.total = total;
    pl.n_pieces = n < n_pieces ? n : n_pieces;
    pl.seg_cost = seg_cost;
    // the skew needs the eight XCD parts to hold the same number of pieces, and pieces long enough for a
    // few per cent of them to be a block or more
    const bool can_skew = xcd_skew > 0 && pl.n_pieces % 8 == 0 && total / pl.n_pieces >= kMinSkewPiece;
    pl.xcd_skew = can_skew ? (xcd_skew < kMaxXcdSkew ? xcd_skew : kMaxXcdSkew) : 0;
    return pl;
}

// floor(i * span / m) in 32-bit arithmetic: i * (span / m) + i * (span % m) / m, with i <= m <= 65536
// so that i * (span % m) < m^2 <= 2^32.
XATTN_HD uint32_t scaled_index(uint32_t i, uint32_t span, uint32_t m) { return i * (span / m) + i * (span % m) / m; }

// The chip's eight XCDs do not stream at the same rate: measured on MI355X, the odd-numbered ones
// take about 7 % longer than the even-numbered ones for the same bytes, whatever data they are given.
// The kernels hand XCD x the pieces x * n / 8 .. (x + 1) * n / 8 - 1 (consecutive workgroup ids go to
// consecutive XCDs), so the stream is first cut into eight XCD parts, part x starting at
// N * (x + (x odd ? skew : 0)) / 8 (skew = xcd_skew / 1000: even parts are longer by that fraction, odd
// parts shorter), and every part into n / 8 equal pieces.  xcd_skew = 0: eight equal parts.
XATTN_HD uint32_t xcd_part_start(const Plan& pl, int x) {
    // 32-bit arithmetic: N * x / 8 and N * skew / 8000, each as quotient part plus remainder part
    const uint32_t t = (uint32_t)pl.total, ux = (uint32_t)x, sk = (uint32_t)pl.xcd_skew;
    const uint32_t even = (t / 8u) * ux + (t % 8u) * ux / 8u;
    return (x & 1) ? even + (t / 8000u) * sk + (t % 8000u) * sk / 8000u : even;
}

// Piece p owns stream positions [piece_bound(p), piece_bound(p + 1)): floor(p * N / n_pieces) (or its
// skewed counterpart) rounded to the nearest multiple of the 16-key block, so every piece is within
// 16 positions of its exact share and all are used.
XATTN_HD int piece_bound(const Plan& pl, int p) {
    if (p >= pl.n_pieces) return pl.total;
    uint32_t x;
    if (pl.xcd_skew == 0) {
        x = scaled_index((uint32_t)p, (uint32_t)pl.total, (uint32_t)pl.n_pieces);
    } else {
        const uint32_t m = (uint32_t)pl.n_pieces / 8u, part = (uint32_t)p / m;
        const uint32_t a = xcd_part_start(pl, (int)part), b = xcd_part_start(pl, (int)part + 1);
        x = a + scaled_index((uint32_t)p - part * m, b - a, m);
    }
    const uint32_t rounded = (x + kPlanRound / 2) / kPlanRound * kPlanRound;
    return rounded < (uint32_t)pl.total ? (int)rounded : pl.total;
}

// The piece that owns stream position x (0 <= x < N): an estimate, corrected against piece_bound.
XATTN_HD int piece_of(const Plan& pl, int x) {
    int p;
    if (pl.xcd_skew == 0) {
        p = (int)((float)x * (float)pl.n_pieces / (float)pl.total);
    } else {
        const int m = pl.n_pieces / 8;
        int part = 0;
        while (part < 7 && xcd_part_start(pl, part + 1) <= (uint32_t)x) ++part;
        const uint32_t a = xcd_part_start(pl, part), b = xcd_part_start(pl, part + 1);
        p = part * m + (int)((float)((uint32_t)x - a) * (float)m / (float)(b - a));
    }
    p = p < 0 ? 0 : (p > pl.n_pieces - 1 ? pl.n_pieces - 1 : p);
    while (p + 1 < pl.n_pieces && piece_bound(pl, p + 1) <= x) ++p;
    while (p > 0 && piece_bound(pl, p) > x) --p;
    return p;
}

// What the merge kernel needs to know of a sequence that starts at stream position `start` and has
// `len` tokens: its first partial-result slot and its number of (piece, sequence) segments, i.e. the
// pieces from the one with its first token to the one with its last.  Slot of a segment = piece +
// sequence index (unique: piece and sequence index never both stand still between two segments).
struct SeqMeta { int first_slot, n_seg; };
XATTN_HD SeqMeta seq_meta(const Plan& pl, int b, int start, int len) {
    SeqMeta m;
    if (len <= 0) { m.first_slot = b; m.n_seg = 0; return m; }
    const int first = piece_of(pl, start);
    m.first_slot = first + b;
    m.n_seg = piece_of(pl, start + len - 1) - first + 1;
    return m;
}

// A piece's walk over the sequences it intersects, in stream order.
struct Walk {
    int b;            // next sequence to look at
    int j;            // offset into that sequence's L + seg_cost positions
    int remaining;    // stream positions left in the piece
};
struct PieceSeg {
    int b, L;         // sequence and its length
    int j0, j1;       // tokens [j0, j1) of it
    bool whole;       // the segment is the whole sequence: no partial result, no merge
};
// len_of(b) returns clamp_len(kv_lens[b]).  Returns false when the piece is exhausted.
template <typename LenFn>
XATTN_HD bool next_segment(Walk& w, int batch, int seg_cost, LenFn len_of, PieceSeg& out) {
    while (w.remaining > 0 && w.b < batch) {
        const int L = len_of(w.b);
        if (L == 0) { ++w.b; continue; }
        // the piece's share of this sequence's L + seg_cost positions, and the tokens among them
        const int left = L + seg_cost - w.j;
        const int n_pos = left < w.remaining ? left : w.remaining;
        const int j0 = w.j < L ? w.j : L, j1 = w.j + n_pos < L ? w.j + n_pos : L;
        w.remaining -= n_pos;
        const int bb = w.b;
        ++w.b;
        w.j = 0;
        if (j1 <= j0) continue;                    // only the sequence's extra positions: no tokens
        out.b = bb;
        out.L = L;
        out.j0 = j0;
        out.j1 = j1;
        out.whole = (j0 == 0 && j1 == L);
        return true;
    }
    return false;
}

}  // namespace xattn
#endif
