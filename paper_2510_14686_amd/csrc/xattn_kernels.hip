// Split-KV decode attention and its log-sum-exp merge for gfx950 (MI355X).
//
// Work decomposition (paper section 4.4.3, "Layer 3": balance compute units by token count, split
// long sequences, let short ones share a unit).  The keys of the whole batch form one stream of
// N = sum_b kv_lens[b] tokens, cut into P pieces of N / P tokens (to within one 16-key block);
// workgroup p owns one piece of that stream, whatever sequences it falls in.  Inside a workgroup wave w owns
// KV head w, so a workgroup streams one contiguous byte range of K and one of V (no block table:
// section 4.3, "Operator Adaptation").  Each (piece, sequence) intersection is a segment.  A segment
// that covers its whole sequence writes the final result; any other writes an un-normalised partial
// (o, m, l) to slot piece + sequence_index, and the merge kernel combines a sequence's slots (the
// aggregation step of section 4.4.3, "Layer 2").  Combining inside the decode kernel by the last wave
// to finish a sequence was tried and is slower: that wave alone reads all of a long sequence's
// partials with dependent device-scope loads, while the merge kernel spreads them over the chip.
//
// Loads: 16 lanes hold one 256-byte K (or V) row, 8 bf16 each, one 128-bit non-temporal buffer load
// per lane, so a wave load covers four rows; the buffer descriptor's size is the sequence's byte
// length, so a ragged last block reads zeros instead of memory past the sequence (which an xTensor
// range may not have mapped).  All query rows that share the KV head (GQA group x new tokens:
// section 4.4.1, K is loaded once for all of them and Q stays in registers) use the row from
// registers.  Two inner loops:
//   * vector path (up to 8 rows): q.k by bf16 dot2 into fp32, reduced over the 16 lanes with DPP;
//     online softmax in fp32 (log2 domain); p.v by fp32 FMA.
//   * matrix path (tiles of 16 rows, the multi-token verification case): the K block is transposed
//     through wave-private LDS into the MFMA operand layout, S^T = K Q^T by bf16 MFMA 16x16x32;
//     softmax on the accumulator layout (a lane holds 4 keys of one row); O^T += V^T P^T by bf16 MFMA
//     16x16x16 straight from the V registers (V never touches LDS), with p fed as hi + lo bf16 parts
//     so that it keeps 16 significant bits.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xattn_device.h"
#include "xattn_kernels.h"

namespace xattn {
namespace {

// One (piece, sequence) intersection as seen by one wave.
struct Segment {
    int b, L;            // sequence and its length
    int j0, j1;          // keys [j0, j1) of the sequence
    const void* kp;      // the sequence's K and V ranges
    const void* vp;
    int slot;            // partial-result slot (piece + sequence index)
    bool whole;          // the segment is the whole sequence: write the final result
    int kvh;             // this wave's KV head
    int row0, n_rows;    // query rows [row0, row0 + n_rows) of the head's group * q_len rows
};

// Sequence length in bytes for the buffer descriptor (sequences of 4 GiB or more are not supported).
__device__ __forceinline__ uint32_t seq_bytes(const DecodeParams& prm, int L) {
    const unsigned long long b = (unsigned long long)L * (unsigned)prm.n_kv_heads * kRowBytes;
    return b > 0xffffffffull ? 0xffffffffu : (uint32_t)b;
}

// ---------------------------------------------------------------------------------- vector path
template <int R>
struct RowState {
    float m[R];        // running max of the scaled scores, log2 domain
    float l[R];        // running sum of exp2(s - m)
    float o[R][8];     // running sum of exp2(s - m) * v, this lane's 8 of the 128 columns
};

struct KvBlock {
    u32x4_t k[kU];
    u32x4_t v[kU];
};

// Key rows j_first + 4u + (lane / 16), u = 0..3; soffset carries the wave-uniform part.
__device__ __forceinline__ void load_block(KvBlock& blk, __amdgpu_buffer_rsrc_t rk, __amdgpu_buffer_rsrc_t rv,
                                           uint32_t voffset, uint32_t row_stride, int j_first) {
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        const uint32_t so = (uint32_t)(j_first + 4 * u) * row_stride;
        blk.k[u] = load_b128_nt(rk, voffset, so);
        blk.v[u] = load_b128_nt(rv, voffset, so);
    }
}

// One block of kU key rows per 16-lane group against R query rows.
// j_sub: absolute key index of this lane's row for u = 0 (rows u are 4 apart).  lim_of(r): first key
// index row r may NOT see (segment end and causal limit); used only when kMasked.
template <int R, bool kMasked, typename LimFn>
__device__ __forceinline__ void compute_block(RowState<R>& st, const KvBlock& blk, const uint32_t (&q)[R][4],
                                              float scale_log2, int j_sub, LimFn lim_of) {
    float s[R][kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        const uint32_t k0 = blk.k[u].x, k1 = blk.k[u].y, k2 = blk.k[u].z, k3 = blk.k[u].w;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float acc = dot2_bf16(q[r][0], k0, 0.0f);
            acc = dot2_bf16(q[r][1], k1, acc);
            acc = dot2_bf16(q[r][2], k2, acc);
            acc = dot2_bf16(q[r][3], k3, acc);
            acc = row16_sum(acc) * scale_log2;
            if (kMasked) acc = (j_sub + 4 * u < lim_of(r)) ? acc : kNegInf;
            s[r][u] = acc;
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float mb = s[r][0];
#pragma unroll
        for (int u = 1; u < kU; ++u) mb = fmaxf(mb, s[r][u]);
        const float m_new = fmaxf(st.m[r], mb);
        // While a row has seen no key yet its max is -inf: subtract 0 instead so that exp2 sees
        // -inf (-> 0), not -inf - -inf.
        const float m_use = (kMasked && m_new == kNegInf) ? 0.0f : m_new;
        const float alpha = fast_exp2(st.m[r] - m_use);
        float sum = 0.0f;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            s[r][u] = fast_exp2(s[r][u] - m_use);
            sum += s[r][u];
        }
        st.l[r] = st.l[r] * alpha + sum;
        st.m[r] = m_new;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[r][e] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        float v[8];
        v[0] = bf16_lo(blk.v[u].x); v[1] = bf16_hi(blk.v[u].x);
        v[2] = bf16_lo(blk.v[u].y); v[3] = bf16_hi(blk.v[u].y);
        v[4] = bf16_lo(blk.v[u].z); v[5] = bf16_hi(blk.v[u].z);
        v[6] = bf16_lo(blk.v[u].w); v[7] = bf16_hi(blk.v[u].w);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) st.o[r][e] = __builtin_fmaf(s[r][u], v[e], st.o[r][e]);
    }
}

// Rows r >= seg.n_rows are padding: they repeat the tile's first row and are never stored.
template <int R>
__device__ __forceinline__ void vector_segment(const DecodeParams& prm, const Segment& seg, int lane) {
    const int sub = lane >> 4, ds = lane & 15;
    const int G = prm.group, T = prm.q_len, Hq = prm.n_q_heads;
    const uint32_t row_stride = (uint32_t)prm.n_kv_heads * kRowBytes;
    const __amdgpu_buffer_rsrc_t rk = make_rsrc(seg.kp, seq_bytes(prm, seg.L));
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(seg.vp, seq_bytes(prm, seg.L));
    const uint32_t voffset = (uint32_t)sub * row_stride + (uint32_t)seg.kvh * kRowBytes + ds * 16;

    // Q rows of this KV head: row r <-> (token t = r / G, head kvh*G + r % G); lane takes columns ds*8..+8.
    auto row_token = [&](int r) { return (seg.row0 + (r < seg.n_rows ? r : 0)) / G; };
    auto row_index = [&](int r) {      // row of [batch*T*Hq]
        const int rr = seg.row0 + (r < seg.n_rows ? r : 0);
        const int t = rr / G;
        return (seg.b * T + t) * Hq + seg.kvh * G + (rr - t * G);
    };
    auto lim_of = [&](int r) {
        const int causal = seg.L - T + row_token(r) + 1;
        return causal < seg.j1 ? causal : seg.j1;
    };
    uint32_t q[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint4 qv = *reinterpret_cast<const uint4*>(prm.q + (long)row_index(r) * kHeadDim + ds * 8);
        q[r][0] = qv.x; q[r][1] = qv.y; q[r][2] = qv.z; q[r][3] = qv.w;
    }
    // token 0 of the tile has the tightest causal limit
    const int causal0 = seg.L - T + seg.row0 / G + 1;
    const int min_lim = causal0 < seg.j1 ? causal0 : seg.j1;

    RowState<R> st;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        st.m[r] = kNegInf;
        st.l[r] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[r][e] = 0.0f;
    }

    // Full blocks: every key visible to every row.  Two register buffers, the next block's loads are
    // issued before the current block's arithmetic.
    const int n_full = min_lim > seg.j0 ? (min_lim - seg.j0) / kBlockKeys : 0;
    KvBlock A, Bk;
    int blk = 0;
    if (n_full > 0) {
        load_block(A, rk, rv, voffset, row_stride, seg.j0);
        for (; blk + 2 <= n_full; blk += 2) {
            load_block(Bk, rk, rv, voffset, row_stride, seg.j0 + (blk + 1) * kBlockKeys);
            compute_block<R, false>(st, A, q, prm.scale_log2, 0, lim_of);
            if (blk + 2 < n_full) load_block(A, rk, rv, voffset, row_stride, seg.j0 + (blk + 2) * kBlockKeys);
            compute_block<R, false>(st, Bk, q, prm.scale_log2, 0, lim_of);
        }
        if (blk < n_full) compute_block<R, false>(st, A, q, prm.scale_log2, 0, lim_of);
    }
    // Ragged tail and the causally masked last keys.
    for (int jt = seg.j0 + n_full * kBlockKeys; jt < seg.j1; jt += kBlockKeys) {
        load_block(A, rk, rv, voffset, row_stride, jt);
        compute_block<R, true>(st, A, q, prm.scale_log2, jt + sub, lim_of);
    }

    // Combine the four 16-lane groups (each saw every fourth key) into one state per row.
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float m = st.m[r];
        m = fmaxf(m, __shfl_xor(m, 16, 64));
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        const float m_use = (m == kNegInf) ? 0.0f : m;
        const float w = fast_exp2(st.m[r] - m_use);
        float l = st.l[r] * w;
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        st.m[r] = m;
        st.l[r] = l;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float o = st.o[r][e] * w;
            o += __shfl_xor(o, 16, 64);
            o += __shfl_xor(o, 32, 64);
            st.o[r][e] = o;
        }
    }

    // Store: group `sub` stores rows r with r % 4 == sub.
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r >= seg.n_rows || (r & 3) != sub) continue;
        if (seg.whole) {
            const long orow = row_index(r);
            const float inv = st.l[r] > 0.0f ? 1.0f / st.l[r] : 0.0f;
            uint4 w;
            w.x = pack_bf16(st.o[r][0] * inv, st.o[r][1] * inv);
            w.y = pack_bf16(st.o[r][2] * inv, st.o[r][3] * inv);
            w.z = pack_bf16(st.o[r][4] * inv, st.o[r][5] * inv);
            w.w = pack_bf16(st.o[r][6] * inv, st.o[r][7] * inv);
            *reinterpret_cast<uint4*>(prm.out + orow * kHeadDim + ds * 8) = w;
            if (prm.lse && ds == 0)
                prm.lse[orow] = st.l[r] > 0.0f ? (st.m[r] + __log2f(st.l[r])) * kLn2 : kNegInf;
        } else {
            const int t = (seg.row0 + r) / G, g = (seg.row0 + r) - t * G;
            const long prow = (long)seg.slot * (T * Hq) + t * Hq + seg.kvh * G + g;
            float4* po = reinterpret_cast<float4*>(prm.part_o + prow * kHeadDim + ds * 8);
            po[0] = make_float4(st.o[r][0], st.o[r][1], st.o[r][2], st.o[r][3]);
            po[1] = make_float4(st.o[r][4], st.o[r][5], st.o[r][6], st.o[r][7]);
            if (ds == 0) reinterpret_cast<float2*>(prm.part_ml)[prow] = make_float2(st.m[r], st.l[r]);
        }
    }
}

// ---------------------------------------------------------------------------------- matrix path
// Lane (kb, n) = (lane / 16, lane % 16).  Loads: lane holds 16 bytes (chunk n of 16) of key rows
// 4*kb + i, i = 0..3, of the 16-key block.  MFMA index maps (any consistent map of the 128 columns
// to the contraction index, and of output columns to physical columns, is allowed):
//   S^T[key][row] = sum_c K[key][c] Q[row][c]: 16x16x32 step s, lane (kb, x) contracts chunk 4*s + kb
//   O^T_e[x][row] += V[key][8*x + e] P[row][key]: 16x16x4 call (i, e) contracts keys 4*kb + i
struct KvRegs {
    u32x4_t k[4];
    u32x4_t v[4];
};

__device__ __forceinline__ void load_regs(KvRegs& r, __amdgpu_buffer_rsrc_t rk, __amdgpu_buffer_rsrc_t rv,
                                          uint32_t voffset, uint32_t row_stride, int j_block) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t so = (uint32_t)(j_block + i) * row_stride;
        r.k[i] = load_b128_nt(rk, voffset, so);
        r.v[i] = load_b128_nt(rv, voffset, so);
    }
}

struct MatrixState {
    f32x4_t o[8];     // O^T tiles: o[e][j] = column 8*(4*kb + j) + e of row n
    float m, l;       // row n: running max (all kb groups agree), this lane's share of the running sum
};

template <int kPv>
__device__ __forceinline__ void matrix_block(MatrixState& st, const KvRegs& r, const bf16x8_t (&qop)[4],
                                             char* lds_wave, float scale_log2, int j_block, int lim, int kb,
                                             int n) {
    // K block -> LDS as [key][chunk ^ (key & 7)] (16-byte chunks), then back as the MFMA A operand.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int key = 4 * kb + i;
        *reinterpret_cast<u32x4_t*>(lds_wave + key * kRowBytes + ((n ^ (key & 7)) << 4)) = r.k[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    f32x4_t s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int step = 0; step < 4; ++step) {
        const int c = 4 * step + kb;
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(lds_wave + n * kRowBytes + ((c ^ (n & 7)) << 4));
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qop[step], s, 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // s[i] = score of key j_block + 4*kb + i for row n
    float p[4];
    float mx = kNegInf;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        p[i] = (j_block + 4 * kb + i < lim) ? s[i] * scale_log2 : kNegInf;
        mx = fmaxf(mx, p[i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(st.m, mx);
    const float m_use = (m_new == kNegInf) ? 0.0f : m_new;
    const float alpha = fast_exp2(st.m - m_use);
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        p[i] = fast_exp2(p[i] - m_use);
        sum += p[i];
    }
    st.l = st.l * alpha + sum;
    st.m = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[e] *= alpha;
    }
    if (kPv == kPvFp32) {
        // O^T_e += V_i[e] (x) p_i over the 4 key groups: fp32 MFMA, p exact.
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v[8];
            v[0] = bf16_lo(r.v[i].x); v[1] = bf16_hi(r.v[i].x);
            v[2] = bf16_lo(r.v[i].y); v[3] = bf16_hi(r.v[i].y);
            v[4] = bf16_lo(r.v[i].z); v[5] = bf16_hi(r.v[i].z);
            v[6] = bf16_lo(r.v[i].w); v[7] = bf16_hi(r.v[i].w);
#pragma unroll
            for (int e = 0; e < 8; ++e) st.o[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(v[e], p[i], st.o[e], 0, 0, 0);
        }
    } else {
        // bf16 MFMA 16x16x16 contracts the block's 16 keys at once: lane (kb, x) supplies keys 4*kb + i,
        // i = 0..3, of column 8*x + e (the e-th bf16 of its four V registers) and of row n (its four p).
        // kPvBf16x2 feeds p as hi + lo bf16 parts in two MFMAs, which keeps p to 16 significant bits.
        const f32x2_t p01 = {p[0], p[1]}, p23 = {p[2], p[3]};
        const bf16x2_t h01 = __builtin_convertvector(p01, bf16x2_t), h23 = __builtin_convertvector(p23, bf16x2_t);
        const u32x2_t ph = {__builtin_bit_cast(uint32_t, h01), __builtin_bit_cast(uint32_t, h23)};
        u32x2_t pl = {0u, 0u};
        if (kPv == kPvBf16x2) {
            const f32x2_t r01 = p01 - __builtin_convertvector(h01, f32x2_t);
            const f32x2_t r23 = p23 - __builtin_convertvector(h23, f32x2_t);
            pl.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(r01, bf16x2_t));
            pl.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(r23, bf16x2_t));
        }
        const uint32_t vw[4][4] = {{r.v[0].x, r.v[0].y, r.v[0].z, r.v[0].w}, {r.v[1].x, r.v[1].y, r.v[1].z, r.v[1].w},
                                   {r.v[2].x, r.v[2].y, r.v[2].z, r.v[2].w}, {r.v[3].x, r.v[3].y, r.v[3].z, r.v[3].w}};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;      // high or low halves of both words
            const u32x2_t a = {__builtin_amdgcn_perm(vw[1][e >> 1], vw[0][e >> 1], sel),
                               __builtin_amdgcn_perm(vw[3][e >> 1], vw[2][e >> 1], sel)};
            st.o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a),
                                                                __builtin_bit_cast(s16x4_t, ph), st.o[e], 0, 0, 0);
            if (kPv == kPvBf16x2)
                st.o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a),
                                                                    __builtin_bit_cast(s16x4_t, pl), st.o[e], 0, 0, 0);
        }
    }
}

// A segment in flight on the matrix path: its per-lane constants, its Q operand and the loads of its
// first block.  matrix_begin issues the loads, matrix_run consumes the blocks, matrix_finish stores.
// The kernel begins the next segment before it finishes the current one, so that the new
// segment's first loads are not queued behind the old segment's stores (a wave's memory operations
// complete in order, and a store's completion takes several microseconds under a saturated read
// stream) and the read stream does not drain at a segment boundary.
struct MatrixCtx {
    Segment seg;
    __amdgpu_buffer_rsrc_t rk, rv;
    uint32_t voffset;
    bf16x8_t qop[4];
    int lim;          // first key index row n may not see
    bool row_ok;      // row n of the tile exists
    int t, g;         // row n <-> (token, head within the group)
    long orow;        // output row of row n
    KvRegs first;     // block 0
};

__device__ __forceinline__ void matrix_begin(MatrixCtx& c, const DecodeParams& prm, const Segment& seg, int lane) {
    const int kb = lane >> 4, n = lane & 15;
    const int G = prm.group, T = prm.q_len, Hq = prm.n_q_heads;
    const uint32_t row_stride = (uint32_t)prm.n_kv_heads * kRowBytes;
    c.seg = seg;
    c.rk = make_rsrc(seg.kp, seq_bytes(prm, seg.L));
    c.rv = make_rsrc(seg.vp, seq_bytes(prm, seg.L));
    c.voffset = (uint32_t)(4 * kb) * row_stride + (uint32_t)seg.kvh * kRowBytes + n * 16;
    load_regs(c.first, c.rk, c.rv, c.voffset, row_stride, seg.j0);
    // Row n of the tile <-> (token t, head kvh*G + g); rows past n_rows are zero padding.
    c.row_ok = n < seg.n_rows;
    const int rr = seg.row0 + (c.row_ok ? n : 0);
    c.t = rr / G;
    c.g = rr - c.t * G;
    c.orow = (long)(seg.b * T + c.t) * Hq + seg.kvh * G + c.g;
#pragma unroll
    for (int step = 0; step < 4; ++step) {
        u32x4_t qv = {0u, 0u, 0u, 0u};
        if (c.row_ok) qv = *reinterpret_cast<const u32x4_t*>(prm.q + c.orow * kHeadDim + (4 * step + kb) * 8);
        c.qop[step] = __builtin_bit_cast(bf16x8_t, qv);
    }
    const int causal = seg.L - T + c.t + 1;
    c.lim = causal < seg.j1 ? causal : seg.j1;
}

template <int kPv>
__device__ __forceinline__ void matrix_run(MatrixState& st, MatrixCtx& c, const DecodeParams& prm, int lane,
                                           char* lds_wave) {
    const int kb = lane >> 4, n = lane & 15;
    const uint32_t row_stride = (uint32_t)prm.n_kv_heads * kRowBytes;
    const Segment& seg = c.seg;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.o[e] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    st.m = kNegInf;
    st.l = 0.0f;
    // Two register buffers: the next block's 8 loads per lane are issued before the current block's
    // arithmetic.
    const int n_blocks = (seg.j1 - seg.j0 + kBlockKeys - 1) / kBlockKeys;
    auto key0 = [&](int blk) { return seg.j0 + blk * kBlockKeys; };
    KvRegs Bk;
    int blk = 0;
    for (; blk + 2 <= n_blocks; blk += 2) {
        load_regs(Bk, c.rk, c.rv, c.voffset, row_stride, key0(blk + 1));
        matrix_block<kPv>(st, c.first, c.qop, lds_wave, prm.scale_log2, key0(blk), c.lim, kb, n);
        if (blk + 2 < n_blocks) load_regs(c.first, c.rk, c.rv, c.voffset, row_stride, key0(blk + 2));
        matrix_block<kPv>(st, Bk, c.qop, lds_wave, prm.scale_log2, key0(blk + 1), c.lim, kb, n);
    }
    if (blk < n_blocks) matrix_block<kPv>(st, c.first, c.qop, lds_wave, prm.scale_log2, key0(blk), c.lim, kb, n);
}

template <bool kWriteThrough>
__device__ __forceinline__ void matrix_finish(const MatrixState& st, const MatrixCtx& c, const DecodeParams& prm,
                                              int lane, char* lds_wave) {
    const int kb = lane >> 4, n = lane & 15;
    const int G = prm.group, T = prm.q_len, Hq = prm.n_q_heads;
    const Segment& seg = c.seg;
    float l = st.l;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    // Store through LDS so that every store instruction writes whole contiguous rows (a lane's own
    // accumulators are 16-byte pieces of 16 different rows).
    auto fence = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto row_of = [&](int r, long* out_row, int* seq_row) {      // tile row r -> output row, row within the sequence
        const int rr2 = seg.row0 + r;
        const int t2 = rr2 / G, g2 = rr2 - t2 * G;
        *seq_row = t2 * Hq + seg.kvh * G + g2;
        *out_row = (long)seg.b * T * Hq + *seq_row;
    };
    fence();      // the last block's LDS reads are done
    if (seg.whole) {
        constexpr int kPitch = kRowBytes + 16;                   // bf16 rows, padded against bank conflicts
        const float inv = l > 0.0f ? 1.0f / l : 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint4 w;
            w.x = pack_bf16(st.o[0][j] * inv, st.o[1][j] * inv);
            w.y = pack_bf16(st.o[2][j] * inv, st.o[3][j] * inv);
            w.z = pack_bf16(st.o[4][j] * inv, st.o[5][j] * inv);
            w.w = pack_bf16(st.o[6][j] * inv, st.o[7][j] * inv);
            *reinterpret_cast<uint4*>(lds_wave + n * kPitch + (4 * kb + j) * 16) = w;
        }
        fence();
#pragma unroll
        for (int i = 0; i < 4; ++i) {                             // 4 rows of 256 bytes per store instruction
            const int r = 4 * i + (lane >> 4);
            if (r < seg.n_rows) {
                long orow2;
                int th2;
                row_of(r, &orow2, &th2);
                const u32x4_t w = *reinterpret_cast<const u32x4_t*>(lds_wave + r * kPitch + (lane & 15) * 16);
                store_b128<kWriteThrough>(prm.out + (long)seg.b * T * Hq * kHeadDim, (uint32_t)(T * Hq * kRowBytes),
                              (uint32_t)(th2 * kRowBytes + (lane & 15) * 16), w);
            }
        }
        if (c.row_ok && prm.lse && kb == 0) prm.lse[c.orow] = l > 0.0f ? (st.m + __log2f(l)) * kLn2 : kNegInf;
    } else {
        constexpr int kPitch = kHeadDim * 4 + 16;                // fp32 rows, padded
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float4* w = reinterpret_cast<float4*>(lds_wave + n * kPitch + (4 * kb + j) * 32);
            w[0] = make_float4(st.o[0][j], st.o[1][j], st.o[2][j], st.o[3][j]);
            w[1] = make_float4(st.o[4][j], st.o[5][j], st.o[6][j], st.o[7][j]);
        }
        fence();
#pragma unroll
        for (int i = 0; i < 8; ++i) {                             // 2 rows of 512 bytes per store instruction
            const int r = 2 * i + (lane >> 5);
            if (r < seg.n_rows) {
                long orow2;
                int th2;
                row_of(r, &orow2, &th2);
                const u32x4_t w = *reinterpret_cast<const u32x4_t*>(lds_wave + r * kPitch + (lane & 31) * 16);
                store_b128<kWriteThrough>(prm.part_o + (long)seg.slot * (T * Hq) * kHeadDim, (uint32_t)(T * Hq * kHeadDim * 4),
                              (uint32_t)(th2 * kHeadDim * 4 + (lane & 31) * 16), w);
            }
        }
        if (c.row_ok && kb == 0) {
            const long prow = (long)seg.slot * (T * Hq) + c.t * Hq + seg.kvh * G + c.g;
            reinterpret_cast<float2*>(prm.part_ml)[prow] = make_float2(st.m, l);
        }
    }
    fence();      // the next segment's K blocks reuse this LDS
}

// ---------------------------------------------------------------------------------- decode kernel
// grid.x = pieces, grid.y = row tiles of R rows, grid.z = groups of up to 8 KV heads; block = 64 * heads.
// kMatrix selects the matrix path (R must be 16 then).
// Fixed work of a (piece, sequence) segment in token units for the partition (0 = pieces of equal token
// count; 16 measured best of 0 / 16 / 48: 0.2 to 1 % on the four large workloads).
constexpr int kGqaSegCost = 16;

template <int R, bool kMatrix, int kPv>
__global__ __launch_bounds__(512) void split_decode_kernel(DecodeParams prm) {
    __shared__ __attribute__((aligned(16))) char lds[kMatrix ? kMaxWavesPerBlock * kLdsPerWave : 16];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int kvh = blockIdx.z * kMaxWavesPerBlock + wave;
    if (kvh >= prm.n_kv_heads) return;
    const WavePlan wp = wave_plan(prm.kv_lens, nullptr, nullptr, prm.batch, prm.n_pieces, prm.min_piece_tokens, kGqaSegCost,
                                  prm.xcd_skew, lane, nullptr);
    const Plan& pl = wp.pl;

    // Piece index: consecutive workgroups go to different XCDs, so give each XCD one contiguous
    // eighth of the token stream.
    const int per_xcd = (pl.n_pieces + 7) >> 3;
    const int bid = blockIdx.x;
    const int p = (bid & 7) * per_xcd + (bid >> 3);
    const int s0 = piece_bound(pl, p), s1 = piece_bound(pl, p + 1);
    const bool active = (bid >> 3) < per_xcd && p < pl.n_pieces && s0 < s1;

    if (blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x < 64) {
        // For the merge kernel: first partial slot and number of segments of every sequence, 64
        // sequences per wave, the groups of 64 dealt out over the workgroups.
        for (int g = bid; 64 * g < prm.batch; g += gridDim.x) wave_write_meta(wp, prm.kv_lens, prm.batch, g, lane, prm.meta);
    }
    if (!active) return;

    Walk walk;
    wave_locate(wp, prm.kv_lens, nullptr, nullptr, prm.batch, s0, lane, nullptr, walk.b, walk.j);
    walk.remaining = s1 - s0;

    const int rows_total = prm.group * prm.q_len;
    Segment seg;
    seg.kvh = kvh;
    seg.row0 = blockIdx.y * R;
    seg.n_rows = rows_total - seg.row0 < R ? rows_total - seg.row0 : R;
    // Next (piece, sequence) intersection of this piece, in stream order; false when the piece is done.
    auto next_seg = [&](Segment& out) {
        PieceSeg ps;
        if (!next_segment(walk, prm.batch, pl.seg_cost,
                          [&](int b) { return __builtin_amdgcn_readfirstlane(clamp_len(prm.kv_lens[b])); }, ps))
            return false;
        out = seg;
        out.b = ps.b;
        out.kp = prm.k_ptrs[ps.b];
        out.vp = prm.v_ptrs[ps.b];
        out.L = ps.L;
        out.j0 = ps.j0;
        out.j1 = ps.j1;
        out.slot = p + ps.b;
        out.whole = ps.whole;
        return true;
    };
    if (kMatrix) {
        char* lds_wave = lds + wave * kLdsPerWave;
        Segment cur_seg;
        if (!next_seg(cur_seg)) return;
        MatrixCtx cur;
        matrix_begin(cur, prm, cur_seg, lane);
        for (;;) {
            MatrixState st;
            matrix_run<kPv>(st, cur, prm, lane, lds_wave);
            Segment nxt_seg;
            const bool more = next_seg(nxt_seg);
            MatrixCtx nxt;
            if (more) matrix_begin(nxt, prm, nxt_seg, lane);     // its loads go out before cur's stores
            if (more) matrix_finish<true>(st, cur, prm, lane, lds_wave);
            else matrix_finish<false>(st, cur, prm, lane, lds_wave);
            if (!more) break;
            cur = nxt;
        }
    } else {
        Segment s2;
        while (next_seg(s2)) vector_segment<R>(prm, s2, lane);
    }
}

// ---------------------------------------------------------------------------------- merge kernel
// Aggregation of the partial results of split sequences (section 4.4.3, "Layer 2"):
//   M = max_s m_s;  l = sum_s l_s 2^(m_s - M);  out = sum_s o_s 2^(m_s - M) / l;  lse = (M + log2 l) ln 2
// One wave per output row (b, t, h); lane holds columns 2*lane, 2*lane+1.  Sequences with a single
// segment were finished by the decode kernel and are skipped; sequences without keys get out = 0 and
// lse = -inf here.  All loads of a round are issued before any is used.
__global__ __launch_bounds__(256) void merge_kernel(DecodeParams prm) {
    const int lane = threadIdx.x & 63;
    const long stride_rows = (long)prm.q_len * prm.n_q_heads;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long)prm.batch * stride_rows) return;
    const int b = (int)(row / stride_rows);
    const int th = (int)(row - (long)b * stride_rows);
    const int2 fs = reinterpret_cast<const int2*>(prm.meta)[b];
    const int n = fs.y;
    if (n == 1) return;
    uint32_t* outp = reinterpret_cast<uint32_t*>(prm.out + row * kHeadDim) + lane;
    if (n == 0) {
        *outp = 0u;
        if (prm.lse && lane == 0) prm.lse[row] = kNegInf;
        return;
    }
    const float2* ml = reinterpret_cast<const float2*>(prm.part_ml) + (long)fs.x * stride_rows + th;
    const float2* po = reinterpret_cast<const float2*>(prm.part_o + ((long)fs.x * stride_rows + th) * kHeadDim) + lane;
    // Lane s holds (m_s, l_s) of slot s of the current group of 64 slots; the first 8 slots' partial
    // rows are requested in the same breath, so a typical row (up to 8 segments) costs one round trip.
    float2 mine = make_float2(kNegInf, 0.0f);
    if (lane < n) mine = ml[lane * stride_rows];
    float2 o[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) o[u] = po[(u < n ? u : n - 1) * stride_rows * (kHeadDim / 2)];
    float M = mine.x;
    for (int base = 64; base < n; base += 64)
        if (base + lane < n) M = fmaxf(M, ml[(base + lane) * stride_rows].x);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    const float m_use = (M == kNegInf) ? 0.0f : M;
    float l = 0.0f, o0 = 0.0f, o1 = 0.0f;
    for (int s0 = 0; s0 < n; s0 += 8) {
        if (s0 > 0) {
            if ((s0 & 63) == 0) mine = (s0 + lane < n) ? ml[(s0 + lane) * stride_rows] : make_float2(kNegInf, 0.0f);
#pragma unroll
            for (int u = 0; u < 8; ++u) o[u] = po[(s0 + u < n ? s0 + u : n - 1) * stride_rows * (kHeadDim / 2)];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float m_s = __shfl(mine.x, (s0 + u) & 63, 64), l_s = __shfl(mine.y, (s0 + u) & 63, 64);
            const float w = s0 + u < n ? fast_exp2(m_s - m_use) : 0.0f;      // past the end: weight 0
            l = __builtin_fmaf(l_s, w, l);
            o0 = __builtin_fmaf(o[u].x, w, o0);
            o1 = __builtin_fmaf(o[u].y, w, o1);
        }
    }
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    *outp = pack_bf16(o0 * inv, o1 * inv);
    if (prm.lse && lane == 0) prm.lse[row] = l > 0.0f ? (M + __log2f(l)) * kLn2 : kNegInf;
}

// ---------------------------------------------------------------------------------- write_kvcache
// One workgroup per (sequence, new token): copies the token's K row and V row (n_kv_heads * 256 bytes
// each) to row kv_len - q_len + t of the sequence's ranges, 16 bytes per lane.
__global__ __launch_bounds__(256) void write_kvcache_kernel(WriteParams prm) {
    const int b = blockIdx.x / prm.q_len, t = blockIdx.x - b * prm.q_len;
    const long pos = (long)prm.kv_lens[b] - prm.q_len + t;
    if (pos < 0) return;
    const long src = (long)blockIdx.x * prm.row_bytes;
    char* kd = static_cast<char*>(prm.k_ptrs[b]) + pos * prm.row_bytes;
    char* vd = static_cast<char*>(prm.v_ptrs[b]) + pos * prm.row_bytes;
    const char* ks = reinterpret_cast<const char*>(prm.k_new) + src;
    const char* vs = reinterpret_cast<const char*>(prm.v_new) + src;
    for (int i = threadIdx.x * 16; i < prm.row_bytes; i += blockDim.x * 16) {
        *reinterpret_cast<uint4*>(kd + i) = *reinterpret_cast<const uint4*>(ks + i);
        *reinterpret_cast<uint4*>(vd + i) = *reinterpret_cast<const uint4*>(vs + i);
    }
}

template <int R, bool kMatrix, int kPv = kPvBf16x2>
hipError_t launch_decode_r(const DecodeParams& prm, dim3 grid, dim3 block, hipStream_t stream) {
    hipLaunchKernelGGL((split_decode_kernel<R, kMatrix, kPv>), grid, block, 0, stream, prm);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_write_kvcache(const WriteParams& prm, hipStream_t stream) {
    hipLaunchKernelGGL(write_kvcache_kernel, dim3((unsigned)(prm.batch * prm.q_len)), dim3(256), 0, stream, prm);
    return hipGetLastError();
}

// Measured on MI355X: the matrix path is the faster one from 4 query rows per KV head upwards
// (Qwen-style groups of 4, 5 and 8 at q_len 1, and every multi-token case); below that most of a
// 16-row MFMA tile would be padding and the vector path does less work.
bool use_matrix_path(int rows_total, int path) {
    return path == kPathMatrix || (path == kPathAuto && rows_total >= 4);
}

int rows_per_tile(int rows_total, int path) {
    if (use_matrix_path(rows_total, path)) return 16;
    static const int kSizes[] = {1, 2, 3, 4, 5, 6, 8};
    for (int s : kSizes)
        if (rows_total <= s) return s;
    return 8;
}

hipError_t launch_decode(const DecodeParams& prm, hipStream_t stream, hipEvent_t* events) {
    const int rows_total = prm.group * prm.q_len;
    const bool matrix = use_matrix_path(rows_total, prm.path);
    const int R = rows_per_tile(rows_total, prm.path);
    const int heads_per_block = prm.n_kv_heads < kMaxWavesPerBlock ? prm.n_kv_heads : kMaxWavesPerBlock;
    dim3 grid((prm.n_pieces + 7) / 8 * 8, (rows_total + R - 1) / R,
              (prm.n_kv_heads + kMaxWavesPerBlock - 1) / kMaxWavesPerBlock);
    dim3 block(64 * heads_per_block);
    hipError_t e;
    if (events && (e = hipEventRecord(events[0], stream)) != hipSuccess) return e;
    if (matrix) {
        switch (prm.pv_mode) {
            case kPvBf16: e = launch_decode_r<16, true, kPvBf16>(prm, grid, block, stream); break;
            case kPvFp32: e = launch_decode_r<16, true, kPvFp32>(prm, grid, block, stream); break;
            default: e = launch_decode_r<16, true, kPvBf16x2>(prm, grid, block, stream); break;
        }
    } else {
        switch (R) {
            case 1: e = launch_decode_r<1, false>(prm, grid, block, stream); break;
            case 2: e = launch_decode_r<2, false>(prm, grid, block, stream); break;
            case 3: e = launch_decode_r<3, false>(prm, grid, block, stream); break;
            case 4: e = launch_decode_r<4, false>(prm, grid, block, stream); break;
            case 5: e = launch_decode_r<5, false>(prm, grid, block, stream); break;
            case 6: e = launch_decode_r<6, false>(prm, grid, block, stream); break;
            default: e = launch_decode_r<8, false>(prm, grid, block, stream); break;
        }
    }
    if (e != hipSuccess) return e;
    if (events && (e = hipEventRecord(events[1], stream)) != hipSuccess) return e;
    const long rows = (long)prm.batch * prm.q_len * prm.n_q_heads;
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, prm);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (events && (e = hipEventRecord(events[2], stream)) != hipSuccess) return e;
    return hipSuccess;
}

}  // namespace xattn
