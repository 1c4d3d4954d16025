// Split-KV decode attention and its log-sum-exp merge for gfx950 (MI355X).
//
// Work decomposition (paper section 4.4.3, "Layer 3": balance compute units by token count, split
// long sequences, let short ones share a unit).  The keys of the whole batch form one stream of
// N = sum_b kv_lens[b] tokens, cut into equal pieces of C tokens; workgroup p owns tokens
// [p*C, (p+1)*C) of that stream, whatever sequences they belong to.  Inside a workgroup wave w owns
// KV head w, so a workgroup streams one contiguous byte range of K and one of V (no block table:
// section 4.3, "Operator Adaptation").  Each (piece, sequence) intersection is a segment.  A segment
// that covers its whole sequence writes the final result; any other writes an un-normalised partial
// (o, m, l) to slot piece + sequence_index, and the merge kernel combines a sequence's slots.
//
// Inner loop: 16 lanes hold one 256-byte K (or V) row, 8 bf16 each, loaded with one 128-bit load per
// lane, so a wave load covers four rows.  All query rows that share the KV head (GQA group x new
// tokens: section 4.4.1, K is loaded once for all of them and Q stays in registers) are multiplied
// with the row in registers: q.k via bf16 dot2 into fp32, reduced over the 16 lanes with DPP;
// softmax is online in fp32 in the log2 domain; p.v accumulates in fp32.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xattn_kernels.h"

namespace xattn {
namespace {

constexpr int kU = 4;                 // key rows per 16-lane group per block
constexpr int kBlockKeys = 4 * kU;    // key rows per wave per block
constexpr float kNegInf = -__builtin_inff();

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// ---------------------------------------------------------------------------------- lane helpers
template <int kCtrl>
__device__ __forceinline__ float dpp_f(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, true));
}
// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_f<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp_f<0x4E>(x);    // quad_perm [2,3,0,1]
    x += dpp_f<0x141>(x);   // row_half_mirror
    x += dpp_f<0x140>(x);   // row_mirror
    return x;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int wave_incl_scan_i(int v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(v, o, 64);
        if (lane >= o) v += n;
    }
    return v;
}
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c,
                                           false);
}
__device__ __forceinline__ float bf16_lo(uint32_t x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t x) { return __uint_as_float(x & 0xffff0000u); }
// fp32 -> bf16 bits, round to nearest even (finite inputs and infinities; NaN keeps a quiet NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------------------------- the plan
struct Plan {
    int total;      // N: tokens of the whole batch
    int piece;      // C: tokens per piece
    int n_active;   // pieces that hold at least one token
};

__device__ __forceinline__ int clamp_len(int v) { return v > 0 ? v : 0; }

__device__ __forceinline__ Plan make_plan(const int32_t* __restrict__ kv_lens, int batch, int n_pieces,
                                          int min_piece, int lane) {
    int total = 0;
    for (int base = 0; base < batch; base += 64) {
        const int i = base + lane;
        total += wave_sum_i(i < batch ? clamp_len(kv_lens[i]) : 0);
    }
    total = __builtin_amdgcn_readfirstlane(total);
    int c = (total + n_pieces - 1) / n_pieces;
    if (c < min_piece) c = min_piece;
    c = (c + kBlockKeys - 1) / kBlockKeys * kBlockKeys;
    Plan pl;
    pl.total = total;
    pl.piece = c;
    pl.n_active = (total + c - 1) / c;
    return pl;
}

// ---------------------------------------------------------------------------------- one segment
template <int R>
struct RowState {
    float m[R];        // running max of the scaled scores, log2 domain
    float l[R];        // running sum of exp2(s - m)
    float o[R][8];     // running sum of exp2(s - m) * v, this lane's 8 of the 128 columns
};

struct KvBlock {
    uint4 k[kU];
    uint4 v[kU];
};

// Loads of a block whose rows all lie inside the segment.
__device__ __forceinline__ void load_block(KvBlock& blk, const char* kbase, const char* vbase, long row_stride,
                                           int j_first) {
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        const long off = (long)(j_first + 4 * u) * row_stride;
        blk.k[u] = *reinterpret_cast<const uint4*>(kbase + off);
        blk.v[u] = *reinterpret_cast<const uint4*>(vbase + off);
    }
}
// Loads of the ragged last block: rows past the segment's end re-read its last row (never memory
// beyond the sequence, which may be unmapped) and are masked out of the scores by the caller.
__device__ __forceinline__ void load_block_clamped(KvBlock& blk, const char* kbase, const char* vbase,
                                                   long row_stride, int j_first, int j_last_valid) {
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        int j = j_first + 4 * u;
        j = j < j_last_valid ? j : j_last_valid;
        const long off = (long)j * row_stride;
        blk.k[u] = *reinterpret_cast<const uint4*>(kbase + off);
        blk.v[u] = *reinterpret_cast<const uint4*>(vbase + off);
    }
}

// One block of kU key rows per 16-lane group against R query rows.
// j_sub: absolute key index of this lane's row for u = 0 (rows u are 4 apart).  lim[r]: first key
// index row r may NOT see (segment end and causal limit); used only when kMasked.
template <int R, bool kMasked>
__device__ __forceinline__ void compute_block(RowState<R>& st, const KvBlock& blk, const uint32_t (&q)[R][4],
                                              float scale_log2, int j_sub, const int (&lim)[R]) {
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
            if (kMasked) acc = (j_sub + 4 * u < lim[r]) ? acc : kNegInf;
            s[r][u] = acc;
        }
    }
    float p[R][kU];
    float alpha[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float mb = s[r][0];
#pragma unroll
        for (int u = 1; u < kU; ++u) mb = fmaxf(mb, s[r][u]);
        const float m_new = fmaxf(st.m[r], mb);
        // While a row has seen no key yet its max is -inf: subtract 0 instead so that exp2 sees
        // -inf (-> 0), not -inf - -inf.
        const float m_use = (kMasked && m_new == kNegInf) ? 0.0f : m_new;
        alpha[r] = fast_exp2(st.m[r] - m_use);
        float sum = 0.0f;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            p[r][u] = fast_exp2(s[r][u] - m_use);
            sum += p[r][u];
        }
        st.l[r] = st.l[r] * alpha[r] + sum;
        st.m[r] = m_new;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[r][e] *= alpha[r];
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
            for (int e = 0; e < 8; ++e) st.o[r][e] = __builtin_fmaf(p[r][u], v[e], st.o[r][e]);
    }
}

// Keys [j0, j1) of sequence b (length L) for this wave's KV head and query rows [row0, row0 + n_rows)
// of the head's G*T rows.  Rows r >= n_rows are padding: they repeat row 0 and are never stored.
template <int R>
__device__ __forceinline__ void process_segment(const DecodeParams& prm, int b, int L, int j0, int j1, int slot,
                                                bool whole_sequence, int kvh, int row0, int n_rows, int lane) {
    const int sub = lane >> 4, ds = lane & 15;
    const int G = prm.group, T = prm.q_len, Hq = prm.n_q_heads;
    const long row_stride = (long)prm.n_kv_heads * (kHeadDim * 2);
    const char* kbase = static_cast<const char*>(prm.k_ptrs[b]) + (long)kvh * (kHeadDim * 2) + ds * 16;
    const char* vbase = static_cast<const char*>(prm.v_ptrs[b]) + (long)kvh * (kHeadDim * 2) + ds * 16;

    // Q rows of this KV head: row r <-> (token t = r / G, head kvh*G + r % G); lane takes columns ds*8..+8.
    uint32_t q[R][4];
    int lim[R];
    int qrow[R];    // row index into [batch*T*Hq]
    int min_lim = j1;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int rr = row0 + (r < n_rows ? r : 0);
        const int t = rr / G, g = rr - t * G;
        qrow[r] = (b * T + t) * Hq + kvh * G + g;
        const uint4 qv = *reinterpret_cast<const uint4*>(prm.q + (long)qrow[r] * kHeadDim + ds * 8);
        q[r][0] = qv.x; q[r][1] = qv.y; q[r][2] = qv.z; q[r][3] = qv.w;
        const int causal = L - T + t + 1;
        lim[r] = causal < j1 ? causal : j1;
        min_lim = lim[r] < min_lim ? lim[r] : min_lim;
    }

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
    const int n_full = min_lim > j0 ? (min_lim - j0) / kBlockKeys : 0;
    const char* kb = kbase + (long)sub * row_stride;
    const char* vb = vbase + (long)sub * row_stride;
    KvBlock A, Bk;
    int blk = 0;
    if (n_full > 0) {
        load_block(A, kb, vb, row_stride, j0);
        for (; blk + 2 <= n_full; blk += 2) {
            load_block(Bk, kb, vb, row_stride, j0 + (blk + 1) * kBlockKeys);
            compute_block<R, false>(st, A, q, prm.scale_log2, 0, lim);
            if (blk + 2 < n_full) load_block(A, kb, vb, row_stride, j0 + (blk + 2) * kBlockKeys);
            compute_block<R, false>(st, Bk, q, prm.scale_log2, 0, lim);
        }
        if (blk < n_full) compute_block<R, false>(st, A, q, prm.scale_log2, 0, lim);
    }
    // Ragged tail and the causally masked last keys.
    for (int jt = j0 + n_full * kBlockKeys; jt < j1; jt += kBlockKeys) {
        load_block_clamped(A, kbase, vbase, row_stride, jt + sub, j1 - 1);
        compute_block<R, true>(st, A, q, prm.scale_log2, jt + sub, lim);
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
        if (r >= n_rows || (r & 3) != sub) continue;
        if (whole_sequence) {
            const float inv = st.l[r] > 0.0f ? 1.0f / st.l[r] : 0.0f;
            uint4 w;
            w.x = pack_bf16(st.o[r][0] * inv, st.o[r][1] * inv);
            w.y = pack_bf16(st.o[r][2] * inv, st.o[r][3] * inv);
            w.z = pack_bf16(st.o[r][4] * inv, st.o[r][5] * inv);
            w.w = pack_bf16(st.o[r][6] * inv, st.o[r][7] * inv);
            *reinterpret_cast<uint4*>(prm.out + (long)qrow[r] * kHeadDim + ds * 8) = w;
            if (prm.lse && ds == 0)
                prm.lse[qrow[r]] = st.l[r] > 0.0f ? (st.m[r] + __log2f(st.l[r])) * 0.6931471805599453f : kNegInf;
        } else {
            const int t = (row0 + r) / G, g = (row0 + r) - t * G;
            const long prow = (long)slot * (T * Hq) + t * Hq + kvh * G + g;
            float4* po = reinterpret_cast<float4*>(prm.part_o + prow * kHeadDim + ds * 8);
            po[0] = make_float4(st.o[r][0], st.o[r][1], st.o[r][2], st.o[r][3]);
            po[1] = make_float4(st.o[r][4], st.o[r][5], st.o[r][6], st.o[r][7]);
            if (ds == 0) reinterpret_cast<float2*>(prm.part_ml)[prow] = make_float2(st.m[r], st.l[r]);
        }
    }
}

// ---------------------------------------------------------------------------------- decode kernel
// grid.x = pieces, grid.y = row tiles of R rows, grid.z = groups of up to 8 KV heads; block = 64 * heads.
template <int R>
__global__ __launch_bounds__(512) void split_decode_kernel(DecodeParams prm) {
    const int lane = threadIdx.x & 63;
    const int kvh = blockIdx.z * kMaxWavesPerBlock + (threadIdx.x >> 6);
    if (kvh >= prm.n_kv_heads) return;
    const Plan pl = make_plan(prm.kv_lens, prm.batch, prm.n_pieces, prm.min_piece_tokens, lane);

    // Piece index: consecutive workgroups go to different XCDs, so give each XCD one contiguous
    // eighth of the token stream.
    const int per_xcd = (pl.n_active + 7) >> 3;
    const int bid = blockIdx.x;
    const int p = (bid & 7) * per_xcd + (bid >> 3);
    const bool active = (bid >> 3) < per_xcd && p < pl.n_active;

    if (bid == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x < 64) {
        // Exclusive prefix sums of the clamped lengths for the merge kernel.
        int run = 0;
        for (int base = 0; base < prm.batch; base += 64) {
            const int i = base + lane;
            const int v = i < prm.batch ? clamp_len(prm.kv_lens[i]) : 0;
            const int incl = wave_incl_scan_i(v, lane) + run;
            if (i < prm.batch) prm.meta[kMetaCum + i] = incl - v;
            run = __shfl(incl, 63, 64);
        }
        if (lane == 0) {
            prm.meta[kMetaTotal] = pl.total;
            prm.meta[kMetaPiece] = pl.piece;
        }
    }
    if (!active) return;

    const int s0 = p * pl.piece;
    const int s1 = (s0 + pl.piece < pl.total) ? s0 + pl.piece : pl.total;

    // Locate the sequence that holds stream token s0.
    int b = 0, j = 0;
    {
        int run = 0;
        for (int base = 0; base < prm.batch; base += 64) {
            const int i = base + lane;
            const int v = i < prm.batch ? clamp_len(prm.kv_lens[i]) : 0;
            const int incl = wave_incl_scan_i(v, lane) + run;
            const unsigned long long hit = __ballot(s0 >= incl - v && s0 < incl);
            if (hit) {
                const int ln = __builtin_ctzll(hit);
                b = base + ln;
                j = s0 - __shfl(incl - v, ln, 64);
                break;
            }
            run = __shfl(incl, 63, 64);
        }
        b = __builtin_amdgcn_readfirstlane(b);
        j = __builtin_amdgcn_readfirstlane(j);
    }

    const int rows_total = prm.group * prm.q_len;
    const int row0 = blockIdx.y * R;
    const int n_rows = rows_total - row0 < R ? rows_total - row0 : R;
    int remaining = s1 - s0;
    while (remaining > 0 && b < prm.batch) {
        const int L = clamp_len(prm.kv_lens[b]);
        if (L == 0) { ++b; continue; }
        const int n = (L - j < remaining) ? L - j : remaining;
        process_segment<R>(prm, b, L, j, j + n, p + b, n == L, kvh, row0, n_rows, lane);
        remaining -= n;
        ++b;
        j = 0;
    }
}

// ---------------------------------------------------------------------------------- merge kernel
// One wave per output row (b, t, h); lane holds columns 2*lane, 2*lane+1.  Sequences with a single
// segment were finished by the decode kernel and are skipped; sequences without keys get out = 0 and
// lse = -inf here.
__global__ __launch_bounds__(256) void merge_kernel(DecodeParams prm) {
    const int lane = threadIdx.x & 63;
    const int T = prm.q_len, Hq = prm.n_q_heads;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long)prm.batch * T * Hq) return;
    const int b = (int)(row / (T * Hq));
    const int th = (int)(row - (long)b * (T * Hq));
    const int L = clamp_len(prm.kv_lens[b]);
    const int piece = prm.meta[kMetaPiece];
    const int start = prm.meta[kMetaCum + b];
    uint32_t* outp = reinterpret_cast<uint32_t*>(prm.out + row * kHeadDim) + lane;
    if (L == 0) {
        *outp = 0u;
        if (prm.lse && lane == 0) prm.lse[row] = kNegInf;
        return;
    }
    const int first = start / piece, last = (start + L - 1) / piece;
    if (first == last) return;
    float M = kNegInf;
    for (int s = first; s <= last; ++s) {
        const float2 ml = reinterpret_cast<const float2*>(prm.part_ml)[(long)(s + b) * (T * Hq) + th];
        M = fmaxf(M, ml.x);
    }
    const float m_use = (M == kNegInf) ? 0.0f : M;
    float l = 0.0f, o0 = 0.0f, o1 = 0.0f;
    for (int s = first; s <= last; ++s) {
        const long prow = (long)(s + b) * (T * Hq) + th;
        const float2 ml = reinterpret_cast<const float2*>(prm.part_ml)[prow];
        const float w = fast_exp2(ml.x - m_use);
        const float2 o = reinterpret_cast<const float2*>(prm.part_o + prow * kHeadDim)[lane];
        l = __builtin_fmaf(ml.y, w, l);
        o0 = __builtin_fmaf(o.x, w, o0);
        o1 = __builtin_fmaf(o.y, w, o1);
    }
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    *outp = pack_bf16(o0 * inv, o1 * inv);
    if (prm.lse && lane == 0) prm.lse[row] = l > 0.0f ? (M + __log2f(l)) * 0.6931471805599453f : kNegInf;
}

template <int R>
hipError_t launch_decode_r(const DecodeParams& prm, dim3 grid, dim3 block, hipStream_t stream) {
    hipLaunchKernelGGL(split_decode_kernel<R>, grid, block, 0, stream, prm);
    return hipGetLastError();
}

}  // namespace

int rows_per_tile(int rows_total) {
    static const int kSizes[] = {1, 2, 3, 4, 5, 6, 8, 12, 16};
    for (int s : kSizes)
        if (rows_total <= s) return s;
    return 16;
}

hipError_t launch_decode(const DecodeParams& prm, hipStream_t stream, hipEvent_t* events) {
    const int rows_total = prm.group * prm.q_len;
    const int R = rows_per_tile(rows_total);
    const int heads_per_block = prm.n_kv_heads < kMaxWavesPerBlock ? prm.n_kv_heads : kMaxWavesPerBlock;
    dim3 grid((prm.n_pieces + 7) / 8 * 8, (rows_total + R - 1) / R,
              (prm.n_kv_heads + kMaxWavesPerBlock - 1) / kMaxWavesPerBlock);
    dim3 block(64 * heads_per_block);
    hipError_t e;
    if (events && (e = hipEventRecord(events[0], stream)) != hipSuccess) return e;
    switch (R) {
        case 1: e = launch_decode_r<1>(prm, grid, block, stream); break;
        case 2: e = launch_decode_r<2>(prm, grid, block, stream); break;
        case 3: e = launch_decode_r<3>(prm, grid, block, stream); break;
        case 4: e = launch_decode_r<4>(prm, grid, block, stream); break;
        case 5: e = launch_decode_r<5>(prm, grid, block, stream); break;
        case 6: e = launch_decode_r<6>(prm, grid, block, stream); break;
        case 8: e = launch_decode_r<8>(prm, grid, block, stream); break;
        case 12: e = launch_decode_r<12>(prm, grid, block, stream); break;
        default: e = launch_decode_r<16>(prm, grid, block, stream); break;
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
