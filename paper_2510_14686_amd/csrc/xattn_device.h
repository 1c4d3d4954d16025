// Device-side helpers shared by the kernels of libxattn.so: vector types, lane operations, buffer
// loads and stores, and the token-stream partition (paper section 4.4.3, "Layer 3").
#ifndef XATTN_DEVICE_H_
#define XATTN_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xattn_kernels.h"
#include "xattn_plan.h"

namespace xattn {
namespace {

constexpr int kU = 4;                 // key rows per 16-lane group per block
constexpr int kBlockKeys = 4 * kU;    // key rows per wave per block
constexpr int kRowBytes = kHeadDim * 2;
// Wave-private LDS of the matrix path: a 16-key K block (4 KiB) during the key loop, a 16-row fp32
// output tile with padded rows (16 x 528 bytes) when a segment is stored.
constexpr int kLdsPerWave = 16 * (kHeadDim * 4 + 16);
constexpr float kNegInf = -__builtin_inff();
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;

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

// Raw buffer descriptor over [base, base + bytes): loads past the end return 0.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
// 128-bit non-temporal load at base + voffset (per lane) + soffset (wave-uniform).
__device__ __forceinline__ u32x4_t load_b128_nt(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t soffset) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voffset, (int)soffset, 2 /* nt */);
}

// Stores of results and partial results: whole rows per instruction (see matrix_finish).  A segment
// that is followed by another one in the same workgroup is written through (sc1): left to the L2's
// write-back policy, its dirty lines are evicted one by one into the saturated read stream later
// (measured on the 16-row workload: 25 MB of partial results cost 37 us of a 400 us kernel, written
// through as full lines 14 us).  A workgroup's last segment keeps the write-back policy: its stores
// complete at the L2 and are flushed in bulk when the kernel ends, which is faster than waiting for
// a write-through at the kernel's tail.
template <bool kWriteThrough>
__device__ __forceinline__ void store_b128(void* base, uint32_t bytes, uint32_t off, u32x4_t v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, make_rsrc(base, bytes), (int)off, 0, kWriteThrough ? 16 /* sc1 */ : 0);
}

// ---------------------------------------------------------------------------------- the plan
// Wave-level front end of the partition in xattn_plan.h.  Every wave computes the plan itself from
// kv_lens (the host never reads the lengths: section 4.2, "Integrating Custom Operators"), in two
// memory round trips and two wave scans whatever the batch: lane l owns the `chunk` consecutive
// sequences l * chunk .. l * chunk + chunk - 1 (chunk = the power of two >= batch / 64, so at most 64
// for the largest batch) and adds up their stream positions from 128-bit loads that are all in
// flight together; one scan over the 64 lane sums gives the total and every chunk's first position;
// a stream position is then located by one ballot (its chunk) and one scan over that chunk's
// sequences.  The loads go through a buffer descriptor over kv_lens, so indices past the batch read 0.
struct WavePlan {
    Plan pl;
    int chunk, chunk_log2;   // sequences per lane
    int mine;                // stream positions of this lane's sequences
    int excl;                // stream positions before this lane's first sequence
};
// Lengths and base addresses of up to 64 consecutive sequences, one per lane: those around the
// position a wave starts at, fetched in the same round trips as the plan, so that a segment's first
// K/V loads do not wait for another two dependent loads (its length, then its pointers).
struct SeqWindow {
    int base, count;         // sequences base .. base + count - 1 are held
    int len;                 // lane l: clamp_len(kv_lens[base + l])
    u32x2_t k, v;            // lane l: k_ptrs[base + l], v_ptrs[base + l] (v unused by kernels with one pointer array)
};

__device__ __forceinline__ u32x2_t load_ptr_entry(const void* const* ptrs, int batch, int idx) {
    const __amdgpu_buffer_rsrc_t r = make_rsrc(ptrs, (uint32_t)batch * 8u);
    return __builtin_bit_cast(u32x2_t, __builtin_amdgcn_raw_buffer_load_b64(r, idx * 8, 0, 0));
}
__device__ __forceinline__ void window_load(SeqWindow& win, const int32_t* __restrict__ kv_lens, const void* const* k_ptrs,
                                            const void* const* v_ptrs, int batch, int base, int count, int lane,
                                            int seg_cost, int& positions) {
    const __amdgpu_buffer_rsrc_t rl = make_rsrc(kv_lens, (uint32_t)batch * 4u);
    const int idx = lane < count ? base + lane : batch;            // past the batch: reads 0
    const int raw = (int)__builtin_amdgcn_raw_buffer_load_b32(rl, idx * 4, 0, 0);
    win.k = load_ptr_entry(k_ptrs, batch, idx);
    win.v = v_ptrs ? load_ptr_entry(v_ptrs, batch, idx) : u32x2_t{0u, 0u};
    win.base = base;
    win.count = count;
    win.len = clamp_len(raw);
    positions = stream_len(raw, seg_cost);
}
// Length and pointers of sequence b: from the window when it holds b, else from memory.  Wave-uniform.
__device__ __forceinline__ int window_len(const SeqWindow& win, const int32_t* __restrict__ kv_lens, int b) {
    const unsigned i = (unsigned)(b - win.base);
    if (i < (unsigned)win.count) return __builtin_amdgcn_readlane(win.len, __builtin_amdgcn_readfirstlane((int)i));
    return __builtin_amdgcn_readfirstlane(clamp_len(kv_lens[b]));
}
__device__ __forceinline__ const void* window_ptr(const SeqWindow& win, const u32x2_t& held, const void* const* ptrs, int b) {
    const unsigned i = (unsigned)(b - win.base);
    uint64_t a;
    if (i < (unsigned)win.count) {
        const int li = __builtin_amdgcn_readfirstlane((int)i);
        a = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)held.x, li) |
            ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)held.y, li) << 32);
    } else {
        const uint64_t m = (uint64_t)(uintptr_t)ptrs[b];
        a = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)m) |
            ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(m >> 32)) << 32);
    }
    return reinterpret_cast<const void*>((uintptr_t)a);
}

template <int kQuads>
__device__ __forceinline__ int chunk_positions(__amdgpu_buffer_rsrc_t rl, int first, int seg_cost) {
    u32x4_t v[kQuads];
#pragma unroll
    for (int k = 0; k < kQuads; ++k) v[k] = __builtin_amdgcn_raw_buffer_load_b128(rl, (first + 4 * k) * 4, 0, 0);
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kQuads; ++k)
        sum += stream_len((int)v[k].x, seg_cost) + stream_len((int)v[k].y, seg_cost) +
               stream_len((int)v[k].z, seg_cost) + stream_len((int)v[k].w, seg_cost);
    return sum;
}

// win (optional): with at most 64 sequences (one per lane) the window is filled here, in the plan's own
// round trip.  (It pays in the latent-KV kernel, whose workgroups wait at a barrier for the first block
// of a segment; the GQA kernel's independent waves hide those two loads and only lose registers to it.)
__device__ __forceinline__ WavePlan wave_plan(const int32_t* __restrict__ kv_lens, const void* const* k_ptrs,
                                              const void* const* v_ptrs, int batch, int n_pieces, int min_piece,
                                              int seg_cost, int xcd_skew, int lane, SeqWindow* win) {
    WavePlan wp;
    int lg = 0;
    while ((64 << lg) < batch) ++lg;                       // wave-uniform: batch is a kernel argument
    wp.chunk_log2 = lg;
    wp.chunk = 1 << lg;
    const __amdgpu_buffer_rsrc_t rl = make_rsrc(kv_lens, (uint32_t)batch * 4u);
    const int first = lane << lg;
    int mine;
    if (win) {
        win->base = 0;
        win->count = 0;
    }
    switch (lg) {
        case 0:
            if (win) window_load(*win, kv_lens, k_ptrs, v_ptrs, batch, 0, batch, lane, seg_cost, mine);
            else mine = stream_len(__builtin_amdgcn_raw_buffer_load_b32(rl, first * 4, 0, 0), seg_cost);
            break;
        case 1: mine = stream_len(__builtin_amdgcn_raw_buffer_load_b32(rl, first * 4, 0, 0), seg_cost) +
                       stream_len(__builtin_amdgcn_raw_buffer_load_b32(rl, first * 4 + 4, 0, 0), seg_cost); break;
        case 2: mine = chunk_positions<1>(rl, first, seg_cost); break;
        case 3: mine = chunk_positions<2>(rl, first, seg_cost); break;
        case 4: mine = chunk_positions<4>(rl, first, seg_cost); break;
        case 5: mine = chunk_positions<8>(rl, first, seg_cost); break;
        default: mine = chunk_positions<16>(rl, first, seg_cost); break;   // batch <= 4096 (checked by the host)
    }
    const int incl = wave_incl_scan_i(mine, lane);
    wp.mine = mine;
    wp.excl = incl - mine;
    wp.pl = plan_for_total(__builtin_amdgcn_readlane(incl, 63), n_pieces, min_piece, seg_cost, xcd_skew);
    return wp;
}

// The sequence b that holds stream position s (0 <= s < N) and the offset j of s within that
// sequence's L + seg_cost positions.  Both wave-uniform.  With more than 64 sequences the window is
// filled here with the located chunk.
__device__ __forceinline__ void wave_locate(const WavePlan& wp, const int32_t* __restrict__ kv_lens, const void* const* k_ptrs,
                                            const void* const* v_ptrs, int batch, int s, int lane, SeqWindow* win, int& b,
                                            int& j) {
    const unsigned long long hit = __ballot(s >= wp.excl && s < wp.excl + wp.mine);
    const int ln = hit ? __builtin_ctzll(hit) : 0;
    const int off = s - __shfl(wp.excl, ln, 64);
    if (wp.chunk_log2 == 0) {
        b = __builtin_amdgcn_readfirstlane(ln);
        j = __builtin_amdgcn_readfirstlane(off);
        return;
    }
    const int base = ln << wp.chunk_log2;
    int v;
    if (win) {
        window_load(*win, kv_lens, k_ptrs, v_ptrs, batch, base, wp.chunk, lane, wp.pl.seg_cost, v);
    } else {
        const __amdgpu_buffer_rsrc_t rl = make_rsrc(kv_lens, (uint32_t)batch * 4u);
        v = lane < wp.chunk ? stream_len(__builtin_amdgcn_raw_buffer_load_b32(rl, (base + lane) * 4, 0, 0), wp.pl.seg_cost) : 0;
    }
    const int incl = wave_incl_scan_i(v, lane);
    const unsigned long long hit2 = __ballot(off >= incl - v && off < incl);
    const int ln2 = hit2 ? __builtin_ctzll(hit2) : 0;
    b = __builtin_amdgcn_readfirstlane(base + ln2);
    j = __builtin_amdgcn_readfirstlane(off - __shfl(incl - v, ln2, 64));
}

// For the merge kernel: (first partial slot, number of segments) of sequences 64 g .. 64 g + 63, one
// per lane.  A group of 64 sequences holds 64 / chunk whole chunks; a sequence's first position is its
// chunk's first position plus the positions of the chunk's earlier sequences.
__device__ __forceinline__ void wave_write_meta(const WavePlan& wp, const int32_t* __restrict__ kv_lens, int batch, int g,
                                                int lane, int32_t* __restrict__ meta) {
    const int seq = 64 * g + lane;
    const __amdgpu_buffer_rsrc_t rl = make_rsrc(kv_lens, (uint32_t)batch * 4u);
    const int len = clamp_len(__builtin_amdgcn_raw_buffer_load_b32(rl, seq * 4, 0, 0));
    const int v = stream_len(len, wp.pl.seg_cost);
    const int before = wave_incl_scan_i(v, lane) - v;                       // within the group
    const int chunk_first = __shfl(wp.excl, (seq >> wp.chunk_log2) & 63, 64);
    const int start = chunk_first + before - __shfl(before, lane & ~(wp.chunk - 1), 64);
    if (seq < batch) {
        const SeqMeta m = seq_meta(wp.pl, seq, start, len);
        reinterpret_cast<int2*>(meta)[seq] = make_int2(m.first_slot, m.n_seg);
    }
}

}  // namespace
}  // namespace xattn
#endif
