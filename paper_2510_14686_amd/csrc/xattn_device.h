// Device-side helpers shared by the kernels of libxattn.so: vector types, lane operations, buffer
// loads and stores, and the token-stream partition (paper section 4.4.3, "Layer 3").
#ifndef XATTN_DEVICE_H_
#define XATTN_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xattn_kernels.h"

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
// All keys of the batch form one stream that is cut into pieces of equal COST.  A sequence of L > 0
// tokens occupies L + seg_cost positions of the stream: its tokens, then seg_cost positions that stand
// for the fixed work every (piece, sequence) segment costs (first loads, Q, the stores of its result),
// so a workgroup whose piece spans a sequence boundary gets correspondingly fewer tokens.  A piece
// bound that falls into those extra positions means "the end of that sequence".  seg_cost = 0 gives
// pieces of equal token count.
struct Plan {
    int total;      // N: positions of the whole stream
    int n_pieces;   // pieces in use: min(launched pieces, N / minimum piece size), at least 1
    int seg_cost;
};

__device__ __forceinline__ int clamp_len(int v) { return v > 0 ? v : 0; }
// Stream positions of a sequence of `len` tokens (any sign).
__device__ __forceinline__ int stream_len(int len, int seg_cost) { return len > 0 ? len + seg_cost : 0; }

__device__ __forceinline__ Plan make_plan(const int32_t* __restrict__ kv_lens, int batch, int n_pieces,
                                          int min_piece, int seg_cost, int lane) {
    int total = 0;
    for (int base = 0; base < batch; base += 64) {
        const int i = base + lane;
        total += wave_sum_i(i < batch ? stream_len(kv_lens[i], seg_cost) : 0);
    }
    total = __builtin_amdgcn_readfirstlane(total);
    int n = total / min_piece;
    n = n < 1 ? 1 : n;
    Plan pl;
    pl.total = total;
    pl.n_pieces = n < n_pieces ? n : n_pieces;
    pl.seg_cost = seg_cost;
    return pl;
}

// Piece p owns stream positions [piece_bound(p), piece_bound(p + 1)): p * N / n_pieces rounded to a
// multiple of the 16-key block, so every piece is within 16 positions of N / n_pieces and all are used.
__device__ __forceinline__ int piece_bound(const Plan& pl, int p) {
    if (p >= pl.n_pieces) return pl.total;
    const long x = (long)p * pl.total / pl.n_pieces;
    const int r = (int)((x + kBlockKeys / 2) / kBlockKeys) * kBlockKeys;
    return r < pl.total ? r : pl.total;
}
// The piece that owns stream position x (0 <= x < N).
__device__ __forceinline__ int piece_of(const Plan& pl, int x) {
    int p = (int)((long)x * pl.n_pieces / pl.total);
    while (p + 1 < pl.n_pieces && piece_bound(pl, p + 1) <= x) ++p;
    while (p > 0 && piece_bound(pl, p) > x) --p;
    return p;
}

}  // namespace
}  // namespace xattn
#endif
