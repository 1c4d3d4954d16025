// Latent-KV (MLA-shaped) split-KV decode attention for gfx950 (MI355X).
//
// The operator the paper itself adapts (section 4.3 "Operator Adaptation": attention on a contiguous
// virtual range, no block table; section 4.4.1 "MLA Optimization": the m+1 query tokens and all
// heads are multiplied with the same cached rows, K is loaded once for all of them and Q stays
// resident).  Per token the cache holds one row of 576 bf16 (512 latent + 64 rope) that is the key of
// every head, and whose first 512 values are every head's value.  With 128 heads that is 242 flop per
// cached byte: the path is bound by the matrix cores and by the LDS that feeds them, not by HBM.
//
// Partition: the same token-stream pieces as the GQA kernel (section 4.4.3, "Layer 3").  A workgroup
// owns one piece and up to 128 query rows (row = token * n_heads + head).  It has at most four waves,
// one per SIMD, so that a wave may use the whole 512-entry register file: a wave owns one or two
// tiles of 16 rows and keeps their Q (72 registers per tile) and their output accumulators (16 x 512
// fp32 = 128 registers per tile) resident for the whole piece.  All waves share each 32-key block of
// the cache through LDS:
//   * the block (32 x 1152 bytes, contiguous in memory) goes from HBM straight into LDS (buffer loads
//     with the LDS destination, 1 KiB per wave instruction, no staging registers), once per
//     workgroup, two LDS buffers, one barrier per block, the next block in flight during the
//     arithmetic.  Rows sit 1184 bytes apart in LDS (two 16-byte pad chunks; the pad is made through
//     the global address each lane fetches, since the LDS side of such a load is fixed to lane order):
//     measured, a pitch of 2 * odd chunks modulo 16 serves both read patterns below without bank
//     conflicts, an odd pitch (1168) halves the rate of both;
//   * S^T = C Q^T: per 16-key tile 18 bf16 MFMA 16x16x32, the A operand (keys) read from LDS and used
//     for both row tiles of the wave;
//   * softmax on the accumulator layout: lane (kb, n) holds, of row n, the keys 4 kb + i of both key
//     tiles, which is exactly the B operand (8 keys per lane) of the next product, so the weights
//     never leave the lane; row maxima cross the four lane groups with lane-swap instructions;
//   * O^T += C[:, 0:512]^T P^T: bf16 MFMA 16x16x32 over the 32 keys, the A operand (16 value columns x
//     8 keys per lane) fetched with LDS transposing reads, again used for both row tiles; P goes in as
//     hi + lo bf16 parts (two MFMAs) unless the caller asks for one rounded bf16.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xattn_device.h"
#include "xattn_kernels.h"

namespace xattn {
namespace {

constexpr int kDqk = 576;                        // key width: latent + rope
constexpr int kDv = 512;                         // value width: the latent part
constexpr int kRowB = kDqk * 2;                  // 1152 bytes per cached token
constexpr int kMlaKeys = 32;                     // keys per LDS block
constexpr int kRowChunks = kRowB / 16;           // 72 chunks of 16 bytes per row
constexpr int kPitchChunks = kRowChunks + 2;     // 74: the pitch in chunks is 2 * odd modulo 16 (see block_to_lds)
constexpr int kPitch = kPitchChunks * 16;        // 1184 bytes between rows in LDS
constexpr int kDmaPerBlock = (kMlaKeys * kPitchChunks + 63) / 64;   // 37 wave-wide loads of 64 x 16 bytes
constexpr int kLdsBlock = kDmaPerBlock * 1024;   // 37888 bytes (the last row's pad is not inside)
constexpr int kTileB = 16 * kPitch;              // from key tile 0 to key tile 1 of a block
constexpr int kQSteps = kDqk / 32;               // 18 MFMA steps of 32 columns
constexpr int kQRegSteps = 9;                    // Q columns 0 .. 32 * 9 - 1 stay in registers, the rest of Q in LDS
constexpr int kQLdsWave = (kQSteps - kQRegSteps) * 1024;   // per 16-row tile: one 16-byte chunk per lane and step
constexpr int kQAhead = 3;                       // key fragments in flight ahead of the MFMAs, in steps
constexpr int kVAhead = 2;                       // value fragments in flight ahead of the MFMAs, in tile pairs
constexpr int kColTiles = kDv / 16;              // 32 tiles of 16 value columns
constexpr int kOutPitch = 128 * 4 + 16;          // epilogue: 16 rows x 128 fp32 columns, padded
constexpr int kLdsOutPerWave = 16 * kOutPitch;

typedef short s16x4v_t __attribute__((ext_vector_type(4)));

// Running state of one 16-row tile.  Lane (kb, n) holds row n.
struct MlaTile {
    f32x4_t o[kColTiles];      // o[ct][i]: column 16 ct + 4 kb + i
    float m, l;                // running maximum (log2 domain) and this lane's share of the sum
};

// The loads are written as assembly so that the compiler does not order them against LDS reads: it
// cannot tell the two halves of the double buffer apart and would wait for every outstanding load
// before each read.  dma_wait() before the workgroup barrier is what makes a block visible.
__device__ __forceinline__ void dma16(u32x4_t rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 1\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// This wave's share of the loads of one 32-key block into LDS: load q fills LDS bytes
// [q * 1024, (q + 1) * 1024) of the block in lane order, i.e. chunk position 64 q + lane = 74 row +
// slot; the lane fetches chunk `slot` of that row (bytes past the sequence's end read as zero), pad
// positions and positions past row 31 fetch nothing.
template <int NW>
__device__ __forceinline__ void block_to_lds(char* lds_block, u32x4_t rc, int j_block, int wave, int lane) {
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_block;
#pragma unroll
    for (int q = 0; q < (kDmaPerBlock + NW - 1) / NW; ++q) {
        const int qq = wave + q * NW;            // wave-uniform
        if (qq < kDmaPerBlock) {
            const int pos = qq * 64 + lane;
            const int row = pos / kPitchChunks, slot = pos - row * kPitchChunks;
            if (slot < kRowChunks && row < kMlaKeys)
                dma16(rc, lds0 + qq * 1024, (uint32_t)(row * kRowB + slot * 16), (uint32_t)j_block * kRowB);
        }
    }
}

// max / sum over the four lanes (kb = 0..3) that hold the same row: lane-swap instructions, no LDS.
// The swap exchanges, between its two register operands, lane group 1 (3) of the first with lane
// group 0 (2) of the second (16-lane form), or the upper half of the first with the lower half of
// the second (32-lane form): called on (x, x), the two results together hold both partners' values.
// (The results are copied to scalars before the bit cast: a bit cast applied directly to an element
// of the result vector read element 0 for both.)
__device__ __forceinline__ void swap16(float x, float& r0, float& r1) {
    const uint32_t a = __builtin_bit_cast(uint32_t, x);
    const u32x2_t t = __builtin_amdgcn_permlane16_swap(a, a, false, false);
    const uint32_t t0 = t.x, t1 = t.y;
    r0 = __builtin_bit_cast(float, t0);
    r1 = __builtin_bit_cast(float, t1);
}
__device__ __forceinline__ void swap32(float x, float& r0, float& r1) {
    const uint32_t a = __builtin_bit_cast(uint32_t, x);
    const u32x2_t t = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const uint32_t t0 = t.x, t1 = t.y;
    r0 = __builtin_bit_cast(float, t0);
    r1 = __builtin_bit_cast(float, t1);
}
__device__ __forceinline__ float kb_max(float x) {
    float a, b;
    swap16(x, a, b);
    x = fmaxf(a, b);
    swap32(x, a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float kb_sum(float x) {
    float a, b;
    swap16(x, a, b);
    x = a + b;
    swap32(x, a, b);
    return a + b;
}

// Scheduling groups (the group sizes must be compile-time constants, hence the templates).
template <int N> __device__ __forceinline__ void sched_ds() { __builtin_amdgcn_sched_group_barrier(0x100, N, 0); }
template <int N> __device__ __forceinline__ void sched_mfma() { __builtin_amdgcn_sched_group_barrier(0x008, N, 0); }
constexpr int qk_reads_of(int step, int rt) { return 2 + (step >= kQRegSteps ? rt : 0); }
constexpr int qk_reads_before(int steps, int rt) {
    int n = 0;
    for (int i = 0; i < steps; ++i) n += qk_reads_of(i, rt);
    return n;
}
template <int STEP, int RT>
struct QkSched {
    static __device__ __forceinline__ void run() {
        sched_mfma<2 * RT>();
        if constexpr (STEP + kQAhead < kQSteps) sched_ds<qk_reads_of(STEP + kQAhead, RT)>();
        if constexpr (STEP + 1 < kQSteps) QkSched<STEP + 1, RT>::run();
    }
};

// One 32-key block from LDS against this wave's RT tiles of 16 rows.  Every operand read from LDS is
// used for all RT tiles.  kHiLo: the softmax weights go into the value product as hi + lo bf16 parts
// (two MFMAs, 16 significant bits) instead of one rounded bf16.
//   qk_base = block + n * kPitch + kb * 16                     (key row n of a tile, chunk kb)
//   pv_base = block + (4 kb + n / 4) * kPitch + (n % 4) * 8    (transposing read, see below)
template <int RT, bool kHiLo>
__device__ __forceinline__ void mla_block(MlaTile (&st)[RT], const char* qk_base, const char* pv_base,
                                          const bf16x8_t (&qop)[RT][kQRegSteps], const char* q_lds, float scale_log2,
                                          int j_block, const int (&lim)[RT], int kb) {
    // S^T tile kt: A = keys 16 kt .. 16 kt + 15 of the block (lane (kb, n): key n, columns 32 step +
    // 8 kb .. + 7), B = Q; the result at lane (kb, n) is key 16 kt + 4 kb + i against row n.
    f32x4_t s[RT][2];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) s[rt][0] = s[rt][1] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    // The key fragments (and, from step kQRegSteps on, the lane's Q chunks, which it parked in LDS at
    // q_lds + tile * kQLdsWave + (step - kQRegSteps) * 1024) are fetched kQAhead steps before the MFMAs
    // that use them.
    bf16x8_t ka[kQSteps][2], ql[RT][kQSteps - kQRegSteps];
    auto load_step = [&](int step) {
        ka[step][0] = *reinterpret_cast<const bf16x8_t*>(qk_base + step * 64);
        ka[step][1] = *reinterpret_cast<const bf16x8_t*>(qk_base + kTileB + step * 64);
        if (step >= kQRegSteps) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                ql[rt][step - kQRegSteps] = *reinterpret_cast<const bf16x8_t*>(q_lds + rt * kQLdsWave + (step - kQRegSteps) * 1024);
        }
    };
#pragma unroll
    for (int step = 0; step < kQAhead; ++step) load_step(step);
#pragma unroll
    for (int step = 0; step < kQSteps; ++step) {
        if (step + kQAhead < kQSteps) load_step(step + kQAhead);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const bf16x8_t qv = step < kQRegSteps ? qop[rt][step < kQRegSteps ? step : 0] : ql[rt][step < kQRegSteps ? 0 : step - kQRegSteps];
            s[rt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[step][0], qv, s[rt][0], 0, 0, 0);
            s[rt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[step][1], qv, s[rt][1], 0, 0, 0);
        }
    }
    // Pin that order for the instruction scheduler: the first reads, then MFMAs and reads in turn.
    sched_ds<qk_reads_before(kQAhead, RT)>();
    QkSched<0, RT>::run();
    // O^T tile ct: A = value columns 16 ct .. + 15 (lane (kb, n): column n, keys as in the softmax
    // below), B = P^T.  A transposing read hands lane n of a 16-lane group, from the 64 values that
    // the group's lanes point at taken in lane order, the values n, n + 16, n + 32, n + 48: lanes 4 j ..
    // 4 j + 3 point at 16 consecutive columns of key 4 kb + j, so lane n receives column n of keys
    // 4 kb .. 4 kb + 3.  The first value fragments are fetched here, ahead of the softmax.
    bf16x8_t va[kColTiles];
    auto load_v = [&](int ct) {
        const s16x4v_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4v_t*)(pv_base + ct * 32));
        const s16x4v_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4v_t*)(pv_base + kTileB + ct * 32));
        const u32x2_t w0 = __builtin_bit_cast(u32x2_t, v0), w1 = __builtin_bit_cast(u32x2_t, v1);
        return __builtin_bit_cast(bf16x8_t, u32x4_t{w0.x, w0.y, w1.x, w1.y});
    };
#pragma unroll
    for (int ct = 0; ct < 2 * kVAhead; ++ct) va[ct] = load_v(ct);
    // Softmax.  The lane's 8 weights of a row, ordered (kt, i), are the B operand of the value product
    // when contraction index 8 kb + 4 kt + i stands for key 16 kt + 4 kb + i.
    bf16x8_t ph[RT], pl[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float p[8];
        float mx = kNegInf;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int key = j_block + 16 * (t >> 2) + 4 * kb + (t & 3);
            p[t] = key < lim[rt] ? s[rt][t >> 2][t & 3] * scale_log2 : kNegInf;
            mx = fmaxf(mx, p[t]);
        }
        mx = kb_max(mx);
        const float m_new = fmaxf(st[rt].m, mx);
        const float m_use = (m_new == kNegInf) ? 0.0f : m_new;
        const float alpha = fast_exp2(st[rt].m - m_use);
        float sum = 0.0f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            p[t] = fast_exp2(p[t] - m_use);
            sum += p[t];
        }
        st[rt].l = st[rt].l * alpha + sum;
        st[rt].m = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int ct = 0; ct < kColTiles; ++ct) st[rt].o[ct] *= alpha;
        }
        uint32_t h[4], lo[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const f32x2_t pp = {p[2 * u], p[2 * u + 1]};
            const bf16x2_t hh = __builtin_convertvector(pp, bf16x2_t);
            h[u] = __builtin_bit_cast(uint32_t, hh);
            if (kHiLo) lo[u] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp - __builtin_convertvector(hh, f32x2_t), bf16x2_t));
        }
        ph[rt] = __builtin_bit_cast(bf16x8_t, u32x4_t{h[0], h[1], h[2], h[3]});
        pl[rt] = __builtin_bit_cast(bf16x8_t, u32x4_t{lo[0], lo[1], lo[2], lo[3]});
    }
    // Value product, fragments kVAhead tile pairs ahead; per pair the hi parts of both tiles (and row
    // tiles) first, then the lo parts, so that no MFMA waits for the one just before it.
#pragma unroll
    for (int c2 = 0; c2 < kColTiles; c2 += 2) {
        if (c2 + 2 * kVAhead < kColTiles) {
            va[c2 + 2 * kVAhead] = load_v(c2 + 2 * kVAhead);
            va[c2 + 2 * kVAhead + 1] = load_v(c2 + 2 * kVAhead + 1);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                st[rt].o[c2 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c2 + u], ph[rt], st[rt].o[c2 + u], 0, 0, 0);
        if (kHiLo) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    st[rt].o[c2 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c2 + u], pl[rt], st[rt].o[c2 + u], 0, 0, 0);
        }
    }
#pragma unroll
    for (int c2 = 0; c2 < kColTiles; c2 += 2) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * RT * (kHiLo ? 2 : 1), 0);
        if (c2 + 2 * kVAhead < kColTiles) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    }
}

// grid.x = pieces, grid.y = groups of 16 * RT * NW rows; block = 64 * NW.  Wave w owns row tiles
// w * RT .. w * RT + RT - 1 of its group.
template <int NW, int RT, bool kHiLo>
__global__ __launch_bounds__(64 * NW) void mla_decode_kernel(MlaParams prm) {
    __shared__ __attribute__((aligned(16))) char lds_c[2 * kLdsBlock];
    // Per wave and tile: the Q chunks of steps kQRegSteps.. (each lane reads back what it wrote); the
    // same bytes stage the output at the end of a segment, when Q is no longer needed.
    __shared__ __attribute__((aligned(16))) char lds_q[NW * RT * kQLdsWave];
    static_assert(kQLdsWave >= kLdsOutPerWave, "output staging must fit the wave's Q area");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = lane >> 4, n = lane & 15;
    const int T = prm.q_len, H = prm.n_heads, rows_total = T * H;
    const Plan pl = make_plan(prm.kv_lens, prm.batch, prm.n_pieces, prm.min_piece_tokens, lane);
    const int per_xcd = (pl.n_pieces + 7) >> 3;
    const int bid = blockIdx.x;
    const int p = (bid & 7) * per_xcd + (bid >> 3);
    const int s0 = piece_bound(pl, p), s1 = piece_bound(pl, p + 1);
    const bool active = (bid >> 3) < per_xcd && p < pl.n_pieces && s0 < s1;

    if (bid == 0 && blockIdx.y == 0 && tid < 64) {
        // For the merge kernel: first partial slot and number of segments of every sequence.
        int run = 0;
        for (int base = 0; base < prm.batch; base += 64) {
            const int i = base + lane;
            const int v = i < prm.batch ? clamp_len(prm.kv_lens[i]) : 0;
            const int incl = wave_incl_scan_i(v, lane) + run;
            if (i < prm.batch) {
                const int first = v > 0 ? piece_of(pl, incl - v) : 0;
                const int n_seg = v > 0 ? piece_of(pl, incl - 1) - first + 1 : 0;
                reinterpret_cast<int2*>(prm.meta)[i] = make_int2(first + i, n_seg);
            }
            run = __shfl(incl, 63, 64);
        }
    }
    if (!active) return;       // the whole workgroup: every wave computed the same plan

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

    // Row n of tile rt of this wave: row index within the sequence's T * H rows.
    const int wave_row0 = blockIdx.y * (16 * RT * NW) + wave * (16 * RT);
    char* q_lds = lds_q + wave * (RT * kQLdsWave) + lane * 16;
    char* out_lds = lds_q + wave * (RT * kQLdsWave);
    const int qk_off = n * kPitch + kb * 16;
    const int pv_off = (4 * kb + (n >> 2)) * kPitch + (n & 3) * 8;
    auto fence = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    int remaining = s1 - s0;
    while (remaining > 0 && b < prm.batch) {
        const int L = __builtin_amdgcn_readfirstlane(clamp_len(prm.kv_lens[b]));
        if (L == 0) { ++b; continue; }
        const int n_tok = (L - j < remaining) ? L - j : remaining;
        const int j0 = j, j1 = j + n_tok;
        const bool whole = (n_tok == L);
        const long slot = (long)p + b;
        const unsigned long long cbytes = (unsigned long long)L * kRowB;
        const uint64_t caddr = (uint64_t)(uintptr_t)prm.c_ptrs[b];
        // raw buffer descriptor: base, no stride, bytes, 32-bit raw format
        const u32x4_t rc = {(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)caddr),
                            (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(caddr >> 32) & 0xffffu)),
                            cbytes > 0xffffffffull ? 0xffffffffu : (uint32_t)cbytes, 0x00020000u};

        block_to_lds<NW>(lds_c, rc, j0, wave, lane);        // block 0 -> buffer 0
        // Q operand: lane (kb, n) holds columns 32 step + 8 kb .. + 7 of row n of each tile.
        bf16x8_t qop[RT][kQRegSteps];
        int lim[RT];
        MlaTile st[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int row = wave_row0 + 16 * rt + n;
            const bool row_ok = row < rows_total;
            const long qrow = (long)b * rows_total + (row_ok ? row : 0);
#pragma unroll
            for (int step = 0; step < kQSteps; ++step) {
                u32x4_t qv = {0u, 0u, 0u, 0u};
                if (row_ok) qv = *reinterpret_cast<const u32x4_t*>(prm.q + qrow * kDqk + (4 * step + kb) * 8);
                if (step < kQRegSteps) qop[rt][step < kQRegSteps ? step : 0] = __builtin_bit_cast(bf16x8_t, qv);
                else *reinterpret_cast<u32x4_t*>(q_lds + rt * kQLdsWave + (step - kQRegSteps) * 1024) = qv;
            }
            const int causal = L - T + (row_ok ? row : 0) / H + 1;
            lim[rt] = causal < j1 ? causal : j1;
#pragma unroll
            for (int ct = 0; ct < kColTiles; ++ct) st[rt].o[ct] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
            st[rt].m = kNegInf;
            st[rt].l = 0.0f;
        }

        // Q is used here, before the loop, so that the wait for its loads sits here as well: a wait
        // inside the loop would also wait for the block loads that were just issued.
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int step = 0; step < kQRegSteps; ++step) asm volatile("" : "+v"(qop[rt][step]));
        fence();                  // the Q chunks in LDS are read back by the lane that wrote them

        const int n_blocks = (j1 - j0 + kMlaKeys - 1) / kMlaKeys;
        for (int blk = 0; blk < n_blocks; ++blk) {
            const char* cur = lds_c + (blk & 1) * kLdsBlock;
            // Every wave waits for its own loads of block blk, then the barrier: block blk is in LDS
            // and everyone is done reading block blk - 1, whose buffer the next loads may overwrite.
            dma_wait();
            __syncthreads();
            if (blk + 1 < n_blocks)
                block_to_lds<NW>(lds_c + ((blk + 1) & 1) * kLdsBlock, rc, j0 + (blk + 1) * kMlaKeys, wave, lane);
            mla_block<RT, kHiLo>(st, cur + qk_off, cur + pv_off, qop, q_lds, prm.scale_log2, j0 + blk * kMlaKeys, lim, kb);
        }
        __syncthreads();          // the next segment's first block reuses buffer 0

        // Store, 128 columns at a time through this wave's LDS so that stores write whole rows.
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const float l = kb_sum(st[rt].l);
            const float sc = whole ? (l > 0.0f ? 1.0f / l : 0.0f) : 1.0f;
            const int tile_row0 = wave_row0 + 16 * rt;
#pragma unroll
            for (int g = 0; g < kDv / 128; ++g) {
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const f32x4_t o = st[rt].o[8 * g + c] * sc;
                    *reinterpret_cast<float4*>(out_lds + n * kOutPitch + (16 * c + 4 * kb) * 4) = make_float4(o[0], o[1], o[2], o[3]);
                }
                fence();
#pragma unroll
                for (int i = 0; i < 8; ++i) {          // 2 rows x 128 fp32 columns per instruction
                    const int rr = tile_row0 + 2 * i + (lane >> 5);
                    if (rr < rows_total) {
                        const float4 w = *reinterpret_cast<const float4*>(out_lds + (2 * i + (lane >> 5)) * kOutPitch +
                                                                          (lane & 31) * 16);
                        if (whole) {
                            uint2 o2;
                            o2.x = pack_bf16(w.x, w.y);
                            o2.y = pack_bf16(w.z, w.w);
                            *reinterpret_cast<uint2*>(prm.out + ((long)b * rows_total + rr) * kDv + g * 128 + (lane & 31) * 4) = o2;
                        } else {
                            *reinterpret_cast<float4*>(prm.part_o + (slot * rows_total + rr) * kDv + g * 128 + (lane & 31) * 4) = w;
                        }
                    }
                }
                fence();
            }
            const int row = tile_row0 + n;
            if (row < rows_total && kb == 0) {
                if (whole) {
                    if (prm.lse) prm.lse[(long)b * rows_total + row] = l > 0.0f ? (st[rt].m + __log2f(l)) * kLn2 : kNegInf;
                } else {
                    reinterpret_cast<float2*>(prm.part_ml)[slot * rows_total + row] = make_float2(st[rt].m, l);
                }
            }
        }
        remaining -= n_tok;
        ++b;
        j = 0;
    }
}

// One wave per output row of 512 columns; lane holds columns 8*lane .. 8*lane+7.
__global__ __launch_bounds__(256) void mla_merge_kernel(MlaParams prm) {
    const int lane = threadIdx.x & 63;
    const long rows_total = (long)prm.q_len * prm.n_heads;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long)prm.batch * rows_total) return;
    const int b = (int)(row / rows_total);
    const long th = row - (long)b * rows_total;
    const int2 fs = reinterpret_cast<const int2*>(prm.meta)[b];
    const int n = fs.y;
    if (n == 1) return;
    uint4* outp = reinterpret_cast<uint4*>(prm.out + row * kDv) + lane;
    if (n == 0) {
        *outp = make_uint4(0u, 0u, 0u, 0u);
        if (prm.lse && lane == 0) prm.lse[row] = kNegInf;
        return;
    }
    const float2* ml = reinterpret_cast<const float2*>(prm.part_ml) + (long)fs.x * rows_total + th;
    const float4* po = reinterpret_cast<const float4*>(prm.part_o + ((long)fs.x * rows_total + th) * kDv) + 2 * lane;
    const long po_stride = rows_total * (kDv / 4);
    float M = kNegInf;
    for (int base = 0; base < n; base += 64)
        if (base + lane < n) M = fmaxf(M, ml[(base + lane) * rows_total].x);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    const float m_use = (M == kNegInf) ? 0.0f : M;
    float l = 0.0f;
    float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int s0 = 0; s0 < n; s0 += 4) {
        float2 a[4];
        float4 o[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u < n ? s0 + u : n - 1;
            a[u] = ml[s * rows_total];
            o[u][0] = po[s * po_stride];
            o[u][1] = po[s * po_stride + 1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = s0 + u < n ? fast_exp2(a[u].x - m_use) : 0.0f;
            l = __builtin_fmaf(a[u].y, w, l);
            acc[0] = __builtin_fmaf(o[u][0].x, w, acc[0]); acc[1] = __builtin_fmaf(o[u][0].y, w, acc[1]);
            acc[2] = __builtin_fmaf(o[u][0].z, w, acc[2]); acc[3] = __builtin_fmaf(o[u][0].w, w, acc[3]);
            acc[4] = __builtin_fmaf(o[u][1].x, w, acc[4]); acc[5] = __builtin_fmaf(o[u][1].y, w, acc[5]);
            acc[6] = __builtin_fmaf(o[u][1].z, w, acc[6]); acc[7] = __builtin_fmaf(o[u][1].w, w, acc[7]);
        }
    }
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    uint4 w;
    w.x = pack_bf16(acc[0] * inv, acc[1] * inv);
    w.y = pack_bf16(acc[2] * inv, acc[3] * inv);
    w.z = pack_bf16(acc[4] * inv, acc[5] * inv);
    w.w = pack_bf16(acc[6] * inv, acc[7] * inv);
    *outp = w;
    if (prm.lse && lane == 0) prm.lse[row] = l > 0.0f ? (M + __log2f(l)) * kLn2 : kNegInf;
}

template <int NW, int RT>
hipError_t launch_mla_cfg(const MlaParams& prm, dim3 grid, hipStream_t stream) {
    if (prm.hi_lo) hipLaunchKernelGGL((mla_decode_kernel<NW, RT, true>), grid, dim3(64 * NW), 0, stream, prm);
    else hipLaunchKernelGGL((mla_decode_kernel<NW, RT, false>), grid, dim3(64 * NW), 0, stream, prm);
    return hipGetLastError();
}

}  // namespace

// Workgroup shape for rows_total = q_len * n_heads query rows per sequence: (waves, 16-row tiles per
// wave).  Automatic: one tile per wave, 8 waves from 65 rows on (two waves per SIMD, 256 registers
// each).  layout 1: at most 4 waves of one tile (64 rows per workgroup); layout 2: 4 waves of two
// tiles from 65 rows on (one wave per SIMD; its accumulators do not fit the register file and spill).
void mla_block_shape(int rows_total, int layout, int* waves, int* tiles_per_wave) {
    const int tiles = (rows_total + 15) / 16;
    *tiles_per_wave = (tiles > 4 && layout == 2) ? 2 : 1;
    *waves = (layout != 1 && layout != 2 && tiles > 4) ? 8 : tiles >= 3 ? 4 : tiles;
}

hipError_t launch_mla_decode(const MlaParams& prm, hipStream_t stream, hipEvent_t* events) {
    const int rows_total = prm.q_len * prm.n_heads;
    int nw = 1, rt = 1;
    mla_block_shape(rows_total, prm.layout, &nw, &rt);
    dim3 grid((prm.n_pieces + 7) / 8 * 8, (rows_total + 16 * rt * nw - 1) / (16 * rt * nw));
    hipError_t e;
    if (events && (e = hipEventRecord(events[0], stream)) != hipSuccess) return e;
    if (rt == 2) e = launch_mla_cfg<4, 2>(prm, grid, stream);
    else if (nw == 8) e = launch_mla_cfg<8, 1>(prm, grid, stream);
    else if (nw == 4) e = launch_mla_cfg<4, 1>(prm, grid, stream);
    else if (nw == 2) e = launch_mla_cfg<2, 1>(prm, grid, stream);
    else e = launch_mla_cfg<1, 1>(prm, grid, stream);
    if (e != hipSuccess) return e;
    if (events && (e = hipEventRecord(events[1], stream)) != hipSuccess) return e;
    const long rows = (long)prm.batch * rows_total;
    hipLaunchKernelGGL(mla_merge_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, prm);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (events && (e = hipEventRecord(events[2], stream)) != hipSuccess) return e;
    return hipSuccess;
}

}  // namespace xattn
