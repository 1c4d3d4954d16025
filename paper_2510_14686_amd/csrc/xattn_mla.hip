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
// owns one piece and up to 128 query rows (row = token * n_heads + head): eight waves, two per SIMD
// (256 registers each), a wave owning one tile of 16 rows whose output accumulators (16 x 512 fp32 =
// 128 registers) stay resident for the whole piece.  Of the tile's Q, 13 of the 18 MFMA steps stay in
// registers (52); each lane parks its chunks of the other 5 in LDS and reads them back per block,
// which leaves the registers for fetching operands ahead of the MFMAs.  (Workgroups of four waves,
// one per SIMD with 512 registers and two tiles each, read every LDS operand half as often: built
// below as mla_block_pp and selectable, but a lone wave per SIMD has nobody to cover its softmax and
// its longer prologue and epilogue, and it measures about 10 % slower.)
// All waves share each 32-key block of the cache through LDS:
//   * the block (32 x 1152 bytes, contiguous in memory) goes from HBM straight into LDS (buffer loads
//     with the LDS destination, 1 KiB per wave instruction, no staging registers), once per
//     workgroup; three LDS buffers, one barrier per block, two blocks in flight during the
//     arithmetic.  In LDS the latent and the rope part of the rows sit in two areas with padded
//     pitches chosen against bank conflicts (the LDS side of such a load is fixed to lane order, so
//     the layout is made through the global address each lane fetches);
//   * S^T = C Q^T: per 16-key tile 18 bf16 MFMA 16x16x32, the A operand (keys) read from LDS;
//   * softmax on the accumulator layout: lane (kb, n) holds, of row n, the keys 4 kb + i of both key
//     tiles, which is exactly the B operand (8 keys per lane) of the next product, so the weights
//     never leave the lane; row maxima cross the four lane groups with lane-swap instructions; the
//     reference maximum of a row moves only when a block exceeds it by more than 2^8, so the 128
//     accumulators are rescaled about once per segment instead of in most blocks;
//   * O^T += C[:, 0:512]^T P^T: bf16 MFMA 16x16x32 over the 32 keys, the A operand (16 value columns x
//     8 keys per lane) fetched with LDS transposing reads.  A weight enters the product as one bf16
//     where it is small against the row's sum, and as hi + lo bf16 parts (two MFMAs, 16 significant
//     bits) where it is not: in the first kExactBlocks blocks of every segment, whose keys' share of
//     the final sum is not yet known, and in any later block that holds a key with at least 1/4 of
//     the row's running sum.  The output is normalised by the sum of the weights as they entered
//     the product.  (Rounding every weight to one bf16 costs nothing on diffuse rows, where the
//     errors average out; where a few keys carry the row, outputs are large enough for bf16 output
//     rounding to use up most of the tolerance, and the weights' own 2^-9 no longer fits beside it.)
// LDS reads are issued a few steps ahead of the MFMAs that use them, pinned with scheduling groups.
// A segment that is not a whole sequence leaves its rows in the workspace as fp16, scaled by the
// row's largest magnitude, with (m, l, lq, 1 / scale) in fp32; the merge kernel combines them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "xattn_device.h"
#include "xattn_kernels.h"

namespace xattn {
namespace {

constexpr int kDqk = 576;                        // key width: latent + rope
constexpr int kDv = 512;                         // value width: the latent part
constexpr int kRowB = kDqk * 2;                  // 1152 bytes per cached token
constexpr int kMlaKeys = 32;                     // keys per LDS block
// LDS image of a block: the first 1024 bytes of each row (the latent part, 64 chunks of 16 bytes) at
// pitch kPitch, the last 128 bytes (the rope part) in a tail area at pitch kTailPitch.  Both pitches are
// 2 * odd chunks modulo 16: measured, that serves the operand reads below without bank conflicts (an
// odd pitch halves their rate).
constexpr int kPitch = 1024 + 32;                // 1056
constexpr int kTailPitch = 128 + 32;             // 160
constexpr int kTailRowsPerLoad = 6;              // one wave-wide load fills the tails of 6 rows (60 lanes)
constexpr int kTailLoads = (kMlaKeys + kTailRowsPerLoad - 1) / kTailRowsPerLoad;          // 6
constexpr int kTailOff = kMlaKeys * kPitch;      // 33792: start of the tail area
constexpr int kLdsBlock = kTailOff + (kTailLoads - 1) * kTailRowsPerLoad * kTailPitch + 1024;   // 39616
constexpr int kDmaPerBlock = kMlaKeys + kTailLoads;   // 38 wave-wide loads of 64 x 16 bytes
constexpr int kTileB = 16 * kPitch;              // from key tile 0 to key tile 1 of a block
constexpr int kTailTileB = 16 * kTailPitch;
constexpr int kMainSteps = 1024 / 64;            // MFMA steps 0..15 read the latent part, 16..17 the tail
constexpr int kQSteps = kDqk / 32;               // 18 MFMA steps of 32 columns
constexpr int kQRegSteps = 13;                   // Q columns 0 .. 32 * 13 - 1 stay in registers, the rest of Q in LDS
constexpr int kQLdsWave = (kQSteps - kQRegSteps) * 1024;   // per 16-row tile: one 16-byte chunk per lane and step
constexpr int kQAhead = 2;                       // key fragments in flight ahead of the MFMAs, in steps
constexpr int kVAhead = 2;                       // value fragments in flight ahead of the MFMAs, in tile pairs
constexpr int kColTiles = kDv / 16;              // 32 tiles of 16 value columns
constexpr int kStagePitch = (kDv / 2) * 2 + 16;  // epilogue: 16 rows x 256 16-bit columns at a time per wave, padded rows
constexpr int kStageWave = 16 * kStagePitch;     // 8448 bytes
// A segment's fixed work (first block's latency, Q, output staging and stores; measured: workgroups
// with two segments finish 13 us later than their token count says) in units of one token's share of
// the block loop (2.3 us per 32 tokens).
constexpr int kMlaSegCost = 192;
constexpr float kLazyLog2 = 8.0f;                // slack of the softmax reference maximum, in powers of two
// Precision of the softmax weights in the value product (see the header comment).
constexpr int kLoNever = 0;                      // one bf16 per weight everywhere
constexpr int kLoAlways = 1;                     // hi + lo bf16 parts everywhere
constexpr int kLoDynamic = 2;                    // hi + lo parts only in blocks with a dominant key
constexpr int kExactBlocks = 4;                  // default mode: the first blocks of a segment run as kLoAlways
constexpr float kDominantShare = 4.0f;           // a key is dominant from 1 / 4 of the row's running sum
// Eight waves: the first wave of each SIMD issues its loads of the block after next behind the block's
// arithmetic, the second one ahead of it, so the two run a fraction of a phase apart and one's vector
// work falls on the other's MFMAs more often (measured: 3-4 % of the kernel).
constexpr bool kSkewWaves = true;
constexpr int kStages = 3;                       // LDS block buffers: two blocks in flight behind the one in use

typedef short s16x4v_t __attribute__((ext_vector_type(4)));

// Running state of one 16-row tile.  Lane (kb, n) holds row n.
struct MlaTile {
    f32x4_t o[kColTiles];      // o[ct][i]: column 16 ct + 4 kb + i
    float m, l;                // reference maximum (log2 domain) and the running sum over all keys of the row
    float lq;                  // this lane's share of the sum over the weights as they entered the value product
};

template <typename F, int... I>
__device__ __forceinline__ void static_for(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>()), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) { static_for(f, std::make_integer_sequence<int, N>()); }

// The loads are written as assembly so that the compiler does not order them against LDS reads: it
// cannot tell the two halves of the double buffer apart and would wait for every outstanding load
// before each read.  dma_wait() before the workgroup barrier is what makes a block visible.
__device__ __forceinline__ void dma16(u32x4_t rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
    // m0 carries the LDS address of the load.  The compiler keeps values of its own in m0 (lane
    // indices, LDS-DMA bases) and does not accept m0 in a clobber list, so the statement saves and
    // restores it; the load has read m0 by the time it is issued.
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 1\n\tbuffer_load_dwordx4 %2, %3, %4 offen nt lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
// Waits until at most n of this wave's loads are outstanding (they complete in order): n = the number
// of loads of the newest block leaves the block before it complete.
__device__ __forceinline__ void dma_wait(int n) {
    switch (n) {           // n is wave-uniform; the instruction takes an immediate
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
        case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
        case 9: asm volatile("s_waitcnt vmcnt(9)" ::: "memory"); break;
        case 10: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
        case 19: asm volatile("s_waitcnt vmcnt(19)" ::: "memory"); break;
        case 38: asm volatile("s_waitcnt vmcnt(38)" ::: "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
}

// This wave's share of the loads of one 32-key block into LDS.  A load fills 1024 consecutive LDS
// bytes in lane order.  Load r < 32: the latent part of row r, lane l fetching chunk l.  Load 32 + p:
// the tails of rows 6 p .. 6 p + 5, lane l = 10 i + c fetching chunk 64 + c of row 6 p + i (c < 8;
// lanes with c >= 8, l >= 60 or a row past the block fetch nothing).  Bytes past the sequence's end
// read as zero.  The per-lane parts of the addresses (dma.main_off, dma.tail_off) do not depend on
// the load, the rest is scalar.
struct DmaLane {
    uint32_t main_off, tail_off;
    int tail_row;                // 6 p + tail_row is the lane's row in a tail load; 64 for lanes that fetch nothing
};
__device__ __forceinline__ DmaLane dma_lane(int lane) {
    DmaLane d;
    const int i = lane / 10, c = lane - 10 * i;
    d.main_off = (uint32_t)lane * 16;
    d.tail_off = (uint32_t)(i * kRowB + 1024 + c * 16);
    d.tail_row = (c < 8 && i < kTailRowsPerLoad) ? i : 64;
    return d;
}
// Load q (of this wave's (kDmaPerBlock + NW - 1) / NW) of a block.
template <int NW>
__device__ __forceinline__ void block_load(char* lds_block, u32x4_t rc, int j_block, int wave, const DmaLane& dma, int q) {
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_block;
    const int g = wave + q * NW;             // wave-uniform
    if (g < kMlaKeys) {
        dma16(rc, lds0 + g * kPitch, dma.main_off, (uint32_t)(j_block + g) * kRowB);
    } else if (g < kDmaPerBlock) {
        const int p = g - kMlaKeys;
        if (p * kTailRowsPerLoad + dma.tail_row < kMlaKeys)
            dma16(rc, lds0 + kTailOff + p * (kTailRowsPerLoad * kTailPitch), dma.tail_off,
                  (uint32_t)(j_block + p * kTailRowsPerLoad) * kRowB);
    }
}
// The same for workgroups of four or eight waves with as few scalar instructions as possible: which
// loads fill the tail area is then known from q alone, and the tail loads run with all lanes.  The
// lanes that "fetch nothing" above then fetch bytes that do no harm: chunks 72 and 73 of a row (the
// start of the next row) land in the padding of the tail pitch, lanes 60-63 fetch what the next tail
// load puts in the same place, and rows past the block land behind the tail area, inside the buffer
// (kLdsBlock counts the last load in full).  Bytes past the sequence read as zero.
struct DmaWave {
    uint32_t lds_main, lds_tail;       // LDS address of this wave's first main / tail load
    uint32_t mem_main, mem_tail;       // byte offsets of the same in the sequence's cache
};
__device__ __forceinline__ DmaWave dma_wave_for(char* lds_block, int j_block, int wave) {
    DmaWave d;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_block;
    d.lds_main = lds0 + wave * kPitch;
    d.lds_tail = lds0 + kTailOff + wave * (kTailRowsPerLoad * kTailPitch);
    d.mem_main = (uint32_t)(j_block + wave) * kRowB;
    d.mem_tail = (uint32_t)(j_block + wave * kTailRowsPerLoad) * kRowB;
    return d;
}
template <int NW, int Q>
__device__ __forceinline__ void block_load_static(const DmaWave& d, u32x4_t rc, const DmaLane& dma, int wave) {
    static_assert(NW == 4 || NW == 8, "the main rows must divide among the waves");
    constexpr int kMainLoads = kMlaKeys / NW;        // loads 0 .. kMainLoads - 1 of a wave are rows wave + NW q
    if constexpr (Q < kMainLoads) {
        dma16(rc, d.lds_main + Q * NW * kPitch, dma.main_off, d.mem_main + Q * NW * kRowB);
    } else if constexpr (NW * (Q - kMainLoads + 1) <= kTailLoads) {    // tail loads wave + NW (Q - kMainLoads), all waves
        dma16(rc, d.lds_tail + (Q - kMainLoads) * NW * (kTailRowsPerLoad * kTailPitch), dma.tail_off,
              d.mem_tail + (Q - kMainLoads) * NW * kTailRowsPerLoad * kRowB);
    } else if constexpr (NW * (Q - kMainLoads) < kTailLoads) {         // the last ones: the first waves only
        if (wave + NW * (Q - kMainLoads) < kTailLoads)
            dma16(rc, d.lds_tail + (Q - kMainLoads) * NW * (kTailRowsPerLoad * kTailPitch), dma.tail_off,
                  d.mem_tail + (Q - kMainLoads) * NW * kTailRowsPerLoad * kRowB);
    }
}
template <int NW>
__device__ __forceinline__ void block_to_lds(char* lds_block, u32x4_t rc, int j_block, int wave, const DmaLane& dma) {
    if constexpr (NW == 4 || NW == 8) {
        const DmaWave d = dma_wave_for(lds_block, j_block, wave);
        static_for<(kDmaPerBlock + NW - 1) / NW>([&](auto q_c) { block_load_static<NW, decltype(q_c)::value>(d, rc, dma, wave); });
    } else {
#pragma unroll
        for (int q = 0; q < (kDmaPerBlock + NW - 1) / NW; ++q) block_load<NW>(lds_block, rc, j_block, wave, dma, q);
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

// Two values rounded to fp16 (nearest even) and packed.
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}

// Two values rounded to bf16 (nearest even) and packed: the conversion instruction.
__device__ __forceinline__ uint32_t cvt_bf16(float a, float b) {
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
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
// used for all RT tiles.  kLo: how the softmax weights go into the value product (kLoNever, kLoAlways,
// kLoDynamic).
//   qk_base = block + n * kPitch + kb * 16                     (key row n of a tile, chunk kb)
//   qt_base = block + kTailOff + n * kTailPitch + kb * 16      (the same for the rope part)
//   pv_base = block + (4 kb + n / 4) * kPitch + (n % 4) * 8    (transposing read, see below)
template <int RT, int kLo>
__device__ __forceinline__ void mla_block(MlaTile (&st)[RT], const char* qk_base, const char* qt_base, const char* pv_base,
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
        if (step < kMainSteps) {
            ka[step][0] = *reinterpret_cast<const bf16x8_t*>(qk_base + step * 64);
            ka[step][1] = *reinterpret_cast<const bf16x8_t*>(qk_base + kTileB + step * 64);
        } else {
            ka[step][0] = *reinterpret_cast<const bf16x8_t*>(qt_base + (step - kMainSteps) * 64);
            ka[step][1] = *reinterpret_cast<const bf16x8_t*>(qt_base + kTailTileB + (step - kMainSteps) * 64);
        }
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
    bool with_lo[RT];                // the tile's weights go in as hi + lo parts in this block
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        // Keys at or past lim[rt] (the end of the segment, or the causal limit of the row) count as
        // -inf; only the blocks that reach that far pay for the comparison.  scale_log2 > 0, so the
        // maximum is taken before scaling, and one fused multiply-add scales and shifts.
        float p[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) p[t] = s[rt][t >> 2][t & 3];
        if (__builtin_amdgcn_ballot_w64(j_block + kMlaKeys > lim[rt]) != 0) {
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int key = j_block + 16 * (t >> 2) + 4 * kb + (t & 3);
                p[t] = key < lim[rt] ? p[t] : kNegInf;
            }
        }
        float mx = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])), fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
        mx = kb_max(mx) * scale_log2;
        // The reference maximum follows the row's maximum lazily: it moves only when a block exceeds
        // it by more than kLazyLog2, so weights reach 2^kLazyLog2 at most (harmless in fp32 sums and in
        // bf16's relative precision) and the rescaling of the 128 accumulators below, which would
        // otherwise run in most blocks (some row of the tile sees a new maximum), runs about once.
        const float m_new = mx > st[rt].m + kLazyLog2 ? mx : st[rt].m;
        const float m_use = (m_new == kNegInf) ? 0.0f : m_new;
        const float alpha = fast_exp2(st[rt].m - m_use);
        float sum = 0.0f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            p[t] = fast_exp2(__builtin_fmaf(p[t], scale_log2, -m_use));
            sum += p[t];
        }
        st[rt].l = st[rt].l * alpha + kb_sum(sum);
        st[rt].m = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int ct = 0; ct < kColTiles; ++ct) st[rt].o[ct] *= alpha;
        }
        // Dominant key: the block's largest weight of a row against the row's sum so far (this block
        // included), which is at most the sum the output is divided by in the end.  The tile adds the
        // lo parts if any of its rows has one.
        with_lo[rt] = kLo == kLoAlways ||
                      (kLo == kLoDynamic && __builtin_amdgcn_ballot_w64(fast_exp2(mx - m_use) * kDominantShare >= st[rt].l) != 0);
        // Where a weight goes in as one bf16 the output is normalised by the sum of the ROUNDED weights:
        // a softmax over slightly perturbed scores (relative weight error 2^-9, the same for equal
        // weights, none for a lone key) instead of rounded weights over an exact sum.
        uint32_t h[4], lo[4] = {0u, 0u, 0u, 0u};
        float sum_q = 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const f32x2_t pp = {p[2 * u], p[2 * u + 1]};
            const bf16x2_t hh = __builtin_convertvector(pp, bf16x2_t);
            const f32x2_t back = __builtin_convertvector(hh, f32x2_t);
            h[u] = __builtin_bit_cast(uint32_t, hh);
            sum_q += back[0] + back[1];
            p[2 * u] -= back[0];
            p[2 * u + 1] -= back[1];
        }
        if (with_lo[rt]) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const f32x2_t rest = {p[2 * u], p[2 * u + 1]};
                lo[u] = __builtin_bit_cast(uint32_t, __builtin_convertvector(rest, bf16x2_t));
            }
        }
        st[rt].lq = st[rt].lq * alpha + (with_lo[rt] ? sum : sum_q);
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
        if (kLo == kLoAlways) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    st[rt].o[c2 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c2 + u], pl[rt], st[rt].o[c2 + u], 0, 0, 0);
        }
    }
#pragma unroll
    for (int c2 = 0; c2 < kColTiles; c2 += 2) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * RT * (kLo == kLoAlways ? 2 : 1), 0);
        if (c2 + 2 * kVAhead < kColTiles) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    }
    if (kLo == kLoDynamic) {
        // The rare block with a dominant key: a second pass over the value fragments with the lo parts.
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            if (!with_lo[rt]) continue;
#pragma unroll
            for (int ct = 0; ct < kColTiles; ++ct)      // fully unrolled: the accumulators are registers
                st[rt].o[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(load_v(ct), pl[rt], st[rt].o[ct], 0, 0, 0);
        }
    }
}

// ----------------------------------------------------------------------- two row tiles per wave
// One wave per SIMD with 512 registers: the output accumulators of two 16-row tiles (256) in the
// accumulation registers, everything else in the ordinary ones.  Every operand fragment read from LDS
// feeds the MFMAs of both tiles where the order of the work allows it: with one tile per wave each
// MFMA needs a fragment of its own, 1 KiB per 16 cycles and SIMD, which is all the LDS delivers.
// A block runs as scores of both tiles (every key fragment feeds two MFMAs), the two softmaxes slice
// by slice in turn (two independent chains of dependent instructions), values of both tiles (every
// value fragment feeds two MFMAs).
// The MFMAs are assembly statements: their accumulators can then be named (scores in ordinary
// registers, outputs in accumulation registers; through the builtin the compiler puts every MFMA
// result into the accumulation registers, which the outputs fill alone), and such statements keep
// their order among themselves and against memory operations, so LDS reads stay where they are
// written, a fixed number of MFMAs ahead of their use.  Vector instructions do move across them;
// the softmax is therefore cut into slices of a few instructions whose results pass through an empty
// statement of the same kind (pin): a slice cannot start before the pin its inputs came through nor
// end after its own.
//
// What the compiler cannot see of an MFMA inside a statement: a vector instruction may read a result
// register only once the MFMA has left the pipe, so a few idle cycles (mfma_drain) stand between the
// last score MFMA and the softmax, and between the last value MFMA of a segment and the epilogue; a
// rescaling reads accumulators a phase or more after the MFMA that wrote them.
constexpr int kFrags = 2 * kQSteps;              // key fragments per block, ordered (step, key tile)
constexpr int kPpKAhead = 6;                     // key fragments in flight ahead of their MFMAs
constexpr int kPpVAhead = 6;                     // value fragments (two reads each) in flight ahead of theirs
constexpr int kPpDmaEvery = 3;                   // key fragments between two loads of the block after next
constexpr int kSoftSlices = 27;

__device__ __forceinline__ void mfma_first_v(f32x4_t& acc, bf16x8_t a, bf16x8_t b) {      // acc = a b
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_v(f32x4_t& acc, bf16x8_t a, bf16x8_t b) {            // acc += a b
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_a(f32x4_t& acc, bf16x8_t a, bf16x8_t b) {            // the same on accumulation registers
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// Between the last MFMA statements and the first vector instructions that read their results: the 16
// cycles an MFMA spends in the pipe and the write-back behind them, with a margin.  The results pass
// through the statement, so their readers stay behind it.
__device__ __forceinline__ void mfma_drain(f32x4_t& a, f32x4_t& b, f32x4_t& c, f32x4_t& d) {
    asm volatile("s_nop 15\n\ts_nop 7" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
__device__ __forceinline__ void mfma_drain_acc(f32x4_t& a, f32x4_t& b, f32x4_t& c, f32x4_t& d) {
    asm volatile("s_nop 15\n\ts_nop 7" : "+a"(a), "+a"(b), "+a"(c), "+a"(d));
}
template <typename A> __device__ __forceinline__ void pin(A& a) { asm volatile("" : "+v"(a)); }
template <typename A, typename B> __device__ __forceinline__ void pin(A& a, B& b) { asm volatile("" : "+v"(a), "+v"(b)); }
template <typename A, typename B, typename C> __device__ __forceinline__ void pin(A& a, B& b, C& c) {
    asm volatile("" : "+v"(a), "+v"(b), "+v"(c));
}
// max(a, b) of two scores (finite or -inf, no NaNs) as one instruction, the median of (a, b, largest
// finite float): fmaxf() first quiets each operand it cannot prove to be the result of arithmetic
// (matrix results, swapped lanes), an instruction apiece.
__device__ __forceinline__ float max_num(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, 0x1.fffffep+127f); }

// o *= alpha for a tile whose accumulators live in the accumulation registers: each passes through
// ordinary registers, one after the other (the pins keep the compiler from fetching all 128 first,
// which would evict everything else that lives in ordinary registers).
__device__ __forceinline__ void rescale_acc(MlaTile& st, float alpha) {
#pragma unroll
    for (int ct = 0; ct < kColTiles; ++ct) {
        if (ct > 0) asm volatile("" : "+a"(st.o[ct]), "+a"(st.o[ct - 1]));
        st.o[ct] *= alpha;
    }
}

// The softmax of one row tile over one block, between slices.
struct SoftRow {
    float p[8];                      // scores, then weights: keys 16 kt + 4 kb + i at index 4 kt + i
    float t0, t1, t2, t3, sw0, sw1;
    float mx, m_new, m_use, alpha, sum, sum_q, dom;
    uint32_t h[4], lo[4];            // the weights as bf16 pairs, and what the rounding left
    bool with_lo;
};
// Slice K of kSoftSlices.  s: the tile's scores (per key tile); st: its running state.
template <int K, int kLo, bool kMasked, bool kPinned>
__device__ __forceinline__ void soft_slice(SoftRow& r, MlaTile& st, const f32x4_t (&s)[2], float scale_log2, int j_block,
                                           int lim, int kb) {
    if constexpr (K == 0) {
#pragma unroll
        for (int t = 0; t < 8; ++t) r.p[t] = s[t >> 2][t & 3];
        if (kMasked) {               // keys at or past lim (end of the segment, causal limit of the row) count as -inf
#pragma unroll
            for (int t = 0; t < 8; ++t) r.p[t] = (j_block + 16 * (t >> 2) + 4 * kb + (t & 3) < lim) ? r.p[t] : kNegInf;
        }
        r.t0 = max_num(r.p[0], r.p[1]);
        r.t1 = max_num(r.p[2], r.p[3]);
        if (kPinned) pin(r.t0, r.t1);
    } else if constexpr (K == 1) {
        r.t2 = max_num(r.p[4], r.p[5]);
        r.t3 = max_num(r.p[6], r.p[7]);
        if (kPinned) pin(r.t2, r.t3);
    } else if constexpr (K == 2) {
        r.t0 = max_num(r.t0, r.t1);
        r.t2 = max_num(r.t2, r.t3);
        if (kPinned) pin(r.t0, r.t2);
    } else if constexpr (K == 3) {
        swap16(max_num(r.t0, r.t2), r.sw0, r.sw1);
        if (kPinned) pin(r.sw0, r.sw1);
    } else if constexpr (K == 4) {
        swap32(max_num(r.sw0, r.sw1), r.sw0, r.sw1);
        if (kPinned) pin(r.sw0, r.sw1);
    } else if constexpr (K == 5) {   // the reference maximum follows lazily, see mla_block
        r.mx = max_num(r.sw0, r.sw1) * scale_log2;
        r.m_new = r.mx > st.m + kLazyLog2 ? r.mx : st.m;
        if (kPinned) pin(r.mx, r.m_new);
    } else if constexpr (K == 6) {
        r.m_use = (r.m_new == kNegInf) ? 0.0f : r.m_new;
        r.alpha = fast_exp2(st.m - r.m_use);
        if (kPinned) pin(r.m_use, r.alpha);
    } else if constexpr (K >= 7 && K <= 14) {
        r.p[K - 7] = fast_exp2(__builtin_fmaf(r.p[K - 7], scale_log2, -r.m_use));
        if (kPinned) pin(r.p[K - 7], r.m_use);
    } else if constexpr (K == 15) {
        r.t0 = r.p[0] + r.p[1];
        r.t1 = r.p[2] + r.p[3];
        if (kPinned) pin(r.t0, r.t1);
    } else if constexpr (K == 16) {
        r.t2 = r.p[4] + r.p[5];
        r.t3 = r.p[6] + r.p[7];
        if (kPinned) pin(r.t2, r.t3);
    } else if constexpr (K == 17) {
        r.sum = (r.t0 + r.t1) + (r.t2 + r.t3);
        swap16(r.sum, r.sw0, r.sw1);
        if (kPinned) pin(r.sum, r.sw0, r.sw1);
    } else if constexpr (K == 18) {
        swap32(r.sw0 + r.sw1, r.sw0, r.sw1);
        if (kPinned) pin(r.sw0, r.sw1);
    } else if constexpr (K == 19) {
        st.l = st.l * r.alpha + (r.sw0 + r.sw1);
        st.m = r.m_new;
        if (kPinned) pin(st.l, st.m);
    } else if constexpr (K == 20) {  // a key with at least 1 / kDominantShare of the row's sum so far
        if (kLo == kLoDynamic) {
            r.dom = fast_exp2(r.mx - r.m_use) * kDominantShare >= st.l ? 1.0f : 0.0f;
            if (kPinned) pin(r.dom);
        }
    } else if constexpr (K == 21 || K == 22) {
#pragma unroll
        for (int u = 2 * (K - 21); u < 2 * (K - 21) + 2; ++u) {
            const f32x2_t pp = {r.p[2 * u], r.p[2 * u + 1]};
            r.h[u] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, bf16x2_t));
        }
        if (kPinned) pin(r.h[2 * (K - 21)], r.h[2 * (K - 21) + 1]);
    } else if constexpr (K == 23) {  // the sum of the rounded weights: each pair times (1, 1), added in fp32
        r.sum_q = 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) r.sum_q = dot2_bf16(r.h[u], 0x3f803f80u, r.sum_q);
        if (kPinned) pin(r.sum_q);
    } else if constexpr (K == 24 || K == 25) {
        if (kLo != kLoNever) {
#pragma unroll
            for (int u = 2 * (K - 24); u < 2 * (K - 24) + 2; ++u) {
                const f32x2_t pp = {r.p[2 * u], r.p[2 * u + 1]};
                const f32x2_t back = __builtin_convertvector(__builtin_bit_cast(bf16x2_t, r.h[u]), f32x2_t);
                r.lo[u] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp - back, bf16x2_t));
            }
            if (kPinned) pin(r.lo[2 * (K - 24)], r.lo[2 * (K - 24) + 1]);
        }
    } else if constexpr (K == 26) {
        r.with_lo = kLo == kLoAlways || (kLo == kLoDynamic && __builtin_amdgcn_ballot_w64(r.dom != 0.0f) != 0);
        st.lq = st.lq * r.alpha + (r.with_lo ? r.sum : r.sum_q);
        if (kPinned) pin(st.lq);
    }
}

// issue(q): the caller's load q of the block after next (a wave-wide load into LDS); they are spread
// over the score phase, one every kPpDmaEvery fragments: issued together behind the barrier they queue
// up in front of the memory pipeline and hold every wave until the last one is accepted.
template <int kLo, bool kMasked, typename Issue>
__device__ __forceinline__ void mla_block_pp(MlaTile (&st)[2], const char* qk_base, const char* qt_base, const char* pv_base,
                                             const bf16x8_t (&qop)[2][kQRegSteps], const char* q_lds, float scale_log2,
                                             int j_block, const int (&lim)[2], int kb, Issue issue) {
    f32x4_t s[2][2];                 // [row tile][key tile]
    bf16x8_t ka[kFrags], ql[2][kQSteps - kQRegSteps], va[kColTiles];
    SoftRow sr[2];
    // Key fragment F = (step, key tile); with key tile 0 of a step from kQRegSteps on come the lane's
    // parked chunks of Q for both row tiles.
    auto load_k = [&](auto f_c) {
        constexpr int F = decltype(f_c)::value, step = F >> 1, kt = F & 1;
        if constexpr (step < kMainSteps) ka[F] = *reinterpret_cast<const bf16x8_t*>(qk_base + kt * kTileB + step * 64);
        else ka[F] = *reinterpret_cast<const bf16x8_t*>(qt_base + kt * kTailTileB + (step - kMainSteps) * 64);
        if constexpr (kt == 0 && step >= kQRegSteps) {
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
                ql[rt][step - kQRegSteps] =
                    *reinterpret_cast<const bf16x8_t*>(q_lds + rt * kQLdsWave + (step - kQRegSteps) * 1024);
        }
    };
    // Value fragment of column tile ct: see mla_block for the layout.
    auto read_v = [&](int ct) {
        const s16x4v_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4v_t*)(pv_base + ct * 32));
        const s16x4v_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4v_t*)(pv_base + kTileB + ct * 32));
        const u32x2_t w0 = __builtin_bit_cast(u32x2_t, v0), w1 = __builtin_bit_cast(u32x2_t, v1);
        return __builtin_bit_cast(bf16x8_t, u32x4_t{w0.x, w0.y, w1.x, w1.y});
    };
    auto load_v = [&](auto i_c) { va[decltype(i_c)::value] = read_v(decltype(i_c)::value); };

    // Scores of both tiles: every key fragment feeds two MFMAs (four independent accumulators).
    static_for<kPpKAhead>(load_k);
    static_for<kFrags>([&](auto f_c) {
        constexpr int F = decltype(f_c)::value, step = F >> 1, kt = F & 1;
        if constexpr (F + kPpKAhead < kFrags) load_k(std::integral_constant<int, F + kPpKAhead>());
        else if constexpr (F + kPpKAhead - kFrags < kPpVAhead) load_v(std::integral_constant<int, F + kPpKAhead - kFrags>());
        if constexpr (F % kPpDmaEvery == kPpDmaEvery - 1) issue(std::integral_constant<int, F / kPpDmaEvery>());
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            bf16x8_t qv;
            if constexpr (step < kQRegSteps) qv = qop[rt][step];
            else qv = ql[rt][step - kQRegSteps];
            if constexpr (step == 0) mfma_first_v(s[rt][kt], ka[F], qv);
            else mfma_v(s[rt][kt], ka[F], qv);
        }
    });
    static_assert(kPpVAhead <= kPpKAhead, "the first value fragments are fetched in the last score steps");
    mfma_drain(s[0][0], s[0][1], s[1][0], s[1][1]);
    // Softmax of both tiles, slice by slice in turn: two independent chains of dependent instructions.
    static_for<kSoftSlices>([&](auto k_c) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
            soft_slice<decltype(k_c)::value, kLo, kMasked, false>(sr[rt], st[rt], s[rt], scale_log2, j_block, lim[rt], kb);
    });
    bf16x8_t ph[2], pl[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        if (__builtin_amdgcn_ballot_w64(sr[rt].alpha != 1.0f) != 0) rescale_acc(st[rt], sr[rt].alpha);       // about once per segment
        ph[rt] = __builtin_bit_cast(bf16x8_t, u32x4_t{sr[rt].h[0], sr[rt].h[1], sr[rt].h[2], sr[rt].h[3]});
        if (kLo != kLoNever) pl[rt] = __builtin_bit_cast(bf16x8_t, u32x4_t{sr[rt].lo[0], sr[rt].lo[1], sr[rt].lo[2], sr[rt].lo[3]});
    }
    // Values of both tiles: every value fragment feeds two MFMAs (four with the lo parts).
    static_for<kColTiles>([&](auto i_c) {
        constexpr int I = decltype(i_c)::value;
        if constexpr (I + kPpVAhead < kColTiles) load_v(std::integral_constant<int, I + kPpVAhead>());
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) mfma_a(st[rt].o[I], va[I], ph[rt]);
        if (kLo == kLoAlways) {
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) mfma_a(st[rt].o[I], va[I], pl[rt]);
        }
    });
    if (kLo == kLoDynamic) {
        // The rare block with a dominant key: a second pass over the value fragments with the lo parts.
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            if (!sr[rt].with_lo) continue;
#pragma unroll
            for (int ct = 0; ct < kColTiles; ++ct) mfma_a(st[rt].o[ct], read_v(ct), pl[rt]);
        }
    }
}

// kMode: 0 = default (hi + lo weights in the first kExactBlocks blocks of a segment and wherever a key
// dominates its row), 1 = hi + lo weights everywhere, 2 = one bf16 per weight everywhere.
template <int NW, int RT, int kMode>
__global__ __launch_bounds__(64 * NW) void mla_decode_kernel(MlaParams prm) {
    __shared__ __attribute__((aligned(16))) char lds_c[kStages * kLdsBlock];
    // Per wave and tile: the Q chunks of steps kQRegSteps.. (each lane reads back what it wrote).
    __shared__ __attribute__((aligned(16))) char lds_q[NW * RT * kQLdsWave];
    static_assert(NW * kStageWave <= kStages * kLdsBlock, "output staging must fit the block buffers");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = lane >> 4, n = lane & 15;
    const int T = prm.q_len, H = prm.n_heads, rows_total = T * H;
    SeqWindow win;
    const WavePlan wp = wave_plan(prm.kv_lens, prm.c_ptrs, nullptr, prm.batch, prm.n_pieces, prm.min_piece_tokens, kMlaSegCost,
                                  prm.xcd_skew, lane, &win);
    const Plan& pl = wp.pl;
    const int per_xcd = (pl.n_pieces + 7) >> 3;
    // Workgroup ids go round-robin over the 8 XCDs.  Of an XCD's workgroups, consecutive ones are the
    // row groups of one piece: they run at the same time on the same XCD and share its L2, so the
    // piece's cache rows come from HBM once.
    const int bid = blockIdx.x;
    const int n_groups = (rows_total + 16 * RT * NW - 1) / (16 * RT * NW);
    const int slot_in_xcd = bid >> 3;
    const int row_group = slot_in_xcd % n_groups;
    const int p = (bid & 7) * per_xcd + slot_in_xcd / n_groups;
    const int s0 = piece_bound(pl, p), s1 = piece_bound(pl, p + 1);
    const bool active = slot_in_xcd / n_groups < per_xcd && p < pl.n_pieces && s0 < s1;

    if (tid < 64) {
        // For the merge kernel: first partial slot and number of segments of every sequence, 64
        // sequences per wave, the groups of 64 dealt out over the workgroups.
        for (int g = bid; 64 * g < prm.batch; g += gridDim.x) wave_write_meta(wp, prm.kv_lens, prm.batch, g, lane, prm.meta);
    }
    if (!active) return;       // the whole workgroup: every wave computed the same plan

    Walk walk;
    wave_locate(wp, prm.kv_lens, prm.c_ptrs, nullptr, prm.batch, s0, lane, &win, walk.b, walk.j);
    walk.remaining = s1 - s0;

    // Row n of tile rt of this wave: row index within the sequence's T * H rows.
    const int wave_row0 = row_group * (16 * RT * NW) + wave * (16 * RT);
    char* q_lds = lds_q + wave * (RT * kQLdsWave) + lane * 16;
    char* stage = lds_c + wave * kStageWave;
    const DmaLane dma = dma_lane(lane);
    const int my_loads = (kDmaPerBlock - wave + NW - 1) / NW;      // block loads this wave issues per block
    const int qk_off = n * kPitch + kb * 16;
    const int qt_off = kTailOff + n * kTailPitch + kb * 16;
    const int pv_off = (4 * kb + (n >> 2)) * kPitch + (n & 3) * 8;
    auto fence = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    PieceSeg ps;
    while (next_segment(walk, prm.batch, pl.seg_cost,
                        [&](int bb) { return window_len(win, prm.kv_lens, bb); }, ps)) {
        const int b = ps.b, L = ps.L, j0 = ps.j0, j1 = ps.j1;
        const bool whole = ps.whole;
        const long slot = (long)p + b;
        const unsigned long long cbytes = (unsigned long long)L * kRowB;
        const uint64_t caddr = (uint64_t)(uintptr_t)window_ptr(win, win.k, prm.c_ptrs, b);
        // raw buffer descriptor: base, no stride, bytes, 32-bit raw format
        const u32x4_t rc = {(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)caddr),
                            (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(caddr >> 32) & 0xffffu)),
                            cbytes > 0xffffffffull ? 0xffffffffu : (uint32_t)cbytes, 0x00020000u};

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
            st[rt].lq = 0.0f;
        }

        // Block 0 -> buffer 0, behind the Q loads: those do not need the sequence's base address, whose
        // own load they now cover.
        block_to_lds<NW>(lds_c, rc, j0, wave, dma);
        // Q is used here, before the loop, so that the wait for its loads sits here as well: a wait
        // inside the loop would also wait for the block loads that were just issued.
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int step = 0; step < kQRegSteps; ++step) asm volatile("" : "+v"(qop[rt][step]));
        fence();                  // the Q chunks in LDS are read back by the lane that wrote them

        const int n_blocks = (j1 - j0 + kMlaKeys - 1) / kMlaKeys;
        if constexpr (RT == 2) {
            // block 1 -> buffer 1; with two tiles per wave every block has its loads, past the segment's
            // end against an empty buffer (see the block loop), so that the waits need no case.
            u32x4_t rc1 = rc;
            if (n_blocks <= 1) rc1[2] = 0u;
            block_to_lds<NW>(lds_c + kLdsBlock, rc1, j0 + kMlaKeys, wave, dma);
        } else {
            if (n_blocks > 1) block_to_lds<NW>(lds_c + kLdsBlock, rc, j0 + kMlaKeys, wave, dma);   // block 1 -> buffer 1
        }
        int cur_buf = 0, next_buf = 2;         // block blk sits in buffer blk % 3, block blk + 2 goes to next_buf
        // One block: every wave waits for its own loads of block blk (those of block blk + 1 may stay
        // in flight), then the barrier: block blk is in LDS and everyone is done reading block
        // blk - 1, whose buffer the loads of block blk + 2 may overwrite.
        auto step = [&](int blk, auto lo_mode, auto masked) {
            const char* cur = lds_c + cur_buf * kLdsBlock;
            dma_wait(RT == 2 || blk + 1 < n_blocks ? my_loads : 0);
            __syncthreads();
            if constexpr (RT == 2) {
                static_assert(RT != 2 || (kDmaPerBlock + NW - 1) / NW <= kFrags / kPpDmaEvery, "a slot for every load");
                // The loads of block blk + 2, spread over the score phase.  Past the segment's end they
                // run against an empty buffer (nothing is fetched, zeros land in the free LDS buffer),
                // so that every block issues the same number of loads and the slots need no branch.
                u32x4_t rc_next = rc;
                if (blk + 2 >= n_blocks) rc_next[2] = 0u;
                const DmaWave d4 = dma_wave_for(lds_c + next_buf * kLdsBlock, j0 + (blk + 2) * kMlaKeys, wave);
                mla_block_pp<decltype(lo_mode)::value, decltype(masked)::value>(
                    st, cur + qk_off, cur + qt_off, cur + pv_off, qop, q_lds, prm.scale_log2, j0 + blk * kMlaKeys, lim, kb,
                    [&](auto q_c) { block_load_static<NW, decltype(q_c)::value>(d4, rc_next, dma, wave); });
            } else {
                const bool late = kSkewWaves && NW == 8 && wave < 4;
                if (blk + 2 < n_blocks && !late)
                    block_to_lds<NW>(lds_c + next_buf * kLdsBlock, rc, j0 + (blk + 2) * kMlaKeys, wave, dma);
                mla_block<RT, decltype(lo_mode)::value>(st, cur + qk_off, cur + qt_off, cur + pv_off, qop, q_lds, prm.scale_log2,
                                                        j0 + blk * kMlaKeys, lim, kb);
                if (blk + 2 < n_blocks && late)
                    block_to_lds<NW>(lds_c + next_buf * kLdsBlock, rc, j0 + (blk + 2) * kMlaKeys, wave, dma);
            }
            cur_buf = cur_buf == kStages - 1 ? 0 : cur_buf + 1;
            next_buf = next_buf == kStages - 1 ? 0 : next_buf + 1;
        };
        // Default mode: the first blocks of a segment with hi + lo weights, the others with hi + lo
        // only where a key dominates.
        const int n_exact = kMode == 1 ? n_blocks : kMode == 2 ? 0 : (n_blocks < kExactBlocks ? n_blocks : kExactBlocks);
        // Two tiles per wave: blocks that end at or below every row's limit (the end of the segment, the
        // causal limit of the wave's first row) run without masking, the few others in the masked form.
        int first_masked = n_blocks;
        if constexpr (RT == 2) {
            const int causal_min = L - T + wave_row0 / H + 1;
            const int clear = ((causal_min < j1 ? causal_min : j1) - j0) / kMlaKeys;
            first_masked = clear < 0 ? 0 : (clear < n_blocks ? clear : n_blocks);
        }
        const int n_exact_clear = n_exact < first_masked ? n_exact : first_masked;
        int blk = 0;
        for (; blk < n_exact_clear; ++blk) step(blk, std::integral_constant<int, kLoAlways>(), std::false_type());
        for (; blk < first_masked; ++blk)
            step(blk, std::integral_constant<int, kMode == 0 ? kLoDynamic : (kMode == 1 ? kLoAlways : kLoNever)>(), std::false_type());
        for (; blk < n_blocks; ++blk) step(blk, std::integral_constant<int, kMode == 2 ? kLoNever : kLoAlways>(), std::true_type());
        if constexpr (RT == 2) dma_wait(0);      // the empty loads behind the last block: they write (zeros) to the buffers
        if constexpr (RT == 2)        // the accumulators are read below; all but the last were written long ago
            mfma_drain_acc(st[0].o[kColTiles - 2], st[0].o[kColTiles - 1], st[1].o[kColTiles - 2], st[1].o[kColTiles - 1]);
        __syncthreads();          // everyone is done with the block buffers: they stage the output now

#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const float l = st[rt].l;
            const float lq = kb_sum(st[rt].lq);
            // A partial row goes out as fp16 after scaling its largest magnitude to 2^15 (the scale's
            // inverse is kept in fp32 beside the row's m and l): half the bytes of fp32 to write here
            // and to read back in the merge.  Every element keeps 11 significant bits of its own
            // (down to 2^-29 of the row's maximum), so a few large columns cost the others nothing.
            // The scale is capped so that rows of denormal size do not overflow it.
            float sc, inv_scale = 0.0f;
            if (whole) {
                sc = lq > 0.0f ? 1.0f / lq : 0.0f;
            } else {
                float amax = 0.0f;
#pragma unroll
                for (int ct = 0; ct < kColTiles; ++ct)
#pragma unroll
                    for (int i = 0; i < 4; ++i) amax = fmaxf(amax, __builtin_fabsf(st[rt].o[ct][i]));
                amax = kb_max(amax);
                sc = amax > 0.0f ? fminf(32768.0f / amax, 0x1.0p100f) : 0.0f;
                inv_scale = amax > 0.0f ? 1.0f / sc : 0.0f;
            }
            const int tile_row0 = wave_row0 + 16 * rt;
            // Rounded to 16 bits (bf16 results, fp16 partial rows), half a row at a time through the
            // block buffers, which are free between the segment's last block and the next segment's
            // first: two rounds per tile, each store instruction writing two whole 512-byte half rows.
            // The stores go through a buffer descriptor over the sequence's (or slot's) rows: 32-bit
            // offsets, and rows past rows_total fall outside and are dropped, so the loop has no branch.
            uint16_t* dst = whole ? prm.out + (long)b * rows_total * kDv : prm.part_o + slot * rows_total * kDv;
            const uint64_t daddr = (uint64_t)(uintptr_t)dst;
            const __amdgpu_buffer_rsrc_t rd = make_rsrc(
                reinterpret_cast<void*>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(daddr >> 32)) << 32) |
                                        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)daddr)),
                (uint32_t)rows_total * (kDv * 2));
            const uint32_t lane_dst = (uint32_t)((tile_row0 + (lane >> 5)) * (kDv * 2) + (lane & 31) * 16);
            const char* lane_stage = stage + (lane >> 5) * kStagePitch + (lane & 31) * 16;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int c = 0; c < kColTiles / 2; ++c) {
                    const f32x4_t o = st[rt].o[(kColTiles / 2) * h + c] * sc;
                    uint2 w;
                    w.x = whole ? cvt_bf16(o[0], o[1]) : pack_f16(o[0], o[1]);
                    w.y = whole ? cvt_bf16(o[2], o[3]) : pack_f16(o[2], o[3]);
                    *reinterpret_cast<uint2*>(stage + n * kStagePitch + (16 * c + 4 * kb) * 2) = w;
                }
                fence();
#pragma unroll
                for (int i = 0; i < 8; ++i) {          // rows 2 i and 2 i + 1, 256 columns each, per instruction
                    const u32x4_t w = *reinterpret_cast<const u32x4_t*>(lane_stage + 2 * i * kStagePitch);
                    __builtin_amdgcn_raw_buffer_store_b128(w, rd, (int)(lane_dst + 2 * i * (kDv * 2) + h * kDv), 0, 0);
                }
                fence();
            }
            const int row = tile_row0 + n;
            if (row < rows_total && kb == 0) {
                if (whole) {
                    if (prm.lse) prm.lse[(long)b * rows_total + row] = l > 0.0f ? (st[rt].m + __log2f(l)) * kLn2 : kNegInf;
                } else {
                    reinterpret_cast<float4*>(prm.part_ml)[slot * rows_total + row] = make_float4(st[rt].m, l, lq, inv_scale);
                }
            }
        }
        __syncthreads();          // the next segment's first block goes to buffer 0, which staged output until here
    }
}

// One wave per output row of 512 columns; lane holds columns 8*lane .. 8*lane+7.  A partial row is 512
// fp16 values times its own scale (the fourth value of its (m, l, lq, 1 / scale) record).
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
    const float4* ml = reinterpret_cast<const float4*>(prm.part_ml) + (long)fs.x * rows_total + th;   // (m, l, lq, 1 / scale)
    const uint4* po = reinterpret_cast<const uint4*>(prm.part_o + ((long)fs.x * rows_total + th) * kDv) + lane;
    const long po_stride = rows_total * (kDv / 8);
    float M = kNegInf;
    for (int base = 0; base < n; base += 64)
        if (base + lane < n) M = fmaxf(M, ml[(base + lane) * rows_total].x);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    const float m_use = (M == kNegInf) ? 0.0f : M;
    float l = 0.0f, lq = 0.0f;
    float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int s0 = 0; s0 < n; s0 += 4) {
        float4 a[4];
        uint4 o[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u < n ? s0 + u : n - 1;
            a[u] = ml[s * rows_total];
            const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(&po[s * po_stride]));   // read once
            o[u] = make_uint4(t.x, t.y, t.z, t.w);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = s0 + u < n ? fast_exp2(a[u].x - m_use) : 0.0f;
            l = __builtin_fmaf(a[u].y, w, l);
            lq = __builtin_fmaf(a[u].z, w, lq);
            const float ws = w * a[u].w;             // weight times the inverse of the row's scale
            const uint32_t q[4] = {o[u].x, o[u].y, o[u].z, o[u].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const f32x2_t v = __builtin_convertvector(__builtin_bit_cast(f16x2_t, q[c]), f32x2_t);
                acc[2 * c] = __builtin_fmaf(v[0], ws, acc[2 * c]);
                acc[2 * c + 1] = __builtin_fmaf(v[1], ws, acc[2 * c + 1]);
            }
        }
    }
    const float inv = lq > 0.0f ? 1.0f / lq : 0.0f;
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
    if (prm.weight_mode == 1) hipLaunchKernelGGL((mla_decode_kernel<NW, RT, 1>), grid, dim3(64 * NW), 0, stream, prm);
    else if (prm.weight_mode == 2) hipLaunchKernelGGL((mla_decode_kernel<NW, RT, 2>), grid, dim3(64 * NW), 0, stream, prm);
    else hipLaunchKernelGGL((mla_decode_kernel<NW, RT, 0>), grid, dim3(64 * NW), 0, stream, prm);
    return hipGetLastError();
}

}  // namespace

// Workgroup shape for rows_total = q_len * n_heads query rows per sequence: (waves, 16-row tiles per
// wave).  Automatic: one tile per wave, 8 waves from 65 rows on (two waves per SIMD, 256 registers
// each).  layout 1: at most 4 waves of one tile (64 rows per workgroup); layout 2: 4 waves of two
// tiles from 65 rows on (one wave per SIMD, 512 registers).
void mla_block_shape(int rows_total, int layout, int* waves, int* tiles_per_wave) {
    const int tiles = (rows_total + 15) / 16;
    *tiles_per_wave = (tiles > 4 && layout == 2) ? 2 : 1;
    *waves = (layout != 1 && layout != 2 && tiles > 4) ? 8 : tiles >= 3 ? 4 : tiles;
}

hipError_t launch_mla_decode(const MlaParams& prm, hipStream_t stream, hipEvent_t* events) {
    const int rows_total = prm.q_len * prm.n_heads;
    int nw = 1, rt = 1;
    mla_block_shape(rows_total, prm.layout, &nw, &rt);
    dim3 grid((unsigned)((prm.n_pieces + 7) / 8 * 8 * ((rows_total + 16 * rt * nw - 1) / (16 * rt * nw))));
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
