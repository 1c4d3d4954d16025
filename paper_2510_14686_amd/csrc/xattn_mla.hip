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
// owns one piece and up to 128 query rows (row = token * n_heads + head): wave w owns rows 16w..16w+15,
// keeps their Q (72 VGPRs) and their output accumulators (16 x 512 fp32 = 128 VGPRs) in registers for
// the whole piece, and all waves share each 16-key block of the cache through LDS:
//   * the block (16 x 1152 bytes, contiguous in memory) goes from HBM straight into LDS (buffer loads
//     with the LDS destination, 1 KiB per wave instruction, no staging registers), once per
//     workgroup, two LDS buffers, one barrier per block, the next block in flight during the
//     arithmetic; 16-byte chunks are XOR-swizzled by row (through the global address each lane
//     fetches, since the LDS side of such a load is fixed to lane order) against bank conflicts;
//   * S^T = C Q^T: 18 bf16 MFMA 16x16x32 on two accumulators, the A operand read from LDS;
//   * softmax on the accumulator layout, as in the GQA matrix path;
//   * O^T += C[:, 0:512]^T P^T: per 128-column group a lane reads the same 8 columns of its four keys
//     (4 x 128 bits) and builds the A operands of 8 column tiles with byte permutes; P goes in as
//     hi + lo bf16 parts (bf16 MFMA 16x16x16).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xattn_device.h"
#include "xattn_kernels.h"

namespace xattn {
namespace {

constexpr int kDqk = 576;                        // key width: latent + rope
constexpr int kDv = 512;                         // value width: the latent part
constexpr int kRowB = kDqk * 2;                  // 1152 bytes per cached token
constexpr int kChunksPerRow = kRowB / 16;        // 72
constexpr int kBlockChunks = kBlockKeys * kChunksPerRow;   // 1152 16-byte chunks per 16-key block
constexpr int kLdsBlock = kBlockKeys * kRowB;    // 18 KiB, rows unpadded: chunk slot c of row r holds chunk c ^ (r & 7)
constexpr int kDmaPerBlock = kLdsBlock / 1024;   // 18 wave-wide loads of 64 x 16 bytes
constexpr int kQSteps = kDqk / 32;               // 18 MFMA steps of 32 columns
constexpr int kVGroups = kDv / 128;              // 4 groups of 128 value columns
constexpr int kOutPitch = 128 * 4 + 16;          // epilogue: 16 rows x 128 fp32 columns, padded
constexpr int kLdsOutPerWave = 16 * kOutPitch;
constexpr int kMaxWaves = 8;

// Running state of one 16-row tile.
struct MlaTile {
    f32x4_t o[kVGroups * 8];   // o[g * 8 + e][j]: column 128 g + 8 (4 kb + j) + e of row n
    float m, l;
};

// This wave's share of the loads of one 16-key block into LDS: load q fills LDS bytes
// [q * 1024, (q + 1) * 1024) of the block in lane order, i.e. linear chunk position P = 64 q + lane
// = (row, slot); the lane fetches the global chunk that belongs there, slot ^ (row & 7) of that row.
// The loads are written as assembly so that the compiler does not order them against LDS reads: it
// cannot tell the two halves of the double buffer apart and would wait for every outstanding load
// before each read.  dma_wait() before the workgroup barrier is what makes a block visible.
__device__ __forceinline__ void dma16(u32x4_t rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 1\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int NW>
__device__ __forceinline__ void block_to_lds(char* lds_block, u32x4_t rc, int j_block, int wave, int lane) {
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_block;
#pragma unroll
    for (int q = 0; q < (kDmaPerBlock + NW - 1) / NW; ++q) {
        const int qq = wave + q * NW;            // wave-uniform
        if (qq < kDmaPerBlock) {
            const int pos = qq * 64 + lane;
            const int row = pos / kChunksPerRow, slot = pos - row * kChunksPerRow;
            const uint32_t voff = (uint32_t)(row * kChunksPerRow + (slot ^ (row & 7))) * 16;
            dma16(rc, lds0 + qq * 1024, voff, (uint32_t)j_block * kRowB);
        }
    }
}

// One 16-key block from LDS against this wave's RT tiles of 16 rows.  Every operand read from LDS (a
// key fragment, a value fragment) is used for all RT tiles.  kHiLo: the softmax weights go into the
// value product as hi + lo bf16 parts (two MFMAs, 16 significant bits) instead of one rounded bf16.
template <int RT, bool kHiLo>
__device__ __forceinline__ void mla_block(MlaTile (&st)[RT], const char* lds_block,
                                          const bf16x8_t (&qop)[RT][kQSteps], float scale_log2, int j_block,
                                          const int (&lim)[RT], int kb, int n) {
    // Key n, chunk 4 * step + kb sits in slot (4 * step + kb) ^ (n & 7): the XOR touches the low three
    // bits only, which alternate between kb and 4 + kb with the step's parity.
    const char* arow = lds_block + n * kRowB;
    const int a_even = (kb ^ (n & 7)) * 16, a_odd = ((4 + kb) ^ (n & 7)) * 16;
    f32x4_t s0[RT], s1[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) s0[rt] = s1[rt] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int step = 0; step < kQSteps; step += 2) {
        const bf16x8_t a0 = *reinterpret_cast<const bf16x8_t*>(arow + a_even + (step >> 1) * 128);
        const bf16x8_t a1 = *reinterpret_cast<const bf16x8_t*>(arow + a_odd + (step >> 1) * 128);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            s0[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qop[rt][step], s0[rt], 0, 0, 0);
            s1[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qop[rt][step + 1], s1[rt], 0, 0, 0);
        }
    }
    u32x2_t ph[RT], pl[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const f32x4_t s = s0[rt] + s1[rt];      // s[i] = score of key j_block + 4*kb + i for row n of tile rt
        float p[4];
        float mx = kNegInf;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] = (j_block + 4 * kb + i < lim[rt]) ? s[i] * scale_log2 : kNegInf;
            mx = fmaxf(mx, p[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(st[rt].m, mx);
        const float m_use = (m_new == kNegInf) ? 0.0f : m_new;
        const float alpha = fast_exp2(st[rt].m - m_use);
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] = fast_exp2(p[i] - m_use);
            sum += p[i];
        }
        st[rt].l = st[rt].l * alpha + sum;
        st[rt].m = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int t = 0; t < kVGroups * 8; ++t) st[rt].o[t] *= alpha;
        }
        const f32x2_t p01 = {p[0], p[1]}, p23 = {p[2], p[3]};
        const bf16x2_t h01 = __builtin_convertvector(p01, bf16x2_t), h23 = __builtin_convertvector(p23, bf16x2_t);
        ph[rt] = u32x2_t{__builtin_bit_cast(uint32_t, h01), __builtin_bit_cast(uint32_t, h23)};
        pl[rt] = u32x2_t{0u, 0u};
        if (kHiLo) {
            const f32x2_t r01 = p01 - __builtin_convertvector(h01, f32x2_t);
            const f32x2_t r23 = p23 - __builtin_convertvector(h23, f32x2_t);
            pl[rt] = u32x2_t{__builtin_bit_cast(uint32_t, __builtin_convertvector(r01, bf16x2_t)),
                             __builtin_bit_cast(uint32_t, __builtin_convertvector(r23, bf16x2_t))};
        }
    }
    // Values: lane (kb, x) reads, for keys 4 kb + i, chunk 16 g + x (columns 128 g + 8 x .. + 7), which
    // sits in slot 16 g + (x ^ (key & 7)); half a chunk (4 columns, 64 bits) at a time to keep the
    // live registers down.  Column tile e of the group takes the e-th bf16 of the four keys' chunks.
    int vaddr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) vaddr[i] = (4 * kb + i) * kRowB + ((n ^ ((4 * kb + i) & 7)) * 16);
#pragma unroll
    for (int g = 0; g < kVGroups; ++g) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u32x2_t v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = *reinterpret_cast<const u32x2_t*>(lds_block + vaddr[i] + g * 256 + h * 8);
            u32x2_t a[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const uint32_t sel = (e2 & 1) ? 0x07060302u : 0x05040100u;
                a[e2] = u32x2_t{__builtin_amdgcn_perm(v[1][e2 >> 1], v[0][e2 >> 1], sel),
                                __builtin_amdgcn_perm(v[3][e2 >> 1], v[2][e2 >> 1], sel)};
            }
            // independent accumulators back to back; the lo parts follow once all hi parts are issued
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2)
                    st[rt].o[g * 8 + 4 * h + e2] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
                        __builtin_bit_cast(s16x4_t, a[e2]), __builtin_bit_cast(s16x4_t, ph[rt]),
                        st[rt].o[g * 8 + 4 * h + e2], 0, 0, 0);
            if (kHiLo) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int e2 = 0; e2 < 4; ++e2)
                        st[rt].o[g * 8 + 4 * h + e2] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
                            __builtin_bit_cast(s16x4_t, a[e2]), __builtin_bit_cast(s16x4_t, pl[rt]),
                            st[rt].o[g * 8 + 4 * h + e2], 0, 0, 0);
            }
        }
    }
}

// grid.x = pieces, grid.y = groups of 16 * RT * NW rows; block = 64 * NW.  Wave w owns row tiles
// w * RT .. w * RT + RT - 1 of its group.
template <int NW, int RT, bool kHiLo>
__global__ __launch_bounds__(64 * NW) void mla_decode_kernel(MlaParams prm) {
    __shared__ __attribute__((aligned(16))) char lds_c[2 * kLdsBlock];
    __shared__ __attribute__((aligned(16))) char lds_out[NW * kLdsOutPerWave];
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
    char* out_lds = lds_out + wave * kLdsOutPerWave;
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
        // Q operand: lane (kb, n) holds chunk 4 * step + kb of row n of each tile.
        bf16x8_t qop[RT][kQSteps];
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
                qop[rt][step] = __builtin_bit_cast(bf16x8_t, qv);
            }
            const int causal = L - T + (row_ok ? row : 0) / H + 1;
            lim[rt] = causal < j1 ? causal : j1;
#pragma unroll
            for (int i = 0; i < kVGroups * 8; ++i) st[rt].o[i] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
            st[rt].m = kNegInf;
            st[rt].l = 0.0f;
        }

        const int n_blocks = (j1 - j0 + kBlockKeys - 1) / kBlockKeys;
        for (int blk = 0; blk < n_blocks; ++blk) {
            char* cur = lds_c + (blk & 1) * kLdsBlock;
            // Every wave waits for its own loads of block blk, then the barrier: block blk is in LDS
            // and everyone is done reading block blk - 1, whose buffer the next loads may overwrite.
            dma_wait();
            __syncthreads();
            if (blk + 1 < n_blocks)
                block_to_lds<NW>(lds_c + ((blk + 1) & 1) * kLdsBlock, rc, j0 + (blk + 1) * kBlockKeys, wave, lane);
            mla_block<RT, kHiLo>(st, cur, qop, prm.scale_log2, j0 + blk * kBlockKeys, lim, kb, n);
        }
        __syncthreads();          // the next segment's first block reuses buffer 0

        // Store, 128 columns at a time through this wave's LDS so that stores write whole rows.
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float l = st[rt].l;
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            const float sc = whole ? (l > 0.0f ? 1.0f / l : 0.0f) : 1.0f;
            const int tile_row0 = wave_row0 + 16 * rt;
#pragma unroll
            for (int g = 0; g < kVGroups; ++g) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    float4* w = reinterpret_cast<float4*>(out_lds + n * kOutPitch + (4 * kb + jj) * 32);
                    w[0] = make_float4(st[rt].o[g * 8 + 0][jj] * sc, st[rt].o[g * 8 + 1][jj] * sc,
                                       st[rt].o[g * 8 + 2][jj] * sc, st[rt].o[g * 8 + 3][jj] * sc);
                    w[1] = make_float4(st[rt].o[g * 8 + 4][jj] * sc, st[rt].o[g * 8 + 5][jj] * sc,
                                       st[rt].o[g * 8 + 6][jj] * sc, st[rt].o[g * 8 + 7][jj] * sc);
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
// wave).  layout 1 forces one tile per wave (up to 8 waves), layout 2 two tiles per wave (4 waves).
void mla_block_shape(int rows_total, int layout, int* waves, int* tiles_per_wave) {
    const int tiles = (rows_total + 15) / 16;
    if (tiles >= 8 && layout == 2) { *waves = 4; *tiles_per_wave = 2; return; }
    *tiles_per_wave = 1;
    if (layout == 3 && tiles >= 4) { *waves = 4; return; }
    *waves = tiles >= 8 ? 8 : tiles >= 4 ? 4 : tiles >= 2 ? 2 : 1;
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
