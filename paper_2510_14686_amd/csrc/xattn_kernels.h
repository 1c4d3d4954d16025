// Internal interface between the C-ABI host code and the gfx950 kernels.
#ifndef XATTN_KERNELS_H_
#define XATTN_KERNELS_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xattn {

constexpr int kHeadDim = 128;
// Default share (per mille) moved from the odd-numbered XCDs' parts of the token stream to the
// even-numbered ones: on MI355X the odd XCDs need about 7 % longer for the same bytes (measured per
// wave with clock stamps on several machines; rotating the data among the XCDs moves nothing), so
// equal parts leave the even XCDs idle at the end of the kernel.
constexpr int kDefaultXcdSkewGqa = 32;
constexpr int kDefaultXcdSkewMla = 0;
constexpr int kMaxWavesPerBlock = 8;   // one wave per KV head, up to 8 KV heads per workgroup

// Workspace header: per sequence two int32 words, (first partial slot, number of segments), written
// by the decode kernel for the merge kernel.  0 segments = no keys; 1 = finished by the decode kernel.

struct DecodeParams {
    const uint16_t* q;               // bf16 [batch, q_len, n_q_heads, 128]
    const void* const* k_ptrs;       // device array[batch] of device pointers
    const void* const* v_ptrs;
    const int32_t* kv_lens;          // device int32[batch]
    int batch, q_len, n_q_heads, n_kv_heads, group;
    float scale_log2;                // scale * log2(e)
    uint16_t* out;                   // bf16 [batch, q_len, n_q_heads, 128]
    float* lse;                      // fp32 [batch, q_len, n_q_heads] or null
    float* part_o;                   // fp32 [slots, q_len * n_q_heads, 128]
    float* part_ml;                  // fp32 [slots, q_len * n_q_heads, 2]  (max, sum)
    int32_t* meta;                   // int32 [batch, 2]
    int n_pieces;                    // pieces the token stream is cut into (upper bound on active ones)
    int min_piece_tokens;
    int xcd_skew;                    // per mille: share taken from the odd XCDs' parts of the stream and given to the even ones
    int path;                        // kPathAuto, kPathVector or kPathMatrix
    int pv_mode;                     // matrix path: kPvBf16x2, kPvFp32 or kPvBf16
};

// How the matrix path multiplies the softmax weights p with V.
constexpr int kPvBf16x2 = 0;   // default: bf16 MFMA 16x16x16 twice, p as hi + lo bf16 parts (16 significant bits)
constexpr int kPvFp32 = 1;     // fp32 MFMA 16x16x4, p exact; 4x the matrix-core time, measurably slower
constexpr int kPvBf16 = 2;     // bf16 MFMA 16x16x16 once, p rounded to bf16; same speed as the default, less exact

// Inner-loop choice: automatic = vector path below 4 query rows per KV head, matrix path from 4 up.
constexpr int kPathAuto = 0;
constexpr int kPathVector = 1;
constexpr int kPathMatrix = 2;

bool use_matrix_path(int rows_total, int path);

// Query rows one workgroup pass handles for a KV head with rows_total = group * q_len rows.
int rows_per_tile(int rows_total, int path);

// Enqueues the split-KV decode kernel and the merge kernel on `stream`.  If `events` is not null it
// holds three events, recorded before the decode kernel, between the kernels and after the merge.
hipError_t launch_decode(const DecodeParams& prm, hipStream_t stream, hipEvent_t* events);

// Latent-KV (MLA-shaped) decode: every head reads the same cached row of 576 bf16 per token.
struct MlaParams {
    const uint16_t* q;               // bf16 [batch, q_len, n_heads, 576]
    const void* const* c_ptrs;       // device array[batch] of device pointers: bf16 [kv_len, 576]
    const int32_t* kv_lens;
    int batch, q_len, n_heads;
    float scale_log2;
    uint16_t* out;                   // bf16 [batch, q_len, n_heads, 512]
    float* lse;                      // fp32 [batch, q_len, n_heads] or null
    uint16_t* part_o;                // fp16 [slots, q_len * n_heads, 512]: partial rows, each times its own scale
    float* part_ml;                  // fp32 [slots, q_len * n_heads, 4]: (max, sum, sum of rounded weights, 1 / scale)
    int32_t* meta;                   // int32 [batch, 2]
    int n_pieces, min_piece_tokens;
    int xcd_skew;                    // as in DecodeParams
    int layout;                      // 0 automatic, 1 one 16-row tile per wave, 2 two tiles per wave
    int weight_mode;                 // softmax weights in the value product: 0 default (hi + lo bf16 parts where a key
                                     // dominates, one bf16 elsewhere), 1 hi + lo everywhere, 2 one bf16 everywhere
};
void mla_block_shape(int rows_total, int layout, int* waves, int* tiles_per_wave);
// Enqueues the decode kernel and its merge kernel; events as for launch_decode.
hipError_t launch_mla_decode(const MlaParams& prm, hipStream_t stream, hipEvent_t* events);

// Appends q_len new K/V rows per sequence at rows [kv_lens[b] - q_len, kv_lens[b]).
struct WriteParams {
    const uint16_t* k_new;           // bf16 [batch, q_len, row_elems]
    const uint16_t* v_new;
    void* const* k_ptrs;
    void* const* v_ptrs;
    const int32_t* kv_lens;
    int batch, q_len;
    int row_bytes;                   // n_kv_heads * head_dim * 2
};
hipError_t launch_write_kvcache(const WriteParams& prm, hipStream_t stream);

}  // namespace xattn
#endif
