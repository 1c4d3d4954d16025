/*
 * xattn -- decode attention over xTensor-style KV memory on one AMD MI355X (gfx950).
 *
 * C ABI of libxattn.so.  Plain pointers and sizes only; every pointer says whether it is a HOST
 * or a DEVICE pointer.  No exception crosses this boundary: every call returns an xattn_status
 * (0 = success, negative = failure) and leaves a message for xattn_last_error().
 *
 * Paper: "xLLM Technical Report" (arXiv 2510.14686).  Passages cited below:
 *   section 4.3   "Efficient Memory Management" (xTensor): a request's KV cache is contiguous in a
 *                 reserved virtual range and is backed on demand by discrete fixed-size physical
 *                 pages; operators receive the starting virtual address and offsets, no block table
 *                 (paragraphs "Physical Memory Page Management ...", "On-demand Memory Mapping",
 *                 "Operator Adaptation", and the address -> (page, offset) equation).
 *   section 4.4.1 "MLA Optimization": the m+1 query tokens of a speculative step are multiplied with
 *                 the same K, which is loaded once for all of them and Q stays resident.
 *   section 4.4.3 "Layer 3: Fine-Grained Kernel-Level Optimization": work is balanced across compute
 *                 units by token count and long sequences are split; "Layer 2": partial attention
 *                 results are combined by an aggregation operator.
 *   section 4.2   "Integrating Custom Operators": runtime shapes reach the kernels as arguments, so
 *                 nothing on the host depends on their values (no host read of kv_lens, no sync).
 */
#ifndef XATTN_H_
#define XATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XATTN_OK = 0,
    XATTN_EINVAL = -1,       /* null pointer, non-positive size, inconsistent arguments */
    XATTN_EUNSUPPORTED = -2, /* a valid request outside the supported set (see xattn_decode) */
    XATTN_ENOMEM = -3,       /* device or virtual-address space exhausted */
    XATTN_EHIP = -4          /* a HIP runtime call failed; the message names it */
} xattn_status;

/* Message of the calling thread's last failed call. HOST string, never NULL, valid until that
 * thread's next failing call. */
const char* xattn_last_error(void);

/*
 * Batched grouped-query decode attention (section 4.3 "Operator Adaptation", section 4.4.1).
 *
 * For sequence b, new query token t in [0, q_len) and query head h (KV head g = h / (n_q_heads /
 * n_kv_heads)), with Lv = kv_lens[b] - q_len + t + 1 visible keys (the cached prefix plus new tokens
 * 0..t: a causal mask inside the block of new tokens):
 *     s_j = scale * <Q[b,t,h,:], K_b[j,g,:]>,  j in [0, Lv)
 *     out[b,t,h,:] = sum_j softmax(s)_j * V_b[j,g,:]        lse[b,t,h] = ln sum_j exp(s_j)
 * The key range is partitioned over the GPU's compute units by token count (sequences are split and
 * short ones share a workgroup, section 4.4.3 Layer 3) and partial results are combined exactly by
 * a log-sum-exp merge; accumulation is fp32, results are rounded to bf16 (nearest even).
 *
 * q        DEVICE  bf16 [batch, q_len, n_q_heads, head_dim], contiguous
 * k_ptrs   DEVICE  array[batch] of DEVICE pointers; k_ptrs[b] -> bf16 [>= kv_lens[b], n_kv_heads,
 *                  head_dim], row-major, 16-byte aligned.  Any device-accessible address works: an
 *                  xtensor_map range or an ordinary allocation.  Rows past kv_lens[b] are never read.
 * v_ptrs   DEVICE  same layout as K
 * kv_lens  DEVICE  int32[batch]; keys visible to the LAST new token, i.e. prefix + q_len (the new
 *                  tokens' K/V are already written).  Read on the device only.  A value < q_len
 *                  leaves the tokens without visible keys with out = 0 and lse = -inf.  The device
 *                  adds the lengths up in 32 bits: the sum over the batch of (kv_lens[b] + 16) must
 *                  stay below 2^31 (for xattn_mla_decode: kv_lens[b] + 192).  The host cannot check
 *                  it and results are undefined beyond, but lengths whose caches fit one GPU's
 *                  memory cannot reach it (2^31 rows of the smallest K/V row pair are 1 TiB).
 * batch    1..4096;  q_len 1..16;  head_dim must be 128;  n_q_heads a multiple of n_kv_heads;
 *          (n_q_heads / n_kv_heads) * q_len <= 64.  Otherwise XATTN_EUNSUPPORTED.
 * scale    multiplies the scores before the softmax (the caller's fp32 value, e.g. 1/sqrt(128))
 * out      DEVICE  bf16 [batch, q_len, n_q_heads, head_dim]
 * lse      DEVICE  fp32 [batch, q_len, n_q_heads], natural log; may be NULL
 * stream   hipStream_t (NULL = the default stream).  The call only enqueues work: it never
 *          synchronises and never reads device memory on the host.
 *
 * Graph capture (section 4.2, "Integrating Custom Operators"): the call may be recorded into a HIP
 * graph and replayed with other lengths, pointers and data in the same device buffers, since nothing
 * on the host depends on their values.  The stream's workspace must be large enough beforehand (one
 * eager call of the shape ON THAT STREAM, or xattn_set_workspace); a call that would have to grow it
 * during capture returns XATTN_ENOMEM and records nothing.  A recorded graph stays valid when later
 * calls grow the workspace: outgrown buffers are kept until the process ends, never freed.
 *
 * Ownership: the caller owns every buffer and keeps it alive and unmodified until the enqueued work
 * has finished.  The library keeps one workspace per stream (see below), so calls on different
 * streams of a device may overlap; calls on ONE stream are ordered by the stream.  With a caller
 * workspace (xattn_set_workspace) all streams share it and must not overlap.  On failure nothing is
 * enqueued.
 */
int xattn_decode(const void* q, const void* const* k_ptrs, const void* const* v_ptrs,
                 const int32_t* kv_lens, int batch, int q_len, int n_q_heads, int n_kv_heads,
                 int head_dim, float scale, void* out, float* lse, void* stream);

/*
 * xattn_decode for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels, partition and results
 * (bit for bit) as xattn_decode; the partial results of split sequences go to a device array of
 * XATTN_NOALLOC_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs
 * on holds its copy until the process ends) instead of a workspace from hipMalloc.  The call
 * allocates nothing: no hipMalloc, hipFree or event creation; xattn_set_workspace and
 * XATTN_CFG_TIMING do not apply to it.
 * A shape whose partial results need more than the array holds (see xattn_workspace_bytes; all five
 * benchmark configurations fit) returns XATTN_EUNSUPPORTED and enqueues nothing.  All calls on a GPU
 * share that GPU's array, whatever their stream: calls that overlap in time on one GPU race; calls
 * on one stream are ordered by it.  Nothing in the array has to start at zero (every word that is
 * read was written by the same call before).  The array's address is resolved on the first call on a
 * device; make that first call outside graph capture.
 */
#define XATTN_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
int xattn_decode_noalloc(const void* q, const void* const* k_ptrs, const void* const* v_ptrs,
                         const int32_t* kv_lens, int batch, int q_len, int n_q_heads, int n_kv_heads,
                         int head_dim, float scale, void* out, float* lse, void* stream);

/*
 * Latent-KV decode attention, the MLA-shaped operator the paper itself adapts (section 4.3
 * "Operator Adaptation"; section 4.4.1 "MLA Optimization": with m speculated tokens, m+1 query
 * tokens per sequence, all heads, are multiplied with the same cached rows).  Per token the cache
 * holds ONE row of d_latent + d_rope bf16 shared by all heads: the whole row is every head's key, its
 * first d_latent values are every head's value (K and V alias one buffer):
 *     s_j = scale * <Q[b,t,h,:], C_b[j,:]>,  j < kv_lens[b] - q_len + t + 1
 *     out[b,t,h,:] = sum_j softmax(s)_j * C_b[j, 0:d_latent]      lse[b,t,h] = ln sum_j exp(s_j)
 * q       DEVICE bf16 [batch, q_len, n_heads, d_latent + d_rope]
 * c_ptrs  DEVICE array[batch] of DEVICE pointers; c_ptrs[b] -> bf16 [>= kv_lens[b], d_latent + d_rope],
 *         16-byte aligned; an xTensor range or any other device memory
 * kv_lens DEVICE int32[batch], as for xattn_decode
 * scale   positive and finite (XATTN_EINVAL otherwise)
 * out     DEVICE bf16 [batch, q_len, n_heads, d_latent];  lse DEVICE fp32 [batch, q_len, n_heads] or NULL
 * Supported: d_latent = 512, d_rope = 64, q_len * n_heads <= 4096, batch <= 4096; otherwise
 * XATTN_EUNSUPPORTED.  Same partition, workspace, stream, capture and ownership rules as xattn_decode.
 * Numerics: fp32 accumulation; the softmax weights enter the value product as bf16, with 16
 * significant bits where a key dominates its row and 8 elsewhere (see XATTN_CFG_PV_MODE), and the
 * output is divided by the sum of the weights as they entered; the partial output rows of a sequence that is split over several compute units
 * pass through the workspace as fp16 scaled by the row's largest magnitude (11 significant bits per
 * element).  q and the cached rows must be finite: an infinity or NaN makes the rows it reaches
 * unspecified.
 */
int xattn_mla_decode(const void* q, const void* const* c_ptrs, const int32_t* kv_lens, int batch, int q_len,
                     int n_heads, int d_latent, int d_rope, float scale, void* out, float* lse, void* stream);

/*
 * Workspace for the partial results of split sequences (section 4.4.3: the parts of a split
 * sequence are computed by different compute units and aggregated afterwards).
 * xattn_workspace_bytes:     upper bound on the bytes one xattn_decode call of this shape uses
 *                            (0 and a message for an unsupported shape).
 * xattn_mla_workspace_bytes: the same for one xattn_mla_decode call.
 * xattn_set_workspace:       hand the library a DEVICE buffer (256-byte aligned) for the current
 *                            device, used by calls on every stream; the caller keeps ownership and
 *                            keeps it alive while calls are in flight or graphs that recorded them
 *                            exist.  (NULL, 0) returns to the library-owned workspaces: one per
 *                            stream (up to 64 streams per device), allocated with hipMalloc by the
 *                            first call on the stream that needs more than it has.  An outgrown
 *                            buffer is not freed before the process ends, because work in flight and
 *                            recorded graphs may still use it; growth is geometric, so the outgrown
 *                            buffers of a stream add up to less than four times its live one.
 */
size_t xattn_workspace_bytes(int batch, int q_len, int n_q_heads, int n_kv_heads, int head_dim);
size_t xattn_mla_workspace_bytes(int batch, int q_len, int n_heads, int d_latent, int d_rope);
int xattn_set_workspace(void* dev_ptr, size_t bytes);

/*
 * Tuning knobs of the partition (section 4.4.3 Layer 3), for sweeps and for tests that show the
 * result does not depend on the partition.  key:
 *   XATTN_CFG_PIECES            number of equal-token pieces the batch's keys are cut into
 *                               (= workgroups launched); 0 = automatic (the CU count; xattn_mla_decode,
 *                               where a piece is worked on by one workgroup per 128 query rows of a
 *                               sequence: the CU count divided by that number)
 *   XATTN_CFG_MIN_PIECE_TOKENS  lower bound on a piece's tokens; 0 = default (64); values below 16
 *                               count as 16
 *   XATTN_CFG_TIMING            1 = record per-kernel events (see xattn_timing_read); 0 = off
 *   XATTN_CFG_PATH              inner loop of the decode kernel: 0 = automatic (vector path below 4
 *                               query rows per KV head, i.e. group * q_len < 4; matrix-core path
 *                               from 4 up), 1 = vector path, 2 = matrix-core path (section 4.4.1)
 *   XATTN_CFG_PV_MODE           matrix-core path, product of softmax weights and V: 0 = default, bf16
 *                               MFMA on hi + lo bf16 parts of the weights (16 significant bits);
 *                               1 = fp32 MFMA (weights exact, slower); 2 = one bf16 MFMA (weights
 *                               rounded to bf16)
 *                               (xattn_mla_decode: 0 = default, hi + lo bf16 parts for the first 128 keys
 *                               of every segment and wherever a key carries 1/4 or more of its row's
 *                               running sum, one bf16 elsewhere; 1 = hi + lo parts everywhere;
 *                               2 = one bf16 per weight everywhere, less exact on peaked rows)
 *   XATTN_CFG_MLA_LAYOUT        xattn_mla_decode workgroup shape for more than 64 query rows per sequence:
 *                               0 = automatic (8 waves of one 16-row tile), 1 = 4 waves of one tile,
 *                               2 = 4 waves of two tiles; for experiments, results do not depend on it
 *   XATTN_CFG_XCD_SKEW          the chip's eight XCDs do not stream at the same rate (the odd-numbered ones
 *                               are slower), so the stream is cut into eight XCD parts of unequal length
 *                               before each part is cut into equal pieces: 0 = the kernel's default,
 *                               n = 1..201: the even XCDs' parts are longer and the odd ones' shorter by
 *                               (n - 1) per mille (1 = equal parts).  Applies when the pieces in use are a
 *                               multiple of 8 and hold 512 positions or more; results do not depend on it.
 * Values outside [0, 65536] give XATTN_EINVAL.  Process-wide.
 */
enum { XATTN_CFG_PIECES = 0, XATTN_CFG_MIN_PIECE_TOKENS = 1, XATTN_CFG_TIMING = 2, XATTN_CFG_PATH = 3,
       XATTN_CFG_PV_MODE = 4, XATTN_CFG_MLA_LAYOUT = 5, XATTN_CFG_XCD_SKEW = 6 };
int xattn_configure(int key, int value);

/*
 * Per-kernel timing for benchmarks.  While XATTN_CFG_TIMING is 1, every xattn_decode call records
 * HIP events on its stream before the split-KV decode kernel, between it and the merge kernel, and
 * after the merge kernel (at most 4096 calls between two reads; later calls are not timed).
 * xattn_timing_read waits for the recorded events, returns the number of timed calls since the last
 * read and the SUMS of the two kernels' durations in milliseconds (HOST outputs, any may be NULL),
 * and starts a new series.  Events cost a little time themselves: measure whole-call throughput
 * with timing off.
 */
int xattn_timing_read(int* n_calls, float* decode_kernel_ms, float* merge_kernel_ms);

/*
 * xTensor range (section 4.3): reserve `reserve_bytes` of virtual address space for one tensor of
 * one request (the paper's MaxSeqLen worth), unbacked, then back its first `mapped_bytes` with
 * physical chunks of XTENSOR_CHUNK_BYTES each, created one by one and mapped in a pseudo-random
 * order drawn from `seed` (so that neighbouring virtual chunks are not physically adjacent), and
 * make them readable and writable from `device`.  Both sizes are rounded up to whole chunks;
 * mapped_bytes may be 0 and must not exceed reserve_bytes.
 *
 * base_out   HOST out: DEVICE virtual address of the range's first byte (chunk-aligned)
 * handle_out HOST out: opaque handle, owned by the library until xtensor_unmap
 * Errors: XATTN_EINVAL (sizes, null outputs), XATTN_EUNSUPPORTED (the device's mapping granularity
 * does not divide the chunk size), XATTN_ENOMEM, XATTN_EHIP.  On failure everything already
 * created is released again and the outputs are left NULL.
 */
#define XTENSOR_CHUNK_BYTES ((size_t)2 << 20)
int xtensor_map(size_t reserve_bytes, size_t mapped_bytes, uint64_t seed, int device,
                void** base_out, void** handle_out);

/* Unmap every chunk, release the physical memory and free the virtual range.  The caller makes
 * sure no kernel still uses the range.  A handle that is NULL or was already unmapped gives
 * XATTN_EINVAL and changes nothing. */
int xtensor_unmap(void* handle);

/*
 * Description of a mapped range, for tests of the address identity of section 4.3
 * (page = floor((va - va_start) / page_size), offset = (va - va_start) mod page_size):
 * order_out[i] (HOST int32[n], n >= mapped chunk count) receives the creation index of the
 * physical chunk that backs virtual chunk i.  Returns the mapped chunk count, or a negative status.
 */
int xtensor_chunk_order(void* handle, int32_t* order_out, int n);

/*
 * A second, read-write view of the physical chunks of `handle` in creation order (virtual chunk i of
 * the view is physical chunk i): the same memory under another address, which lets a test read back
 * through physical order what it wrote through the permuted range.  The view is owned by the
 * handle and disappears with xtensor_unmap.  view_out: HOST out, DEVICE address.
 */
int xtensor_physical_view(void* handle, void** view_out);

/*
 * xTensor page pool (section 4.3, "Physical Memory Page Management and Virtual Memory Tensor
 * Management", "On-demand Memory Mapping", "Low Overhead Allocation").
 *
 * xtensor_pool_create  creates n_pages physical pages of XTENSOR_CHUNK_BYTES on `device` up front.
 *                      Every page carries <PageID, Status, OwnerSession>; PageID is its index.
 *                      Pages are handed out in a pseudo-random order drawn from `seed`.
 * xtensor_pool_destroy unmaps Reusable sets and releases every page; fails with XATTN_EINVAL while
 *                      a range is still open.
 * xtensor_pool_counts  counts_out (HOST size_t[4]) receives the number of pages per status, indexed
 *                      by XTENSOR_PAGE_*.
 * xtensor_page_info    status and owner session of one page (outputs may be NULL).
 *
 * xtensor_open         a request's tensor: reserve `reserve_bytes` of virtual addresses (MaxSeqLen
 *                      worth; nothing backed) and back the first `mapped_bytes`.  Page reuse: if a
 *                      Reusable set of exactly ceil(mapped_bytes / page) pages sits in a range at
 *                      least as large, that range is handed over as it is (no Map/Unmap call) and
 *                      *reused_out = 1.  `session` is recorded as the pages' owner.
 * xtensor_grow         on-demand mapping: make the first `mapped_bytes` of the range backed by
 *                      mapping free pages at the next addresses; returns the number of pages newly
 *                      mapped (>= 0).  When no page is free, the oldest Reusable set is unmapped
 *                      first; with none left: XATTN_ENOMEM (the range keeps what it had).
 * xtensor_premap_async the same request handed to the pool's background thread; returns at once.
 *                      Meant to be called while the current decode step runs, for the pages the
 *                      next tokens will need.  xtensor_premap_wait blocks until the range's requests
 *                      are done and returns the last one's status.  xtensor_grow and xtensor_close
 *                      wait for pending requests of their range first.
 * xtensor_close        the request is finished.  keep_reusable != 0: the pages stay mapped and become
 *                      Reusable (the handle stays known to the pool, not to the caller);
 *                      keep_reusable == 0: unmap at once, pages become Free.
 * xtensor_range_pages  page ids behind virtual pages 0, 1, ... of a range (HOST int64[n]); returns
 *                      the count.  With the identity page = floor((va - base) / page_size) this is
 *                      the whole address translation.
 * Pool and ranges are thread-safe against each other; the caller makes sure no kernel uses a range
 * that is being closed.  Errors as for xtensor_map.
 */
enum { XTENSOR_PAGE_FREE = 0, XTENSOR_PAGE_ALLOCATED = 1, XTENSOR_PAGE_MAPPED = 2, XTENSOR_PAGE_REUSABLE = 3 };
int xtensor_pool_create(int device, size_t n_pages, uint64_t seed, void** pool_out);
int xtensor_pool_destroy(void* pool);
int xtensor_pool_counts(void* pool, size_t* counts_out);
int xtensor_page_info(void* pool, size_t page_id, int* status_out, uint64_t* owner_out);
int xtensor_open(void* pool, uint64_t session, size_t reserve_bytes, size_t mapped_bytes, void** base_out,
                 void** range_out, int* reused_out);
int xtensor_grow(void* range, size_t mapped_bytes);
int xtensor_premap_async(void* range, size_t mapped_bytes);
int xtensor_premap_wait(void* range);
int xtensor_close(void* range, int keep_reusable);
int xtensor_range_pages(void* range, int64_t* page_ids_out, int n);

/*
 * write_kvcache (section 4.3, "Operator Adaptation": the operator that appends new tokens' K and V
 * takes the range's starting address and an offset, no block table).  Copies the q_len new rows of
 * every sequence to rows [kv_lens[b] - q_len, kv_lens[b]) of its K and V ranges, i.e. kv_lens holds
 * the lengths AFTER the append, the same array xattn_decode takes next.  Rows whose index would be
 * negative are skipped.  The destination rows must be backed (xtensor_grow first).
 * k_new, v_new  DEVICE bf16 [batch, q_len, n_kv_heads, head_dim], 16-byte aligned
 * k_ptrs, v_ptrs DEVICE arrays[batch] of DEVICE pointers (as for xattn_decode, written here)
 * kv_lens       DEVICE int32[batch].  Asynchronous on `stream`; head_dim * n_kv_heads * 2 must be a
 * multiple of 16.
 */
int xattn_write_kvcache(const void* k_new, const void* v_new, void* const* k_ptrs, void* const* v_ptrs,
                        const int32_t* kv_lens, int batch, int q_len, int n_kv_heads, int head_dim,
                        void* stream);

/* Synchronous copies between HOST memory and any DEVICE address (mapped ranges included). */
int xtensor_upload(void* dst_device, const void* src_host, size_t bytes);
int xtensor_download(void* dst_host, const void* src_device, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* XATTN_H_ */
