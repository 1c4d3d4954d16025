// C-ABI entry points of libxattn.so: argument checks, workspace, kernel launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>
#include <vector>

#include "../../include/xattn.h"
#include "xattn_hip_error.h"
#include "xattn_host.h"
#include "xattn_kernels.h"
#include "xattn_plan.h"

namespace xattn {

namespace {

constexpr int kMaxDevices = 16;
constexpr int kMaxBatch = 4096;
constexpr int kMaxQLen = 16;
constexpr int kMaxRows = 64;
constexpr int kDefaultMinPieceTokens = 64;

// The library's own workspaces: one per (device, stream), so that calls on different streams of a
// device may overlap.  A buffer that has become too small is RETIRED, not freed: a HIP graph recorded
// earlier may hold its address in the arguments of its kernel nodes, and replaying such a graph must
// stay valid.  Buffers grow geometrically, so the retired ones add up to less than the live one
// times four; all of them are released when the process ends.
struct StreamWorkspace {
    hipStream_t stream = nullptr;
    void* ptr = nullptr;
    size_t bytes = 0;
};
constexpr int kMaxStreamWorkspaces = 64;

struct DeviceState {
    int n_cu = 0;
    std::vector<StreamWorkspace> owned;   // library-owned workspaces, one per stream seen
    std::vector<void*> retired;           // outgrown buffers, kept alive (see above)
    void* user_ws = nullptr;              // caller-provided workspace, if any: used for every stream
    size_t user_bytes = 0;
};

std::mutex g_mutex;
DeviceState g_dev[kMaxDevices];
int g_cfg_pieces = 0;
int g_cfg_min_piece = 0;
int g_cfg_timing = 0;
int g_cfg_path = 0;
int g_cfg_pv_mode = 0;
int g_cfg_mla_layout = 0;
int g_cfg_xcd_skew = 0;              // 0 = the kernel's default, n > 0 = n - 1 per mille

constexpr int kMaxTimedCalls = 4096;
std::vector<hipEvent_t> g_events;     // three per timed call, created on demand, reused across series
int g_timed_calls = 0;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int pieces_for(int n_cu) { return g_cfg_pieces > 0 ? g_cfg_pieces : n_cu; }

struct WorkspaceLayout {
    size_t meta_off, ml_off, o_off, total;
};

// Pieces of a latent-KV call: as many as give one workgroup per compute unit when a piece is worked
// on by several workgroups (one per group of query rows; they sit side by side on one XCD and share
// the piece's cache rows in its L2).  More pieces than that only add partial rows: measured with 256
// query rows per sequence, 128 pieces against 256 take 8 % off the call and 20 % off the merge.
int mla_pieces_for(int n_cu, int q_len, int n_heads) {
    if (g_cfg_pieces > 0) return g_cfg_pieces;
    int waves = 1, tiles = 1;
    mla_block_shape(q_len * n_heads, g_cfg_mla_layout, &waves, &tiles);
    const int rows_per_group = 16 * waves * tiles;
    const int n_groups = (q_len * n_heads + rows_per_group - 1) / rows_per_group;
    const int pieces = n_cu / n_groups / 8 * 8;
    return pieces < 8 ? 8 : pieces;
}

WorkspaceLayout layout_for(int batch, int q_len, int n_q_heads, int n_pieces) {
    const size_t slots = (size_t)n_pieces + (size_t)batch;
    const size_t rows = (size_t)q_len * (size_t)n_q_heads;
    WorkspaceLayout w;
    w.meta_off = 0;
    w.ml_off = align_up((size_t)batch * 2 * sizeof(int32_t), 256);
    w.o_off = w.ml_off + align_up(slots * rows * 2 * sizeof(float), 256);
    w.total = w.o_off + align_up(slots * rows * kHeadDim * sizeof(float), 256);
    return w;
}

// Latent-KV call: per-sequence table, (m, l, lq, 1 / scale) per partial row, partial rows of 512 fp16.
struct MlaWorkspaceLayout {
    size_t ml_off, o_off, total;
};
MlaWorkspaceLayout mla_layout_for(int batch, int q_len, int n_heads, int n_pieces) {
    const size_t slots = (size_t)n_pieces + (size_t)batch;
    const size_t rows = (size_t)q_len * (size_t)n_heads;
    MlaWorkspaceLayout w;
    w.ml_off = align_up((size_t)batch * 2 * sizeof(int32_t), 256);
    w.o_off = w.ml_off + align_up(slots * rows * 4 * sizeof(float), 256);
    w.total = w.o_off + align_up(slots * rows * 512 * sizeof(uint16_t), 256);
    return w;
}

int check_mla_shape(int batch, int q_len, int n_heads, int d_latent, int d_rope) {
    if (batch < 1 || q_len < 1 || n_heads < 1)
        return fail(XATTN_EINVAL, "xattn_mla_decode: batch, q_len and n_heads must be positive");
    if (d_latent != 512 || d_rope != 64)
        return fail(XATTN_EUNSUPPORTED, "xattn_mla_decode: latent %d + rope %d: only 512 + 64 is supported", d_latent, d_rope);
    if (batch > kMaxBatch) return fail(XATTN_EUNSUPPORTED, "batch %d exceeds %d", batch, kMaxBatch);
    if (q_len > kMaxQLen) return fail(XATTN_EUNSUPPORTED, "q_len %d exceeds %d", q_len, kMaxQLen);
    if ((long)q_len * n_heads > 4096) return fail(XATTN_EUNSUPPORTED, "q_len * n_heads = %ld exceeds 4096", (long)q_len * n_heads);
    return XATTN_OK;
}

int check_shape(int batch, int q_len, int n_q_heads, int n_kv_heads, int head_dim) {
    if (batch < 1 || q_len < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1)
        return fail(XATTN_EINVAL, "batch, q_len, n_q_heads, n_kv_heads and head_dim must be positive");
    if (n_q_heads % n_kv_heads != 0)
        return fail(XATTN_EUNSUPPORTED, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", n_q_heads, n_kv_heads);
    if (head_dim != kHeadDim) return fail(XATTN_EUNSUPPORTED, "head_dim %d: only 128 is supported", head_dim);
    if (batch > kMaxBatch) return fail(XATTN_EUNSUPPORTED, "batch %d exceeds %d", batch, kMaxBatch);
    if (q_len > kMaxQLen) return fail(XATTN_EUNSUPPORTED, "q_len %d exceeds %d", q_len, kMaxQLen);
    if ((n_q_heads / n_kv_heads) * q_len > kMaxRows)
        return fail(XATTN_EUNSUPPORTED, "(n_q_heads / n_kv_heads) * q_len = %d exceeds %d",
                    (n_q_heads / n_kv_heads) * q_len, kMaxRows);
    return XATTN_OK;
}

int device_state(DeviceState** out, int* dev_out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(XATTN_EUNSUPPORTED, "device index %d not supported", dev);
    DeviceState& d = g_dev[dev];
    if (d.n_cu == 0) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return fail_hip(e, "hipDeviceGetAttribute(MultiprocessorCount)");
        d.n_cu = n > 0 ? n : 256;
    }
    *out = &d;
    if (dev_out) *dev_out = dev;
    return XATTN_OK;
}

// A workspace of at least `total` bytes for a call on `stream`: the caller's if one was handed
// over, else the library's own for that stream, grown when needed (never while `stream` is being
// captured: growing allocates).
int acquire_workspace(DeviceState* d, size_t total, hipStream_t stream, const char* who, char** ws_out) {
    if (d->user_ws) {
        if (d->user_bytes < total)
            return fail(XATTN_ENOMEM, "%s: caller workspace has %zu bytes, this call needs %zu", who, d->user_bytes, total);
        *ws_out = static_cast<char*>(d->user_ws);
        return XATTN_OK;
    }
    StreamWorkspace* w = nullptr;
    for (auto& cand : d->owned)
        if (cand.stream == stream) w = &cand;
    if (!w || w->bytes < total) {
        hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &capture) == hipSuccess && capture != hipStreamCaptureStatusNone)
            return fail(XATTN_ENOMEM,
                        "%s: this stream's workspace must grow to %zu bytes but the stream is being captured; "
                        "run one call of this shape on the stream before the capture or hand over a workspace",
                        who, total);
        if (!w) {
            if ((int)d->owned.size() >= kMaxStreamWorkspaces)
                return fail(XATTN_ENOMEM, "%s: more than %d streams with a library-owned workspace on this device; "
                                          "hand over a workspace with xattn_set_workspace", who, kMaxStreamWorkspaces);
            d->owned.push_back(StreamWorkspace{stream, nullptr, 0});
            w = &d->owned.back();
        }
        const size_t want = total + total / 4;
        void* fresh = nullptr;
        const hipError_t e = hipMalloc(&fresh, want);
        if (e != hipSuccess) return fail_hip(e, "hipMalloc(workspace)");
        // Work already enqueued, and graphs already recorded, keep using the old buffer.
        if (w->ptr) d->retired.push_back(w->ptr);
        w->ptr = fresh;
        w->bytes = want;
    }
    *ws_out = static_cast<char*>(w->ptr);
    return XATTN_OK;
}

// Events for the current call when timing is on (three per call), else null.
int timing_events(hipEvent_t** events_out) {
    *events_out = nullptr;
    if (!g_cfg_timing || g_timed_calls >= kMaxTimedCalls) return XATTN_OK;
    while ((int)g_events.size() < 3 * (g_timed_calls + 1)) {
        hipEvent_t ev;
        hipError_t ee = hipEventCreate(&ev);
        if (ee != hipSuccess) return fail_hip(ee, "hipEventCreate");
        g_events.push_back(ev);
    }
    *events_out = &g_events[3 * g_timed_calls];
    return XATTN_OK;
}

}  // namespace

// xattn_decode and its variants: argument checks, workspace, launch.  `fixed_workspace`, when given,
// supplies the workspace instead of the per-stream one (and the call is never timed: events allocate).
int decode_call(const char* who, FixedWorkspaceFn fixed_workspace, const void* q, const void* const* k_ptrs,
                const void* const* v_ptrs, const int32_t* kv_lens, int batch, int q_len, int n_q_heads,
                int n_kv_heads, int head_dim, float scale, void* out, float* lse, void* stream) {
    if (!q || !k_ptrs || !v_ptrs || !kv_lens || !out)
        return fail(XATTN_EINVAL, "%s: q, k_ptrs, v_ptrs, kv_lens and out must not be NULL", who);
    int st = check_shape(batch, q_len, n_q_heads, n_kv_heads, head_dim);
    if (st != XATTN_OK) return st;
    if (!std::isfinite(scale)) return fail(XATTN_EINVAL, "%s: scale is not finite", who);
    if (reinterpret_cast<uintptr_t>(q) % 16 != 0 || reinterpret_cast<uintptr_t>(out) % 16 != 0)
        return fail(XATTN_EINVAL, "%s: q and out must be 16-byte aligned", who);

    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState* d = nullptr;
    int dev = 0;
    st = device_state(&d, &dev);
    if (st != XATTN_OK) return st;

    const int n_pieces = pieces_for(d->n_cu);
    const WorkspaceLayout w = layout_for(batch, q_len, n_q_heads, n_pieces);
    char* ws = nullptr;
    st = fixed_workspace ? fixed_workspace(who, dev, w.total, &ws)
                         : acquire_workspace(d, w.total, static_cast<hipStream_t>(stream), who, &ws);
    if (st != XATTN_OK) return st;

    DecodeParams prm;
    prm.q = static_cast<const uint16_t*>(q);
    prm.k_ptrs = k_ptrs;
    prm.v_ptrs = v_ptrs;
    prm.kv_lens = kv_lens;
    prm.batch = batch;
    prm.q_len = q_len;
    prm.n_q_heads = n_q_heads;
    prm.n_kv_heads = n_kv_heads;
    prm.group = n_q_heads / n_kv_heads;
    prm.scale_log2 = (float)((double)scale * 1.4426950408889634074);
    prm.out = static_cast<uint16_t*>(out);
    prm.lse = lse;
    prm.meta = reinterpret_cast<int32_t*>(ws + w.meta_off);
    prm.part_ml = reinterpret_cast<float*>(ws + w.ml_off);
    prm.part_o = reinterpret_cast<float*>(ws + w.o_off);
    prm.n_pieces = n_pieces;
    prm.min_piece_tokens = g_cfg_min_piece > 0 ? g_cfg_min_piece : kDefaultMinPieceTokens;
    if (prm.min_piece_tokens < 16) prm.min_piece_tokens = 16;      // one 16-key block at least
    prm.xcd_skew = g_cfg_xcd_skew > 0 ? g_cfg_xcd_skew - 1 : kDefaultXcdSkewGqa;
    prm.path = g_cfg_path;
    prm.pv_mode = g_cfg_pv_mode;

    hipEvent_t* events = nullptr;
    if (!fixed_workspace) {
        st = timing_events(&events);
        if (st != XATTN_OK) return st;
    }
    hipError_t e = launch_decode(prm, static_cast<hipStream_t>(stream), events);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    if (events) ++g_timed_calls;
    return XATTN_OK;
}

}  // namespace xattn

using namespace xattn;

extern "C" {

int xattn_configure(int key, int value) {
    if (value < 0 || value > 65536) return fail(XATTN_EINVAL, "xattn_configure: value %d outside [0, 65536]", value);
    std::lock_guard<std::mutex> lock(g_mutex);
    switch (key) {
        case XATTN_CFG_PIECES: g_cfg_pieces = value; return XATTN_OK;
        case XATTN_CFG_MIN_PIECE_TOKENS: g_cfg_min_piece = value; return XATTN_OK;
        case XATTN_CFG_TIMING: g_cfg_timing = value ? 1 : 0; return XATTN_OK;
        case XATTN_CFG_PATH:
            if (value > 2) return fail(XATTN_EINVAL, "xattn_configure: path %d is not 0, 1 or 2", value);
            g_cfg_path = value;
            return XATTN_OK;
        case XATTN_CFG_MLA_LAYOUT:
            if (value > 2) return fail(XATTN_EINVAL, "xattn_configure: MLA layout %d is not 0, 1 or 2", value);
            g_cfg_mla_layout = value;
            return XATTN_OK;
        case XATTN_CFG_XCD_SKEW:
            if (value > kMaxXcdSkew + 1) return fail(XATTN_EINVAL, "xattn_configure: XCD skew %d is not in [0, %d]", value, kMaxXcdSkew + 1);
            g_cfg_xcd_skew = value;
            return XATTN_OK;
        case XATTN_CFG_PV_MODE:
            if (value > 2) return fail(XATTN_EINVAL, "xattn_configure: pv mode %d is not 0, 1 or 2", value);
            g_cfg_pv_mode = value;
            return XATTN_OK;
        default: return fail(XATTN_EINVAL, "xattn_configure: unknown key %d", key);
    }
}

size_t xattn_workspace_bytes(int batch, int q_len, int n_q_heads, int n_kv_heads, int head_dim) {
    if (check_shape(batch, q_len, n_q_heads, n_kv_heads, head_dim) != XATTN_OK) return 0;
    // Upper bound over the automatic piece count of any supported device and the configured one.
    int pieces = g_cfg_pieces > 0 ? g_cfg_pieces : 256;
    DeviceState* d = nullptr;
    if (g_cfg_pieces == 0 && device_state(&d, nullptr) == XATTN_OK) pieces = pieces_for(d->n_cu);
    return layout_for(batch, q_len, n_q_heads, pieces).total;
}

size_t xattn_mla_workspace_bytes(int batch, int q_len, int n_heads, int d_latent, int d_rope) {
    if (check_mla_shape(batch, q_len, n_heads, d_latent, d_rope) != XATTN_OK) return 0;
    DeviceState* d = nullptr;
    const int n_cu = device_state(&d, nullptr) == XATTN_OK ? d->n_cu : 256;
    return mla_layout_for(batch, q_len, n_heads, mla_pieces_for(n_cu, q_len, n_heads)).total;
}

int xattn_set_workspace(void* dev_ptr, size_t bytes) {
    if ((dev_ptr == nullptr) != (bytes == 0))
        return fail(XATTN_EINVAL, "xattn_set_workspace: pointer and size must both be given or both be zero");
    if (reinterpret_cast<uintptr_t>(dev_ptr) % 256 != 0)
        return fail(XATTN_EINVAL, "xattn_set_workspace: pointer is not 256-byte aligned");
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState* d = nullptr;
    int st = device_state(&d, nullptr);
    if (st != XATTN_OK) return st;
    d->user_ws = dev_ptr;
    d->user_bytes = bytes;
    return XATTN_OK;
}

int xattn_decode(const void* q, const void* const* k_ptrs, const void* const* v_ptrs, const int32_t* kv_lens,
                 int batch, int q_len, int n_q_heads, int n_kv_heads, int head_dim, float scale, void* out,
                 float* lse, void* stream) {
    return decode_call("xattn_decode", nullptr, q, k_ptrs, v_ptrs, kv_lens, batch, q_len, n_q_heads, n_kv_heads,
                       head_dim, scale, out, lse, stream);
}

int xattn_timing_read(int* n_calls, float* decode_kernel_ms, float* merge_kernel_ms) {
    std::lock_guard<std::mutex> lock(g_mutex);
    float decode_ms = 0.0f, merge_ms = 0.0f;
    for (int i = 0; i < g_timed_calls; ++i) {
        hipError_t e = hipEventSynchronize(g_events[3 * i + 2]);
        if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize");
        float a = 0.0f, b = 0.0f;
        e = hipEventElapsedTime(&a, g_events[3 * i], g_events[3 * i + 1]);
        if (e != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
        e = hipEventElapsedTime(&b, g_events[3 * i + 1], g_events[3 * i + 2]);
        if (e != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
        decode_ms += a;
        merge_ms += b;
    }
    if (n_calls) *n_calls = g_timed_calls;
    if (decode_kernel_ms) *decode_kernel_ms = decode_ms;
    if (merge_kernel_ms) *merge_kernel_ms = merge_ms;
    g_timed_calls = 0;
    return XATTN_OK;
}

int xattn_mla_decode(const void* q, const void* const* c_ptrs, const int32_t* kv_lens, int batch, int q_len,
                     int n_heads, int d_latent, int d_rope, float scale, void* out, float* lse, void* stream) {
    if (!q || !c_ptrs || !kv_lens || !out)
        return fail(XATTN_EINVAL, "xattn_mla_decode: q, c_ptrs, kv_lens and out must not be NULL");
    int st = check_mla_shape(batch, q_len, n_heads, d_latent, d_rope);
    if (st != XATTN_OK) return st;
    if (!std::isfinite(scale) || !(scale > 0.0f)) return fail(XATTN_EINVAL, "xattn_mla_decode: scale %g is not a positive finite number", (double)scale);
    if (reinterpret_cast<uintptr_t>(q) % 16 != 0 || reinterpret_cast<uintptr_t>(out) % 16 != 0)
        return fail(XATTN_EINVAL, "xattn_mla_decode: q and out must be 16-byte aligned");

    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState* d = nullptr;
    st = device_state(&d, nullptr);
    if (st != XATTN_OK) return st;
    const int n_pieces = mla_pieces_for(d->n_cu, q_len, n_heads);
    const MlaWorkspaceLayout w = mla_layout_for(batch, q_len, n_heads, n_pieces);
    char* ws = nullptr;
    st = acquire_workspace(d, w.total, static_cast<hipStream_t>(stream), "xattn_mla_decode", &ws);
    if (st != XATTN_OK) return st;

    MlaParams prm;
    prm.q = static_cast<const uint16_t*>(q);
    prm.c_ptrs = c_ptrs;
    prm.kv_lens = kv_lens;
    prm.batch = batch;
    prm.q_len = q_len;
    prm.n_heads = n_heads;
    prm.scale_log2 = (float)((double)scale * 1.4426950408889634074);
    prm.out = static_cast<uint16_t*>(out);
    prm.lse = lse;
    prm.meta = reinterpret_cast<int32_t*>(ws);
    prm.part_ml = reinterpret_cast<float*>(ws + w.ml_off);
    prm.part_o = reinterpret_cast<uint16_t*>(ws + w.o_off);
    prm.n_pieces = n_pieces;
    prm.min_piece_tokens = g_cfg_min_piece > 0 ? g_cfg_min_piece : kDefaultMinPieceTokens;
    if (prm.min_piece_tokens < 16) prm.min_piece_tokens = 16;
    prm.xcd_skew = g_cfg_xcd_skew > 0 ? g_cfg_xcd_skew - 1 : kDefaultXcdSkewMla;
    prm.layout = g_cfg_mla_layout;
    prm.weight_mode = g_cfg_pv_mode;
    hipEvent_t* events = nullptr;
    st = timing_events(&events);
    if (st != XATTN_OK) return st;
    hipError_t e = launch_mla_decode(prm, static_cast<hipStream_t>(stream), events);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    if (events) ++g_timed_calls;
    return XATTN_OK;
}

int xattn_write_kvcache(const void* k_new, const void* v_new, void* const* k_ptrs, void* const* v_ptrs,
                        const int32_t* kv_lens, int batch, int q_len, int n_kv_heads, int head_dim, void* stream) {
    if (!k_new || !v_new || !k_ptrs || !v_ptrs || !kv_lens)
        return fail(XATTN_EINVAL, "xattn_write_kvcache: NULL argument");
    if (batch < 1 || q_len < 1 || n_kv_heads < 1 || head_dim < 1)
        return fail(XATTN_EINVAL, "xattn_write_kvcache: batch, q_len, n_kv_heads and head_dim must be positive");
    const long row_bytes = (long)n_kv_heads * head_dim * 2;
    if (row_bytes % 16 != 0 || row_bytes > (1 << 24))
        return fail(XATTN_EUNSUPPORTED, "xattn_write_kvcache: a token row of %ld bytes is not a multiple of 16", row_bytes);
    if (reinterpret_cast<uintptr_t>(k_new) % 16 != 0 || reinterpret_cast<uintptr_t>(v_new) % 16 != 0)
        return fail(XATTN_EINVAL, "xattn_write_kvcache: k_new and v_new must be 16-byte aligned");
    if ((long)batch * q_len > (1L << 30)) return fail(XATTN_EUNSUPPORTED, "xattn_write_kvcache: batch * q_len too large");
    WriteParams prm;
    prm.k_new = static_cast<const uint16_t*>(k_new);
    prm.v_new = static_cast<const uint16_t*>(v_new);
    prm.k_ptrs = k_ptrs;
    prm.v_ptrs = v_ptrs;
    prm.kv_lens = kv_lens;
    prm.batch = batch;
    prm.q_len = q_len;
    prm.row_bytes = (int)row_bytes;
    hipError_t e = launch_write_kvcache(prm, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return XATTN_OK;
}

int xtensor_upload(void* dst_device, const void* src_host, size_t bytes) {
    if (bytes == 0) return XATTN_OK;
    if (!dst_device || !src_host) return fail(XATTN_EINVAL, "xtensor_upload: NULL pointer");
    hipError_t e = hipMemcpy(dst_device, src_host, bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail_hip(e, "hipMemcpy(host to device)");
    return XATTN_OK;
}

int xtensor_download(void* dst_host, const void* src_device, size_t bytes) {
    if (bytes == 0) return XATTN_OK;
    if (!dst_host || !src_device) return fail(XATTN_EINVAL, "xtensor_download: NULL pointer");
    hipError_t e = hipMemcpy(dst_host, src_device, bytes, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(e, "hipMemcpy(device to host)");
    return XATTN_OK;
}

}  // extern "C"
