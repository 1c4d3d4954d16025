"""ctypes binding of libxattn.so: the same names and arguments as include/xattn.h.

Argument marshalling only -- every step of the path runs in the library's kernels.  Device
pointers may be given as integers or as torch tensors (their ``data_ptr()`` is taken).  There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

from . import build as _build

XATTN_OK, XATTN_EINVAL, XATTN_EUNSUPPORTED, XATTN_ENOMEM, XATTN_EHIP = 0, -1, -2, -3, -4
XATTN_CFG_PIECES, XATTN_CFG_MIN_PIECE_TOKENS, XATTN_CFG_TIMING, XATTN_CFG_PATH, XATTN_CFG_PV_MODE, XATTN_CFG_MLA_LAYOUT = 0, 1, 2, 3, 4, 5
XATTN_CFG_XCD_SKEW = 6
XTENSOR_CHUNK_BYTES = 2 << 20

EXPORTS = ["xattn_last_error", "xattn_decode", "xattn_decode_noalloc", "xattn_workspace_bytes", "xattn_set_workspace",
           "xattn_configure", "xattn_timing_read", "xtensor_map", "xtensor_unmap", "xtensor_chunk_order",
           "xtensor_physical_view", "xtensor_upload", "xtensor_download",
           "xtensor_pool_create", "xtensor_pool_destroy", "xtensor_pool_counts", "xtensor_page_info",
           "xtensor_open", "xtensor_grow", "xtensor_premap_async", "xtensor_premap_wait", "xtensor_close",
           "xtensor_range_pages", "xattn_write_kvcache", "xattn_mla_decode", "xattn_mla_workspace_bytes", "xbeam_select"]
XBEAM_FULL_SORT, XBEAM_CHECK_INPUT = 1, 2
XTENSOR_PAGE_FREE, XTENSOR_PAGE_ALLOCATED, XTENSOR_PAGE_MAPPED, XTENSOR_PAGE_REUSABLE = 0, 1, 2, 3


class XattnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("xattn status %d: %s" % (status, message))
        self.status = status


_lib = None


def _signatures():
    vp, i32, sz, u64, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_float
    P = ctypes.POINTER
    return {
        "xattn_last_error": (ctypes.c_char_p, []),
        "xattn_decode": (i32, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp]),
        "xattn_decode_noalloc": (i32, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp]),
        "xattn_workspace_bytes": (sz, [i32] * 5),
        "xattn_mla_workspace_bytes": (sz, [i32] * 5),
        "xattn_set_workspace": (i32, [vp, sz]),
        "xattn_configure": (i32, [i32, i32]),
        "xattn_timing_read": (i32, [P(i32), P(f32), P(f32)]),
        "xtensor_map": (i32, [sz, sz, u64, i32, P(vp), P(vp)]),
        "xtensor_unmap": (i32, [vp]),
        "xtensor_chunk_order": (i32, [vp, vp, i32]),
        "xtensor_physical_view": (i32, [vp, P(vp)]),
        "xtensor_upload": (i32, [vp, vp, sz]),
        "xtensor_download": (i32, [vp, vp, sz]),
        "xtensor_pool_create": (i32, [i32, sz, u64, P(vp)]),
        "xtensor_pool_destroy": (i32, [vp]),
        "xtensor_pool_counts": (i32, [vp, P(sz)]),
        "xtensor_page_info": (i32, [vp, sz, P(i32), P(u64)]),
        "xtensor_open": (i32, [vp, u64, sz, sz, P(vp), P(vp), P(i32)]),
        "xtensor_grow": (i32, [vp, sz]),
        "xtensor_premap_async": (i32, [vp, sz]),
        "xtensor_premap_wait": (i32, [vp]),
        "xtensor_close": (i32, [vp, i32]),
        "xtensor_range_pages": (i32, [vp, vp, i32]),
        "xattn_mla_decode": (i32, [vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp]),
        "xbeam_select": (i32, [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]),
        "xattn_write_kvcache": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]),
    }


def bind(lib: ctypes.CDLL, required=None) -> ctypes.CDLL:
    """Set the C signatures on `lib` for every declared entry point it exports; the names in `required`
    (default: all of EXPORTS) must be there."""
    sigs = _signatures()
    for name in (EXPORTS if required is None else required):
        if not hasattr(lib, name):
            raise AttributeError("%s does not export %s" % (lib._name, name))
    for name, (restype, argtypes) in sigs.items():
        if hasattr(lib, name):
            fn = getattr(lib, name)
            fn.restype = restype
            fn.argtypes = argtypes
    return lib


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libxattn.so (building it only if no built library exists)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or os.environ.get("XATTN_LIBRARY") or _build.LIB_PATH      # XATTN_LIBRARY: another build of libxattn.so
    if not os.path.exists(p):
        if p != _build.LIB_PATH:
            raise FileNotFoundError(p)
        p = _build.build()
    elif p == _build.LIB_PATH and _build.is_stale():
        # a built library is loaded as it is (builds happen in build(), not here); say so when it is old
        import warnings
        warnings.warn("libxattn.so is older than its sources; run paper_2510_14686_amd/build.py to rebuild it")
    lib = bind(ctypes.CDLL(p))
    if path is None:
        _lib = lib
    return lib


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    raise TypeError("expected an integer address or a tensor, got %r" % type(x))


def _check(status: int) -> int:
    if status < 0:
        raise XattnError(status, xattn_last_error())
    return status


def xattn_last_error() -> str:
    return load_library().xattn_last_error().decode("utf-8", "replace")


def xattn_decode(q, k_ptrs, v_ptrs, kv_lens, batch: int, q_len: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, scale: float, out, lse=None, stream=None) -> None:
    """Enqueue decode attention; see include/xattn.h.  All pointers are device addresses."""
    if stream is not None and not isinstance(stream, int):
        stream = int(stream.cuda_stream)
    _check(load_library().xattn_decode(_ptr(q), _ptr(k_ptrs), _ptr(v_ptrs), _ptr(kv_lens), batch, q_len,
                                       n_q_heads, n_kv_heads, head_dim, ctypes.c_float(scale), _ptr(out),
                                       _ptr(lse), stream))


def xattn_decode_noalloc(q, k_ptrs, v_ptrs, kv_lens, batch: int, q_len: int, n_q_heads: int, n_kv_heads: int,
                         head_dim: int, scale: float, out, lse=None, stream=None) -> None:
    """xattn_decode without any device allocation (fixed scratch array); see include/xattn.h."""
    if stream is not None and not isinstance(stream, int):
        stream = int(stream.cuda_stream)
    _check(load_library().xattn_decode_noalloc(_ptr(q), _ptr(k_ptrs), _ptr(v_ptrs), _ptr(kv_lens), batch, q_len,
                                               n_q_heads, n_kv_heads, head_dim, ctypes.c_float(scale), _ptr(out),
                                               _ptr(lse), stream))


XATTN_NOALLOC_SCRATCH_BYTES = 32 << 20


def xattn_workspace_bytes(batch: int, q_len: int, n_q_heads: int, n_kv_heads: int, head_dim: int) -> int:
    n = int(load_library().xattn_workspace_bytes(batch, q_len, n_q_heads, n_kv_heads, head_dim))
    if n == 0:
        raise XattnError(XATTN_EUNSUPPORTED, xattn_last_error())
    return n


def xattn_mla_workspace_bytes(batch: int, q_len: int, n_heads: int, d_latent: int = 512, d_rope: int = 64) -> int:
    n = int(load_library().xattn_mla_workspace_bytes(batch, q_len, n_heads, d_latent, d_rope))
    if n == 0:
        raise XattnError(XATTN_EUNSUPPORTED, xattn_last_error())
    return n


def xattn_set_workspace(dev_ptr, nbytes: int) -> None:
    _check(load_library().xattn_set_workspace(_ptr(dev_ptr), nbytes))


def xattn_configure(key: int, value: int) -> None:
    _check(load_library().xattn_configure(key, value))


def xattn_timing_read() -> Tuple[int, float, float]:
    """(timed calls, sum of decode-kernel ms, sum of merge-kernel ms) since the last read."""
    n, a, b = ctypes.c_int(), ctypes.c_float(), ctypes.c_float()
    _check(load_library().xattn_timing_read(ctypes.byref(n), ctypes.byref(a), ctypes.byref(b)))
    return int(n.value), float(a.value), float(b.value)


def xtensor_map(reserve_bytes: int, mapped_bytes: int, seed: int, device: int) -> Tuple[int, int]:
    """Returns (base device address, handle)."""
    base, handle = ctypes.c_void_p(), ctypes.c_void_p()
    _check(load_library().xtensor_map(reserve_bytes, mapped_bytes, seed, device, ctypes.byref(base),
                                      ctypes.byref(handle)))
    return int(base.value), int(handle.value)


def xtensor_unmap(handle: int) -> None:
    _check(load_library().xtensor_unmap(handle))


def xtensor_chunk_order(handle: int) -> np.ndarray:
    lib = load_library()
    # ask with a generous buffer: a range of MaxSeqLen tokens has at most a few thousand chunks
    buf = np.empty(1 << 16, dtype=np.int32)
    n = _check(lib.xtensor_chunk_order(handle, buf.ctypes.data, buf.size))
    return buf[:n].copy()


def xtensor_physical_view(handle: int) -> int:
    view = ctypes.c_void_p()
    _check(load_library().xtensor_physical_view(handle, ctypes.byref(view)))
    return int(view.value)


def xtensor_upload(dst_device: int, src: np.ndarray) -> None:
    src = np.ascontiguousarray(src)
    _check(load_library().xtensor_upload(dst_device, src.ctypes.data, src.nbytes))


def xtensor_download(dst: np.ndarray, src_device: int) -> None:
    assert dst.flags["C_CONTIGUOUS"]
    _check(load_library().xtensor_download(dst.ctypes.data, src_device, dst.nbytes))


def xtensor_pool_create(device: int, n_pages: int, seed: int) -> int:
    pool = ctypes.c_void_p()
    _check(load_library().xtensor_pool_create(device, n_pages, seed, ctypes.byref(pool)))
    return int(pool.value)


def xtensor_pool_destroy(pool: int) -> None:
    _check(load_library().xtensor_pool_destroy(pool))


def xtensor_pool_counts(pool: int) -> Tuple[int, int, int, int]:
    """(free, allocated, mapped, reusable) pages."""
    c = (ctypes.c_size_t * 4)()
    _check(load_library().xtensor_pool_counts(pool, c))
    return tuple(int(x) for x in c)


def xtensor_page_info(pool: int, page_id: int) -> Tuple[int, int]:
    """(status, owner session) of one page."""
    st, owner = ctypes.c_int(), ctypes.c_uint64()
    _check(load_library().xtensor_page_info(pool, page_id, ctypes.byref(st), ctypes.byref(owner)))
    return int(st.value), int(owner.value)


def xtensor_open(pool: int, session: int, reserve_bytes: int, mapped_bytes: int) -> Tuple[int, int, bool]:
    """Returns (base device address, range handle, reused)."""
    base, rng, reused = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_int()
    _check(load_library().xtensor_open(pool, session, reserve_bytes, mapped_bytes, ctypes.byref(base),
                                       ctypes.byref(rng), ctypes.byref(reused)))
    return int(base.value), int(rng.value), bool(reused.value)


def xtensor_grow(rng: int, mapped_bytes: int) -> int:
    return _check(load_library().xtensor_grow(rng, mapped_bytes))


def xtensor_premap_async(rng: int, mapped_bytes: int) -> None:
    _check(load_library().xtensor_premap_async(rng, mapped_bytes))


def xtensor_premap_wait(rng: int) -> None:
    _check(load_library().xtensor_premap_wait(rng))


def xtensor_close(rng: int, keep_reusable: bool) -> None:
    _check(load_library().xtensor_close(rng, 1 if keep_reusable else 0))


def xtensor_range_pages(rng: int) -> np.ndarray:
    buf = np.empty(1 << 16, dtype=np.int64)
    n = _check(load_library().xtensor_range_pages(rng, buf.ctypes.data, buf.size))
    return buf[:n].copy()


def xattn_write_kvcache(k_new, v_new, k_ptrs, v_ptrs, kv_lens, batch: int, q_len: int, n_kv_heads: int,
                        head_dim: int, stream=None) -> None:
    """Enqueue the append of q_len new K/V rows per sequence; see include/xattn.h."""
    if stream is not None and not isinstance(stream, int):
        stream = int(stream.cuda_stream)
    _check(load_library().xattn_write_kvcache(_ptr(k_new), _ptr(v_new), _ptr(k_ptrs), _ptr(v_ptrs), _ptr(kv_lens),
                                              batch, q_len, n_kv_heads, head_dim, stream))


def xattn_mla_decode(q, c_ptrs, kv_lens, batch: int, q_len: int, n_heads: int, d_latent: int, d_rope: int,
                     scale: float, out, lse=None, stream=None) -> None:
    """Enqueue latent-KV (MLA-shaped) decode attention; see include/xattn.h."""
    if stream is not None and not isinstance(stream, int):
        stream = int(stream.cuda_stream)
    _check(load_library().xattn_mla_decode(_ptr(q), _ptr(c_ptrs), _ptr(kv_lens), batch, q_len, n_heads, d_latent,
                                           d_rope, ctypes.c_float(scale), _ptr(out), _ptr(lse), stream))


def xbeam_select(beam_lp, cand_lp, cand_tok=None, flags: int = 0, out_lp=None, out_parent=None, out_tok=None,
                 visited=None):
    """Host beam-search selection on numpy arrays; see include/xbeam.h.  beam_lp float32 [R, W], cand_lp
    float32 [R, W, K] descending along K, cand_tok int32 [R, W, K] or None.  Outputs are written into the
    given arrays (allocated here when omitted) and returned as (out_lp, out_parent, out_tok, visited)."""
    import numpy as np

    def host(a, dtype, shape, name):
        if not (isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous and a.shape == shape):
            raise TypeError("%s must be a C-contiguous %s array of shape %s" % (name, np.dtype(dtype).name, shape))
        return a.ctypes.data

    if not isinstance(cand_lp, np.ndarray) or cand_lp.ndim != 3:
        raise TypeError("cand_lp must be a float32 array [n_req, beam_width, top_k]")
    R, W, K = cand_lp.shape
    out_lp = np.empty((R, W), np.float32) if out_lp is None else out_lp
    out_parent = np.empty((R, W), np.int32) if out_parent is None else out_parent
    out_tok = np.empty((R, W), np.int32) if out_tok is None else out_tok
    visited = np.zeros(R, np.int64) if visited is None else visited
    _check(load_library().xbeam_select(
        host(beam_lp, np.float32, (R, W), "beam_lp"), host(cand_lp, np.float32, (R, W, K), "cand_lp"),
        None if cand_tok is None else host(cand_tok, np.int32, (R, W, K), "cand_tok"), R, W, K, flags,
        host(out_lp, np.float32, (R, W), "out_lp"), host(out_parent, np.int32, (R, W), "out_parent"),
        host(out_tok, np.int32, (R, W), "out_tok"), host(visited, np.int64, (R,), "visited")))
    return out_lp, out_parent, out_tok, visited
